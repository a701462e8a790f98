"""GPU parity: every call goes through the C-ABI (via the thin binding) and is
compared element by element with the CPU oracle on the same seeded inputs.

Bars: fp32 path 1e-5, bf16 / fp8-cache path 2e-2, both as
max|gpu - oracle| / max|oracle| over the tensor; page gather bit-exact.
"""
import math

import numpy as np
import pytest

import oracle
from helpers import TOL, DeviceWorkload, lse_err, max_abs_rel, storage_bits, to_torch, widen_gpu
from workloads import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mla():
    import torch
    assert torch.cuda.is_available()
    from paper_2502_07864_amd import mla as m
    m.lib()  # fails loudly if the HIP library is not built
    return m


def oracle_decode(w, q_abs_np, b_sel=None):
    """Oracle o_lat / lse for (a subset of) the sequences, given q_abs in its stored dtype."""
    sel = slice(None) if b_sel is None else np.asarray(b_sel)
    return oracle.decode_absorbed(q_abs_np[sel], w.q_rope[sel], w.pool, w.kv_scale,
                                  w.page_table[sel], w.seq_lens[sel], w.softmax_scale)


def gpu_q_abs(mla, d):
    return mla.absorb_q(d.q_nope, d.W_UK)


def q_abs_storage(t):
    """GPU q_abs tensor -> numpy storage array the oracle wrapper understands."""
    bits = storage_bits(t)
    return bits if bits.dtype == np.uint16 else bits.view(np.float32)


def run_decode(mla, d, q_abs, num_splits, flags=0):
    w = d.w
    o, lse = mla.decode_paged(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                              num_splits=num_splits, kv_scale=d.kv_scale, return_lse=True, flags=flags)
    return o, lse


def check_decode(mla, w, num_splits, flags=0, b_sel=None, tol=None):
    import torch
    d = DeviceWorkload(w)
    q_abs = gpu_q_abs(mla, d)
    o, lse = run_decode(mla, d, q_abs, num_splits, flags)
    torch.cuda.synchronize()
    ref_o, ref_lse = oracle_decode(w, q_abs_storage(q_abs), b_sel)
    sel = slice(None) if b_sel is None else np.asarray(b_sel)
    got_o, got_lse = widen_gpu(o)[sel], widen_gpu(lse)[sel]
    assert np.isfinite(got_o).all()
    tol = tol or TOL[w.io_dtype]
    err = max_abs_rel(got_o, ref_o)
    assert err <= tol, f"{w.name} splits={num_splits} flags={flags}: o_lat err {err:.3e} > {tol}"
    le = lse_err(got_lse, ref_lse)
    assert le <= (1e-4 if w.io_dtype == "f32" else 2e-2), f"lse err {le:.3e}"
    return err


# ------------------------------------------------------------------ gather

@pytest.mark.parametrize("name,shrink", [("C3", 16), ("C5", 64), ("C2", 4), ("C1", 1)])
def test_gather_bit_exact(mla, name, shrink):
    import torch
    w = synth.config(name, shrink=shrink)
    d = DeviceWorkload(w)
    max_len = int(w.seq_lens.max())
    dense = mla.gather_paged(d.pool, d.page_table, d.seq_lens, max_len)
    torch.cuda.synchronize()
    want = oracle.gather_paged(w.pool, w.page_table, w.seq_lens, max_len)
    assert dense.cpu().numpy().tobytes() == want.tobytes()


@pytest.mark.parametrize("d_c,H,num_splits", [(512, 32, 1), (512, 32, 7), (256, 28, 2)])
def test_stream_probe_reads_only(mla, d_c, H, num_splits):
    """The diagnostic stream kernel (tile traffic of the bf16 decode kernel, nothing else) over
    ragged lengths, an empty sequence, NaN-poisoned free pages and a page id outside the pool:
    it completes, and the cache, the tables and a decode call afterwards are what they were."""
    import torch
    w = ragged_workload(d_c=d_c, H=H, lens=[300, 0, 64, 1000, 65, 1], seed=61)
    d = DeviceWorkload(w)
    table = d.page_table.clone()
    table[3, 2] = w.num_pages + 5          # skipped by the kernel, never dereferenced
    before = d.pool.clone()
    mla.diag_stream_tiles(d.pool, table, d.seq_lens, num_splits)
    mla.diag_stream_tiles(d.pool, d.page_table, d.seq_lens, num_splits)
    torch.cuda.synchronize()
    assert d.pool.view(torch.int16).equal(before.view(torch.int16))
    check_decode(mla, w, num_splits)


# ------------------------------------------------------- the two projections

@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("B,H,d_head,d_c", [(1, 32, 128, 512), (16, 32, 128, 512), (37, 28, 128, 256),
                                            (3, 5, 24, 40), (130, 4, 128, 512), (128, 28, 128, 256),
                                            (64, 32, 128, 512)])
def test_absorb_and_out_proj(mla, io, B, H, d_head, d_c):
    import torch
    r = synth.stream(7, B * 1000 + H)
    q = synth.store(synth.normal(r, (B, H, d_head)), io)
    Wk = synth.store(synth.normal(r, (H, d_head, d_c), 1 / math.sqrt(d_c)), io)
    o = synth.store(synth.normal(r, (B, H, d_c)), io)
    Wv = synth.store(synth.normal(r, (H, d_c, d_head), 1 / math.sqrt(d_c)), io)
    got_a = mla.absorb_q(to_torch(q, io), to_torch(Wk, io))
    got_o = mla.out_proj(to_torch(o, io), to_torch(Wv, io))
    torch.cuda.synchronize()
    assert max_abs_rel(widen_gpu(got_a), oracle.absorb_q(q, Wk)) <= TOL[io]
    assert max_abs_rel(widen_gpu(got_o), oracle.out_proj(o, Wv)) <= TOL[io]


def test_offline_fold_of_W_UK_into_the_query_projection(mla):
    """App. A.2.2: W'^Q_h = (W^{UK}_h)^T W^Q_h can be built offline with the absorb call itself,
    by passing the rows of W^Q (one per model dimension) as the batch:  fold[D, h, :] =
    W^Q[D, h, :] . W_UK[h].  The folded route x . fold then equals absorb(x . W^Q)."""
    import torch
    D, H, d_head, d_c, B = 384, 8, 128, 512, 5
    r = synth.stream(11, 3)
    WQ = synth.store(synth.normal(r, (D, H, d_head), 1 / math.sqrt(D)), "bf16")     # [D, H, d_head]
    Wk = synth.store(synth.normal(r, (H, d_head, d_c), 1 / math.sqrt(d_c)), "bf16")
    x = synth.normal(r, (B, D)).astype(np.float64)
    fold = mla.absorb_q(to_torch(WQ, "bf16"), to_torch(Wk, "bf16"))                 # [D, H, d_c] on the GPU
    torch.cuda.synchronize()
    want_fold = oracle.absorb_q(WQ, Wk)                                             # fp64, from the stored values
    assert max_abs_rel(widen_gpu(fold), want_fold) <= TOL["bf16"]
    q_folded = np.einsum("bD,Dhc->bhc", x, widen_gpu(fold).astype(np.float64))
    q_nope = np.einsum("bD,Dhk->bhk", x, oracle.widen(WQ).astype(np.float64))
    q_two_step = np.einsum("bhk,hkc->bhc", q_nope, oracle.widen(Wk).astype(np.float64))
    assert max_abs_rel(q_folded, q_two_step) <= TOL["bf16"]


def test_offline_fold_of_W_UV_into_the_output_projection(mla):
    """App. A.2.2 (the second rewrite): y = W^O [W^{UV}_h o_h]_h = sum_h W'^O_h o^_h with
    W'^O_h = W^{UV}_h W^O_h, built offline with the library's own per-head product by passing the d_c
    rows of every W^{UV}_h as the batch:  fold[c, h, :] = W_UV[h][c, :] . W^O[h].  The folded route
    sum_h o^_h . fold[:, h, :] then equals W^O applied to out_proj's result."""
    import torch
    D, H, d_head, d_c, B = 384, 8, 128, 512, 5
    r = synth.stream(12, 3)
    Wv = synth.store(synth.normal(r, (H, d_c, d_head), 1 / math.sqrt(d_c)), "bf16")      # [H, d_c, d_head]
    WO = synth.store(synth.normal(r, (H, d_head, D), 1 / math.sqrt(H * d_head)), "bf16") # [H, d_head, D]
    o_lat = synth.normal(r, (B, H, d_c)).astype(np.float64)
    rows = np.ascontiguousarray(np.transpose(Wv, (1, 0, 2)))                              # [d_c, H, d_head]: the batch
    fold = mla.absorb_q(to_torch(rows, "bf16"), to_torch(WO, "bf16"))                     # [d_c, H, D] on the GPU
    torch.cuda.synchronize()
    want_fold = oracle.absorb_q(rows, WO)                                                  # fp64, from the stored values
    assert max_abs_rel(widen_gpu(fold), want_fold) <= TOL["bf16"]
    y_folded = np.einsum("bhc,chD->bD", o_lat, widen_gpu(fold).astype(np.float64))
    o_head = np.einsum("bhc,hck->bhk", o_lat, oracle.widen(Wv).astype(np.float64))
    y_two_step = np.einsum("bhk,hkD->bD", o_head, oracle.widen(WO).astype(np.float64))
    assert max_abs_rel(y_folded, y_two_step) <= TOL["bf16"]


# ------------------------------------------------------------ decode, fp32

@pytest.mark.parametrize("num_splits", [1, 4, 16])
def test_decode_C1_fp32_full(mla, num_splits):
    """Config 1 at full size: fp32 cache and io, 1024 tokens, identity page table."""
    w = synth.config("C1")
    err = check_decode(mla, w, num_splits)
    assert err <= 1e-5


def test_step_C1_fp32_three_calls(mla):
    import torch
    w = synth.config("C1")
    d = DeviceWorkload(w)
    q_abs = mla.absorb_q(d.q_nope, d.W_UK)
    o_lat = run_decode(mla, d, q_abs, 4)[0]
    out = mla.out_proj(o_lat, d.W_UV)
    torch.cuda.synchronize()
    ref = oracle.mla_step(w.q_nope, w.q_rope, w.W_UK, w.W_UV, w.pool, None, w.page_table,
                          w.seq_lens, w.softmax_scale)
    assert max_abs_rel(widen_gpu(q_abs), ref["q_abs"]) <= 1e-5
    assert max_abs_rel(widen_gpu(o_lat), ref["o_lat"]) <= 1e-5
    assert max_abs_rel(widen_gpu(out), ref["out"]) <= 1e-5


# ------------------------------------- decode, bf16: matrix-core + portable

RAGGED = [1, 63, 64, 65, 127, 128, 129, 700, 1, 2048, 33, 1000]


def ragged_workload(d_c=512, H=32, lens=RAGGED, seed=3, cache="bf16", io="bf16", **kw):
    return synth.make_workload("ragged", B=len(lens), H=H, d_head=128, d_c=d_c, d_rope=64,
                               seq_lens=lens, io_dtype=io, cache_dtype=cache, placement="random",
                               free_frac=0.2, seed=seed, **kw)


@pytest.mark.parametrize("num_splits", [1, 2, 7, 32])
@pytest.mark.parametrize("flags", [0, 1])
def test_decode_bf16_ragged(mla, num_splits, flags):
    """Lengths around the page size, several pages, ragged tails, NaN-poisoned
    free pages and tail slots; both kernels."""
    check_decode(mla, ragged_workload(), num_splits, flags)


@pytest.mark.parametrize("num_splits", [1, 3])
def test_decode_bf16_long_uniform_chunks(mla, num_splits):
    """Chunks of several hundred tiles in the two-stage kernel (d_c = 512 takes it at every chunk
    length), beside a short and a one-tile sequence."""
    w = ragged_workload(lens=[20000, 5000, 33], seed=11)
    check_decode(mla, w, num_splits)


@pytest.mark.parametrize("flags", [0, 1])
def test_decode_bf16_C4_shape(mla, flags):
    """28 heads (padded to the 32-row tile), d_c = 256."""
    w = ragged_workload(d_c=256, H=28, lens=[4096 // 4, 100, 640, 64, 1], seed=4)
    check_decode(mla, w, 2, flags)
    check_decode(mla, w, 5, flags)


def test_decode_bf16_C3_shrunk(mla):
    """Variable lengths, 10 % of the pool free, k_rope x4."""
    w = synth.config("C3", shrink=8)
    check_decode(mla, w, w.num_splits)
    check_decode(mla, w, 1, flags=1)


def test_decode_fp8_cache(mla):
    """fp8 e4m3 cache with one fp32 scale per token, bf16 and fp32 io."""
    w = synth.config("C5", shrink=32)
    for flags in (0, 1):                      # matrix-core kernel and portable kernel
        check_decode(mla, w, w.num_splits, flags)
        check_decode(mla, w, 3, flags)
    # ragged lengths, poisoned tails (NaN codes and NaN scales), 28 heads / d_c 256
    check_decode(mla, ragged_workload(cache="fp8_e4m3", seed=21), 5)
    check_decode(mla, ragged_workload(cache="fp8_e4m3", d_c=256, H=28, lens=[1, 64, 65, 1000, 31, 33], seed=22), 2)
    w2 = ragged_workload(cache="fp8_e4m3", io="f32", lens=[1, 65, 300, 64], seed=9)
    check_decode(mla, w2, 2, tol=1e-5)


def test_decode_fp8_chunks_longer_than_the_page_registers(mla):
    """256 sequences with one chunk each (nothing is cut again): the two long ones run 141 and 129
    tiles in one workgroup, past the 64 + 64 page ids a wavefront holds at a time.  Then the same with
    queries dominated by a key near the end of the long sequences: the second pass walks the page
    blocks again from the start."""
    import torch
    lens = [9000, 8200] + [1] * 254
    w = ragged_workload(cache="fp8_e4m3", lens=lens, seed=23)
    sel = [0, 1, 2, 255]
    check_decode(mla, w, 1, b_sel=sel)
    d = DeviceWorkload(w)
    q = oracle.widen(q_abs_storage(gpu_q_abs(mla, d))).astype(np.float32)
    for b, j in ((0, 8990), (1, 8150)):
        page, slot = int(w.page_table[b, j // 64]), j % 64
        row = np.array([oracle.widen_e4m3_code(c) for c in w.pool[page, slot, :512]]) * float(w.kv_scale[page, slot])
        q[b] = 30.0 * row[None, :] / max(1e-6, float(np.abs(row).max()))
    q_bits = synth.to_bf16_bits(q)
    o, lse = mla.decode_paged(to_torch(q_bits, "bf16"), d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                              num_splits=1, kv_scale=d.kv_scale, return_lse=True)
    torch.cuda.synchronize()
    ref_o, ref_lse = oracle.decode_absorbed(q_bits[sel], w.q_rope[sel], w.pool, w.kv_scale, w.page_table[sel],
                                            w.seq_lens[sel], w.softmax_scale)
    assert max_abs_rel(widen_gpu(o)[sel], ref_o) <= 2e-2
    assert lse_err(widen_gpu(lse)[sel], ref_lse) <= 2e-2


def test_decode_f32_io_bf16_cache(mla):
    w = ragged_workload(cache="bf16", io="f32", lens=[130, 64, 7], seed=10)
    check_decode(mla, w, 2, tol=1e-5)


def test_mfma_matches_portable_kernel(mla):
    """Two independent GPU implementations of the same call agree far inside the bar."""
    import torch
    w = ragged_workload(seed=11)
    d = DeviceWorkload(w)
    q_abs = gpu_q_abs(mla, d)
    a = widen_gpu(run_decode(mla, d, q_abs, 4, 0)[0])
    b = widen_gpu(run_decode(mla, d, q_abs, 4, 1)[0])
    torch.cuda.synchronize()
    assert max_abs_rel(a, b) <= 1e-2


def test_fused_merge_out_proj_matches_separate_calls(mla):
    """mla_merge_out_proj = mla_merge_partials + mla_out_proj: identical o_lat / lse bits, out within
    rounding of the separate path and inside the bar against the oracle."""
    import torch
    cases = [(ragged_workload(seed=31), 7), (synth.config("C2", shrink=8), 4),
             (ragged_workload(d_c=256, H=28, lens=[300, 1, 64, 0, 999], seed=32), 3),
             (synth.config("C1", shrink=4), 2)]     # fp32: the unfused fallback inside the call
    for w, S in cases:
        d = DeviceWorkload(w)
        q_abs = mla.absorb_q(d.q_nope, d.W_UK)
        ws = mla.decode_paged(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                              num_splits=S, kv_scale=d.kv_scale, flags=mla.FLAG_SKIP_MERGE)
        o1, l1 = mla.merge_partials(ws, w.B, w.H, w.d_c, S, q_abs.dtype, return_lse=True)
        out1 = mla.out_proj(o1, d.W_UV)
        o2, out2, l2 = mla.merge_out_proj(ws, d.W_UV, w.B, S, return_lse=True)
        torch.cuda.synchronize()
        assert storage_bits(o1).tobytes() == storage_bits(o2).tobytes()
        assert storage_bits(l1).tobytes() == storage_bits(l2).tobytes()
        ref = oracle.out_proj(q_abs_storage(o2), w.W_UV)
        tol = TOL[w.io_dtype]
        assert max_abs_rel(widen_gpu(out2), ref) <= tol
        assert max_abs_rel(widen_gpu(out2), widen_gpu(out1)) <= tol / 2


def test_page_table_longer_than_any_sequence(mla):
    """Every sequence uses only the first part of its page-table row, so the trailing chunks of
    every sequence are empty (regular pattern of empty workgroups in the grid): results as usual,
    for chunk counts that leave a quarter, half and most of the chunks empty."""
    w = synth.make_workload("wide-table", B=6, H=32, d_head=128, d_c=512, d_rope=64,
                            seq_lens=[1500, 2048, 700, 2047, 64, 1], io_dtype="bf16", cache_dtype="bf16",
                            placement="random", max_pages_per_seq=128, num_splits=8, seed=41)
    for S in (4, 8, 32):
        check_decode(mla, w, S)
    check_decode(mla, w, 8, flags=1)


# ------------------------------------------------ balanced partition (flag 4)

BAL = 4


@pytest.mark.parametrize("num_splits", [1, 2, 7, 32])
def test_decode_balanced_ragged(mla, num_splits):
    """Equal page ranges per workgroup over the concatenated page lists: ranges cross sequence
    boundaries, short sequences share a workgroup, long ones span many."""
    check_decode(mla, ragged_workload(seed=71), num_splits, flags=BAL)


def test_decode_balanced_shapes_and_caches(mla):
    check_decode(mla, ragged_workload(d_c=256, H=28, lens=[300, 1, 64, 0, 999, 4096], seed=72), 3, flags=BAL)
    check_decode(mla, synth.config("C3", shrink=16), 4, flags=BAL)
    check_decode(mla, synth.config("C5", shrink=64), 8, flags=BAL)          # fp8 cache
    check_decode(mla, ragged_workload(lens=[5000], seed=73), 16, flags=BAL)  # one sequence, many workgroups
    check_decode(mla, ragged_workload(lens=[3, 2, 1], seed=74), 64, flags=BAL)   # more workgroups than pages
    check_decode(mla, ragged_workload(lens=[0, 1, 0, 64, 5, 0], seed=75), 3, flags=BAL)
    w = ragged_workload(lens=[700] * 70, seed=76)                            # more than 64 sequences: two scan blocks
    check_decode(mla, w, 2, flags=BAL, b_sel=[0, 1, 63, 64, 65, 69])
    w = ragged_workload(lens=[9000, 1, 130, 0] + [70] * 60, seed=78)         # many segments in one workgroup
    check_decode(mla, w, 1, flags=BAL, b_sel=[0, 1, 2, 3, 4, 63])
    w = ragged_workload(d_c=256, H=28, lens=[9000, 1, 130, 0] + [70] * 60, seed=79)
    check_decode(mla, w, 1, flags=BAL, b_sel=[0, 1, 2, 3, 4, 63])


@pytest.mark.parametrize("num_splits", [1, 2, 7, 32])
def test_decode_fp8_balanced_ragged(mla, num_splits):
    """fp8 cache under the balanced partition (the kernel that contracts the codes as they are, run
    segment by segment): ranges that cross sequence boundaries, short sequences sharing a workgroup,
    NaN-poisoned free pages, tail slots and scales."""
    check_decode(mla, ragged_workload(cache="fp8_e4m3", seed=81), num_splits, flags=BAL)


def test_decode_fp8_balanced_shapes(mla):
    check_decode(mla, ragged_workload(cache="fp8_e4m3", d_c=256, H=28, lens=[300, 1, 64, 0, 999, 4096], seed=82), 3, flags=BAL)
    check_decode(mla, ragged_workload(cache="fp8_e4m3", lens=[5000], seed=83), 16, flags=BAL)        # one sequence, many workgroups
    check_decode(mla, ragged_workload(cache="fp8_e4m3", lens=[3, 2, 1], seed=84), 64, flags=BAL)     # more workgroups than pages
    check_decode(mla, ragged_workload(cache="fp8_e4m3", lens=[0, 1, 0, 64, 5, 0], seed=85), 3, flags=BAL)
    w = ragged_workload(cache="fp8_e4m3", lens=[700] * 70, seed=86)                                  # two scan blocks
    check_decode(mla, w, 2, flags=BAL, b_sel=[0, 1, 63, 64, 65, 69])
    w = ragged_workload(cache="fp8_e4m3", lens=[9000, 1, 130, 0] + [70] * 60, seed=87)               # many segments in one workgroup
    check_decode(mla, w, 1, flags=BAL, b_sel=[0, 1, 2, 3, 4, 63])
    check_bench_step(mla, synth.config("C5", shrink=16), 8, flags=BAL)                               # with the fused tail


@pytest.mark.parametrize("cache", ["bf16", "fp8_e4m3"])
def test_decode_balanced_all_sequences_empty(mla, cache):
    import torch
    w = ragged_workload(lens=[0, 0, 0], seed=77, cache=cache)
    d = DeviceWorkload(w)
    o, lse = run_decode(mla, d, gpu_q_abs(mla, d), 2, BAL)
    torch.cuda.synchronize()
    assert not widen_gpu(o).any() and np.isneginf(widen_gpu(lse)).all()


def test_balanced_matches_uniform_and_fused_tail_call(mla):
    """Same inputs through both partitions: equal within fp32 merge rounding of the bf16 output;
    and the separate merge / tail calls accept the balanced workspace."""
    import torch
    w = ragged_workload(seed=78)
    d = DeviceWorkload(w)
    q_abs = gpu_q_abs(mla, d)
    o_u, lse_u = run_decode(mla, d, q_abs, 7, 0)
    o_b, lse_b = run_decode(mla, d, q_abs, 7, BAL)
    ws = mla.decode_paged(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                          num_splits=7, flags=mla.FLAG_SKIP_MERGE | BAL)
    o_m, lse_m = mla.merge_partials(ws, w.B, w.H, w.d_c, 7, q_abs.dtype, return_lse=True, flags=BAL)
    o_t, out_t, lse_t = mla.merge_out_proj(ws, d.W_UV, w.B, 7, return_lse=True, flags=BAL)
    torch.cuda.synchronize()
    assert max_abs_rel(widen_gpu(o_b), widen_gpu(o_u)) <= 2 ** -7
    assert lse_err(widen_gpu(lse_b), widen_gpu(lse_u)) <= 5e-3     # each sums bf16-rounded weights, chunked differently
    for o_x, lse_x in ((o_m, lse_m), (o_t, lse_t)):
        assert storage_bits(o_x).tobytes() == storage_bits(o_b).tobytes()
        assert storage_bits(lse_x).tobytes() == storage_bits(lse_b).tobytes()
    ref = oracle.out_proj(q_abs_storage(o_t), w.W_UV)
    assert max_abs_rel(widen_gpu(out_t), ref) <= TOL["bf16"]


def test_balanced_more_than_64_chunks_of_one_sequence(mla):
    """One long sequence among short ones with many workgroups: the plan gives it well over 64
    chunks (the merge walks them 64 at a time).  Decode + merge against the oracle, and the fused
    tail bit for bit the separate merge."""
    import torch
    w = ragged_workload(lens=[6000, 1, 130, 0], seed=79)
    check_decode(mla, w, 40, flags=BAL)          # 4 x 40 = 160 workgroups over 98 pages; sequence 0 holds 94 of them
    check_decode(mla, w, 25, flags=BAL)          # 4 x 25 x 4 (cut again to fill the chip) = 400 workgroups
    d = DeviceWorkload(w)
    q_abs = gpu_q_abs(mla, d)
    ws = mla.decode_paged(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                          num_splits=40, flags=mla.FLAG_SKIP_MERGE | BAL)
    o_m, lse_m = mla.merge_partials(ws, w.B, w.H, w.d_c, 40, q_abs.dtype, return_lse=True, flags=BAL)
    o_t, out_t, lse_t = mla.merge_out_proj(ws, d.W_UV, w.B, 40, return_lse=True, flags=BAL)
    torch.cuda.synchronize()
    plan_off = mla.decode_workspace_bytes(w.B, w.H, w.d_c, 40) - 256
    counts = ws[plan_off:plan_off + 8 * w.B].view(torch.int32).cpu().numpy().reshape(w.B, 2)[:, 1]
    assert counts[0] > 64 and counts[3] == 0, counts
    assert storage_bits(o_t).tobytes() == storage_bits(o_m).tobytes()
    assert storage_bits(lse_t).tobytes() == storage_bits(lse_m).tobytes()
    assert max_abs_rel(widen_gpu(out_t), oracle.out_proj(q_abs_storage(o_t), w.W_UV)) <= TOL["bf16"]


def test_balanced_needs_the_matrix_core_kernel(mla):
    w = synth.config("C1", shrink=4)          # fp32: portable kernel only
    d = DeviceWorkload(w)
    with pytest.raises(mla.MlaError) as e:
        run_decode(mla, d, gpu_q_abs(mla, d), 2, BAL)
    assert e.value.status == -3


# ------------------------------------------------------------- edge cases

def test_empty_and_single_token_sequences(mla):
    import torch
    w = ragged_workload(lens=[0, 1, 0, 64, 5], seed=12)
    for flags in (0, 1):
        d = DeviceWorkload(w)
        q_abs = gpu_q_abs(mla, d)
        o, lse = run_decode(mla, d, q_abs, 3, flags)
        torch.cuda.synchronize()
        o, lse = widen_gpu(o), widen_gpu(lse)
        assert (o[0] == 0).all() and (o[2] == 0).all()
        assert np.isneginf(lse[0]).all() and np.isneginf(lse[2]).all()
        ref_o, ref_lse = oracle_decode(w, q_abs_storage(q_abs))
        assert max_abs_rel(o, ref_o) <= 2e-2
        # one cached token: the output is that token's latent row (softmax over one element)
        row = oracle.widen(w.pool.reshape(-1, 576)[int(w.page_table[1, 0]) * 64])[:512]
        assert np.abs(o[1] - row[None, :]).max() <= 2 ** -8 * np.abs(row).max()
        assert lse_err(lse, ref_lse) <= 2e-2


def test_out_of_pool_page_ids_are_skipped_not_dereferenced(mla):
    """A page id outside [0, num_pages) inside the live range: its tokens are skipped."""
    import torch
    w = ragged_workload(lens=[256, 200], seed=13)
    bad = w.page_table.copy()
    bad[0, 1] = -1
    bad[1, 2] = w.num_pages + 7
    # oracle view: the same sequences with those pages removed
    keep0 = [0, 2, 3]
    keep1 = [0, 1, 3]
    w_ref = ragged_workload(lens=[256, 200], seed=13)
    pt = np.full_like(w.page_table, -1)
    pt[0, :3] = w.page_table[0, keep0]
    pt[1, :3] = w.page_table[1, keep1]
    # sequence 1: pages 0,1 full, page 3 has 200-192 = 8 rows -> 136 tokens
    lens_ref = np.array([192, 136], dtype=np.int32)
    for flags in (0, 1):
        d = DeviceWorkload(w)
        d.page_table = to_torch(bad, "i32")
        q_abs = gpu_q_abs(mla, d)
        o, _ = run_decode(mla, d, q_abs, 2, flags)
        torch.cuda.synchronize()
        ref_o, _ = oracle.decode_absorbed(q_abs_storage(q_abs), w.q_rope, w_ref.pool, None, pt,
                                          lens_ref, w.softmax_scale)
        assert max_abs_rel(widen_gpu(o), ref_o) <= 2e-2


def test_placement_invariance_and_determinism_bitwise(mla):
    """Same logical rows at different physical pages -> identical output bits; and
    the same call twice -> identical bits (fixed reduction order)."""
    import torch
    lens = [500, 64, 129]
    a = ragged_workload(lens=lens, seed=14)
    d = DeviceWorkload(a)
    q_abs = gpu_q_abs(mla, d)
    # rebuild the same rows under another placement: permute pages of the pool
    perm = synth.stream(99, 1).permutation(a.num_pages).astype(np.int32)   # new index of page p
    pool2 = np.empty_like(a.pool)
    pool2[perm] = a.pool
    pt2 = np.where(a.page_table >= 0, perm[np.maximum(a.page_table, 0)], -1).astype(np.int32)
    for flags in (0, 1):
        o1, l1 = run_decode(mla, d, q_abs, 3, flags)
        o1b, _ = run_decode(mla, d, q_abs, 3, flags)
        d2 = DeviceWorkload(a)
        d2.pool = to_torch(pool2, "bf16")
        d2.page_table = to_torch(pt2, "i32")
        o2, l2 = run_decode(mla, d2, q_abs, 3, flags)
        torch.cuda.synchronize()
        assert storage_bits(o1).tobytes() == storage_bits(o1b).tobytes()
        assert storage_bits(o1).tobytes() == storage_bits(o2).tobytes()
        assert storage_bits(l1).tobytes() == storage_bits(l2).tobytes()


def test_dominant_score_and_uniform_weights(mla):
    """Closed forms on the GPU: a zero query averages the rows; one score far above
    the rest selects its row (no overflow in the running softmax)."""
    import torch
    w = ragged_workload(lens=[300, 300], seed=15)
    d = DeviceWorkload(w)
    rows = oracle.widen(oracle.gather_paged(w.pool, w.page_table, w.seq_lens, 300).view(np.uint16))
    for flags in (0, 1):
        q0 = torch.zeros((2, 32, 512), dtype=torch.bfloat16, device="cuda")
        r0 = torch.zeros((2, 32, 64), dtype=torch.bfloat16, device="cuda")
        o, lse = mla.decode_paged(q0, r0, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                                  num_splits=2, return_lse=True, flags=flags)
        torch.cuda.synchronize()
        mean = rows[:, :, :512].mean(axis=1)
        assert np.abs(widen_gpu(o) - mean[:, None, :]).max() <= 2e-2 * np.abs(mean).max() + 1e-3
        assert np.abs(widen_gpu(lse) - math.log(300)).max() <= 1e-3
        # query = 40 x (row 217's latent): its score dominates all others by a wide margin
        target = rows[:, 217, :512]
        q1 = to_torch(synth.to_bf16_bits((40.0 * target[:, None, :].repeat(32, 1)).astype(np.float32)), "bf16")
        o, lse = mla.decode_paged(q1, r0, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                                  num_splits=2, return_lse=True, flags=flags)
        torch.cuda.synchronize()
        assert np.isfinite(widen_gpu(o)).all() and np.isfinite(widen_gpu(lse)).all()
        assert np.abs(widen_gpu(o) - target[:, None, :]).max() <= 2e-2 * np.abs(target).max()


@pytest.mark.parametrize("flags", [0, BAL])
@pytest.mark.parametrize("d_c", [512, 256])
def test_dominant_late_score_takes_the_careful_pass(mla, flags, d_c):
    """One chunk per sequence, and the one score that dominates sits in its seventh tile: the fixed
    reference of the fast pass (the first tile's maximum) is exceeded by far more than it
    tolerates, so the chunk is redone with a moving reference.  Both partitions, both latent widths;
    the result is the dominant row itself and the whole output matches the oracle."""
    import torch
    w = ragged_workload(d_c=d_c, lens=[300, 2000, 217], seed=16)
    d = DeviceWorkload(w)
    rows = oracle.widen(oracle.gather_paged(w.pool, w.page_table, w.seq_lens, 2000).view(np.uint16))
    target = np.stack([rows[0, 217, :d_c], rows[1, 1900, :d_c], rows[2, 216, :d_c]])
    q1 = to_torch(synth.to_bf16_bits((40.0 * target[:, None, :].repeat(32, 1)).astype(np.float32)), "bf16")
    r0 = torch.zeros((3, 32, 64), dtype=torch.bfloat16, device="cuda")
    o, lse = mla.decode_paged(q1, r0, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                              num_splits=1, return_lse=True, flags=flags)
    torch.cuda.synchronize()
    assert np.isfinite(widen_gpu(o)).all() and np.isfinite(widen_gpu(lse)).all()
    assert np.abs(widen_gpu(o) - target[:, None, :]).max() <= 2e-2 * np.abs(target).max()
    ref_o, ref_lse = oracle.decode_absorbed(q_abs_storage(q1), q_abs_storage(r0), w.pool, w.kv_scale,
                                            w.page_table, w.seq_lens, w.softmax_scale)
    assert max_abs_rel(widen_gpu(o), ref_o) <= TOL["bf16"]
    assert lse_err(widen_gpu(lse), ref_lse) <= 2e-2


def test_GQA_reduction_on_gpu(mla):
    """Sec. 4.1 at GPU size: H = 32 heads in g = 2 groups, d_head = 128, latent
    = [k_1 k_2 v_1 v_2] (d_c = 512), selector-identity W_UK / W_UV: the three
    calls reproduce textbook grouped-query attention."""
    import torch
    H, g, dh, d_c = 32, 2, 128, 512
    w = ragged_workload(lens=[200, 77], seed=16, softmax_scale=1 / math.sqrt(dh))
    Wk = np.zeros((H, dh, d_c), dtype=np.float32)
    Wv = np.zeros((H, d_c, dh), dtype=np.float32)
    for i in range(1, H + 1):
        kk = math.ceil(i / (H / g))
        Wk[i - 1, :, (kk - 1) * dh:kk * dh] = np.eye(dh)
        Wv[i - 1, (g + kk - 1) * dh:(g + kk) * dh, :] = np.eye(dh)
    d = DeviceWorkload(w)
    d.W_UK, d.W_UV = to_torch(synth.to_bf16_bits(Wk), "bf16"), to_torch(synth.to_bf16_bits(Wv), "bf16")
    zero_rope = torch.zeros_like(d.q_rope)
    q_abs = mla.absorb_q(d.q_nope, d.W_UK)
    o_lat = mla.decode_paged(q_abs, zero_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale, num_splits=2)
    out = widen_gpu(mla.out_proj(o_lat, d.W_UV))
    torch.cuda.synchronize()
    q = oracle.widen(w.q_nope)
    want = np.zeros((2, H, dh))
    dense = oracle.widen(oracle.gather_paged(w.pool, w.page_table, w.seq_lens, 200).view(np.uint16))
    for b, L in enumerate([200, 77]):
        rows = dense[b, :L]
        for i in range(H):
            kk = i // (H // g)
            K, V = rows[:, kk * dh:(kk + 1) * dh], rows[:, (g + kk) * dh:(g + kk + 1) * dh]
            s = (K @ q[b, i]) * w.softmax_scale
            p = np.exp(s - s.max())
            want[b, i] = (p / p.sum()) @ V
    assert max_abs_rel(out, want) <= 2e-2


# ---------------------------------- full-size configurations (sampled rows)

def test_step_C2_full_three_calls(mla):
    """Headline configuration at full size, launch configuration of the benchmark:
    batch 16, context 8192, bf16, random page placement, 16 chunks.  The oracle
    checks every sequence and head."""
    import torch
    w = synth.config("C2")
    d = DeviceWorkload(w)
    q_abs = mla.absorb_q(d.q_nope, d.W_UK)
    o_lat, lse = run_decode(mla, d, q_abs, w.num_splits)
    out = mla.out_proj(o_lat, d.W_UV)
    torch.cuda.synchronize()
    ref_q = oracle.absorb_q(w.q_nope, w.W_UK)
    assert max_abs_rel(widen_gpu(q_abs), ref_q) <= 2e-2
    ref_o, ref_lse = oracle_decode(w, q_abs_storage(q_abs))
    assert max_abs_rel(widen_gpu(o_lat), ref_o) <= 2e-2
    assert lse_err(widen_gpu(lse), ref_lse) <= 2e-2
    ref_out = oracle.out_proj(storage_bits(o_lat), w.W_UV)
    assert max_abs_rel(widen_gpu(out), ref_out) <= 2e-2
    # and the whole chain against the un-rounded fp64 chain
    chain = oracle.mla_step(w.q_nope, w.q_rope, w.W_UK, w.W_UV, w.pool, None, w.page_table,
                            w.seq_lens, w.softmax_scale)
    assert max_abs_rel(widen_gpu(out), chain["out"]) <= 2e-2
    # the benchmark's own call sequence: split-KV kernel with the partials left in the workspace,
    # then merge + W_UV in one kernel -- same o_lat / lse bits, out against the oracle
    ws = mla.decode_paged(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                          num_splits=w.num_splits, flags=mla.FLAG_SKIP_MERGE)
    o2, out2, lse2 = mla.merge_out_proj(ws, d.W_UV, w.B, w.num_splits, return_lse=True)
    torch.cuda.synchronize()
    assert storage_bits(o2).tobytes() == storage_bits(o_lat).tobytes()
    assert storage_bits(lse2).tobytes() == storage_bits(lse).tobytes()
    assert max_abs_rel(widen_gpu(out2), ref_out) <= 2e-2
    assert max_abs_rel(widen_gpu(out2), chain["out"]) <= 2e-2


def check_bench_step(mla, w, num_splits, flags=0):
    """The call sequence the benchmark times -- mla_absorb_q, mla_decode_paged with the partials left
    in the workspace (plus `flags`), mla_merge_out_proj -- at full size, every sequence and head
    against the oracle: q_abs, o_lat and lse from the stored q_abs, out from the stored o_lat, and
    out against the un-rounded fp64 chain.  Also the plain mla_decode_paged call (decode + merge)."""
    import torch
    d = DeviceWorkload(w)
    q_abs = mla.absorb_q(d.q_nope, d.W_UK)
    ws = mla.decode_paged(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                          num_splits=num_splits, kv_scale=d.kv_scale, flags=mla.FLAG_SKIP_MERGE | flags)
    o_lat, out, lse = mla.merge_out_proj(ws, d.W_UV, w.B, num_splits, return_lse=True, flags=flags)
    o_call, lse_call = run_decode(mla, d, q_abs, num_splits, flags)
    torch.cuda.synchronize()
    assert max_abs_rel(widen_gpu(q_abs), oracle.absorb_q(w.q_nope, w.W_UK)) <= 2e-2
    ref_o, ref_lse = oracle_decode(w, q_abs_storage(q_abs))
    for o_x, lse_x in ((o_lat, lse), (o_call, lse_call)):
        got = widen_gpu(o_x)
        assert np.isfinite(got).all()
        assert max_abs_rel(got, ref_o) <= 2e-2
        # per sequence as well: a short sequence must not hide behind the batch's largest value
        for b in range(w.B):
            assert max_abs_rel(got[b], ref_o[b]) <= 2e-2, f"sequence {b} (length {int(w.seq_lens[b])})"
        assert lse_err(widen_gpu(lse_x), ref_lse) <= 2e-2
    assert storage_bits(o_call).tobytes() == storage_bits(o_lat).tobytes()
    ref_out = oracle.out_proj(storage_bits(o_lat), w.W_UV)
    assert max_abs_rel(widen_gpu(out), ref_out) <= 2e-2
    chain = oracle.mla_step(w.q_nope, w.q_rope, w.W_UK, w.W_UV, w.pool, w.kv_scale, w.page_table,
                            w.seq_lens, w.softmax_scale)
    got_out = widen_gpu(out)
    assert np.isfinite(got_out).all()
    assert max_abs_rel(got_out, chain["out"]) <= 2e-2
    for b in range(w.B):
        assert max_abs_rel(got_out[b], chain["out"][b]) <= 2e-2, f"sequence {b} (length {int(w.seq_lens[b])})"


def test_step_C4_full_bench_sequence(mla):
    """Batch 128 x 4096 tokens, 28 heads, d_c 256, 2 chunks: all 128 sequences."""
    w = synth.config("C4")
    check_bench_step(mla, w, w.num_splits)


def test_step_C3_full_bench_sequence(mla):
    """64 sequences of 1024 .. 32768 tokens, balanced partition with 4 workgroups per sequence (the
    benchmark's launch) and the uniform partition with the configuration's 16 chunks: all sequences."""
    w = synth.config("C3")
    check_bench_step(mla, w, 4, flags=BAL)
    check_bench_step(mla, w, w.num_splits)


def test_step_C5_full_bench_sequence(mla):
    """fp8 cache, 4 sequences of 131072 tokens, 32 chunks: all four sequences."""
    w = synth.config("C5")
    check_bench_step(mla, w, w.num_splits)


@pytest.mark.parametrize("B,H,d_c,S,flags", [(128, 28, 256, 2, 0),      # the wide-batch shape: 16 batch rows per workgroup
                                             (137, 28, 256, 3, 0),      # last row group partly filled
                                             (130, 32, 512, 2, 0),      # 8 batch rows per workgroup, last group of 2
                                             (64, 32, 512, 4, 4),       # balanced partition, 64 sequences
                                             (70, 32, 512, 2, 4)])      # balanced, two scan blocks
def test_fused_tail_wide_batches(mla, B, H, d_c, S, flags):
    """mla_merge_out_proj on batches wide enough that a workgroup takes 8 or 16 batch rows (several
    tasks per wavefront): o_lat / lse bit for bit those of mla_merge_partials, out against the
    oracle's projection of the stored o_lat and against mla_out_proj."""
    import torch
    lens = [int(x) for x in (np.arange(B) * 37 % 190 + 1)]
    lens[3], lens[B - 1] = 0, 64
    w = synth.make_workload("wide-tail", B=B, H=H, d_head=128, d_c=d_c, d_rope=64, seq_lens=lens,
                            io_dtype="bf16", cache_dtype="bf16", placement="random", free_frac=0.1, seed=B + d_c)
    d = DeviceWorkload(w)
    q_abs = mla.absorb_q(d.q_nope, d.W_UK)
    ws = mla.decode_paged(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                          num_splits=S, flags=mla.FLAG_SKIP_MERGE | flags)
    o1, l1 = mla.merge_partials(ws, B, H, d_c, S, q_abs.dtype, return_lse=True, flags=flags)
    out1 = mla.out_proj(o1, d.W_UV)
    o2, out2, l2 = mla.merge_out_proj(ws, d.W_UV, B, S, return_lse=True, flags=flags)
    torch.cuda.synchronize()
    assert storage_bits(o1).tobytes() == storage_bits(o2).tobytes()
    assert storage_bits(l1).tobytes() == storage_bits(l2).tobytes()
    ref_o, ref_lse = oracle_decode(w, q_abs_storage(q_abs))
    assert max_abs_rel(widen_gpu(o2), ref_o) <= 2e-2
    assert lse_err(widen_gpu(l2), ref_lse) <= 2e-2
    ref = oracle.out_proj(storage_bits(o2), w.W_UV)
    got = widen_gpu(out2)
    assert max_abs_rel(got, ref) <= 2e-2
    for b in range(B):
        assert max_abs_rel(got[b], ref[b]) <= 2e-2, f"batch row {b}"
    assert max_abs_rel(got, widen_gpu(out1)) <= 1e-2


# ------------------------------------------------------------ cache append

def _append_inputs(cache_dtype, D, seed, lens=(0, 63, 64, 1000, 4095), page_size=64):
    io = "f32" if cache_dtype == "f32" else "bf16"
    w = synth.make_workload("append", B=len(lens), H=4, d_head=128, d_c=512, d_rope=64, seq_lens=list(lens),
                            io_dtype=io, cache_dtype=cache_dtype, placement="random", free_frac=0.3,
                            max_pages_per_seq=65, seed=seed)
    pt = w.page_table.copy()
    used = set(pt[pt >= 0].tolist())
    free = [p for p in range(w.pool.shape[0]) if p not in used]
    for b, L in enumerate(lens):            # the page the new token goes to must be in the table
        if pt[b, L // page_size] < 0:
            pt[b, L // page_size] = free.pop()
    r = synth.stream(seed, 91)
    x = synth.store(synth.normal(r, (len(lens), D)), io)
    W = synth.store(synth.normal(r, (D, 576), 1 / math.sqrt(D)), io)
    return w, pt, x, W, io


def _decoded_rows(pool_np, scale_np, pt, pos):
    rows = []
    for b in range(len(pos)):
        p, s = pt[b, pos[b] // 64], pos[b] % 64
        if pool_np.dtype == np.uint8:
            rows.append(np.array([oracle.widen_e4m3_code(int(c)) for c in pool_np[p, s]]) * float(scale_np[p, s]))
        else:
            rows.append(oracle.widen(pool_np[p, s]))
    return np.stack(rows)


@pytest.mark.parametrize("cache_dtype,D", [("bf16", 4096), ("bf16", 1024), ("bf16", 200), ("fp8_e4m3", 4096),
                                           ("f32", 1024), ("f32", 96)])
def test_cache_append_matches_oracle(mla, cache_dtype, D):
    """New rows against the fp64 oracle rows (one rounding to the cache dtype apart); every other
    byte of the pool and of the scale pool untouched."""
    import torch
    w, pt, x, W, io = _append_inputs(cache_dtype, D, seed=61)
    d = DeviceWorkload(w)
    pool = d.pool.clone()
    scale = None if d.kv_scale is None else d.kv_scale.clone()
    pos = w.seq_lens.copy()
    mla.cache_append(to_torch(x, io), to_torch(W, io), pool, to_torch(pt, "i32"), to_torch(pos, "i32"), 512,
                     kv_scale=scale)
    torch.cuda.synchronize()
    ref_pool, ref_scale, rows = oracle.cache_append(x, W, w.pool, w.kv_scale, pt, pos, 512)
    got_pool = storage_bits(pool) if cache_dtype != "f32" else pool.cpu().numpy()
    got_scale = None if scale is None else scale.cpu().numpy()
    got = _decoded_rows(got_pool, got_scale, pt, pos)
    if cache_dtype == "f32":
        assert max_abs_rel(got, rows) <= 1e-5
    elif cache_dtype == "bf16":
        assert max_abs_rel(got, rows) <= 2 ** -8        # one bf16 rounding (2^-9) and fp32 accumulation
        assert (np.abs(got - rows) <= 2 ** -8 * np.abs(rows) + 1e-6).all()
    else:
        sref = np.array([ref_scale[pt[b, pos[b] // 64], pos[b] % 64] for b in range(w.B)])
        sgot = np.array([got_scale[pt[b, pos[b] // 64], pos[b] % 64] for b in range(w.B)])
        assert np.abs(sgot - sref).max() <= 1e-5 * sref.max()
        assert (np.abs(got - rows) <= 2 ** -4 * np.abs(rows) + sgot[:, None] * 2 ** -9 * 1.01).all()   # half a step
        ref_codes = np.stack([ref_pool[pt[b, pos[b] // 64], pos[b] % 64] for b in range(w.B)])
        got_codes = np.stack([got_pool[pt[b, pos[b] // 64], pos[b] % 64] for b in range(w.B)])
        assert (ref_codes != got_codes).mean() < 0.02   # only values within rounding of a code boundary differ
    changed = np.zeros(w.pool.shape[:2], dtype=bool)
    for b in range(w.B):
        changed[pt[b, pos[b] // 64], pos[b] % 64] = True
    a = w.pool.view(np.uint8).reshape(*w.pool.shape[:2], -1)
    g = np.ascontiguousarray(got_pool).view(np.uint8).reshape(*w.pool.shape[:2], -1)
    assert (a[~changed] == g[~changed]).all()
    if got_scale is not None:
        assert np.array_equal(got_scale[~changed], w.kv_scale[~changed], equal_nan=True)


@pytest.mark.parametrize("cache_dtype", ["bf16", "fp8_e4m3", "f32"])
def test_cache_append_encoders_bitwise(mla, cache_dtype):
    """x = 64 e_k makes the projection exact (one product per column) and position 0 makes the
    rotation the identity: the stored row must then equal the oracle's bit for bit (bf16 rounding,
    e4m3 codes and per-token scale take their decisions on the same fp32 values)."""
    import torch
    w, pt, x, W, io = _append_inputs(cache_dtype, 256, seed=62, lens=(3, 3, 3))   # position 0 is overwritten
    xf = np.zeros((3, 256), dtype=np.float32)
    xf[0, 5], xf[1, 200], xf[2, 77] = 64.0, -0.5, 1024.0
    x = synth.store(xf, io)
    Wf = synth.normal(synth.stream(62, 5), (256, 576), 37.0)      # spread over many binades
    Wf[200, :8] = 0.0
    Wf[77, 100:108] = [448.0, 449.0, 1e-3, -1e-3, 3.0e-3, 0.0, -0.0, 464.0]
    W = synth.store(Wf, io)
    d = DeviceWorkload(w)
    pool = d.pool.clone()
    scale = None if d.kv_scale is None else d.kv_scale.clone()
    pos = np.zeros(3, dtype=np.int32)
    mla.cache_append(to_torch(x, io), to_torch(W, io), pool, to_torch(pt, "i32"), to_torch(pos, "i32"), 512,
                     kv_scale=scale)
    torch.cuda.synchronize()
    ref_pool, ref_scale, _ = oracle.cache_append(x, W, w.pool, w.kv_scale, pt, pos, 512)
    got_pool = storage_bits(pool) if cache_dtype != "f32" else pool.cpu().numpy()
    for b in range(3):
        p = pt[b, 0]
        assert np.array_equal(np.ascontiguousarray(got_pool[p, 0]).view(np.uint8),
                              np.ascontiguousarray(ref_pool[p, 0]).view(np.uint8)), (cache_dtype, b)
        if scale is not None:
            assert scale.cpu().numpy()[p, 0] == ref_scale[p, 0]


def test_cache_append_then_decode(mla):
    """Append on the GPU, then decode over seq_len + 1 tokens: equals the oracle's decode over the
    oracle-appended cache (the new token is part of the softmax)."""
    import torch
    w, pt, x, W, io = _append_inputs("bf16", 1024, seed=63, lens=(0, 63, 64, 700, 2048))
    d = DeviceWorkload(w)
    pool = d.pool.clone()
    pos = w.seq_lens.copy()
    mla.cache_append(to_torch(x, io), to_torch(W, io), pool, to_torch(pt, "i32"), to_torch(pos, "i32"), 512)
    q_abs = gpu_q_abs(mla, d)
    lens1 = (w.seq_lens + 1).astype(np.int32)
    o, lse = mla.decode_paged(q_abs, d.q_rope, pool, to_torch(pt, "i32"), to_torch(lens1, "i32"), w.softmax_scale,
                              num_splits=4, return_lse=True)
    torch.cuda.synchronize()
    ref_pool, _, _ = oracle.cache_append(x, W, w.pool, None, pt, pos, 512)
    ref_o, ref_lse = oracle.decode_absorbed(q_abs_storage(q_abs), w.q_rope, ref_pool, None, pt, lens1, w.softmax_scale)
    assert max_abs_rel(widen_gpu(o), ref_o) <= TOL["bf16"]
    assert lse_err(widen_gpu(lse), ref_lse) <= 2e-2


def test_cache_append_skips_bad_positions(mla):
    import torch
    w, pt, x, W, io = _append_inputs("bf16", 256, seed=64, lens=(5, 70, 130))
    pos = np.array([65 * 64, 70, 130], dtype=np.int32)       # first: one past the table
    pt2 = pt.copy(); pt2[1, 1] = w.pool.shape[0] + 3; pt2[2, 2] = -1
    d = DeviceWorkload(w)
    pool = d.pool.clone()
    mla.cache_append(to_torch(x, io), to_torch(W, io), pool, to_torch(pt2, "i32"), to_torch(pos, "i32"), 512)
    torch.cuda.synchronize()
    assert np.array_equal(storage_bits(pool), w.pool)


# ------------------------------------------------------------- graph capture

def test_step_captured_in_a_hip_graph(mla):
    """The library only enqueues kernels on the current stream and allocates nothing, so the whole
    step can be captured; every replay (with eager work and synchronisation in between, and with
    the inputs changed between replays) must give the bits of the eager run on the same inputs."""
    import torch
    w = synth.config("C2", shrink=8)
    d = DeviceWorkload(w)
    B, H, d_c, S = w.B, w.H, w.d_c, w.num_splits
    q_nope = d.q_nope.clone()
    q_abs = torch.empty((B, H, d_c), dtype=torch.bfloat16, device="cuda")
    o_lat = torch.empty_like(q_abs)
    out = torch.empty((B, H, w.d_head), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(mla.decode_workspace_bytes(B, H, d_c, S), dtype=torch.uint8, device="cuda")

    def step():
        mla.absorb_q(q_nope, d.W_UK, out=q_abs)
        mla.decode_paged(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                         num_splits=S, workspace=ws, flags=mla.FLAG_SKIP_MERGE)
        mla.merge_out_proj(ws, d.W_UV, B, S, o_lat=o_lat, out=out)

    step()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        q_nope.copy_(torch.roll(d.q_nope, shifts=rep, dims=1))       # new inputs, same buffers
        step()
        torch.cuda.synchronize()
        want_o, want_out = storage_bits(o_lat).copy(), storage_bits(out).copy()
        o_lat.zero_(); out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(storage_bits(o_lat), want_o), f"replay {rep}: o_lat differs"
        assert np.array_equal(storage_bits(out), want_out), f"replay {rep}: out differs"
    ref = oracle.mla_step(w.q_nope, w.q_rope, w.W_UK, w.W_UV, w.pool, None, w.page_table, w.seq_lens, w.softmax_scale)
    q_nope.copy_(d.q_nope)
    graph.replay()
    torch.cuda.synchronize()
    assert max_abs_rel(widen_gpu(out), ref["out"]) <= TOL["bf16"]


# ------------------------------------------------------- seeded random sweep

def test_random_shapes_partitions_and_caches(mla):
    """Forty seeded random cases: batch 1..9, heads 1..32, d_c 256 / 512, lengths 0..3000 (many
    of them around page and tile boundaries), bf16 / fp8 caches, 1..40 chunks, both partitions,
    both kernels (the portable one with the uniform partition)."""
    rng = np.random.default_rng(2024)
    special = [0, 1, 31, 32, 33, 63, 64, 65, 95, 96, 127, 128, 129, 191, 192, 193]
    for case in range(40):
        B = int(rng.integers(1, 10))
        H = int(rng.choice([1, 5, 16, 17, 28, 32]))
        d_c = int(rng.choice([256, 512]))
        lens = [int(rng.choice(special)) if rng.random() < 0.5 else int(rng.integers(0, 3000)) for _ in range(B)]
        cache = "fp8_e4m3" if rng.random() < 0.35 else "bf16"
        S = int(rng.integers(1, 41))
        flags = int(rng.choice([0, 0, 4, 4, 1]))
        w = synth.make_workload(f"rand{case}", B=B, H=H, d_head=128, d_c=d_c, d_rope=64, seq_lens=lens,
                                io_dtype="bf16", cache_dtype=cache, placement="random", free_frac=0.25,
                                seed=1000 + case)
        try:
            check_decode(mla, w, S, flags=flags)
        except AssertionError as e:
            raise AssertionError(f"case {case}: B={B} H={H} d_c={d_c} lens={lens} cache={cache} S={S} flags={flags}: {e}")


# ----------------------------------------------- several query tokens per sequence

def check_multi(mla, w, T, num_splits, flags=0, tol=None, fused_tail=False):
    """q_len = T query tokens per sequence against the oracle's Eq. "mqa" with one upper limit of
    the sum per token; returns what the GPU produced."""
    import torch
    d = DeviceWorkload(w)
    qn, qr = synth.multi_queries(w, T)
    qn_t, qr_t = to_torch(qn, w.io_dtype), to_torch(qr, w.io_dtype)
    q_abs = mla.absorb_q(qn_t.view(w.B * T, w.H, w.d_head), d.W_UK).view(w.B, T, w.H, w.d_c)
    out = None
    if fused_tail:
        ws = mla.decode_paged_multi(q_abs, qr_t, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                                    num_splits=num_splits, kv_scale=d.kv_scale, flags=flags | mla.FLAG_SKIP_MERGE)
        o, out, lse = mla.merge_out_proj_multi(ws, d.W_UV, w.B, T, num_splits, return_lse=True, flags=flags)
    else:
        o, lse = mla.decode_paged_multi(q_abs, qr_t, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                                        num_splits=num_splits, kv_scale=d.kv_scale, return_lse=True, flags=flags)
    torch.cuda.synchronize()
    ref_o, ref_lse = oracle.decode_absorbed_multi(q_abs_storage(q_abs), qr, w.pool, w.kv_scale, w.page_table,
                                                  w.seq_lens, w.softmax_scale)
    got_o, got_lse = widen_gpu(o), widen_gpu(lse)
    assert got_o.shape == ref_o.shape and np.isfinite(got_o).all()
    tol = tol or TOL[w.io_dtype]
    err = max_abs_rel(got_o, ref_o)
    assert err <= tol, f"{w.name} q_len={T} splits={num_splits} flags={flags}: o_lat err {err:.3e} > {tol}"
    assert lse_err(got_lse, ref_lse) <= (1e-4 if w.io_dtype == "f32" else 2e-2)
    if out is not None:
        ref_out = oracle.out_proj(q_abs_storage(o).reshape(w.B * T, w.H, w.d_c), w.W_UV).reshape(w.B, T, w.H, w.d_head)
        assert max_abs_rel(widen_gpu(out), ref_out) <= tol
    return o, lse


@pytest.mark.parametrize("T", [2, 3])
def test_multi_token_fp32_portable(mla, T):
    """fp32 cache and io (portable kernel), C1 shape and a ragged batch."""
    check_multi(mla, synth.config("C1"), T, 4)
    check_multi(mla, ragged_workload(cache="f32", io="f32", lens=[130, 64, 7, 1, 65], seed=31), T, 3)


@pytest.mark.parametrize("T,flags", [(2, 0), (3, 0), (4, 0), (2, 1), (3, BAL)])
def test_multi_token_bf16_ragged(mla, T, flags):
    """Matrix-core kernel (64, 96, 128 query rows: 2 to 4 groups of 32), portable kernel and the
    balanced partition on lengths around the tile, page and chunk boundaries: the newest T rows
    straddle them, so the per-token limits fall in different tiles, pages and chunks."""
    w = ragged_workload(lens=[64 * 3 + 1, 64 * 2 + 33, 32, 129, 64, 2, 1000, 31], seed=32)
    check_multi(mla, w, T, 4, flags)
    check_multi(mla, w, T, 1, flags)
    check_multi(mla, w, T, 16, flags)


def test_multi_token_few_heads_share_a_group(mla):
    """5 heads x 3 tokens = 15 rows and 8 heads x 4 tokens = 32 rows in one group of 32: lanes of
    one wavefront belong to different query tokens."""
    check_multi(mla, ragged_workload(H=5, lens=[200, 66, 3, 64], seed=33), 3, 2)
    check_multi(mla, ragged_workload(H=8, lens=[200, 66, 3, 64], seed=34), 4, 3)
    check_multi(mla, ragged_workload(H=28, d_c=256, lens=[500, 65, 4096 // 4], seed=35), 2, 2)     # 56 rows: 32 + 24


def test_multi_token_fewer_rows_than_tokens_and_empty(mla):
    """seq_len < q_len: the tokens before position 0 see nothing (zeros, -inf); seq_len 0."""
    w = ragged_workload(lens=[2, 0, 3, 70], seed=36)
    o, lse = check_multi(mla, w, 4, 2)
    o, lse = widen_gpu(o), widen_gpu(lse)
    assert not o[0, :2].any() and np.isneginf(lse[0, :2]).all() and np.isfinite(lse[0, 2:]).all()
    assert not o[1].any() and np.isneginf(lse[1]).all()
    assert np.isneginf(lse[2, 0]).all() and np.isfinite(lse[2, 1:]).all()
    check_multi(mla, w, 4, 2, flags=1)


def test_multi_token_fp8_cache_and_fused_tail(mla):
    check_multi(mla, synth.config("C5", shrink=64), 2, 8)
    check_multi(mla, synth.config("C5", shrink=64), 2, 8, flags=1)
    # fp8 under the balanced partition, several groups of 32 query rows per segment
    check_multi(mla, synth.config("C5", shrink=64), 2, 8, flags=BAL)
    check_multi(mla, ragged_workload(cache="fp8_e4m3", lens=[300, 2, 64, 0, 999, 65], seed=38), 3, 3, flags=BAL, fused_tail=True)
    w = synth.config("C2", shrink=8)
    check_multi(mla, w, 2, 4, fused_tail=True)                 # one kernel for merge + W_UV
    check_multi(mla, w, 3, 4, flags=BAL, fused_tail=True)      # balanced: merge, then the projection
    check_multi(mla, ragged_workload(cache="f32", io="f32", lens=[130, 7], seed=37), 2, 2, fused_tail=True)


@pytest.mark.parametrize("H,exact", [(8, True), (32, False)])
def test_multi_token_last_token_is_the_single_token_decode(mla, H, exact):
    """Token q_len - 1 sees the whole sequence: its result must equal the one-token call on the same
    query.  16 query rows run on the same kernel as one token does (same chunks, same order of
    operations per query row): bit for bit.  64 rows run on the 64-row kernel, which sums in another
    order: equal within the rounding of the bf16 output."""
    import torch
    w = ragged_workload(H=H, lens=[300, 64, 129], seed=38)
    T = 2
    d = DeviceWorkload(w)
    qn, qr = synth.multi_queries(w, T)
    qn_t, qr_t = to_torch(qn, "bf16"), to_torch(qr, "bf16")
    q_abs = mla.absorb_q(qn_t.view(w.B * T, w.H, w.d_head), d.W_UK).view(w.B, T, w.H, w.d_c)
    o, lse = mla.decode_paged_multi(q_abs, qr_t, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                                    num_splits=4, return_lse=True)
    o1, lse1 = mla.decode_paged(q_abs[:, T - 1].contiguous(), qr_t[:, T - 1].contiguous(), d.pool, d.page_table,
                                d.seq_lens, w.softmax_scale, num_splits=4, return_lse=True)
    torch.cuda.synchronize()
    if exact:
        assert storage_bits(o[:, T - 1]).tobytes() == storage_bits(o1).tobytes()
        assert storage_bits(lse[:, T - 1]).tobytes() == storage_bits(lse1).tobytes()
    else:
        assert max_abs_rel(widen_gpu(o[:, T - 1]), widen_gpu(o1)) <= 2 ** -7
        assert lse_err(widen_gpu(lse[:, T - 1]), widen_gpu(lse1)) <= 5e-3


def test_multi_token_dominant_late_score_takes_the_careful_route(mla):
    """A score far above the first tile's maximum, met late in the chunk, sends the 64-row kernel
    through its second route (exact maxima first, then the accumulation): the query of token 0 is
    40 x the latent of row 217, that of token 1 is 40 x the latent of the newest row (which token 0
    must not see), both checked against the oracle and against the closed form (the dominant row)."""
    import torch
    L, T = 300, 2
    w = ragged_workload(lens=[L, L], seed=39)
    d = DeviceWorkload(w)
    rows = oracle.widen(oracle.gather_paged(w.pool, w.page_table, w.seq_lens, L).view(np.uint16))
    q = np.zeros((2, T, 32, 512), dtype=np.float32)
    q[:, 0] = 40.0 * rows[:, 217, None, :512]
    q[:, 1] = 40.0 * rows[:, L - 1, None, :512]
    q_bits = synth.to_bf16_bits(q)
    q1 = to_torch(q_bits, "bf16")
    r0 = torch.zeros((2, T, 32, 64), dtype=torch.bfloat16, device="cuda")
    for splits in (1, 2):
        o, lse = mla.decode_paged_multi(q1, r0, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                                        num_splits=splits, return_lse=True)
        torch.cuda.synchronize()
        got, got_lse = widen_gpu(o), widen_gpu(lse)
        assert np.isfinite(got).all() and np.isfinite(got_lse).all()
        ref_o, ref_lse = oracle.decode_absorbed_multi(q_bits, np.zeros((2, T, 32, 64), dtype=np.float32).view(np.float32),
                                                      w.pool, None, w.page_table, w.seq_lens, w.softmax_scale)
        assert max_abs_rel(got, ref_o) <= TOL["bf16"]
        assert np.abs(got_lse - ref_lse).max() <= 2e-2 * np.abs(ref_lse).max()
        assert np.abs(got[:, 0] - rows[:, 217, None, :512]).max() <= 2e-2 * np.abs(rows[:, 217, :512]).max()
        assert np.abs(got[:, 1] - rows[:, L - 1, None, :512]).max() <= 2e-2 * np.abs(rows[:, L - 1, :512]).max()


def test_multi_token_random_sweep(mla):
    """Thirty seeded random cases with 2..5 query tokens: batch 1..6, heads 1..40 (so 2..200 query
    rows: one to four groups on either matrix-core kernel, lanes of mixed tokens), d_c 256 / 512,
    lengths 0..2000 around page, tile and chunk boundaries and below q_len, bf16 / fp8 caches,
    1..24 chunks, both partitions, both kernel families, with and without the fused tail."""
    rng = np.random.default_rng(4048)
    special = [0, 1, 2, 3, 31, 32, 33, 34, 63, 64, 65, 66, 67, 127, 128, 129, 130, 192, 193, 194]
    for case in range(30):
        B = int(rng.integers(1, 7))
        H = int(rng.choice([1, 5, 8, 16, 17, 28, 32, 40]))
        T = int(rng.integers(2, 6))
        d_c = int(rng.choice([256, 512]))
        lens = [int(rng.choice(special)) if rng.random() < 0.6 else int(rng.integers(0, 2000)) for _ in range(B)]
        cache = "fp8_e4m3" if rng.random() < 0.3 else "bf16"
        S = int(rng.integers(1, 25))
        flags = int(rng.choice([0, 0, 0, 4, 1]))
        fused = bool(rng.random() < 0.4)
        w = synth.make_workload(f"mrand{case}", B=B, H=H, d_head=128, d_c=d_c, d_rope=64, seq_lens=lens,
                                io_dtype="bf16", cache_dtype=cache, placement="random", free_frac=0.25,
                                seed=3000 + case)
        try:
            check_multi(mla, w, T, S, flags=flags, fused_tail=fused)
        except AssertionError as e:
            raise AssertionError(f"case {case}: B={B} H={H} T={T} d_c={d_c} lens={lens} cache={cache} S={S} "
                                 f"flags={flags} fused={fused}: {e}")


# ----------------------------------------------- prefill in the MHA paradigm

def check_prefill(mla, w, T, tol=None):
    """mla_prefill_mha for the T newest tokens of every sequence against the oracle's Eq. "mha"
    (keys and values materialised per head in fp64); returns the GPU output."""
    import torch
    d = DeviceWorkload(w)
    qn, qr = synth.multi_queries(w, T)
    qn_t, qr_t = to_torch(qn, w.io_dtype), to_torch(qr, w.io_dtype)
    out, lse = mla.prefill_mha(qn_t, qr_t, d.W_UK, d.W_UV, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                               return_lse=True)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.prefill_explicit(qn, qr, w.W_UK, w.W_UV, w.pool, None, w.page_table, w.seq_lens,
                                           w.softmax_scale, w.d_c)
    got, got_lse = widen_gpu(out), widen_gpu(lse)
    assert got.shape == ref.shape and np.isfinite(got).all()
    err = max_abs_rel(got, ref)
    tol = tol or TOL["bf16"]
    assert err <= tol, f"{w.name} q_len={T}: out err {err:.3e} > {tol}"
    assert lse_err(got_lse, ref_lse) <= 2e-2
    return out, lse, qn_t, qr_t, d


@pytest.mark.parametrize("T", [1, 64, 200, 300])
def test_prefill_mha_ragged(mla, T):
    """Lengths around tile and page boundaries; q_len from one token to the whole prompt of the
    longest sequence (shorter sequences then have tokens before position 0: zeros, -inf);
    one to five groups of 64 query rows per (sequence, head)."""
    w = ragged_workload(H=8, lens=[300, 64, 129, 1, 65, 33], seed=51)
    check_prefill(mla, w, T)


def test_prefill_mha_whole_prompts_32_heads_and_C4_shape(mla):
    w = ragged_workload(H=32, lens=[256, 192], seed=52)
    check_prefill(mla, w, 256)
    w4 = ragged_workload(H=28, d_c=256, lens=[150, 70, 2], seed=53)
    check_prefill(mla, w4, 150)


def test_prefill_mha_matches_the_absorbed_calls_on_the_gpu(mla):
    """Same inputs through both paradigms on the GPU (Sec. 3.3: the Absorb operation changes the
    order of the products, not the function): equal within the bf16 roundings of either route."""
    import torch
    w = ragged_workload(H=16, lens=[200, 96, 40], seed=54)
    T = 40
    out, lse, qn_t, qr_t, d = check_prefill(mla, w, T)
    q_abs = mla.absorb_q(qn_t.view(w.B * T, w.H, w.d_head), d.W_UK).view(w.B, T, w.H, w.d_c)
    o_lat, lse_a = mla.decode_paged_multi(q_abs, qr_t, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                                          num_splits=2, return_lse=True)
    out_a = mla.out_proj(o_lat.view(w.B * T, w.H, w.d_c), d.W_UV).view(w.B, T, w.H, w.d_head)
    torch.cuda.synchronize()
    assert max_abs_rel(widen_gpu(out), widen_gpu(out_a)) <= 2e-2
    assert lse_err(widen_gpu(lse), widen_gpu(lse_a)) <= 2e-2


def test_prefill_mha_empty_sequence_and_dominant_late_key(mla):
    """seq_len 0 gives zeros and -inf.  A key whose score lies far above the first tile's maximum,
    met late, sends the attention kernel through its second route (exact maxima first): queries
    built from that key's own materialised k = W_UK c, checked against the oracle."""
    import torch
    w = ragged_workload(H=4, lens=[0, 200, 70], seed=55)
    out, lse, _, _, _ = check_prefill(mla, w, 70)
    assert not widen_gpu(out)[0].any() and np.isneginf(widen_gpu(lse)[0]).all()
    # queries of every token = 10 x k_nope of row 150 of sequence 1 (row 50 of sequence 2), per head: its score lies
    # ~90 powers of two above the first tile's maximum (more would only amplify the bf16 rounding of the keys)
    T = 70
    d = DeviceWorkload(w)
    rows = oracle.widen(oracle.gather_paged(w.pool, w.page_table, w.seq_lens, 200).view(np.uint16))   # [B, 200, 576]
    Wk = oracle.widen(w.W_UK)                                                                         # [H, 128, 512]
    qn = np.zeros((3, T, 4, 128), dtype=np.float32)
    qn[1] = 10.0 * np.einsum("hdc,c->hd", Wk, rows[1, 150, :512])[None]
    qn[2] = 10.0 * np.einsum("hdc,c->hd", Wk, rows[2, 50, :512])[None]
    qn_bits = synth.to_bf16_bits(qn)
    qr = np.zeros((3, T, 4, 64), dtype=np.float32)
    out, lse = mla.prefill_mha(to_torch(qn_bits, "bf16"), to_torch(synth.to_bf16_bits(qr), "bf16"), d.W_UK, d.W_UV,
                               d.pool, d.page_table, d.seq_lens, w.softmax_scale, return_lse=True)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.prefill_explicit(qn_bits, synth.to_bf16_bits(qr), w.W_UK, w.W_UV, w.pool, None, w.page_table,
                                           w.seq_lens, w.softmax_scale, w.d_c)
    got = widen_gpu(out)
    assert np.isfinite(got).all()
    assert max_abs_rel(got, ref) <= TOL["bf16"]
    fin = np.isfinite(ref_lse)
    assert (np.isfinite(widen_gpu(lse)) == fin).all()
    assert np.abs(widen_gpu(lse)[fin] - ref_lse[fin]).max() <= 2e-2 * np.abs(ref_lse[fin]).max()


def test_prefill_mha_random_sweep(mla):
    """Twenty seeded random prefill cases: batch 1..4, heads 1..32, d_c 256 / 512, lengths 0..700 around
    tile, page and query-group boundaries, q_len from 1 to beyond the longest sequence."""
    rng = np.random.default_rng(777)
    special = [0, 1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 130, 191, 192, 193, 255, 256, 257]
    for case in range(20):
        B = int(rng.integers(1, 5))
        H = int(rng.choice([1, 3, 8, 16, 28, 32]))
        d_c = int(rng.choice([256, 512]))
        lens = [int(rng.choice(special)) if rng.random() < 0.6 else int(rng.integers(0, 700)) for _ in range(B)]
        T = int(rng.choice([1, 2, 17, 64, 127, 128, 129, 300, max(1, max(lens)), max(lens) + 5]))
        w = synth.make_workload(f"prand{case}", B=B, H=H, d_head=128, d_c=d_c, d_rope=64, seq_lens=lens,
                                io_dtype="bf16", cache_dtype="bf16", placement="random", free_frac=0.25,
                                seed=5000 + case)
        try:
            check_prefill(mla, w, T)
        except AssertionError as e:
            raise AssertionError(f"case {case}: B={B} H={H} d_c={d_c} lens={lens} T={T}: {e}")


# ----------------------------------------------- the new calls at full size

def test_multi_token_C2_full_fused_tail(mla):
    """Headline cache at full size (batch 16, context 8192, 16 chunks), two query tokens per sequence,
    the call sequence bench.py --q-len 2 times: 64-row kernel with the partials left in the
    workspace, then merge + W_UV in one kernel.  Every sequence, token and head against the oracle."""
    w = synth.config("C2")
    check_multi(mla, w, 2, w.num_splits, fused_tail=True)


def test_prefill_mha_2048_token_prompts(mla):
    """Whole prompts of 2048 and 2000 tokens, 32 heads: 16 groups of 128 queries per (sequence, head),
    64 key tiles for the last group; every row against the oracle."""
    w = ragged_workload(H=32, lens=[2048, 2000], seed=56)
    check_prefill(mla, w, 2048)
