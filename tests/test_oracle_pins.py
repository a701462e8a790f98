"""Pins for the CPU oracle: it is checked against things other than itself.

Every test states the passage or the mathematics that fixes the expected
value.  Expected values are computed inside the tests with separately written
numpy / pure-Python code (textbook attention, scalar brute force, closed
forms), never with the oracle's own routines.
"""
import math
from pathlib import Path

import numpy as np
import pytest

import oracle
from workloads import synth

GOLDEN = Path(__file__).parent / "golden"
RNG = np.random.default_rng(1234)


# ---------------------------------------------------------------- helpers

def dense_cache(c_kv, k_rope, page_size=4, shuffle=True, extra_pages=1, seed=0):
    """Pack per-sequence fp64/fp32 rows into a float32 paged pool.

    c_kv: list of [L_b, d_c]; k_rope: list of [L_b, d_rope].  Returns
    (pool f32, page_table, seq_lens).  Unused slots hold NaN."""
    B = len(c_kv)
    d_c = c_kv[0].shape[1]
    d_rope = k_rope[0].shape[1]
    lens = np.array([x.shape[0] for x in c_kv], dtype=np.int32)
    npg = (lens + page_size - 1) // page_size
    total = int(npg.sum()) + extra_pages
    order = np.random.default_rng(seed).permutation(total) if shuffle else np.arange(total)
    pool = np.full((total, page_size, d_c + d_rope), np.nan, dtype=np.float32)
    table = np.full((B, max(1, int(npg.max()))), -1, dtype=np.int32)
    cur = 0
    for b in range(B):
        pages = order[cur:cur + npg[b]]
        cur += npg[b]
        table[b, :npg[b]] = pages
        for j in range(lens[b]):
            pool[pages[j // page_size], j % page_size, :d_c] = c_kv[b][j]
            pool[pages[j // page_size], j % page_size, d_c:] = k_rope[b][j]
    return pool, table, lens


def f32(x):
    """Round to float32 and back so stored inputs are exactly representable."""
    return np.asarray(x, dtype=np.float32).astype(np.float64)


def textbook_attention(q, K, V, scale):
    """softmax(q K^T * scale) V for one head; q [d], K [L,d], V [L,dv]."""
    s = (K @ q) * scale
    s = s - s.max()
    p = np.exp(s)
    p /= p.sum()
    return p @ V, p


def random_case(B=2, H=3, d_head=4, d_c=6, d_rope=2, lens=(5, 3), page_size=2, seed=0):
    r = np.random.default_rng(seed)
    c = [f32(r.standard_normal((L, d_c))) for L in lens]
    k = [f32(r.standard_normal((L, d_rope))) for L in lens]
    qn = f32(r.standard_normal((B, H, d_head)))
    qr = f32(r.standard_normal((B, H, d_rope)))
    Wk = f32(r.standard_normal((H, d_head, d_c)))
    Wv = f32(r.standard_normal((H, d_c, d_head)))
    pool, table, sl = dense_cache(c, k, page_size, seed=seed)
    return dict(c=c, k=k, qn=qn, qr=qr, Wk=Wk, Wv=Wv, pool=pool, table=table, sl=sl,
                d_c=d_c, d_rope=d_rope, scale=1.0 / math.sqrt(d_head + d_rope))


def absorbed_chain(cs):
    return oracle.mla_step(cs["qn"], cs["qr"], cs["Wk"], cs["Wv"], cs["pool"], None,
                           cs["table"], cs["sl"], cs["scale"])


# ------------------------------------------------- P8: scalar brute force

def brute_force(cs):
    """Scalar reference written out by hand from Eq. "mha": pure Python
    floats, exactly rounded sums (math.fsum)."""
    B, H, d_head = cs["qn"].shape
    out = np.zeros((B, H, d_head))
    lse = np.zeros((B, H))
    for b in range(B):
        L = cs["c"][b].shape[0]
        for h in range(H):
            scores = []
            vals = []
            for j in range(L):
                cj = [float(x) for x in cs["c"][b][j]]
                kc = [math.fsum(float(cs["Wk"][h, d, c]) * cj[c] for c in range(cs["d_c"]))
                      for d in range(d_head)]
                vj = [math.fsum(cj[c] * float(cs["Wv"][h, c, d]) for c in range(cs["d_c"]))
                      for d in range(d_head)]
                dot = math.fsum([float(cs["qn"][b, h, d]) * kc[d] for d in range(d_head)] +
                                [float(cs["qr"][b, h, r]) * float(cs["k"][b][j, r])
                                 for r in range(cs["d_rope"])])
                scores.append(cs["scale"] * dot)
                vals.append(vj)
            m = max(scores)
            e = [math.exp(s - m) for s in scores]
            z = math.fsum(e)
            for d in range(d_head):
                out[b, h, d] = math.fsum(e[j] / z * vals[j][d] for j in range(L))
            lse[b, h] = m + math.log(z)
    return out, lse


@pytest.mark.parametrize("seed,d_rope,page_size", [(0, 2, 2), (1, 0, 2), (2, 2, 3), (3, 2, 1)])
def test_P8_brute_force_tiny(seed, d_rope, page_size):
    cs = random_case(d_rope=d_rope, page_size=page_size, seed=seed)
    want, want_lse = brute_force(cs)
    got, got_lse = oracle.decode_explicit(cs["qn"], cs["qr"], cs["Wk"], cs["Wv"], cs["pool"], None,
                                          cs["table"], cs["sl"], cs["scale"], cs["d_c"])
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got_lse, want_lse, rtol=1e-12, atol=1e-13)
    ch = absorbed_chain(cs)
    np.testing.assert_allclose(ch["out"], want, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(ch["lse"], want_lse, rtol=1e-12, atol=1e-12)


# ----------------------------------- P1: absorbed form == explicit form

@pytest.mark.parametrize("seed", range(4))
def test_P1_absorbed_equals_explicit_random(seed):
    """Sec. 3.3: the "MQA paradigm" is an exact re-association of the
    "MHA paradigm"; both routines are written separately and must agree."""
    r = np.random.default_rng(seed)
    B, H = 3, 5
    lens = tuple(int(x) for x in r.integers(1, 40, size=B))
    cs = random_case(B=B, H=H, d_head=8, d_c=16, d_rope=4, lens=lens, page_size=4, seed=seed)
    e_out, e_lse = oracle.decode_explicit(cs["qn"], cs["qr"], cs["Wk"], cs["Wv"], cs["pool"], None,
                                          cs["table"], cs["sl"], cs["scale"], cs["d_c"])
    ch = absorbed_chain(cs)
    scale = np.abs(e_out).max()
    assert np.abs(ch["out"] - e_out).max() <= 1e-12 * scale
    np.testing.assert_allclose(ch["lse"], e_lse, rtol=1e-12, atol=1e-12)


def test_P1_absorbed_equals_explicit_C1_full():
    """Config 1 at full size (fp32 storage, 1024 tokens, 32 heads)."""
    w = synth.config("C1")
    e_out, e_lse = oracle.decode_explicit(w.q_nope, w.q_rope, w.W_UK, w.W_UV, w.pool, None,
                                          w.page_table, w.seq_lens, w.softmax_scale, w.d_c)
    ch = oracle.mla_step(w.q_nope, w.q_rope, w.W_UK, w.W_UV, w.pool, None, w.page_table,
                         w.seq_lens, w.softmax_scale)
    assert np.abs(ch["out"] - e_out).max() <= 1e-12 * np.abs(e_out).max()
    np.testing.assert_allclose(ch["lse"], e_lse, rtol=1e-12)


def test_P1_subsample_bf16_and_fp8_caches():
    """Explicit vs absorbed on a sub-sample of sequences and heads, reading
    bf16 and fp8 caches through a randomly placed page table."""
    for name in ("C3", "C5"):
        w = synth.config(name, shrink=64)
        b_sel, h_sel = [0, w.B - 1], [0, 7, 31]
        e_out, e_lse = oracle.decode_explicit(w.q_nope, w.q_rope, w.W_UK, w.W_UV, w.pool,
                                              w.kv_scale, w.page_table, w.seq_lens,
                                              w.softmax_scale, w.d_c, b_sel, h_sel)
        ch = oracle.mla_step(w.q_nope, w.q_rope, w.W_UK, w.W_UV, w.pool, w.kv_scale,
                             w.page_table, w.seq_lens, w.softmax_scale)
        sub = ch["out"][np.ix_(b_sel, h_sel)]
        assert np.isfinite(sub).all()
        assert np.abs(sub - e_out).max() <= 1e-11 * np.abs(e_out).max()
        np.testing.assert_allclose(ch["lse"][np.ix_(b_sel, h_sel)], e_lse, rtol=1e-12)


# ------------------------- P2: reduction to textbook MHA / GQA (Sec. 4.1)

def test_P2_block_identity_reduces_to_MHA():
    """d_c = H*d_head, W_UK[h] / W_UV[h] = identity on block h, no RoPE part,
    scale 1/sqrt(d_head): the layer is plain multi-head attention whose key
    and value of head h are both block h of the latent."""
    r = np.random.default_rng(7)
    B, H, d = 2, 4, 8
    d_c = H * d
    lens = (9, 6)
    c = [f32(r.standard_normal((L, d_c))) for L in lens]
    k = [np.zeros((L, 2)) for L in lens]
    qn = f32(r.standard_normal((B, H, d)))
    qr = np.zeros((B, H, 2))
    Wk = np.zeros((H, d, d_c))
    Wv = np.zeros((H, d_c, d))
    for h in range(H):
        Wk[h, :, h * d:(h + 1) * d] = np.eye(d)
        Wv[h, h * d:(h + 1) * d, :] = np.eye(d)
    pool, table, sl = dense_cache(c, k, page_size=4)
    scale = 1.0 / math.sqrt(d)
    got = oracle.mla_step(qn, qr, Wk, Wv, pool, None, table, sl, scale)["out"]
    got_e, _ = oracle.decode_explicit(qn, qr, Wk, Wv, pool, None, table, sl, scale, d_c)
    for b in range(B):
        for h in range(H):
            blk = c[b][:, h * d:(h + 1) * d]
            want, _ = textbook_attention(qn[b, h], blk, blk, scale)
            np.testing.assert_allclose(got[b, h], want, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(got_e[b, h], want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("H,g", [(8, 2), (6, 3), (4, 4), (4, 1)])
def test_P2_selector_matrices_reduce_to_GQA(H, g):
    """Sec. 4.1 / App. A.2.1: c = [k_1..k_g ; v_1..v_g] (r_kv = 2gd),
    W^{UK}_i selects key block ceil(i/(h/g)), W^{UV}_i selects value block
    g + ceil(i/(h/g)); the layer equals grouped-query attention with
    distinct keys and values (g = h: MHA, g = 1: MQA)."""
    r = np.random.default_rng(100 + H * 10 + g)
    B, d = 2, 4
    d_c = 2 * g * d
    lens = (7, 10)
    Ks = [f32(r.standard_normal((L, g, d))) for L in lens]
    Vs = [f32(r.standard_normal((L, g, d))) for L in lens]
    c = [np.concatenate([Ks[b].reshape(L, g * d), Vs[b].reshape(L, g * d)], axis=1)
         for b, L in enumerate(lens)]
    k = [np.zeros((L, 2)) for L in lens]
    qn = f32(r.standard_normal((B, H, d)))
    qr = f32(r.standard_normal((B, H, 2)))  # multiplies a zero key part: no effect
    Wk = np.zeros((H, d, d_c))
    Wv = np.zeros((H, d_c, d))
    for i in range(1, H + 1):  # 1-based head index as in the paper
        kk = math.ceil(i / (H / g))
        Wk[i - 1, :, (kk - 1) * d:kk * d] = np.eye(d)
        Wv[i - 1, (g + kk - 1) * d:(g + kk) * d, :] = np.eye(d)
    pool, table, sl = dense_cache(c, k, page_size=4)
    scale = 1.0 / math.sqrt(d)
    got = oracle.mla_step(qn, qr, Wk, Wv, pool, None, table, sl, scale)["out"]
    for b in range(B):
        for i in range(1, H + 1):
            kk = math.ceil(i / (H / g)) - 1
            want, _ = textbook_attention(qn[b, i - 1], Ks[b][:, kk], Vs[b][:, kk], scale)
            np.testing.assert_allclose(got[b, i - 1], want, rtol=1e-12, atol=1e-13)


def test_P3_zero_WUK_is_MQA_on_the_rope_part():
    """App. A.3: the positional term is an MQA structure -- h query parts
    against one shared key part.  With W_UK = 0 only that term is left."""
    cs = random_case(B=2, H=4, d_head=4, d_c=6, d_rope=4, lens=(8, 5), seed=11)
    cs["Wk"] = np.zeros_like(cs["Wk"])
    got = absorbed_chain(cs)["out"]
    for b in range(2):
        for h in range(4):
            V = cs["c"][b] @ cs["Wv"][h]
            want, _ = textbook_attention(cs["qr"][b, h], cs["k"][b], V, cs["scale"])
            np.testing.assert_allclose(got[b, h], want, rtol=1e-12, atol=1e-13)


def test_T3_prefolded_query_route():
    """App. A.2.2: scores can be taken with W'^Q_i = (W^{UK}_i)^T W^Q_i
    applied to the hidden state; pins the orientation of W_UK in absorb_q."""
    r = np.random.default_rng(5)
    B, H, d, d_c, D = 2, 3, 4, 6, 10
    x = f32(r.standard_normal((B, D)))
    WQ = f32(r.standard_normal((H, d, D)))
    Wk = f32(r.standard_normal((H, d, d_c)))
    q = np.einsum("hdD,bD->bhd", WQ, x)
    Wfold = np.einsum("hdc,hdD->hcD", Wk, WQ)       # (W^{UK}_h)^T W^Q_h : [d_c, D]
    want = np.einsum("hcD,bD->bhc", Wfold, x)
    got = oracle.absorb_q(q, Wk)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_P7_projections_match_einsum():
    r = np.random.default_rng(6)
    q = f32(r.standard_normal((3, 5, 7)))
    Wk = f32(r.standard_normal((5, 7, 11)))
    np.testing.assert_allclose(oracle.absorb_q(q, Wk), np.einsum("bhd,hdc->bhc", q, Wk),
                               rtol=1e-13, atol=1e-13)
    o = f32(r.standard_normal((3, 5, 11)))
    Wv = f32(r.standard_normal((5, 11, 7)))
    np.testing.assert_allclose(oracle.out_proj(o, Wv), np.einsum("bhc,hcd->bhd", o, Wv),
                               rtol=1e-13, atol=1e-13)
    # a non-symmetric hand example: 1 head, d_head 2, d_c 3
    got = oracle.absorb_q(np.array([[[1.0, 10.0]]]), np.array([[[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]]]))
    np.testing.assert_array_equal(got, [[[41.0, 52.0, 63.0]]])
    got = oracle.out_proj(np.array([[[1.0, 10.0, 100.0]]]),
                          np.array([[[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]]]))
    np.testing.assert_array_equal(got, [[[531.0, 642.0]]])


# ------------------------------------- T4: content + positional split

def test_T4_score_is_content_plus_positional():
    """App. A.3: score = q^C.k^C + q^R.k^R.  The log-sum-exp of a one-token
    cache *is* the scaled score, so it exposes the score directly."""
    r = np.random.default_rng(8)
    H, d, d_c, d_r = 3, 4, 6, 2
    c = [f32(r.standard_normal((1, d_c)))]
    k = [f32(r.standard_normal((1, d_r)))]
    qn = f32(r.standard_normal((1, H, d)))
    qr = f32(r.standard_normal((1, H, d_r)))
    Wk = f32(r.standard_normal((H, d, d_c)))
    pool, table, sl = dense_cache(c, k, page_size=2)
    qa = oracle.absorb_q(qn, Wk)
    scale = 0.37
    _, lse_full = oracle.decode_absorbed(qa, qr, pool, None, table, sl, scale)
    _, lse_content = oracle.decode_absorbed(qa, 0 * qr, pool, None, table, sl, scale)
    _, lse_pos = oracle.decode_absorbed(0 * qa, qr, pool, None, table, sl, scale)
    np.testing.assert_allclose(lse_full, lse_content + lse_pos, rtol=1e-13, atol=1e-13)
    want_content = scale * np.einsum("hd,hdc,c->h", qn[0], Wk, c[0][0])
    want_pos = scale * qr[0] @ k[0][0]
    np.testing.assert_allclose(lse_content[0], want_content, rtol=1e-12)
    np.testing.assert_allclose(lse_pos[0], want_pos, rtol=1e-12)


# ----------------------------------------- P4 / P5: softmax properties

def test_P4_rows_sum_to_one_and_convexity():
    cs = random_case(B=2, H=3, d_head=4, d_c=6, d_rope=2, lens=(33, 17), page_size=4, seed=21)
    _, _, probs = oracle.decode_explicit(cs["qn"], cs["qr"], cs["Wk"], cs["Wv"], cs["pool"], None,
                                         cs["table"], cs["sl"], cs["scale"], cs["d_c"],
                                         return_probs=True)
    assert (probs >= 0).all()
    np.testing.assert_allclose(probs.sum(-1), 1.0, rtol=0, atol=1e-15 * 40)
    assert (probs[1, :, 17:] == 0).all()
    qa = oracle.absorb_q(cs["qn"], cs["Wk"])
    o, _ = oracle.decode_absorbed(qa, cs["qr"], cs["pool"], None, cs["table"], cs["sl"], cs["scale"])
    for b in range(2):
        lo, hi = cs["c"][b].min(0), cs["c"][b].max(0)
        assert (o[b] >= lo - 1e-12).all() and (o[b] <= hi + 1e-12).all()


def test_P5_closed_forms():
    r = np.random.default_rng(9)
    H, d_c, d_r = 3, 6, 2
    scale = 0.25
    # one cached token: o = c_0, lse = s_0
    c = [f32(r.standard_normal((1, d_c)))]
    k = [f32(r.standard_normal((1, d_r)))]
    pool, table, sl = dense_cache(c, k, page_size=2)
    qa = f32(r.standard_normal((1, H, d_c)))
    qr = f32(r.standard_normal((1, H, d_r)))
    o, lse = oracle.decode_absorbed(qa, qr, pool, None, table, sl, scale)
    np.testing.assert_allclose(o[0], np.broadcast_to(c[0][0], (H, d_c)), rtol=1e-15)
    np.testing.assert_allclose(lse[0], scale * (qa[0] @ c[0][0] + qr[0] @ k[0][0]), rtol=1e-13)
    # zero query: uniform weights -> mean of the rows, lse = log L
    L = 11
    c = [f32(r.standard_normal((L, d_c)))]
    k = [f32(r.standard_normal((L, d_r)))]
    pool, table, sl = dense_cache(c, k, page_size=4)
    o, lse = oracle.decode_absorbed(np.zeros((1, H, d_c)), np.zeros((1, H, d_r)), pool, None,
                                    table, sl, scale)
    np.testing.assert_allclose(o[0], np.broadcast_to(c[0].mean(0), (H, d_c)), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse[0], math.log(L), rtol=1e-14)
    # all rows equal: o = that row whatever the query
    row = f32(r.standard_normal(d_c))
    c = [np.tile(row, (L, 1))]
    k = [np.tile(f32(r.standard_normal(d_r)), (L, 1))]
    pool, table, sl = dense_cache(c, k, page_size=4)
    o, _ = oracle.decode_absorbed(qa, qr, pool, None, table, sl, scale)
    np.testing.assert_allclose(o[0], np.broadcast_to(row, (H, d_c)), rtol=1e-14)
    # one score far above the rest: o -> that row
    c = [f32(r.standard_normal((L, d_c)))]
    k = [np.zeros((L, d_r))]
    k[0][4, 0] = 1.0
    pool, table, sl = dense_cache(c, k, page_size=4)
    qr_big = np.zeros((1, H, d_r))
    qr_big[..., 0] = 800.0  # scaled score of token 4 exceeds the others by 200
    o, lse = oracle.decode_absorbed(np.zeros((1, H, d_c)), qr_big, pool, None, table, sl, scale)
    np.testing.assert_allclose(o[0], np.broadcast_to(c[0][4], (H, d_c)), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(lse[0], 200.0, rtol=1e-13)


def test_P5_empty_sequence():
    """seq_len = 0: nothing to attend to -> zeros and lse = -inf."""
    cs = random_case(B=2, H=3, lens=(5, 3), seed=2)
    sl = cs["sl"].copy()
    sl[1] = 0
    qa = oracle.absorb_q(cs["qn"], cs["Wk"])
    o, lse = oracle.decode_absorbed(qa, cs["qr"], cs["pool"], None, cs["table"], sl, cs["scale"])
    assert (o[1] == 0).all() and np.isneginf(lse[1]).all()
    assert np.isfinite(o[0]).all()


# ------------------------------------------------------ P6: invariances

def test_P6_token_order_and_page_placement():
    r = np.random.default_rng(31)
    cs = random_case(B=2, H=3, d_head=4, d_c=6, d_rope=2, lens=(13, 9), page_size=4, seed=31)
    base = absorbed_chain(cs)
    # another physical placement of the same logical rows
    pool2, table2, sl2 = dense_cache(cs["c"], cs["k"], page_size=4, seed=99, extra_pages=5)
    alt = oracle.mla_step(cs["qn"], cs["qr"], cs["Wk"], cs["Wv"], pool2, None, table2, sl2, cs["scale"])
    np.testing.assert_array_equal(alt["out"], base["out"])  # same op order -> same bits
    # identity placement
    pool3, table3, sl3 = dense_cache(cs["c"], cs["k"], page_size=4, shuffle=False, extra_pages=0)
    alt = oracle.mla_step(cs["qn"], cs["qr"], cs["Wk"], cs["Wv"], pool3, None, table3, sl3, cs["scale"])
    np.testing.assert_array_equal(alt["out"], base["out"])
    # a different page size changes nothing either
    pool4, table4, sl4 = dense_cache(cs["c"], cs["k"], page_size=5, seed=3)
    alt = oracle.mla_step(cs["qn"], cs["qr"], cs["Wk"], cs["Wv"], pool4, None, table4, sl4, cs["scale"])
    np.testing.assert_array_equal(alt["out"], base["out"])
    # permuting the logical order of the cached rows (RoPE is baked into them)
    perm = [r.permutation(13), r.permutation(9)]
    c2 = [cs["c"][b][perm[b]] for b in range(2)]
    k2 = [cs["k"][b][perm[b]] for b in range(2)]
    pool5, table5, sl5 = dense_cache(c2, k2, page_size=4, seed=5)
    alt = oracle.mla_step(cs["qn"], cs["qr"], cs["Wk"], cs["Wv"], pool5, None, table5, sl5, cs["scale"])
    np.testing.assert_allclose(alt["out"], base["out"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(alt["lse"], base["lse"], rtol=1e-13)


def test_P6_shift_invariance_of_softmax():
    """A component shared by every key (constant cache column) shifts all
    scores of a head by the same amount: o unchanged, lse moves by it."""
    cs = random_case(B=1, H=3, d_head=4, d_c=6, d_rope=2, lens=(12,), page_size=4, seed=41)
    qa = oracle.absorb_q(cs["qn"], cs["Wk"])
    o0, l0 = oracle.decode_absorbed(qa, cs["qr"], cs["pool"], None, cs["table"], cs["sl"], cs["scale"])
    k2 = [np.concatenate([cs["k"][0], np.full((12, 2), 3.0)], axis=1)]
    qr2 = np.concatenate([cs["qr"], np.full((1, 3, 2), 0.5)], axis=2)
    pool, table, sl = dense_cache(cs["c"], k2, page_size=4, seed=41)
    o1, l1 = oracle.decode_absorbed(qa, qr2, pool, None, table, sl, cs["scale"])
    np.testing.assert_allclose(o1, o0, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(l1 - l0, cs["scale"] * 3.0, rtol=1e-12)


@pytest.mark.parametrize("n_splits,chunk_pages", [(1, 100), (2, 5), (7, 2), (32, 1), (3, 1)])
def test_P6_split_kv_merge_agrees(n_splits, chunk_pages):
    """Softmax over a union of chunks = log-sum-exp-weighted mix of the
    chunk-local softmaxes (the identity the split-KV reduction relies on)."""
    cs = random_case(B=3, H=3, d_head=4, d_c=6, d_rope=2, lens=(37, 1, 20), page_size=4, seed=51)
    qa = oracle.absorb_q(cs["qn"], cs["Wk"])
    o0, l0 = oracle.decode_absorbed(qa, cs["qr"], cs["pool"], None, cs["table"], cs["sl"], cs["scale"])
    o1, l1, op, lp = oracle.decode_split(qa, cs["qr"], cs["pool"], None, cs["table"], cs["sl"],
                                         cs["scale"], n_splits, chunk_pages, return_partials=True)
    covered = n_splits * chunk_pages * 4
    for b, L in enumerate((37, 1, 20)):
        if covered >= L:
            np.testing.assert_allclose(o1[b], o0[b], rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(l1[b], l0[b], rtol=1e-13)
    assert np.isfinite(o1).all()
    # empty chunks carry -inf and zero
    used = -(-np.array([37, 1, 20]) // (chunk_pages * 4))
    for b in range(3):
        for s in range(n_splits):
            if s >= used[b]:
                assert np.isneginf(lp[b, :, s]).all() and (op[b, :, s] == 0).all()


def test_merge_lse_against_direct_formula():
    r = np.random.default_rng(61)
    op = r.standard_normal((5, 4))
    lp = np.array([0.3, -np.inf, 2.0, -1.0, 700.0])
    o, l = oracle.merge_lse(op, lp)
    # 700 dominates completely in fp64
    np.testing.assert_allclose(o, op[4], rtol=1e-13)
    assert l == pytest.approx(700.0, rel=1e-15)
    lp = np.array([0.3, -np.inf, 2.0, -1.0, 0.0])
    o, l = oracle.merge_lse(op, lp)
    w = np.exp(lp)
    np.testing.assert_allclose(l, math.log(w.sum()), rtol=1e-14)
    np.testing.assert_allclose(o, (w[:, None] * op).sum(0) / w.sum(), rtol=1e-13)
    o, l = oracle.merge_lse(op, np.full(5, -np.inf))
    assert (o == 0).all() and l == -math.inf


# ------------------------------------------------ P9: RoPE (generator)

def test_P9_rope_matches_equation_and_relative_identity():
    """Sec. 3.1 Eq. 1 (interleaved pairs, theta_k = 10000^(-2(k-1)/d)) and
    App. B: <RoPE(q,t), RoPE(k,j)> depends on t-j only, equal to
    sum_l cos((t-j)th_l)(q_x k_x + q_y k_y) + sin((t-j)th_l)(q_x k_y - q_y k_x)."""
    r = np.random.default_rng(71)
    d = 8
    q = r.standard_normal(d)
    k = r.standard_normal(d)
    # element-wise form of Eq. 1 written out directly
    t = 5
    th = np.array([10000.0 ** (-2.0 * (i - 1) / d) for i in range(1, d // 2 + 1)])
    want = np.empty(d)
    for i in range(d // 2):
        want[2 * i] = q[2 * i] * math.cos(t * th[i]) - q[2 * i + 1] * math.sin(t * th[i])
        want[2 * i + 1] = q[2 * i + 1] * math.cos(t * th[i]) + q[2 * i] * math.sin(t * th[i])
    np.testing.assert_allclose(synth.rope(q[None, :], np.array([t]))[0], want, rtol=1e-13)
    # batch of positions + relative identity
    for (t, j) in [(9, 2), (107, 100), (7, 0), (1023, 1016)]:
        a = synth.rope(q[None, :], np.array([t]))[0]
        b = synth.rope(k[None, :], np.array([j]))[0]
        rel = sum(math.cos((t - j) * th[i]) * (q[2 * i] * k[2 * i] + q[2 * i + 1] * k[2 * i + 1]) +
                  math.sin((t - j) * th[i]) * (q[2 * i] * k[2 * i + 1] - q[2 * i + 1] * k[2 * i])
                  for i in range(d // 2))
        assert a @ b == pytest.approx(rel, rel=1e-11, abs=1e-11)
    # position 0 is the identity; norms are preserved
    np.testing.assert_array_equal(synth.rope(q[None, :], np.array([0]))[0], q)
    x = r.standard_normal((6, d))
    np.testing.assert_allclose(np.linalg.norm(synth.rope(x, np.arange(6)), axis=1),
                               np.linalg.norm(x, axis=1), rtol=1e-13)


# ------------------------------------------------------- P10: codecs

def _golden_pairs(fname):
    pairs = []
    for line in (GOLDEN / fname).read_text().splitlines():
        line = line.split("#")[0].strip()
        if line:
            a, b = line.split()
            pairs.append((int(a, 16), b))
    return pairs


def test_P10_e4m3_decode_table():
    """OCP 8-bit float E4M3: bias 7, subnormals m*2^-9, max 448, NaN at
    S.1111.111 only, no infinities."""
    for code, val in _golden_pairs("e4m3_ocp_values.txt"):
        got = oracle.widen_e4m3_code(code)
        if val == "nan":
            assert math.isnan(got)
        else:
            assert got == float(val), (hex(code), got, val)
            assert math.copysign(1.0, got) == math.copysign(1.0, float(val))
    vals = [oracle.widen_e4m3_code(c) for c in range(256)]
    finite = [v for v in vals if not math.isnan(v)]
    assert len(finite) == 254 and max(finite) == 448.0 and min(finite) == -448.0
    assert not any(math.isinf(v) for v in finite)
    pos = vals[:0x7F]
    assert all(b > a for a, b in zip(pos, pos[1:]))          # strictly monotone
    assert all(vals[c + 128] == -vals[c] for c in range(0x7F))
    # cross-check with the tensor library's independent decoder
    import torch
    t = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(torch.float8_e4m3fn).double().numpy()
    np.testing.assert_array_equal(np.nan_to_num(t, nan=12345.0), np.nan_to_num(np.array(vals), nan=12345.0))


def test_P10_e4m3_encode_roundtrip_ties_saturation():
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    vals = np.array([oracle.widen_e4m3_code(int(c)) for c in codes], dtype=np.float32)
    back = synth.encode_e4m3(vals)
    np.testing.assert_array_equal(back, codes)
    # midpoints go to the even mantissa
    for lo in (0x38, 0x39, 0x01, 0x45, 0x7C):
        a, b = oracle.widen_e4m3_code(lo), oracle.widen_e4m3_code(lo + 1)
        got = int(synth.encode_e4m3(np.array([(a + b) / 2], dtype=np.float32))[0])
        assert got == (lo if lo % 2 == 0 else lo + 1)
    assert list(synth.encode_e4m3(np.array([1e6, -1e6, 449.0, 464.0], dtype=np.float32))) == \
        [0x7E, 0xFE, 0x7E, 0x7E]
    # per-token quantiser: scale = absmax/448, absmax itself maps to +-448
    x = np.array([[0.5, -2.0, 1.0], [0.0, 0.0, 0.0]], dtype=np.float32)
    q, s = synth.quant_e4m3_per_token(x)
    assert s[0] == np.float32(2.0 / 448.0) and s[1] == 1.0
    assert q[0, 1] == 0xFE and (q[1] == 0).all()
    assert oracle.widen_e4m3_code(int(q[0, 0])) * float(s[0]) == pytest.approx(0.5, rel=2 ** -4)


def test_P10_bf16_all_codes():
    """bfloat16 = top half of binary32: check all 65536 patterns against the
    tensor library's widening, and the encoder's round-to-nearest-even."""
    import torch
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.widen(bits)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).double().numpy()
    np.testing.assert_array_equal(np.nan_to_num(got, nan=7.0), np.nan_to_num(want, nan=7.0))
    assert oracle.widen_bf16_code(0x3F80) == 1.0 and oracle.widen_bf16_code(0xC000) == -2.0
    finite = np.isfinite(want)
    re = synth.to_bf16_bits(want[finite].astype(np.float32))
    np.testing.assert_array_equal(re, bits[finite])
    x = np.random.default_rng(3).standard_normal(100000).astype(np.float32) * 37.0
    np.testing.assert_array_equal(synth.to_bf16_bits(x).view(np.int16),
                                  torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy())
    # exact ties: 1 + 2^-8 -> 1 (even), 1 + 3*2^-8 -> 1 + 2^-6
    assert synth.to_bf16_bits(np.array([1 + 2 ** -8, 1 + 3 * 2 ** -8], dtype=np.float32)).tolist() == \
        [0x3F80, 0x3F82]


# ------------------------------------------------------ P11: page gather

def test_P11_gather_is_byte_exact():
    w = synth.config("C3", shrink=64)
    max_len = int(w.seq_lens.max())
    dense = oracle.gather_paged(w.pool, w.page_table, w.seq_lens, max_len)
    flat = w.pool.reshape(-1, w.pool.shape[2])
    for b in (0, w.B - 1):
        L = int(w.seq_lens[b])
        for j in (0, 1, 63, 64, L - 1):
            if j >= L:
                continue
            row = flat[int(w.page_table[b, j // 64]) * 64 + j % 64]
            assert dense[b, j].tobytes() == row.tobytes()
        assert not dense[b, L:].any()
    # no poison (NaN pattern 0x7FC0) inside the valid region
    v = dense[0, :int(w.seq_lens[0])].view(np.uint16)
    assert not (v == 0x7FC0).any()


# ------------------------------------- shapes vs the paper's KV budget

def test_config_shapes_match_paper_kv_budget():
    """Table 1 / Sec. 5: LLaMA-2-7B keeps 7.03 % of 2*32*128 = 8192 cache
    values per token at -92.97 %, i.e. 576 = d_c + d_rope."""
    rows = {}
    for line in (GOLDEN / "kv_budget.txt").read_text().splitlines():
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split()
            rows[k] = float(v)
    w = synth.config("C2", shrink=64)
    kept = (w.d_c + w.d_rope) / (2 * 32 * 128)
    assert round(100 * (1 - kept), 2) == rows["llama2_7b_max_compression_percent"]
    assert round(100 * kept, 2) == rows["llama2_7b_kept_percent"]
    assert w.softmax_scale == pytest.approx(1 / math.sqrt(192))
    assert w.row_bytes == 1152
    w5 = synth.config("C5", shrink=64)
    assert w5.row_bytes == 576 and w5.kv_scale is not None
    w4 = synth.config("C4", shrink=64)
    assert (w4.H, w4.d_c, w4.row_bytes) == (28, 256, 640)


def test_generator_is_seeded_and_poisoned():
    a = synth.config("C3", shrink=64, seed=0)
    b = synth.config("C3", shrink=64, seed=0)
    c = synth.config("C3", shrink=64, seed=1)
    assert a.pool.tobytes() == b.pool.tobytes() and (a.page_table == b.page_table).all()
    assert a.pool.tobytes() != c.pool.tobytes()
    used = set(a.page_table[a.page_table >= 0].tolist())
    assert len(used) == int(((a.seq_lens + 63) // 64).sum())         # no page shared
    free = [p for p in range(a.num_pages) if p not in used]
    assert free and all((a.pool[p] == 0x7FC0).all() for p in free)   # free pages poisoned
    assert len(free) >= int(0.08 * a.num_pages)
    # weights have variance 1/d_c, cache ~ N(0,1) with rope part x4
    W = oracle.widen(a.W_UK)
    assert W.var() == pytest.approx(1 / 512, rel=0.05)
    L0 = int(a.seq_lens[0])
    rows = oracle.widen(oracle.gather_paged(a.pool, a.page_table, a.seq_lens, L0)[0].view(np.uint16))
    assert rows[:, :512].std() == pytest.approx(1.0, rel=0.05)
    assert rows[:, 512:].std() == pytest.approx(4.0, rel=0.05)


def test_stored_cache_values_are_widened_exactly():
    """With a single cached token the output is that token's latent row
    (softmax over one element is 1), which exposes how the oracle reads each
    storage dtype: bf16 bits, and fp8 code times the token's scale."""
    import torch
    r = np.random.default_rng(81)
    B, H, d_c, d_r = 3, 2, 8, 2
    x = (r.standard_normal((B, 1, d_c + d_r)) * 3).astype(np.float32)
    table = np.arange(B, dtype=np.int32).reshape(B, 1)[::-1].copy()
    sl = np.ones(B, dtype=np.int32)
    qa = r.standard_normal((B, H, d_c))
    qr = r.standard_normal((B, H, d_r))
    # bf16
    pool = np.full((B, 4, d_c + d_r), 0x7FC0, dtype=np.uint16)
    bits = synth.to_bf16_bits(x)
    pool[:, 0:1, :] = bits
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).double().numpy()
    o, lse = oracle.decode_absorbed(qa, qr, pool, None, table, sl, 0.5)
    for b in range(B):
        p = table[b, 0]
        np.testing.assert_array_equal(o[b], np.broadcast_to(want[p, 0, :d_c], (H, d_c)))
        np.testing.assert_allclose(lse[b], 0.5 * (qa[b] @ want[p, 0, :d_c] + qr[b] @ want[p, 0, d_c:]),
                                   rtol=1e-13)
    # fp8 + per-token scale
    codes, sc = synth.quant_e4m3_per_token(x.reshape(B, -1))
    pool = np.full((B, 4, d_c + d_r), 0x7F, dtype=np.uint8)
    pool[:, 0, :] = codes
    kv_scale = np.full((B, 4), np.nan, dtype=np.float32)
    kv_scale[:, 0] = sc
    dec = torch.from_numpy(codes).view(torch.float8_e4m3fn).double().numpy() * sc.astype(np.float64)[:, None]
    o, lse = oracle.decode_absorbed(qa, qr, pool, kv_scale, table, sl, 0.5)
    for b in range(B):
        p = table[b, 0]
        np.testing.assert_array_equal(o[b], np.broadcast_to(dec[p, :d_c], (H, d_c)))
        np.testing.assert_allclose(lse[b], 0.5 * (qa[b] @ dec[p, :d_c] + qr[b] @ dec[p, d_c:]), rtol=1e-13)
    assert np.abs(dec - x.reshape(B, -1)).max() <= np.abs(x).max() * 2 ** -4  # sanity: it is a quantisation of x


# ------------------------------------------------------------ cache append
# Sec. 3.3 (MLA equations): c^{KV} = W^{DKV} x, k^R = RoPE(W^{KR} x, t); Sec. 3.1 Eq. 1 for RoPE.

def test_A1_rope_closed_forms():
    """Eq. 1: position 0 is the identity; the first pair (theta = 1) of (1, 0) at position
    pi/2 is (0, 1); with base 1 every pair turns by the position itself; pair norms are kept."""
    v = RNG.standard_normal(64)
    assert np.array_equal(oracle.rope(v, 0.0), v)
    e = np.zeros(8); e[0] = 1.0
    np.testing.assert_allclose(oracle.rope(e, math.pi / 2)[:2], [0.0, 1.0], atol=1e-15)
    r = oracle.rope(v, 0.75, base=1.0)
    z = (v[0::2] + 1j * v[1::2]) * np.exp(1j * 0.75)          # complex multiplication, base 1
    np.testing.assert_allclose(r[0::2] + 1j * r[1::2], z, rtol=0, atol=1e-14)
    w = oracle.rope(v, 1234.0)
    np.testing.assert_allclose(np.hypot(w[0::2], w[1::2]), np.hypot(v[0::2], v[1::2]), rtol=1e-13)


def test_A2_rope_group_and_relative_position_properties():
    """Rotations compose additively in the position, and <RoPE(q, m), RoPE(k, n)> depends on
    m - n only (the property App. B builds on)."""
    q, k = RNG.standard_normal(64), RNG.standard_normal(64)
    np.testing.assert_allclose(oracle.rope(oracle.rope(q, 17.0), 25.0), oracle.rope(q, 42.0), atol=1e-12)
    d1 = oracle.rope(q, 100.0) @ oracle.rope(k, 93.0)
    d2 = oracle.rope(q, 5007.0) @ oracle.rope(k, 5000.0)
    d3 = oracle.rope(q, 7.0) @ k
    np.testing.assert_allclose([d1, d2], [d3, d3], atol=1e-9)


def test_A3_rope_frequencies_against_the_input_generator():
    """Independent implementation (the workload generator's vectorised numpy RoPE) at the
    frequencies of Eq. 1, theta_i = 10000^(-2i/d)."""
    v = RNG.standard_normal((5, 64))
    for pos in (1.0, 63.0, 8191.0, 131071.0):
        np.testing.assert_allclose(oracle.rope(v, pos), synth.rope(v, np.full(5, pos)), rtol=0, atol=1e-9)


def test_A4_bf16_encoder_against_the_tensor_library_and_ties():
    import torch
    x = np.concatenate([RNG.standard_normal(4000).astype(np.float32) * 3,
                        np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -65504.0])])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.encode_bf16(x), want)
    # ties go to the even mantissa: 1 + 2^-8 -> 1.0, 1 + 3*2^-8 -> 1 + 2^-6
    assert oracle.encode_bf16(np.float32([1.00390625]))[0] == 0x3F80
    assert oracle.encode_bf16(np.float32([1.01171875]))[0] == 0x3F82


def test_A5_e4m3_encoder_round_trip_ties_saturation():
    """Every finite code's value encodes to that code (table of the OCP format in
    tests/golden); the midpoint of two neighbours goes to the even mantissa; beyond 448 -> 448."""
    for code, sval in _golden_pairs("e4m3_ocp_values.txt"):
        if sval == "nan":
            continue
        got = int(oracle.encode_e4m3(np.float32([float(sval)]))[0])
        assert got == code, (hex(code), sval, hex(got))
    # all neighbouring finite codes (their values come from the decoder pinned by P10)
    for c0 in range(0x00, 0x7E):
        v0, v1 = oracle.widen_e4m3_code(c0), oracle.widen_e4m3_code(c0 + 1)
        assert int(oracle.encode_e4m3(np.float32([v0]))[0]) == c0
        mid = np.float32((v0 + v1) / 2)                      # exact in fp32
        want = c0 if c0 % 2 == 0 else c0 + 1
        assert int(oracle.encode_e4m3(np.float32([mid]))[0]) == want
        assert int(oracle.encode_e4m3(np.float32([-mid]))[0]) == (want | 0x80)
        eps = np.float32((v1 - v0) / 64)
        assert int(oracle.encode_e4m3(np.float32([mid - eps]))[0]) == c0
        assert int(oracle.encode_e4m3(np.float32([mid + eps]))[0]) == c0 + 1
    assert list(oracle.encode_e4m3(np.float32([449.0, 1e9, -1e9, 464.0]))) == [0x7E, 0x7E, 0xFE, 0x7E]


def test_A6_e4m3_encoder_and_row_scale_against_the_tensor_library():
    import torch
    x = (RNG.standard_normal(6000) * 100).astype(np.float32)
    want = torch.from_numpy(np.clip(x, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.encode_e4m3(x), want)
    row = RNG.standard_normal(576).astype(np.float32)
    codes, scale = oracle.encode_row(row, oracle.FP8_E4M3)
    wc, ws = synth.quant_e4m3_per_token(row[None])
    assert np.array_equal(codes, wc[0]) and np.float32(scale) == ws[0]
    assert int(codes[np.argmax(np.abs(row))]) & 0x7F == 0x7E     # the largest magnitude lands on 448
    codes0, scale0 = oracle.encode_row(np.zeros(16, np.float32), oracle.FP8_E4M3)
    assert scale0 == 1.0 and not codes0.any()


def _append_case(cache_dtype, seed=5):
    w = synth.make_workload("append", B=3, H=2, d_head=8, d_c=32, d_rope=8, seq_lens=[5, 64, 130],
                            io_dtype="bf16", cache_dtype=cache_dtype, page_size=64, placement="random",
                            free_frac=0.5, max_pages_per_seq=3, seed=seed)
    r = synth.stream(seed, 77)
    D = 24
    x = synth.normal(r, (w.B, D))
    W = synth.normal(r, (D, w.d_c + w.d_rope), 1 / math.sqrt(D))
    return w, x, W


@pytest.mark.parametrize("cache_dtype", ["f32", "bf16", "fp8_e4m3"])
def test_A7_append_writes_exactly_one_row_per_sequence(cache_dtype):
    """After the append the logical view holds the new row at position seq_len and every
    other byte of the pool (and scale pool) is unchanged; the row is [x W_c ; RoPE(x W_r, t)]
    computed here with numpy and the generator's RoPE."""
    w, x, W = _append_case(cache_dtype)
    # sequence 1 is exactly one full page: its new token opens page index 1 of its table
    pt = w.page_table.copy()
    used = set(pt[pt >= 0].tolist())
    free = [p for p in range(w.pool.shape[0]) if p not in used]
    if pt[1, 1] < 0:
        assert free, "the generator leaves a spare page"
        pt[1, 1] = free[0]
    pool2, sc2, rows = oracle.cache_append(x, W, w.pool, w.kv_scale, pt, w.seq_lens, w.d_c)
    y = x.astype(np.float64) @ W.astype(np.float64)
    want = y.copy()
    for b in range(w.B):
        want[b, w.d_c:] = synth.rope(y[b, w.d_c:][None], np.array([float(w.seq_lens[b])]))[0]
    np.testing.assert_allclose(rows, want, rtol=0, atol=1e-10)
    changed = np.zeros(w.pool.shape[:2], dtype=bool)
    for b in range(w.B):
        t = int(w.seq_lens[b])
        changed[pt[b, t // 64], t % 64] = True
        stored = oracle.widen(pool2[pt[b, t // 64], t % 64]) if cache_dtype != "fp8_e4m3" else None
        if cache_dtype == "f32":
            assert np.array_equal(pool2[pt[b, t // 64], t % 64], want[b].astype(np.float32))
        elif cache_dtype == "bf16":
            np.testing.assert_allclose(stored, want[b], rtol=2 ** -8, atol=1e-30)
        else:
            s = sc2[pt[b, t // 64], t % 64]
            dec = np.array([oracle.widen_e4m3_code(int(c)) for c in pool2[pt[b, t // 64], t % 64]]) * float(s)
            assert abs(float(s) - np.abs(want[b]).max() / 448) <= 1e-6 * float(s)
            np.testing.assert_allclose(dec, want[b], rtol=0, atol=np.abs(want[b]).max() / 448 * 16 + 1e-12)
    a, b2 = w.pool.view(np.uint8).reshape(*w.pool.shape[:2], -1), pool2.view(np.uint8).reshape(*w.pool.shape[:2], -1)
    same = (a == b2).all(axis=-1) | (np.isnan(w.pool).all(axis=-1) & np.isnan(pool2).all(axis=-1) if cache_dtype == "f32" else False)
    assert same[~changed].all()
    if sc2 is not None:
        assert np.array_equal(sc2[~changed], w.kv_scale[~changed], equal_nan=True)


def test_A8_append_then_decode_sees_the_new_token():
    """x = 64 e_3 picks 64 times a row of W exactly; that row dwarfs the cached ones, so a query
    aligned with it puts all the weight on the appended token: o_lat equals its latent part."""
    w, x, W = _append_case("f32", seed=9)
    x = np.zeros_like(x); x[:, 3] = 64.0
    pt = w.page_table.copy()
    if pt[1, 1] < 0:
        used = set(pt[pt >= 0].tolist())
        pt[1, 1] = [p for p in range(w.pool.shape[0]) if p not in used][0]
    pool2, _, rows = oracle.cache_append(x, W, w.pool, None, pt, w.seq_lens, w.d_c)
    np.testing.assert_allclose(rows[:, :w.d_c], np.tile(64.0 * W[3, :w.d_c].astype(np.float64), (w.B, 1)), atol=0)
    q_abs = np.repeat(rows[:, None, :w.d_c], w.H, axis=1)
    q_rope = np.zeros((w.B, w.H, w.d_rope))
    o, _ = oracle.decode_absorbed(q_abs, q_rope, pool2, None, pt, w.seq_lens + 1, 1.0)
    np.testing.assert_allclose(o, np.repeat(rows[:, None, :w.d_c].astype(np.float32), w.H, axis=1), rtol=1e-6, atol=1e-7)


def test_A9_append_skips_positions_outside_the_table_or_pool():
    w, x, W = _append_case("bf16")
    pos = w.seq_lens.copy(); pos[0] = 3 * 64            # one past the table
    pt = w.page_table.copy(); pt[2, 130 // 64] = w.pool.shape[0] + 7     # page id outside the pool
    pt[1, 1] = -1
    pool2, _, _ = oracle.cache_append(x, W, w.pool, None, pt, pos, w.d_c)
    assert np.array_equal(pool2, w.pool)


# ---------------------------------------------------------------------------
# M: several query tokens per sequence (multi-token prediction; Eq. "mqa" read for the T newest
# positions at once, each with its own upper limit of the sum over j)
# ---------------------------------------------------------------------------

def _multi_case(T, lens, H=3, d_head=4, d_c=6, d_rope=2, page_size=2, seed=0):
    r = np.random.default_rng(100 + seed)
    B = len(lens)
    c = [f32(r.standard_normal((L, d_c))) for L in lens]
    k = [f32(r.standard_normal((L, d_rope))) for L in lens]
    pool, table, sl = dense_cache(c, k, page_size, seed=seed)
    return dict(c=c, k=k, pool=pool, table=table, sl=sl, d_c=d_c, d_rope=d_rope,
                qn=f32(r.standard_normal((B, T, H, d_head))), qr=f32(r.standard_normal((B, T, H, d_rope))),
                Wk=f32(r.standard_normal((H, d_head, d_c))), Wv=f32(r.standard_normal((H, d_c, d_head))),
                scale=1.0 / math.sqrt(d_head + d_rope))


def _multi_chain(cs):
    """absorb -> multi-token decode -> up-projection, all through the oracle."""
    B, T, H, d_head = cs["qn"].shape
    qa = oracle.absorb_q(cs["qn"].reshape(B * T, H, d_head), cs["Wk"]).reshape(B, T, H, cs["d_c"])
    o, lse = oracle.decode_absorbed_multi(qa, cs["qr"], cs["pool"], None, cs["table"], cs["sl"], cs["scale"])
    out = oracle.out_proj(o.reshape(B * T, H, cs["d_c"]), cs["Wv"]).reshape(B, T, H, d_head)
    return qa, o, lse, out


@pytest.mark.parametrize("T,lens,page_size,seed", [(2, (7, 4), 2, 0), (3, (9, 3, 5), 4, 1), (4, (6, 13), 3, 2),
                                                   (1, (5, 3), 2, 3)])
def test_M1_multi_token_equals_masked_attention_in_the_MHA_paradigm(T, lens, page_size, seed):
    """Eq. "mha" written as the textbook masked attention of a whole sequence: keys and values
    materialised per head, one score matrix [T x L], entry (i, j) allowed iff j <= L - T + i."""
    cs = _multi_case(T, lens, page_size=page_size, seed=seed)
    _, _, lse, out = _multi_chain(cs)
    for b, L in enumerate(lens):
        for h in range(cs["Wk"].shape[0]):
            K = np.concatenate([cs["c"][b] @ cs["Wk"][h].T, cs["k"][b]], axis=1)     # [L, d + d^R]
            V = cs["c"][b] @ cs["Wv"][h]                                               # [L, d]
            Q = np.concatenate([cs["qn"][b, :, h], cs["qr"][b, :, h]], axis=1)         # [T, d + d^R]
            S = (Q @ K.T) * cs["scale"]
            allowed = np.arange(L)[None, :] <= (L - T + np.arange(T))[:, None]
            S = np.where(allowed, S, -np.inf)
            m = S.max(axis=1, keepdims=True)
            E = np.exp(S - m)
            Z = E.sum(axis=1, keepdims=True)
            np.testing.assert_allclose(out[b, :, h], (E / Z) @ V, rtol=1e-11, atol=1e-12)
            np.testing.assert_allclose(lse[b, :, h], (m + np.log(Z))[:, 0], rtol=1e-12, atol=1e-12)


def test_M2_each_token_is_a_single_token_decode_of_the_truncated_sequence():
    """Token i of T is the (separately pinned) one-token decode at length L - (T-1-i)."""
    T = 3
    cs = _multi_case(T, (10, 6, 3), page_size=4, seed=5)
    qa, o, lse, _ = _multi_chain(cs)
    for i in range(T):
        sl_i = np.maximum(cs["sl"] - (T - 1 - i), 0).astype(np.int32)
        o1, l1 = oracle.decode_absorbed(qa[:, i], cs["qr"][:, i], cs["pool"], None, cs["table"], sl_i, cs["scale"])
        assert np.array_equal(o[:, i], o1) and np.array_equal(lse[:, i], l1)


def test_M3_multi_token_closed_forms():
    T, H, d_c, d_r = 3, 2, 6, 2
    r = np.random.default_rng(77)
    scale = 0.3
    # L = T: token 0 sees row 0 alone -> o = c_0, lse = its score; token 1 sees rows 0 and 1 ...
    L = T
    c = [f32(r.standard_normal((L, d_c)))]
    k = [f32(r.standard_normal((L, d_r)))]
    pool, table, sl = dense_cache(c, k, page_size=2)
    qa = f32(r.standard_normal((1, T, H, d_c)))
    qr = f32(r.standard_normal((1, T, H, d_r)))
    o, lse = oracle.decode_absorbed_multi(qa, qr, pool, None, table, sl, scale)
    np.testing.assert_allclose(o[0, 0], np.broadcast_to(c[0][0], (H, d_c)), rtol=1e-15)
    np.testing.assert_allclose(lse[0, 0], scale * (qa[0, 0] @ c[0][0] + qr[0, 0] @ k[0][0]), rtol=1e-13)
    s01 = scale * (qa[0, 1] @ c[0][:2].T + qr[0, 1] @ k[0][:2].T)                     # [H, 2]
    w = np.exp(s01 - s01.max(1, keepdims=True)); w /= w.sum(1, keepdims=True)
    np.testing.assert_allclose(o[0, 1], w @ c[0][:2], rtol=1e-13, atol=1e-14)
    # zero queries: token i averages the first L - (T-1-i) rows, lse = log of that count
    L = 9
    c = [f32(r.standard_normal((L, d_c)))]
    k = [f32(r.standard_normal((L, d_r)))]
    pool, table, sl = dense_cache(c, k, page_size=4)
    o, lse = oracle.decode_absorbed_multi(np.zeros((1, T, H, d_c)), np.zeros((1, T, H, d_r)), pool, None, table, sl, scale)
    for i in range(T):
        n = L - (T - 1 - i)
        np.testing.assert_allclose(o[0, i], np.broadcast_to(c[0][:n].mean(0), (H, d_c)), rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(lse[0, i], math.log(n), rtol=1e-14)
    # fewer cached rows than query tokens: the tokens before position 0 see nothing
    sl2 = np.array([2], dtype=np.int32)
    o, lse = oracle.decode_absorbed_multi(qa, qr, pool, None, table, sl2, scale)
    assert (o[0, 0] == 0).all() and np.isneginf(lse[0, 0]).all()
    np.testing.assert_allclose(o[0, 1], np.broadcast_to(c[0][0], (H, d_c)), rtol=1e-15)
    assert np.isfinite(lse[0, 1:]).all()


def test_M4_later_rows_do_not_reach_an_earlier_token_and_its_own_row_does():
    T = 3
    cs = _multi_case(T, (8,), page_size=4, seed=8)
    _, o, lse, _ = _multi_chain(cs)
    L = 8
    for i in range(T):
        t_i = L - T + i
        # overwrite every row after t_i: token i must not move by a bit
        c2 = [cs["c"][0].copy()]; k2 = [cs["k"][0].copy()]
        c2[0][t_i + 1:] = 1e6; k2[0][t_i + 1:] = -1e6
        pool2, table2, sl2 = dense_cache(c2, k2, 4, seed=8)
        cs2 = dict(cs, c=c2, k=k2, pool=pool2, table=table2, sl=sl2)
        _, o2, lse2, _ = _multi_chain(cs2)
        assert np.array_equal(o2[0, i], o[0, i]) and np.array_equal(lse2[0, i], lse[0, i])
        # overwrite its own row: it must move (the limit is inclusive)
        c3 = [cs["c"][0].copy()]; c3[0][t_i] += 1.0
        pool3, table3, sl3 = dense_cache(c3, cs["k"], 4, seed=8)
        _, o3, _, _ = _multi_chain(dict(cs, c=c3, pool=pool3, table=table3, sl=sl3))
        assert np.abs(o3[0, i] - o[0, i]).max() > 1e-3


# ---------------------------------------------------------------------------
# F: prefill in the MHA paradigm (Eq. "mha" with keys and values materialised per head)
# ---------------------------------------------------------------------------

def _prefill(cs):
    return oracle.prefill_explicit(cs["qn"], cs["qr"], cs["Wk"], cs["Wv"], cs["pool"], None, cs["table"],
                                   cs["sl"], cs["scale"], cs["d_c"])


def test_F1_prefill_scalar_brute_force():
    """Pure-Python scalar evaluation of Eq. "mha" with exactly rounded sums, every query token with
    its own upper limit j <= t_i."""
    T, lens = 3, (5, 3, 2)
    cs = _multi_case(T, lens, page_size=2, seed=11)
    out, lse = _prefill(cs)
    B, _, H, d_head = cs["qn"].shape
    for b, L in enumerate(lens):
        for h in range(H):
            keys, vals = [], []
            for j in range(L):
                cj = [float(x) for x in cs["c"][b][j]]
                kc = [math.fsum(float(cs["Wk"][h, d, c]) * cj[c] for c in range(cs["d_c"])) for d in range(d_head)]
                keys.append(kc + [float(x) for x in cs["k"][b][j]])
                vals.append([math.fsum(cj[c] * float(cs["Wv"][h, c, d]) for c in range(cs["d_c"])) for d in range(d_head)])
            for i in range(T):
                vis = max(0, L - (T - 1 - i))
                q = [float(x) for x in cs["qn"][b, i, h]] + [float(x) for x in cs["qr"][b, i, h]]
                sc = [cs["scale"] * math.fsum(q[d] * keys[j][d] for d in range(len(q))) for j in range(vis)]
                if vis == 0:
                    assert (out[b, i, h] == 0).all() and np.isneginf(lse[b, i, h])
                    continue
                m = max(sc)
                e = [math.exp(x - m) for x in sc]
                z = math.fsum(e)
                want = [math.fsum(e[j] / z * vals[j][d] for j in range(vis)) for d in range(d_head)]
                np.testing.assert_allclose(out[b, i, h], want, rtol=1e-12, atol=1e-13)
                np.testing.assert_allclose(lse[b, i, h], m + math.log(z), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("T,lens,page_size,seed", [(1, (6, 2), 2, 0), (4, (9, 4, 6), 4, 1), (7, (7, 12), 3, 2)])
def test_F2_prefill_equals_the_absorbed_form(T, lens, page_size, seed):
    """Sec. 3.3: the two paradigms compute the same function (the Absorb operation only moves
    W^{UK} to the query side and W^{UV} behind the sum)."""
    cs = _multi_case(T, lens, page_size=page_size, seed=seed)
    out, lse = _prefill(cs)
    _, _, lse_abs, out_abs = _multi_chain(cs)
    np.testing.assert_allclose(out, out_abs, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(lse, lse_abs, rtol=1e-12, atol=1e-12)


def test_F3_whole_prompt_against_the_tensor_library_causal_attention():
    """T = L (prefill of a whole prompt) is textbook causal self-attention over the materialised
    keys and values: checked against torch's scaled_dot_product_attention(is_causal=True) in fp64.
    T = 1 is the one-token explicit decode (pinned separately)."""
    import torch
    L = 11
    cs = _multi_case(L, (L, L), H=2, page_size=4, seed=21)
    out, _ = _prefill(cs)
    for b in range(2):
        for h in range(2):
            K = torch.from_numpy(np.concatenate([cs["c"][b] @ cs["Wk"][h].T, cs["k"][b]], axis=1))
            V = torch.from_numpy(cs["c"][b] @ cs["Wv"][h])
            Q = torch.from_numpy(np.concatenate([cs["qn"][b, :, h], cs["qr"][b, :, h]], axis=1))
            want = torch.nn.functional.scaled_dot_product_attention(Q[None], K[None], V[None], is_causal=True,
                                                                    scale=cs["scale"])[0].numpy()
            np.testing.assert_allclose(out[b, :, h], want, rtol=1e-10, atol=1e-11)
    cs1 = _multi_case(1, (6, 3), page_size=2, seed=22)
    out1, lse1 = _prefill(cs1)
    want, want_lse = oracle.decode_explicit(cs1["qn"][:, 0], cs1["qr"][:, 0], cs1["Wk"], cs1["Wv"], cs1["pool"], None,
                                            cs1["table"], cs1["sl"], cs1["scale"], cs1["d_c"])
    np.testing.assert_allclose(out1[:, 0], want, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse1[:, 0], want_lse, rtol=1e-13, atol=1e-14)
