"""mla_decode_paged_static (scratch in the library's static device array, no allocation) against
mla_decode_paged (caller's workspace), through the C-ABI: two calls in a row, the second on a
smaller input, so that what the first left in the array must not reach the second's result."""
import numpy as np
import pytest

import oracle
from helpers import DeviceWorkload, lse_err, max_abs_rel, storage_bits, widen_gpu
from workloads import synth

pytestmark = pytest.mark.gpu


def _both(mla, w, num_splits, flags=0):
    import torch
    d = DeviceWorkload(w)
    q_abs = mla.absorb_q(d.q_nope, d.W_UK)
    want_o, want_lse = mla.decode_paged(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                                        num_splits=num_splits, kv_scale=d.kv_scale, return_lse=True, flags=flags)
    got_o = torch.full_like(want_o, float("nan"))
    got_lse = torch.full_like(want_lse, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    mla.decode_paged_static(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale, got_o,
                            num_splits=num_splits, kv_scale=d.kv_scale, lse=got_lse, flags=flags)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before   # the binding allocated nothing either
    return q_abs, want_o, want_lse, got_o, got_lse


def test_static_scratch_decode_matches_the_workspace_call_twice_in_a_row():
    import torch
    assert torch.cuda.is_available()
    from paper_2502_07864_amd import mla
    mla.lib()
    torch.cuda.set_device(0)
    # first call: the headline shape, shrunk in context only (16 sequences x 32 heads x 16 chunks: the
    # full 17.9 MB of partials); second call: a smaller, ragged batch with fewer chunks, whose partial
    # slots lie inside the region the first call filled
    big = synth.make_workload("static-big", B=16, H=32, d_head=128, d_c=512, d_rope=64, seq_lens=[2048] * 16,
                              io_dtype="bf16", cache_dtype="bf16", placement="random", num_splits=16, seed=76)
    small = synth.make_workload("static-small", B=3, H=32, d_head=128, d_c=512, d_rope=64,
                                seq_lens=[700, 65, 1], io_dtype="bf16", cache_dtype="bf16",
                                placement="random", free_frac=0.2, max_pages_per_seq=16, seed=77)
    for w, splits in ((big, big.num_splits), (small, 4)):
        q_abs, want_o, want_lse, got_o, got_lse = _both(mla, w, splits)
        # same kernels, same partial layout: the two entry points agree bit for bit
        assert storage_bits(got_o).tobytes() == storage_bits(want_o).tobytes()
        assert storage_bits(got_lse).tobytes() == storage_bits(want_lse).tobytes()
        # and both meet the oracle's bar
        qa = storage_bits(q_abs)
        ref_o, ref_lse = oracle.decode_absorbed(qa, w.q_rope, w.pool, w.kv_scale, w.page_table, w.seq_lens,
                                                w.softmax_scale)
        assert max_abs_rel(widen_gpu(got_o), ref_o) <= 2e-2
        assert lse_err(widen_gpu(got_lse), ref_lse) <= 2e-2


def test_static_scratch_decode_rejects_what_does_not_fit():
    import torch
    from paper_2502_07864_amd import mla
    # 64 sequences x 17 slots x 32 heads x 513 floats = 71 MB
    w = synth.make_workload("static-wide", B=64, H=32, d_head=128, d_c=512, d_rope=64, seq_lens=[64] * 64,
                            io_dtype="bf16", cache_dtype="bf16", placement="random", seed=78)
    d = DeviceWorkload(w)
    q_abs = mla.absorb_q(d.q_nope, d.W_UK)
    out = torch.zeros_like(q_abs)
    assert mla.decode_workspace_bytes(w.B, w.H, w.d_c, 16) > mla.static_scratch_bytes()
    with pytest.raises(mla.MlaError) as e:
        mla.decode_paged_static(q_abs, d.q_rope, d.pool, d.page_table, d.seq_lens, w.softmax_scale, out,
                                num_splits=16)
    assert e.value.status == -7 and "SCRATCH" in str(e.value)
    torch.cuda.synchronize()
    assert not out.any()                             # nothing was launched
