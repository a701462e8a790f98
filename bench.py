#!/usr/bin/env python3
"""Benchmark of the absorbed MLA decode step on one MI355X.

A step = mla_absorb_q -> mla_decode_paged (split-KV kernel, partials left in the
workspace) -> mla_merge_out_proj (split-KV merge + W_UV, fused) on one stream, for one batch of synthetic input already resident
in HBM.  Workload: LLaMA-2-7B-shaped converted layer, batch 16, every
sequence at context 8192, bf16 storage / fp32 accumulate, 64-token pages in a
random physical order (H=32, d_head=128, d_c=512, d_rope=64).

The timed loop cycles over several distinct copies of the cache so every step
streams its 151 MB from HBM rather than from the 256 MB last-level cache.

Prints ONE JSON line: us/step for the whole step, plus
  roofline     - the split-KV decode kernel against the 8 TB/s HBM peak,
                 its launches timed with events on the launch stream (mean of
                 back-to-back launches; kernels_us holds the per-step event
                 brackets, which include the gap around a single launch);
  cpu_baseline - the fp64 CPU oracle timed on a bounded sample (reported
                 baseline only).
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

HBM_PEAK_GBPS = 8000.0

METRICS = {
    "C2": "MLA decode us/step (absorb + paged split-KV decode + out-proj), bs16 ctx8K bf16, 1 GPU",
    "C1": "MLA decode us/step, bs1 ctx1K fp32, 1 GPU",
    "C3": "MLA decode us/step, bs64 ctx U[1K,32K] bf16, 1 GPU",
    "C4": "MLA decode us/step, bs128 ctx4K H28 d_c256 bf16, 1 GPU",
    "C5": "MLA decode us/step, bs4 ctx128K fp8 cache, 1 GPU",
}
WORKLOADS = {
    "C2": "C2: LLaMA-2-7B-shaped converted layer, batch 16 x context 8192, H=32 d_head=128 d_c=512 "
          "d_rope=64, bf16 cache in 64-token pages (random placement), 16 KV chunks per sequence",
    "C1": "C1: batch 1 x context 1024, H=32 d_c=512 d_rope=64, fp32 cache and io, identity page table",
    "C3": "C3: batch 64, context uniform in [1024, 32768], bf16, random placement with 10% of the pool free",
    "C4": "C4: batch 128 x context 4096, H=28 d_c=256 d_rope=64, bf16",
    "C5": "C5: batch 4 x context 131072, fp8 e4m3 cache with one fp32 scale per token, 32 KV chunks",
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults long enough for the clocks to settle: a step is tens of microseconds, and with 200 steps
    # behind 20 the timed region (8 ms at C2) still sat on the ramp (C2 41.0 against 39.2 us/step, C5
    # 86.6 against 75.2 with these counts on the same box)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--copies", type=int, default=0,
                    help="distinct cache copies cycled through (0 = enough to exceed 900 MB)")
    ap.add_argument("--unfused-tail", action="store_true",
                    help="merge and out-projection as two calls instead of mla_merge_out_proj")
    ap.add_argument("--splits", type=int, default=0, help="override the configuration's KV chunk count")
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C4", "C5"],
                    help="C2 is the headline configuration; the others are secondary rows")
    ap.add_argument("--partition", default="auto", choices=["auto", "uniform", "balanced"],
                    help="uniform: equal chunks per sequence; balanced (MLA_FLAG_BALANCED): equal page ranges "
                         "per workgroup over the concatenated sequences, --splits workgroups per sequence on "
                         "average; auto: balanced with 4 per sequence for the ragged batch C3, uniform otherwise")
    ap.add_argument("--q-len", type=int, default=1,
                    help="query tokens per sequence and step (multi-token prediction / speculative decoding); "
                         "above 1 the step uses mla_decode_paged_multi and mla_merge_out_proj_multi and is a "
                         "secondary row, not the headline metric")
    ap.add_argument("--prefill-len", type=int, default=0,
                    help="instead of the decode step, time mla_prefill_mha (MHA paradigm: keys and values "
                         "materialised per head, causal attention) for this many newest tokens of every sequence "
                         "of the workload (-1: the whole prompt); secondary row, MFMA roofline")
    ap.add_argument("--convert", action="store_true",
                    help="secondary row: the offline GQA->MLA conversion of one LLaMA-2-7B-shaped layer (fp64) "
                         "instead of the decode step")
    ap.add_argument("--convert-iters", type=int, default=20, help="block power iterations of the joint basis")
    ap.add_argument("--freqfold", type=int, default=2, help="FreqFold group size M of the conversion")
    ap.add_argument("--convert-keep", type=int, default=1,
                    help="components per FreqFold group that stay under RoPE: the RoPE key is keep * 128 / M wide "
                         "(default M = 2, keep = 1: 64, the decode path's 512 + 64 row)")
    ap.add_argument("--convert-block", type=int, default=768,
                    help="block width p of the power iteration (>= r_kv = 512; 768 with 20 iterations reaches a smaller "
                         "residual than 576 with 60 in 70 %% of the time on the synthetic spectrum)")
    ap.add_argument("--convert-products-only", action="store_true",
                    help="with --convert: only the two large fp64 products of the layer shape (moment C^T C and S Q), "
                         "a few launches each, for counter passes of the profiler")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=16, help="sequences in the CPU-oracle sample")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch the page-gather kernel (a plain copy of the whole cache, "
                         "known size) so hardware byte counters can be scaled against it")
    ap.add_argument("--traffic-json", default=str(ROOT / "profiles" / "decode_traffic.json"),
                    help="HBM traffic per launch of the decode kernels from rocprofv3 counters, per workload, if recorded")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (collectives and sharding are not part "
              "of it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from workloads.device import DeviceWorkload
    from paper_2502_07864_amd import mla
    from workloads import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    mla.lib()

    if args.prefill_len:
        return prefill_main(args)
    if args.convert:
        return convert_main(args)
    args.balanced = args.partition == "balanced" or (args.partition == "auto" and args.workload == "C3")
    if args.balanced and args.partition == "auto" and not args.splits:
        args.splits = 4          # 64 sequences x 4 = one workgroup per CU
    w = synth.config(args.workload)
    d = DeviceWorkload(w, "cuda:0")
    B, H, d_c, S = w.B, w.H, w.d_c, (args.splits or w.num_splits)
    io_t = torch.bfloat16 if w.io_dtype == "bf16" else torch.float32
    if args.copies <= 0:
        args.copies = max(2, min(6, -(-900_000_000 // max(1, w.cache_bytes_per_step))))
    # distinct HBM copies of cache + page table (copy i: pages rotated by i within the pool)
    pools, tables, scales = [], [], []
    for i in range(max(1, args.copies)):
        if i == 0:
            pools.append(d.pool)
            tables.append(d.page_table)
            scales.append(d.kv_scale)
        else:
            shift = (i * 977) % w.num_pages
            pools.append(torch.roll(d.pool, shifts=shift, dims=0).contiguous())
            shifted = torch.where(d.page_table >= 0, (d.page_table + shift) % w.num_pages, d.page_table)
            tables.append(shifted.to(torch.int32).contiguous())
            scales.append(None if d.kv_scale is None else torch.roll(d.kv_scale, shifts=shift, dims=0).contiguous())
    T = args.q_len
    assert T >= 1
    ws = torch.empty(mla.decode_workspace_bytes(B, T * H, d_c, S), dtype=torch.uint8, device="cuda:0")
    bal = mla.FLAG_BALANCED if args.balanced else 0
    if T == 1:
        q_abs = torch.empty((B, H, d_c), dtype=io_t, device="cuda:0")
        o_lat = torch.empty((B, H, d_c), dtype=io_t, device="cuda:0")
        out = torch.empty((B, H, w.d_head), dtype=io_t, device="cuda:0")
        q_nope, q_rope = d.q_nope, d.q_rope
        absorb = lambda: mla.absorb_q(q_nope, d.W_UK, out=q_abs)
        decode = mla.decode_paged
        def tail():
            if args.unfused_tail:
                mla.merge_partials(ws, B, H, d_c, S, io_t, out=o_lat, flags=bal)
                mla.out_proj(o_lat, d.W_UV, out=out)
            else:
                mla.merge_out_proj(ws, d.W_UV, B, S, o_lat=o_lat, out=out, flags=bal)
    else:
        # the q_len newest tokens of every sequence query the cache at once; their own rows are
        # the last q_len rows the cache already holds
        from workloads.device import to_torch
        qn, qr = synth.multi_queries(w, T)
        q_nope, q_rope = to_torch(qn, w.io_dtype, "cuda:0"), to_torch(qr, w.io_dtype, "cuda:0")
        q_abs = torch.empty((B, T, H, d_c), dtype=io_t, device="cuda:0")
        o_lat = torch.empty((B, T, H, d_c), dtype=io_t, device="cuda:0")
        out = torch.empty((B, T, H, w.d_head), dtype=io_t, device="cuda:0")
        absorb = lambda: mla.absorb_q(q_nope.view(B * T, H, w.d_head), d.W_UK, out=q_abs.view(B * T, H, d_c))
        decode = mla.decode_paged_multi
        def tail():
            if args.unfused_tail:
                mla.merge_partials(ws, B, T * H, d_c, S, io_t, out=o_lat.view(B, T * H, d_c), flags=bal)
                mla.out_proj(o_lat.view(B * T, H, d_c), d.W_UV, out=out.view(B * T, H, w.d_head))
            else:
                mla.merge_out_proj_multi(ws, d.W_UV, B, T, S, o_lat=o_lat, out=out, flags=bal)

    def step(i, events=None):
        k = i % len(pools)
        absorb()
        if events is not None:
            events[0].record()
        decode(q_abs, q_rope, pools[k], tables[k], d.seq_lens, w.softmax_scale,
               num_splits=S, kv_scale=scales[k], workspace=ws, flags=mla.FLAG_SKIP_MERGE | bal)
        if events is not None:
            events[1].record()
        tail()
        if events is not None:
            events[2].record()

    if args.calib_copy:
        for _ in range(3):
            mla.gather_paged(d.pool, d.page_table, d.seq_lens, int(w.seq_lens.max()))
        torch.cuda.synchronize()

    # untimed: the warm-up steps asked for, and as many more as it takes to have about 500 behind the
    # timed region (the clocks settle over tens of milliseconds of load; see the note at --steps)
    settle_steps = max(0, 500 - args.warmup)
    for i in range(args.warmup + settle_steps):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    assert torch.isfinite(out.float()).all()

    # second pass over the same steps with events around the decode kernel and the merge
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for i in range(args.steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    dec_us = np.array([e[0].elapsed_time(e[1]) * 1e3 for e in evs])
    mrg_us = np.array([e[1].elapsed_time(e[2]) * 1e3 for e in evs])

    # third pass: the decode kernel alone, launched back to back between two events on the same
    # stream (same cache rotation).  The per-step events above also contain the gap the event
    # packets themselves add around a single launch; this average does not, and it is the one the
    # roofline uses (it is the figure a kernel trace reports as the kernel's average duration).
    def decode_only(i):
        k = i % len(pools)
        decode(q_abs, q_rope, pools[k], tables[k], d.seq_lens, w.softmax_scale,
               num_splits=S, kv_scale=scales[k], workspace=ws, flags=mla.FLAG_SKIP_MERGE | bal)
    for i in range(min(args.warmup, 10)):
        decode_only(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        decode_only(i)
    e1.record()
    torch.cuda.synchronize()
    dec_b2b_us = e0.elapsed_time(e1) * 1e3 / args.steps

    # fourth pass: the whole mla_decode_paged call (split-KV kernel + merge kernel), back to back
    def decode_call(i):
        k = i % len(pools)
        decode(q_abs, q_rope, pools[k], tables[k], d.seq_lens, w.softmax_scale,
               num_splits=S, kv_scale=scales[k], workspace=ws, out=o_lat, flags=bal)
    for i in range(min(args.warmup, 10)):
        decode_call(i)
    e0.record()
    for i in range(args.steps):
        decode_call(i)
    e1.record()
    torch.cuda.synchronize()
    dec_call_us = e0.elapsed_time(e1) * 1e3 / args.steps

    # the bf16 stream kernel's launch shape with everything but the tile traffic taken out (same
    # grid, ring, requests, waits and barriers; no query rows, arithmetic or output): what reading
    # the cached rows once costs in this shape, the floor the decode kernel's time is read against
    stream_only_us = None
    if (w.io_dtype == "bf16" and w.cache_dtype == "bf16" and T == 1 and not args.balanced
            and 2 * (-(-d.page_table.shape[1] // S)) <= 32):
        def probe(i):
            k = i % len(pools)
            mla.diag_stream_tiles(pools[k], tables[k], d.seq_lens, S)
        for i in range(min(args.warmup, 10)):
            probe(i)
        e0.record()
        for i in range(args.steps):
            probe(i)
        e1.record()
        torch.cuda.synchronize()
        stream_only_us = e0.elapsed_time(e1) * 1e3 / args.steps

    # last pass (after everything above, it overwrites B cache rows): the cache-append call that
    # produces the next token's row, model dimension 4096, back to back
    append = None
    if w.io_dtype == "bf16":
        D_MODEL = 4096
        g = torch.Generator(device="cuda:0").manual_seed(1)
        xa = torch.randn((B, D_MODEL), generator=g, device="cuda:0").to(torch.bfloat16)
        Wa = (torch.randn((D_MODEL, d_c + w.d_rope), generator=g, device="cuda:0") / D_MODEL ** 0.5).to(torch.bfloat16)
        pos = torch.clamp(d.seq_lens - 1, min=0).to(torch.int32)
        aws = torch.empty(max(16, mla.append_workspace_bytes(B, D_MODEL, d_c, w.d_rope)), dtype=torch.uint8, device="cuda:0")
        def append_call():
            mla.cache_append(xa, Wa, pools[0], tables[0], pos, d_c, kv_scale=scales[0], workspace=aws)
        for _ in range(5):
            append_call()
        torch.cuda.synchronize()
        # the call is two short kernels: launched one by one the host cannot keep the GPU busy, so
        # 20 calls are captured into a HIP graph (the library allocates nothing and enqueues only
        # kernels on the current stream) and the graph is replayed
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            append_call()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(20):
                    append_call()
        torch.cuda.synchronize()
        reps = max(1, args.steps // 20)
        graph.replay()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        a_us = e0.elapsed_time(e1) * 1e3 / (reps * 20)
        a_bytes = Wa.numel() * 2 + xa.numel() * 2
        append = {"us": round(a_us, 2), "model_dim": D_MODEL, "weight_and_input_bytes": a_bytes,
                  "hbm_frac": round(a_bytes / (a_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                  "note": "mla_cache_append (projection + RoPE + store of one row per sequence), two kernels, "
                          "20 calls per HIP graph replay; not part of the step"}

    cache_bytes = w.cache_bytes_per_step                      # C2: 1152 B x 131072 tokens
    dec_avg_us = float(dec_b2b_us)
    achieved = cache_bytes / (dec_avg_us * 1e-6) / 1e9
    # which kernel mla_decode_paged launches for this call (the library's dispatch rule, restated)
    fp8 = w.cache_dtype == "fp8_e4m3"
    if w.io_dtype != "bf16":
        kernel_name = "decode_portable_kernel<float, float>"
    elif T > 1:
        kernel_name = f"decode_mfma_wide_kernel<{d_c}>"
    elif fp8:
        kernel_name = f"decode_stream_fp8_kernel<{d_c}, {'true' if args.balanced else 'false'}>"
    elif args.balanced:
        tiles = 2 * d.page_table.shape[1] // max(1, S)
        kernel_name = (f"decode_stream_kernel<{d_c}, false, true>" if d_c == 512 else
                       f"decode_mfma_kernel<{d_c}, {'3' if tiles <= 64 else '4'}, 1, true>")
    else:
        tiles = 2 * (-(-d.page_table.shape[1] // S))
        kernel_name = (f"decode_stream_kernel<{d_c}, false, false>" if (d_c == 512 or tiles <= 32) else
                       f"decode_mfma_kernel<{d_c}, {'3' if tiles <= 64 else '4'}, 1, false>")
    # HBM bytes per launch from the committed rocprofv3 counter summary; only valid for the default
    # launch configuration of the workload and while the kernel sources are the ones the counters
    # were taken on
    traffic, traffic_source = None, None
    tp = Path(args.traffic_json)
    default_config = args.partition == "auto" and T == 1 and not args.unfused_tail and S == (4 if args.workload == "C3" else w.num_splits)
    if tp.exists() and default_config:
        try:
            import hashlib
            tj = json.loads(tp.read_text()).get(args.workload)
            if tj and tj.get("kernel") == kernel_name:
                csrc = ROOT / "paper_2502_07864_amd" / "csrc"
                same = all(hashlib.sha256((csrc / f).read_bytes()).hexdigest()[:16] == h
                           for f, h in tj.get("source_sha256_16", {}).items())
                if same:
                    traffic = tj.get("hbm_bytes_per_launch")
                    traffic_source = ("rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE (one pass each), scaled by the page-gather "
                                      f"copy of the same run; {tj.get('summary')}")
                else:
                    traffic_source = "null: the kernel source has changed since the counters in profiles/decode_traffic.json were taken"
        except Exception:
            traffic, traffic_source = None, None

    rec = {
        "metric": METRICS[args.workload] + (f", {T} query tokens per sequence" if T > 1 else ""),
        "value": round(ms_per_step * 1e3, 3),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_steps": settle_steps,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.io_dtype == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": WORKLOADS[args.workload],
                   "batch": B, "context_max": int(w.seq_lens.max()), "tokens": w.tokens,
                   "cache_dtype": w.cache_dtype, "num_splits": S, "cache_copies_cycled": len(pools),
                   "partition": "balanced" if args.balanced else "uniform", "q_len": T},
        "tokens_per_s": round(B * T / (ms_per_step * 1e-3), 1),
        "step_hbm_GBps": round(cache_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "step_hbm_frac": round(cache_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "decode_call_us": round(float(dec_call_us), 2),
        "decode_call_hbm_frac": round(cache_bytes / (dec_call_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
        "kernels_us": {"decode_split_kv": {"avg": round(float(dec_us.mean()), 2),
                                           "p10": round(float(np.percentile(dec_us, 10)), 2),
                                           "p50": round(float(np.percentile(dec_us, 50)), 2),
                                           "p90": round(float(np.percentile(dec_us, 90)), 2)},
                       ("merge+out_proj" if args.unfused_tail else "merge_out_proj_fused"):
                           {"avg": round(float(mrg_us.mean()), 2)}},
        "roofline": {"bound": "hbm", "kernel": kernel_name,
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": cache_bytes,
                     "launch_us": round(dec_avg_us, 2),
                     "timing": f"mean of {args.steps} back-to-back launches between two HIP events on the launch stream"},
    }

    if stream_only_us is not None:
        rec["roofline"]["stream_only"] = {
            "kernel": f"decode_stream_kernel<{d_c}, true, false>", "launch_us": round(float(stream_only_us), 2),
            "frac": round(cache_bytes / (stream_only_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
            "note": "mla_diag_stream_tiles: the decode kernel's grid, tile ring, loads, waits and barriers with no "
                    "arithmetic and no output, back to back like launch_us"}
    if append is not None:
        rec["cache_append"] = append

    if not args.no_cpu_baseline and T > 1:
        import oracle
        n = max(1, min(args.cpu_seqs, B))
        t0 = time.perf_counter()
        qa = oracle.absorb_q(qn[:n].reshape(n * T, H, w.d_head), w.W_UK).reshape(n, T, H, d_c)
        o64, _ = oracle.decode_absorbed_multi(qa, qr[:n], w.pool, w.kv_scale, w.page_table[:n], w.seq_lens[:n],
                                              w.softmax_scale)
        oracle.out_proj(o64.reshape(n * T, H, d_c), w.W_UV)
        t_cpu = time.perf_counter() - t0
        rec["cpu_baseline"] = {
            "value": round(t_cpu * (B / n) * 1e6, 1), "unit": "us/step", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{n} of {B} sequences, {T} query tokens each, fp64 absorbed oracle (absorb + decode + "
                      f"out-proj), one run = {t_cpu:.2f} s, scaled by {B}/{n}"}
    elif not args.no_cpu_baseline:
        import oracle
        n = max(1, min(args.cpu_seqs, B))
        sel = np.arange(n)
        times = []
        for _ in range(3):
            t0 = time.perf_counter()
            oracle.mla_step(w.q_nope[sel], w.q_rope[sel], w.W_UK, w.W_UV, w.pool, w.kv_scale,
                            w.page_table[sel], w.seq_lens[sel], w.softmax_scale)
            times.append(time.perf_counter() - t0)
        t_cpu = sorted(times)[1]
        # the same routine on one thread, one sequence (bounded: a few tenths of a second at C2)
        oracle.set_num_threads(1)
        t0 = time.perf_counter()
        oracle.mla_step(w.q_nope[:1], w.q_rope[:1], w.W_UK, w.W_UV, w.pool, w.kv_scale,
                        w.page_table[:1], w.seq_lens[:1], w.softmax_scale)
        t_one = time.perf_counter() - t0
        oracle.set_num_threads(0)
        tok1 = max(1, int(w.seq_lens[0]))
        rec["cpu_baseline"] = {
            "value": round(t_cpu * (B / n) * 1e6, 1), "unit": "us/step",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n} of {B} sequences (all {H} heads, {int(w.seq_lens[sel].sum())} tokens), fp64 absorbed oracle "
                      f"(absorb + decode + out-proj), median of 3 runs = {t_cpu:.2f} s, scaled by {B}/{n}",
            "single_thread": {"value": round(t_one * (w.tokens / tok1) * 1e6, 1), "unit": "us/step", "cores": 1,
                              "sample": f"sequence 0 ({tok1} tokens, all {H} heads) = {t_one:.2f} s, scaled by tokens "
                                        f"{w.tokens}/{tok1}"}}
    print(json.dumps(rec))


def prefill_main(args):
    """Secondary row: the MHA-paradigm prefill call on the workload's cache."""
    import numpy as np
    import torch
    from workloads.device import DeviceWorkload, to_torch
    from paper_2502_07864_amd import mla
    from workloads import synth

    w = synth.config(args.workload)
    assert w.io_dtype == "bf16" and w.cache_dtype == "bf16", "prefill runs on bf16 caches"
    d = DeviceWorkload(w, "cuda:0")
    B, H = w.B, w.H
    T = int(w.seq_lens.max()) if args.prefill_len < 0 else args.prefill_len
    qn, qr = synth.multi_queries(w, T)
    qn_t, qr_t = to_torch(qn, "bf16", "cuda:0"), to_torch(qr, "bf16", "cuda:0")
    ws = torch.empty(mla.prefill_workspace_bytes(B, H, w.d_c, w.max_pages_per_seq), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((B, T, H, w.d_head), dtype=torch.bfloat16, device="cuda:0")

    def step():
        mla.prefill_mha(qn_t, qr_t, d.W_UK, d.W_UV, d.pool, d.page_table, d.seq_lens, w.softmax_scale,
                        workspace=ws, out=out)
    steps, warmup = max(1, min(args.steps, 20)), max(1, min(args.warmup, 3))
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    assert torch.isfinite(out.float()).all()
    # algorithmic flops (Eq. "mha"): per (query, visible key, head) 2 (d_head + d_rope) + 2 d_head;
    # materialisation per (key, head) 2 d_c * 2 d_head
    lens = w.seq_lens.astype(np.int64)
    i = np.arange(T, dtype=np.int64)
    visible = np.maximum(lens[:, None] - (T - 1 - i)[None, :], 0).sum()
    attn_flop = float(visible) * H * (2 * (w.d_head + w.d_rope) + 2 * w.d_head)
    mat_flop = float(lens.sum()) * H * 2 * w.d_c * 2 * w.d_head
    tflops = (attn_flop + mat_flop) / (ms * 1e-3) / 1e12
    rec = {"metric": f"MLA prefill ms (MHA paradigm: materialise + causal attention), {args.workload} cache, "
                     f"{T} newest tokens per sequence, 1 GPU",
           "value": round(ms, 3), "unit": "ms/step", "n_gpus": 1, "steps": steps, "warmup": warmup,
           "ms_per_step": round(ms, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": WORKLOADS[args.workload], "batch": B, "q_len": T, "heads": H,
                      "context_max": int(w.seq_lens.max())},
           "tokens_per_s": round(B * T / (ms * 1e-3), 1),
           "roofline": {"bound": "mfma", "kernel": "prefill_attention_kernel<3, 2> + prefill_materialise_kernel<512>",
                        "achieved": round(tflops, 1), "peak": 2500.0, "unit": "TFLOP/s",
                        "frac": round(tflops / 2500.0, 4), "traffic": None,
                        "algorithmic_flop_per_step": attn_flop + mat_flop,
                        "timing": "wall clock around the whole call (weights, materialisation, attention), "
                                  f"{steps} calls back to back"}}
    print(json.dumps(rec))


def convert_main(args):
    """Secondary row: offline conversion of one GQA layer to MLA (Sec. 4, App. B-D) in fp64."""
    import numpy as np
    import torch
    from paper_2502_07864_amd import convert as cv
    from workloads import synth

    g = h = 32
    d, D, n, r_kv, p = 128, 4096, 4096, 512, args.convert_block
    M, keep, iters = args.freqfold, args.convert_keep, args.convert_iters
    d_rope = keep * (d // M)
    mj = 2 * g * d - d_rope
    if args.convert_products_only:
        gen = torch.Generator(device="cuda:0").manual_seed(0)
        C = torch.randn((n, mj), dtype=torch.float64, device="cuda:0", generator=gen)
        one = torch.ones(1, dtype=torch.float64, device="cuda:0")
        Q = torch.randn((mj, p), dtype=torch.float64, device="cuda:0", generator=gen)
        aws = torch.empty(cv.apply_workspace_bytes(mj, p), dtype=torch.uint8, device="cuda:0")
        times = {}
        for name, call in (("moment", lambda: cv.joint_moment(C[:, :mj - g * d].contiguous(), C[:, mj - g * d:].contiguous(), one)),
                           ("S_Q", None)):
            if name == "moment":
                S, _ = call()
                call = None
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                if name == "moment":
                    cv.joint_moment(C[:, :mj - g * d].contiguous(), C[:, mj - g * d:].contiguous(), one)
                else:
                    cv.apply(S, Q, workspace=aws)
            e1.record()
            torch.cuda.synchronize()
            times[name] = e0.elapsed_time(e1) / 3
        print(json.dumps({"products_ms": times, "moment_TFLOPs": 2.0 * mj * mj * n / times["moment"] / 1e9,
                          "S_Q_TFLOPs": 2.0 * mj * mj * p / times["S_Q"] / 1e9}))
        return
    X, W_K, W_V = synth.calibration(n, D, g, d, seed=0)
    Q0 = synth.start_block(mj, p, seed=0)
    dev = lambda a: torch.from_numpy(a).to("cuda:0")
    Xd, Kd, Vd, Qd = dev(X), dev(W_K), dev(W_V), dev(Q0)
    ws = torch.empty(cv.lib().mla_convert_layer_workspace_bytes(n, D, g, h, d, M, keep, r_kv, p), dtype=torch.uint8, device="cuda:0")

    def step():
        return cv.convert_layer(Xd, Kd, Vd, Qd, g, h, d, M, r_kv, iters, workspace=ws, keep=keep)
    steps, warmup = max(1, min(args.steps, 5)), max(1, min(args.warmup, 2))
    for _ in range(warmup):
        out = step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        out = step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    info = out["info"].cpu().numpy()
    assert (info[:-2] >= 1).all() and info[-2] == 0 and info[-1] >= 1, f"conversion did not converge: {info}"

    # what was computed: orthonormal basis, and how far the r_kv Ritz pairs are from eigenpairs of the
    # moment matrix rebuilt here from the library's own step calls (S R - R diag(evals), column norms)
    U = out["U"]
    W_rot = cv.rotate_rows(Kd, U, g, d, M, keep)
    K_nope, V = cv.project(Xd, W_rot[d_rope:].contiguous()), cv.project(Xd, Vd)
    S, _ = cv.joint_moment(K_nope, V, out["alpha"])
    R, ev = out["R_KV"], out["evals_joint"][:r_kv]
    Rp = torch.zeros((mj, p), dtype=torch.float64, device="cuda:0")
    Rp[:, :r_kv] = R
    resid = (cv.apply(S, Rp)[:, :r_kv] - R * ev).norm(dim=0).max().item() / ev[0].item()
    orth = (R.T @ R - torch.eye(r_kv, dtype=torch.float64, device="cuda:0")).abs().max().item()
    captured = ev.sum().item() / torch.trace(S).item()

    # roofline of the dominant kernel: the fp64 matrix product S Q of the block power iteration,
    # timed alone between two events on the launch stream
    Y = torch.empty((mj, p), dtype=torch.float64, device="cuda:0")
    aws = torch.empty(cv.apply_workspace_bytes(mj, p), dtype=torch.uint8, device="cuda:0")
    reps = 20
    for _ in range(3):
        cv.apply(S, Qd, out=Y, workspace=aws)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        cv.apply(S, Qd, out=Y, workspace=aws)
    e1.record()
    torch.cuda.synchronize()
    launch_ms = e0.elapsed_time(e1) / reps
    flop = 2.0 * mj * mj * p
    tflops = flop / (launch_ms * 1e-3) / 1e12
    # algorithmic flop of the chain: activations, moments, iterations (S Q, Gram, Q = Y L^-T), projections
    gd = g * d
    chain_flop = (2.0 * n * D * gd + 2.0 * n * D * (gd - d_rope) + 2.0 * n * D * gd + 2.0 * mj * mj * n
                  + (iters + 1) * flop + (iters + 4) * 2 * (2.0 * mj * p * p)
                  + 2.0 * r_kv * D * mj + 2.0 * h * d * r_kv * (gd - d_rope))
    rec = {"metric": "GQA->MLA conversion of one LLaMA-2-7B-shaped layer, ms (fp64), 1 GPU",
           "value": round(ms, 2), "unit": "ms/layer", "n_gpus": 1, "steps": steps, "warmup": warmup,
           "ms_per_step": round(ms, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
           "dtype": "f64", "data": "synthetic",
           "config": {"workload": f"one layer g=h={g} d={d} D={D}, {n} synthetic calibration tokens, FreqFold M={M} with "
                                  f"{keep} RoPE pair(s) per group (RoPE key {d_rope} wide), r_kv={r_kv}, block width {p}, "
                                  f"{iters} block power iterations",
                      "g": g, "h": h, "d": d, "D": D, "n": n, "M": M, "keep": keep, "d_rope": d_rope, "r_kv": r_kv,
                      "p": p, "iters": iters},
           "chain_TFLOPs": round(chain_flop / (ms * 1e-3) / 1e12, 2),
           "checks": {"ritz_residual_over_lambda1": resid, "orthonormality": orth,
                      "captured_second_moment": round(captured, 6), "alpha": out["alpha"].item(),
                      "rope_basis_sweeps_max": int(info[:-2].max()), "ritz_sweeps": int(info[-1])},
           "roofline": {"bound": "mfma", "kernel": f"gemm_f64_kernel<true, false> (S Q, {mj} x {mj} x {p}, K range in slices) "
                                                   "+ gemm_f64_reduce_kernel",
                        "achieved": round(tflops, 2), "peak": 78.6, "unit": "TFLOP/s", "frac": round(tflops / 78.6, 4),
                        "traffic": None, "algorithmic_flop_per_launch": flop, "launch_us": round(launch_ms * 1e3, 1),
                        "timing": f"mean of {reps} back-to-back mla_conv_apply calls (product kernel, then the kernel "
                                  "that sums the slices) between two HIP events on the launch stream"}}
    if not args.no_cpu_baseline:
        # the numpy chain on a half-size layer (16 heads: moment matrix 3968 x 3968); the GPU chain on the
        # same sample is timed beside it (no scaling applied: the eigensolvers do not scale linearly)
        import oracle.convert_oracle as co
        g2 = h2 = 16
        D2, n2, r2, p2 = 2048, 4096, 256, 384
        X2, K2, V2 = synth.calibration(n2, D2, g2, d, seed=1)
        t0 = time.perf_counter()
        ref = co.convert_layer(X2, K2, V2, g2, h2, d, M, r2, keep)
        cpu_s = time.perf_counter() - t0
        Q2 = dev(synth.start_block(2 * g2 * d - d_rope, p2, seed=1))
        a2 = [dev(a) for a in (X2, K2, V2)]
        cv.convert_layer(*a2, Q2, g2, h2, d, M, r2, iters, keep=keep)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        got = cv.convert_layer(*a2, Q2, g2, h2, d, M, r2, iters, keep=keep)
        torch.cuda.synchronize()
        gpu_s = time.perf_counter() - t0
        ev_err = float(np.abs(got["evals_joint"][:r2].cpu().numpy() - ref["evals_joint"][:r2]).max() / ref["evals_joint"][0])
        import os
        rec["cpu_baseline"] = {"value": round(cpu_s * 1e3, 1), "unit": "ms/layer", "cores": os.cpu_count(), "kind": "oracle",
                               "sample": f"half-size layer g=h={g2} d={d} D={D2}, {n2} tokens, r_kv={r2} (not scaled); "
                                         f"GPU chain on the same sample: {gpu_s * 1e3:.1f} ms, eigenvalue gap to the "
                                         f"oracle {ev_err:.1e} of the largest"}
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
