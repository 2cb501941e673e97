#!/usr/bin/env python3
"""Benchmark of the SamKV hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--ratio R]

A step is one pass of the whole hot path (samkv_score, samkv_topk_select, samkv_gather,
samkv_recompute_attn, samkv_query_attn) over the per-document caches of one layer (for the
32-layer workload: over all 32 layers).  Inputs are seeded synthetic caches already resident in
HBM; enough distinct copies are rotated that the working set exceeds twice the 256 MB Infinity
Cache, so K is streamed from HBM and not from cache.  Prints ONE JSON line.

The timed region launches the calls eagerly and brackets only the dominant call with HIP events (its average
duration feeds the roofline figure); the per-call table comes from a second, untimed pass with every call
bracketed, and `hip_graph` repeats the timed steps as replays of captured HIP graphs.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix cores, published
FP32_VALU_PEAK_TFLOPS = 157.3
KERNELS = ("score", "select", "gather", "recompute_attn", "query_attn")          # the five entry points of the path
STEP = ("score_select_gather", "recompute_attn", "query_attn")                   # what a step launches: the first three fused
EXTRA = ("score_select",)                                                        # also timed per call, outside the step


def algorithmic_work(w, lens, m, n_q_tok):
    """Algorithmic bytes / flops of one pass over one layer (what the method itself must move or compute)."""
    e = 2 if w.dtype == "bf16" else 4
    tot, hkv, hq, d = sum(lens), w.n_kv_heads, w.n_q_heads, w.head_dim
    # score: every key row read once and one float32 written per token-head, plus the Q rows that Eq. 1 pools
    # (the user query's and every document's local Q cache), each read once
    q_rows = hq * n_q_tok + len(lens) * hq * w.w_loc
    return {
        "score": {"bytes": tot * hkv * (d * e + 4) + q_rows * d * e, "flops": 2 * d * tot * hkv},
        "select": {"bytes": tot * hkv * 4 + m * hkv * 4, "flops": 0},
        # fused: K and the Q rows read once, only the kept positions written (the scores stay on chip)
        "score_select": {"bytes": tot * hkv * d * e + q_rows * d * e + m * hkv * 4, "flops": 2 * d * tot * hkv},
        "gather": {"bytes": m * hkv * (4 * d * e + 4), "flops": 0},
        # score, selection and compaction in one call: the two above, the positions written once and read back on chip
        "score_select_gather": {"bytes": tot * hkv * d * e + q_rows * d * e + m * hkv * (4 * d * e + 4),
                                "flops": 2 * d * tot * hkv},
        "recompute_attn": {"bytes": (2 * hq + 2 * hkv) * m * d * e + hq * m * (d + 1) * 4,
                           "flops": 4 * hq * d * m * (m + 1) // 2},
        "query_attn": {"bytes": 2 * m * hkv * d * e + hq * n_q_tok * (d * e + (d + 1) * 4),
                       "flops": 4 * hq * d * n_q_tok * m},
    }


def read_traffic(workload, kernel: str):
    """HBM bytes per launch (read + write) of a kernel, from the committed rocprofv3 --pmc summary of this
    workload (profiles/bench_<workload>.txt: FETCH_SIZE and WRITE_SIZE runs scaled by a plain copy), or None."""
    prefixes = {"score": ["k_score<"], "select": ["k_select"], "gather": ["k_gather<"], "score_select": ["k_score_select"],
                "score_select_gather": ["k_score_select"],
                "recompute_attn": ["k_attn_%s<%d, true" % (workload.dtype, workload.head_dim), "k_attn_%s_dma<true" % workload.dtype],
                "query_attn": ["k_attn_%s<%d, false" % (workload.dtype, workload.head_dim), "k_attn_%s_dma<false" % workload.dtype],
                }[kernel]
    try:
        lines = open(os.path.join(ROOT, "profiles", f"bench_{workload.name}.txt")).read().splitlines()
    except OSError:
        return None
    for line in lines:
        if any(line.startswith(p) for p in prefixes):
            try:
                rd, wr = float(line.split()[-2]), float(line.split()[-1])
                return (rd + wr) * 1e6
            except ValueError:
                return None
    return None


def cpu_baseline(layer, ratio, n_sample_rows, budget_s=30.0):
    """Times the fp64 oracle (as it stands) on the host over the same layer; attention rows are sampled
    when the full computation would not fit the time budget, and extrapolated by pair count."""
    import numpy as np
    from oracle import samkv_oracle as O
    from paper_2508_11661_amd import synth

    w = layer.workload
    n = len(layer.k)
    scale = 1.0 / math.sqrt(w.head_dim)
    rng = np.random.default_rng(0)

    def one_pass():
        """One pass of the oracle over the layer; returns (extrapolated seconds, rows sampled or None, m, fraction)."""
        t0 = time.perf_counter()
        q_hat = O.personalized_query(layer.q_tok, layer.q_loc, n)
        scores = O.score(q_hat, layer.k)
        idx, cu_k = O.select(scores, ratio)
        k_c, v_c = O.gather(layer.k, layer.v, idx, cu_k)
        t_front = time.perf_counter() - t0
        m = int(cu_k[-1])
        q_rec = synth.make_q_rec(w, layer.layer, m)
        if n_sample_rows >= m:
            rows, frac = None, 1.0
        else:
            rows = np.unique(np.concatenate([[0, m - 1], rng.integers(0, m, size=n_sample_rows - 2)]))
            frac = float((rows + 1).sum()) / (m * (m + 1) / 2)
        t1 = time.perf_counter()
        O.attention(q_rec, k_c, v_c, scale, True, rows=rows)
        t_rec = (time.perf_counter() - t1) / frac
        t2 = time.perf_counter()
        O.attention(layer.q_tok, k_c, v_c, scale, False)
        t_q = time.perf_counter() - t2
        return t_front + t_rec + t_q, rows, m, frac

    # a small layer is timed over as many whole passes as about ten seconds hold, a large one over one sampled pass
    w0, c0 = time.perf_counter(), time.process_time()
    totals = []
    while True:
        total, rows, m, frac = one_pass()
        totals.append(total)
        spent = time.perf_counter() - w0
        if rows is not None or spent >= 10.0 or spent + spent / len(totals) > budget_s:
            break
    wall = time.perf_counter() - w0
    cores = max(1, round((time.process_time() - c0) / wall))
    total = sum(totals) / len(totals)
    sample = (f"whole layer, every step of the path, mean of {len(totals)} passes" if rows is None else
              f"score/select/gather/query attention in full; recompute attention on {len(rows)} of {m} rows per "
              f"head ({frac:.3%} of the causal pairs), time extrapolated by pair count")
    return {"value": sum(layer.lens) / total, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": sample, "seconds_measured": round(wall, 2), "ms_per_step_extrapolated": round(total * 1e3, 1)}


def measured_peaks(samkv, iters=7):
    """What this device sustains on a pure-MFMA loop (the bf16 32x32x16 product, 2 and 4 waves per SIMD) and on a
    plain 1 GiB streaming copy: the ceilings a kernel's rate can be read against besides the published peaks."""
    import torch

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(iters):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            work = fn()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return work, sorted(ts)[iters // 2]

    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    out = {}
    for wps in (2, 4):                       # waves per SIMD: a workgroup is 4 waves, one per SIMD
        flop, ms = timed(lambda: samkv.samkv_peak_mfma_bf16(sink, n_cu * wps, 4000 // wps))
        out[f"mfma_bf16_tflops_{wps}_waves_per_simd"] = round(flop / ms / 1e9, 1)
    out["mfma_bf16_tflops"] = max(v for k, v in out.items() if k.startswith("mfma"))
    # the same loop with pseudo-random operands (full mantissas): the device keeps inside its power limit by lowering
    # the clock, and real data toggle far more bits than small integers do.  Sustained figure: launches back to back
    # for about a quarter of a second before the timed ones.
    for _ in range(40):
        samkv.samkv_peak_mfma_bf16_data(sink, n_cu * 4, 1000, 2)
    flop, ms = timed(lambda: samkv.samkv_peak_mfma_bf16_data(sink, n_cu * 4, 1000, 2))
    out["mfma_bf16_tflops_random_operands"] = round(flop / ms / 1e9, 1)
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    nbytes, ms = timed(lambda: samkv.samkv_peak_copy(src, dst))
    out["copy_gbs_read_plus_write"] = round(nbytes / ms / 1e6, 1)
    nbytes, ms = timed(lambda: samkv.samkv_peak_read(src, sink))
    out["read_gbs"] = round(nbytes / ms / 1e6, 1)
    out["compute_units"] = n_cu
    return out


def at_scale(samkv, iters=5):
    """Kernel timings at the shapes of the largest workload (64 documents x 4096 tokens, 64/8 heads, d = 128,
    256 query tokens, 15 % budget), where the kernels are bandwidth- or MFMA-bound instead of latency-bound.
    Shapes only: device-generated Gaussian bf16 tensors, HIP-event timing, the same entry points.  This is
    context for the roofline fractions; the headline value above stays the timed workload's."""
    import torch
    w = __import__("paper_2508_11661_amd.synth", fromlist=["WORKLOADS"]).WORKLOADS["large_cache_stress"]
    g = torch.Generator(device="cuda").manual_seed(1234)
    rnd = lambda *shape: torch.randn(*shape, device="cuda", generator=g).to(torch.bfloat16)
    k = [rnd(w.n_kv_heads, w.ctx_len, w.head_dim) for _ in range(w.n_ctx)]
    v = [rnd(w.n_kv_heads, w.ctx_len, w.head_dim) for _ in range(w.n_ctx)]
    caches = samkv.Caches(k, v, w.n_q_heads)
    q_tok = rnd(w.n_q_heads, w.n_q_tok, w.head_dim)
    q_loc = rnd(w.n_ctx, w.n_q_heads, w.w_loc, w.head_dim)
    m = w.n_ctx * samkv.samkv_kept_count(w.ctx_len, 0.15)
    q_rec = rnd(w.n_q_heads, m, w.head_dim)
    buf = samkv.alloc_layer_buffers(caches, w.n_q_tok, 0.15)
    scale = 1.0 / math.sqrt(w.head_dim)
    calls = {
        "score": lambda: samkv.samkv_score(caches, q_tok, q_loc, buf.scores, buf.ws),
        "select": lambda: samkv.samkv_topk_select(buf.scores, caches, 0.15, 0, 0, buf.idx, buf.cu_k_dev, buf.ws),
        "gather": lambda: samkv.samkv_gather(caches, buf.idx, 0.15, buf.k_c, buf.v_c),
        "recompute_attn": lambda: samkv.samkv_recompute_attn(q_rec, buf.k_c, buf.v_c, scale, buf.rec_out, buf.rec_lse, buf.ws),
        "query_attn": lambda: samkv.samkv_query_attn(q_tok, buf.k_c, buf.v_c, scale, buf.q_out, buf.q_lse, buf.ws),
    }
    work = algorithmic_work(w, w.lens, m, w.n_q_tok)
    res = {"workload": w.name, "data": "device-generated Gaussian bf16, shapes only", "iters": iters}
    for name in KERNELS:                      # in path order, so select/gather/attention see real scores and indices
        calls[name]()
    torch.cuda.synchronize()
    for name in KERNELS:
        ev = []
        for _ in range(iters):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            calls[name]()
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        ms = sorted(x.elapsed_time(y) for x, y in ev)[iters // 2]
        res[name] = {"ms": round(ms, 4), "GB/s": round(work[name]["bytes"] / ms / 1e6, 1),
                     "TFLOP/s": round(work[name]["flops"] / ms / 1e9, 1),
                     "frac_hbm": round(work[name]["bytes"] / ms / 1e6 / HBM_PEAK_GBS, 4),
                     "frac_mfma": round(work[name]["flops"] / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)}
    ss_ms = res["score"]["ms"] + res["select"]["ms"]
    ss_bytes = work["score"]["bytes"] + m * w.n_kv_heads * 4
    ss_gbs = ss_bytes / ss_ms / 1e6
    res["score+select"] = {"ms": round(ss_ms, 4), "GB/s": round(ss_gbs, 1), "frac_hbm": round(ss_gbs / HBM_PEAK_GBS, 4)}
    fused = lambda: samkv.samkv_score_select(caches, q_tok, q_loc, 0.15, 0, 0, None, buf.idx, buf.cu_k_dev, buf.ws)
    fused()
    torch.cuda.synchronize()
    ev = []
    for _ in range(iters):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fused()
        b.record()
        ev.append((a, b))
    torch.cuda.synchronize()
    ms = sorted(x.elapsed_time(y) for x, y in ev)[iters // 2]
    res["score_select_fused"] = {"ms": round(ms, 4), "GB/s": round(ss_bytes / ms / 1e6, 1),
                                 "frac_hbm": round(ss_bytes / ms / 1e6 / HBM_PEAK_GBS, 4)}

    # the causal attention once more on all-zero operands: same instruction stream, far fewer bits toggling.  The
    # difference to the figure above is what the device's power limit costs on real data.
    zq, zk, zv = torch.zeros_like(q_rec), torch.zeros_like(buf.k_c), torch.zeros_like(buf.v_c)
    zcall = lambda: samkv.samkv_recompute_attn(zq, zk, zv, scale, buf.rec_out, buf.rec_lse, buf.ws)
    zcall()
    torch.cuda.synchronize()
    ev = []
    for _ in range(iters):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        zcall()
        b.record()
        ev.append((a, b))
    torch.cuda.synchronize()
    ms = sorted(x.elapsed_time(y) for x, y in ev)[iters // 2]
    res["recompute_attn_zero_operands"] = {"ms": round(ms, 4),
                                           "TFLOP/s": round(work["recompute_attn"]["flops"] / ms / 1e9, 1),
                                           "note": "same launch on all-zero Q, K, V: not power-limited"}
    del zq, zk, zv

    # block-level variant of the selection (64-token blocks, 1 initial + 2 local blocks forced, per-document share
    # 0.15 of the middle blocks), with and without the cross-document filter, and the gather that follows each
    block, p = 64, [0.15] * w.n_ctx
    nb = sum(-(-n // block) for n in w.lens)
    bs = torch.empty((w.n_kv_heads, nb), dtype=torch.float32, device="cuda")
    bws = torch.empty(samkv.samkv_block_workspace_bytes(caches, block), dtype=torch.uint8, device="cuda")
    samkv.samkv_block_scores(buf.scores, caches, block, bs)
    mb = samkv.samkv_block_select_count(caches, block, p, 1, 2)
    idx_b = torch.empty((w.n_kv_heads, mb), dtype=torch.int32, device="cuda")
    cu = samkv.samkv_block_select(bs, caches, block, p, 1, 2, idx_b, None, bws)
    mf = samkv.samkv_block_filter_count(caches, block, p, 1, 2)
    gidx = torch.empty((w.n_kv_heads, mf), dtype=torch.int32, device="cuda")
    kb, vb = (torch.empty((w.n_kv_heads, mb, w.head_dim), dtype=torch.bfloat16, device="cuda") for _ in range(2))
    kf, vf = (torch.empty((w.n_kv_heads, mf, w.head_dim), dtype=torch.bfloat16, device="cuda") for _ in range(2))
    row = w.head_dim * 2
    bcalls = {
        "block_scores": (lambda: samkv.samkv_block_scores(buf.scores, caches, block, bs), 4 * w.n_kv_heads * (sum(w.lens) + nb)),
        "block_select": (lambda: samkv.samkv_block_select(bs, caches, block, p, 1, 2, idx_b, None, bws), 4 * w.n_kv_heads * (nb + mb)),
        "gather_v": (lambda: samkv.samkv_gather_v(caches, idx_b, cu, kb, vb), w.n_kv_heads * mb * (4 * row + 4)),
        "block_select_filter": (lambda: samkv.samkv_block_select_filter(bs, caches, block, p, 1, 2, gidx, bws), 4 * w.n_kv_heads * (nb + mf)),
        "gather_g": (lambda: samkv.samkv_gather_g(caches, gidx, kf, vf), w.n_kv_heads * mf * (4 * row + 4)),
    }
    blk = {"block": block, "kept_tokens": mb, "kept_tokens_after_filter": mf}
    for name, (fn, nbytes) in bcalls.items():
        fn()
        torch.cuda.synchronize()
        ev = []
        for _ in range(iters):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        ms = sorted(x.elapsed_time(y) for x, y in ev)[iters // 2]
        blk[name] = {"ms": round(ms, 4), "GB/s": round(nbytes / ms / 1e6, 1), "frac_hbm": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
    res["block_level"] = blk
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llama3_8b_layer")
    ap.add_argument("--ratio", type=float, default=None)
    ap.add_argument("--layers", type=int, default=None, help="layers of a multi-layer workload to run (default all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=None)
    ap.add_argument("--no-at-scale", action="store_true",
                    help="skip the extra kernel timings at the shapes of the large-cache workload")
    ap.add_argument("--layout", choices=("stacked", "per-layer"), default="stacked",
                    help="multi-layer workloads: all layers in one tensor per document and one call per entry point, "
                         "or one set of calls per layer")
    ap.add_argument("--streams", type=int, default=None,
                    help="HIP streams that consecutive passes alternate between: the layers of a per-layer multi-layer "
                         "step (default 2), or with one call set per step the steps themselves (default 1: a step "
                         "then is also a latency; more streams measure throughput of independent requests)")
    ap.add_argument("--no-two-streams", action="store_true", help="skip the extra two-stream throughput timing")
    ap.add_argument("--no-peaks", action="store_true", help="skip the pure-MFMA and plain-copy micro-kernels")
    ap.add_argument("--no-graph", dest="graph", action="store_false",
                    help="skip the extra timing of the same steps as HIP graph replays")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device copies (known traffic, for scaling rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2508_11661_amd import samkv, synth
    to_dev = samkv.upload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    w = synth.WORKLOADS[args.workload]
    ratio = args.ratio if args.ratio is not None else (0.15 if 0.15 in w.ratios else w.ratios[0])
    n_layers = args.layers or w.n_layers
    e = 2 if w.dtype == "bf16" else 4
    scale = 1.0 / math.sqrt(w.head_dim)

    # ---- inputs: n_layers layers, replicated until the K/V working set passes 512 MB
    layers_np = [synth.make_layer(w, l) for l in range(n_layers)]
    m = sum(samkv.samkv_kept_count(n, ratio) for n in w.lens)
    kv_bytes = 2 * sum(w.lens) * w.n_kv_heads * w.head_dim * e * n_layers
    n_rot = max(1, min(16, math.ceil(512e6 / kv_bytes)))
    # Layout of a multi-layer workload.  "stacked": every document's cache holds all layers, [(layer, KV head)][L][d],
    # and so do the Q tensors; the library knows nothing about layers (a head is a head, query head h reads KV head
    # h / G, which stays inside its layer), so ONE call per entry point serves all layers: 4 launches of full-chip
    # size per step instead of 4 small ones per layer.  "per-layer": one set of calls per layer.
    stacked = n_layers > 1 and args.layout == "stacked"
    layers_per_call = n_layers if stacked else 1
    sets = []
    for rot in range(n_rot):
        if stacked:
            cat = lambda arrs, axis=0: to_dev(np.concatenate(arrs, axis=axis), w.dtype)
            k = [cat([x.k[i] for x in layers_np]) for i in range(w.n_ctx)]
            v = [cat([x.v[i] for x in layers_np]) for i in range(w.n_ctx)]
            sets.append(dict(caches=samkv.Caches(k, v, w.n_q_heads * n_layers), q_tok=cat([x.q_tok for x in layers_np]),
                             q_loc=cat([x.q_loc for x in layers_np], axis=1),
                             q_rec=cat([synth.make_q_rec(w, l, m) for l in range(n_layers)])))
            continue
        for l, x in enumerate(layers_np):
            k = [to_dev(a, w.dtype) for a in x.k]
            v = [to_dev(a, w.dtype) for a in x.v]
            sets.append(dict(caches=samkv.Caches(k, v, w.n_q_heads), q_tok=to_dev(x.q_tok, w.dtype),
                             q_loc=to_dev(x.q_loc, w.dtype),
                             q_rec=to_dev(synth.make_q_rec(w, l, m), w.dtype)))
    calls_per_step = 1 if stacked else n_layers
    # The layers of a multi-layer workload are independent (per-layer caches, stored Q states as inputs), so they are
    # spread over `n_streams` HIP streams of default priority, each with its own buffers: the tail of one layer's
    # causal attention (a few long row tiles) overlaps with the next layer's first kernels.
    n_streams = args.streams or (1 if calls_per_step == 1 else 2)
    bufs = [samkv.alloc_layer_buffers(sets[0]["caches"], w.n_q_tok, ratio) for _ in range(n_streams)]
    streams = [torch.cuda.current_stream()] if n_streams == 1 else [torch.cuda.Stream() for _ in range(n_streams)]
    torch.cuda.synchronize()

    calls = {
        "score": lambda s, b: samkv.samkv_score(s["caches"], s["q_tok"], s["q_loc"], b.scores, b.ws),
        "select": lambda s, b: samkv.samkv_topk_select(b.scores, s["caches"], ratio, 0, 0, b.idx, b.cu_k_dev, b.ws),
        "gather": lambda s, b: samkv.samkv_gather(s["caches"], b.idx, ratio, b.k_c, b.v_c),
        "recompute_attn": lambda s, b: samkv.samkv_recompute_attn(s["q_rec"], b.k_c, b.v_c, scale, b.rec_out, b.rec_lse, b.ws),
        "query_attn": lambda s, b: samkv.samkv_query_attn(s["q_tok"], b.k_c, b.v_c, scale, b.q_out, b.q_lse, b.ws),
        "score_select": lambda s, b: samkv.samkv_score_select(s["caches"], s["q_tok"], s["q_loc"], ratio, 0, 0, None, b.idx,
                                                              b.cu_k_dev, b.ws),
        "score_select_gather": lambda s, b: samkv.samkv_score_select_gather(s["caches"], s["q_tok"], s["q_loc"], ratio, 0, 0,
                                                                            None, b.idx, b.cu_k_dev, b.k_c, b.v_c, b.ws),
    }

    def step(i, events=None, only=None, names=STEP):
        """One pass of the hot path.  `events`: dict name -> list of (start, end) HIP events on the launch stream,
        recorded around every call, or only around the call named `only`."""
        for l in range(calls_per_step):
            s = sets[(i * calls_per_step + l) % len(sets)]
            lane = (i * calls_per_step + l) % n_streams   # consecutive passes (layers, or whole steps) alternate streams
            b = bufs[lane]
            with torch.cuda.stream(streams[lane]):
                for name in names:
                    if events is not None and (only is None or only == name):
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        calls[name](s, b)
                        e1.record()
                        events[name].append((e0, e1))
                    else:
                        calls[name](s, b)

    def mean_ms(evs):
        return float(np.mean([a.elapsed_time(b) for a, b in evs]))

    # untimed: which call dominates (events around every call cost a few microseconds each, so the timed region
    # below carries them only around that one call)
    probe = {name: [] for name in STEP}
    n_probe = 12 if calls_per_step * n_layers <= 4 else 3       # short steps: the first few are not representative
    for name in STEP:                                           # one call bracketed at a time, as in the timed region
        for i in range(n_probe):
            step(i, probe, only=name)
    torch.cuda.synchronize()
    dom = max(STEP, key=lambda n: mean_ms(probe[n][len(probe[n]) // 2:]))

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    dom_events = {dom: []}
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, dom_events, only=dom)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    # untimed again: every call bracketed, for the per-call table (the step's fused call, then the five entry points)
    events = {name: [] for name in STEP + KERNELS + EXTRA}
    for i in range(min(args.steps, 50)):
        step(args.warmup + args.steps + i, events)
        step(args.warmup + args.steps + i, events, names=KERNELS)
        step(args.warmup + args.steps + i, events, names=EXTRA)
    torch.cuda.synchronize()
    events[dom] = dom_events[dom]          # the dominant call's figure is the one from the timed region

    # the same K steps as replays of captured HIP graphs (one graph per rotated input set): what a serving loop
    # would launch.  Reported beside the eager figure, not instead of it.
    graph_ms = None
    if args.graph and len(sets) <= 64 and n_streams == 1:
        side = torch.cuda.Stream()
        graphs = []
        streams[0] = side                  # step() launches on streams[0]: capture on the side stream
        with torch.cuda.stream(side):
            for gi in range(len(sets) // calls_per_step):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step(gi)
                graphs.append(g)
        torch.cuda.synchronize()
        for i in range(args.warmup):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(args.steps):
            graphs[(args.warmup + i) % len(graphs)].replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t1) / args.steps * 1e3

    # independent requests side by side: the same K steps alternating between two streams with their own buffers.
    # A throughput figure for a serving loop (a step here is no longer a latency); reported beside the main one.
    two_ms = None
    if n_streams == 1 and calls_per_step == 1 and not args.no_two_streams and ms_per_step < 5.0:
        saved = (n_streams, bufs, streams)
        n_streams = 2
        bufs = [saved[1][0], samkv.alloc_layer_buffers(sets[0]["caches"], w.n_q_tok, ratio)]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        torch.cuda.synchronize()
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
        two_ms = (time.perf_counter() - t1) / args.steps * 1e3
        n_streams, bufs, streams = saved

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    work = algorithmic_work(w, w.lens, m, w.n_q_tok)
    per_kernel = {}
    for name in STEP + tuple(n for n in KERNELS + EXTRA if n not in STEP):
        # the dominant call: mean over the timed region; the others: median of the untimed pass, whose first call of a
        # kernel pays for loading it and which an occasional host hiccup of tens of milliseconds would distort
        samples = [a.elapsed_time(b) for a, b in events[name]]
        ms = float(np.mean(samples) if name == dom else np.median(samples))
        gbs = work[name]["bytes"] * layers_per_call / (ms * 1e-3) / 1e9
        tfl = work[name]["flops"] * layers_per_call / (ms * 1e-3) / 1e12
        per_kernel[name] = {"ms": round(ms, 5), "GB/s": round(gbs, 1), "TFLOP/s": round(tfl, 2),
                            "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)}
        if name.endswith("attn"):
            peak = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else FP32_VALU_PEAK_TFLOPS
            per_kernel[name]["frac_compute"] = round(tfl / peak, 4)

    ss_ms = per_kernel["score"]["ms"] + per_kernel["select"]["ms"]
    ss_gbs = (work["score"]["bytes"] + m * w.n_kv_heads * 4) * layers_per_call / (ss_ms * 1e-3) / 1e9
    per_kernel["score+select"] = {"ms": round(ss_ms, 5), "GB/s": round(ss_gbs, 1), "frac_hbm": round(ss_gbs / HBM_PEAK_GBS, 4),
                                  "note": "the two separate calls as one K-streaming stage, for comparison with the "
                                          "fused calls (score_select, and score_select_gather that the timed step launches)"}
    if dom.endswith("attn") and w.dtype == "bf16":
        roof = {"kernel": dom, "bound": "mfma", "achieved": per_kernel[dom]["TFLOP/s"], "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(per_kernel[dom]["TFLOP/s"] / MFMA_BF16_PEAK_TFLOPS, 4)}
    elif dom.endswith("attn"):
        roof = {"kernel": dom, "bound": "alu", "achieved": per_kernel[dom]["TFLOP/s"], "peak": FP32_VALU_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(per_kernel[dom]["TFLOP/s"] / FP32_VALU_PEAK_TFLOPS, 4)}
    else:
        roof = {"kernel": dom, "bound": "hbm", "achieved": per_kernel[dom]["GB/s"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(per_kernel[dom]["GB/s"] / HBM_PEAK_GBS, 4)}
    roof["avg_launch_ms"] = per_kernel[dom]["ms"]
    roof["traffic"] = read_traffic(w, dom)
    roof["algorithmic"] = (work[dom]["flops"] if roof["bound"] != "hbm" else work[dom]["bytes"]) * layers_per_call

    out = {
        "metric": "KV tokens scored per second through the whole sparse-prefill hot path "
                  "(score+select+gather+recompute_attn+query_attn)",
        "value": round(sum(w.lens) * n_layers / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_layer": round(ms_per_step / n_layers, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n_layers": n_layers, "n_ctx": w.n_ctx, "ctx_len": w.ctx_len,
                   "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                   "n_q_tok": w.n_q_tok, "budget_ratio": ratio, "kept_per_ctx": m // w.n_ctx, "m_total": m,
                   "input_copies_rotated": n_rot, "streams": n_streams,
                   "layout": "stacked: one call per entry point serves all layers" if stacked else "per-layer calls"},
        "per_kernel": per_kernel,
        "roofline": roof,
    }
    if not args.no_peaks:
        mp = measured_peaks(samkv)
        out["measured_peaks"] = mp
        if roof["bound"] == "mfma":
            roof["frac_of_measured_peak"] = round(roof["achieved"] / mp["mfma_bf16_tflops"], 4)
            roof["frac_of_measured_peak_random_operands"] = round(roof["achieved"] / mp["mfma_bf16_tflops_random_operands"], 4)
        elif roof["bound"] == "hbm":
            roof["frac_of_measured_peak"] = round(roof["achieved"] / mp["read_gbs"], 4)
    if two_ms is not None:
        out["two_streams"] = {"ms_per_step": round(two_ms, 4), "value": round(sum(w.lens) * n_layers / (two_ms * 1e-3), 1),
                              "unit": "tokens/s", "note": "the same steps as independent requests alternating between two "
                                                          "HIP streams: throughput, not the latency of a step"}
    if graph_ms is not None:
        out["hip_graph"] = {"ms_per_step": round(graph_ms, 4), "value": round(sum(w.lens) * n_layers / (graph_ms * 1e-3), 1),
                            "unit": "tokens/s", "note": "the same steps launched as replays of captured HIP graphs"}
    if not args.no_at_scale and w.name != "large_cache_stress":
        out["at_scale"] = at_scale(samkv)
    if not args.no_cpu_baseline:
        rows = args.cpu_sample_rows or (m if m <= 2048 else 48)
        out["cpu_baseline"] = cpu_baseline(layers_np[0], ratio, rows)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
