#!/usr/bin/env python3
"""Benchmark of the SamKV hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--ratio R]

A step is one pass of the whole hot path (score, selection, compaction, recompute attention, query attention) over
the per-document caches of one layer (for the 32-layer workload: over all 32 layers).  Inputs are the seeded
synthetic caches of `paper_2508_11661_amd/synth.py`, already resident in HBM; enough distinct copies are rotated
that the working set exceeds twice the 256 MB Infinity Cache, so K is streamed from HBM and not from cache.
Prints ONE JSON line.

Default workload: `large_cache_stress` (64 documents x 4096 tokens, 64/8 heads, d = 128, 256 query tokens, 15 %),
the largest single-GPU configuration.  Beside the headline the line carries
  secondary   the same step on the small `llama3_8b_layer` workload (launch- and latency-bound; context only)
  sweep       the five separate calls on `mistral_7b_sweep` at 5, 10, 15 and 25 % budget (the crossover table)
  measured_peaks, cpu_baseline

The timed region launches the calls eagerly and brackets only the dominant call with HIP events (its average
duration feeds the roofline figure); the per-call table comes from a second, untimed pass with every call bracketed.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix cores, published
FP32_VALU_PEAK_TFLOPS = 157.3
RIDGE = MFMA_BF16_PEAK_TFLOPS / HBM_PEAK_GBS * 1e3   # flop per byte above which a bf16 kernel is MFMA-bound
KERNELS = ("score", "select", "gather", "recompute_attn", "query_attn")          # the five entry points of the path
STEP = ("score_select_gather", "recompute_query_attn")                            # what a step launches: two fused calls
EXTRA = ("score_select",)                                                        # also timed per call, outside the step
ATTN_PAIR = "recompute_query_attn"


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
        # both attentions in one call: the sum of the two
        "recompute_query_attn": {"bytes": (2 * hq + 2 * hkv) * m * d * e + hq * m * (d + 1) * 4
                                          + 2 * m * hkv * d * e + hq * n_q_tok * (d * e + (d + 1) * 4),
                                 "flops": 4 * hq * d * m * (m + 1) // 2 + 4 * hq * d * n_q_tok * m},
    }


def bound_of(name, w, work):
    """Which roofline bounds a call: HBM for score / select / gather; the matrix cores for the causal attention; for
    the query attention whichever its arithmetic intensity puts lower (HBM below the ridge of about 310 flop/B)."""
    if not name.endswith("attn"):
        return "hbm"
    if w.dtype != "bf16":
        return "alu"
    if name == "query_attn" and work[name]["flops"] / work[name]["bytes"] < RIDGE:
        return "hbm"
    return "mfma"


def kernel_row(name, w, work, ms, layers_per_call=1):
    gbs = work[name]["bytes"] * layers_per_call / (ms * 1e-3) / 1e9
    tfl = work[name]["flops"] * layers_per_call / (ms * 1e-3) / 1e12
    bound = bound_of(name, w, work)
    row = {"ms": round(ms, 5), "GB/s": round(gbs, 1), "TFLOP/s": round(tfl, 2), "bound": bound,
           "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)}
    if name.endswith("attn"):
        peak = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else FP32_VALU_PEAK_TFLOPS
        row["frac_compute"] = round(tfl / peak, 4)
    row["frac"] = row["frac_hbm"] if bound == "hbm" else row["frac_compute"]
    return row


def read_traffic(workload, kernel: str):
    """HBM bytes per launch (read + write) of a call's main kernel(s), from the committed rocprofv3 --pmc summary of
    this workload (profiles/bench_<workload>.txt: FETCH_SIZE and WRITE_SIZE runs scaled by a plain copy), or None."""
    causal = ["k_attn_%s<%d, true" % (workload.dtype, workload.head_dim), "k_attn_%s_dma<true" % workload.dtype]
    plain = ["k_attn_%s<%d, false" % (workload.dtype, workload.head_dim), "k_attn_%s_dma<false" % workload.dtype]
    pair = ["k_attn_%s_pair<%d" % (workload.dtype, workload.head_dim), "k_attn_%s_dma_pair" % workload.dtype]
    groups = {"score": [["k_score<"]], "select": [["k_select"]], "gather": [["k_gather<"]],
              "score_select": [["k_score_select"]], "score_select_gather": [["k_score_select"]],
              "recompute_attn": [causal], "query_attn": [plain],
              # bf16: one launch runs both attentions; float32: the two kernels one after the other
              "recompute_query_attn": [pair] if workload.dtype == "bf16" else [causal, plain]}[kernel]
    try:
        lines = open(os.path.join(ROOT, "profiles", f"bench_{workload.name}.txt")).read().splitlines()
    except OSError:
        return None
    total = 0.0
    for prefixes in groups:
        for line in lines:
            if any(line.startswith(p) for p in prefixes):
                try:
                    total += (float(line.split()[-2]) + float(line.split()[-1])) * 1e6
                except ValueError:
                    return None
                break
        else:
            return None
    return total


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
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return {"value": sum(layer.lens) / total, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": sample, "seconds_measured": round(wall, 2), "ms_per_step_extrapolated": round(total * 1e3, 1),
            "host": {"nproc": os.cpu_count(), "cpus_usable_by_this_process": usable,
                     "OMP_NUM_THREADS": os.environ.get("OMP_NUM_THREADS"),
                     "note": "`cores` = process CPU time / wall time of the oracle run: numpy's own loops run on one "
                             "thread, its matrix products on as many as the BLAS it links takes"}}


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


class Workbench:
    """Device inputs and buffers of one workload at one budget, and the calls of the path on them."""

    def __init__(self, samkv, synth, w, ratio, n_layers, layout, n_streams_arg, caches_from=None):
        """`caches_from`: another Workbench of the same single-layer workload whose uploaded caches and query tensors
        are reused (they do not depend on the budget); only the kept tokens' query states and the buffers are new."""
        import torch
        self.samkv, self.w, self.ratio, self.n_layers = samkv, w, ratio, n_layers
        to_dev = samkv.upload
        e = 2 if w.dtype == "bf16" else 4
        self.scale = scale = 1.0 / math.sqrt(w.head_dim)
        self.m = m = sum(samkv.samkv_kept_count(n, ratio) for n in w.lens)
        if caches_from is not None:
            o = caches_from
            self.layers_np, self.n_rot, self.stacked, self.layers_per_call = o.layers_np, o.n_rot, False, 1
            q_rec = to_dev(synth.make_q_rec(w, 0, m), w.dtype)
            self.sets = [dict(s, q_rec=q_rec) for s in o.sets]
        else:
            self._upload(synth, w, n_layers, layout, m, e)
        self._finish(samkv, w, ratio, scale, n_streams_arg)

    def _upload(self, synth, w, n_layers, layout, m, e):
        samkv = self.samkv
        to_dev = samkv.upload
        # ---- inputs: n_layers layers, replicated until the K/V working set passes 512 MB
        self.layers_np = []
        for l in range(n_layers):
            self.layers_np.append(synth.make_layer(w, l))
            if n_layers > 1 and l % 4 == 3:          # a long host-side phase: say that the run is alive
                print(f"bench.py: {w.name}: layers 0..{l} drawn", file=sys.stderr, flush=True)
        kv_bytes = 2 * sum(w.lens) * w.n_kv_heads * w.head_dim * e * n_layers
        self.n_rot = max(1, min(16, math.ceil(512e6 / kv_bytes)))
        # Layout of a multi-layer workload.  "stacked": every document's cache holds all layers, [(layer, KV head)][L][d],
        # and so do the Q tensors (synth.stack_layers); ONE call per entry point serves all layers: 4 launches of
        # full-chip size per step instead of 4 small ones per layer.  "per-layer": one set of calls per layer.
        self.stacked = n_layers > 1 and layout == "stacked"
        self.layers_per_call = n_layers if self.stacked else 1
        self.sets = []
        for rot in range(self.n_rot):
            if self.stacked:
                k, v, q_tok, q_loc, q_rec = synth.stack_layers(w, self.layers_np,
                                                               [synth.make_q_rec(w, l, m) for l in range(n_layers)])
                self.sets.append(dict(caches=samkv.Caches([to_dev(a, w.dtype) for a in k], [to_dev(a, w.dtype) for a in v],
                                                          w.n_q_heads * n_layers),
                                      q_tok=to_dev(q_tok, w.dtype), q_loc=to_dev(q_loc, w.dtype), q_rec=to_dev(q_rec, w.dtype)))
                del k, v
                continue
            for l, x in enumerate(self.layers_np):
                k = [to_dev(a, w.dtype) for a in x.k]
                v = [to_dev(a, w.dtype) for a in x.v]
                self.sets.append(dict(caches=samkv.Caches(k, v, w.n_q_heads), q_tok=to_dev(x.q_tok, w.dtype),
                                      q_loc=to_dev(x.q_loc, w.dtype),
                                      q_rec=to_dev(synth.make_q_rec(w, l, m), w.dtype)))

    def _finish(self, samkv, w, ratio, scale, n_streams_arg):
        import torch
        n_layers, m = self.n_layers, self.m
        self.calls_per_step = 1 if self.stacked else n_layers
        # The layers of a multi-layer workload are independent (per-layer caches, stored Q states as inputs), so they
        # may be spread over `n_streams` HIP streams of default priority, each with its own buffers.
        self.n_streams = n_streams_arg or (1 if self.calls_per_step == 1 else 2)
        self.bufs = [samkv.alloc_layer_buffers(self.sets[0]["caches"], w.n_q_tok, ratio) for _ in range(self.n_streams)]
        self.streams = ([torch.cuda.current_stream()] if self.n_streams == 1
                        else [torch.cuda.Stream() for _ in range(self.n_streams)])
        torch.cuda.synchronize()
        S = samkv
        self.calls = {
            "score": lambda s, b: S.samkv_score(s["caches"], s["q_tok"], s["q_loc"], b.scores, b.ws),
            "select": lambda s, b: S.samkv_topk_select(b.scores, s["caches"], ratio, 0, 0, b.idx, b.cu_k_dev, b.ws),
            "gather": lambda s, b: S.samkv_gather(s["caches"], b.idx, ratio, b.k_c, b.v_c),
            "recompute_attn": lambda s, b: S.samkv_recompute_attn(s["q_rec"], b.k_c, b.v_c, scale, b.rec_out, b.rec_lse, b.ws),
            "query_attn": lambda s, b: S.samkv_query_attn(s["q_tok"], b.k_c, b.v_c, scale, b.q_out, b.q_lse, b.ws),
            "score_select": lambda s, b: S.samkv_score_select(s["caches"], s["q_tok"], s["q_loc"], ratio, 0, 0, None, b.idx,
                                                              b.cu_k_dev, b.ws),
            "score_select_gather": lambda s, b: S.samkv_score_select_gather(s["caches"], s["q_tok"], s["q_loc"], ratio, 0, 0,
                                                                            None, b.idx, b.cu_k_dev, b.k_c, b.v_c, b.ws),
            "recompute_query_attn": lambda s, b: S.samkv_recompute_query_attn(s["q_rec"], s["q_tok"], b.k_c, b.v_c, scale,
                                                                              b.rec_out, b.rec_lse, b.q_out, b.q_lse, b.ws),
        }
        self.work = algorithmic_work(w, w.lens, m, w.n_q_tok)

    def step(self, i, events=None, only=None, names=STEP):
        """One pass of the hot path.  `events`: dict name -> list of (start, end) HIP events on the launch stream,
        recorded around every call, or only around the call named `only`."""
        import torch
        for l in range(self.calls_per_step):
            s = self.sets[(i * self.calls_per_step + l) % len(self.sets)]
            lane = (i * self.calls_per_step + l) % self.n_streams   # consecutive passes alternate streams
            b = self.bufs[lane]
            with torch.cuda.stream(self.streams[lane]):
                for name in names:
                    if events is not None and (only is None or only == name):
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        self.calls[name](s, b)
                        e1.record()
                        events[name].append((e0, e1))
                    else:
                        self.calls[name](s, b)

    def run(self, steps, warmup, per_call_steps=50):
        """Probe for the dominant call, warm up, time `steps` steps (events around the dominant call only), then an
        untimed pass with every call bracketed.  Returns (ms_per_step, dominant call, per_kernel table)."""
        import numpy as np
        import torch
        mean_ms = lambda evs: float(np.mean([a.elapsed_time(b) for a, b in evs]))
        probe = {name: [] for name in STEP}
        n_probe = 12 if self.calls_per_step * self.n_layers <= 4 and self.m < 8192 else 3
        for name in STEP:                                           # one call bracketed at a time, as in the timed region
            for i in range(n_probe):
                self.step(i, probe, only=name)
        torch.cuda.synchronize()
        dom = max(STEP, key=lambda n: mean_ms(probe[n][len(probe[n]) // 2:]))

        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        dom_events = {dom: []}
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(warmup + i, dom_events, only=dom)
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) / steps * 1e3

        events = {name: [] for name in STEP + KERNELS + EXTRA}
        for i in range(min(steps, per_call_steps)):
            self.step(warmup + steps + i, events)
            self.step(warmup + steps + i, events, names=KERNELS)
            self.step(warmup + steps + i, events, names=EXTRA)
        torch.cuda.synchronize()
        events[dom] = dom_events[dom]          # the dominant call's figure is the one from the timed region
        w, work = self.w, self.work
        per_kernel = {}
        for name in STEP + tuple(n for n in KERNELS + EXTRA if n not in STEP):
            # the dominant call: mean over the timed region; the others: median of the untimed pass
            samples = [a.elapsed_time(b) for a, b in events[name]]
            ms = float(np.mean(samples) if name == dom else np.median(samples))
            per_kernel[name] = kernel_row(name, w, work, ms, self.layers_per_call)
        ss_ms = per_kernel["score"]["ms"] + per_kernel["select"]["ms"]
        ss_gbs = (work["score"]["bytes"] + self.m * w.n_kv_heads * 4) * self.layers_per_call / (ss_ms * 1e-3) / 1e9
        per_kernel["score+select"] = {"ms": round(ss_ms, 5), "GB/s": round(ss_gbs, 1), "frac_hbm": round(ss_gbs / HBM_PEAK_GBS, 4),
                                      "note": "the two separate calls as one K-streaming stage, for comparison with the "
                                              "fused calls (score_select, and score_select_gather that the timed step launches)"}
        return ms_per_step, dom, per_kernel

    def graph_ms(self, steps, warmup):
        """The same steps as replays of captured HIP graphs (one per rotated input set)."""
        import torch
        if len(self.sets) > 64 or self.n_streams != 1:
            return None
        side = torch.cuda.Stream()
        graphs = []
        saved = self.streams[0]
        self.streams[0] = side                  # step() launches on streams[0]: capture on the side stream
        with torch.cuda.stream(side):
            for gi in range(len(self.sets) // self.calls_per_step):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    self.step(gi)
                graphs.append(g)
        torch.cuda.synchronize()
        for i in range(warmup):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(steps):
            graphs[(warmup + i) % len(graphs)].replay()
        torch.cuda.synchronize()
        self.streams[0] = saved
        return (time.perf_counter() - t1) / steps * 1e3

    def two_stream_ms(self, steps, warmup):
        """Independent requests side by side: the same steps alternating between two streams with their own buffers."""
        import torch
        if self.n_streams != 1 or self.calls_per_step != 1:
            return None
        saved = (self.n_streams, self.bufs, self.streams)
        self.n_streams = 2
        self.bufs = [saved[1][0], self.samkv.alloc_layer_buffers(self.sets[0]["caches"], self.w.n_q_tok, self.ratio)]
        self.streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        torch.cuda.synchronize()
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(steps):
            self.step(warmup + i)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t1) / steps * 1e3
        self.n_streams, self.bufs, self.streams = saved
        return ms


def next_rows(samkv, wb, iters=20, warmup=3):
    """The entry points beyond the five of the step (cache update, block-level retrieval with the cross-document
    filter, gathers by explicit counts / global positions / of the Q caches, query attention with its own tail), each
    timed alone on the workload's shapes: median of `iters` event-bracketed calls after `warmup`.  HBM-bound rows
    report their algorithmic bytes against the HBM peak; the small selection kernels are latency-bound."""
    import numpy as np
    import torch
    w, S = wb.w, samkv
    if wb.stacked or w.dtype != "bf16":
        return None
    s, b = wb.sets[0], wb.bufs[0]
    caches = s["caches"]
    n, hq, hkv, d, e = w.n_ctx, w.n_q_heads, w.n_kv_heads, w.head_dim, 2
    total, m, block = sum(w.lens), wb.m, 64
    gen = torch.Generator(device="cuda").manual_seed(0x5A4D)
    rnd = lambda *shape: torch.randn(*shape, device="cuda", generator=gen).to(torch.bfloat16)

    # the calls repeat on the same buffers: a 512 MB copy ahead of every timed call pushes them out of the 256 MB
    # Infinity Cache, so that every call finds its inputs in HBM as it would inside a step
    flush_src = torch.empty((512 << 20,), dtype=torch.uint8, device="cuda").fill_(1)
    flush_dst = torch.empty_like(flush_src)

    def timed(fn):
        for _ in range(warmup):
            fn()
        ev = []
        for _ in range(iters):
            flush_dst.copy_(flush_src)
            a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            z.record()
            ev.append((a, z))
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(z) for a, z in ev]))

    def row(ms, nbytes=None, flops=None):
        r = {"us": round(ms * 1e3, 1)}
        if nbytes is not None:
            r["GB/s"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
            r["frac_hbm"] = round(r["GB/s"] / HBM_PEAK_GBS, 4)
        if flops is not None:
            r["TFLOP/s"] = round(flops / (ms * 1e-3) / 1e12, 1)
            r["frac_mfma"] = round(r["TFLOP/s"] / MFMA_BF16_PEAK_TFLOPS, 4)
        return r

    out = {"workload": w.name, "block": block, "note": "each call alone, inputs resident in HBM; a 512 MB device copy "
           "ahead of every timed call empties the 256 MB Infinity Cache"}
    wb.step(0)                                   # the compacted cache and the buffers hold a step's results
    S.samkv_score(caches, s["q_tok"], s["q_loc"], b.scores, b.ws)
    torch.cuda.synchronize()
    # ---- cache update after recomputation (Eq. 4): rows of the compacted cache against new rows
    k_new, v_new = rnd(hkv, m, d), rnd(hkv, m, d)
    rows_bytes = 2 * hkv * m * d * e             # K and V
    out["kv_update_overwrite"] = row(timed(lambda: S.samkv_kv_update(b.k_c, b.v_c, k_new, v_new, 0)), 2 * rows_bytes)
    out["kv_update_fusion"] = row(timed(lambda: S.samkv_kv_update(b.k_c, b.v_c, k_new, v_new, 1)), 3 * rows_bytes)
    # ---- block-level retrieval (64-token blocks, one initial and two local blocks forced, share 0.15 of the rest)
    n_blk = sum(-(-x // block) for x in w.lens)
    bscores = torch.empty((hkv, n_blk), dtype=torch.float32, device="cuda")
    out["block_scores"] = row(timed(lambda: S.samkv_block_scores(b.scores, caches, block, bscores)),
                              hkv * (total + n_blk) * 4)
    p = [0.15] * n
    ws_b = torch.empty((max(S.samkv_block_workspace_bytes(caches, block), 256),), dtype=torch.uint8, device="cuda")
    m_b = S.samkv_block_select_count(caches, block, p, 1, 2)
    idx_b = torch.empty((hkv, m_b), dtype=torch.int32, device="cuda")
    cu = S.samkv_block_select(bscores, caches, block, p, 1, 2, idx_b, None, ws_b)
    out["block_select"] = row(timed(lambda: S.samkv_block_select(bscores, caches, block, p, 1, 2, idx_b, None, ws_b)))
    out["block_select"]["kept_tokens"] = m_b
    k2 = torch.empty((hkv, m_b, d), dtype=torch.bfloat16, device="cuda")
    v2 = torch.empty_like(k2)
    gather_bytes = lambda mm: hkv * mm * (4 * d * e + 4)
    out["gather_v"] = row(timed(lambda: S.samkv_gather_v(caches, idx_b, cu, k2, v2)), gather_bytes(m_b))
    m_f = S.samkv_block_filter_count(caches, block, p, 1, 2)
    gidx = torch.empty((hkv, m_f), dtype=torch.int32, device="cuda")
    out["block_select_filter"] = row(timed(lambda: S.samkv_block_select_filter(bscores, caches, block, p, 1, 2, gidx, ws_b)))
    out["block_select_filter"]["kept_tokens"] = m_f
    k3 = torch.empty((hkv, m_f, d), dtype=torch.bfloat16, device="cuda")
    v3 = torch.empty_like(k3)
    out["gather_g"] = row(timed(lambda: S.samkv_gather_g(caches, gidx, k3, v3)), gather_bytes(m_f))
    del k2, v2, k3, v3
    # ---- the stored Q caches compacted at the kept positions of the step
    q_cache = [rnd(hq, x, d) for x in w.lens]
    q_rec = torch.empty((hq, m, d), dtype=torch.bfloat16, device="cuda")
    out["gather_q"] = row(timed(lambda: S.samkv_gather_q(caches, q_cache, b.idx, wb.ratio, q_rec)),
                          hq * m * 2 * d * e + hkv * m * 4)
    del q_cache, q_rec
    # ---- query attention with the query tokens' own K/V appended causally
    lq = w.n_q_tok
    k_self, v_self = rnd(hkv, lq, d), rnd(hkv, lq, d)
    out["query_attn_self"] = row(timed(lambda: S.samkv_query_attn_self(s["q_tok"], b.k_c, b.v_c, k_self, v_self, wb.scale,
                                                                       b.q_out, b.q_lse, b.ws)),
                                 flops=4.0 * hq * d * lq * (m + (lq + 1) / 2))
    return out



def sweep(samkv, synth, iters=30, warmup=8):
    """The five separate calls of the path on `mistral_7b_sweep` at each of its budgets: score is flat in the budget,
    gather and the query attention grow with r, the recompute attention with r^2.  Per call: median of `iters`
    event-bracketed launches after `warmup`, inputs rotated past the Infinity Cache."""
    import numpy as np
    import torch
    w = synth.WORKLOADS["mistral_7b_sweep"]
    names = KERNELS + STEP
    rows, first = [], None
    for ratio in w.ratios:
        wb = Workbench(samkv, synth, w, ratio, 1, "per-layer", 1, caches_from=first)
        first = first or wb
        for i in range(warmup):
            wb.step(i, names=names)
        events = {n: [] for n in names}
        for i in range(iters):
            wb.step(warmup + i, events, names=names)
        torch.cuda.synchronize()
        row = {"ratio": ratio, "kept_per_ctx": wb.m // w.n_ctx, "m_total": wb.m}
        for n in names:
            ms = float(np.median([a.elapsed_time(b) for a, b in events[n]]))
            row[n] = kernel_row(n, w, wb.work, ms)
        row["five_calls_ms"] = round(sum(row[n]["ms"] for n in KERNELS), 5)
        row["step_ms"] = round(sum(row[n]["ms"] for n in STEP), 5)
        hbm = {n: row[n]["ms"] for n in ("score", "select", "gather")}
        row["largest_hbm_bound_call"] = max(hbm, key=hbm.get)
        row["gather_bytes_over_score_bytes"] = round(wb.work["gather"]["bytes"] / wb.work["score"]["bytes"], 3)
        row["recompute_over_score_time"] = round(row["recompute_attn"]["ms"] / row["score"]["ms"], 2)
        rows.append(row)
        if wb is not first:
            del wb
        torch.cuda.empty_cache()
    return {"workload": w.name, "iters": iters, "warmup": warmup, "input_copies_rotated": first.n_rot, "rows": rows,
            "note": "score streams all of K whatever the budget; gather bytes reach score bytes at r = 0.25 "
                    "(4 d e r against d e per token-head); the recompute attention grows with r^2"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="large_cache_stress")
    ap.add_argument("--ratio", type=float, default=None)
    ap.add_argument("--layers", type=int, default=None, help="layers of a multi-layer workload to run (default all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=None)
    ap.add_argument("--no-secondary", action="store_true", help="skip the extra timing of the small llama3_8b_layer workload")
    ap.add_argument("--no-sweep", action="store_true", help="skip the budget sweep on mistral_7b_sweep")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="skip the timing of the entry points beyond the step (cache update, block-level retrieval, ...)")
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

    import torch
    from paper_2508_11661_amd import samkv, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    w = synth.WORKLOADS[args.workload]
    ratio = args.ratio if args.ratio is not None else (0.15 if 0.15 in w.ratios else w.ratios[0])
    n_layers = args.layers or w.n_layers

    wb = Workbench(samkv, synth, w, ratio, n_layers, args.layout, args.streams)
    ms_per_step, dom, per_kernel = wb.run(args.steps, args.warmup)
    m, work = wb.m, wb.work
    short = ms_per_step < 5.0
    graph_ms = wb.graph_ms(args.steps, args.warmup) if args.graph and short else None
    two_ms = wb.two_stream_ms(args.steps, args.warmup) if not args.no_two_streams and short else None

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    bound = per_kernel[dom]["bound"]
    if bound == "hbm":
        roof = {"kernel": dom, "bound": "hbm", "achieved": per_kernel[dom]["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        roof = {"kernel": dom, "bound": bound, "achieved": per_kernel[dom]["TFLOP/s"],
                "peak": MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = round(roof["achieved"] / roof["peak"], 4)
    roof["avg_launch_ms"] = per_kernel[dom]["ms"]
    roof["traffic"] = read_traffic(w, dom)
    roof["algorithmic"] = (work[dom]["flops"] if bound != "hbm" else work[dom]["bytes"]) * wb.layers_per_call
    if dom == ATTN_PAIR:
        rec, qry = per_kernel["recompute_attn"], per_kernel["query_attn"]
        roof["note"] = ("the dominant call runs both attentions: the launches that rewrite V as scaled half precision "
                        "(not counted as algorithmic work), then ONE kernel launch whose first workgroups are the query "
                        "attention (all keys in one chunk) and whose others are the causal attention; "
                        "achieved = algorithmic flop of both attentions / duration of the call")
        roof["components"] = {"recompute_attn": {"ms_as_a_separate_call": rec["ms"], "TFLOP/s": rec["TFLOP/s"],
                                                 "frac": rec["frac"], "flop": work["recompute_attn"]["flops"] * wb.layers_per_call},
                              "query_attn": {"ms_as_a_separate_call": qry["ms"], "TFLOP/s": qry["TFLOP/s"], "bound": qry["bound"],
                                             "frac": qry["frac"], "flop": work["query_attn"]["flops"] * wb.layers_per_call}}

    tokens = sum(w.lens) * n_layers
    out = {
        "metric": "KV tokens scored per second through the whole sparse-prefill hot path "
                  "(score+select+gather+recompute_attn+query_attn)",
        "value": round(tokens / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_layer": round(ms_per_step / n_layers, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n_layers": n_layers, "n_ctx": w.n_ctx, "ctx_len": w.ctx_len,
                   "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                   "n_q_tok": w.n_q_tok, "budget_ratio": ratio, "kept_per_ctx": m // w.n_ctx, "m_total": m,
                   "input_copies_rotated": wb.n_rot, "streams": wb.n_streams,
                   "layout": "stacked: one call per entry point serves all layers" if wb.stacked else "per-layer calls",
                   "step": "samkv_score_select_gather (scores = NULL: the scores stay on chip, only the kept positions "
                           "and the compacted rows are written), samkv_recompute_query_attn (both attentions, V prepared once)",
                   "inputs": "seeded synthetic caches (synth.make_layer), resident in HBM"},
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
        out["two_streams"] = {"ms_per_step": round(two_ms, 4), "value": round(tokens / (two_ms * 1e-3), 1),
                              "unit": "tokens/s", "note": "the same steps as independent requests alternating between two "
                                                          "HIP streams: throughput, not the latency of a step"}
    if graph_ms is not None:
        out["hip_graph"] = {"ms_per_step": round(graph_ms, 4), "value": round(tokens / (graph_ms * 1e-3), 1),
                            "unit": "tokens/s", "note": "the same steps launched as replays of captured HIP graphs"}
    layer0 = wb.layers_np[0]
    if not args.no_next_rows:
        nr = next_rows(samkv, wb)
        if nr is not None:
            out["next_rows"] = nr
    del wb
    torch.cuda.empty_cache()
    if not args.no_secondary and w.name != "llama3_8b_layer":
        w2 = synth.WORKLOADS["llama3_8b_layer"]
        wb2 = Workbench(samkv, synth, w2, 0.15, 1, "per-layer", 1)
        ms2, dom2, pk2 = wb2.run(200, 20)
        out["secondary"] = {"workload": w2.name, "steps": 200, "warmup": 20, "ms_per_step": round(ms2, 4),
                            "value": round(sum(w2.lens) / (ms2 * 1e-3), 1), "unit": "tokens/s", "m_total": wb2.m,
                            "input_copies_rotated": wb2.n_rot, "dominant_call": dom2, "per_kernel": pk2,
                            "note": "small single-layer workload: launch- and latency-bound, reported for context"}
        g2 = wb2.graph_ms(200, 20)
        if g2 is not None:
            out["secondary"]["hip_graph_ms_per_step"] = round(g2, 4)
        del wb2
        torch.cuda.empty_cache()
    if not args.no_sweep:
        out["sweep"] = sweep(samkv, synth)
    if not args.no_cpu_baseline:
        rows = args.cpu_sample_rows or (m if m <= 2048 else 48)
        out["cpu_baseline"] = cpu_baseline(layer0, ratio, rows)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
