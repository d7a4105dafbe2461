#!/usr/bin/env python3
"""Benchmark of the Head-Centric Sparse Attention hot path on one MI355X.

One "step" is one pass of the whole hot path over resident synthetic inputs:
    select  + attend   on the batched Reuse workload   (16 seqs, KV 512..4096, keep 10..50 %)
    dense Refresh      on the Refresh workload          (8 x L=2048, 32 heads x 128)
    select  + attend   on the mixed GQA burst           (24 Reuse + 8 Refresh sequences in one call)
plus the paper's own Reuse layout on the first workload: pack the kept rows once, attend over the packed cache.
and the gather attend with one kept set shared by all heads (the head-summed selection of Eq. 5).
All inputs are on the GPU before the timed region.  A step's calls are timed call by call: the K launches
of one call follow each other on the stream, each on the next of several copies of its inputs, so every
launch reads its data from HBM and not from the 256 MB memory-side cache; event pairs on that stream
bracket runs of a few launches.  Rates are algorithmic bytes (or flops) divided by the mean launch duration.

Prints ONE JSON line.  `value` is the Reuse sparse-attention rate in GB/s of algorithmic bytes
(the headline of the metric); the Refresh TFLOP/s and the other calls are reported beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published

# HBM bytes per launch (reads + writes) from two rocprofv3 --pmc runs of this script (FETCH_SIZE, then
# WRITE_SIZE, each scaled by what it reads for the --copy-probe launch of known size); the summary,
# with the commands, is profiles/hbm_traffic_pmc.md.  They are properties of the workload shapes
# above, not of the timing, so they are recorded here rather than re-measured on every run.
TRAFFIC_BYTES = {
    "attend_dense_bf16_kernel": 537.3e6,     # Refresh c4: 403.0 MB read + 134.3 MB written
    "attend_sparse_multi_bf16_kernel": 197.7e6,   # Reuse c3: 193.8 MB read + 4.2 MB written, less rounding
    "score_kernel": 287.6e6,                 # Reuse c3: 283.1 MB read + 4.5 MB written
}

# What plain kernels reach on this GPU (python -m paper_2512_17077_amd.ceilings; profiles/ceilings_microbench.md):
# context for the fractions of the published peaks, never used as the roofline denominator.
MEASURED_CEILINGS = {"hbm_stream_read_grid_stride_GBps": 5085.0, "hbm_stream_read_spans_nontemporal_GBps": 6530.0,
                     "hbm_row_gather_GBps": 4718.0, "mfma_bf16_sustained_TFLOPs": 2002.0,
                     "shader_clock_under_mfma_MHz": 1970.0}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device copy (reference launch for scaling rocprofv3 byte counters)")
    ap.add_argument("--warm", action="store_true",
                    help="afterwards time every call again on one copy without flushes (warm caches), for contrast")
    ap.add_argument("--isolated", action="store_true",
                    help="afterwards time every call again one launch at a time, each after a cache flush "
                         "and on an otherwise idle GPU, for contrast")
    ap.add_argument("--only", choices=["all", "reuse", "refresh", "mixed"], default="all",
                    help="restrict the step to one workload (for profiling runs)")
    return ap.parse_args()


class Train:
    """One library call, launched back to back on rotating copies of its inputs.

    Launches follow each other on the stream with no gap, so an event pair around a run of `chunk`
    launches measures their kernels' durations (a pair around a single launch adds the few
    microseconds the command processor takes between an event and the next dispatch).  Each copy has
    its own tensors, and a call returns to a copy only after the other copies' launches have moved more
    than the 256 MB memory-side cache holds, so every launch finds its inputs in HBM; an untimed
    read-only pass over 512 MiB before the run evicts what earlier work left behind."""

    flush_buf = None
    flush_out = None
    chunk = 5

    def __init__(self, name, fns):
        import torch
        self.name, self.fns, self.pairs, self.torch, self.turn = name, list(fns), [], torch, 0
        if Train.flush_buf is None:
            Train.flush_buf = torch.zeros(1 << 27, dtype=torch.int32, device="cuda:0")
            Train.flush_out = torch.zeros((), dtype=torch.int32, device="cuda:0")

    def launch(self):
        self.fns[self.turn % len(self.fns)]()
        self.turn += 1

    def run(self, n, record, flush=True):
        if flush:
            self.torch.max(Train.flush_buf, out=Train.flush_out)
        done = 0
        while done < n:
            m = min(Train.chunk, n - done)
            if record:
                a = self.torch.cuda.Event(enable_timing=True)
                b = self.torch.cuda.Event(enable_timing=True)
                a.record()
            for _ in range(m):
                self.launch()
            if record:
                b.record()
                self.pairs.append((a, b, m))
            done += m

    def run_isolated(self, n):
        """n launches, each after its own flush and inside its own event pair: the duration of a
        call that starts on an idle GPU (clocks recovered, plus the event-to-dispatch latency)."""
        for _ in range(n):
            self.run(1, True)

    def ms(self):
        """(mean per launch over all timed launches, best per-launch mean of any one event pair)"""
        t = [(a.elapsed_time(b), m) for a, b, m in self.pairs]
        if not t:
            return float("nan"), float("nan")
        return sum(x for x, _ in t) / sum(m for _, m in t), min(x / m for x, m in t)

    def reset(self):
        self.pairs = []


def cpu_baseline(w3, w4):
    """The oracle as it stands, timed on this host: the full Reuse workload (selection and attention),
    repeated for a steadier clock, and one whole Refresh sequence (all heads)."""
    import numpy as np
    import oracle
    from paper_2512_17077_amd import synth
    q, k, v = synth.to_bits(w3.q), synth.to_bits(w3.k), synth.to_bits(w3.v)
    reps = 30
    t_sel = t_att = 0.0
    for _ in range(reps):
        t0 = time.perf_counter()
        idx = oracle.select(q, k, w3.cu_q, w3.cu_kv, w3.cu_k)
        t1 = time.perf_counter()
        oracle.attend(q, k, v, w3.cu_q, w3.cu_kv, idx, w3.cu_k, None, w3.softmax_scale)
        t2 = time.perf_counter()
        t_sel += t1 - t0
        t_att += t2 - t1
    t_sel /= reps
    t_att /= reps
    # Refresh sample: the first sequence, all query rows and heads, against its full K/V
    L = int(w4.kv_lens[0])
    n = int(w4.q_lens[0])
    sub_q = synth.to_bits(w4.q[:n])
    sub_k, sub_v = synth.to_bits(w4.k[:L]), synth.to_bits(w4.v[:L])
    t3 = time.perf_counter()
    oracle.attend(sub_q, sub_k, sub_v, np.array([0, n], np.int32), np.array([0, L], np.int32), None, None,
                  np.ones(1, np.uint8), w4.softmax_scale)
    t4 = time.perf_counter()
    dense_flops = 4.0 * n * L * w4.head_dim * w4.n_q_heads
    return {
        "value": w3.attend_sparse_bytes() / t_att / 1e9,
        "unit": "GB/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"full Reuse workload {w3.name}, mean of {reps} runs: attend {t_att:.3f} s, select {t_sel:.3f} s; "
                  f"Refresh: one whole L={L} sequence ({n} query rows x {w4.n_q_heads} heads) {t4 - t3:.2f} s",
        "select_gbps": w3.select_bytes() / t_sel / 1e9,
        "refresh_tflops": dense_flops / (t4 - t3) / 1e12,
    }


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (asked for --gpus {args.gpus}); "
              "the path shards by sequence or by KV head with no exchange between GPUs", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2512_17077_amd import hcsa, synth
    hcsa.lib()   # raises if the HIP library is not built: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)

    w3, w4, w5 = synth.config(3), synth.config(4), synth.config(5)
    reuse, refresh, mixed = (args.only in ("all", w) for w in ("reuse", "refresh", "mixed"))
    # Copies per workload: a launch must not find what the launch before last left in the 256 MB
    # memory-side cache.  A Reuse attend touches about 200 MB of its copy, a Reuse select about 290 MB:
    # three copies; the Refresh and mixed calls move more than 500 MB each: two copies.
    d3 = [hcsa.DeviceWorkload(w3, "cuda:0") for _ in range(3 if reuse else 0)]
    d4 = [hcsa.DeviceWorkload(w4, "cuda:0") for _ in range(2 if refresh else 0)]
    d5 = [hcsa.DeviceWorkload(w5, "cuda:0") for _ in range(2 if mixed else 0)]

    def ws(nbytes):
        return torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda:0")

    calls = {}
    if reuse:
        ws3s = ws(hcsa.dllm_hcsa_select_workspace(d3[0].batch, d3[0].max_k))
        ws3a = ws(hcsa.dllm_hcsa_attend_workspace(d3[0].batch, d3[0].max_k))
        # the kept-row indices, the packed cache and the shared (head-summed, Section 2.4 Eq. 5) lists of every copy
        shared = []
        for d in d3:
            sh = torch.empty_like(d.idx)
            hcsa.dllm_hcsa_select_ex(d.batch, d.cu_k, d.total_k, d.max_k, sh, head_sum=True, workspace=ws3s)
            shared.append(sh)
            d.select(workspace=ws3s)
            d.pack()
        calls["attend_reuse"] = Train("attend_reuse", [lambda d=d: d.attend(workspace=ws3a) for d in d3])
        calls["select_reuse"] = Train("select_reuse", [lambda d=d: d.select(workspace=ws3s) for d in d3])
        calls["pack_reuse"] = Train("pack_reuse", [lambda d=d: d.pack() for d in d3])
        calls["attend_packed_reuse"] = Train("attend_packed_reuse",
                                             [lambda d=d: d.attend_packed(workspace=ws3a) for d in d3])
        calls["attend_shared_list_reuse"] = Train("attend_shared_list_reuse",
                                                  [lambda d=d, sh=sh: d.attend(sh, workspace=ws3a)
                                                   for d, sh in zip(d3, shared)])
    if refresh:
        calls["dense_refresh"] = Train("dense_refresh", [lambda d=d: d.dense_refresh() for d in d4])
    if mixed:
        ws5s = ws(hcsa.dllm_hcsa_select_workspace(d5[0].batch, d5[0].max_k))
        ws5a = ws(hcsa.dllm_hcsa_attend_workspace(d5[0].batch, d5[0].max_k))
        for d in d5:
            d.select(workspace=ws5s)
        calls["select_mixed"] = Train("select_mixed", [lambda d=d: d.select(workspace=ws5s) for d in d5])
        calls["attend_mixed"] = Train("attend_mixed", [lambda d=d: d.attend(workspace=ws5a) for d in d5])
        # each part of the mixed batch as a batch of its own, against its own roofline
        w5s = synth.subset(w5, np.flatnonzero(w5.seq_mode == 0), "c5_reuse_part")
        w5d = synth.subset(w5, np.flatnonzero(w5.seq_mode == 1), "c5_refresh_part")
        d5s = [hcsa.DeviceWorkload(w5s, "cuda:0") for _ in range(2)]
        d5d = [hcsa.DeviceWorkload(w5d, "cuda:0") for _ in range(2)]
        ws5p = ws(hcsa.dllm_hcsa_attend_workspace(d5s[0].batch, d5s[0].max_k))
        for d in d5s:
            d.select(workspace=ws5s)
        calls["attend_mixed_reuse_part_alone"] = Train("attend_mixed_reuse_part_alone",
                                                       [lambda d=d: d.attend(workspace=ws5p) for d in d5s])
        calls["attend_mixed_refresh_part_alone"] = Train("attend_mixed_refresh_part_alone",
                                                         [lambda d=d: d.dense_refresh() for d in d5d])
    order = [calls[n] for n in ("select_reuse", "attend_reuse", "pack_reuse", "attend_packed_reuse",
                                "attend_shared_list_reuse", "dense_refresh", "select_mixed", "attend_mixed",
                                "attend_mixed_reuse_part_alone", "attend_mixed_refresh_part_alone")
             if n in calls]
    torch.cuda.synchronize()

    if args.copy_probe:
        # one plain elementwise pass of known size: reads 1 GiB, writes 1 GiB (dst = src + 1 on int32)
        src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # K steps = K launches of every call; the launches of one call run as a train (see Train)
    for c in order:
        c.run(args.warmup, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for c in order:
        c.run(args.steps, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    T = {c.name: c.ms() for c in order}

    isolated = None
    if args.isolated:
        for c in order:
            c.reset()
        for _ in range(args.steps):
            for c in order:
                c.run_isolated(1)
        torch.cuda.synchronize()
        isolated = {c.name: [round(x, 5) for x in c.ms()] for c in order}

    warm = None
    if args.warm:
        # for contrast: the same calls with every launch on ONE copy and no flush, so that whatever
        # fits stays in the memory-side cache between launches
        for c in order:
            c.reset()
            c.fns = c.fns[:1]
            c.run(args.warmup, False, flush=False)
            c.run(args.steps, True, flush=False)
        torch.cuda.synchronize()
        warm = {c.name: [round(x, 5) for x in c.ms()] for c in order}

    def rate_gbps(nbytes, name):
        return nbytes / (T[name][0] * 1e-3) / 1e9 if name in T else None

    def rate_tflops(flops, name):
        return flops / (T[name][0] * 1e-3) / 1e12 if name in T else None

    reuse_gbps = rate_gbps(w3.attend_sparse_bytes(), "attend_reuse")
    select_gbps = rate_gbps(w3.select_bytes(), "select_reuse")
    refresh_tflops = rate_tflops(w4.attend_dense_flops(), "dense_refresh")
    mixed_sel_gbps = rate_gbps(w5.select_bytes(), "select_mixed")
    pack_gbps = rate_gbps(w3.pack_bytes(), "pack_reuse")
    packed_gbps = rate_gbps(w3.attend_packed_bytes(), "attend_packed_reuse")

    def roof(bound, achieved, peak, unit, kernel, algorithmic):
        if achieved is None:
            return None
        return {"bound": bound, "kernel": kernel, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "algorithmic_per_launch": algorithmic,
                "traffic": TRAFFIC_BYTES.get(kernel)}

    out = {
        "metric": "Reuse sparse-attn HBM GB/s (% of peak) + Refresh attn TFLOP/s, 1 MI355X",
        "value": reuse_gbps if reuse_gbps is not None else refresh_tflops,
        "unit": "GB/s" if reuse_gbps is not None else "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "c3_batched_reuse (value: Reuse attend) + c4_refresh_dense (Refresh TFLOP/s) + "
                        "c5_mixed_burst_gqa (one-call mixed dispatch)",
            "step": [c.name for c in order],
            "protocol": f"per call: {args.steps} launches back to back on rotating input copies, "
                        f"one event pair per {Train.chunk} launches, cold memory-side cache",
            "reuse": {"batch": w3.batch, "heads": w3.n_q_heads, "head_dim": w3.head_dim, "block": 32,
                      "sum_kv": w3.total_kv, "sum_keep": w3.total_k,
                      "attend_bytes": w3.attend_sparse_bytes(), "select_bytes": w3.select_bytes(),
                      "pack_bytes": w3.pack_bytes(), "attend_packed_bytes": w3.attend_packed_bytes()},
            "refresh": {"batch": w4.batch, "heads": w4.n_q_heads, "head_dim": w4.head_dim,
                        "L": int(w4.kv_lens[0]), "flops": w4.attend_dense_flops()},
            "mixed": {"batch": w5.batch, "q_heads": w5.n_q_heads, "kv_heads": w5.n_kv_heads,
                      "reuse_seqs": int((w5.seq_mode == 0).sum()), "refresh_seqs": int((w5.seq_mode == 1).sum()),
                      "sparse_bytes": w5.attend_sparse_bytes(), "dense_flops": w5.attend_dense_flops()},
        },
        "reuse_attend_gbps": reuse_gbps,
        "reuse_attend_pct_of_hbm_peak": None if reuse_gbps is None else 100.0 * reuse_gbps / HBM_PEAK_GBPS,
        "reuse_select_gbps": select_gbps,
        "refresh_tflops": refresh_tflops,
        "refresh_pct_of_mfma_peak": None if refresh_tflops is None else 100.0 * refresh_tflops / MFMA_BF16_PEAK_TFLOPS,
        "mixed_select_gbps": mixed_sel_gbps,
        # the paper's layout (pack once at Refresh, then read the packed cache sequentially) beside the gather design
        "reuse_pack_gbps": pack_gbps,
        "reuse_attend_packed_gbps": packed_gbps,
        # gather attend when all heads of a sequence share one kept set (head-summed selection, Eq. 5)
        "reuse_attend_shared_list_gbps": rate_gbps(w3.attend_sparse_bytes(), "attend_shared_list_reuse"),
        "call_ms_mean_min": {k: [round(v[0], 5), round(v[1], 5)] for k, v in T.items()},
        "call_ms_mean_min_warm": warm,
        "call_ms_mean_min_isolated": isolated,
        # the kernel that dominates the step's time is the dense Refresh kernel (one launch per call)
        "roofline": roof("mfma", refresh_tflops, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s", "attend_dense_bf16_kernel",
                         w4.attend_dense_flops()),
        "roofline_reuse": roof("hbm", reuse_gbps, HBM_PEAK_GBPS, "GB/s", "attend_sparse_multi_bf16_kernel",
                               w3.attend_sparse_bytes()),
        "roofline_select": roof("hbm", select_gbps, HBM_PEAK_GBPS, "GB/s", "score_kernel", w3.select_bytes()),
        "peaks": {"hbm_GBps": HBM_PEAK_GBPS, "mfma_bf16_dense_TFLOPs": MFMA_BF16_PEAK_TFLOPS},
        "measured_ceilings_context": MEASURED_CEILINGS,
        "paper_context": "dLLM-Serve reports end-to-end serving gains only (1.61-1.81x on RTX 4090, "
                         "1.60-1.74x on L40S); no kernel-level number exists for this path",
    }
    if "attend_mixed" in T:
        bound_ms = max(w5.attend_dense_flops() / (MFMA_BF16_PEAK_TFLOPS * 1e12),
                       w5.attend_sparse_bytes() / (HBM_PEAK_GBPS * 1e9)) * 1e3
        sparse_ms, dense_ms = T["attend_mixed_reuse_part_alone"][0], T["attend_mixed_refresh_part_alone"][0]
        out["mixed_attend"] = {
            "ms": T["attend_mixed"][0], "lower_bound_ms": bound_ms,
            # the two parts as batches of their own, each against its own roofline
            "reuse_part_alone_ms": sparse_ms,
            "reuse_part_alone_gbps": w5.attend_sparse_bytes() / (sparse_ms * 1e-3) / 1e9,
            "refresh_part_alone_ms": dense_ms,
            "refresh_part_alone_tflops": w5.attend_dense_flops() / (dense_ms * 1e-3) / 1e12,
            # the one call launches the dense part, then the sparse part, on the same stream
            "sparse_part_hidden_under_dense_part": bool(T["attend_mixed"][0] < dense_ms + 0.5 * sparse_ms),
            "one_call_over_sum_of_parts": T["attend_mixed"][0] / (dense_ms + sparse_ms)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w3, w4)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
