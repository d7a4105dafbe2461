#!/usr/bin/env python3
"""Benchmark of the Head-Centric Sparse Attention hot path on one MI355X.

One "step" is one pass of the whole hot path over resident synthetic inputs:
    select  + attend   on the batched Reuse workload   (16 seqs, KV 512..4096, keep 10..50 %)
    dense Refresh      on the Refresh workload          (8 x L=2048, 32 heads x 128)
    select  + attend   on the mixed GQA burst           (24 Reuse + 8 Refresh sequences in one call)
plus, on the first workload, the paper's own Reuse layout (pack the kept rows once, attend over the packed
cache), the gather attend with one kept set shared by all heads (the head-summed selection of Eq. 5) and the
selection options (pooling window 3, the block's own 32 positions forced, head-summed), and select + attend
on the two small configurations, where a call is a launch latency and not a bandwidth.
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

# HBM bytes per launch (reads, writes) from rocprofv3 --pmc runs of this script, one call and one counter per run
# (FETCH_SIZE, then WRITE_SIZE, each scaled by what it reads for the --copy-probe launch of known size).
# bench_traffic.py turns the profiler's CSV files into profiles/hbm_traffic.json (and the summary beside it, with
# the commands); the figures are properties of the workload shapes, not of the timing, so they are loaded from
# that file rather than re-measured on every run.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def load_traffic():
    """{call: {kernel: {"read_bytes": r, "write_bytes": w, ...}}} or {} when the file is not there."""
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f)["calls"]
    except (OSError, ValueError, KeyError):
        return {}


def traffic_of(traffic, call, kernel_prefix):
    """read + write bytes per launch of the kernel whose name starts with kernel_prefix in `call`, else None"""
    for name, t in traffic.get(call, {}).items():
        if name.startswith(kernel_prefix):
            return t["read_bytes"] + t["write_bytes"]
    return None


# What plain kernels reach on this GPU (python ceilings.py; profiles/ceilings_microbench.md):
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
    ap.add_argument("--no-warm", action="store_true",
                    help="skip the contrast pass that times every call again on one copy without flushes (warm caches)")
    ap.add_argument("--calls", default="",
                    help="comma-separated call names: launch only these in the warm-up and timed regions (profiling runs)")
    ap.add_argument("--isolated", action="store_true",
                    help="afterwards time every call again one launch at a time, each after a cache flush "
                         "and on an otherwise idle GPU, for contrast")
    ap.add_argument("--only", choices=["all", "reuse", "refresh", "mixed", "small"], default="all",
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
        """(mean per launch over all timed launches, best and median per-launch mean of the event pairs)"""
        t = [(a.elapsed_time(b), m) for a, b, m in self.pairs]
        if not t:
            return float("nan"), float("nan"), float("nan")
        per = sorted(x / m for x, m in t)
        mid = per[len(per) // 2] if len(per) % 2 else 0.5 * (per[len(per) // 2 - 1] + per[len(per) // 2])
        return sum(x for x, _ in t) / sum(m for _, m in t), per[0], mid

    def reset(self):
        self.pairs = []


def cpu_baseline(w3, w4, w5):
    """The oracle as it stands, timed on this host: the full Reuse workload (selection and attention),
    repeated for a steadier clock, one whole Refresh sequence (all heads), the mixed workload's selection
    and Reuse part once, and select + attend of the layer-shaped configuration on one thread (a child
    process with OMP_NUM_THREADS=1, started before anything here touches the GPU)."""
    import subprocess
    import numpy as np
    import oracle
    from paper_2512_17077_amd import synth
    one_thread_c2 = """
import sys, time
sys.path.insert(0, {root!r})
import ctypes, oracle, torch
from paper_2512_17077_amd import synth
w = synth.config(2)
q, k, v = synth.to_bits(w.q), synth.to_bits(w.k), synth.to_bits(w.v)
oracle.select(q, k, w.cu_q, w.cu_kv, w.cu_k)           # loads the oracle (and with it the OpenMP runtime)
torch.set_num_threads(1)                               # torch sets the runtime's team size when it is first used
ctypes.CDLL("libgomp.so.1").omp_set_num_threads(1)
t0 = time.perf_counter()
for _ in range(3):
    idx = oracle.select(q, k, w.cu_q, w.cu_kv, w.cu_k)
    oracle.attend(q, k, v, w.cu_q, w.cu_kv, idx, w.cu_k, None, w.softmax_scale)
print((time.perf_counter() - t0) / 3, oracle.num_threads())
"""
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
    # mixed workload: selection of all Reuse sequences, attention of the Reuse part
    w5s = synth.subset(w5, np.flatnonzero(w5.seq_mode == 0), "c5_reuse_part")
    q5, k5, v5 = synth.to_bits(w5s.q), synth.to_bits(w5s.k), synth.to_bits(w5s.v)
    t5 = time.perf_counter()
    idx5 = oracle.select(q5, k5, w5s.cu_q, w5s.cu_kv, w5s.cu_k)
    t6 = time.perf_counter()
    oracle.attend(q5, k5, v5, w5s.cu_q, w5s.cu_kv, idx5, w5s.cu_k, None, w5s.softmax_scale)
    t7 = time.perf_counter()
    env = dict(os.environ, OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-c", one_thread_c2.format(root=ROOT)], env=env, capture_output=True, text=True,
                       timeout=300)
    one = r.stdout.split() if r.returncode == 0 else []
    return {
        "value": w3.attend_sparse_bytes() / t_att / 1e9,
        "unit": "GB/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"full Reuse workload {w3.name}, mean of {reps} runs: attend {t_att:.3f} s, select {t_sel:.3f} s; "
                  f"Refresh: one whole L={L} sequence ({n} query rows x {w4.n_q_heads} heads) {t4 - t3:.2f} s; "
                  f"mixed workload once: select {t6 - t5:.2f} s, Reuse-part attend {t7 - t6:.2f} s",
        "select_gbps": w3.select_bytes() / t_sel / 1e9,
        "refresh_tflops": dense_flops / (t4 - t3) / 1e12,
        "c5_select_s": t6 - t5,
        "c5_select_gbps": w5.select_bytes() / (t6 - t5) / 1e9,
        "c5_reuse_part_attend_s": t7 - t6,
        "c2_one_thread_s": float(one[0]) if len(one) == 2 else None,
        "c2_one_thread_threads": int(one[1]) if len(one) == 2 else None,
    }


def gqa_union_bytes(w, idx):
    """Bytes the Reuse part would move if the query heads that share a KV head fetched the union of their kept
    rows once: one K and one V row per (sequence, KV head, position kept by any head of the group), plus Q in,
    O out and the per-head indices (idx: the selection's output, [Hq, total_k] on any device)."""
    import torch
    G = w.n_q_heads // w.n_kv_heads
    rows = 0
    for b in range(w.batch):
        lo, hi = int(w.cu_k[b]), int(w.cu_k[b + 1])
        if hi == lo or int(w.seq_mode[b]) != 0:
            continue
        part = idx[:, lo:hi].reshape(w.n_kv_heads, G * (hi - lo))
        rows += sum(int(torch.unique(part[g]).numel()) for g in range(w.n_kv_heads))
    sp = w.seq_mode == 0
    nq, nk = int(w.q_lens[sp].sum()), int(w.keep[sp].sum())
    e, d = w.elem_bytes, w.head_dim
    return 2 * rows * d * e + 2 * nq * w.n_q_heads * d * e + nk * w.n_q_heads * 4


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (asked for --gpus {args.gpus}); "
              "the path shards by sequence or by KV head with no exchange between GPUs", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2512_17077_amd import hcsa, synth, workload
    hcsa.lib()   # raises if the HIP library is not built: there is no fallback

    w1, w2, w3, w4, w5 = (synth.config(c) for c in (1, 2, 3, 4, 5))
    only_calls = [c for c in args.calls.split(",") if c]
    # the oracle is timed first: its one-thread leg starts a child process, and no process is started once the
    # GPU is in use
    cpu = None if (args.no_cpu_baseline or only_calls) else cpu_baseline(w3, w4, w5)

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)

    def wanted(group, names):
        if only_calls:
            return any(n in only_calls for n in names)
        return args.only in ("all", group)

    REUSE = ("select_reuse", "attend_reuse", "pack_reuse", "attend_packed_reuse", "attend_shared_list_reuse",
             "select_pool3_reuse", "select_forced32_reuse", "select_headsum_reuse", "select_reuse_one_launch")
    REFRESH = ("dense_refresh", "dense_refresh_zero_inputs")
    MIXED = ("select_mixed", "attend_mixed", "attend_mixed_reuse_part_alone", "attend_mixed_refresh_part_alone",
             "select_mixed_two_launches", "select_pool3_mixed")
    SMALL = ("select_c1", "attend_c1", "select_c2", "attend_c2")
    reuse, refresh, mixed = wanted("reuse", REUSE), wanted("refresh", REFRESH), wanted("mixed", MIXED)
    small = wanted("small", SMALL) if only_calls else args.only == "all"
    # Copies per workload: a launch must not find what the launch before last left in the 256 MB
    # memory-side cache.  A Reuse attend touches about 200 MB of its copy, a Reuse select about 290 MB:
    # three copies; the Refresh and mixed calls move more than 500 MB each: two copies.
    d3 = [workload.DeviceWorkload(w3, "cuda:0") for _ in range(3 if reuse else 0)]
    d4 = [workload.DeviceWorkload(w4, "cuda:0") for _ in range(2 if refresh else 0)]
    d5 = [workload.DeviceWorkload(w5, "cuda:0") for _ in range(2 if mixed else 0)]

    def ws(nbytes):
        return torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda:0")

    calls = {}

    def add(name, fns):
        calls[name] = Train(name, fns)

    def in_form(form, fn):
        """fn with selection forced into one of its two forms (the library chooses by shape otherwise)"""
        def run():
            hcsa.dllm_hcsa_set_select_form(form)
            fn()
            hcsa.dllm_hcsa_set_select_form(hcsa.DLLM_SELECT_FORM_AUTO)
        return run

    if reuse:
        ws3s = ws(hcsa.dllm_hcsa_select_workspace(d3[0].batch, d3[0].max_k))
        ws3a = ws(hcsa.dllm_hcsa_attend_workspace(d3[0].batch, d3[0].max_k))
        # the kept-row indices, the packed cache and the shared (head-summed, Section 2.4 Eq. 5) lists of every copy
        shared, scratch_idx = [], []
        for d in d3:
            sh = torch.empty_like(d.idx)
            hcsa.dllm_hcsa_select_ex(d.batch, d.cu_k, d.total_k, d.max_k, sh, head_sum=True, workspace=ws3s)
            shared.append(sh)
            scratch_idx.append(torch.empty_like(d.idx))   # where the timed option calls write, so d.idx stays the plain selection
            d.select(workspace=ws3s)
            d.pack()
        add("attend_reuse", [lambda d=d: d.attend(workspace=ws3a) for d in d3])
        add("select_reuse", [lambda d=d: d.select(workspace=ws3s) for d in d3])
        add("select_reuse_one_launch", [in_form(hcsa.DLLM_SELECT_FORM_ONE_LAUNCH, lambda d=d, out=out: hcsa.dllm_hcsa_select(
            d.batch, d.cu_k, d.total_k, d.max_k, out, workspace=ws3s)) for d, out in zip(d3, scratch_idx)])
        add("pack_reuse", [lambda d=d: d.pack() for d in d3])
        add("attend_packed_reuse", [lambda d=d: d.attend_packed(workspace=ws3a) for d in d3])
        add("attend_shared_list_reuse", [lambda d=d, sh=sh: d.attend(sh, workspace=ws3a) for d, sh in zip(d3, shared)])
        # the selection options on the same workload (Table 2's pooling window; Eq. 4's forced block; Eq. 5's head sum)
        for name, opt in (("select_pool3_reuse", dict(pool_w=3)), ("select_forced32_reuse", dict(forced_tail=32)),
                          ("select_headsum_reuse", dict(head_sum=True))):
            add(name, [lambda d=d, out=out, opt=opt: hcsa.dllm_hcsa_select_ex(d.batch, d.cu_k, d.total_k, d.max_k, out,
                                                                               workspace=ws3s, **opt)
                       for d, out in zip(d3, scratch_idx)])
    if refresh:
        add("dense_refresh", [lambda d=d: d.dense_refresh() for d in d4])
        if not only_calls or "dense_refresh_zero_inputs" in only_calls:
            # the same launches on all-zero Q, K, V: the same instructions and bytes, fewer bits toggling; the board's
            # power limit sets the clock of this kernel, so the difference is what the data costs
            d4z = [workload.DeviceWorkload(w4, "cuda:0") for _ in range(2)]
            for d in d4z:
                d.q.zero_(), d.k.zero_(), d.v.zero_()
            add("dense_refresh_zero_inputs", [lambda d=d: d.dense_refresh() for d in d4z])
    union_bytes = None
    if mixed:
        ws5s = ws(hcsa.dllm_hcsa_select_workspace(d5[0].batch, d5[0].max_k))
        ws5a = ws(hcsa.dllm_hcsa_attend_workspace(d5[0].batch, d5[0].max_k))
        for d in d5:
            d.select(workspace=ws5s)
        torch.cuda.synchronize()
        union_bytes = gqa_union_bytes(w5, d5[0].idx)
        add("select_mixed", [lambda d=d: d.select(workspace=ws5s) for d in d5])
        add("select_mixed_two_launches", [in_form(hcsa.DLLM_SELECT_FORM_TWO_LAUNCHES, lambda d=d: d.select(workspace=ws5s))
                                          for d in d5])
        # the paper's default pooling window (Table 2) on the grouped-query workload; results go to a scratch list
        pool_idx = [torch.empty_like(d.idx) for d in d5]
        add("select_pool3_mixed", [lambda d=d, out=out: hcsa.dllm_hcsa_select(d.batch, d.cu_k, d.total_k, d.max_k, out, 3,
                                                                               workspace=ws5s) for d, out in zip(d5, pool_idx)])
        add("attend_mixed", [lambda d=d: d.attend(workspace=ws5a) for d in d5])
        # each part of the mixed batch as a batch of its own, against its own roofline
        w5s = synth.subset(w5, np.flatnonzero(w5.seq_mode == 0), "c5_reuse_part")
        w5d = synth.subset(w5, np.flatnonzero(w5.seq_mode == 1), "c5_refresh_part")
        d5s = [workload.DeviceWorkload(w5s, "cuda:0") for _ in range(2)]
        d5d = [workload.DeviceWorkload(w5d, "cuda:0") for _ in range(2)]
        ws5p = ws(hcsa.dllm_hcsa_attend_workspace(d5s[0].batch, d5s[0].max_k))
        for d in d5s:
            d.select(workspace=ws5s)
        add("attend_mixed_reuse_part_alone", [lambda d=d: d.attend(workspace=ws5p) for d in d5s])
        add("attend_mixed_refresh_part_alone", [lambda d=d: d.dense_refresh() for d in d5d])
    if small:
        # the two small configurations: a call here is launch latency (their inputs stay in cache whatever is done)
        for tag, w in (("c1", w1), ("c2", w2)):
            ds = [workload.DeviceWorkload(w, "cuda:0") for _ in range(2)]
            wss = ws(hcsa.dllm_hcsa_select_workspace(ds[0].batch, ds[0].max_k))
            wsa = ws(hcsa.dllm_hcsa_attend_workspace(ds[0].batch, ds[0].max_k))
            for d in ds:
                d.select(workspace=wss)
            add(f"select_{tag}", [lambda d=d, wss=wss: d.select(workspace=wss) for d in ds])
            add(f"attend_{tag}", [lambda d=d, wsa=wsa: d.attend(workspace=wsa) for d in ds])
    names = REUSE[:5] + REFRESH[:1] + MIXED[:4] + REUSE[5:] + MIXED[4:] + REFRESH[1:] + SMALL
    order = [calls[n] for n in names if n in calls and (not only_calls or n in only_calls)]
    # what BASELINE's metric counts as the step: the whole hot path on the three workloads
    step_calls = ("select_reuse", "attend_reuse", "dense_refresh", "select_mixed", "attend_mixed")
    torch.cuda.synchronize()

    if args.copy_probe:
        # one plain elementwise pass of known size: reads 1 GiB, writes 1 GiB (dst = src + 1 on int32)
        src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # K steps = K launches of every call of the step; the launches of one call run as a train (see Train).
    # The timed region holds the step's calls only; the other calls are timed the same way right after it.
    in_step = [c for c in order if c.name in step_calls]
    beside = [c for c in order if c.name not in step_calls]
    for c in in_step:
        c.run(args.warmup, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for c in in_step:
        c.run(args.steps, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    for c in beside:
        c.run(args.warmup, False)
        c.run(args.steps, True)
    torch.cuda.synchronize()
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
    if not args.no_warm:
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
    traffic = load_traffic()

    def roof(bound, achieved, peak, unit, call, kernel, algorithmic):
        if achieved is None:
            return None
        return {"bound": bound, "kernel": kernel, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "algorithmic_per_launch": algorithmic,
                "traffic": traffic_of(traffic, call, kernel)}

    out = {
        "metric": "Reuse sparse-attn HBM GB/s (% of peak) + Refresh attn TFLOP/s, 1 MI355X",
        "value": reuse_gbps if reuse_gbps is not None else refresh_tflops,
        "unit": "GB/s" if reuse_gbps is not None else "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        # one step = select + attend on c3, dense Refresh on c4, select + attend on c5: wall clock of the timed region
        # over the steps (cache flushes between the calls' trains included); the other calls (packed layout, selection
        # options, parts of the mixed batch alone, small configurations) are timed after it and reported beside it
        "ms_per_step": ms_per_step,
        "ms_per_step_sum_of_mean_launches": sum(T[n][0] for n in step_calls if n in T),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "c3_batched_reuse (value: Reuse attend) + c4_refresh_dense (Refresh TFLOP/s) + "
                        "c5_mixed_burst_gqa (one-call mixed dispatch)",
            "step": [n for n in step_calls if n in T],
            "also_timed": [c.name for c in order if c.name not in step_calls],
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
                      "select_bytes": w5.select_bytes(), "sparse_bytes": w5.attend_sparse_bytes(),
                      "sparse_bytes_gqa_union": union_bytes, "dense_flops": w5.attend_dense_flops()},
        },
        "reuse_attend_gbps": reuse_gbps,
        "reuse_attend_pct_of_hbm_peak": None if reuse_gbps is None else 100.0 * reuse_gbps / HBM_PEAK_GBPS,
        "reuse_select_gbps": select_gbps,
        "reuse_select_pct_of_hbm_peak": None if select_gbps is None else 100.0 * select_gbps / HBM_PEAK_GBPS,
        "refresh_tflops": refresh_tflops,
        "refresh_tflops_zero_inputs": rate_tflops(w4.attend_dense_flops(), "dense_refresh_zero_inputs"),
        "refresh_pct_of_mfma_peak": None if refresh_tflops is None else 100.0 * refresh_tflops / MFMA_BF16_PEAK_TFLOPS,
        "mixed_select_gbps": mixed_sel_gbps,
        "mixed_select_pct_of_hbm_peak": None if mixed_sel_gbps is None else 100.0 * mixed_sel_gbps / HBM_PEAK_GBPS,
        # the paper's layout (pack once at Refresh, then read the packed cache sequentially) beside the gather design
        "reuse_pack_gbps": pack_gbps,
        "reuse_attend_packed_gbps": packed_gbps,
        # gather attend when all heads of a sequence share one kept set (head-summed selection, Eq. 5)
        "reuse_attend_shared_list_gbps": rate_gbps(w3.attend_sparse_bytes(), "attend_shared_list_reuse"),
        # selection with its options on the Reuse workload (same algorithmic bytes as the plain call)
        "reuse_select_options_gbps": {n: rate_gbps(w3.select_bytes(), n)
                                      for n in ("select_pool3_reuse", "select_forced32_reuse", "select_headsum_reuse")},
        # selection in the form the library does not choose for the workload: one launch on the ragged Reuse batch
        # (it takes two there), two launches on the mixed grouped-query burst (it takes one there)
        "select_other_form_gbps": {"select_reuse_one_launch": rate_gbps(w3.select_bytes(), "select_reuse_one_launch"),
                                   "select_mixed_two_launches": rate_gbps(w5.select_bytes(), "select_mixed_two_launches")},
        "mixed_select_pool3_gbps": rate_gbps(w5.select_bytes(), "select_pool3_mixed"),
        # the small configurations: microseconds per call (launch latency, not a bandwidth)
        "small_config_call_us": {n: round(T[n][0] * 1e3, 2) for n in SMALL if n in T},
        "call_ms_mean_min_median": {k: [round(x, 5) for x in v] for k, v in T.items()},
        "call_ms_mean_min_median_warm": warm,
        "call_ms_mean_min_median_isolated": isolated,
        # the kernel that dominates the step's time is the dense Refresh kernel (one launch per call)
        "roofline": roof("mfma", refresh_tflops, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s", "dense_refresh",
                         "attend_dense_bf16_kernel", w4.attend_dense_flops()),
        "roofline_reuse": roof("hbm", reuse_gbps, HBM_PEAK_GBPS, "GB/s", "attend_reuse",
                               "attend_sparse_multi_bf16_kernel", w3.attend_sparse_bytes()),
        "roofline_select": roof("hbm", select_gbps, HBM_PEAK_GBPS, "GB/s", "select_reuse", "score_kernel",
                                w3.select_bytes()),
        "roofline_select_mixed": roof("hbm", mixed_sel_gbps, HBM_PEAK_GBPS, "GB/s", "select_mixed", "select_fused_kernel",
                                      w5.select_bytes()),
        "peaks": {"hbm_GBps": HBM_PEAK_GBPS, "mfma_bf16_dense_TFLOPs": MFMA_BF16_PEAK_TFLOPS},
        "measured_ceilings_context": MEASURED_CEILINGS,
        "paper_context": "dLLM-Serve reports end-to-end serving gains only (1.61-1.81x on RTX 4090, "
                         "1.60-1.74x on L40S); no kernel-level number exists for this path",
    }
    if "attend_mixed" in T and "attend_mixed_reuse_part_alone" in T and "attend_mixed_refresh_part_alone" in T:
        bound_ms = max(w5.attend_dense_flops() / (MFMA_BF16_PEAK_TFLOPS * 1e12),
                       w5.attend_sparse_bytes() / (HBM_PEAK_GBPS * 1e9)) * 1e3
        sparse_ms, dense_ms = T["attend_mixed_reuse_part_alone"][0], T["attend_mixed_refresh_part_alone"][0]
        dense_t = traffic.get("attend_mixed_refresh_part_alone", {})
        dense_t = next((t for k, t in dense_t.items() if k.startswith("attend_dense")), None)
        # algorithmic reads of the dense part with grouped queries: Q once, K and V of the KV heads once
        nd = int((w5.seq_mode == 1).sum())
        Ld = int(w5.kv_lens[w5.seq_mode == 1][0])
        dense_read_alg = nd * Ld * (w5.n_q_heads + 2 * w5.n_kv_heads) * w5.head_dim * 2
        out["mixed_attend"] = {
            "ms": T["attend_mixed"][0], "lower_bound_ms": bound_ms,
            # the two parts as batches of their own, each against its own roofline
            "reuse_part_alone_ms": sparse_ms,
            # every query head gathers its own kept rows: the per-head sum is what the kernel moves; the smaller
            # figure counts a row kept by several heads of a KV-head group once
            "reuse_part_bytes_per_head": w5.attend_sparse_bytes(),
            "reuse_part_bytes_gqa_union": union_bytes,
            "reuse_part_alone_gbps": w5.attend_sparse_bytes() / (sparse_ms * 1e-3) / 1e9,
            "reuse_part_alone_gbps_gqa_union": union_bytes / (sparse_ms * 1e-3) / 1e9,
            "reuse_part_alone_pct_of_hbm_peak": 100.0 * w5.attend_sparse_bytes() / (sparse_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "reuse_part_alone_pct_of_hbm_peak_gqa_union": 100.0 * union_bytes / (sparse_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "refresh_part_alone_ms": dense_ms,
            "refresh_part_alone_tflops": w5.attend_dense_flops() / (dense_ms * 1e-3) / 1e12,
            "refresh_part_read_bytes_counter": None if dense_t is None else dense_t["read_bytes"],
            "refresh_part_read_bytes_algorithmic": dense_read_alg,
            # the one call launches the dense part, then the sparse part, on the same stream
            "sparse_part_hidden_under_dense_part": bool(T["attend_mixed"][0] < dense_ms + 0.5 * sparse_ms),
            "one_call_over_sum_of_parts": T["attend_mixed"][0] / (dense_ms + sparse_ms)}
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
