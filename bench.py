#!/usr/bin/env python3
"""Benchmark of the SpecTr-GBV verification hot path on one MI355X.

A step is one specgbv_verify call (statistics + sums of Eq. (hik), Algorithm 1's decision
scan, residual / bonus draw) over one synthetic batch already resident in HBM.  Prints ONE
JSON line with whole-call throughput (verifications/s), the HBM roofline figures of the
dominant (vocabulary-streaming) kernel measured with HIP events, and the CPU oracle timed
on the host cores of the same machine as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ProcessPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from specgbv_synth import WORKLOADS, make_prefix, with_batch  # noqa: E402

HBM_PEAK_GBS = 8000.0


def _gen(args):
    name, seed, b = args
    return make_prefix(WORKLOADS[name], seed, b)


def generate(name: str, seed: int, workers: int, batch: int = 0):
    w = WORKLOADS[name]
    if batch > 0:
        w = with_batch(w, batch)                       # the first `batch` prefixes of the workload
    store = np.uint16 if w.dtype == "bf16" else np.float32
    target = np.empty((w.batch, w.K, w.L + 1, w.V), dtype=store)
    draft = np.empty((w.batch, w.K, w.L, w.V), dtype=store)
    tokens = np.empty((w.batch, w.K, w.L), dtype=np.int32)
    jobs = [(name, seed, b) for b in range(w.batch)]
    if workers > 1:
        with ProcessPoolExecutor(max_workers=workers) as ex:
            for b, (t, d, k) in enumerate(ex.map(_gen, jobs)):
                target[b], draft[b], tokens[b] = t, d, k
    else:
        for b, j in enumerate(jobs):
            target[b], draft[b], tokens[b] = _gen(j)
    return target, draft, tokens


FULL_WORKLOAD = True        # False with --batch: the committed traffic figures are those of the whole workload


def committed_traffic(tag: str):
    """HBM bytes per call from the committed rocprofv3 --pmc summary profiles/hbm_traffic_<tag>.txt (FETCH_SIZE +
    WRITE_SIZE, calibrated against a plain copy), or None.  The figure is NOT measured in this run (counters need
    the profiler): traffic_source() says which file it comes from and what that file says about its origin."""
    if not FULL_WORKLOAD:
        return None
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % tag)
    if os.path.exists(path):
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    return None


def traffic_source(tag: str):
    """Provenance of committed_traffic(tag): the file and its `measured:` line (date, kernel source revision)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % tag)
    if not FULL_WORKLOAD or not os.path.exists(path):
        return None
    measured = [ln.split(":", 1)[1].strip() for ln in open(path) if ln.startswith("measured:")]
    return {"file": "profiles/hbm_traffic_%s.txt" % tag, "measured": measured[0] if measured else "not recorded",
            "note": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command, not of this run"}


def bench_modify(a, w, sg, torch, tl, dl, tk, ws, out):
    """One step = one specgbv_modify_target call over the whole batch: M = L draft rows plus the bonus row per
    draft, float32 log-probabilities of both models written.  The carried ratios and row counts are those a
    verification of the same batch leaves in its workspace (the tensors stand in for the next iteration's)."""
    sg.specgbv_verify_ex(tl, dl, tk, w.temperature, a.seed, 0, workspace=ws, out=out, algo=a.algo)
    carry_ptr, count_ptr = sg.specgbv_workspace_carry(ws, w.batch, w.K, w.L, w.V)
    torch.cuda.synchronize()
    dt = 1 if w.dtype == "bf16" else 0
    counts = sg.specgbv_read_intermediates(ws, w.batch, w.K, w.L, w.V, dt)["modify_count"]
    res = sg.specgbv_modify_target(tl, dl, tk, w.temperature, carry_ptr, count_ptr, want_logp=True)
    for _ in range(a.warmup):
        sg.specgbv_modify_target(tl, dl, tk, w.temperature, carry_ptr, count_ptr, want_logp=True, out=res)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(a.steps)]
    t0 = time.perf_counter()
    for e0, e1 in evs:
        e0.record()
        sg.specgbv_modify_target(tl, dl, tk, w.temperature, carry_ptr, count_ptr, want_logp=True, out=res)
        e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / a.steps
    ker = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    avg = sum(ker) / len(ker)
    rows_d, rows_t = w.batch * w.K * w.L, w.batch * w.K * (w.L + 1)
    read_b = (rows_d + rows_t) * w.V * w.elem_bytes          # every input row once
    write_b = (rows_d + rows_t) * w.V * 4                    # float32 log-probabilities of both models
    achieved = (read_b + write_b) / (avg * 1e-3) / 1e9
    return {
        "metric": "distribution modifications/sec (Algorithm 2) and achieved HBM GB/s (% of peak) at K=8, L=8, V=128256",
        "value": w.batch / (ms_per_step * 1e-3), "unit": "prefixes/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: batch %d, K=%d, M=L=%d plus bonus row, V=%d, %s logits, T=%g" % (
                       w.name, w.batch, w.K, w.L, w.V, w.dtype, w.temperature),
                   "mean_rows_modified": float(np.mean(counts)), "outputs": "logq [B,K,L+1,V] and logp [B,K,L,V], float32"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": committed_traffic("modify_" + w.name),
                     "kernel": "k_mod_row + k_mod_norm + k_mod_write",
                     "kernel_ms_avg": avg, "kernel_ms_min": ker[0],
                     "algorithmic_bytes_per_launch": read_b + write_b,
                     "algorithmic_read_bytes": read_b, "algorithmic_write_bytes": write_b},
    }


def bench_pending(a, w, sg, torch, tl, dl, tk, ws, out):
    """One step = one specgbv_verify_ex call that applies a pending distribution modification on the fly
    (Algorithm 2 inside the verification of the next iteration).  The carried ratios and row counts are those
    a verification of the same batch leaves in its workspace (the tensors stand in for the next iteration's)."""
    sg.specgbv_verify_ex(tl, dl, tk, w.temperature, a.seed, 0, workspace=ws, out=out, algo=a.algo)
    torch.cuda.synchronize()
    dt = 1 if w.dtype == "bf16" else 0
    inter = sg.specgbv_read_intermediates(ws, w.batch, w.K, w.L, w.V, dt)
    pend = (torch.from_numpy(inter["carry_log_nu"]).to(tl.device), torch.from_numpy(inter["modify_count"]).to(tl.device))
    for i in range(a.warmup):
        sg.specgbv_verify_ex(tl, dl, tk, w.temperature, a.seed, 1 + i, workspace=ws, out=out, pending=pend, algo=a.algo)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(a.steps)]
    t0 = time.perf_counter()
    for i, (e0, e1) in enumerate(evs):
        e0.record()
        sg.specgbv_verify_ex(tl, dl, tk, w.temperature, a.seed, 1 + a.warmup + i, workspace=ws, out=out, pending=pend, algo=a.algo)
        e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / a.steps
    ker = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    avg = sum(ker) / len(ker)
    bytes_ = w.batch * w.K * w.L * 2 * w.V * w.elem_bytes     # every (target, draft) row pair once
    achieved = bytes_ / (avg * 1e-3) / 1e9
    return {
        "metric": "verifications/sec under a pending distribution modification applied on the fly (Algorithms 1 + 2) "
                  "and achieved HBM GB/s (% of peak) at K=8, L=8, V=128256",
        "value": w.batch / (ms_per_step * 1e-3), "unit": "verifications/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: batch %d, K=%d, L=%d, V=%d, %s logits, T=%g" % (
                       w.name, w.batch, w.K, w.L, w.V, w.dtype, w.temperature),
                   "mean_rows_modified": float(np.mean(inter["modify_count"])),
                   "schedule": "chain" if a.algo == "chain" else "two-pass"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": committed_traffic("pending_" + w.name),
                     "kernel": "k_row_stats + k_pend_norm + k_ot_sum + k_final (whole call)",
                     "kernel_ms_avg": avg, "kernel_ms_min": ker[0], "algorithmic_bytes_per_launch": bytes_},
    }


def bench_iterate(a, w, sg, torch, sets, ws, out):
    """One step = one specgbv_verify_ex call with the pending state: the verification under every distribution
    modification still pending for each prefix, and Algorithm 3's bookkeeping, all on the device.  The state
    starts empty and evolves from call to call.  With one input set the same synthetic tensors stand in for every
    iteration's drafts, so a prefix accepts about the same length every time and modifications pile up more than
    they would behind real models (a pessimistic steady state); with --input-sets N the iterations cycle through
    N independent sets, so accepted lengths vary from iteration to iteration as they do in decoding."""
    tl = sets[0][0]
    state = torch.zeros(sg.specgbv_pending_state_bytes(w.batch), dtype=torch.uint8, device=tl.device)
    nwarm = max(a.warmup, 2 * w.L)                           # long enough for the number of levels to settle
    for i in range(nwarm):
        tl, dl, tk = sets[i % len(sets)]
        sg.specgbv_verify_ex(tl, dl, tk, w.temperature, a.seed, i, workspace=ws, out=out, pending_state=state, algo=a.algo)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(a.steps)]
    t0 = time.perf_counter()
    for i, (e0, e1) in enumerate(evs):
        tl, dl, tk = sets[(nwarm + i) % len(sets)]
        e0.record()
        sg.specgbv_verify_ex(tl, dl, tk, w.temperature, a.seed, 1000 + i, workspace=ws, out=out, pending_state=state, algo=a.algo)
        e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / a.steps
    ker = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    avg = sum(ker) / len(ker)
    # levels and rows pending, averaged over one more cycle of untimed iterations
    lev, rows_mod, lev_max = [], [], 0
    for i in range(max(len(sets), 4)):
        cnt = sg.pending_state_views(state.cpu().numpy(), w.batch)[1]
        lev.append(float((cnt > 0).sum(0).mean())); rows_mod.append(float(cnt.max(0).mean()))
        lev_max = max(lev_max, int((cnt > 0).sum(0).max()))
        tl, dl, tk = sets[(nwarm + a.steps + i) % len(sets)]
        sg.specgbv_verify_ex(tl, dl, tk, w.temperature, a.seed, 5000 + i, workspace=ws, out=out, pending_state=state, algo=a.algo)
    torch.cuda.synchronize()
    bytes_ = w.batch * w.K * w.L * 2 * w.V * w.elem_bytes     # every (target, draft) row pair once
    achieved = bytes_ / (avg * 1e-3) / 1e9
    return {
        "metric": "decoding iterations/sec: verification under all pending distribution modifications plus Algorithm 3's "
                  "bookkeeping on the device, and achieved HBM GB/s (% of peak) at K=8, L=8, V=128256",
        "value": w.batch / (ms_per_step * 1e-3), "unit": "verifications/s", "n_gpus": 1, "steps": a.steps,
        "warmup": nwarm, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: batch %d, K=%d, L=%d, V=%d, %s logits, T=%g" % (
                       w.name, w.batch, w.K, w.L, w.V, w.dtype, w.temperature),
                   "input_sets": len(sets), "mean_levels_pending": sum(lev) / len(lev), "max_levels_pending": lev_max,
                   "mean_rows_modified": sum(rows_mod) / len(rows_mod), "schedule": "chain" if a.algo == "chain" else "two-pass"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": committed_traffic("iterate_" + w.name) if len(sets) == 1 else None,
                     "kernel": "k_row_stats + (L-1) x k_pend_norm + k_ot_sum + k_final (whole call)",
                     "kernel_ms_avg": avg, "kernel_ms_min": ker[0], "algorithmic_bytes_per_launch": bytes_},
    }


def bench_sample(a, w, sg, torch, dl):
    """One step = one specgbv_sample_tokens call: one token for each of the batch * K draft rows of one position."""
    rows = dl[:, :, 0].contiguous().view(w.batch * w.K, w.V)
    tok, ws = sg.specgbv_sample_tokens(rows, w.temperature, a.seed, 0, 0)
    for i in range(a.warmup):
        sg.specgbv_sample_tokens(rows, w.temperature, a.seed, i, 0, out=tok, workspace=ws)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(a.steps)]
    t0 = time.perf_counter()
    for i, (e0, e1) in enumerate(evs):
        e0.record()
        sg.specgbv_sample_tokens(rows, w.temperature, a.seed, a.warmup + i, 0, out=tok, workspace=ws)
        e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / a.steps
    ker = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    avg = sum(ker) / len(ker)
    n = w.batch * w.K
    bytes_ = n * w.V * w.elem_bytes                         # every row once
    achieved = bytes_ / (avg * 1e-3) / 1e9
    return {
        "metric": "draft tokens drawn/sec (Algorithm 3 drafting step) and achieved HBM GB/s (% of peak) at V=128256",
        "value": n / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %d draft rows (batch %d x K=%d) of one position, V=%d, %s logits, T=%g" % (
            w.name, n, w.batch, w.K, w.V, w.dtype, w.temperature)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": committed_traffic("sample_" + w.name),
                     "kernel": "k_sample_rows",
                     "kernel_ms_avg": avg, "kernel_ms_min": ker[0], "algorithmic_bytes_per_launch": bytes_},
    }


def bench_compare(a, w, sg, torch, tl, dl, tk):
    """Accepted tokens per iteration and verification time of the four verifiers the paper compares (its Table 1 /
    Table 2 / Fig. 2, on synthetic logits): token-level speculative decoding (Section 3.1, draft 0), greedy block
    verification (Section 3.3 = the main verifier at K = 1, draft 0), SpecTr K-SEQ (Section 3.2) and SpecTr-GBV
    (Algorithm 1), each with the first k of the K drafts for k in a small sweep.  One 'call' verifies the whole
    batch; accepted lengths are averaged over the batch and over --steps calls with different Philox offsets."""
    dev = tl.device
    ks = sorted({k for k in (1, 2, 3, 4, 5, 8, 16) if k <= w.K} | {w.K})
    rows = []

    def run(name, k, fn):
        t_k = tl[:, :k].contiguous() if k < w.K else tl
        d_k = dl[:, :k].contiguous() if k < w.K else dl
        tok_k = tk[:, :k].contiguous() if k < w.K else tk
        dt = 1 if w.dtype == "bf16" else 0
        ws = torch.empty(sg.specgbv_workspace_bytes(w.batch, k, w.L, w.V, dt), dtype=torch.uint8, device=dev)
        out = (torch.empty(w.batch, dtype=torch.int32, device=dev), torch.empty(w.batch, dtype=torch.int32, device=dev),
               torch.empty((w.batch, w.L + 1), dtype=torch.int32, device=dev))
        acc = torch.zeros((), dtype=torch.float64, device=dev)
        for i in range(max(a.warmup, 3)):                  # (the reductions below are warmed up too)
            fn(t_k, d_k, tok_k, i, ws, out)
            acc += out[0].double().mean()
        torch.cuda.synchronize()
        # time: the verifier calls alone, back to back on the stream
        t0 = time.perf_counter()
        for i in range(a.steps):
            fn(t_k, d_k, tok_k, 100 + i, ws, out)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / a.steps
        # accepted lengths: the same calls again, each followed by the batch mean of its result
        acc.zero_()
        for i in range(a.steps):
            fn(t_k, d_k, tok_k, 100 + i, ws, out)
            acc += out[0].double().mean()
        torch.cuda.synchronize()
        rows.append({"verifier": name, "drafts": k, "mean_accepted_len": float(acc.item()) / a.steps,
                     "tokens_per_iteration": float(acc.item()) / a.steps + 1.0, "ms_per_call": ms})

    gbv = lambda t, d, tok, off, ws, out: sg.specgbv_verify_ex(t, d, tok, w.temperature, a.seed, off, workspace=ws, out=out)
    kseq = lambda t, d, tok, off, ws, out: sg.specgbv_verify_kseq(t, d, tok, w.temperature, a.seed, off, workspace=ws, out=out)
    run("token-level SD (Section 3.1)", 1, kseq)
    run("GBV (Section 3.3)", 1, gbv)
    for k in ks:
        if k > 1:
            run("SpecTr K-SEQ (Section 3.2)", k, kseq)
            run("SpecTr-GBV (Algorithm 1)", k, gbv)
    best = max(r["tokens_per_iteration"] for r in rows)
    return {
        "metric": "accepted tokens per iteration and verification ms per call of the four verifiers of the paper's comparison",
        "value": best, "unit": "tokens/iteration (best verifier)", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": rows[-1]["ms_per_call"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: batch %d, K=%d, L=%d, V=%d, %s logits, T=%g" % (
            w.name, w.batch, w.K, w.L, w.V, w.dtype, w.temperature)},
        "table": rows,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: 0.15 s of GPU work.  Under the streaming kernel's load the shader clock takes some tens of
    # milliseconds to settle (a serving GPU runs such kernels all the time); 50 steps after 5 warm-up calls, 15 ms
    # in all, measure mostly that transient and read 8 - 10 % slower
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="cfg4", choices=sorted(WORKLOADS))
    ap.add_argument("--algo", default="auto", choices=["auto", "split", "chain"])
    ap.add_argument("--op", default="verify", choices=["verify", "modify", "sample", "pending", "iterate", "compare"],
                    help="verify: the verification call (the benchmark); modify: the distribution modification "
                         "(Algorithm 2) for the drafts of the next iteration, on the same tensors; "
                         "sample: the draft-side token draw of one position (Algorithm 3) over the batch * K draft rows; "
                         "pending: the verification with a pending modification applied on the fly; "
                         "iterate: the verification with the pending state (all pending modifications and their bookkeeping); "
                         "compare: accepted lengths and times of token-level SD, GBV, SpecTr K-SEQ and SpecTr-GBV on the same inputs")
    ap.add_argument("--shared-row0", type=int, default=0, choices=[0, 1],
                    help="verify only: tell the library that rows 0 of a prefix's K drafts are copies of one another "
                         "(they are in these inputs, as in Algorithm 3); the chain schedule then reads them once per "
                         "prefix, and the algorithmic bytes are counted accordingly")
    ap.add_argument("--input-sets", type=int, default=1,
                    help="iterate only: cycle through this many independent input sets (seeds seed, seed+1, ...)")
    ap.add_argument("--batch", type=int, default=0,
                    help="use only the first N prefixes of the workload (0 = all); a reduced batch is not the benchmark "
                         "configuration: for latency measurements at small batches")
    ap.add_argument("--settle-ms", type=float, default=80.0,
                    help="verify only: before the --warmup calls, keep issuing the same call for this many milliseconds "
                         "(untimed): under this kernel's load the shader clock takes some tens of milliseconds to settle, "
                         "and a serving GPU is always in the settled state; 0 switches it off.  Reported in the JSON")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--workers", type=int, default=0, help="input-generation processes (0 = one per CPU, at most 16)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also run a plain device-to-device copy of this many MiB (three times) before the timed "
                         "region: under rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings calibrate the counters")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build measures one GPU only (the path is independent over prefixes: more GPUs would "
              "each verify their share of the batch); run with --gpus 1", file=sys.stderr)
        return 2

    w = WORKLOADS[a.workload]
    if a.batch > 0:
        if a.batch > w.batch:
            print("bench.py: --batch exceeds the workload's %d prefixes" % w.batch, file=sys.stderr)
            return 2
        w = with_batch(w, a.batch)
        global FULL_WORKLOAD
        FULL_WORKLOAD = False
    # inputs are generated on the host before the GPU is touched (worker processes fork here)
    t0 = time.time()
    target, draft, tokens = generate(a.workload, a.seed, workers=a.workers or min(16, os.cpu_count() or 1), batch=a.batch)
    gen_s = time.time() - t0
    more_sets = []
    if a.op == "iterate":
        more_sets = [generate(a.workload, a.seed + j, workers=a.workers or min(16, os.cpu_count() or 1), batch=a.batch)
                     for j in range(1, max(1, a.input_sets))]

    import torch
    import paper_2604_25925_amd as sg
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")

    def up(x):
        if x.dtype == np.uint16:
            return torch.from_numpy(x.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(x).to(dev)

    tl, dl, tk = up(target), up(draft), up(tokens)
    dt = 1 if w.dtype == "bf16" else 0
    ws = torch.empty(sg.specgbv_workspace_bytes(w.batch, w.K, w.L, w.V, dt), dtype=torch.uint8, device=dev)
    out = (torch.empty(w.batch, dtype=torch.int32, device=dev), torch.empty(w.batch, dtype=torch.int32, device=dev),
           torch.empty((w.batch, w.L + 1), dtype=torch.int32, device=dev))

    def step(offset, events=None):
        sg.specgbv_verify_ex(tl, dl, tk, w.temperature, a.seed, offset, workspace=ws, out=out, algo=a.algo,
                             events=events, shared_row0=bool(a.shared_row0))

    if a.calibrate_copy_mib > 0:
        src = torch.empty(a.calibrate_copy_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if a.op == "sample":
        print(json.dumps(bench_sample(a, w, sg, torch, dl)))
        return 0
    if a.op == "compare":
        print(json.dumps(bench_compare(a, w, sg, torch, tl, dl, tk)))
        return 0
    if a.op == "modify":
        print(json.dumps(bench_modify(a, w, sg, torch, tl, dl, tk, ws, out)))
        return 0
    if a.op == "pending":
        print(json.dumps(bench_pending(a, w, sg, torch, tl, dl, tk, ws, out)))
        return 0
    if a.op == "iterate":
        sets = [(tl, dl, tk)] + [tuple(up(x) for x in more) for more in more_sets]
        print(json.dumps(bench_iterate(a, w, sg, torch, sets, ws, out)))
        return 0

    # untimed calls that let the shader clock reach its state under load.  The GPU's power management reacts to
    # every idle gap (a host synchronisation is one): some milliseconds at the boost clock, then a dip, settled
    # after 15 - 40 ms.  The calls are therefore enqueued in one go, with no synchronisation inside.
    settle_calls = 0
    if a.settle_ms > 0:
        for _ in range(16):                                # first calls: module load, allocator
            step(1 << 20)
        torch.cuda.synchronize()
        t_cal = time.perf_counter()
        for _ in range(16):
            step(1 << 20)
        torch.cuda.synchronize()
        per_call = (time.perf_counter() - t_cal) / 16
        settle_calls = int(min(max(a.settle_ms * 1e-3 / max(per_call, 1e-6), 1), 20000))
        for _ in range(settle_calls):
            step(1 << 20)
    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(a.warmup + i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / a.steps
    tau_mean = float(out[0].float().mean().item())

    # dominant kernel(s): HIP events recorded by the library on the launch stream, around the
    # vocabulary-streaming kernels only
    evs = []
    for i in range(a.steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); e1.record()                    # materialise the hipEvent_t handles
        evs.append((e0, e1))
    torch.cuda.synchronize()
    for _ in range(settle_calls):                   # the synchronisation above was an idle gap: settle again, and go
        step(1 << 20)                               # on to the bracketed calls without another one
    for i, (e0, e1) in enumerate(evs):
        step(a.warmup + a.steps + i, events=(e0.cuda_event, e1.cuda_event))
    torch.cuda.synchronize()
    series = [e0.elapsed_time(e1) for e0, e1 in evs]        # in call order: shows the clock settling, if it does
    main_ms = sorted(series)
    main_avg = sum(main_ms) / len(main_ms)
    main_bytes = w.row_pairs * w.V * 2 * w.elem_bytes       # every (target, draft) row pair once
    dedup = bool(a.shared_row0) and a.algo != "split" and w.L >= 2
    if dedup:                                               # rows 0 once per prefix instead of once per draft
        main_bytes = w.batch * (w.K * (w.L - 1) + 1) * w.V * 2 * w.elem_bytes
    achieved = main_bytes / (main_avg * 1e-3) / 1e9

    # HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE +
    # WRITE_SIZE, calibrated against a plain copy), if one exists for this workload and schedule
    ttag = a.workload + ("_shared_row0" if dedup else "")
    traffic = committed_traffic(ttag) if a.algo != "split" else None

    res = {
        "metric": "verifications/sec and achieved HBM GB/s (% of peak) at K=8, L=8, V=128256",
        "value": w.batch / (ms_per_step * 1e-3),
        "unit": "verifications/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: batch %d, K=%d, L=%d, V=%d, %s logits, T=%g" % (
                       w.name, w.batch, w.K, w.L, w.V, w.dtype, w.temperature),
                   "algo": a.algo, "shared_row0": bool(a.shared_row0), "row_pairs_per_s": w.row_pairs / (ms_per_step * 1e-3),
                   "whole_call_algorithmic_GBps": w.algorithmic_bytes / (ms_per_step * 1e-3) / 1e9,
                   "mean_accepted_len": tau_mean, "input_generation_s": round(gen_s, 1),
                   "settle": {"ms": a.settle_ms, "calls": settle_calls,
                              "note": "untimed calls enqueued in one go before the warm-up calls, and again before the event-bracketed calls of the roofline figure, so that the shader clock is in its state under load"}},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "the vocabulary-streaming kernel(s) that compute the statistics and the sums of Eq. (hik) "
                               "for every row: k_chain on the chain schedule (with k_row0_parts under --shared-row0), "
                               "k_row_stats + k_ot_sum (or their _parts variants) on the two-pass schedule; the chain "
                               "schedule's follow-up kernel for rows summed a second time (4 us when there is none) and "
                               "the final-token kernel are outside the event bracket and inside ms_per_step",
                     "kernel_ms_avg": main_avg, "kernel_ms_min": main_ms[0],
                     "kernel_ms_median": main_ms[len(main_ms) // 2],
                     "kernel_ms_first5": [round(v, 4) for v in series[:5]],
                     "kernel_ms_last5": [round(v, 4) for v in series[-5:]],
                     "kernel_calls_above_1.05x_min": sum(1 for v in series if v > 1.05 * main_ms[0]),
                     "kernel_calls": len(series),
                     "traffic_source": traffic_source(ttag) if traffic is not None else None,
                     # fetched + written bytes of the committed counter run over this run's kernel time
                     "traffic_GBps": (traffic / (main_avg * 1e-3) / 1e9) if traffic is not None else None,
                     "algorithmic_bytes_per_launch": main_bytes},
    }

    # The same kernel against the vector-ALU issue rate (it is limited by instruction issue, not by HBM, for
    # bfloat16 logits): lane-instructions the formulation needs per (target, draft) entry pair -- v_exp_f32
    # counts two issue slots -- over the 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz the chip issues without packed
    # float32 instructions.
    unpack = 2 if w.dtype == "bf16" else 0
    nmul = (w.K.bit_length() - 1) + bin(w.K).count("1") - 1
    pairs1 = w.batch * (w.K * (w.L - 1) + 1) if dedup else w.row_pairs      # row pairs that get statistics
    pairs2 = w.batch * w.K * (w.L - 1)                                      # row pairs that get an Eq. (hik) sum
    slots = ((unpack + 8) * pairs1 + (unpack + 9 + nmul) * pairs2) / pairs1
    alu_peak = 256 * 4 * 16 * 2.4e9 / 1e12
    alu_ach = slots * pairs1 * w.V / (main_avg * 1e-3) / 1e12
    res["roofline_alu"] = {"bound": "alu", "achieved": alu_ach, "peak": alu_peak, "unit": "Tlane-instr/s",
                           "frac": alu_ach / alu_peak, "slots_per_entry_pair": slots,
                           "note": "unpacked float32 issue rate; the published 157.3 TFLOP/s counts packed FMA"}

    if not a.no_cpu_baseline:
        import oracle
        # bounded sample: time two prefixes, then as many as fit the CPU-time target
        t0 = time.perf_counter()
        oracle.verify(target[:2], draft[:2], tokens[:2], w.temperature, a.seed, 0, nthreads=1)
        per = (time.perf_counter() - t0) / 2
        n = int(max(2, min(w.batch, a.cpu_seconds / max(per, 1e-9))))
        t0 = time.perf_counter()
        ref = oracle.verify(target[:n], draft[:n], tokens[:n], w.temperature, a.seed, a.warmup + a.steps - 1,
                            nthreads=1, debug=True)
        cpu_s = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": n / cpu_s, "unit": "verifications/s", "cores": 1, "kind": "oracle",
                               "sample": "first %d of %d prefixes of the same batch, float64, 1 thread, %.1f s" % (
                                   n, w.batch, cpu_s),
                               "host_cpus": os.cpu_count()}
        # the same oracle with one thread per host core (prefixes distributed over threads), whole batch
        nthr = min(os.cpu_count() or 1, oracle.num_procs(), w.batch)
        if nthr > 1:
            t0 = time.perf_counter()
            oracle.verify(target, draft, tokens, w.temperature, a.seed, 0, nthreads=nthr)
            res["cpu_baseline"]["all_cores"] = {"value": w.batch / (time.perf_counter() - t0), "cores": nthr,
                                                "sample": "all %d prefixes" % w.batch}
        # the last timed step used the same counters: report agreement on the sample
        step(a.warmup + a.steps - 1)
        torch.cuda.synchronize()
        got = out[0][:n].cpu().numpy()
        res["config"]["sample_accepted_len_agree"] = int((got == ref["accepted_len"]).sum())
        res["config"]["sample_size"] = n
        # the parity bar's counted events on the same sample: decisions and final tokens whose margin is below 1e-6
        # (they may differ), and the differences actually seen
        inter = sg.specgbv_read_intermediates(ws, w.batch, w.K, w.L, w.V, dt)
        g_f, g_tok = out[1][:n].cpu().numpy(), out[2][:n].cpu().numpy()
        tested = (ref["state"] == 1) | (inter["state"][:n] == 1)
        dist = np.minimum(np.abs(ref["eta"] - ref["h"]), np.abs(inter["eta"][:n] - inter["h"][:n]))
        low_dec = np.array([bool(np.any(dist[b][tested[b]] < 1e-6)) for b in range(n)])
        same_dec = (got == ref["accepted_len"]) & (g_f == ref["accepted_draft_idx"])
        low_tok = (ref["margin"] < 1e-6) | (inter["margin"][:n] < 1e-6)
        same_tok = np.array([np.array_equal(g_tok[b], ref["out_tokens"][b]) for b in range(n)])
        res["parity_sample"] = {
            "prefixes": n, "low_margin_decisions": int(low_dec.sum()), "decision_mismatches": int((~same_dec).sum()),
            "decision_mismatches_outside_margin": int((~same_dec & ~low_dec).sum()),
            "low_margin_tokens": int((same_dec & low_tok).sum()), "token_mismatches": int((same_dec & ~same_tok).sum()),
            "token_mismatches_outside_margin": int((same_dec & ~same_tok & ~low_tok).sum()),
            "max_h_error_over_bar": float((np.abs(inter["h"][:n] - ref["h"]) / (1e-5 * np.abs(ref["h"]) + 1e-9)).max()),
            "bar": "tau, f, tokens bit-exact unless a margin is below 1e-6; h within 1e-5 |h| + 1e-9"}
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
