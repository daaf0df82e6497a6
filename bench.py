#!/usr/bin/env python3
"""Benchmark of the DistFlashAttn per-worker hot path on one MI355X.

One "step" = one pass of the whole hot path for the heaviest worker (worker P-1) of the
Llama-7B attention shape at N = 32768, P = 8 (chunk 4096, 32 heads x d128, bf16): the causal
diagonal chunk, its four OWN off-diagonal pairs (each continuing from the running (O, lse)
state: dfa_chunk_fwd_acc), the merges of the three partials that helpers send, the D pre-pass and
the backward of the same five pairs.
Inputs are resident in HBM before the timed region; the helpers' partials are produced
beforehand (they arrive over the network in the distributed setting).

Prints ONE JSON line: causal-adjusted TFLOP/s (14 d H nnz / t), the MFMA roofline of the
dominant kernel measured with HIP events inside the timed region, and the fp64 CPU oracle
timed on a bounded sample of the same workload.
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

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0
EVENT_EVERY = 4                 # timed steps between two steps instrumented with HIP events


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="index into dfa_inputs.CONFIGS (1 = the metric's workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap-copy", action="store_true",
                    help="stage the key/value chunk of each OWN forward pair one step ahead with a device-to-device "
                         "copy on a second stream (emulates the communication overlap; forward only)")
    ap.add_argument("--schedule", choices=("balanced", "ring"), default="balanced",
                    help="balanced: the load-balanced schedule (the metric's workload); ring: the plain ring "
                         "schedule, where worker P-1 computes all P of its pairs itself (ablation)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain elementwise kernel that reads 1 GiB and writes 1 GiB, "
                         "the known-size reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--cpu-heads", type=int, default=16, help="heads of the share the oracle is timed on")
    return ap.parse_args()


def share_pairs(sched):
    return [(s.q_chunk, s.kv_chunk, s.kind) for s in sched if s.kind != 0]


def traffic_from_profiles(name):
    """HBM bytes per launch of the dominant kernel, measured offline with rocprofv3 --pmc
    (FETCH_SIZE + WRITE_SIZE) and recorded in profiles/; None when not recorded."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


def cpu_baseline(w, worker, heads, q, k, v, do, mode="balanced"):
    """Times the fp64 oracle (as it stands) on `heads` heads of the worker's share: pair
    forward + pair backward of its five pairs.  Returns the cpu_baseline JSON object."""
    import numpy as np
    from oracle import attention as A
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    c = w.chunk
    kvh = max(1, heads // (w.h_q // w.h_kv))
    q64 = q[:heads].double().numpy(); do64 = do[:heads].double().numpy()
    k64 = k[:kvh].double().numpy(); v64 = v[:kvh].double().numpy()
    # global logsumexp and D of the worker's rows (untimed set-up: the backward's saved inputs)
    rows = slice(worker * c, (worker + 1) * c)
    O = np.empty((heads, c, w.d)); L = np.empty((heads, c))
    for h in range(heads):
        O[h], L[h] = A.rows_fwd(q64[h, rows], np.arange(worker * c, (worker + 1) * c), k64[h // (heads // kvh)],
                                v64[h // (heads // kvh)], w.scale)
    Lfull = np.zeros((heads, w.n_total)); Dfull = np.zeros((heads, w.n_total))
    Lfull[:, rows] = L; Dfull[:, rows] = A.delta_rows(O, do64[:, rows])
    import paper_2310_03294_amd as dfa
    pairs = share_pairs(dfa.dfa_schedule(w.p, worker, mode))
    t0 = time.perf_counter()
    for (qc, kc, _kind) in pairs:
        A.pair_fwd(q64, k64, v64, w.scale, qc, kc, c)
        A.pair_bwd(q64, k64, v64, do64, Lfull, Dfull, w.scale, qc, kc, c)
    dt = time.perf_counter() - t0
    nnz = sum(c * (c + 1) // 2 if qc == kc else c * c for qc, kc, _ in pairs)
    flops = 14.0 * w.d * heads * nnz
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{heads} of {w.h_q} heads of worker {worker}'s share ({len(pairs)} pairs fwd+bwd, fp64 numpy), "
                      f"{dt:.1f} s"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the P workers are virtual); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import dfa_inputs
    import paper_2310_03294_amd as dfa
    from paper_2310_03294_amd import driver, binding as B

    dfa.load_library()           # fails loudly if the HIP extension is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    w = dfa_inputs.CONFIGS[args.config]
    worker = w.p - 1
    c = w.chunk

    q, k, v, do = (dfa_inputs.full_sequence(w, t) for t in range(4))
    Q, K, V, dO = (t.to(dev) for t in (q, k, v, do))
    bufs = driver.Buffers(w.h_q, w.h_kv, w.n_total, w.d, w.p, dev)
    remote = driver.helper_partials_for(Q, K, V, w.scale, w.p, worker, bufs) if args.schedule == "balanced" else {}
    sched = dfa.dfa_schedule(w.p, worker, args.schedule)
    pairs = share_pairs(sched)
    nnz = sum(c * (c + 1) // 2 if qc == kc else c * c for qc, kc, _ in pairs)
    flops_step = 14.0 * w.d * w.h_q * nnz

    def chunk(t, i):
        return t[:, i * c:(i + 1) * c]

    # HIP events on the stream the kernels run on (torch's current stream; the binding passes
    # that stream to the library): one pair per backward kernel launch, one around the forward.
    ev = {"k_bwd_dkdv_bf16": [], "k_bwd_dq_bf16": [], "forward": []}

    def timed(name, record, flops, fn):
        if not record:
            fn()
            return
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record(); fn(); e1.record()
        ev[name].append((e0, e1, flops))

    fwd_flops = 4.0 * w.d * w.h_q * nnz
    prefetch = driver.KVPrefetcher(K, V, c) if args.overlap_copy else None

    def step(record):
        timed("forward", record, fwd_flops,
              lambda: driver.forward_worker(Q, K, V, w.scale, w.p, worker, bufs, remote=remote or None,
                                            mode=args.schedule, prefetch=prefetch))
        B.dfa_delta(chunk(bufs.O, worker), chunk(dO, worker), delta=chunk(bufs.delta, worker))
        seen_q, seen_kv = set(), set()     # first contribution to a gradient chunk overwrites, the rest accumulate
        for (qc, kc, kind) in pairs:
            n = c * (c + 1) // 2 if qc == kc else c * c
            common = (chunk(Q, qc), chunk(K, kc), chunk(V, kc), chunk(bufs.L, qc), chunk(bufs.delta, qc), chunk(dO, qc))
            diag = kind == B.DFA_STEP_DIAG
            acc_kv, acc_q = kc in seen_kv, qc in seen_q
            seen_kv.add(kc); seen_q.add(qc)
            # the two kernels of one dfa_chunk_bwd, launched through the same entry point one at a
            # time so that each gets its own event pair: S, dP, dV, dK = 8 d nnz; dQ (with S, dP
            # recomputed) = 2 d nnz algorithmic, 6 d nnz executed
            timed("k_bwd_dkdv_bf16", record, 8.0 * w.d * w.h_q * n,
                  lambda: B.dfa_chunk_bwd(*common, None, chunk(bufs.dK, kc), chunk(bufs.dV, kc), diag, w.scale,
                                          accumulate=acc_kv))
            timed("k_bwd_dq_bf16", record, 2.0 * w.d * w.h_q * n,
                  lambda: B.dfa_chunk_bwd(*common, chunk(bufs.dQ, qc), None, None, diag, w.scale, accumulate=acc_q))

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)     # one dispatch: 2^30 B read, 2^30 B written
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    # Event pairs serialise the stream around each timed launch (about 10 us per pair), so only
    # every EVENT_EVERY-th timed step carries them; the other steps run as a caller would run them.
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i % EVENT_EVERY == 0)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt * 1e3 / args.steps
    tflops = flops_step / (ms * 1e-3) / 1e12

    def summary(name):
        tot_ms = sum(a.elapsed_time(b) for a, b, _ in ev[name])
        tot_fl = sum(f for _, _, f in ev[name])
        return tot_ms, tot_fl, len(ev[name])

    kv_ms, kv_fl, kv_n = summary("k_bwd_dkdv_bf16")
    dq_ms, dq_fl, dq_n = summary("k_bwd_dq_bf16")
    fw_ms, fw_fl, fw_n = summary("forward")
    achieved = kv_fl / (kv_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "k_bwd_dkdv_bf16", "achieved": round(achieved, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "avg_launch_ms": round(kv_ms / kv_n, 4), "flop_per_launch": kv_fl / kv_n,
                "traffic": traffic_from_profiles("k_bwd_dkdv_bf16_cfg2_pmc.txt"),
                "share_of_step": round(kv_ms / (kv_n / len(pairs)) / ms, 3),
                "others": {
                    "k_bwd_dq_bf16": {"avg_launch_ms": round(dq_ms / dq_n, 4),
                                      "algorithmic_tflops": round(dq_fl / (dq_ms * 1e-3) / 1e12, 2),
                                      "executed_tflops": round(3.0 * dq_fl / (dq_ms * 1e-3) / 1e12, 2),
                                      "share_of_step": round(dq_ms / (dq_n / len(pairs)) / ms, 3)},
                    f"forward (k_fwd_bf16 x{len(pairs)} + k_merge x{len(remote)})": {"ms_per_step": round(fw_ms / fw_n, 4),
                                                            "tflops": round(fw_fl / (fw_ms * 1e-3) / 1e12, 2),
                                                            "share_of_step": round(fw_ms / fw_n / ms, 3)}}}

    # On-box ceiling of the matrix pipes (after the timed region): a register-resident MFMA stream
    # at the clock the device sustains under that load, next to the published peak.
    probe_out = torch.empty(512 * 256, dtype=torch.float32, device=dev)
    B.dfa_mfma_probe(probe_out, 2000)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    probe_flop = B.dfa_mfma_probe(probe_out, 20000)
    e1.record()
    torch.cuda.synchronize()
    ceiling = probe_flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    roofline["onbox_mfma_ceiling"] = round(ceiling, 1)
    roofline["frac_of_onbox_ceiling"] = round(achieved / ceiling, 4)

    out = {
        "metric": "causal-adjusted attention TFLOP/s fwd+bwd per worker share; % of bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: worker {worker} share ({args.schedule} schedule), {len(pairs)} pairs fwd+bwd + "
                               f"{len(remote)} remote merges, H={w.h_q}/{w.h_kv} d={w.d} C={c}",
                   "n_total": w.n_total, "P": w.p, "chunk": c},
        "pct_of_bf16_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "pct_of_onbox_mfma_ceiling": round(100.0 * tflops / ceiling, 2),
        "flop_per_step": flops_step,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, worker, args.cpu_heads, q, k, v, do, args.schedule)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
