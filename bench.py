#!/usr/bin/env python3
"""Benchmark of the DistFlashAttn per-worker hot path on one MI355X.

One "step" = one pass of the whole hot path for the heaviest worker (worker P-1) of a Llama-7B
attention configuration (32 heads x d128, bf16, P = 8): the causal diagonal chunk, its four OWN
off-diagonal pairs (each continuing from the running (O, lse) state: dfa_chunk_fwd_acc), the
merges of the three partials that helpers send, the D pre-pass and the backward of the same five
pairs.  The headline workload is the largest single-GPU worker share, N = 524288 (chunk 65536);
the shares at N = 131072 and N = 32768 are timed in the same run and reported under "per_config".
Inputs are resident in HBM before the timed region; the helpers' partials are produced
beforehand (they arrive over the network in the distributed setting).  Only the chunks the share
touches are generated (the recipe of dfa_inputs, chunk by chunk).

Prints ONE JSON line: causal-adjusted TFLOP/s (14 d H nnz / t), the MFMA roofline of the
dominant kernel measured with HIP events inside the timed region, and the fp64 CPU oracle
timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0
HEADLINE_CONFIG = 3             # index into dfa_inputs.CONFIGS: N = 524288, P = 8, chunk 65536
ALSO_TIMED = (1, 2)             # the smaller worker-share configurations, reported under per_config
CPU_SAMPLE_SCORES = 6.0e8       # scores of the slab the oracle is timed on (about 10-20 s of fp64 numpy)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=HEADLINE_CONFIG,
                    help="index into dfa_inputs.CONFIGS (3 = the largest single-GPU worker share, the default)")
    ap.add_argument("--no-per-config", action="store_true", help="skip the smaller worker-share configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap-copy", action="store_true",
                    help="stage the key/value chunk of each OWN forward pair one step ahead with a device-to-device "
                         "copy on a second stream (emulates the communication overlap; forward only)")
    ap.add_argument("--schedule", choices=("balanced", "ring"), default="balanced",
                    help="balanced: the load-balanced schedule (the metric's workload); ring: the plain ring "
                         "schedule, where worker P-1 computes all P of its pairs itself (ablation)")
    ap.add_argument("--zero-operand-steps", type=int, default=3,
                    help="after the timed region, time this many steps of the same share on all-zero operands "
                         "(evidence of the power limit; 0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain elementwise kernel that reads 1 GiB and writes 1 GiB, "
                         "the known-size reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    return ap.parse_args()


def share_pairs(sched):
    return [(s.q_chunk, s.kv_chunk, s.kind) for s in sched if s.kind != 0]


def traffic_from_profiles(kernel, cfg_index):
    """HBM bytes per launch of a kernel at THIS configuration, measured offline with rocprofv3 --pmc
    (FETCH_SIZE + WRITE_SIZE) and recorded in profiles/; None when no profile of it is recorded."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_cfg{cfg_index + 1}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


class Share:
    """Device tensors of one worker's share: full-sequence views of which only the chunks the share
    touches are filled (Q, dO: the worker's chunk; K, V: every chunk, the earliest ones only feed
    the helpers' partials).  keep_head: fp64 host copies of that head, for the CPU baseline."""

    def __init__(self, w, worker, dev, keep_head=None):
        import numpy as np
        import torch
        import dfa_inputs
        c, n = w.chunk, w.n_total
        self.Q = torch.empty((w.h_q, n, w.d), dtype=torch.bfloat16, device=dev)
        self.dO = torch.empty_like(self.Q)
        self.K = torch.empty((w.h_kv, n, w.d), dtype=torch.bfloat16, device=dev)
        self.V = torch.empty_like(self.K)
        self.host = {}
        g = w.h_q // w.h_kv
        for tid, dst, chunks in ((dfa_inputs.TENSOR_Q, self.Q, [worker]), (dfa_inputs.TENSOR_DO, self.dO, [worker]),
                                 (dfa_inputs.TENSOR_K, self.K, range(w.p)), (dfa_inputs.TENSOR_V, self.V, range(w.p))):
            for ci in chunks:
                t = dfa_inputs.workload_chunk(w, tid, ci)
                dst[:, ci * c:(ci + 1) * c] = t.to(dev)
                if keep_head is not None:
                    h = keep_head if tid in (dfa_inputs.TENSOR_Q, dfa_inputs.TENSOR_DO) else keep_head // g
                    self.host[(tid, ci)] = t[h].to(torch.float64).numpy()
                del t


def cpu_baseline(w, worker, share, mode):
    """Times the fp64 oracle (as it stands) on a slab of the worker's share: the last R query rows
    of one head against the share's whole key range - forward partial (rows_fwd), dq (rows_dq) and
    dk, dv (cols_dkdv) of that slab.  Returns the cpu_baseline JSON object."""
    import numpy as np
    import dfa_inputs
    from oracle import attention as A
    from oracle import schedule as S
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    c, n = w.chunk, w.n_total
    sched = (S.balanced(w.p) if mode == "balanced" else S.ring(w.p))[worker]
    kv_chunks = sorted(s["kv_chunk"] for s in sched if s["kind"] != S.IDLE)
    lo = kv_chunks[0] * c                       # the share's keys are the contiguous range [lo, n)
    assert kv_chunks == list(range(kv_chunks[0], worker + 1))
    R = int(min(c, max(64, CPU_SAMPLE_SCORES // (n - lo) // 64 * 64)))
    rows = np.arange(n - R, n)
    q = share.host[(dfa_inputs.TENSOR_Q, worker)][c - R:]
    do = share.host[(dfa_inputs.TENSOR_DO, worker)][c - R:]
    k = np.concatenate([share.host[(dfa_inputs.TENSOR_K, i)] for i in range(w.p)])
    v = np.concatenate([share.host[(dfa_inputs.TENSOR_V, i)] for i in range(w.p)])
    # untimed set-up: the rows' global logsumexp and D (the backward's saved inputs)
    o_r = np.empty((R, w.d)); l_r = np.empty(R)
    for r0 in range(0, R, 256):            # in row blocks, to bound the fp64 temporaries
        o_r[r0:r0 + 256], l_r[r0:r0 + 256] = A.rows_fwd(q[r0:r0 + 256], rows[r0:r0 + 256], k, v, w.scale)
    d_r = A.delta_rows(o_r, do)
    cols = np.arange(lo, n)
    t0 = time.perf_counter()
    A.rows_fwd(q, rows, k[lo:], v[lo:], w.scale, col_lo=lo)
    A.rows_dq(q, rows, do, l_r, d_r, k[lo:], v[lo:], w.scale, col_lo=lo)
    A.cols_dkdv(k[lo:], v[lo:], cols, q, do, l_r, d_r, w.scale, row_lo=n - R)
    dt = time.perf_counter() - t0
    nnz = int(sum(int(i) - lo + 1 for i in rows))
    flops = 14.0 * w.d * nnz
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 of {w.h_q} heads, the last {R} query rows of worker {worker}'s chunk against the share's "
                      f"{n - lo} keys ({nnz} unmasked scores): rows_fwd + rows_dq + cols_dkdv, fp64 numpy, {dt:.1f} s"}


def run_share(w, cfg_index, args, steps, warmup, dev, keep_head=None, zero_steps=0):
    """Times `steps` passes of worker P-1's share of workload w.  Returns (result dict, Share).
    zero_steps > 0: afterwards the inputs are zeroed and that many more steps are timed (the Share's
    device tensors are then no longer the workload)."""
    import torch
    import paper_2310_03294_amd as dfa
    from paper_2310_03294_amd import driver, binding as B

    worker = w.p - 1
    c = w.chunk
    share = Share(w, worker, dev, keep_head)
    Q, K, V, dO = share.Q, share.K, share.V, share.dO
    bufs = driver.Buffers(w.h_q, w.h_kv, w.n_total, w.d, w.p, dev)
    remote = driver.helper_partials_for(Q, K, V, w.scale, w.p, worker, bufs) if args.schedule == "balanced" else {}
    sched = dfa.dfa_schedule(w.p, worker, args.schedule)
    pairs = share_pairs(sched)
    nnz = sum(c * (c + 1) // 2 if qc == kc else c * c for qc, kc, _ in pairs)
    flops_step = 14.0 * w.d * w.h_q * nnz
    fwd_flops = 4.0 * w.d * w.h_q * nnz
    # event pairs serialise the stream around a launch (about 10 us per pair): every launch carries
    # them when launches take milliseconds, every 4th step otherwise
    event_every = 1 if c >= 16384 else 4

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

    prefetch = driver.KVPrefetcher(K, V, c) if args.overlap_copy else None
    kv_bytes = []     # algorithmic HBM bytes of every dk/dv launch of a step

    def step(record):
        timed("forward", record, fwd_flops,
              lambda: driver.forward_worker(Q, K, V, w.scale, w.p, worker, bufs, remote=remote or None,
                                            mode=args.schedule, prefetch=prefetch))
        B.dfa_delta(chunk(bufs.O, worker), chunk(dO, worker), delta=chunk(bufs.delta, worker))
        seen_q, seen_kv = set(), set()     # first contribution to a gradient chunk overwrites, the rest accumulate
        kv_bytes.clear()
        for (qc, kc, kind) in pairs:
            n = c * (c + 1) // 2 if qc == kc else c * c
            common = (chunk(Q, qc), chunk(K, kc), chunk(V, kc), chunk(bufs.L, qc), chunk(bufs.delta, qc), chunk(dO, qc))
            diag = kind == B.DFA_STEP_DIAG
            acc_kv, acc_q = kc in seen_kv, qc in seen_q
            seen_kv.add(kc); seen_q.add(qc)
            # q, dO, k, v (bf16) and lse, D (fp32) read once, dk, dv (fp32) written once (and read when accumulating)
            kv_bytes.append(c * w.d * 2 * (2 * w.h_q + 2 * w.h_kv) + 2 * w.h_q * c * 4
                            + 2 * w.h_kv * c * w.d * 4 * (2 if acc_kv else 1))
            # the two kernels of one dfa_chunk_bwd, launched through the same entry point one at a
            # time so that each gets its own event pair: S, dP, dV, dK = 8 d nnz; dQ (with S, dP
            # recomputed) = 2 d nnz algorithmic, 6 d nnz executed
            timed("k_bwd_dkdv_bf16", record, 8.0 * w.d * w.h_q * n,
                  lambda: B.dfa_chunk_bwd(*common, None, chunk(bufs.dK, kc), chunk(bufs.dV, kc), diag, w.scale,
                                          accumulate=acc_kv))
            timed("k_bwd_dq_bf16", record, 2.0 * w.d * w.h_q * n,
                  lambda: B.dfa_chunk_bwd(*common, chunk(bufs.dQ, qc), None, None, diag, w.scale, accumulate=acc_q))

    for _ in range(warmup):
        step(False)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        step(i % event_every == 0)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt * 1e3 / steps
    per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
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
                "traffic": traffic_from_profiles("k_bwd_dkdv_bf16", cfg_index),
                "algorithmic_bytes_per_launch": sum(kv_bytes) / len(kv_bytes),
                "share_of_step": round(kv_ms / (kv_n / len(pairs)) / ms, 3),
                "others": {
                    "k_bwd_dq_bf16": {"avg_launch_ms": round(dq_ms / dq_n, 4),
                                      "algorithmic_tflops": round(dq_fl / (dq_ms * 1e-3) / 1e12, 2),
                                      "executed_tflops": round(3.0 * dq_fl / (dq_ms * 1e-3) / 1e12, 2),
                                      "share_of_step": round(dq_ms / (dq_n / len(pairs)) / ms, 3)},
                    f"forward (k_fwd_bf16 x{len(pairs)} + k_merge x{len(remote)})": {
                        "ms_per_step": round(fw_ms / fw_n, 4), "tflops": round(fw_fl / (fw_ms * 1e-3) / 1e12, 2),
                        "share_of_step": round(fw_ms / fw_n / ms, 3)}}}
    zero_ops = None
    if zero_steps > 0:
        # The same launches on all-zero operands (wrong for the method, same instruction streams):
        # what these kernels do when operand values cost no power.  After the timed region.
        for t in (Q, K, V, dO):
            t.zero_()
        step(False)
        torch.cuda.synchronize()
        z0 = time.perf_counter()
        for _ in range(zero_steps):
            step(False)
        torch.cuda.synchronize()
        zms = (time.perf_counter() - z0) * 1e3 / zero_steps
        zero_ops = {"value": round(flops_step / (zms * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "ms_per_step": round(zms, 4),
                    "steps": zero_steps,
                    "note": "same share, same launches, every operand zero: the device holds its power limit by "
                            "lowering the clock, and N(0,1) operands draw far more power per MFMA than zeros"}
    res = {"value": round(tflops, 2), "ms_per_step": round(ms, 4),
           "ms_per_step_median": round(statistics.median(per_step), 4), "ms_per_step_min": round(min(per_step), 4),
           "steps": steps, "warmup": warmup, "flop_per_step": flops_step,
           "pct_of_bf16_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
           "workload": f"{w.name}: worker {worker} share ({args.schedule} schedule), {len(pairs)} pairs fwd+bwd + "
                       f"{len(remote)} remote merges, H={w.h_q}/{w.h_kv} d={w.d} C={c}",
           "roofline": roofline}
    if zero_ops is not None:
        res["zero_operands"] = zero_ops
    del bufs, remote, prefetch
    return res, share


def mfma_ceiling(dev):
    """On-box ceilings of the matrix pipes: register-resident MFMA streams at the clock the device
    sustains under them.  (a) near-constant operands, a few milliseconds: what the pipes do when power
    is no limit; (b) i.i.d. N(0, 1) bf16 operands (the workload's values), rotating, > 100 ms: the
    device holds its power limit by lowering the clock, and operands with many toggling bits draw
    more power per MFMA, so this is the rate an attention kernel on this data could at best reach
    with every operand already in registers.  Median, min and max of several launches each."""
    import torch
    from paper_2310_03294_amd import binding as B
    out = torch.empty(512 * 256, dtype=torch.float32, device=dev)

    def rate(launch, reps):
        launch(True)
        vals = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flop = launch(False)
            e1.record()
            torch.cuda.synchronize()
            vals.append(flop / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        return statistics.median(vals), min(vals), max(vals)

    plain = rate(lambda warm: B.dfa_mfma_probe(out, 4000 if warm else 20000), 7)
    ops = torch.randn(1 << 22, generator=torch.Generator(device="cpu").manual_seed(4321)).to(torch.bfloat16).to(dev)
    data = rate(lambda warm: B.dfa_mfma_probe_data(ops, out, 20000 if warm else 400000), 3)
    return plain, data


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the P workers are virtual); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import dfa_inputs
    import paper_2310_03294_amd as dfa

    dfa.load_library()           # fails loudly if the HIP extension is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    w = dfa_inputs.CONFIGS[args.config]
    if w.dtype != "bf16":
        print("bench.py times the bf16 worker-share configurations (indices 1-4)", file=sys.stderr)
        sys.exit(2)

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)     # one dispatch: 2^30 B read, 2^30 B written
        torch.cuda.synchronize()
        del src, dst

    keep = None if args.no_cpu_baseline else 0
    res, share = run_share(w, args.config, args, args.steps, args.warmup, dev, keep_head=keep,
                           zero_steps=args.zero_operand_steps)
    roofline = res.pop("roofline")
    (ceiling, c_min, c_max), (ceil_data, d_min, d_max) = mfma_ceiling(dev)
    roofline["onbox_mfma_ceiling"] = round(ceiling, 1)
    roofline["onbox_mfma_ceiling_range"] = [round(c_min, 1), round(c_max, 1)]
    roofline["frac_of_onbox_ceiling"] = round(roofline["achieved"] / ceiling, 4)
    roofline["onbox_mfma_ceiling_n01_operands"] = round(ceil_data, 1)
    roofline["onbox_mfma_ceiling_n01_operands_range"] = [round(d_min, 1), round(d_max, 1)]
    roofline["frac_of_onbox_ceiling_n01_operands"] = round(roofline["achieved"] / ceil_data, 4)

    out = {
        "metric": "causal-adjusted attention TFLOP/s fwd+bwd per worker share; % of bf16 MFMA peak",
        "value": res["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "ms_per_step_median": res["ms_per_step_median"],
        "ms_per_step_min": res["ms_per_step_min"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": res["workload"], "n_total": w.n_total, "P": w.p, "chunk": w.chunk},
        "pct_of_bf16_peak": res["pct_of_bf16_peak"],
        "pct_of_onbox_mfma_ceiling": round(100.0 * res["value"] / ceiling, 2),
        "pct_of_onbox_mfma_ceiling_n01_operands": round(100.0 * res["value"] / ceil_data, 2),
        "flop_per_step": res["flop_per_step"],
        "roofline": roofline,
    }
    if "zero_operands" in res:
        out["zero_operands"] = res["zero_operands"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, w.p - 1, share, args.schedule)
    del share
    torch.cuda.empty_cache()
    if not args.no_per_config and args.config == HEADLINE_CONFIG:
        per = {}
        for ci in ALSO_TIMED:
            wc = dfa_inputs.CONFIGS[ci]
            r, s = run_share(wc, ci, args, 20, 5, dev)
            del s
            torch.cuda.empty_cache()
            rf = r.pop("roofline")
            r["k_bwd_dkdv_bf16_frac_of_peak"] = rf["frac"]
            r["k_bwd_dq_bf16_executed_tflops"] = rf["others"]["k_bwd_dq_bf16"]["executed_tflops"]
            r["forward_tflops"] = [v for k_, v in rf["others"].items() if k_.startswith("forward")][0]["tflops"]
            per[wc.name] = r
        out["per_config"] = per
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
