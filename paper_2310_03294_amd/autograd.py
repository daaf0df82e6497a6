"""Causal attention over P virtual workers as a torch.autograd.Function, with the
rematerialization-aware placement of the gradient checkpoint (Section 3.3).

The forward runs the load-balanced schedule (Section 3.2) through the library and saves
(q, k, v, O, logsumexp); the backward needs nothing else (Appendix A): it never re-runs the
attention forward.  `CheckpointedBlock` shows the two checkpoint placements of Section 3.3 on a
block  y = f(attention(q, k, v))  whose activations are dropped in the forward pass:

  * placement "layer_boundary" (the usual one): the backward first recomputes the whole block,
    attention included, then back-propagates: attention costs 2 forwards + 1 backward;
  * placement "attention_output" (remat-aware): the attention output is the checkpoint; only f is
    recomputed, attention costs 1 forward + 1 backward.

Host-side sequencing only; every computation of the attention is a call into libdfa.so.
"""
from __future__ import annotations

import torch

from . import binding as B
from . import driver

# pairs computed by dfa_chunk_fwd / dfa_chunk_fwd_acc since the last reset (for tests and for
# showing what each checkpoint placement re-runs)
forward_pair_calls = 0
# When set, every backward leaves its gradients here as the library produced them (fp32 dq, dk, dv),
# before they are rounded to the dtype of the inputs they are handed to.
keep_fp32_grads = False
last_fp32_grads = None


def _forward(q, k, v, scale, P):
    """Runs the whole balanced schedule; returns the merged output and logsumexp, both fp32 (the
    state the schedule carries and the backward reuses; callers get the output in q's dtype)."""
    global forward_pair_calls
    h_q, n, d = q.shape
    bufs = driver.Buffers(h_q, k.shape[0], n, d, P, q.device, grads=False)
    driver.run_all_workers(q, k, v, None, scale, P, bufs, backward=False)
    forward_pair_calls += P * (P + 1) // 2
    return bufs.O, bufs.L


class DistFlashAttnFunction(torch.autograd.Function):
    """o = causal_attention(q, k, v) for [heads, N, d] bf16 / fp32 tensors, N divisible by P.
    o has q's dtype; what is saved for the backward is the fp32 output and its logsumexp."""

    @staticmethod
    def forward(ctx, q, k, v, scale, P):
        o, lse = _forward(q, k, v, scale, P)
        ctx.save_for_backward(q, k, v, o, lse)
        ctx.scale, ctx.P = scale, P
        return o.to(q.dtype)

    @staticmethod
    def backward(ctx, d_o):
        q, k, v, o, lse = ctx.saved_tensors
        return (*_backward(q, k, v, o, lse, d_o, ctx.scale, ctx.P), None, None)


def _backward(q, k, v, o, lse, d_o, scale, P):
    """Gradients from the saved (q, k, v, O, logsumexp) and dO, which is rounded to the dtype of q
    (the kernels read dO in the inputs' dtype).  The library's gradients are fp32; autograd hands a
    tensor gradients of its own dtype, so they are rounded to it on return."""
    global last_fp32_grads
    h_q, n, d = q.shape
    c = n // P
    d_o = d_o.to(q.dtype).contiguous()
    bufs = driver.Buffers(h_q, k.shape[0], n, d, P, q.device, grads=True, outputs=False)
    bufs.O, bufs.L = o, lse
    for w in range(P):
        B.dfa_delta(o[:, w * c:(w + 1) * c], d_o[:, w * c:(w + 1) * c], delta=bufs.delta[:, w * c:(w + 1) * c])
    touched = driver.new_pass()
    for w in range(P):
        driver.backward_worker(q, k, v, d_o, scale, P, w, bufs, with_delta=False, touched=touched)
    if keep_fp32_grads:
        last_fp32_grads = (bufs.dQ, bufs.dK, bufs.dV)
    return bufs.dQ.to(q.dtype), bufs.dK.to(k.dtype), bufs.dV.to(v.dtype)


def dist_flash_attn(q, k, v, scale, P):
    return DistFlashAttnFunction.apply(q, k, v, scale, P)


class _BlockFunction(torch.autograd.Function):
    """y = f(attention(q, k, v)) with the block's activations dropped in the forward pass."""

    @staticmethod
    def forward(ctx, q, k, v, scale, P, f, placement):
        o, lse = _forward(q, k, v, scale, P)
        with torch.no_grad():
            y = f(o.to(q.dtype))
        if placement == "attention_output":
            ctx.save_for_backward(q, k, v, o, lse)        # the checkpoint is the attention output
        else:
            ctx.save_for_backward(q, k, v)                 # the checkpoint is the block input
        ctx.scale, ctx.P, ctx.f, ctx.placement = scale, P, f, placement
        return y

    @staticmethod
    def backward(ctx, d_y):
        if ctx.placement == "attention_output":
            q, k, v, o, lse = ctx.saved_tensors
        else:
            q, k, v = ctx.saved_tensors
            o, lse = _forward(q, k, v, ctx.scale, ctx.P)   # recomputation re-runs the attention forward
        with torch.enable_grad():
            o_in = o.detach().to(q.dtype).requires_grad_(True)
            y = ctx.f(o_in)                                # recompute f only
        (d_o,) = torch.autograd.grad(y, o_in, d_y)
        return (*_backward(q, k, v, o, lse, d_o, ctx.scale, ctx.P), None, None, None, None)


class CheckpointedBlock(torch.nn.Module):
    """A checkpointed block around the attention; `placement` selects where the checkpoint sits."""

    def __init__(self, f, scale, P, placement="attention_output"):
        super().__init__()
        if placement not in ("attention_output", "layer_boundary"):
            raise ValueError(placement)
        self.f, self.scale, self.P, self.placement = f, scale, P, placement

    def forward(self, q, k, v):
        return _BlockFunction.apply(q, k, v, self.scale, self.P, self.f, self.placement)


def _main():
    """Times one forward + backward of the checkpointed block under both placements:
    python -m paper_2310_03294_amd.autograd [--config I] [--steps K]."""
    import argparse
    import json
    import time

    import dfa_inputs

    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    args = ap.parse_args()
    w = dfa_inputs.CONFIGS[args.config]
    dev = torch.device("cuda:0")
    q, k, v, d_y = (dfa_inputs.full_sequence(w, t).to(dev) for t in range(4))
    q.requires_grad_(True); k.requires_grad_(True); v.requires_grad_(True)
    out = {"workload": w.name, "P": w.p, "steps": args.steps}
    for placement in ("attention_output", "layer_boundary"):
        block = CheckpointedBlock(lambda o: o, w.scale, w.p, placement)
        for i in range(args.steps + 1):
            if i == 1:
                torch.cuda.synchronize(); t0 = time.perf_counter()
            q.grad = k.grad = v.grad = None
            block(q, k, v).backward(d_y)
        torch.cuda.synchronize()
        out[placement + "_ms"] = round((time.perf_counter() - t0) * 1e3 / args.steps, 3)
    out["ratio"] = round(out["layer_boundary_ms"] / out["attention_output_ms"], 3)
    print(json.dumps(out))


if __name__ == "__main__":
    _main()
