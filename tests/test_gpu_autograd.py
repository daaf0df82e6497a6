"""The autograd wrapper and the two checkpoint placements of Section 3.3 (GPU, through the C ABI)."""
import math

import numpy as np
import pytest
import torch

import dfa_inputs
from gpu_util import dev, maxerr, np64
from oracle import attention as A

pytestmark = pytest.mark.gpu


def _f(o):                      # the rest of the block: any differentiable function of the attention output
    return torch.tanh(o) * 0.5 + o


def _oracle(q, k, v, d_y, scale):
    q64, k64, v64 = np64(q), np64(k), np64(v)
    O, _ = A.attention_fwd(q64, k64, v64, scale)
    o_t = torch.tensor(O, dtype=torch.float64, requires_grad=True)
    y = _f(o_t)
    (d_o,) = torch.autograd.grad(y, o_t, torch.tensor(np64(d_y)))
    dq, dk, dv = A.attention_bwd(q64, k64, v64, d_o.numpy(), scale)
    return y.detach().numpy(), dq, dk, dv


@pytest.mark.parametrize("dtype,d,tol", [(torch.float32, 64, 2e-5), (torch.bfloat16, 128, 6e-2)])
@pytest.mark.parametrize("placement", ["attention_output", "layer_boundary"])
def test_checkpointed_block(dtype, d, tol, placement):
    from paper_2310_03294_amd import autograd as AG
    w = dfa_inputs.Workload("t_autograd", 4, 2, d, 512, 4, "f32" if dtype == torch.float32 else "bf16", 99)
    q, k, v, d_y = (dfa_inputs.full_sequence(w, t) for t in range(4))
    Q, K, V = (t.to(dev()).requires_grad_(True) for t in (q, k, v))
    block = AG.CheckpointedBlock(_f, w.scale, w.p, placement)
    AG.forward_pair_calls = 0
    y = block(Q, K, V)
    pairs = w.p * (w.p + 1) // 2
    assert AG.forward_pair_calls == pairs
    y.backward(d_y.to(dev()).to(y.dtype))
    torch.cuda.synchronize()
    # the remat-aware placement re-runs no attention forward; the usual one re-runs all of it
    assert AG.forward_pair_calls == (pairs if placement == "attention_output" else 2 * pairs)
    ry, rq, rk, rv = _oracle(q, k, v, d_y, w.scale)
    errs = dict(y=maxerr(y, ry), dq=maxerr(Q.grad, rq), dk=maxerr(K.grad, rk), dv=maxerr(V.grad, rv))
    assert all(e <= tol for e in errs.values()), errs


def test_function_matches_oracle_fp32():
    from paper_2310_03294_amd import autograd as AG
    w = dfa_inputs.CONFIGS[0]
    q, k, v, d_o = (dfa_inputs.full_sequence(w, t) for t in range(4))
    Q, K, V = (t.to(dev()).requires_grad_(True) for t in (q, k, v))
    o = AG.dist_flash_attn(Q, K, V, w.scale, w.p)
    o.backward(d_o.to(dev()))
    torch.cuda.synchronize()
    O, _ = A.attention_fwd(np64(q), np64(k), np64(v), w.scale)
    dq, dk, dv = A.attention_bwd(np64(q), np64(k), np64(v), np64(d_o), w.scale)
    assert maxerr(o, O) <= 1e-5 and maxerr(Q.grad, dq) <= 1e-5 and maxerr(K.grad, dk) <= 1e-5 and maxerr(V.grad, dv) <= 1e-5
