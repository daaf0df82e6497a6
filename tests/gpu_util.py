"""Helpers for the GPU parity tests (no attention arithmetic here)."""
import numpy as np
import torch

import dfa_inputs

TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}   # max abs error vs the fp64 oracle


def dev():
    return torch.device("cuda:0")


def np64(t):
    return t.detach().to("cpu", torch.float64).numpy()


def maxerr(got, want):
    g = np64(got) if isinstance(got, torch.Tensor) else np.asarray(got, np.float64)
    return float(np.abs(g - want).max()) if g.size else 0.0


def case(seed, h_q, h_kv, s_q, s_k, d, dtype):
    """q, dO: [h_q, s_q, d]; k, v: [h_kv, s_k, d] on the CPU in `dtype`."""
    q = dfa_inputs.chunk_tensor(seed, dfa_inputs.TENSOR_Q, 0, h_q, s_q, d, dtype)
    k = dfa_inputs.chunk_tensor(seed, dfa_inputs.TENSOR_K, 0, h_kv, s_k, d, dtype)
    v = dfa_inputs.chunk_tensor(seed, dfa_inputs.TENSOR_V, 0, h_kv, s_k, d, dtype)
    do = dfa_inputs.chunk_tensor(seed, dfa_inputs.TENSOR_DO, 0, h_q, s_q, d, dtype)
    return q, k, v, do
