"""Seeded synthetic inputs shared by the tests, the bench and the smoke check.

This module only draws random numbers and describes workload shapes.  It holds
none of the attention arithmetic and is imported by both the CPU oracle's
callers and the HIP path's callers, so that the two sides see bit-identical
inputs without sharing any code of the method itself.

Recipe: every tensor is produced chunk by chunk (one chunk = the C = N/P tokens
one sequence-parallel worker owns, Section 3.1 of the DistFlashAttn paper).
A chunk of tensor `tensor_id` (0=Q, 1=K, 2=V, 3=dO) is
`torch.randn(heads, C, d, fp32)` from a CPU `torch.Generator` seeded with
`seed + 1000 * tensor_id + chunk_id`, then rounded to the workload dtype.  Any
chunk can therefore be regenerated on its own without holding the whole
sequence on the host.  The paper uses no dataset for this path (it times
training iterations on random-shaped Llama-7B attention), so i.i.d. N(0,1)
tensors of the Llama-7B attention shape are the workload itself.
"""
from __future__ import annotations

import dataclasses
import math

import torch

TENSOR_Q, TENSOR_K, TENSOR_V, TENSOR_DO = 0, 1, 2, 3


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark/parity configuration (shapes only)."""

    name: str
    h_q: int
    h_kv: int
    d: int
    n_total: int      # N, tokens in the whole sequence
    p: int            # P, number of (virtual) workers
    dtype: str        # "f32" or "bf16"
    seed: int

    @property
    def chunk(self) -> int:
        return self.n_total // self.p

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


# The five configurations the build is measured on (index = config number).
CONFIGS = (
    Workload("cfg1_f32_h1_d64_n1k_p4", 1, 1, 64, 1024, 4, "f32", 1234),
    Workload("cfg2_llama7b_n32k_p8", 32, 32, 128, 32768, 8, "bf16", 1235),
    Workload("cfg3_llama7b_n128k_p8", 32, 32, 128, 131072, 8, "bf16", 1236),
    Workload("cfg4_llama7b_n512k_p8", 32, 32, 128, 524288, 8, "bf16", 1237),
    Workload("cfg5_gqa_n256k_p16", 32, 8, 128, 262144, 16, "bf16", 1238),
)


def chunk_tensor(seed: int, tensor_id: int, chunk_id: int, heads: int, c: int,
                 d: int, dtype: torch.dtype) -> torch.Tensor:
    """Chunk `chunk_id` of tensor `tensor_id`: [heads, c, d], values N(0,1) rounded to dtype."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed) + 1000 * int(tensor_id) + int(chunk_id))
    x = torch.randn((heads, c, d), generator=g, dtype=torch.float32)
    return x.to(dtype)


def workload_chunk(w: Workload, tensor_id: int, chunk_id: int) -> torch.Tensor:
    heads = w.h_q if tensor_id in (TENSOR_Q, TENSOR_DO) else w.h_kv
    return chunk_tensor(w.seed, tensor_id, chunk_id, heads, w.chunk, w.d, w.torch_dtype)


def full_sequence(w: Workload, tensor_id: int) -> torch.Tensor:
    """All P chunks of a tensor concatenated along the sequence axis: [heads, N, d]."""
    return torch.cat([workload_chunk(w, tensor_id, c) for c in range(w.p)], dim=1)


def small_case(seed: int, h_q: int, h_kv: int, n: int, d: int,
               dtype: torch.dtype = torch.float32):
    """Q, K, V, dO for an ad-hoc small problem (single chunk id 0 per tensor)."""
    q = chunk_tensor(seed, TENSOR_Q, 0, h_q, n, d, dtype)
    k = chunk_tensor(seed, TENSOR_K, 0, h_kv, n, d, dtype)
    v = chunk_tensor(seed, TENSOR_V, 0, h_kv, n, d, dtype)
    do = chunk_tensor(seed, TENSOR_DO, 0, h_q, n, d, dtype)
    return q, k, v, do
