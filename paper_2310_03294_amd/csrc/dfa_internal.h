// Internal declarations shared by the translation units of libdfa (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dfa.h"

namespace dfa {

// Launch wrappers: every one validates nothing (the ABI layer did) and returns a dfa_status.
int launch_merge(const dfa_merge_desc& md, void* o_a, float* lse_a, const void* o_b, const float* lse_b,
                 hipStream_t st);
int launch_delta(const dfa_shape& sh, const void* o, const void* dO, float* delta, hipStream_t st);
int launch_fill_zero_rows(float* p, int heads, int rows, int d, int64_t stride_h, int64_t stride_s,
                          hipStream_t st);
int launch_fill_empty_fwd(const dfa_shape& sh, void* o, float* lse, hipStream_t st);

// accumulate != 0: (o, lse) hold the state of earlier key/value chunks on entry and are updated in place
int launch_fwd_f32(const dfa_shape& sh, const float* q, const float* k, const float* v,
                   void* o, float* lse, int accumulate, hipStream_t st);
int launch_bwd_f32(const dfa_shape& sh, const float* q, const float* k, const float* v,
                   const float* lse, const float* delta, const float* dO,
                   float* dq, float* dk, float* dv, int accumulate, hipStream_t st);

int launch_fwd_bf16(const dfa_shape& sh, const void* q, const void* k, const void* v,
                    void* o, float* lse, int accumulate, hipStream_t st);
int launch_bwd_bf16(const dfa_shape& sh, const void* q, const void* k, const void* v,
                    const float* lse, const float* delta, const void* dO,
                    float* dq, float* dk, float* dv, int accumulate, hipStream_t st);

inline int hip_status(hipError_t e) { return e == hipSuccess ? DFA_OK : DFA_ERR_HIP; }
inline int last_launch_status() { return hip_status(hipGetLastError()); }

}  // namespace dfa
