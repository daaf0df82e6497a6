// Measurement aid for the MFMA roofline: a register-resident stream of
// v_mfma_f32_32x32x16_bf16 on every SIMD of the device (2 wavefronts per SIMD, four independent
// accumulator tiles each, no memory traffic inside the loop).  Timed by the caller, it gives what
// the matrix pipes deliver at the clock the device sustains under this load, which sits below the
// published peak (that one assumes the maximum clock).
#include <hip/hip_runtime.h>
#include "dfa.h"
#include "dfa_mfma.h"

namespace dfa {
namespace {
constexpr int PROBE_GRID = 512;      // 2 workgroups of 4 wavefronts per CU on 256 CUs
constexpr int PROBE_BLOCK = 256;

__global__ void __launch_bounds__(PROBE_BLOCK, 2) k_mfma_probe(float* out, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = static_cast<__bf16>(1.0f / 1024.0f * static_cast<float>((lane + i) & 7));
    b[i] = static_cast<__bf16>(1.0f / 1024.0f * static_cast<float>((lane * 3 + i) & 7));
  }
  f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  for (int it = 0; it < iters; ++it) {
    c0 = mfma32(a, b, c0);
    c1 = mfma32(a, b, c1);
    c2 = mfma32(a, b, c2);
    c3 = mfma32(a, b, c3);
  }
  out[blockIdx.x * PROBE_BLOCK + threadIdx.x] = c0[0] + c1[5] + c2[10] + c3[15];
}
}  // namespace
}  // namespace dfa

extern "C" int dfa_mfma_probe(float* out, int64_t n_out, int32_t iters, double* flop, void* stream) {
  using namespace dfa;
  if (out == nullptr) return DFA_ERR_NULL;
  if (iters < 1 || n_out < static_cast<int64_t>(PROBE_GRID) * PROBE_BLOCK) return DFA_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  k_mfma_probe<<<PROBE_GRID, PROBE_BLOCK, 0, st>>>(out, iters);
  if (hipGetLastError() != hipSuccess) return DFA_ERR_HIP;
  if (flop != nullptr)
    *flop = 2.0 * 32 * 32 * 16 * 4.0 * iters * (PROBE_GRID * (PROBE_BLOCK / 64));   // 4 MFMAs per iteration and wavefront
  return DFA_OK;
}
