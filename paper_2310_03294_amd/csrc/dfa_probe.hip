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

// The same stream fed with caller-supplied operand values: every wavefront loads eight A and eight B
// operands (16 bytes per lane each) from `ops` once and rotates through them, so that consecutive
// MFMAs see different operands, as they do in the attention kernels.  What the matrix pipes sustain
// depends on the operand VALUES: the device holds a power limit by lowering its clock, and operands
// with many toggling bits draw more power per MFMA than the near-constant ones of the plain probe.
__global__ void __launch_bounds__(PROBE_BLOCK, 2) k_mfma_probe_data(const uint4* __restrict__ ops, uint32_t mask,
                                                                    float* out, int iters) {
  const uint32_t t = blockIdx.x * PROBE_BLOCK + threadIdx.x;
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, ops[(t + i * 4099u) & mask]);
    b[i] = __builtin_bit_cast(bf16x8, ops[(t + i * 4099u + 31337u) & mask]);
  }
  f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; i += 4) {
      c0 = mfma32(a[i], b[i], c0);
      c1 = mfma32(a[i + 1], b[i + 1], c1);
      c2 = mfma32(a[i + 2], b[i + 2], c2);
      c3 = mfma32(a[i + 3], b[i + 3], c3);
    }
    if ((it & 255) == 255) {      // keep the accumulators in range, whatever the operands are
#pragma unroll
      for (int j = 0; j < 16; ++j) { c0[j] *= 0.001f; c1[j] *= 0.001f; c2[j] *= 0.001f; c3[j] *= 0.001f; }
    }
  }
  out[t] = c0[0] + c1[5] + c2[10] + c3[15];
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

extern "C" int dfa_mfma_probe_data(const void* operands, int64_t operand_bytes, float* out, int64_t n_out,
                                   int32_t iters, double* flop, void* stream) {
  using namespace dfa;
  if (out == nullptr || operands == nullptr) return DFA_ERR_NULL;
  if (iters < 1 || n_out < static_cast<int64_t>(PROBE_GRID) * PROBE_BLOCK) return DFA_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(operands) & 15u) != 0) return DFA_ERR_SHAPE;
  // the largest power of two of 16-byte pieces that fits, at least 64 K of them (1 MiB)
  int64_t pieces = 65536;
  if (operand_bytes < pieces * 16) return DFA_ERR_ARG;
  while (pieces * 2 * 16 <= operand_bytes && pieces < (int64_t{1} << 30)) pieces *= 2;
  hipStream_t st = static_cast<hipStream_t>(stream);
  k_mfma_probe_data<<<PROBE_GRID, PROBE_BLOCK, 0, st>>>(static_cast<const uint4*>(operands),
                                                        static_cast<uint32_t>(pieces - 1), out, iters);
  if (hipGetLastError() != hipSuccess) return DFA_ERR_HIP;
  if (flop != nullptr)
    *flop = 2.0 * 32 * 32 * 16 * 8.0 * iters * (PROBE_GRID * (PROBE_BLOCK / 64));   // 8 MFMAs per iteration and wavefront
  return DFA_OK;
}
