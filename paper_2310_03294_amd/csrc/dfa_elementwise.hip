// HBM-bound row kernels: the merge (rescale) of two partial results, the D = rowsum(dO o O)
// pre-pass of the backward, and small fill kernels.  One query row is d values wide; a row is
// handled by d/8 adjacent lanes, each moving 8 elements (16 B of bf16 or 2 x 16 B of fp32), so
// every global access of a wavefront is a run of full cache lines.
#include "dfa_internal.h"

namespace dfa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct Vec8 { float v[8]; };

template <bool BF16>
__device__ inline Vec8 load8(const void* base, int64_t elem_off) {
  Vec8 r;
  if constexpr (BF16) {
    const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const __bf16*>(base) + elem_off);
    bf16x8 b = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
    for (int i = 0; i < 8; ++i) r.v[i] = static_cast<float>(b[i]);
  } else {
    const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem_off);
    const float4 a = p[0], b = p[1];
    r.v[0] = a.x; r.v[1] = a.y; r.v[2] = a.z; r.v[3] = a.w;
    r.v[4] = b.x; r.v[5] = b.y; r.v[6] = b.z; r.v[7] = b.w;
  }
  return r;
}

template <bool BF16>
__device__ inline void store8(void* base, int64_t elem_off, const Vec8& r) {
  if constexpr (BF16) {
    bf16x8 b;
#pragma unroll
    for (int i = 0; i < 8; ++i) b[i] = static_cast<__bf16>(r.v[i]);
    *reinterpret_cast<uint4*>(static_cast<__bf16*>(base) + elem_off) = __builtin_bit_cast(uint4, b);
  } else {
    float4* p = reinterpret_cast<float4*>(static_cast<float*>(base) + elem_off);
    p[0] = make_float4(r.v[0], r.v[1], r.v[2], r.v[3]);
    p[1] = make_float4(r.v[4], r.v[5], r.v[6], r.v[7]);
  }
}

// (o_a, lse_a) <- merge((o_a, lse_a), (o_b, lse_b)), Section 3.2 rescale(.)
template <int D, bool BF16>
__global__ void __launch_bounds__(256) k_merge(dfa_merge_desc md, void* __restrict__ o_a, float* __restrict__ lse_a,
                                               const void* __restrict__ o_b, const float* __restrict__ lse_b) {
  constexpr int LPR = D / 8;           // lanes per row
  constexpr int RPB = 256 / LPR;       // rows per block iteration
  const int lane = threadIdx.x % LPR;
  const int rib = threadIdx.x / LPR;
  const int h = blockIdx.y;
  float* la_p = lse_a + h * md.lse_a_stride_h;
  const float* lb_p = lse_b + h * md.lse_b_stride_h;
  for (int row = blockIdx.x * RPB + rib; row < md.rows; row += gridDim.x * RPB) {
    const float la = la_p[row], lb = lb_p[row];
    const float m = fmaxf(la, lb);
    float wa = 0.f, wb = 0.f, l = -INFINITY;
    if (m > -INFINITY) {
      const float ea = expf(la - m), eb = expf(lb - m);   // one of them is exactly 1
      const float s = ea + eb;
      l = m + logf(s);
      const float inv = 1.f / s;
      wa = ea * inv; wb = eb * inv;
    }
    const int64_t offa = h * md.a_stride_h + static_cast<int64_t>(row) * md.a_stride_s + lane * 8;
    const int64_t offb = h * md.b_stride_h + static_cast<int64_t>(row) * md.b_stride_s + lane * 8;
    const Vec8 a = load8<BF16>(o_a, offa);
    const Vec8 b = load8<BF16>(o_b, offb);
    Vec8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r.v[i] = wa * a.v[i] + wb * b.v[i];
    store8<BF16>(o_a, offa, r);
    if (lane == 0) la_p[row] = l;
  }
}

// D_i = sum_c dO_ic * O_ic  (Section 3.3: the saved output feeds the backward)
template <int D, bool DO_BF16, bool O_BF16>
__global__ void __launch_bounds__(256) k_delta(int s_q, const void* __restrict__ o, int64_t o_sh, int64_t o_ss,
                                               const void* __restrict__ dO, int64_t q_sh, int64_t q_ss,
                                               float* __restrict__ delta, int64_t l_sh) {
  constexpr int LPR = D / 8;
  constexpr int RPB = 256 / LPR;
  const int lane = threadIdx.x % LPR;
  const int h = blockIdx.y;
  const int row = blockIdx.x * RPB + threadIdx.x / LPR;
  float acc = 0.f;
  if (row < s_q) {
    const Vec8 a = load8<O_BF16>(o, h * o_sh + static_cast<int64_t>(row) * o_ss + lane * 8);
    const Vec8 b = load8<DO_BF16>(dO, h * q_sh + static_cast<int64_t>(row) * q_ss + lane * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc = fmaf(a.v[i], b.v[i], acc);
  }
#pragma unroll
  for (int off = LPR / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
  if (row < s_q && lane == 0) delta[h * l_sh + row] = acc;
}

__global__ void __launch_bounds__(256) k_zero_rows(float* __restrict__ p, int rows, int d4, int64_t sh, int64_t ss) {
  const int h = blockIdx.y;
  const int per_row = d4;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < static_cast<int64_t>(rows) * per_row;
       i += static_cast<int64_t>(gridDim.x) * 256) {
    const int64_t r = i / per_row; const int c = static_cast<int>(i % per_row);
    reinterpret_cast<float4*>(p + h * sh + r * ss)[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
}

template <bool BF16>
__global__ void __launch_bounds__(256) k_empty_fwd(int s_q, int d8, void* __restrict__ o, int64_t o_sh, int64_t o_ss,
                                                   float* __restrict__ lse, int64_t l_sh) {
  const int h = blockIdx.y;
  Vec8 z; for (int i = 0; i < 8; ++i) z.v[i] = 0.f;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < static_cast<int64_t>(s_q) * d8;
       i += static_cast<int64_t>(gridDim.x) * 256) {
    const int64_t r = i / d8; const int c = static_cast<int>(i % d8);
    store8<BF16>(o, h * o_sh + r * o_ss + c * 8, z);
    if (c == 0) lse[h * l_sh + r] = -INFINITY;
  }
}

int grid_for(int64_t items, int per_block) {
  int64_t g = (items + per_block - 1) / per_block;
  const int64_t cap = 256 * 16;   // 256 CUs, a few blocks each; kernels are grid-stride
  return static_cast<int>(g < 1 ? 1 : (g > cap ? cap : g));
}

}  // namespace

int launch_merge(const dfa_merge_desc& md, void* o_a, float* lse_a, const void* o_b, const float* lse_b,
                 hipStream_t st) {
  const int rpb = 256 / (md.d / 8);
  int gx = (md.rows + rpb - 1) / rpb;
  const int cap = (256 * 16 + md.heads - 1) / md.heads;   // a few blocks per CU in total; rows are grid-strided
  if (gx > cap) gx = cap;
  dim3 grid(gx < 1 ? 1 : gx, md.heads);
  if (md.d == 128) {
    if (md.o_dtype == DFA_BF16) k_merge<128, true><<<grid, 256, 0, st>>>(md, o_a, lse_a, o_b, lse_b);
    else k_merge<128, false><<<grid, 256, 0, st>>>(md, o_a, lse_a, o_b, lse_b);
  } else {
    if (md.o_dtype == DFA_BF16) k_merge<64, true><<<grid, 256, 0, st>>>(md, o_a, lse_a, o_b, lse_b);
    else k_merge<64, false><<<grid, 256, 0, st>>>(md, o_a, lse_a, o_b, lse_b);
  }
  return last_launch_status();
}

int launch_delta(const dfa_shape& sh, const void* o, const void* dO, float* delta, hipStream_t st) {
  const int rpb = 256 / (sh.d / 8);
  dim3 grid((sh.s_q + rpb - 1) / rpb, sh.h_q);
  const bool dob = sh.dtype == DFA_BF16, ob = sh.o_dtype == DFA_BF16;
#define DFA_DELTA(DD, A, B) k_delta<DD, A, B><<<grid, 256, 0, st>>>(sh.s_q, o, sh.o_stride_h, sh.o_stride_s, dO, \
                                sh.q_stride_h, sh.q_stride_s, delta, sh.lse_stride_h)
  if (sh.d == 128) {
    if (dob && ob) DFA_DELTA(128, true, true); else if (dob) DFA_DELTA(128, true, false);
    else if (ob) DFA_DELTA(128, false, true); else DFA_DELTA(128, false, false);
  } else {
    if (dob && ob) DFA_DELTA(64, true, true); else if (dob) DFA_DELTA(64, true, false);
    else if (ob) DFA_DELTA(64, false, true); else DFA_DELTA(64, false, false);
  }
#undef DFA_DELTA
  return last_launch_status();
}

int launch_fill_zero_rows(float* p, int heads, int rows, int d, int64_t stride_h, int64_t stride_s, hipStream_t st) {
  dim3 grid(grid_for(static_cast<int64_t>(rows) * (d / 4), 256), heads);
  k_zero_rows<<<grid, 256, 0, st>>>(p, rows, d / 4, stride_h, stride_s);
  return last_launch_status();
}

int launch_fill_empty_fwd(const dfa_shape& sh, void* o, float* lse, hipStream_t st) {
  dim3 grid(grid_for(static_cast<int64_t>(sh.s_q) * (sh.d / 8), 256), sh.h_q);
  if (sh.o_dtype == DFA_BF16) k_empty_fwd<true><<<grid, 256, 0, st>>>(sh.s_q, sh.d / 8, o, sh.o_stride_h, sh.o_stride_s, lse, sh.lse_stride_h);
  else k_empty_fwd<false><<<grid, 256, 0, st>>>(sh.s_q, sh.d / 8, o, sh.o_stride_h, sh.o_stride_s, lse, sh.lse_stride_h);
  return last_launch_status();
}

}  // namespace dfa
