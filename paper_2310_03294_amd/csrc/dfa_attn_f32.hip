// fp32 mode of the chunk kernels: plain fp32 FMA arithmetic, LDS-tiled, any s_q / s_k.
// This is the precision-reference mode of the library (small problems, 1e-5 agreement with
// fp64); the bf16 MFMA kernels are the fast path.  Tiling: a workgroup of 256 threads owns
// 64 query rows (forward) or 64 key rows (backward) and streams the other operand in tiles
// through LDS; online softmax follows the forward pseudo-code of Appendix A (running row
// maximum m and row sum l, old terms multiplied by exp(m_old - m_new)).
#include "dfa_internal.h"

namespace dfa {
namespace {

constexpr int kThreads = 256;

struct F32Params {
  const float *q, *k, *v, *dO, *lse_in, *delta;
  void* o; float* lse;
  float *dq, *dk, *dv;
  int s_q, s_k, group, causal, o_bf16, accumulate;
  float scale;
  int64_t q_sh, q_ss, kv_sh, kv_ss, o_sh, o_ss, l_sh, dq_sh, dq_ss, dkv_sh, dkv_ss;
};

// rows x D tile from global (row stride ss) into LDS (row stride LD); rows >= nrows become 0
template <int D, int ROWS, int LD>
__device__ inline void load_tile(float* dst, const float* src, int64_t ss, int row0, int nrows) {
  constexpr int C4 = D / 4;
  for (int i = threadIdx.x; i < ROWS * C4; i += kThreads) {
    const int r = i / C4, c = i % C4;
    float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row0 + r < nrows) x = *reinterpret_cast<const float4*>(src + static_cast<int64_t>(row0 + r) * ss + c * 4);
    *reinterpret_cast<float4*>(dst + r * LD + c * 4) = x;
  }
}

template <int D>
__global__ void __launch_bounds__(kThreads) k_fwd_f32(F32Params p) {
  constexpr int BQ = 64, BK = 64, LD = D + 4, LS = BK + 1, NC = D / 16;
  extern __shared__ __align__(16) float smem[];
  float* Qs = smem;
  float* Ks = Qs + BQ * LD;
  float* Vs = Ks + BK * LD;
  float* Ss = Vs + BK * LD;
  float* row_m = Ss + BQ * LS;
  float* row_l = row_m + BQ;
  float* row_a = row_l + BQ;
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  const int h = blockIdx.y, kh = h / p.group, q0 = blockIdx.x * BQ;
  const float* qg = p.q + h * p.q_sh;
  const float* kg = p.k + kh * p.kv_sh;
  const float* vg = p.v + kh * p.kv_sh;

  load_tile<D, BQ, LD>(Qs, qg, p.q_ss, q0, p.s_q);
  // Empty state, or (accumulate) the state of the earlier key/value chunks: the normalised output
  // with its logsumexp is the running (o, m, l) with m = lse and l = 1.
  if (tid < BQ) {
    float m0 = -INFINITY;
    if (p.accumulate && q0 + tid < p.s_q) m0 = p.lse[h * p.l_sh + q0 + tid];
    row_m[tid] = m0; row_l[tid] = m0 > -INFINITY ? 1.f : 0.f;
  }
  float acc[4][NC];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int qi = q0 + ty * 4 + a;
    const bool have = p.accumulate && qi < p.s_q && p.lse[h * p.l_sh + qi] > -INFINITY;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      float x = 0.f;
      if (have) {
        const int64_t off = h * p.o_sh + static_cast<int64_t>(qi) * p.o_ss + tx + 16 * c;
        x = p.o_bf16 ? static_cast<float>(static_cast<const __bf16*>(p.o)[off]) : static_cast<const float*>(p.o)[off];
      }
      acc[a][c] = x;
    }
  }

  const int k_end = p.causal ? min(p.s_k, q0 + BQ) : p.s_k;
  for (int k0 = 0; k0 < k_end; k0 += BK) {
    __syncthreads();
    load_tile<D, BK, LD>(Ks, kg, p.kv_ss, k0, p.s_k);
    load_tile<D, BK, LD>(Vs, vg, p.kv_ss, k0, p.s_k);
    __syncthreads();
    // s = scale * q k^T on a 4x4 micro-tile per thread
    float s[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) s[a][b] = 0.f;
    for (int c = 0; c < D; c += 4) {
      float4 qa[4], kb[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) qa[a] = *reinterpret_cast<const float4*>(Qs + (ty * 4 + a) * LD + c);
#pragma unroll
      for (int b = 0; b < 4; ++b) kb[b] = *reinterpret_cast<const float4*>(Ks + (tx * 4 + b) * LD + c);
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          s[a][b] = fmaf(qa[a].x, kb[b].x, s[a][b]); s[a][b] = fmaf(qa[a].y, kb[b].y, s[a][b]);
          s[a][b] = fmaf(qa[a].z, kb[b].z, s[a][b]); s[a][b] = fmaf(qa[a].w, kb[b].w, s[a][b]);
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int qi = q0 + ty * 4 + a, kj = k0 + tx * 4 + b;
        const bool vis = kj < p.s_k && (!p.causal || kj <= qi);
        Ss[(ty * 4 + a) * LS + tx * 4 + b] = vis ? s[a][b] * p.scale : -INFINITY;
      }
    __syncthreads();
    {  // online softmax: 4 adjacent lanes per row, 16 columns each
      const int row = tid / 4, part = tid % 4;
      float* sr = Ss + row * LS + part * 16;
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < 16; ++j) mx = fmaxf(mx, sr[j]);
      mx = fmaxf(mx, __shfl_xor(mx, 1)); mx = fmaxf(mx, __shfl_xor(mx, 2));
      const float m_old = row_m[row];
      const float m_new = fmaxf(m_old, mx);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 16; ++j) { const float e = expf(sr[j] - m_safe); sr[j] = e; sum += e; }
      sum += __shfl_xor(sum, 1); sum += __shfl_xor(sum, 2);
      const float alpha = expf(m_old - m_safe);   // exp(-inf) = 0 on the first tile
      const float l_old = row_l[row];
      __builtin_amdgcn_wave_barrier();
      if (part == 0) { row_m[row] = m_new; row_l[row] = l_old * alpha + sum; row_a[row] = alpha; }
    }
    __syncthreads();
    float al[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) al[a] = row_a[ty * 4 + a];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int c = 0; c < NC; ++c) acc[a][c] *= al[a];
    for (int j = 0; j < BK; ++j) {
      float pj[4], vv[NC];
#pragma unroll
      for (int a = 0; a < 4; ++a) pj[a] = Ss[(ty * 4 + a) * LS + j];
#pragma unroll
      for (int c = 0; c < NC; ++c) vv[c] = Vs[j * LD + tx + 16 * c];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[a][c] = fmaf(pj[a], vv[c], acc[a][c]);
    }
  }
  __syncthreads();
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int r = ty * 4 + a, qi = q0 + r;
    if (qi >= p.s_q) continue;
    const float l = row_l[r];
    const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const float val = acc[a][c] * inv;
      const int64_t off = h * p.o_sh + static_cast<int64_t>(qi) * p.o_ss + tx + 16 * c;
      if (p.o_bf16) static_cast<__bf16*>(p.o)[off] = static_cast<__bf16>(val);
      else static_cast<float*>(p.o)[off] = val;
    }
    if (tx == 0) p.lse[h * p.l_sh + qi] = l > 0.f ? row_m[r] + logf(l) : -INFINITY;
  }
}

// Backward, key-stationary: a workgroup owns 64 key rows of one kv head and walks over the
// query heads of its group and their query tiles (32 rows).  dk, dv are accumulated in
// registers and written once; dq contributions are added to global memory with fp32 atomics.
template <int D>
__global__ void __launch_bounds__(kThreads) k_bwd_f32(F32Params p) {
  constexpr int BK = 64, BQ = 32, LD = D + 4, LS = BK + 1, NC = D / 16, NQ = D / 8;
  extern __shared__ __align__(16) float smem[];
  float* Ks = smem;
  float* Vs = Ks + BK * LD;
  float* Qs = Vs + BK * LD;
  float* Gs = Qs + BQ * LD;       // dO tile
  float* Ps = Gs + BQ * LD;       // P
  float* Ts = Ps + BQ * LS;       // scale * dS
  float* row_L = Ts + BQ * LS;
  float* row_D = row_L + BQ;
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  const int kh = blockIdx.y, k0 = blockIdx.x * BK;
  load_tile<D, BK, LD>(Ks, p.k + kh * p.kv_sh, p.kv_ss, k0, p.s_k);
  load_tile<D, BK, LD>(Vs, p.v + kh * p.kv_sh, p.kv_ss, k0, p.s_k);
  float dk[4][NC], dv[4][NC];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int c = 0; c < NC; ++c) { dk[a][c] = 0.f; dv[a][c] = 0.f; }

  const int q_begin = p.causal ? (k0 / BQ) * BQ : 0;
  for (int hq = kh * p.group; hq < (kh + 1) * p.group; ++hq) {
    for (int q0 = q_begin; q0 < p.s_q; q0 += BQ) {
      __syncthreads();
      load_tile<D, BQ, LD>(Qs, p.q + hq * p.q_sh, p.q_ss, q0, p.s_q);
      load_tile<D, BQ, LD>(Gs, p.dO + hq * p.q_sh, p.q_ss, q0, p.s_q);
      if (tid < BQ) {
        const bool ok = q0 + tid < p.s_q;
        row_L[tid] = ok ? p.lse_in[hq * p.l_sh + q0 + tid] : -INFINITY;
        row_D[tid] = ok ? p.delta[hq * p.l_sh + q0 + tid] : 0.f;
      }
      __syncthreads();
      {  // s = q k^T and dp = dO v^T on a 2x4 micro-tile: rows ty*2+a, cols tx*4+b
        float s[2][4], dp[2][4];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int b = 0; b < 4; ++b) { s[a][b] = 0.f; dp[a][b] = 0.f; }
        for (int c = 0; c < D; c += 4) {
          float4 qa[2], ga[2], kb[4], vb[4];
#pragma unroll
          for (int a = 0; a < 2; ++a) {
            qa[a] = *reinterpret_cast<const float4*>(Qs + (ty * 2 + a) * LD + c);
            ga[a] = *reinterpret_cast<const float4*>(Gs + (ty * 2 + a) * LD + c);
          }
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            kb[b] = *reinterpret_cast<const float4*>(Ks + (tx * 4 + b) * LD + c);
            vb[b] = *reinterpret_cast<const float4*>(Vs + (tx * 4 + b) * LD + c);
          }
#pragma unroll
          for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
              s[a][b] = fmaf(qa[a].x, kb[b].x, s[a][b]); s[a][b] = fmaf(qa[a].y, kb[b].y, s[a][b]);
              s[a][b] = fmaf(qa[a].z, kb[b].z, s[a][b]); s[a][b] = fmaf(qa[a].w, kb[b].w, s[a][b]);
              dp[a][b] = fmaf(ga[a].x, vb[b].x, dp[a][b]); dp[a][b] = fmaf(ga[a].y, vb[b].y, dp[a][b]);
              dp[a][b] = fmaf(ga[a].z, vb[b].z, dp[a][b]); dp[a][b] = fmaf(ga[a].w, vb[b].w, dp[a][b]);
            }
        }
#pragma unroll
        for (int a = 0; a < 2; ++a) {
          const int r = ty * 2 + a, qi = q0 + r;
          const float L = row_L[r], Dl = row_D[r];
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            const int kj = k0 + tx * 4 + b;
            const bool vis = qi < p.s_q && kj < p.s_k && (!p.causal || kj <= qi) && L > -INFINITY;
            const float pr = vis ? expf(s[a][b] * p.scale - L) : 0.f;
            Ps[r * LS + tx * 4 + b] = pr;
            Ts[r * LS + tx * 4 + b] = pr * (dp[a][b] - Dl) * p.scale;
          }
        }
      }
      __syncthreads();
      // dv_j += sum_i P_ij dO_i ; dk_j += sum_i (scale dS_ij) q_i   (key rows ty*4+a, cols tx+16c)
      for (int i = 0; i < BQ; ++i) {
        float pj[4], tj[4], gv[NC], qv[NC];
#pragma unroll
        for (int a = 0; a < 4; ++a) { pj[a] = Ps[i * LS + ty * 4 + a]; tj[a] = Ts[i * LS + ty * 4 + a]; }
#pragma unroll
        for (int c = 0; c < NC; ++c) { gv[c] = Gs[i * LD + tx + 16 * c]; qv[c] = Qs[i * LD + tx + 16 * c]; }
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
          for (int c = 0; c < NC; ++c) { dv[a][c] = fmaf(pj[a], gv[c], dv[a][c]); dk[a][c] = fmaf(tj[a], qv[c], dk[a][c]); }
      }
      if (p.dq) {  // dq_i += sum_j (scale dS_ij) k_j : row tid/8, cols (tid%8) + 8c
        const int r = tid / 8, cx = tid % 8;
        float dqa[NQ];
#pragma unroll
        for (int c = 0; c < NQ; ++c) dqa[c] = 0.f;
        for (int j = 0; j < BK; ++j) {
          const float t = Ts[r * LS + j];
#pragma unroll
          for (int c = 0; c < NQ; ++c) dqa[c] = fmaf(t, Ks[j * LD + cx + 8 * c], dqa[c]);
        }
        if (q0 + r < p.s_q) {
          float* dst = p.dq + hq * p.dq_sh + static_cast<int64_t>(q0 + r) * p.dq_ss;
#pragma unroll
          for (int c = 0; c < NQ; ++c) atomicAdd(dst + cx + 8 * c, dqa[c]);
        }
      }
    }
  }
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int kj = k0 + ty * 4 + a;
    if (kj >= p.s_k || !p.dk) continue;
    float* dkp = p.dk + kh * p.dkv_sh + static_cast<int64_t>(kj) * p.dkv_ss;
    float* dvp = p.dv + kh * p.dkv_sh + static_cast<int64_t>(kj) * p.dkv_ss;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int col = tx + 16 * c;
      if (p.accumulate) { dkp[col] += dk[a][c]; dvp[col] += dv[a][c]; }
      else { dkp[col] = dk[a][c]; dvp[col] = dv[a][c]; }
    }
  }
}

F32Params make_params(const dfa_shape& sh) {
  F32Params p{};
  p.s_q = sh.s_q; p.s_k = sh.s_k; p.group = sh.h_q / sh.h_kv; p.causal = sh.causal;
  p.o_bf16 = sh.o_dtype == DFA_BF16; p.scale = sh.scale;
  p.q_sh = sh.q_stride_h; p.q_ss = sh.q_stride_s; p.kv_sh = sh.kv_stride_h; p.kv_ss = sh.kv_stride_s;
  p.o_sh = sh.o_stride_h; p.o_ss = sh.o_stride_s; p.l_sh = sh.lse_stride_h;
  p.dq_sh = sh.dq_stride_h; p.dq_ss = sh.dq_stride_s; p.dkv_sh = sh.dkv_stride_h; p.dkv_ss = sh.dkv_stride_s;
  return p;
}

template <typename K>
int set_smem(K kernel, size_t bytes) {
  return hip_status(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes)));
}

}  // namespace

int launch_fwd_f32(const dfa_shape& sh, const float* q, const float* k, const float* v,
                   void* o, float* lse, int accumulate, hipStream_t st) {
  F32Params p = make_params(sh);
  p.q = q; p.k = k; p.v = v; p.o = o; p.lse = lse; p.accumulate = accumulate;
  dim3 grid((sh.s_q + 63) / 64, sh.h_q);
  const int D = sh.d;
  const size_t smem = sizeof(float) * (3 * 64 * (D + 4) + 64 * 65 + 3 * 64);
  int rc;
  if (D == 128) { if ((rc = set_smem(k_fwd_f32<128>, smem))) return rc; k_fwd_f32<128><<<grid, kThreads, smem, st>>>(p); }
  else { if ((rc = set_smem(k_fwd_f32<64>, smem))) return rc; k_fwd_f32<64><<<grid, kThreads, smem, st>>>(p); }
  return last_launch_status();
}

int launch_bwd_f32(const dfa_shape& sh, const float* q, const float* k, const float* v,
                   const float* lse, const float* delta, const float* dO,
                   float* dq, float* dk, float* dv, int accumulate, hipStream_t st) {
  F32Params p = make_params(sh);
  p.q = q; p.k = k; p.v = v; p.lse_in = lse; p.delta = delta; p.dO = dO;
  p.dq = dq; p.dk = dk; p.dv = dv; p.accumulate = accumulate;
  int rc;
  if (!accumulate && dq) {
    rc = launch_fill_zero_rows(dq, sh.h_q, sh.s_q, sh.d, sh.dq_stride_h, sh.dq_stride_s, st);
    if (rc) return rc;
  }
  dim3 grid((sh.s_k + 63) / 64, sh.h_kv);
  const int D = sh.d;
  const size_t smem = sizeof(float) * (2 * 64 * (D + 4) + 2 * 32 * (D + 4) + 2 * 32 * 65 + 2 * 32);
  if (D == 128) { if ((rc = set_smem(k_bwd_f32<128>, smem))) return rc; k_bwd_f32<128><<<grid, kThreads, smem, st>>>(p); }
  else { if ((rc = set_smem(k_bwd_f32<64>, smem))) return rc; k_bwd_f32<64><<<grid, kThreads, smem, st>>>(p); }
  return last_launch_status();
}

}  // namespace dfa
