// bf16 backward chunk kernel for gfx950: dq, dk, dv contributions of one chunk pair from the
// saved logsumexp and D = rowsum(dO o O), without re-running the forward (Section 3.3).
//
// Key-stationary decomposition.  A workgroup of 4 wavefronts owns 128 key rows of one kv head
// (32 per wavefront, their K and V held in registers as MFMA B operands) and walks over the
// query heads of the group and their query tiles of 64 rows, staged (Q, dO, lse, D) in LDS.
// Per tile and wavefront, five products on v_mfma_f32_32x32x16_bf16:
//   S  = Q K^T, dP = dO V^T            (queries x keys: each lane holds 16 queries of ONE key)
//   P  = exp2(S c - lse log2e), dS = P o (dP - D)        (registers only)
//   dV^T += dO^T P,  dK^T += Q^T dS    (P, dS fed back from registers as B operands; dO^T, Q^T
//                                       gathered from LDS with the transposing read)
//   dQ = dS K                          (contraction over keys: dS goes through LDS once so that
//                                       each wavefront reduces over all 128 keys of the workgroup
//                                       for its 32 output columns, then fp32 atomics to dq)
// dk, dv are written once per workgroup (summed over the group's query heads in registers).
#include "dfa_internal.h"
#include "dfa_mfma.h"

namespace dfa {
namespace {

constexpr int D = 128;
constexpr int BN = 128;    // key rows per workgroup
constexpr int BM = 64;     // query rows per LDS tile
constexpr int NTHREADS = 256;
constexpr int QTILE_BYTES = BM * kRowBytes;       // rows padded to 272 B
constexpr int DST_BYTES = (BN / 2) * kRowBytes;   // dS^T as 64 padded rows, two keys per row
constexpr float LOG2E = 1.4426950408889634f;

struct BwdParams {
  const __bf16 *q, *k, *v, *dO;
  const float *lse, *delta;
  float *dq, *dk, *dv;
  int s_q, s_k, h_kv, group, causal, accumulate, ntk, total, per_xcd;
  float scale;
  int64_t q_sh, q_ss, kv_sh, kv_ss, l_sh, dq_sh, dq_ss, dkv_sh, dkv_ss;
};

struct QTileRegs { uint4 q[4], g[4]; float ld; };

__device__ __forceinline__ void qtile_load(QTileRegs& t, const BwdParams& p, int hq, int q0, int tid) {
  const int c = tid & 15;
  const __bf16* qg = p.q + hq * p.q_sh;
  const __bf16* gg = p.dO + hq * p.q_sh;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (tid >> 4) + 16 * i;
    if (q0 + r < p.s_q) {
      const int64_t off = static_cast<int64_t>(q0 + r) * p.q_ss + c * 8;
      t.q[i] = *reinterpret_cast<const uint4*>(qg + off);
      t.g[i] = *reinterpret_cast<const uint4*>(gg + off);
    } else {
      t.q[i] = make_uint4(0, 0, 0, 0);
      t.g[i] = make_uint4(0, 0, 0, 0);
    }
  }
  // threads 0..63 fetch lse (pre-multiplied by log2 e), threads 64..127 fetch D
  t.ld = 0.f;
  if (tid < 128) {
    const int r = tid & 63;
    const bool ok = q0 + r < p.s_q;
    if (tid < 64) {
      const float L = ok ? p.lse[hq * p.l_sh + q0 + r] : INFINITY;
      t.ld = (L > -INFINITY) ? L * LOG2E : INFINITY;   // +inf makes P exactly 0 for that row
    } else {
      t.ld = ok ? p.delta[hq * p.l_sh + q0 + r] : 0.f;
    }
  }
}

__device__ __forceinline__ void qtile_store(const QTileRegs& t, char* Qs, char* Gs, float* LDs, int tid) {
  const int c = tid & 15;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (tid >> 4) + 16 * i;
    const int off = tile_off(r, c);
    *reinterpret_cast<uint4*>(Qs + off) = t.q[i];
    *reinterpret_cast<uint4*>(Gs + off) = t.g[i];
  }
  if (tid < 128) LDs[tid] = t.ld;
}

// dS^T tile: key kv (0..127), query column qc (0..63) -> byte offset; two keys share a padded row
__device__ __forceinline__ int dst_off(int kv, int qc) {
  return tile_off(kv >> 1, 0) + ((kv & 1) << 7) + (qc << 1);
}

__device__ __forceinline__ bf16x8 cat8(bf16x4 lo, bf16x4 hi) {
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__global__ void __launch_bounds__(NTHREADS, 1) k_bwd_bf16(BwdParams p) {
  extern __shared__ __align__(16) char smem[];
  char* Qs = smem;                         // 16 KB
  char* Gs = smem + QTILE_BYTES;           // 16 KB  (dO tile)
  char* Ts = smem + 2 * QTILE_BYTES;       // 16 KB  (dS^T tile)
  float* LDs = reinterpret_cast<float*>(smem + 2 * QTILE_BYTES + DST_BYTES);   // lse'[64], D[64]

  const int bid = blockIdx.x;
  const int item = (bid & 7) * p.per_xcd + (bid >> 3);
  if (item >= p.total) return;
  const int kh = item / p.ntk;
  int tk = item % p.ntk;
  // causal: key tile 0 meets every query tile, so low tiles are the long ones and go first
  const int k0 = tk * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r32 = lane & 31, hh = lane >> 5;
  const int kvl = wave * 32 + r32;          // key index within the workgroup's tile
  const int kvrow = k0 + kvl;
  const bool kvalid = kvrow < p.s_k;
  // per-lane LDS bases; everything else in an LDS address is a compile-time constant
  const int a_base = tile_off(r32, hh);                       // row reads (A operand of S, dP)
  const int g_base = gather_base(lane);                       // transposed gathers of Q, dO
  const int w_base = dst_off(kvl, hh * 4);                    // dS^T writes of this lane's key
  const int t_base = dst_off(4 * (lane >> 5) + ((lane & 15) >> 2), 16 * ((lane >> 4) & 1) + 4 * (lane & 3));

  // K^T and V^T B operands of this wavefront's 32 keys (contraction over d)
  bf16x8 kT[8], vT[8];
  {
    const int64_t off = kh * p.kv_sh + static_cast<int64_t>(kvrow) * p.kv_ss + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 a = make_uint4(0, 0, 0, 0), b = make_uint4(0, 0, 0, 0);
      if (kvalid) {
        a = *reinterpret_cast<const uint4*>(p.k + off + 16 * ks);
        b = *reinterpret_cast<const uint4*>(p.v + off + 16 * ks);
      }
      kT[ks] = __builtin_bit_cast(bf16x8, a);
      vT[ks] = __builtin_bit_cast(bf16x8, b);
    }
  }
  // K as B operand of dQ = dS K (contraction over the 128 keys, this wavefront's 32 columns):
  // stage the whole K tile in LDS once (it fits the Q + dO buffers) and gather it transposed.
  bf16x8 kB[8];
  {
    const int c = tid & 15;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = (tid >> 4) + 16 * i;
      uint4 x = make_uint4(0, 0, 0, 0);
      if (k0 + r < p.s_k)
        x = *reinterpret_cast<const uint4*>(p.k + kh * p.kv_sh + static_cast<int64_t>(k0 + r) * p.kv_ss + c * 8);
      *reinterpret_cast<uint4*>(smem + tile_off(r, c)) = x;
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kB[ks] = lds_gather(smem, g_base + ks * 16 * kRowBytes + wave * 64);
    __syncthreads();
  }

  f32x16 dvT[4], dkT[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) { dvT[i][j] = 0.f; dkT[i][j] = 0.f; }

  const float c2 = p.scale * LOG2E;
  const int q_begin = p.causal ? k0 : 0;            // k0 is a multiple of BM
  const int ntq = (p.s_q - q_begin + BM - 1) / BM;  // query tiles per head for this key tile
  const int niter = ntq * p.group;

  QTileRegs tr;
  if (niter > 0) {
    qtile_load(tr, p, kh * p.group, q_begin, tid);
    qtile_store(tr, Qs, Gs, LDs, tid);
  }
  __syncthreads();

  for (int it = 0; it < niter; ++it) {
    const int hq = kh * p.group + it / ntq;
    const int q0 = q_begin + (it % ntq) * BM;
    const bool more = it + 1 < niter;
    if (more) qtile_load(tr, p, kh * p.group + (it + 1) / ntq, q_begin + ((it + 1) % ntq) * BM, tid);

    // S = Q K^T and dP = dO V^T for two 32-query blocks
    f32x16 s[2], dp[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
      for (int j = 0; j < 16; ++j) { s[qb][j] = 0.f; dp[qb][j] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const int off = a_base + qb * 32 * kRowBytes + ks * 32;
        s[qb] = mfma32(lds_read_b128(Qs, off), kT[ks], s[qb]);
        dp[qb] = mfma32(lds_read_b128(Gs, off), vT[ks], dp[qb]);
      }
    }
    // P and dS (in place: s <- P, dp <- dS)
    const bool need_mask = (k0 + BN > p.s_k) || (p.causal && q0 < k0 + BN - 1);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int qi = qb * 32 + g4 * 8 + hh * 4;       // first of 4 consecutive query rows
        const f32x4 L4 = *reinterpret_cast<const f32x4*>(LDs + qi);
        const f32x4 D4 = *reinterpret_cast<const f32x4*>(LDs + 64 + qi);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = g4 * 4 + e;
          float pr = __builtin_amdgcn_exp2f(fmaf(s[qb][j], c2, -L4[e]));
          if (need_mask) {
            const int qrow = q0 + qi + e;
            if (!kvalid || (p.causal && kvrow > qrow)) pr = 0.f;
          }
          s[qb][j] = pr;
          dp[qb][j] = pr * (dp[qb][j] - D4[e]);
        }
      }
    // dV^T += dO^T P ; dK^T += Q^T dS
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8 pb = pack8(s[qb], u * 8);
        const bf16x8 db_ = pack8(dp[qb], u * 8);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const int goff = g_base + (qb * 32 + u * 16) * kRowBytes + db * 64;
          dvT[db] = mfma32(lds_gather(Gs, goff), pb, dvT[db]);
          dkT[db] = mfma32(lds_gather(Qs, goff), db_, dkT[db]);
        }
      }
    // dS^T -> LDS (8-byte pieces: 4 consecutive queries of this lane's key)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        bf16x4 b;
#pragma unroll
        for (int e = 0; e < 4; ++e) b[e] = static_cast<__bf16>(dp[qb][g4 * 4 + e]);
        *reinterpret_cast<bf16x4*>(Ts + w_base + (qb * 32 + g4 * 8) * 2) = b;
      }
    __syncthreads();
    if (more) qtile_store(tr, Qs, Gs, LDs, tid);
    // dQ block (32 queries x this wavefront's 32 columns) over all 128 keys, then atomics
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 dq;
#pragma unroll
      for (int j = 0; j < 16; ++j) dq[j] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        // keys +16 per step = logical rows +8: physical +16 rows on even steps, +2 more on odd
        // ones; the second half of the operand (keys +8) sits one physical row further
        const int off = t_base + ((ks >> 1) * 16 + (ks & 1) * 2) * kRowBytes + qb * 64;
        dq = mfma32(cat8(lds_read_tr(Ts, off), lds_read_tr(Ts, off + kRowBytes)), kB[ks], dq);
      }
      float* dst = p.dq + hq * p.dq_sh + wave * 32 + r32;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int qrow = q0 + qb * 32 + (j >> 2) * 8 + hh * 4 + (j & 3);
        if (qrow < p.s_q) atomicAdd(dst + static_cast<int64_t>(qrow) * p.dq_ss, dq[j] * p.scale);
      }
    }
    __syncthreads();
  }

  if (kvalid) {
    float* dkp = p.dk + kh * p.dkv_sh + static_cast<int64_t>(kvrow) * p.dkv_ss;
    float* dvp = p.dv + kh * p.dkv_sh + static_cast<int64_t>(kvrow) * p.dkv_ss;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = db * 32 + g4 * 8 + hh * 4;
        float4 a = make_float4(dkT[db][g4 * 4] * p.scale, dkT[db][g4 * 4 + 1] * p.scale,
                               dkT[db][g4 * 4 + 2] * p.scale, dkT[db][g4 * 4 + 3] * p.scale);
        float4 b = make_float4(dvT[db][g4 * 4], dvT[db][g4 * 4 + 1], dvT[db][g4 * 4 + 2], dvT[db][g4 * 4 + 3]);
        if (p.accumulate) {
          const float4 a0 = *reinterpret_cast<const float4*>(dkp + col);
          const float4 b0 = *reinterpret_cast<const float4*>(dvp + col);
          a.x += a0.x; a.y += a0.y; a.z += a0.z; a.w += a0.w;
          b.x += b0.x; b.y += b0.y; b.z += b0.z; b.w += b0.w;
        }
        *reinterpret_cast<float4*>(dkp + col) = a;
        *reinterpret_cast<float4*>(dvp + col) = b;
      }
  }
}

}  // namespace

int launch_bwd_bf16(const dfa_shape& sh, const void* q, const void* k, const void* v,
                    const float* lse, const float* delta, const void* dO,
                    float* dq, float* dk, float* dv, int accumulate, hipStream_t st) {
  BwdParams p{};
  p.q = static_cast<const __bf16*>(q); p.k = static_cast<const __bf16*>(k); p.v = static_cast<const __bf16*>(v);
  p.dO = static_cast<const __bf16*>(dO); p.lse = lse; p.delta = delta; p.dq = dq; p.dk = dk; p.dv = dv;
  p.s_q = sh.s_q; p.s_k = sh.s_k; p.h_kv = sh.h_kv; p.group = sh.h_q / sh.h_kv; p.causal = sh.causal;
  p.accumulate = accumulate; p.scale = sh.scale;
  p.q_sh = sh.q_stride_h; p.q_ss = sh.q_stride_s; p.kv_sh = sh.kv_stride_h; p.kv_ss = sh.kv_stride_s;
  p.l_sh = sh.lse_stride_h; p.dq_sh = sh.dq_stride_h; p.dq_ss = sh.dq_stride_s;
  p.dkv_sh = sh.dkv_stride_h; p.dkv_ss = sh.dkv_stride_s;
  p.ntk = (sh.s_k + BN - 1) / BN;
  const int64_t total = static_cast<int64_t>(p.ntk) * sh.h_kv;
  if (total > (1 << 30)) return DFA_ERR_SHAPE;
  p.total = static_cast<int>(total);
  p.per_xcd = (p.total + 7) / 8;
  if (!accumulate) {
    const int rc = launch_fill_zero_rows(dq, sh.h_q, sh.s_q, sh.d, sh.dq_stride_h, sh.dq_stride_s, st);
    if (rc) return rc;
  }
  const size_t smem = 2 * QTILE_BYTES + DST_BYTES + 128 * sizeof(float);
  k_bwd_bf16<<<p.per_xcd * 8, NTHREADS, smem, st>>>(p);
  return last_launch_status();
}

}  // namespace dfa
