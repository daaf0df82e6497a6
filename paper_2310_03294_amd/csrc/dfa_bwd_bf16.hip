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
//
// The tile body exists twice: an interior version without any bounds or mask logic (one
// straight-line block the scheduler can software-pipeline: the MFMAs of one 32-query block
// run under the exp/VALU work of the other) and an edge version for ragged or diagonal tiles.
#include "dfa_internal.h"
#include "dfa_mfma.h"

namespace dfa {
namespace {

constexpr int D = 128;
constexpr int BN = 128;    // key rows per workgroup
constexpr int BM = 64;     // query rows per LDS tile
constexpr int NTHREADS = 256;
constexpr int QTILE_BYTES = BM * kRowBytes;    // 17 KB (rows padded to 272 B)
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

template <bool EDGE>
__device__ __forceinline__ void qtile_load(QTileRegs& t, const BwdParams& p, int hq, int q0, int tid) {
  const int c = tid & 15;
  const __bf16* qg = p.q + hq * p.q_sh;
  const __bf16* gg = p.dO + hq * p.q_sh;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (tid >> 4) + 16 * i;
    if (!EDGE || q0 + r < p.s_q) {
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
    const bool ok = !EDGE || q0 + r < p.s_q;
    const int idx = ok ? q0 + r : 0;
    if (tid < 64) {
      const float L = p.lse[hq * p.l_sh + idx];
      t.ld = (ok && L > -INFINITY) ? L * LOG2E : INFINITY;   // +inf makes P exactly 0 for that row
    } else {
      const float dl = p.delta[hq * p.l_sh + idx];
      t.ld = ok ? dl : 0.f;
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

  // XCD-aware mapping: workgroup ids go round-robin over the 8 XCDs; give every XCD a contiguous
  // range of (kv head, key tile) items so that the tiles of one head share Q/dO in one L2.
  const int bid = blockIdx.x;
  const int item = (bid & 7) * p.per_xcd + (bid >> 3);
  if (item >= p.total) return;
  const int kh = item / p.ntk;
  const int tk = item % p.ntk;       // causal: low key tiles meet the most query tiles and come first
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
    const int64_t off = kh * p.kv_sh + static_cast<int64_t>(kvalid ? kvrow : 0) * p.kv_ss + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 a = *reinterpret_cast<const uint4*>(p.k + off + 16 * ks);
      uint4 b = *reinterpret_cast<const uint4*>(p.v + off + 16 * ks);
      if (!kvalid) { a = make_uint4(0, 0, 0, 0); b = make_uint4(0, 0, 0, 0); }
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
  const bool k_edge = k0 + BN > p.s_k;

  QTileRegs tr;
  if (niter > 0) {
    qtile_load<true>(tr, p, kh * p.group, q_begin, tid);
    qtile_store(tr, Qs, Gs, LDs, tid);
  }
  __syncthreads();

  // ---- tile body -------------------------------------------------------------------------
  auto phase_a = [&](int qb, f32x16& s, f32x16& dp) {     // S = Q K^T, dP = dO V^T (32 queries)
#pragma unroll
    for (int j = 0; j < 16; ++j) { s[j] = 0.f; dp[j] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const int off = a_base + qb * 32 * kRowBytes + ks * 32;
      s = mfma32(lds_read_b128(Qs, off), kT[ks], s);
      dp = mfma32(lds_read_b128(Gs, off), vT[ks], dp);
    }
  };
  auto phase_c = [&](int qb, const f32x16& pr, const f32x16& ds) {   // dV^T += dO^T P, dK^T += Q^T dS
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bf16x8 pb = pack8(pr, u * 8);
      const bf16x8 sb = pack8(ds, u * 8);
      const int roff = g_base + (qb * 32 + u * 16) * kRowBytes;
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        dvT[db] = mfma32(lds_gather(Gs, roff + db * 64), pb, dvT[db]);
        dkT[db] = mfma32(lds_gather(Qs, roff + db * 64), sb, dkT[db]);
      }
    }
  };
  auto write_ds = [&](int qb, const f32x16& ds) {
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      bf16x4 b;
#pragma unroll
      for (int e = 0; e < 4; ++e) b[e] = static_cast<__bf16>(ds[g4 * 4 + e]);
      *reinterpret_cast<bf16x4*>(Ts + w_base + (qb * 32 + g4 * 8) * 2) = b;
    }
  };
  auto dq_block = [&](int qb, f32x16& dq) {                // dQ (32 queries x 32 columns) over 128 keys
#pragma unroll
    for (int j = 0; j < 16; ++j) dq[j] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      // keys +16 per step = logical rows +8: physical +16 rows on even steps, +2 more on odd ones;
      // the second half of the operand (keys +8 = logical rows +4) sits one physical row further
      const int off = t_base + ((ks >> 1) * 16 + (ks & 1) * 2) * kRowBytes + qb * 64;
      dq = mfma32(cat8(lds_read_tr(Ts, off), lds_read_tr(Ts, off + kRowBytes)), kB[ks], dq);
    }
  };

  for (int it = 0; it < niter; ++it) {
    const int hq = kh * p.group + it / ntq;
    const int q0 = q_begin + (it % ntq) * BM;
    const bool more = it + 1 < niter;
    if (more) {
      const int hq_n = kh * p.group + (it + 1) / ntq;
      const int q0_n = q_begin + ((it + 1) % ntq) * BM;
      if (q0_n + BM <= p.s_q) qtile_load<false>(tr, p, hq_n, q0_n, tid);
      else qtile_load<true>(tr, p, hq_n, q0_n, tid);
    }
    const bool edge = k_edge || (q0 + BM > p.s_q) || (p.causal && q0 < k0 + BN - 1);

    f32x16 s0, dp0, s1, dp1;
    if (!edge) {
      // interior tile: straight-line code, MFMAs of one query block under the VALU work of the other
      phase_a(0, s0, dp0);
      phase_a(1, s1, dp1);
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const f32x4 L4 = *reinterpret_cast<const f32x4*>(LDs + g4 * 8 + hh * 4);
        const f32x4 D4 = *reinterpret_cast<const f32x4*>(LDs + 64 + g4 * 8 + hh * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = g4 * 4 + e;
          const float pr = __builtin_amdgcn_exp2f(fmaf(s0[j], c2, -L4[e]));
          s0[j] = pr;
          dp0[j] = pr * (dp0[j] - D4[e]);
        }
      }
      phase_c(0, s0, dp0);
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const f32x4 L4 = *reinterpret_cast<const f32x4*>(LDs + 32 + g4 * 8 + hh * 4);
        const f32x4 D4 = *reinterpret_cast<const f32x4*>(LDs + 96 + g4 * 8 + hh * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = g4 * 4 + e;
          const float pr = __builtin_amdgcn_exp2f(fmaf(s1[j], c2, -L4[e]));
          s1[j] = pr;
          dp1[j] = pr * (dp1[j] - D4[e]);
        }
      }
      write_ds(0, dp0);
      phase_c(1, s1, dp1);
      write_ds(1, dp1);
    } else {
      // edge tile (ragged sizes or the causal diagonal): one query block at a time, masked
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        phase_a(qb, s0, dp0);
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int qi = qb * 32 + g4 * 8 + hh * 4;
          const f32x4 L4 = *reinterpret_cast<const f32x4*>(LDs + qi);
          const f32x4 D4 = *reinterpret_cast<const f32x4*>(LDs + 64 + qi);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int j = g4 * 4 + e;
            float pr = __builtin_amdgcn_exp2f(fmaf(s0[j], c2, -L4[e]));
            const int qrow = q0 + qi + e;
            pr = (!kvalid || (p.causal && kvrow > qrow)) ? 0.f : pr;
            s0[j] = pr;
            dp0[j] = pr * (dp0[j] - D4[e]);
          }
        }
        phase_c(qb, s0, dp0);
        write_ds(qb, dp0);
      }
    }
    __syncthreads();
    if (more) qtile_store(tr, Qs, Gs, LDs, tid);
    {
      f32x16 dq0, dq1;
      dq_block(0, dq0);
      dq_block(1, dq1);
      float* dst = p.dq + hq * p.dq_sh + static_cast<int64_t>(q0) * p.dq_ss + wave * 32 + r32;
      if (q0 + BM <= p.s_q) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int rr = (j >> 2) * 8 + hh * 4 + (j & 3);
          atomicAdd(dst + static_cast<int64_t>(rr) * p.dq_ss, dq0[j] * p.scale);
          atomicAdd(dst + static_cast<int64_t>(rr + 32) * p.dq_ss, dq1[j] * p.scale);
        }
      } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int rr = (j >> 2) * 8 + hh * 4 + (j & 3);
          if (q0 + rr < p.s_q) atomicAdd(dst + static_cast<int64_t>(rr) * p.dq_ss, dq0[j] * p.scale);
          if (q0 + rr + 32 < p.s_q) atomicAdd(dst + static_cast<int64_t>(rr + 32) * p.dq_ss, dq1[j] * p.scale);
        }
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
