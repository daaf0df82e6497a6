// bf16 backward chunk kernels for gfx950: dq, dk, dv contributions of one chunk pair from the
// saved logsumexp and D = rowsum(dO o O), without re-running the forward (Section 3.3).
//
// Two kernels, no atomics, deterministic:
//
//  k_bwd_dkdv_bf16 (key-stationary).  A workgroup of 4 wavefronts owns 128 key rows of one kv
//  head (32 per wavefront, their K and V held in registers as MFMA B operands) and walks over the
//  query heads of the group and their query tiles of 64 rows, staged (Q, dO, lse, D) in a
//  double-buffered LDS tile.  Per tile and wavefront, on v_mfma_f32_32x32x16_bf16:
//    S = Q K^T, dP = dO V^T         (queries x keys: each lane holds 16 queries of ONE key)
//    P = exp2(S c - lse log2e), dS = P o (dP - D)          (registers only)
//    dV^T += dO^T P, dK^T += Q^T dS (P, dS fed back from registers as B operands; dO^T, Q^T
//                                    gathered from LDS with the transposing read)
//  dk, dv are written once per workgroup (summed over the group's query heads in registers).
//
//  k_bwd_dq_bf16 (query-stationary).  A workgroup of 4 wavefronts owns 128 query rows of one head
//  (Q^T, dO^T, lse, D in registers) and walks over the key/value chunk in tiles of 64 rows in
//  LDS: S^T = K Q^T, dP^T = V dO^T (keys x queries: each lane holds 16 keys of ONE query, so lse
//  and D are per-lane scalars), dS^T from registers as the B operand of dQ^T += K^T dS^T.
//
// The fused alternative (one kernel, dq by fp32 atomics) was measured first: the L2 atomic units
// retire about one fp32 atomic per clock and channel (~3.1e11 per second on the whole chip),
// which caps a 128-key workgroup tile at ~400 TFLOP/s no matter how the rest is scheduled.
// Recomputing S and dP in a second kernel costs 7 products instead of 5 but has no such cap.
#include "dfa_internal.h"
#include "dfa_mfma.h"

namespace dfa {
namespace {

constexpr int NTHREADS = 256;
constexpr float LOG2E = 1.4426950408889634f;

struct BwdParams {
  const __bf16 *q, *k, *v, *dO;
  const float *lse, *delta;
  float *dq, *dk, *dv;
  int s_q, s_k, h_q, h_kv, group, causal, accumulate, ntile, total, per_xcd;
  float scale;
  int64_t q_sh, q_ss, kv_sh, kv_ss, l_sh, dq_sh, dq_ss, dkv_sh, dkv_ss;
};

// ============================================================================================
// dK, dV
// ============================================================================================
namespace kv {

constexpr int BN = 128;    // key rows per workgroup
constexpr int BM = 64;     // query rows per LDS tile
constexpr int QTILE_BYTES = BM * kRowBytes;        // rows padded to 272 B
constexpr int BUF_BYTES = 2 * QTILE_BYTES + 512;   // Q tile, dO tile, lse'[64] + D[64]

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

__global__ void __launch_bounds__(NTHREADS, 1) k_bwd_dkdv_bf16(BwdParams p) {
  extern __shared__ __align__(16) char smem[];
  // Buffer b: Q at b*BUF, dO at b*BUF + QTILE, lse'[64] and D[64] at b*BUF + 2*QTILE.

  // XCD-aware mapping: workgroup ids go round-robin over the 8 XCDs; give every XCD a contiguous
  // range of (kv head, key tile) items so that the tiles of one head share Q/dO in one L2.
  const int bid = blockIdx.x;
  const int item = (bid & 7) * p.per_xcd + (bid >> 3);
  if (item >= p.total) return;
  const int kh = item / p.ntile;
  const int tk = item % p.ntile;     // causal: low key tiles meet the most query tiles and come first
  const int k0 = tk * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps tile branches scalar
  const int r32 = lane & 31, hh = lane >> 5;
  const int kvrow = k0 + wave * 32 + r32;
  const bool kvalid = kvrow < p.s_k;
  // per-lane LDS bases; everything else in an LDS address is a compile-time constant
  const int a_base = tile_off(r32, hh);                       // row reads (A operand of S, dP)
  const int g_base = gather_base(lane);                       // transposed gathers of Q, dO

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
    qtile_store(tr, smem, smem + QTILE_BYTES, reinterpret_cast<float*>(smem + 2 * QTILE_BYTES), tid);
  }
  __syncthreads();

  for (int it = 0; it < niter; ++it) {
    const int q0 = q_begin + (it % ntq) * BM;
    const bool more = it + 1 < niter;
    const int boff = (it & 1) * BUF_BYTES;
    const char* Qs = smem + boff;
    const char* Gs = Qs + QTILE_BYTES;
    const float* LDs = reinterpret_cast<const float*>(Qs + 2 * QTILE_BYTES);
    char* Qn = smem + (BUF_BYTES - boff);              // buffer of the next tile
    const bool edge = k_edge || (q0 + BM > p.s_q) || (p.causal && q0 < k0 + BN - 1);

    // The tile is two blocks of 32 queries, software-pipelined by hand inside the wavefront (one
    // wavefront per SIMD here, so nothing else hides latencies): the MFMAs of one block are
    // issued between slices of the exp/VALU work of the other, and every LDS operand is read
    // 2-4 MFMA steps before it is used.  DFA_SCHED_FENCE pins that order.
#define DFA_RA(QB, KS, SL)                                                         \
  {                                                                                \
    const int off_ = a_base + (QB) * 32 * kRowBytes + (KS) * 32;                   \
    qa[SL] = lds_read_b128(Qs, off_);                                              \
    ga[SL] = lds_read_b128(Gs, off_);                                              \
  }
#define DFA_RG(QB, I, SL)                                                          \
  {                                                                                \
    const int off_ = g_base + ((QB) * 32 + ((I) >> 2) * 16) * kRowBytes + ((I) & 3) * 64; \
    gd[SL] = lds_gather(Gs, off_);                                                 \
    gq[SL] = lds_gather(Qs, off_);                                                 \
  }
#define DFA_RLD(QB, G4, SL)                                                        \
  {                                                                                \
    L4[SL] = *reinterpret_cast<const f32x4*>(LDs + (QB) * 32 + (G4) * 8 + hh * 4); \
    D4[SL] = *reinterpret_cast<const f32x4*>(LDs + 64 + (QB) * 32 + (G4) * 8 + hh * 4); \
  }
#define DFA_BELEM(S, DP, QB, J)                                                    \
  {                                                                                \
    float pr_ = __builtin_amdgcn_exp2f(fmaf(S[J], c2, -L4[((J) >> 2) & 1][(J) & 3])); \
    if (edge) {                                                                    \
      const int qrow_ = q0 + (QB) * 32 + ((J) >> 2) * 8 + hh * 4 + ((J) & 3);       \
      pr_ = (!kvalid || (p.causal && kvrow > qrow_)) ? 0.f : pr_;                  \
    }                                                                              \
    S[J] = pr_;                                                                    \
    DP[J] = pr_ * (DP[J] - D4[((J) >> 2) & 1][(J) & 3]);                           \
  }
    {
      bf16x8 qa[4], ga[4], gd[2], gq[2], pb0[2], sb0[2], pb1[2], sb1[2];
      f32x4 L4[2], D4[2];
      f32x16 s0, dp0, s1, dp1;
#pragma unroll
      for (int j = 0; j < 16; ++j) { s0[j] = 0.f; dp0[j] = 0.f; s1[j] = 0.f; dp1[j] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) DFA_RA(0, ks, ks)
      DFA_RLD(0, 0, 0)
      if (more) {   // global loads of the next tile; stored to the other LDS buffer after the tile
        const int hq_n = kh * p.group + (it + 1) / ntq;
        const int q0_n = q_begin + ((it + 1) % ntq) * BM;
        if (q0_n + BM <= p.s_q) qtile_load<false>(tr, p, hq_n, q0_n, tid);
        else qtile_load<true>(tr, p, hq_n, q0_n, tid);
      }
      DFA_SCHED_FENCE();
      // stage 1: S, dP of block 0
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        s0 = mfma32(qa[ks & 3], kT[ks], s0);
        dp0 = mfma32(ga[ks & 3], vT[ks], dp0);
        if (ks < 4) DFA_RA(0, ks + 4, ks & 3) else DFA_RA(1, ks - 4, ks & 3)
        DFA_SCHED_FENCE();
      }
      // stage 2: S, dP of block 1 between slices of P, dS of block 0
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        s1 = mfma32(qa[ks & 3], kT[ks], s1);
        dp1 = mfma32(ga[ks & 3], vT[ks], dp1);
        if (ks < 4) DFA_RA(1, ks + 4, ks & 3)
        if (ks == 4) DFA_RG(0, 0, 0)
        if (ks == 5) DFA_RG(0, 1, 1)
        if ((ks & 1) == 0 && ks < 6) DFA_RLD(0, ks / 2 + 1, (ks / 2 + 1) & 1)
        if (ks == 6) DFA_RLD(1, 0, 0)
        DFA_BELEM(s0, dp0, 0, 2 * ks)
        DFA_BELEM(s0, dp0, 0, 2 * ks + 1)
        if (ks == 4) pb0[0] = pack8(s0, 0);
        if (ks == 5) sb0[0] = pack8(dp0, 0);
        DFA_SCHED_FENCE();
      }
      // stage 3: dV^T, dK^T of block 0 between slices of P, dS of block 1
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (i == 0) pb0[1] = pack8(s0, 8);       // first used at i == 4
        if (i == 1) sb0[1] = pack8(dp0, 8);
        dvT[i & 3] = mfma32(gd[i & 1], pb0[i >> 2], dvT[i & 3]);
        dkT[i & 3] = mfma32(gq[i & 1], sb0[i >> 2], dkT[i & 3]);
        if (i + 2 < 8) DFA_RG(0, i + 2, i & 1) else DFA_RG(1, i - 6, i & 1)
        if ((i & 1) == 0 && i < 6) DFA_RLD(1, i / 2 + 1, (i / 2 + 1) & 1)
        DFA_BELEM(s1, dp1, 1, 2 * i)
        DFA_BELEM(s1, dp1, 1, 2 * i + 1)
        if (i == 4) pb1[0] = pack8(s1, 0);
        if (i == 5) sb1[0] = pack8(dp1, 0);
        DFA_SCHED_FENCE();
      }
      // stage 4: dV^T, dK^T of block 1
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (i == 0) pb1[1] = pack8(s1, 8);
        if (i == 1) sb1[1] = pack8(dp1, 8);
        dvT[i & 3] = mfma32(gd[i & 1], pb1[i >> 2], dvT[i & 3]);
        dkT[i & 3] = mfma32(gq[i & 1], sb1[i >> 2], dkT[i & 3]);
        if (i + 2 < 8) DFA_RG(1, i + 2, i & 1)
        DFA_SCHED_FENCE();
      }
    }
#undef DFA_RA
#undef DFA_RG
#undef DFA_RLD
#undef DFA_BELEM
    if (more) qtile_store(tr, Qn, Qn + QTILE_BYTES, reinterpret_cast<float*>(Qn + 2 * QTILE_BYTES), tid);
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

}  // namespace kv

// ============================================================================================
// dQ
// ============================================================================================
namespace qs {

constexpr int BM = 128;     // query rows per workgroup
constexpr int BN = 64;      // key rows per LDS tile
constexpr int TILE_BYTES = BN * kRowBytes;

struct TileRegs { uint4 k[4], v[4]; };

__device__ __forceinline__ void tile_load(TileRegs& t, const __bf16* kg, const __bf16* vg, int64_t ss,
                                          int k0, int s_k, int tid) {
  const int c = tid & 15;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (tid >> 4) + 16 * i;
    if (k0 + r < s_k) {
      const int64_t off = static_cast<int64_t>(k0 + r) * ss + c * 8;
      t.k[i] = *reinterpret_cast<const uint4*>(kg + off);
      t.v[i] = *reinterpret_cast<const uint4*>(vg + off);
    } else {
      t.k[i] = make_uint4(0, 0, 0, 0);
      t.v[i] = make_uint4(0, 0, 0, 0);
    }
  }
}

__device__ __forceinline__ void tile_store(const TileRegs& t, char* Ks, char* Vs, int tid) {
  const int c = tid & 15;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (tid >> 4) + 16 * i;
    const int off = tile_off(r, c);
    *reinterpret_cast<uint4*>(Ks + off) = t.k[i];
    *reinterpret_cast<uint4*>(Vs + off) = t.v[i];
  }
}

__global__ void __launch_bounds__(NTHREADS, 2) k_bwd_dq_bf16(BwdParams p) {
  extern __shared__ __align__(16) char smem[];
  char* Ks = smem;
  char* Vs = smem + TILE_BYTES;

  const int bid = blockIdx.x;
  const int item = (bid & 7) * p.per_xcd + (bid >> 3);   // contiguous (head, query tile) range per XCD
  if (item >= p.total) return;
  const int head = item / p.ntile;
  int tq = item % p.ntile;
  if (p.causal) tq = p.ntile - 1 - tq;      // longest rows first
  const int kh = head / p.group;
  const int q0 = tq * BM;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps tile branches scalar
  const int r32 = lane & 31, hh = lane >> 5;
  const int q0w = q0 + wave * 32;
  const int qrow = q0w + r32;
  const bool qvalid = qrow < p.s_q;
  const int a_base = tile_off(r32, hh);
  const int g_base = gather_base(lane);

  const __bf16* kg = p.k + kh * p.kv_sh;
  const __bf16* vg = p.v + kh * p.kv_sh;

  // Q^T and dO^T operands: lane holds row qrow, columns 16 ks + 8 hh .. +7; lse' and D of that row
  bf16x8 qB[8], gB[8];
  {
    const int64_t off = head * p.q_sh + static_cast<int64_t>(qvalid ? qrow : 0) * p.q_ss + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 a = *reinterpret_cast<const uint4*>(p.q + off + 16 * ks);
      uint4 b = *reinterpret_cast<const uint4*>(p.dO + off + 16 * ks);
      if (!qvalid) { a = make_uint4(0, 0, 0, 0); b = make_uint4(0, 0, 0, 0); }
      qB[ks] = __builtin_bit_cast(bf16x8, a);
      gB[ks] = __builtin_bit_cast(bf16x8, b);
    }
  }
  float Lr = INFINITY, Dr = 0.f;          // +inf makes P exactly 0 for rows past the end
  if (qvalid) {
    const float L = p.lse[head * p.l_sh + qrow];
    Lr = L > -INFINITY ? L * LOG2E : INFINITY;
    Dr = p.delta[head * p.l_sh + qrow];
  }

  f32x16 dqT[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) dqT[i][j] = 0.f;
  const float c2 = p.scale * LOG2E;

  const int k_end = p.causal ? min(p.s_k, q0 + BM) : p.s_k;
  const int ntiles = (k_end + BN - 1) / BN;

  TileRegs tr;
  tile_load(tr, kg, vg, p.kv_ss, 0, p.s_k, tid);
  tile_store(tr, Ks, Vs, tid);
  __syncthreads();

  for (int it = 0; it < ntiles; ++it) {
    const int k0 = it * BN;
    const bool more = it + 1 < ntiles;
    if (more) tile_load(tr, kg, vg, p.kv_ss, k0 + BN, p.s_k, tid);

    const bool active = !(p.causal && k0 > q0w + 31);
    if (active) {
      const bool need_mask = (k0 + BN > p.s_k) || (p.causal && k0 + BN - 1 > q0w);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        // S^T = K Q^T, dP^T = V dO^T for 32 keys; row reads run 4 steps ahead
        bf16x8 ka[4], va[4];
        f32x16 s, dp;
#pragma unroll
        for (int j = 0; j < 16; ++j) { s[j] = 0.f; dp[j] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const int off = a_base + nb * 32 * kRowBytes + ks * 32;
          ka[ks] = lds_read_b128(Ks, off);
          va[ks] = lds_read_b128(Vs, off);
        }
        DFA_SCHED_FENCE();
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          s = mfma32(ka[ks & 3], qB[ks], s);
          dp = mfma32(va[ks & 3], gB[ks], dp);
          if (ks < 4) {
            const int off = a_base + nb * 32 * kRowBytes + (ks + 4) * 32;
            ka[ks & 3] = lds_read_b128(Ks, off);
            va[ks & 3] = lds_read_b128(Vs, off);
          }
          DFA_SCHED_FENCE();
        }
        // dS^T = P^T o (dP^T - D): lse' and D are per-lane scalars here
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const float pr = __builtin_amdgcn_exp2f(fmaf(s[j], c2, -Lr));
          dp[j] = pr * (dp[j] - Dr);
        }
        if (need_mask) {
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const int kvi = k0 + nb * 32 + (j >> 2) * 8 + hh * 4 + (j & 3);
            if (kvi >= p.s_k || (p.causal && kvi > qrow)) dp[j] = 0.f;
          }
        }
        // dQ^T += K^T dS^T: 2 contraction steps of 16 keys, 4 blocks of 32 columns
        bf16x8 sb[2], gk[2];
        sb[0] = pack8(dp, 0); sb[1] = pack8(dp, 8);
#pragma unroll
        for (int i = 0; i < 2; ++i) gk[i] = lds_gather(Ks, g_base + (nb * 32) * kRowBytes + i * 64);
        DFA_SCHED_FENCE();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int u = i >> 2, db = i & 3;
          dqT[db] = mfma32(gk[i & 1], sb[u], dqT[db]);
          if (i + 2 < 8)
            gk[i & 1] = lds_gather(Ks, g_base + (nb * 32 + ((i + 2) >> 2) * 16) * kRowBytes + ((i + 2) & 3) * 64);
          DFA_SCHED_FENCE();
        }
      }
    }
    __syncthreads();
    if (more) tile_store(tr, Ks, Vs, tid);
    __syncthreads();
  }

  if (qvalid) {
    float* dst = p.dq + head * p.dq_sh + static_cast<int64_t>(qrow) * p.dq_ss;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = db * 32 + g4 * 8 + hh * 4;
        float4 a = make_float4(dqT[db][g4 * 4] * p.scale, dqT[db][g4 * 4 + 1] * p.scale,
                               dqT[db][g4 * 4 + 2] * p.scale, dqT[db][g4 * 4 + 3] * p.scale);
        if (p.accumulate) {
          const float4 a0 = *reinterpret_cast<const float4*>(dst + col);
          a.x += a0.x; a.y += a0.y; a.z += a0.z; a.w += a0.w;
        }
        *reinterpret_cast<float4*>(dst + col) = a;
      }
  }
}

}  // namespace qs
}  // namespace

int launch_bwd_bf16(const dfa_shape& sh, const void* q, const void* k, const void* v,
                    const float* lse, const float* delta, const void* dO,
                    float* dq, float* dk, float* dv, int accumulate, hipStream_t st) {
  BwdParams p{};
  p.q = static_cast<const __bf16*>(q); p.k = static_cast<const __bf16*>(k); p.v = static_cast<const __bf16*>(v);
  p.dO = static_cast<const __bf16*>(dO); p.lse = lse; p.delta = delta; p.dq = dq; p.dk = dk; p.dv = dv;
  p.s_q = sh.s_q; p.s_k = sh.s_k; p.h_q = sh.h_q; p.h_kv = sh.h_kv; p.group = sh.h_q / sh.h_kv;
  p.causal = sh.causal; p.accumulate = accumulate; p.scale = sh.scale;
  p.q_sh = sh.q_stride_h; p.q_ss = sh.q_stride_s; p.kv_sh = sh.kv_stride_h; p.kv_ss = sh.kv_stride_s;
  p.l_sh = sh.lse_stride_h; p.dq_sh = sh.dq_stride_h; p.dq_ss = sh.dq_stride_s;
  p.dkv_sh = sh.dkv_stride_h; p.dkv_ss = sh.dkv_stride_s;

  if (dk) {  // dK, dV
    BwdParams a = p;
    a.ntile = (sh.s_k + kv::BN - 1) / kv::BN;
    const int64_t total = static_cast<int64_t>(a.ntile) * sh.h_kv;
    if (total > (1 << 30)) return DFA_ERR_SHAPE;
    a.total = static_cast<int>(total);
    a.per_xcd = (a.total + 7) / 8;
    const size_t smem = 2 * kv::BUF_BYTES;
    static bool attr_set = false;   // > 64 KB of dynamic LDS needs the opt-in once per process
    if (!attr_set) {
      const int rc = hip_status(hipFuncSetAttribute(reinterpret_cast<const void*>(kv::k_bwd_dkdv_bf16),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                                    static_cast<int>(smem)));
      if (rc) return rc;
      attr_set = true;
    }
    kv::k_bwd_dkdv_bf16<<<a.per_xcd * 8, NTHREADS, smem, st>>>(a);
    const int rc = last_launch_status();
    if (rc) return rc;
  }
  if (dq) {  // dQ
    BwdParams b = p;
    b.ntile = (sh.s_q + qs::BM - 1) / qs::BM;
    const int64_t total = static_cast<int64_t>(b.ntile) * sh.h_q;
    if (total > (1 << 30)) return DFA_ERR_SHAPE;
    b.total = static_cast<int>(total);
    b.per_xcd = (b.total + 7) / 8;
    qs::k_bwd_dq_bf16<<<b.per_xcd * 8, NTHREADS, 2 * qs::TILE_BYTES, st>>>(b);
  }
  return last_launch_status();
}

}  // namespace dfa
