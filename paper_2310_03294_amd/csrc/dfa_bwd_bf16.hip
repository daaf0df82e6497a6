// bf16 backward chunk kernels for gfx950: dq, dk, dv contributions of one chunk pair from the
// saved logsumexp and D = rowsum(dO o O), without re-running the forward (Section 3.3).
//
// Two kernels, no atomics, deterministic:
//
//  k_bwd_dkdv_bf16 (key-stationary).  A workgroup of 8 wavefronts owns 128 key rows of one kv
//  head and walks over the query heads of the group and their query tiles of 64 rows, staged
//  (Q, dO, lse, D) through LDS rings.  The wavefronts are specialised in pairs per 32-key block,
//  one of each kind per SIMD, so that the exponentials of one overlap the MFMAs of the other:
//    "S" wavefront  (K^T in registers):  S = Q K^T, P = exp2(S c - lse log2e), hands P (bf16)
//                                        to its partner through LDS, dV^T += dO^T P
//    "dP" wavefront (V^T in registers):  dP - D = dO V^T - D (the MFMA chains start from -D),
//                                        dS = P o (dP - D), dK^T += Q^T dS
//  (queries x keys tiles on v_mfma_f32_32x32x16_bf16: each lane holds 16 queries of ONE key; P
//  and dS are fed back from registers as B operands; dO^T, Q^T are gathered from LDS with the
//  transposing read).  The dP wavefronts run one tile behind, so one barrier per tile suffices.
//  Wavefronts raise their priority while they issue MFMAs, so that the other kind's VALU work
//  fills the gaps instead of delaying them.
//  dv / dk are written once per workgroup (summed over the group's query heads in registers).
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
#include <mutex>

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

constexpr int NT = 512;     // 8 wavefronts: 4 "S" wavefronts (dV) and 4 "dP" wavefronts (dK)
constexpr int BN = 128;     // key rows per workgroup, 32 per wavefront pair
constexpr int BM = 64;      // query rows per LDS tile
constexpr int QTILE_BYTES = BM * kRowBytes;   // rows padded to 272 B
constexpr int LD_BYTES = 1024;                // lse'[64], -D[64], 128 spare floats
constexpr int PX_BYTES = 4 * 4096;            // P hand-over: 4 key blocks x (64 x 32 bf16)
// LDS map.  Tile t lives in Q slot t % 3, dO slot t % 2, lse/D slot t % 3, P slot t % 2.
constexpr int OFF_Q = 0;
constexpr int OFF_G = OFF_Q + 3 * QTILE_BYTES;
constexpr int OFF_LD = OFF_G + 2 * QTILE_BYTES;
constexpr int OFF_PX = OFF_LD + 3 * LD_BYTES;
constexpr int SMEM_BYTES = OFF_PX + 2 * PX_BYTES;

// The Q and dO tiles go from global memory straight into LDS (global_load_lds_dwordx4: every
// lane supplies its own global address, the wavefront's 64 x 16 bytes land contiguously at the
// LDS address in M0).  A padded tile is 17 such 1 KB pieces; of the four wavefronts that copy a
// tile, wavefront w moves pieces 4w .. 4w + 3 and (w = 0 only) 16.  Byte 16 s of the tile is chunk
// s % 17 of physical row s / 17; chunk 16 is the pad (it receives a copy of chunk 15).  Only
// lse / D pass through a register.  The S wavefronts copy the Q tiles, the dP wavefronts the dO
// tiles, each piece issued from inline assembly between two MFMAs of a product (the memory pipe
// takes ~17 cycles per piece and CU: issued in a burst, the pieces stall the wavefront) and waited
// for just before the slot's barrier.  Measured with time stamps per phase: all staging at the top
// of the slot cost the S wavefronts, which are the critical path, 600-900 of ~3500 cycles per tile.
struct QTileRegs { float ld; bool ld_ok; };

// Where the next (Q, dO, lse, D) tile comes from: wave-uniform head bases, advanced tile by
// tile (no division in the loop), plus per-thread 32-bit byte offsets inside the head.
struct QTileCursor {
  const char *qh, *gh;       // Q and dO of the head
  const float* ldh;          // lse (even wavefronts) or D (odd wavefronts) of the head
  int q0;                    // first query row of the tile
};

// Cursor to the next tile: the next rows, or the next query head of the group.
__device__ __forceinline__ void qtile_advance(QTileCursor& cur, const BwdParams& p, int q_begin, int q_end) {
  cur.q0 += 64;
  if (cur.q0 >= q_end) {
    cur.q0 = q_begin;
    cur.qh += p.q_sh * 2; cur.gh += p.q_sh * 2; cur.ldh += p.l_sh;
  }
}
// The same as selects only (adv false: the cursor stays), for use inside the straight-line loops.
__device__ __forceinline__ void qtile_advance_if(QTileCursor& cur, bool adv, const BwdParams& p, int q_begin,
                                                 int q_end) {
  const int nq = cur.q0 + 64;
  const bool wrap = nq >= q_end;
  const int64_t hs = (adv && wrap) ? p.q_sh * 2 : 0;
  const int64_t ls = (adv && wrap) ? p.l_sh : 0;
  cur.q0 = adv ? (wrap ? q_begin : nq) : cur.q0;
  cur.qh += hs; cur.gh += hs; cur.ldh += ls;
}

// Rows past s_q are clamped to the last row instead of zero-filled: their lse' is +inf, so P and
// dS vanish for them whatever (finite) Q and dO the tile holds.  Qs, Gs: LDS tiles to fill.
__device__ __forceinline__ void qtile_copy(const QTileCursor& cur, const TileLane& m, const BwdParams& p,
                                           char* Qs, char* Gs, int w, int lane) {
  const uint32_t rowbytes = static_cast<uint32_t>(p.q_ss) * 2;
  tile_dma(cur.qh, rowbytes, cur.q0, p.s_q - 1, m, Qs, w, lane);
  tile_dma(cur.gh, rowbytes, cur.q0, p.s_q - 1, m, Gs, w, lane);
}

// lse (S wavefronts 0, 2, 3) or D (S wavefront 1) of the tile's 64 rows, one per lane, into a
// register.  Wavefronts 2 and 3 only go through the motions (their values land in a spare part
// of the slot), which keeps the staging free of branches.
__device__ __forceinline__ void qtile_load_ld(QTileRegs& t, const QTileCursor& cur, const BwdParams& p, int tid) {
  const int last = p.s_q - 1;
  const int r = cur.q0 + (tid & 63);
  t.ld_ok = r <= last;
  t.ld = cur.ldh[static_cast<uint32_t>(min(r, last))];
}

// LDs: the slot's 256 floats: lse'[64], -D[64], 128 spare.
__device__ __forceinline__ void qtile_store(const QTileRegs& t, float* LDs, int tid, bool is_d) {
  // lse pre-multiplied by log2 e; +inf makes P exactly 0 for an absent or empty row
  const float l = (t.ld_ok && t.ld > -INFINITY) ? t.ld * LOG2E : INFINITY;
  const float d = t.ld_ok ? -t.ld : 0.f;      // -D: the value the dP accumulators start from
  LDs[tid] = is_d ? d : l;
}

// C[qb] += X[qb rows] * B^T over d for both 32-row blocks of the tile: X rows are read from LDS
// (A operand), B is the wavefront's K^T or V^T held in registers; the caller sets what the chains
// start from (zero, or -D for the dP products).
struct NoHook { __device__ __forceinline__ void operator()(int) const {} };
// hook(ks) runs after the MFMAs of step ks (the callers issue their tile-copy pieces there)
template <class Hook = NoHook>
__device__ __forceinline__ void row_products(f32x16& c0, f32x16& c1, const char* Xs, int a_base,
                                             const bf16x8 (&bT)[8], Hook hook = Hook()) {
  constexpr int AHEAD = 3;                      // LDS reads run this many d-steps ahead of the MFMAs
  bf16x8 x0[AHEAD + 1], x1[AHEAD + 1];
#pragma unroll
  for (int ks = 0; ks < AHEAD; ++ks) {
    x0[ks] = lds_read_b128(Xs, a_base + ks * 32);
    x1[ks] = lds_read_b128(Xs, a_base + 32 * kRowBytes + ks * 32);
  }
  DFA_SCHED_FENCE();
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    if (ks + AHEAD < 8) {
      x0[(ks + AHEAD) % (AHEAD + 1)] = lds_read_b128(Xs, a_base + (ks + AHEAD) * 32);
      x1[(ks + AHEAD) % (AHEAD + 1)] = lds_read_b128(Xs, a_base + 32 * kRowBytes + (ks + AHEAD) * 32);
    }
    c0 = mfma32(x0[ks % (AHEAD + 1)], bT[ks], c0);
    c1 = mfma32(x1[ks % (AHEAD + 1)], bT[ks], c1);
    hook(ks);
    DFA_SCHED_FENCE();
  }
}

// acc[db] += Y^T[db block of d][64 queries] * W[64 queries][32 keys]: Y^T is gathered from the
// row-major LDS tile with the transposing read, W (P or dS) comes from registers in the order
// an MFMA result tile has (w[qb][half] = rows (e/4)*8 + 4h + e%4 of 16-row half `half`).
constexpr int COL_AHEAD = 4;              // gathers run this many MFMAs ahead
__device__ __forceinline__ int col_off(int g_base, int n) {       // n = qb * 8 + half * 4 + db
  return g_base + ((n >> 3) * 32 + ((n >> 2) & 1) * 16) * kRowBytes + (n & 3) * 64;
}
// The first COL_AHEAD gathers of col_products, issued early (e.g. before a barrier) so that the
// products can start without waiting for LDS.
// (The pieces are kept as raw 32-bit vectors: carried around a loop as bf16 vectors they would be
// taken apart into 16-bit halves and put together again.)
__device__ __forceinline__ void col_prefetch(u32x4 (&y)[COL_AHEAD + 1], const char* Ys, int g_base) {
#pragma unroll
  for (int n = 0; n < COL_AHEAD; ++n) y[n] = __builtin_bit_cast(u32x4, lds_gather(Ys, col_off(g_base, n)));
}
template <bool PRE, class Hook = NoHook>
__device__ __forceinline__ void col_products(f32x16 (&acc)[4], const char* Ys, int g_base,
                                             const bf16x8 (&w)[2][2], u32x4 (&y)[COL_AHEAD + 1],
                                             Hook hook = Hook()) {
  constexpr int AHEAD = COL_AHEAD;
  if (!PRE) col_prefetch(y, Ys, g_base);
  DFA_SCHED_FENCE();
#pragma unroll
  for (int n = 0; n < 16; ++n) {
    if (n + AHEAD < 16)
      y[(n + AHEAD) % (AHEAD + 1)] = __builtin_bit_cast(u32x4, lds_gather(Ys, col_off(g_base, n + AHEAD)));
    acc[n & 3] = mfma32(__builtin_bit_cast(bf16x8, y[n % (AHEAD + 1)]), w[n >> 3][(n >> 2) & 1], acc[n & 3]);
    hook(n);
    DFA_SCHED_FENCE();
  }
}

// RAGGED: s_q is no multiple of the 64-row tile, so a head's last tile has rows past the end.
template <bool RAGGED>
__global__ void __launch_bounds__(NT, 2) k_bwd_dkdv_bf16(BwdParams p) {
  extern __shared__ __align__(16) char smem[];

  // XCD-aware mapping: workgroup ids go round-robin over the 8 XCDs; give every XCD a contiguous
  // range of (kv head, key tile) items so that the tiles of one head share Q/dO in one L2.
  const int bid = blockIdx.x;
  const int item = (bid & 7) * p.per_xcd + (bid >> 3);
  if (item >= p.total) return;
  const int kh = item / p.ntile;
  const int tk = item % p.ntile;     // causal: low key tiles meet the most query tiles and come first
  const int k0 = tk * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: role branches stay scalar
  const int kb = wave & 3;            // 32-key block of this wavefront
  const bool dp_wave = wave >= 4;     // false: S, P, dV;  true: dP, dS, dK
  const int r32 = lane & 31, hh = lane >> 5;
  const int kvrow = k0 + kb * 32 + r32;
  const bool kvalid = kvrow < p.s_k;
  // per-lane LDS bases; everything else in an LDS address is a compile-time constant
  const int a_base = tile_off(r32, hh);                       // row reads (A operand of S, dP)
  const int g_base = gather_base(lane);                       // transposed gathers of Q, dO

  // B operands over d of this wavefront's 32 keys: K^T for an S wavefront, V^T for a dP wavefront
  bf16x8 bT[8];
  {
    const __bf16* src = dp_wave ? p.v : p.k;
    const int64_t off = kh * p.kv_sh + static_cast<int64_t>(kvalid ? kvrow : 0) * p.kv_ss + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 a = *reinterpret_cast<const uint4*>(src + off + 16 * ks);
      if (!kvalid) a = make_uint4(0, 0, 0, 0);
      bT[ks] = __builtin_bit_cast(bf16x8, a);
    }
  }

  // dV^T (S wavefront) or dK^T (dP wavefront): [d block][d within block][key]
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;

  const float c2 = p.scale * LOG2E;
  const int q_begin = p.causal ? k0 : 0;            // k0 is a multiple of BM
  const int ntq = (p.s_q - q_begin + BM - 1) / BM;  // query tiles per head for this key tile
  const int niter = ntq * p.group;

  // Tile staging.  Two cursors: `cur` for the tile copies (tile t + 1 during slot t; Q by the S
  // wavefronts, dO by the dP wavefronts), `curl` for lse / D (S wavefronts), which pass through a
  // register and run one tile further ahead.  Order inside a slot: store the held lse / D, load
  // the next ones, THEN issue the copies - the compiler knows nothing of the copies, so any wait
  // it places for its own loads must come before them or it would wait for them too.
  QTileRegs tr;
  QTileCursor cur, curl;
  {
    const int hq0 = kh * p.group;
    cur.qh = reinterpret_cast<const char*>(p.q + hq0 * p.q_sh);
    cur.gh = reinterpret_cast<const char*>(p.dO + hq0 * p.q_sh);
    cur.ldh = (kb == 1 ? p.delta : p.lse) + hq0 * p.l_sh;
    cur.q0 = q_begin;
    curl = cur;
  }
  const int q_end = q_begin + ntq * BM;
  const uint32_t q_rowbytes = static_cast<uint32_t>(p.q_ss) * 2;
  const TileLane tl = tile_lane(kb, lane, q_rowbytes);
  if (!dp_wave) {
    qtile_load_ld(tr, curl, p, tid);
    qtile_store(tr, reinterpret_cast<float*>(smem + OFF_LD), tid, kb == 1);
    if (niter > 1) {
      qtile_advance(curl, p, q_begin, q_end);
      qtile_load_ld(tr, curl, p, tid);           // lse / D of tile 1, stored in slot 0
    }
    qtile_copy(cur, tl, p, smem + OFF_Q, smem + OFF_G, kb, lane);
    lds_dma_wait();                                // this wavefront's copies into LDS have landed
  }
  __syncthreads();

  // One barrier per tile.  Between two barriers ("slot" t) the S wavefronts take tile t all the
  // way (S, P, hand P over through LDS, dV) while the dP wavefronts finish tile t-1 (dS, dK) and
  // then start tile t (dP).  The two kinds share each SIMD, so the exponentials of one overlap
  // the MFMAs of the other.  Both kinds run niter + 1 slots (the S wavefronts idle in the last,
  // the dP wavefronts have no dS/dK in the first); each kind has its own straight-line loop.
  int slot = 0;            // t % 3
  f32x16 zero;
#pragma unroll
  for (int j = 0; j < 16; ++j) zero[j] = 0.f;
  if (!dp_wave) {
    int q0 = q_begin;      // first query row of tile `it`
    for (int it = 0; it < niter; ++it) {
      const bool more = it + 1 < niter;
      const int next = slot == 2 ? 0 : slot + 1;
      const char* Qs = smem + OFF_Q + slot * QTILE_BYTES;
      const char* Gs = smem + OFF_G + (it & 1) * QTILE_BYTES;
      const float* Ls = reinterpret_cast<const float*>(smem + OFF_LD + slot * LD_BYTES);
      // Staging, all of it inside the S products so that it costs no time of its own, and without
      // branches (past the last tile the cursors stay: the same tile, lse and D go once more into
      // ring slots nobody reads).  First (step 0) lse / D: tile it + 1 from the register into
      // LDS, tile it + 2 into the register - before the first copy of the slot, because the
      // compiler's wait for that register would otherwise wait for the copies too.  Then the Q
      // tile it + 1 into ring slot `next`, one piece every other step.
      qtile_advance_if(cur, more, p, q_begin, q_end);
      const TileCopy cq = tile_copy_plan<RAGGED>(cur.qh, q_rowbytes, cur.q0, p.s_q - 1, tl,
                                                 smem + OFF_Q + next * QTILE_BYTES, kb, lane);
      f32x16 c0 = zero, c1 = zero;
      __builtin_amdgcn_s_setprio(3);
      row_products(c0, c1, Qs, a_base, bT, [&](int ks) {          // S = Q K^T
        if (ks == 0) {
          qtile_store(tr, reinterpret_cast<float*>(smem + OFF_LD + next * LD_BYTES), tid, kb == 1);
          qtile_advance_if(curl, it + 2 < niter, p, q_begin, q_end);
          qtile_load_ld(tr, curl, p, tid);
        }
        if (ks == 1) tile_copy_piece<0>(cq);
        if (ks == 2 && kb == 0) tile_copy_piece<4>(cq);
        if (ks == 3) tile_copy_piece<1>(cq);
        if (ks == 5) tile_copy_piece<2>(cq);
        if (ks == 7) tile_copy_piece<3>(cq);
      });
      __builtin_amdgcn_s_setprio(0);
      // Only the causal diagonal needs a mask: query rows past s_q carry lse' = +inf (P = 0)
      // and key rows past s_k only feed dk/dv rows that are never written.
      if (p.causal && q0 < k0 + BN - 1) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int qrow = q0 + (j >> 2) * 8 + hh * 4 + (j & 3);
          c0[j] = kvrow > qrow ? -INFINITY : c0[j];
          c1[j] = kvrow > qrow + 32 ? -INFINITY : c1[j];
        }
      }
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const f32x4 l0 = *reinterpret_cast<const f32x4*>(Ls + g4 * 8 + hh * 4);
        const f32x4 l1 = *reinterpret_cast<const f32x4*>(Ls + 32 + g4 * 8 + hh * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          c0[g4 * 4 + e] = __builtin_amdgcn_exp2f(fmaf(c0[g4 * 4 + e], c2, -l0[e]));
          c1[g4 * 4 + e] = __builtin_amdgcn_exp2f(fmaf(c1[g4 * 4 + e], c2, -l1[e]));
        }
      }
      bf16x8 w[2][2];
      w[0][0] = pack8(c0, 0); w[0][1] = pack8(c0, 8);
      w[1][0] = pack8(c1, 0); w[1][1] = pack8(c1, 8);
      {  // hand P to the dP wavefront of the same key block: lane-private, any layout will do
        char* px = smem + OFF_PX + (it & 1) * PX_BYTES + kb * 4096 + lane * 16;
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<bf16x8*>(px + j * 1024) = w[j >> 1][j & 1];
      }
      u32x4 y[COL_AHEAD + 1];
      __builtin_amdgcn_s_setprio(3);
      col_products<false>(acc, Gs, g_base, w, y);    // dV^T += dO^T P
      __builtin_amdgcn_s_setprio(0);
      lds_dma_wait();                                // this wavefront's copies into LDS have landed
      __syncthreads();
      slot = next;
      q0 = q0 + BM >= q_end ? q_begin : q0 + BM;
    }
    __syncthreads();      // the dP wavefronts' last slot
  } else {
    f32x16 c0, c1;        // dP of the tile in flight, carried over the barrier
    bf16x8 w[2][2];
    // -D of a tile's 64 query rows in the accumulator layout: the dP chains start from it, so what
    // they end with is dP - D
    auto neg_d = [&](f32x16& d0, f32x16& d1, int ld_slot) {
      const float* Ds = reinterpret_cast<const float*>(smem + OFF_LD + ld_slot * LD_BYTES) + 64;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(Ds + g4 * 8 + hh * 4);
        const f32x4 b = *reinterpret_cast<const f32x4*>(Ds + 32 + g4 * 8 + hh * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { d0[g4 * 4 + e] = a[e]; d1[g4 * 4 + e] = b[e]; }
      }
    };
    auto dS_prev = [&](int it) {                     // dS of tile it - 1 from P (LDS) and dP - D (registers)
      const char* px = smem + OFF_PX + ((it & 1) ^ 1) * PX_BYTES + kb * 4096 + lane * 16;
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j >> 1][j & 1] = *reinterpret_cast<const bf16x8*>(px + j * 1024);
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        c0[j] = static_cast<float>(w[0][j >> 3][j & 7]) * c0[j];
        c1[j] = static_cast<float>(w[1][j >> 3][j & 7]) * c1[j];
      }
      w[0][0] = pack8(c0, 0); w[0][1] = pack8(c0, 8);
      w[1][0] = pack8(c1, 0); w[1][1] = pack8(c1, 8);
    };
    // The first Q^T gathers of the next slot's dK products are issued before the barrier (that Q
    // tile has been in LDS for a whole slot), so after the barrier only P has to be waited for.
    u32x4 y[COL_AHEAD + 1];
    // The dP wavefronts copy the dO tiles: tile t + 1 during slot t, its pieces spread over the
    // products (past the last tile the cursor stays: the same tile goes into the unused slot).
    {  // slot 0: dP of tile 0 only
      qtile_advance_if(cur, niter > 1, p, q_begin, q_end);
      const TileCopy cg = tile_copy_plan<RAGGED>(cur.gh, q_rowbytes, cur.q0, p.s_q - 1, tl,
                                                 smem + OFF_G + QTILE_BYTES, kb, lane);
      if (kb == 0) tile_copy_piece<4>(cg);
      neg_d(c0, c1, 0);
      row_products(c0, c1, smem + OFF_G, a_base, bT, [&](int ks) {
        if (ks == 0) tile_copy_piece<0>(cg);
        if (ks == 2) tile_copy_piece<1>(cg);
        if (ks == 4) tile_copy_piece<2>(cg);
        if (ks == 6) tile_copy_piece<3>(cg);
      });
      col_prefetch(y, smem + OFF_Q, g_base);
      lds_dma_wait();
      DFA_BARRIER_NO_DRAIN();
      slot = 1;
    }
    for (int it = 1; it < niter; ++it) {
      const int prev = slot == 0 ? 2 : slot - 1, next = slot == 2 ? 0 : slot + 1;
      qtile_advance_if(cur, it + 1 < niter, p, q_begin, q_end);
      const TileCopy cg = tile_copy_plan<RAGGED>(cur.gh, q_rowbytes, cur.q0, p.s_q - 1, tl,
                                                 smem + OFF_G + ((it + 1) & 1) * QTILE_BYTES, kb, lane);
      if (kb == 0) tile_copy_piece<4>(cg);
      __builtin_amdgcn_s_setprio(3);
      dS_prev(it);
      neg_d(c0, c1, slot);                       // read straight into the accumulators, under the dK products
      col_products<true>(acc, smem + OFF_Q + prev * QTILE_BYTES, g_base, w, y, [&](int n) {  // dK^T += Q^T dS
        if (n == 1) tile_copy_piece<0>(cg);
        if (n == 5) tile_copy_piece<1>(cg);
        if (n == 9) tile_copy_piece<2>(cg);
        if (n == 13) tile_copy_piece<3>(cg);
      });
      row_products(c0, c1, smem + OFF_G + (it & 1) * QTILE_BYTES, a_base, bT);   // dP - D = dO V^T - D
      col_prefetch(y, smem + OFF_Q + slot * QTILE_BYTES, g_base);
      __builtin_amdgcn_s_setprio(0);
      lds_dma_wait();                            // this wavefront's copies into LDS have landed
      DFA_BARRIER_NO_DRAIN();                    // nothing else it wrote has to be seen by the others
      slot = next;
    }
    dS_prev(niter);
    col_products<true>(acc, smem + OFF_Q + (slot == 0 ? 2 : slot - 1) * QTILE_BYTES, g_base, w, y);
    __syncthreads();
  }


  if (kvalid) {
    float* dst = (dp_wave ? p.dk : p.dv) + kh * p.dkv_sh + static_cast<int64_t>(kvrow) * p.dkv_ss;
    const float f = dp_wave ? p.scale : 1.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = db * 32 + g4 * 8 + hh * 4;
        float4 a = make_float4(acc[db][g4 * 4] * f, acc[db][g4 * 4 + 1] * f, acc[db][g4 * 4 + 2] * f,
                               acc[db][g4 * 4 + 3] * f);
        if (p.accumulate) {
          const float4 a0 = *reinterpret_cast<const float4*>(dst + col);
          a.x += a0.x; a.y += a0.y; a.z += a0.z; a.w += a0.w;
        }
        *reinterpret_cast<float4*>(dst + col) = a;
      }
  }
}

}  // namespace kv

// ============================================================================================
// dQ
// ============================================================================================
namespace qs {

constexpr int BN = 64;      // key rows per LDS tile
constexpr int TILE_BYTES = BN * kRowBytes;

// NW wavefronts of 32 query rows each per workgroup, two wavefronts per SIMD either way: NW = 4 (128
// rows, two workgroups per CU, scheduled independently of each other) or NW = 8 (256 rows, one
// workgroup per CU: every K/V tile copy and every barrier serve twice the rows; measured 2-3 %
// faster on long chunks, where the copies are what the second independent workgroup used to hide, and
// no faster on short ones and on the causal diagonal pair, which keep the 128-row form).
template <int NW>
__global__ void __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) k_bwd_dq_bf16(BwdParams p) {
  constexpr int BM = NW * 32;     // query rows per workgroup
  extern __shared__ __align__(16) char smem[];   // two (K tile, V tile) buffers

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

  const char* kg = reinterpret_cast<const char*>(p.k + kh * p.kv_sh);
  const char* vg = reinterpret_cast<const char*>(p.v + kh * p.kv_sh);
  const uint32_t kv_rowbytes = static_cast<uint32_t>(p.kv_ss) * 2;
  // Tile copies: with 4 wavefronts each moves its quarter of the K tile and of the V tile; with 8,
  // wavefronts 0-3 move the K tile and 4-7 the V tile.
  const int cw = wave & 3;
  const TileLane tl = tile_lane(cw, lane, kv_rowbytes);

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

  // -D of the lane's query row in every element: the accumulator the dP^T products start from,
  // which saves the subtraction per score
  f32x16 negD;
#pragma unroll
  for (int j = 0; j < 16; ++j) negD[j] = -Dr;
  f32x16 dqT[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) dqT[i][j] = 0.f;
  const float c2 = p.scale * LOG2E;

  const int k_end = p.causal ? min(p.s_k, q0 + BM) : p.s_k;
  const int ntiles = (k_end + BN - 1) / BN;

  // K/V tiles go from global memory straight into LDS; key rows past s_k are clamped to the last
  // row and masked below.  Tile t + 1 is on its way while tile t is computed on.
  if (NW == 4 || wave < 4) tile_dma(kg, kv_rowbytes, 0, p.s_k - 1, tl, smem, cw, lane);
  if (NW == 4 || wave >= 4) tile_dma(vg, kv_rowbytes, 0, p.s_k - 1, tl, smem + TILE_BYTES, cw, lane);
  lds_dma_wait();
  __syncthreads();

  for (int it = 0; it < ntiles; ++it) {
    const int k0 = it * BN;
    const char* Ks = smem + (it & 1) * 2 * TILE_BYTES;
    const char* Vs = Ks + TILE_BYTES;
    // The next K and V tiles into the other buffer, their pieces spread between the MFMAs below
    // (issued in a burst they stall the wavefront while the memory pipe takes them in).  After the
    // last tile the same tile goes once more into the idle buffer, which keeps the loop free of
    // branches around the copies.
    const int kn0 = it + 1 < ntiles ? k0 + BN : k0;
    const char* Kn = smem + ((it + 1) & 1) * 2 * TILE_BYTES;
    // ck: the pieces issued under the first 32 keys, cv: those under the second 32 (NW == 4: K and V;
    // NW == 8: this wavefront's one tile under the first, nothing under the second)
    const bool v_wave = NW == 8 && wave >= 4;
    const TileCopy ck = tile_copy_plan(v_wave ? vg : kg, kv_rowbytes, kn0, p.s_k - 1, tl,
                                       v_wave ? Kn + TILE_BYTES : Kn, cw, lane);
    const TileCopy cv = tile_copy_plan(vg, kv_rowbytes, kn0, p.s_k - 1, tl, Kn + TILE_BYTES, cw, lane);

    const bool active = !(p.causal && k0 > q0w + 31);
    if (!active) {      // nothing to compute for this wavefront's rows: only its share of the copies
      tile_copy_piece<0>(ck); tile_copy_piece<1>(ck); tile_copy_piece<2>(ck); tile_copy_piece<3>(ck);
      if (cw == 0) tile_copy_piece<4>(ck);
      if (NW == 4) {
        tile_copy_piece<0>(cv); tile_copy_piece<1>(cv); tile_copy_piece<2>(cv); tile_copy_piece<3>(cv);
        if (cw == 0) tile_copy_piece<4>(cv);
      }
    }
    if (active) {
      const bool need_mask = (k0 + BN > p.s_k) || (p.causal && k0 + BN - 1 > q0w);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        // S^T = K Q^T, dP^T = V dO^T for 32 keys; row reads run 4 steps ahead
        bf16x8 ka[4], va[4];
        f32x16 s, dp;
#pragma unroll
        for (int j = 0; j < 16; ++j) s[j] = 0.f;
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
          dp = mfma32(va[ks & 3], gB[ks], ks == 0 ? negD : dp);      // the chain starts from -D
          if (NW == 4 || nb == 0) {   // one piece of the next tiles every other step
            const TileCopy& c = nb == 0 ? ck : cv;
            if (ks == 0) tile_copy_piece<0>(c);
            if (ks == 2) tile_copy_piece<1>(c);
            if (ks == 4) tile_copy_piece<2>(c);
            if (ks == 6) tile_copy_piece<3>(c);
          }
          if (ks < 4) {
            const int off = a_base + nb * 32 * kRowBytes + (ks + 4) * 32;
            ka[ks & 3] = lds_read_b128(Ks, off);
            va[ks & 3] = lds_read_b128(Vs, off);
          }
          DFA_SCHED_FENCE();
        }
        // dS^T = P^T o (dP^T - D): lse' is a per-lane scalar here, -D came in through the accumulator
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const float pr = __builtin_amdgcn_exp2f(fmaf(s[j], c2, -Lr));
          dp[j] = pr * dp[j];
        }
        if (need_mask) {
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const int kvi = k0 + nb * 32 + (j >> 2) * 8 + hh * 4 + (j & 3);
            if (kvi >= p.s_k || (p.causal && kvi > qrow)) dp[j] = 0.f;
          }
        }
        if (cw == 0 && (NW == 4 || nb == 0)) tile_copy_piece<4>(nb == 0 ? ck : cv);
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
    lds_dma_wait();
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
    const size_t smem = kv::SMEM_BYTES;
    // > 64 KB of dynamic LDS needs the opt-in, once per process (thread-safe)
    static std::once_flag once;
    static int attr_rc = DFA_OK;
    std::call_once(once, [smem] {
      for (const void* f : {reinterpret_cast<const void*>(kv::k_bwd_dkdv_bf16<false>),
                            reinterpret_cast<const void*>(kv::k_bwd_dkdv_bf16<true>)}) {
        const int rc = hip_status(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                      static_cast<int>(smem)));
        if (rc) attr_rc = rc;
      }
    });
    if (attr_rc) return attr_rc;
    if (sh.s_q % kv::BM == 0) kv::k_bwd_dkdv_bf16<false><<<a.per_xcd * 8, kv::NT, smem, st>>>(a);
    else kv::k_bwd_dkdv_bf16<true><<<a.per_xcd * 8, kv::NT, smem, st>>>(a);
    const int rc = last_launch_status();
    if (rc) return rc;
  }
  if (dq) {  // dQ
    BwdParams b = p;
    const size_t smem = 4 * qs::TILE_BYTES;
    static std::once_flag once;
    static int attr_rc = DFA_OK;
    std::call_once(once, [smem] {
      for (const void* f : {reinterpret_cast<const void*>(qs::k_bwd_dq_bf16<4>),
                            reinterpret_cast<const void*>(qs::k_bwd_dq_bf16<8>)}) {
        const int rc = hip_status(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                      static_cast<int>(smem)));
        if (rc) attr_rc = rc;
      }
    });
    if (attr_rc) return attr_rc;
    // 256-row workgroups for long unmasked chunks (at least four of them per CU), 128 rows otherwise
    const bool wide = !sh.causal && static_cast<int64_t>(sh.h_q) * ((sh.s_q + 255) / 256) >= 1024;
    const int bm = wide ? 256 : 128;
    b.ntile = (sh.s_q + bm - 1) / bm;
    const int64_t total = static_cast<int64_t>(b.ntile) * sh.h_q;
    if (total > (1 << 30)) return DFA_ERR_SHAPE;
    b.total = static_cast<int>(total);
    b.per_xcd = (b.total + 7) / 8;
    if (wide) qs::k_bwd_dq_bf16<8><<<b.per_xcd * 8, 512, smem, st>>>(b);
    else qs::k_bwd_dq_bf16<4><<<b.per_xcd * 8, 256, smem, st>>>(b);
  }
  return last_launch_status();
}

}  // namespace dfa
