// bf16 forward chunk kernel for gfx950: attn(q_p, k_r, v_r) of one chunk pair from the empty
// state (forward pseudo-code of Appendix A; Eq. 1 restricted to one key/value chunk).
//
// Work decomposition.  A workgroup of 4 wavefronts owns 128 query rows of one head, each
// wavefront 32 of them, and walks over the key/value chunk in tiles of 64 rows staged in LDS.
// Per tile a wavefront computes S^T = K Q^T (keys x queries) so that every lane holds 32
// scores of ONE query: the running row maximum / row sum of the online softmax are then
// per-lane scalars plus one exchange between lane l and l+32.  The exponentiated tile is fed
// straight back, from registers, as the B operand of O^T += V^T P^T.
// Q stays in registers for the whole kernel; K/V tiles are copied from global memory straight
// into LDS (double-buffered); K is read from LDS with ds_read_b128, V with the transposing
// ds_read_b64_tr_b16.  The causal mask is applied only on tiles that straddle the
// diagonal; tiles above it are skipped.
#include <mutex>
#include <type_traits>

#include "dfa_internal.h"
#include "dfa_mfma.h"

namespace dfa {
namespace {

constexpr int D = 128;
constexpr int BM = 128;     // query rows per workgroup
constexpr int BN = 64;      // key rows per LDS tile
constexpr int NTHREADS = 256;
constexpr int TILE_BYTES = BN * kRowBytes;   // rows padded to 272 B
constexpr float LOG2E = 1.4426950408889634f;

struct FwdParams {
  const __bf16 *q, *k, *v;
  void* o; float* lse;
  int s_q, s_k, h_q, group, causal, o_bf16, accumulate, ntq, total, per_xcd;
  float scale;
  int64_t q_sh, q_ss, kv_sh, kv_ss, o_sh, o_ss, l_sh;
};

__global__ void __launch_bounds__(NTHREADS, 2) k_fwd_bf16(FwdParams p) {
  extern __shared__ __align__(16) char smem[];   // two (K tile, V tile) buffers

  // XCD-aware mapping: consecutive workgroup ids go round-robin over the 8 XCDs, so give every
  // XCD a contiguous range of (head, query tile) items; its workgroups then share K/V in its L2.
  const int bid = blockIdx.x;
  const int item = (bid & 7) * p.per_xcd + (bid >> 3);
  if (item >= p.total) return;
  const int head = item / p.ntq;
  int tq = item % p.ntq;
  if (p.causal) tq = p.ntq - 1 - tq;      // longest rows first
  const int kh = head / p.group;
  const int q0 = tq * BM;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps tile branches scalar
  const int r32 = lane & 31, hh = lane >> 5;
  const int q0w = q0 + wave * 32;
  const int qrow = q0w + r32;
  const bool qvalid = qrow < p.s_q;
  const int a_base = tile_off(r32, hh);     // per-lane LDS bases; the rest of every address is constant
  const int g_base = gather_base(lane);

  const char* kg = reinterpret_cast<const char*>(p.k + kh * p.kv_sh);
  const char* vg = reinterpret_cast<const char*>(p.v + kh * p.kv_sh);
  const uint32_t kv_rowbytes = static_cast<uint32_t>(p.kv_ss) * 2;
  const TileLane tl = tile_lane(wave, lane, kv_rowbytes);

  // Q^T operand: lane holds Q[qrow][16 ks + 8 hh .. +7]
  bf16x8 qreg[8];
  {
    const __bf16* qp = p.q + head * p.q_sh + static_cast<int64_t>(qrow) * p.q_ss + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (qvalid) raw = *reinterpret_cast<const uint4*>(qp + 16 * ks);
      qreg[ks] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  f32x16 o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) o[i][j] = 0.f;
  float m_run = -INFINITY;     // running maximum of the raw scores q.k
  float l_run = 0.f;           // this lane's half of the running row sum
  const float c2 = p.scale * LOG2E;
  if (p.accumulate && qvalid) {
    // State of the earlier key/value chunks: the normalised output with its logsumexp is the
    // running (o, m, l) with m = lse (in raw-score units: lse / scale) and l = 1.
    const float L = p.lse[head * p.l_sh + qrow];
    if (L > -INFINITY) {
      m_run = L / p.scale;
      l_run = hh == 0 ? 1.f : 0.f;
      const int64_t obase = head * p.o_sh + static_cast<int64_t>(qrow) * p.o_ss;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int col = db * 32 + g4 * 8 + hh * 4;
          if (p.o_bf16) {
            const bf16x4 b = *reinterpret_cast<const bf16x4*>(static_cast<const __bf16*>(p.o) + obase + col);
#pragma unroll
            for (int e = 0; e < 4; ++e) o[db][g4 * 4 + e] = static_cast<float>(b[e]);
          } else {
            const float4 x = *reinterpret_cast<const float4*>(static_cast<const float*>(p.o) + obase + col);
            o[db][g4 * 4] = x.x; o[db][g4 * 4 + 1] = x.y; o[db][g4 * 4 + 2] = x.z; o[db][g4 * 4 + 3] = x.w;
          }
        }
    }
  }

  const int k_end = p.causal ? min(p.s_k, q0 + BM) : p.s_k;
  const int ntiles = (k_end + BN - 1) / BN;

  // K/V tiles go from global memory straight into LDS; key rows past s_k are clamped to the last
  // row and masked below.  Tile t + 1 is on its way while tile t is computed on.
  tile_dma(kg, kv_rowbytes, 0, p.s_k - 1, tl, smem, wave, lane);
  tile_dma(vg, kv_rowbytes, 0, p.s_k - 1, tl, smem + TILE_BYTES, wave, lane);
  lds_dma_wait();
  __syncthreads();

  // Online softmax of one 32-key block (exp2 domain, scores scaled by scale*log2 e), with a lazy
  // running maximum: the reference maximum m_run only moves when some row's block maximum exceeds
  // it by more than 2^8 in the exp2 domain (or on the first block).  Until then exponentials are
  // taken against the stale maximum - they stay below 2^8, harmless in fp32 / bf16 - and O needs
  // no rescaling; the final division by the row sum makes the result independent of the reference.
  // Returns the factor O has to be multiplied by (1 when the reference did not move).
  auto softmax_block = [&](f32x16& s) {
    float mx = fmaxf(fmaxf(s[0], s[1]), s[2]);
#pragma unroll
    for (int j = 3; j < 15; j += 2) mx = fmaxf(fmaxf(mx, s[j]), s[j + 1]);
    mx = fmaxf(mx, s[15]);
    float alpha = 1.f;
    if (__any((mx - m_run) * c2 > 8.f)) {          // -inf reference (first block) also lands here
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);
      const float mc_new = (m_new == -INFINITY) ? 0.f : m_new * c2;
      alpha = __builtin_amdgcn_exp2f(m_run * c2 - mc_new);
      m_run = m_new;
      l_run *= alpha;
    }
    const float mc = (m_run == -INFINITY) ? 0.f : m_run * c2;
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float e = __builtin_amdgcn_exp2f(fmaf(s[j], c2, -mc));
      s[j] = e;
      sum += e;
    }
    l_run += sum;
    return alpha;
  };
  auto rescale_o = [&](float alpha) {
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[i][j] *= alpha;
    }
  };
  auto mask_block = [&](f32x16& s, int kbase) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int kvi = kbase + (j >> 2) * 8 + hh * 4 + (j & 3);
      if (kvi >= p.s_k || (p.causal && kvi > qrow)) s[j] = -INFINITY;
    }
  };

  for (int it = 0; it < ntiles; ++it) {
    const int k0 = it * BN;
    const bool more = it + 1 < ntiles;
    const int boff = (it & 1) * 2 * TILE_BYTES;
    const char* Ks = smem + boff;
    const char* Vs = Ks + TILE_BYTES;
    // The next K and V tiles into the other buffer, their pieces issued one at a time between the
    // MFMAs of stages 1 and 4 (in a burst they stall the wavefront while the memory pipe takes them
    // in).  After the last tile the same tile goes once more into the idle buffer: no branch
    // around the copies.
    const char* Kn = smem + (2 * TILE_BYTES - boff);
    const int kn0 = more ? k0 + BN : k0;
    const TileCopy ck = tile_copy_plan(kg, kv_rowbytes, kn0, p.s_k - 1, tl, Kn, wave, lane);
    const TileCopy cv = tile_copy_plan(vg, kv_rowbytes, kn0, p.s_k - 1, tl, Kn + TILE_BYTES, wave, lane);

    const bool active = !(p.causal && k0 > q0w + 31);
    if (!active) {      // nothing to compute for this wavefront's rows: only its share of the copies
      tile_copy_piece<0>(ck); tile_copy_piece<1>(ck); tile_copy_piece<2>(ck); tile_copy_piece<3>(ck);
      tile_copy_piece<0>(cv); tile_copy_piece<1>(cv); tile_copy_piece<2>(cv); tile_copy_piece<3>(cv);
      if (wave == 0) { tile_copy_piece<4>(ck); tile_copy_piece<4>(cv); }
    }
    if (active) {
      const bool need_mask = (k0 + BN > p.s_k) || (p.causal && k0 + BN - 1 > q0w);
      // Software pipeline over the two 32-key blocks of the tile: the MFMAs of one block run
      // under the softmax arithmetic of the other; LDS operand reads run ahead of their MFMAs.
      bf16x8 ka[4], gv[2], pb0[2], pb1[2];
      f32x16 s0, s1;
#pragma unroll
      for (int j = 0; j < 16; ++j) { s0[j] = 0.f; s1[j] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) ka[ks] = lds_read_b128(Ks, a_base + ks * 32);
      DFA_SCHED_FENCE();
      // stage 1: S0^T = K0 Q^T
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        s0 = mfma32(ka[ks & 3], qreg[ks], s0);
        ka[ks & 3] = lds_read_b128(Ks, ks < 4 ? a_base + (ks + 4) * 32 : a_base + 32 * kRowBytes + (ks - 4) * 32);
        if (ks == 0) tile_copy_piece<0>(ck);
        if (ks == 2) tile_copy_piece<1>(ck);
        if (ks == 4) tile_copy_piece<2>(ck);
        if (ks == 6) tile_copy_piece<3>(ck);
        DFA_SCHED_FENCE();
      }
      if (wave == 0) { tile_copy_piece<4>(ck); tile_copy_piece<4>(cv); }
      if (need_mask) mask_block(s0, k0);
      DFA_SCHED_FENCE();
      // stage 2: S1^T = K1 Q^T  ||  softmax of block 0
      float alpha0;
      {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          s1 = mfma32(ka[ks & 3], qreg[ks], s1);
          if (ks < 4) ka[ks & 3] = lds_read_b128(Ks, a_base + 32 * kRowBytes + (ks + 4) * 32);
        }
        gv[0] = lds_gather(Vs, g_base);
        gv[1] = lds_gather(Vs, g_base + 64);
        alpha0 = softmax_block(s0);
        pb0[0] = pack8(s0, 0); pb0[1] = pack8(s0, 8);
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
          __builtin_amdgcn_sched_group_barrier(0x002, 9, 0);   // 9 VALU
        }
      }
      DFA_SCHED_FENCE();
      rescale_o(alpha0);
      if (need_mask) mask_block(s1, k0 + 32);
      DFA_SCHED_FENCE();
      // stage 3: O^T += V0^T P0^T  ||  softmax of block 1
      float alpha1;
      {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          o[i & 3] = mfma32(gv[i & 1], pb0[i >> 2], o[i & 3]);
          const int n = i + 2;    // next gather: block 0 second half, then block 1
          gv[i & 1] = lds_gather(Vs, g_base + (n >> 2) * 16 * kRowBytes + (n & 3) * 64);
        }
        alpha1 = softmax_block(s1);
        pb1[0] = pack8(s1, 0); pb1[1] = pack8(s1, 8);
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 9, 0);
        }
      }
      DFA_SCHED_FENCE();
      rescale_o(alpha1);
      DFA_SCHED_FENCE();
      // stage 4: O^T += V1^T P1^T
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        o[i & 3] = mfma32(gv[i & 1], pb1[i >> 2], o[i & 3]);
        if (i + 2 < 8) {
          const int n = i + 10;
          gv[i & 1] = lds_gather(Vs, g_base + (n >> 2) * 16 * kRowBytes + (n & 3) * 64);
        }
        if (i == 0) tile_copy_piece<0>(cv);
        if (i == 2) tile_copy_piece<1>(cv);
        if (i == 4) tile_copy_piece<2>(cv);
        if (i == 6) tile_copy_piece<3>(cv);
        DFA_SCHED_FENCE();
      }
    }
    lds_dma_wait();
    __syncthreads();
  }

  // epilogue: combine the two half-sums, normalise, write O and the logsumexp
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (qvalid) {
    if (hh == 0) p.lse[head * p.l_sh + qrow] = l_tot > 0.f ? m_run * p.scale + logf(l_tot) : -INFINITY;
    const int64_t obase = head * p.o_sh + static_cast<int64_t>(qrow) * p.o_ss;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = db * 32 + g4 * 8 + hh * 4;
        const float x0 = o[db][g4 * 4 + 0] * inv, x1 = o[db][g4 * 4 + 1] * inv;
        const float x2 = o[db][g4 * 4 + 2] * inv, x3 = o[db][g4 * 4 + 3] * inv;
        if (p.o_bf16) {
          bf16x4 b; b[0] = static_cast<__bf16>(x0); b[1] = static_cast<__bf16>(x1);
          b[2] = static_cast<__bf16>(x2); b[3] = static_cast<__bf16>(x3);
          *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.o) + obase + col) = b;
        } else {
          *reinterpret_cast<float4*>(static_cast<float*>(p.o) + obase + col) = make_float4(x0, x1, x2, x3);
        }
      }
  }
}

// ============================================================================================
// Wavefront-specialised forward for full (unmasked) pairs: 16 wavefronts on 256 query rows, four
// per SIMD.
//   8 "S" wavefronts (32 query rows each, Q^T in registers): S^T = K Q^T, online softmax (one
//     reference update per 64-key tile), and the exponentiated tile P^T handed over through LDS as
//     bf16 together with the factor by which the running maximum moved; wavefronts 0-3 also issue
//     the global -> LDS copies of the K tiles, 4-7 those of the V tiles;
//   8 "PV" wavefronts (the same 32 rows each): O^T = O^T * factor + V^T P^T, one tile behind their
//     S wavefront, so one barrier per tile suffices; with only O^T to hold they read V^T six steps
//     ahead of their MFMAs.
// A wavefront overlaps nothing with itself (measured), different wavefronts of a SIMD do: here the
// exponentials of two S wavefronts run under the MFMAs of all four.  Measured against the
// 4-wavefront kernel above: 10 % faster on a 4096 x 4096 pair in spite of a lower clock under
// load (1.8 GHz); 5 % slower on the causal diagonal pair (256-row granularity), which therefore
// stays with the kernel above.
// ============================================================================================
namespace full_pair {

constexpr int NT = 1024;
constexpr int BMW = 256;                       // query rows per workgroup
constexpr int PX_BYTES = 8 * 4096;             // P^T hand-over: 8 query blocks x (64 keys x 32 queries bf16)
constexpr int AL_BYTES = 8 * 32 * 4;           // rescale factor per query row
// LDS map.  Tile t: K slot t % 2, V slot t % 3, P^T / factor slot t % 2; row statistics at the end.
constexpr int OFF_K = 0;
constexpr int OFF_V = OFF_K + 2 * TILE_BYTES;
constexpr int OFF_PX = OFF_V + 3 * TILE_BYTES;
constexpr int OFF_AL = OFF_PX + 2 * PX_BYTES;
constexpr int OFF_ST = OFF_AL + 2 * AL_BYTES;  // 1 / row sum, written once by the S wavefronts
constexpr int SMEM_BYTES = OFF_ST + AL_BYTES;

// RAGGED: s_k is no multiple of the 64-row tile, so the last K/V tile has rows past the end.
template <bool RAGGED>
__global__ void __launch_bounds__(NT, 1) k_fwd_bf16(FwdParams p) {
  extern __shared__ __align__(16) char smem[];

  const int bid = blockIdx.x;
  const int item = (bid & 7) * p.per_xcd + (bid >> 3);   // contiguous (head, query tile) range per XCD
  if (item >= p.total) return;
  const int head = item / p.ntq;
  int tq = item % p.ntq;
  if (p.causal) tq = p.ntq - 1 - tq;      // longest rows first
  const int kh = head / p.group;
  const int q0 = tq * BMW;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: role branches stay scalar
  const bool pv_wave = wave >= 8;
  const int r32 = lane & 31, hh = lane >> 5;
  const float c2 = p.scale * LOG2E;

  const int k_end = p.causal ? min(p.s_k, q0 + BMW) : p.s_k;
  const int ntiles = (k_end + BN - 1) / BN;

  if (!pv_wave) {
    // ------------------------------------------------------------------ S wavefront
    const int q0w = q0 + wave * 32;
    const int qrow = q0w + r32;
    const bool qvalid = qrow < p.s_q;
    const int a_base = tile_off(r32, hh);
    bf16x8 qreg[8];      // Q^T operand: lane holds Q[qrow][16 ks + 8 hh .. +7]
    {
      const __bf16* qp = p.q + head * p.q_sh + static_cast<int64_t>(qvalid ? qrow : 0) * p.q_ss + 8 * hh;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        uint4 raw = *reinterpret_cast<const uint4*>(qp + 16 * ks);
        if (!qvalid) raw = make_uint4(0, 0, 0, 0);
        qreg[ks] = __builtin_bit_cast(bf16x8, raw);
      }
    }
    float m_run = -INFINITY;     // running maximum of the raw scores q.k
    float l_run = 0.f;           // this lane's half of the running row sum
    if (p.accumulate && qvalid) {
      // state of the earlier key/value chunks: running (o, m, l) with m = lse (raw-score units), l = 1
      const float L = p.lse[head * p.l_sh + qrow];
      if (L > -INFINITY) { m_run = L / p.scale; l_run = hh == 0 ? 1.f : 0.f; }
    }
    float* al = reinterpret_cast<float*>(smem + OFF_AL) + wave * 32 + r32;
    // the S wavefronts (registers to spare) issue the global -> LDS copies of the K/V tiles
    const char* kg = reinterpret_cast<const char*>(p.k + kh * p.kv_sh);
    const char* vg = reinterpret_cast<const char*>(p.v + kh * p.kv_sh);
    const uint32_t kv_rowbytes = static_cast<uint32_t>(p.kv_ss) * 2;
    const TileLane tl = tile_lane(wave & 3, lane, kv_rowbytes);
    const char* cg = wave < 4 ? kg : vg;      // wavefronts 0-3 copy K tiles, 4-7 V tiles
    const int last = p.s_k - 1;
    tile_dma(cg, kv_rowbytes, 0, last, tl, wave < 4 ? smem + OFF_K : smem + OFF_V, wave & 3, lane);
    lds_dma_wait();
    __syncthreads();                         // tile 0 is in LDS
    for (int it = 0; it < ntiles; ++it) {
      const int k0 = it * BN;
      const char* Ks = smem + OFF_K + (it & 1) * TILE_BYTES;
      // This wavefront's pieces of the next K (or V) tile, issued one at a time between the MFMAs
      // below: in a burst they would stall it while the memory pipe takes them in.  After the last
      // tile the same tile goes once more into a ring slot nobody reads (no branch around the copies).
      const TileCopy cn = tile_copy_plan<RAGGED>(cg, kv_rowbytes, it + 1 < ntiles ? k0 + BN : k0, last, tl,
                                         wave < 4 ? smem + OFF_K + ((it + 1) & 1) * TILE_BYTES
                                                  : smem + OFF_V + ((it + 1) % 3) * TILE_BYTES,
                                         wave & 3, lane);
      const bool active = !(p.causal && k0 > q0w + 31);   // else: the whole tile lies above this block's diagonal
      if (!active) {
        tile_copy_piece<0>(cn); tile_copy_piece<1>(cn); tile_copy_piece<2>(cn); tile_copy_piece<3>(cn);
        if ((wave & 3) == 0) tile_copy_piece<4>(cn);
      }
      if (active) {
        f32x16 s0, s1;
        // S^T = K Q^T of the tile's two 32-key blocks.  COPIES: this wavefront's pieces of the next
        // tile's copy go out between the MFMAs (false when the products are done a second time).
        auto s_products = [&](auto copies) {
          constexpr bool COPIES = decltype(copies)::value;
          bf16x8 x0[4], x1[4];
          f32x16 zero;
#pragma unroll
          for (int j = 0; j < 16; ++j) zero[j] = 0.f;
#pragma unroll
          for (int ks = 0; ks < 3; ++ks) {
            x0[ks] = lds_read_b128(Ks, a_base + ks * 32);
            x1[ks] = lds_read_b128(Ks, a_base + 32 * kRowBytes + ks * 32);
          }
          DFA_SCHED_FENCE();
          __builtin_amdgcn_s_setprio(3);         // MFMAs first: the other wavefronts' VALU work fills the gaps
#pragma unroll
          for (int ks = 0; ks < 8; ++ks) {
            if (ks + 3 < 8) {
              x0[(ks + 3) & 3] = lds_read_b128(Ks, a_base + (ks + 3) * 32);
              x1[(ks + 3) & 3] = lds_read_b128(Ks, a_base + 32 * kRowBytes + (ks + 3) * 32);
            }
            s0 = mfma32(x0[ks & 3], qreg[ks], ks == 0 ? zero : s0);
            s1 = mfma32(x1[ks & 3], qreg[ks], ks == 0 ? zero : s1);
            if (COPIES) {
              if (ks == 0) tile_copy_piece<0>(cn);
              if (ks == 2) tile_copy_piece<1>(cn);
              if (ks == 4) tile_copy_piece<2>(cn);
              if (ks == 6) tile_copy_piece<3>(cn);
            }
            DFA_SCHED_FENCE();
          }
          __builtin_amdgcn_s_setprio(0);
          if (COPIES && (wave & 3) == 0) tile_copy_piece<4>(cn);
          if ((k0 + BN > p.s_k) || (p.causal && k0 + BN - 1 > q0w)) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              const int kvi = k0 + (j >> 2) * 8 + hh * 4 + (j & 3);
              if (kvi >= p.s_k || (p.causal && kvi > qrow)) s0[j] = -INFINITY;
              if (kvi + 32 >= p.s_k || (p.causal && kvi + 32 > qrow)) s1[j] = -INFINITY;
            }
          }
        };
        // Moves the reference maximum up to the tile's row maxima; returns the factor by which what
        // has been accumulated against the old reference shrinks.
        auto new_reference = [&]() {
          float mx = fmaxf(s0[0], s1[0]);
#pragma unroll
          for (int j = 1; j < 16; ++j) mx = fmaxf(fmaxf(mx, s0[j]), s1[j]);
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          const float m_new = fmaxf(m_run, mx);
          const float mc_new = (m_new == -INFINITY) ? 0.f : m_new * c2;
          const float a = __builtin_amdgcn_exp2f(m_run * c2 - mc_new);
          m_run = m_new;
          l_run *= a;
          return a;
        };
        // P^T = exp2(S^T c - reference) rounded to bf16, and this lane's half of the tile's row sum, taken
        // over the ROUNDED values (v_dot2c_f32_bf16 against a pair of ones: one instruction per two
        // scores), so that the sum that normalises O is the sum of exactly the weights that multiply V.
        bf16x8 p0, p1, p2, p3;
        auto exponentials = [&]() {
          const float mc = (m_run == -INFINITY) ? 0.f : m_run * c2;
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            s0[j] = __builtin_amdgcn_exp2f(fmaf(s0[j], c2, -mc));
            s1[j] = __builtin_amdgcn_exp2f(fmaf(s1[j], c2, -mc));
          }
          p0 = pack8(s0, 0); p1 = pack8(s0, 8); p2 = pack8(s1, 0); p3 = pack8(s1, 8);
          // two independent chains, so that the adds do not wait for one another
          const float sa = sum8(p2, sum8(p0, 0.f)), sb = sum8(p3, sum8(p1, 0.f));
          const float sum = sa + sb;
          return sum;
        };
        // Online softmax of the 64-key tile (exp2 domain) against a reference maximum that is only
        // moved when it has to be.  A tile is first exponentiated against the reference as it stands,
        // without looking for its maximum: as long as no score lies more than 2^14 above the
        // reference, the exponentials are harmless in fp32 / bf16, O needs no rescaling, and the final
        // division by the row sum removes the reference.  The reference is derived from the scores
        // themselves (row maximum, one exchange between the two half rows) on a row's first tile -
        // so the largest weight seen is at least 1 and later tiles cannot underflow the row sum - and
        // again when a tile's half-row sum shows a score far above it (or is no number): that tile's
        // products are then done once more and the tile is redone with the moved reference.
        float alpha = 1.f;
        s_products(std::true_type{});
        const bool fresh = __any(m_run == -INFINITY);
        if (fresh) alpha = new_reference();
        float sum = exponentials();
        if (!fresh && __any(!(sum <= 16384.f))) {
          s_products(std::false_type{});
          alpha = new_reference();
          sum = exponentials();
        }
        l_run += sum;
        // hand P^T and the factor to the PV wavefront: lane-private, any layout will do
        char* px = smem + OFF_PX + (it & 1) * PX_BYTES + wave * 4096 + lane * 16;
        *reinterpret_cast<bf16x8*>(px) = p0;
        *reinterpret_cast<bf16x8*>(px + 1024) = p1;
        *reinterpret_cast<bf16x8*>(px + 2048) = p2;
        *reinterpret_cast<bf16x8*>(px + 3072) = p3;
        if (hh == 0) al[(it & 1) * (AL_BYTES / 4)] = alpha;
      }
      lds_dma_wait();
      __syncthreads();
    }
    // row statistics: logsumexp to memory, 1 / row sum to the PV wavefront
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (hh == 0) {
      reinterpret_cast<float*>(smem + OFF_ST)[wave * 32 + r32] = l_tot > 0.f ? 1.f / l_tot : 0.f;
      if (qvalid) p.lse[head * p.l_sh + qrow] = l_tot > 0.f ? m_run * p.scale + logf(l_tot) : -INFINITY;
    }
    __syncthreads();                         // the PV wavefronts' last slot
  } else {
    // ------------------------------------------------------------------ PV wavefront
    const int sw = wave - 8;                 // serves S wavefront sw: the same 32 query rows
    const int q0w = q0 + sw * 32;
    const int qrow = q0w + r32;
    const bool qvalid = qrow < p.s_q;
    const int g_base = gather_base(lane);

    f32x16 o[4];         // O^T: [d block][d within block][query]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) o[i][j] = 0.f;
    if (p.accumulate && qvalid && p.lse[head * p.l_sh + qrow] > -INFINITY) {
      const int64_t obase = head * p.o_sh + static_cast<int64_t>(qrow) * p.o_ss;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int col = db * 32 + g4 * 8 + hh * 4;
          if (p.o_bf16) {
            const bf16x4 x = *reinterpret_cast<const bf16x4*>(static_cast<const __bf16*>(p.o) + obase + col);
#pragma unroll
            for (int e = 0; e < 4; ++e) o[db][g4 * 4 + e] = static_cast<float>(x[e]);
          } else {
            const float4 x = *reinterpret_cast<const float4*>(static_cast<const float*>(p.o) + obase + col);
            o[db][g4 * 4] = x.x; o[db][g4 * 4 + 1] = x.y; o[db][g4 * 4 + 2] = x.z; o[db][g4 * 4 + 3] = x.w;
          }
        }
    }
    // O^T = O^T * factor + V^T P^T for tile t (skipped when the tile lies above the block's diagonal)
    auto pv_tile = [&](int t) {
      const int k0 = t * BN;
      if (p.causal && k0 > q0w + 31) return;
      const char* Vs = smem + OFF_V + (t % 3) * TILE_BYTES;
      const char* px = smem + OFF_PX + (t & 1) * PX_BYTES + sw * 4096 + lane * 16;
      const float a = reinterpret_cast<const float*>(smem + OFF_AL)[(t & 1) * (AL_BYTES / 4) + sw * 32 + r32];
      constexpr int AHEAD = 6;               // V^T gathers run this many steps ahead of their MFMAs
      const uint32_t vb = lds_pin(lds_addr(Vs) + g_base);
      auto voff = [&](int n) {               // n = key block * 8 + half * 4 + d block
        return ((n >> 3) * 32 + ((n >> 2) & 1) * 16) * kRowBytes + (n & 3) * 64;
      };
      bf16x8 y[AHEAD + 1], pa[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) pa[j] = *reinterpret_cast<const bf16x8*>(px + j * 1024);
#pragma unroll
      for (int n = 0; n < AHEAD; ++n) y[n] = lds_gather_at(vb, voff(n));
      if (__any(a != 1.f)) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 16; ++j) o[i][j] *= a;
      }
      DFA_SCHED_FENCE();
      __builtin_amdgcn_s_setprio(3);
#pragma unroll
      for (int n = 0; n < 16; ++n) {
        if (n + AHEAD < 16) y[(n + AHEAD) % (AHEAD + 1)] = lds_gather_at(vb, voff(n + AHEAD));
        o[n & 3] = mfma32(y[n % (AHEAD + 1)], pa[n >> 2], o[n & 3]);
        DFA_SCHED_FENCE();
      }
      __builtin_amdgcn_s_setprio(0);
    };

    __syncthreads();                         // tile 0 is in LDS
    for (int it = 0; it < ntiles; ++it) {    // slot it: finish tile it - 1
      if (it > 0) pv_tile(it - 1);
      __syncthreads();
    }
    pv_tile(ntiles - 1);
    __syncthreads();                         // row statistics are in LDS

    if (qvalid) {
      const float inv = reinterpret_cast<const float*>(smem + OFF_ST)[sw * 32 + r32];
      const int64_t obase = head * p.o_sh + static_cast<int64_t>(qrow) * p.o_ss;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int col = db * 32 + g4 * 8 + hh * 4;
          const float x0 = o[db][g4 * 4 + 0] * inv, x1 = o[db][g4 * 4 + 1] * inv;
          const float x2 = o[db][g4 * 4 + 2] * inv, x3 = o[db][g4 * 4 + 3] * inv;
          if (p.o_bf16) {
            bf16x4 x; x[0] = static_cast<__bf16>(x0); x[1] = static_cast<__bf16>(x1);
            x[2] = static_cast<__bf16>(x2); x[3] = static_cast<__bf16>(x3);
            *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.o) + obase + col) = x;
          } else {
            *reinterpret_cast<float4*>(static_cast<float*>(p.o) + obase + col) = make_float4(x0, x1, x2, x3);
          }
        }
    }
  }
}

}  // namespace full_pair

}  // namespace

int launch_fwd_bf16(const dfa_shape& sh, const void* q, const void* k, const void* v,
                    void* o, float* lse, int accumulate, hipStream_t st) {
  FwdParams p{};
  p.q = static_cast<const __bf16*>(q); p.k = static_cast<const __bf16*>(k); p.v = static_cast<const __bf16*>(v);
  p.o = o; p.lse = lse;
  p.s_q = sh.s_q; p.s_k = sh.s_k; p.h_q = sh.h_q; p.group = sh.h_q / sh.h_kv; p.causal = sh.causal;
  p.o_bf16 = sh.o_dtype == DFA_BF16; p.scale = sh.scale; p.accumulate = accumulate;
  p.q_sh = sh.q_stride_h; p.q_ss = sh.q_stride_s; p.kv_sh = sh.kv_stride_h; p.kv_ss = sh.kv_stride_s;
  p.o_sh = sh.o_stride_h; p.o_ss = sh.o_stride_s; p.l_sh = sh.lse_stride_h;
  if (!sh.causal) {   // full pairs: the wavefront-specialised kernel; the diagonal pair keeps the finer 128-row tiling
    p.ntq = (sh.s_q + full_pair::BMW - 1) / full_pair::BMW;
    p.total = p.ntq * sh.h_q;
    p.per_xcd = (p.total + 7) / 8;
    // > 64 KB of dynamic LDS needs the opt-in, once per process (thread-safe)
    static std::once_flag once;
    static int attr_rc = DFA_OK;
    std::call_once(once, [] {
      for (const void* f : {reinterpret_cast<const void*>(full_pair::k_fwd_bf16<false>),
                            reinterpret_cast<const void*>(full_pair::k_fwd_bf16<true>)}) {
        const int rc = hip_status(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                      full_pair::SMEM_BYTES));
        if (rc) attr_rc = rc;
      }
    });
    if (attr_rc) return attr_rc;
    if (sh.s_k % BN == 0)
      full_pair::k_fwd_bf16<false><<<p.per_xcd * 8, full_pair::NT, full_pair::SMEM_BYTES, st>>>(p);
    else
      full_pair::k_fwd_bf16<true><<<p.per_xcd * 8, full_pair::NT, full_pair::SMEM_BYTES, st>>>(p);
    return last_launch_status();
  }
  p.ntq = (sh.s_q + BM - 1) / BM;
  const int64_t total = static_cast<int64_t>(p.ntq) * sh.h_q;
  if (total > (1 << 30)) return DFA_ERR_SHAPE;
  p.total = static_cast<int>(total);
  p.per_xcd = (p.total + 7) / 8;
  const size_t smem = 4 * TILE_BYTES;     // two (K, V) buffers; above 64 KB needs the opt-in once
  static std::once_flag once;
  static int attr_rc = DFA_OK;
  std::call_once(once, [smem] {
    attr_rc = hip_status(hipFuncSetAttribute(reinterpret_cast<const void*>(k_fwd_bf16),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem)));
  });
  if (attr_rc) return attr_rc;
  k_fwd_bf16<<<p.per_xcd * 8, NTHREADS, smem, st>>>(p);
  return last_launch_status();
}

}  // namespace dfa
