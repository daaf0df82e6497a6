// Building blocks for the bf16 MFMA kernels on gfx950 (CDNA4): vector types, the
// v_mfma_f32_32x32x16_bf16 wrapper with its register layouts, and the LDS tile layout.
//
// v_mfma_f32_32x32x16_bf16 computes C[32x32] += A[32x16] B[16x32] per wavefront.  With
// lane l, r = l % 32, h = l / 32:
//   A operand (8 bf16): A[r][8h .. 8h+7]         B operand (8 bf16): B[8h .. 8h+7][r]
//   C/D (16 fp32):      C[(i/4)*8 + 4h + i%4][r] for i = 0..15
// Because the contraction index only has to match between A and B, a C tile can be fed
// back as the B operand of the next product without any data movement: the 8 values
// C[.][r] with i in [8u, 8u+8) become B[8h+e][r], provided the A operand of that product is
// gathered with the same row order, rows (e/4)*8 + 4h + e%4 of the 16-row block u.
//
// LDS tiles hold rows of 128 bf16 padded to 272 bytes, and logical row r is stored at physical
// row prow(r) (a 4x4 transpose of the low four row bits).  With that, both access patterns
// used here are bank-conflict free AND every address is a per-lane base plus a compile-time
// constant: ds_read_b128 of one 16-byte chunk column from 16 consecutive logical rows (their
// physical rows are 16 distinct values mod 16, and 272 = 256 + 16), and ds_read_b64_tr_b16 of
// 4 consecutive logical rows x 64 B (their physical rows are 4 apart: 4 * 272 = 64 mod 256).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dfa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // an operand piece as raw bits (for values carried around a loop)

#define DFA_LDS __attribute__((address_space(3)))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// (Inline-assembly forms of the MFMA with operand register files fixed by hand were tried and
// dropped: hipcc places accumulator copies next to such statements without the wait states the
// hardware needs there, which gave wrong results; the builtin above is the only form used.)

#define DFA_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
// Workgroup barrier without the wait for this wavefront's outstanding memory operations that
// __syncthreads() puts in front of it.  For a wavefront that only READS shared tiles and whose
// reads still in flight target registers it consumes later (the compiler's own counters cover
// those): nothing it wrote has to be visible to the others.  The "memory" clobber keeps the
// compiler from moving memory accesses across it.
#define DFA_BARRIER_NO_DRAIN() asm volatile("s_barrier" ::: "memory")

constexpr int kRowBytes = 272;

__device__ __forceinline__ int prow(int r) { return (r & ~15) | ((r & 3) << 2) | ((r >> 2) & 3); }

// byte offset of 16-byte chunk c of logical row r
__device__ __forceinline__ int tile_off(int r, int c) { return prow(r) * kRowBytes + (c << 4); }

__device__ __forceinline__ bf16x8 lds_read_b128(const char* base, int off) {
  return *reinterpret_cast<const bf16x8*>(base + off);
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane j supplies
// the address of 4 consecutive bf16; lane i receives, for t = 0..3, element (i % 4) of the
// 4 that lane (4t + i/4) of its group addressed.
__device__ __forceinline__ bf16x4 lds_read_tr(const char* base, int off) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (DFA_LDS s16x4*)(base + off));
  return __builtin_bit_cast(bf16x4, v);
}

// Gather for an operand whose contraction runs over tile ROWS (the tile is stored row-major, so
// this is a transposed read).  gather_base(lane) is the per-lane part; lds_gather(base, off)
// with off = row0 * kRowBytes + col0 * 2 (row0 a multiple of 16, col0 a multiple of 32) returns
// the 8 values  tile[row0 + (e/4)*8 + 4h + e%4][col0 + lane%32],  e = 0..7,  h = lane/32,
// which is the row order in which an MFMA result tile is fed back as a B operand.
__device__ __forceinline__ int gather_base(int lane) {
  const int g = lane >> 4, j = lane & 15;
  return tile_off(4 * (g >> 1) + (j >> 2), 2 * (g & 1) + ((j & 3) >> 1)) + ((j & 1) << 3);
}

// The same from a 32-bit LDS address held in a register that the compiler must take as it is
// (see lds_pin): the constant part of every read then goes into the instruction's offset field.
__device__ __forceinline__ bf16x4 lds_read_tr_at(uint32_t addr, int off) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((DFA_LDS s16x4*)(addr + off));
  return __builtin_bit_cast(bf16x4, v);
}
__device__ __forceinline__ bf16x8 lds_gather_at(uint32_t addr, int off) {
  const bf16x4 lo = lds_read_tr_at(addr, off);
  const bf16x4 hi = lds_read_tr_at(addr, off + 2 * kRowBytes);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
// Makes `addr` opaque to the compiler, so that it stays THE base register of the reads that
// follow.  Left alone, the compiler may pick a base above them and spend one v_add per read on
// the (negative, not encodable) differences.
__device__ __forceinline__ uint32_t lds_pin(uint32_t addr) {
  asm volatile("" : "+v"(addr));
  return addr;
}

__device__ __forceinline__ bf16x8 lds_gather(const char* base, int off) {
  const bf16x4 lo = lds_read_tr(base, off);
  const bf16x4 hi = lds_read_tr(base, off + 2 * kRowBytes);   // logical rows +8 = physical rows +2
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// ---- global memory -> LDS tile copy without a register stop-over --------------------------
// global_load_lds_dwordx4: every lane supplies its own global address and the wavefront's
// 64 x 16 bytes land contiguously at the LDS byte address M0 + the instruction's offset.  A
// padded 64-row tile (64 x kRowBytes = 17 KB) is 17 such 1 KB pieces; of 4 copying wavefronts,
// wavefront w moves pieces 4w .. 4w+3 with ONE write of M0 (the immediate offsets 0, 1024, 2048,
// 3072 step through them; measured: 21 instead of 40 cycles of issue per copy) and wavefront 0
// also piece 16.  Byte 16 s of the tile is chunk s % 17 of physical row s / 17; chunk 16 is the
// row's pad and receives a copy of chunk 15.
//
// The copy is issued from inline assembly, so the compiler neither sees it nor waits for it:
// lds_dma_wait() before the barrier that publishes the tile is the caller's duty.  (Compiler-
// tracked loads stay correct next to it: extra loads in flight only make its waits stricter, so
// keep them before the copies in program order.)
//
// The immediate offset also moves the global address, so piece j's lane offset carries
// 3072 - 1024 j and the scalar base is taken 3072 bytes early: voff holds, per lane and piece,
// that adjusted byte offset from the tile's first row for a tile wholly inside the matrix.
struct TileLane { uint32_t voff[5]; };

__device__ __forceinline__ void tile_lane_rc(int w, int lane, int j, int& row, uint32_t& cb) {
  const int s = (j < 4 ? 4 * w + j : 16) * 64 + lane;
  row = prow(s / 17);                              // prow is its own inverse
  const int c = s % 17;
  cb = static_cast<uint32_t>(c < 15 ? c : 15) * 16;
}

__device__ __forceinline__ TileLane tile_lane(int w, int lane, uint32_t rowbytes) {
  TileLane m;
#pragma unroll
  for (int j = 0; j < 5; ++j) {
    int row; uint32_t cb;
    tile_lane_rc(w, lane, j, row, cb);
    m.voff[j] = static_cast<uint32_t>(row) * rowbytes + cb + (j < 4 ? 3072 - 1024 * j : 3072);
  }
  return m;
}

__device__ __forceinline__ uint32_t lds_addr(const char* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((DFA_LDS const char*)p));
}

// gbase and lds must be wave-uniform; v* are this lane's byte offsets from gbase.
__device__ __forceinline__ void lds_dma16(const char* gbase, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds), "v"(voff), "s"(gbase) : "memory", "m0");
}
// four consecutive 1 KB pieces at lds; piece j reads from gbase + vj + 1024 j
__device__ __forceinline__ void lds_dma16x4(const char* gbase, uint32_t v0, uint32_t v1, uint32_t v2,
                                            uint32_t v3, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
               "global_load_lds_dwordx4 %1, %5\n\t"
               "global_load_lds_dwordx4 %2, %5 offset:1024\n\t"
               "global_load_lds_dwordx4 %3, %5 offset:2048\n\t"
               "global_load_lds_dwordx4 %4, %5 offset:3072"
               :: "s"(lds), "v"(v0), "v"(v1), "v"(v2), "v"(v3), "s"(gbase) : "memory", "m0");
}

// Rows row0 .. row0 + 63 of a [rows, d = 128] bf16 matrix at gbase (row pitch rowbytes) into the
// padded LDS tile at `tile`; rows past `last` are clamped to it (callers mask them).  A tile
// inside the matrix costs no vector arithmetic: the tile's position goes into the scalar base.
__device__ __forceinline__ void tile_dma(const char* gbase, uint32_t rowbytes, int row0, int last,
                                         const TileLane& m, const char* tile, int w, int lane) {
  const uint32_t base = lds_addr(tile);
  const char* g3 = gbase - 3072;                   // see TileLane
  if (row0 + 63 <= last) {
    const char* g = g3 + static_cast<uint64_t>(static_cast<uint32_t>(row0)) * rowbytes;
    lds_dma16x4(g, m.voff[0], m.voff[1], m.voff[2], m.voff[3], base + w * 4096);
    if (w == 0) lds_dma16(g, m.voff[4], base + 16 * 1024);
  } else {
    uint32_t v[5];
#pragma unroll
    for (int j = 0; j < 5; ++j) {
      int row; uint32_t cb;
      tile_lane_rc(w, lane, j, row, cb);
      const int r = row0 + row;
      v[j] = static_cast<uint32_t>(r < last ? r : last) * rowbytes + cb + (j < 4 ? 3072 - 1024 * j : 3072);
    }
    lds_dma16x4(g3, v[0], v[1], v[2], v[3], base + w * 4096);
    if (w == 0) lds_dma16(g3, v[4], base + 16 * 1024);
  }
}

// One wavefront's share of a tile copy (pieces 4w .. 4w + 3, and piece 16 for w == 0), resolved
// to a scalar base and per-lane offsets, so that the pieces can be issued one at a time between
// other instructions: the memory pipe takes about 17 cycles per 1 KB piece and CU, and a
// wavefront that issues its pieces in a burst stalls until the pipe has taken them all.
struct TileCopy {
  const char* g;        // scalar base (taken 3072 bytes early, see TileLane)
  uint32_t v[5];        // per-lane byte offsets of the five pieces
  uint32_t lds, lds16;  // LDS addresses of piece 4w and of piece 16
};

// RAGGED false: the caller guarantees that every tile lies wholly inside the matrix.
template <bool RAGGED = true>
__device__ __forceinline__ TileCopy tile_copy_plan(const char* gbase, uint32_t rowbytes, int row0, int last,
                                                   const TileLane& m, const char* tile, int w, int lane) {
  TileCopy c;
  const uint32_t base = lds_addr(tile);
  c.lds = base + w * 4096;
  c.lds16 = base + 16 * 1024;
  const char* g3 = gbase - 3072;
  if (!RAGGED || row0 + 63 <= last) {              // tile inside the matrix: its position goes into the scalar base
    c.g = g3 + static_cast<uint64_t>(static_cast<uint32_t>(row0)) * rowbytes;
#pragma unroll
    for (int j = 0; j < 5; ++j) c.v[j] = m.voff[j];
  } else {                                         // rows past `last` are clamped to it
    c.g = g3;
#pragma unroll
    for (int j = 0; j < 5; ++j) {
      int row; uint32_t cb;
      tile_lane_rc(w, lane, j, row, cb);
      const int r = row0 + row;
      c.v[j] = static_cast<uint32_t>(r < last ? r : last) * rowbytes + cb + (j < 4 ? 3072 - 1024 * j : 3072);
    }
  }
  return c;
}

// Piece J of the plan: J = 0..3 are pieces 4w + J, J = 4 is piece 16 (issue it from one wavefront only).
template <int J>
__device__ __forceinline__ void tile_copy_piece(const TileCopy& c) {
  if constexpr (J == 0)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(c.lds), "v"(c.v[0]), "s"(c.g) : "memory", "m0");
  else if constexpr (J == 1)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:1024"
                 :: "s"(c.lds), "v"(c.v[1]), "s"(c.g) : "memory", "m0");
  else if constexpr (J == 2)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:2048"
                 :: "s"(c.lds), "v"(c.v[2]), "s"(c.g) : "memory", "m0");
  else if constexpr (J == 3)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:3072"
                 :: "s"(c.lds), "v"(c.v[3]), "s"(c.g) : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(c.lds16), "v"(c.v[4]), "s"(c.g) : "memory", "m0");
}

__device__ __forceinline__ void lds_dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// acc + the sum of the eight bf16 values of v, in fp32: v_dot2c_f32_bf16 against a pair of ones adds
// two of them per instruction.
__device__ __forceinline__ float sum8(bf16x8 v, float acc) {
  bf16x2 ones;
  ones[0] = static_cast<__bf16>(1.f); ones[1] = ones[0];
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(v, v, 0, 1), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(v, v, 2, 3), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(v, v, 4, 5), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(v, v, 6, 7), ones, acc, false);
  return acc;
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int first) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = static_cast<__bf16>(v[first + e]);
  return r;
}

}  // namespace dfa
