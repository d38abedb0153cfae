// Building blocks shared by the bf16 matrix-core kernels: vector types, the 32x32x16 MFMA
// wrapper, and the LDS tile layout with its global->LDS staging.
//
// MFMA v_mfma_f32_32x32x16_bf16 (one wavefront, C[32x32] += A[32x16] * B[16x32]):
//   A operand: lane L holds row (L % 32), k = (L / 32) * 8 .. +8      (8 consecutive k)
//   B operand: lane L holds col (L % 32), k = (L / 32) * 8 .. +8
//   C/D:       lane L holds col (L % 32), rows (i / 4) * 8 + (L / 32) * 4 + (i % 4), i = 0..15
// All kernels compute "transposed" products so that the index a softmax reduces over (keys
// in the forward and dQ kernels, queries in the dK/dV kernel) lies along C's rows, i.e. inside
// a lane, and so that C's register layout can be fed back as a B operand: for MFMA k-slot
// (half = L / 32, j = 0..7) of the k-step that consumes C registers 8t..8t+7, the row index is
//   16 t + (j / 4) * 8 + half * 4 + (j % 4).
// The other operand of that second product (V^T, K^T, Q^T, dO^T) is read from the natural-
// orientation tile in LDS by transposing reads that deliver exactly this permuted order (see
// TileS below), so the sum over k pairs matching rows.
#pragma once
#include "common.h"

namespace mmsp {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

__device__ __forceinline__ f32x16 mfma32(const u32x4& a, const u32x4& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ u32x4 mk4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  u32x4 r = {a, b, c, d};
  return r;
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  f32x2 x = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

constexpr int kTileBytes = 64 * 128 * 2;     // 16 KiB: one 64 x 128 bf16 tile

// ---------------------------------------------------------------------------------------
// Asynchronous global -> LDS copies (global_load_lds_dwordx4): every lane supplies its own
// global address; the 64 x 16 bytes of a wavefront land contiguously at a wavefront-uniform LDS
// address.  Completion is tracked by vmcnt.  A swizzled LDS layout is obtained by permuting
// which global chunk each lane fetches.
// ---------------------------------------------------------------------------------------
// The copy is written as inline assembly, not through the compiler's builtin, on purpose.  The
// compiler's wait-count pass treats a global->LDS copy it knows about as an access to both
// memories: while one is in flight it turns every wait for an LDS read into "wait for all LDS
// reads", which defeats reading operands several matrix instructions ahead, and it adds waits
// on the copy counter wherever it cannot tell an LDS read from a copy's target.  The pipelines
// here wait for their copies explicitly (s_waitcnt vmcnt(n) + barrier), so the compiler need
// not know.  A copy it does not count can only make its own vmcnt waits stricter than needed
// (the counter retires in order), never too weak.  M0 (the copy's LDS base) is a register the
// compiler reserves and sets itself right before each of its own uses; nothing else in these
// kernels uses it.
// `lds_array` is a __shared__ array (its LDS address is a constant the compiler folds), `byte_offset`
// a wavefront-uniform offset inside it that the caller keeps in a scalar register.
__device__ __forceinline__ uint32_t lds_address(const void* lds_array) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)lds_array;
}
// Source address = wavefront-uniform `base` (scalar register pair) + this lane's 32-bit byte `offset`.
__device__ __forceinline__ void dma16(const char* base, uint32_t offset, const void* lds_array, int byte_offset) {
  const uint32_t lds = lds_address(lds_array) + (uint32_t)byte_offset;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds), "v"(offset), "s"(base) : "memory");
}
__device__ __forceinline__ void dma4(const char* base, uint32_t offset, const void* lds_array, int byte_offset) {   // 4 bytes per lane
  const uint32_t lds = lds_address(lds_array) + (uint32_t)byte_offset;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(lds), "v"(offset), "s"(base) : "memory");
}

// Bare workgroup barrier for the asynchronous-copy pipelines.  __syncthreads() (and any
// workgroup fence) makes the compiler wait for every outstanding vmcnt operation, including
// the tile copies that are deliberately still in flight.  Here the copies a stage needs are
// awaited explicitly (s_waitcnt vmcnt(n)) before the barrier, every LDS read of the stage being
// recycled has been consumed by an MFMA issued before it, and the empty asm statements keep
// the compiler from moving memory accesses across it.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Same barrier for a wavefront that has just written LDS with ordinary ds_write instructions:
// those are tracked by lgkmcnt, which must drain before the barrier so that the other
// wavefronts see the data (vmcnt, i.e. the tile copies in flight, is left alone).
__device__ __forceinline__ void lds_barrier_after_write() {
  __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
  lds_barrier();
}

// A tile is 16 wavefront-copies of 4 rows; copy j lands rows 4j .. 4j+3.  kCopies = 16 /
// (wavefronts sharing the tile); the wavefront with index w takes copies w, w + W, ...
// Offsets are bytes from the tile's first row and fit 32 bits.
template <int kCopies>
struct DmaOffs { uint32_t o[kCopies]; };

// ---------------------------------------------------------------------------------------
// TileS: a [64 rows][128 cols] bf16 tile in its natural orientation (row = token, col = d),
// 256 bytes per row, the 16-byte chunk c of row r stored at chunk position c ^ swz16(r).
// One copy in LDS serves both operand orientations:
//   * k index along d (rows = MFMA rows): ds_read_b128 of chunk (2 ks + half) of row (lane % 32);
//     the 16 lanes of a phase read one chunk of 16 consecutive rows, and swz16 is a bijection of
//     r & 15, so they hit 16 distinct 16-byte bank groups;
//   * k index along the tokens (rows of the MFMA operand = d): two ds_read_b64_tr_b16 per
//     operand.  In each group of 16 lanes, lane a + 4 m supplies the address of 4 consecutive
//     d (8 bytes) of token row m; the instruction hands lane l of the group the element d = l
//     of the four rows m = 0..3.  The four rows of a read are 4 consecutive tokens, whose
//     swz16 values differ in bits 2..3, i.e. they lie in four different 64-byte bank groups.
// The k-slot order of the second kind follows the C layout of the first product (see the top
// of this file): for the 16 tokens 16 g .. 16 g + 15 of a tile, the lanes of half h take
// tokens 16 g + 4 h + {0..3} (first read) and 16 g + 8 + 4 h + {0..3} (second read).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int swz16(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

__device__ __forceinline__ int tile_s_offset(int row, int chunk /*0..15*/) {
  return row * 256 + ((chunk ^ swz16(row & 15)) << 4);
}

typedef short s16x4 __attribute__((__vector_size__(4 * sizeof(short))));

__device__ __forceinline__ u32x2 lds_read_tr(const char* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(u32x2, v);
}

// Byte offset, inside a TileS tile, of the address this lane supplies to the transposing read
// of d block db (32 rows of the operand), for tokens 4 h + m (sec = 0) or 8 + 4 h + m (sec = 1)
// of token group 0; token group g adds g * 4096 bytes.
__device__ __forceinline__ int tile_s_tr_offset(int lane, int db, int sec) {
  const int grp = lane >> 4, a = lane & 3, m = (lane >> 2) & 3;      // lane = 16 grp + 4 m + a
  const int h = grp >> 1, dsub = grp & 1;
  const int row = sec * 8 + h * 4 + m;
  const int chunk = db * 4 + dsub * 2 + (a >> 1);
  return tile_s_offset(row, chunk) + (a & 1) * 8;
}

// TileS by asynchronous copies: lane l of copy j fetches the logical chunk that belongs at chunk
// position l % 16 of row 4j + l / 16, i.e. chunk (l % 16) ^ swz16(row); rows past the end of the
// tensor repeat the last row.
template <int kCopies>
__device__ __forceinline__ DmaOffs<kCopies> dma_s_offsets(int64_t row_stride_elems, int rows_left, int wave, int lane) {
  constexpr int W = 16 / kCopies;
  DmaOffs<kCopies> t;
#pragma unroll
  for (int i = 0; i < kCopies; ++i) {
    const int row = 4 * (wave + i * W) + (lane >> 4);
    const int chunk = (lane & 15) ^ swz16(row & 15);
    t.o[i] = (uint32_t)(min(row, rows_left - 1) * (int)row_stride_elems * 2 + chunk * 16);
  }
  return t;
}

}  // namespace mmsp
