// Building blocks shared by the bf16 matrix-core kernels: vector types, the 32x32x16 MFMA
// wrapper, and the two LDS tile layouts with their global->LDS staging.
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
// The other operand of that second product (V^T, K^T, Q^T, dO^T) is staged in LDS in exactly
// this permuted order ("TileT"), so the sum over k pairs matching rows.
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

// ---------------------------------------------------------------------------------------
// TileN: a [64 rows][128 cols] bf16 tile in its natural orientation (row = token, col = d),
// 256 bytes per row, 16-byte chunks XOR-swizzled by (row & 15) so that the 16 lanes of a
// ds_read_b128 phase, which read the same chunk of 16 consecutive rows, hit distinct banks.
// Used as an MFMA A operand whose k index runs along d.
// ---------------------------------------------------------------------------------------
constexpr int kTileBytes = 64 * 128 * 2;     // 16 KiB, both layouts

__device__ __forceinline__ int tile_n_offset(int row, int chunk /*0..15*/) {
  return row * 256 + ((chunk ^ (row & 15)) << 4);
}

// ---------------------------------------------------------------------------------------
// TileT: the same 64x128 tile transposed, [128 d][64 token slots].  Token t of the tile sits
// in slot (t & ~15) | swap_bits_2_3(t & 15), which is the k-slot order described above.
// Rows 2j and 2j+1 share one 256-byte bank line; which half a row takes is flipped by bit 3
// of d, and the 16-byte chunks inside the half are XOR-swizzled by (d >> 4) ^ (d >> 1).  With
// this placement both the b128 operand reads (32 consecutive d, one chunk) and the b64
// transposing writes (d = 8 * lane + e, see tile_store_t) touch every bank equally often.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int tile_t_offset(int d, int chunk /*0..7*/) {
  return (d >> 1) * 256 + (((d ^ (d >> 3)) & 1) << 7) + (((chunk ^ (d >> 4) ^ (d >> 1)) & 7) << 4);
}

// Staging registers for one 64x128 tile and 256 threads: thread t owns the token group
// kg = stage_kg(t) (tokens 4kg .. 4kg+3) and d-chunk (t%16)*8 .. +8  ->  four 16-byte global
// loads, each row of the tile being read by 16 consecutive lanes (256 contiguous bytes).
// Within a wavefront the 16-lane groups take token groups 0, 2, 1, 3 so that the first 32
// lanes of a transposing b64 write differ in the 8-byte half of a chunk, not in the chunk.
struct TileRegs { u32x4 r[4]; };

__device__ __forceinline__ int stage_kg(int tid) {
  return (tid >> 6) * 4 + ((tid >> 4) & 1) * 2 + ((tid >> 5) & 1);
}

// rows are clamped to [0, n_rows-1] so that every load is in bounds; clamped duplicates are
// masked (or never stored) by the caller.
__device__ __forceinline__ void tile_load(TileRegs& t, const uint16_t* base, int64_t row_stride, int row0, int n_rows,
                                          int tid) {
  const int tok = stage_kg(tid) * 4, dc = tid & 15;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = min(row0 + tok + r, n_rows - 1);
    t.r[r] = *reinterpret_cast<const u32x4*>(base + (int64_t)row * row_stride + dc * 8);
  }
}

__device__ __forceinline__ uint32_t comp(const u32x4& v, int i) { return v[i]; }   // i constant after unrolling

__device__ __forceinline__ void tile_store_t(const TileRegs& t, char* tile, int tid) {
  const int kg = stage_kg(tid), dc = tid & 15;
  // tokens 4kg..4kg+3: 16-group g16 = kg/4, offset bits (b3,b2) = ((kg%4)>>1, (kg%4)&1);
  // slot = b2*8 + b3*4 + (0..3)  ->  chunk = g16*2 + b2, byte offset inside the chunk = b3*8
  const int chunk = (kg >> 2) * 2 + (kg & 1);
  const int sub = ((kg >> 1) & 1) * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int d = dc * 8 + e;
    const int wi = e >> 1;
    u32x2 out;
    if (e & 1) {   // high halves
      out.x = __builtin_amdgcn_perm(comp(t.r[1], wi), comp(t.r[0], wi), 0x07060302u);
      out.y = __builtin_amdgcn_perm(comp(t.r[3], wi), comp(t.r[2], wi), 0x07060302u);
    } else {       // low halves
      out.x = __builtin_amdgcn_perm(comp(t.r[1], wi), comp(t.r[0], wi), 0x05040100u);
      out.y = __builtin_amdgcn_perm(comp(t.r[3], wi), comp(t.r[2], wi), 0x05040100u);
    }
    *reinterpret_cast<u32x2*>(tile + tile_t_offset(d, chunk) + sub) = out;
  }
}

// ---------------------------------------------------------------------------------------
// Asynchronous global -> LDS copies (global_load_lds_dwordx4): every lane supplies its own
// global address; the 64 x 16 bytes of a wavefront land contiguously at a wavefront-uniform LDS
// address.  Completion is tracked by vmcnt.  A swizzled LDS layout is obtained by permuting
// which global chunk each lane fetches.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void dma16(const char* gptr, char* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
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

// TileN by DMA: the tile is 16 wavefront-copies of 4 rows; copy j of a wavefront lands rows
// 4j .. 4j+3.  Lane l of copy j fetches logical chunk (l % 16) ^ (row & 15) of row 4j + l/16.
// kCopies = 16 / (wavefronts sharing the tile); the wavefront with index w takes copies
// w, w + W, ...  Offsets are bytes from the tile's first row and fit 32 bits.
template <int kCopies>
struct DmaOffs { uint32_t o[kCopies]; };

template <int kCopies>
__device__ __forceinline__ DmaOffs<kCopies> dma_n_offsets(int64_t row_stride_elems, int rows_left, int wave, int lane) {
  constexpr int W = 16 / kCopies;
  DmaOffs<kCopies> t;
#pragma unroll
  for (int i = 0; i < kCopies; ++i) {
    const int row = 4 * (wave + i * W) + (lane >> 4);
    const int chunk = (lane & 15) ^ (row & 15);
    t.o[i] = (uint32_t)(min(row, rows_left - 1) * (int)row_stride_elems * 2 + chunk * 16);
  }
  return t;
}

template <int kCopies>
__device__ __forceinline__ void dma_tile_n(const char* tile_ptr /* uniform */, const DmaOffs<kCopies>& off, char* lds_tile,
                                           int wave) {
  constexpr int W = 16 / kCopies;
#pragma unroll
  for (int i = 0; i < kCopies; ++i) dma16(tile_ptr + off.o[i], lds_tile + (wave + i * W) * 1024);
}

// A pre-built 16 KiB LDS image (see transpose_tiles) copied verbatim.
template <int kCopies>
__device__ __forceinline__ void dma_tile_image(const char* image /* uniform */, char* lds_tile, int wave, int lane) {
  constexpr int W = 16 / kCopies;
#pragma unroll
  for (int i = 0; i < kCopies; ++i) dma16(image + (wave + i * W) * 1024 + lane * 16, lds_tile + (wave + i * W) * 1024);
}

}  // namespace mmsp
