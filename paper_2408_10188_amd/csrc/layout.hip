// HBM-bound data movement around the attention path: the token-level "both ends" sharding of
// a whole sequence into per-rank zigzag shards (and back), and the local re-grouping of heads
// that brackets the all-to-all of the head-sharded mode.  All four are row permutations: rows
// of `row_bytes` (a multiple of 16) are copied whole with 16-byte accesses, consecutive lanes
// on consecutive 16-byte pieces, so reads and writes are fully coalesced; 1 byte read and
// 1 byte written per byte of payload.
#include "common.h"

namespace mmsp {
namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

enum PermKind { kZigzagGather = 0, kZigzagScatter = 1, kSwapOuter = 2 };

// dst row j <- src row perm(j).
//   zigzag: sequence rows are tokens; shard row j = rank * 2C + half * C + i holds token
//           chunk(rank, half) * C + i with chunk(r, 0) = r, chunk(r, 1) = 2N - 1 - r.
//           gather: dst = shards, src = sequence;  scatter: the inverse.
//   swap:   src is [A][B] rows, dst is [B][A] rows: dst row b * A + a <- src row a * B + b.
template <int KIND>
__global__ __launch_bounds__(256) void permute_rows_kernel(const char* __restrict__ src, char* __restrict__ dst,
                                                           int64_t n_rows, int vec_per_row, int64_t p0 /* C or A */,
                                                           int64_t p1 /* N or B */) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = t / vec_per_row;
  if (row >= n_rows) return;
  const int v = (int)(t - row * vec_per_row);
  int64_t src_row, dst_row;
  if (KIND == kSwapOuter) {
    const int64_t b = row / p0, a = row - b * p0;      // dst index
    dst_row = row; src_row = a * p1 + b;
  } else {
    const int64_t C = p0, N = p1;
    const int64_t seg = row / C, i = row - seg * C;    // shard-side index: seg = rank * 2 + half
    const int64_t rank = seg >> 1, half = seg & 1;
    const int64_t token = (half ? 2 * N - 1 - rank : rank) * C + i;
    if (KIND == kZigzagGather) { dst_row = row; src_row = token; } else { dst_row = token; src_row = row; }
  }
  const int64_t rb = (int64_t)vec_per_row * 16;
  *reinterpret_cast<u32x4_t*>(dst + dst_row * rb + v * 16) = *reinterpret_cast<const u32x4_t*>(src + src_row * rb + v * 16);
}

template <int KIND>
hipError_t launch(const void* src, void* dst, int64_t n_rows, int64_t row_bytes, int64_t p0, int64_t p1, hipStream_t stream) {
  const int vec = (int)(row_bytes / 16);
  const int64_t n = n_rows * vec;
  if (n == 0) return hipSuccess;
  permute_rows_kernel<KIND><<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(
      reinterpret_cast<const char*>(src), reinterpret_cast<char*>(dst), n_rows, vec, p0, p1);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_zigzag_gather(const void* seq, void* shards, int64_t T, int N, int64_t row_bytes, hipStream_t stream) {
  return launch<kZigzagGather>(seq, shards, T, row_bytes, T / (2 * (int64_t)N), N, stream);
}
hipError_t launch_zigzag_scatter(const void* shards, void* seq, int64_t T, int N, int64_t row_bytes, hipStream_t stream) {
  return launch<kZigzagScatter>(shards, seq, T, row_bytes, T / (2 * (int64_t)N), N, stream);
}
// src [A][B] rows -> dst [B][A] rows
hipError_t launch_swap_outer(const void* src, void* dst, int64_t A, int64_t B, int64_t row_bytes, hipStream_t stream) {
  return launch<kSwapOuter>(src, dst, A * B, row_bytes, A, B, stream);
}

}  // namespace mmsp
