// Pre-transposition of 64-row tiles into ready-made LDS images.  Every product that contracts
// over tokens (P.V, dS^T.K, P^T.dO, dS^T.Q) needs its LDS operand token-contiguous; building
// that layout once per call here, instead of once per workgroup inside the hot kernels, lets
// those kernels fetch every tile with plain asynchronous global->LDS copies.  HBM-bound:
// 2 bytes read + 2 bytes written per element.
#include "mfma_tiles.h"

namespace mmsp {
namespace {

__global__ __launch_bounds__(256) void transpose_tiles_kernel(const uint16_t* __restrict__ x, int64_t tok_stride,
                                                              int64_t head_stride, int row0, int n_rows,
                                                              char* __restrict__ out) {
  __shared__ __attribute__((aligned(16))) char tile[kTileBytes];
  const int tid = threadIdx.x;
  const int t = blockIdx.x, h = blockIdx.y, n_tiles = gridDim.x;
  TileRegs r;
  tile_load(r, x + (int64_t)row0 * tok_stride + (int64_t)h * head_stride, tok_stride, t * 64, n_rows, tid);
  tile_store_t(r, tile, tid);
  __syncthreads();
  char* dst = out + ((int64_t)h * n_tiles + t) * kTileBytes;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    *reinterpret_cast<u32x4*>(dst + i * 4096 + tid * 16) = *reinterpret_cast<const u32x4*>(tile + i * 4096 + tid * 16);
}

}  // namespace

hipError_t launch_transpose_tiles(const void* x, int64_t tok_stride, int64_t head_stride, int H, int row0, int n_rows,
                                  void* out, hipStream_t stream) {
  if (n_rows <= 0) return hipSuccess;
  const dim3 g((unsigned)tiles_of(n_rows), H), b(256);
  transpose_tiles_kernel<<<g, b, 0, stream>>>(reinterpret_cast<const uint16_t*>(x), tok_stride, head_stride, row0, n_rows,
                                              reinterpret_cast<char*>(out));
  return hipGetLastError();
}

}  // namespace mmsp
