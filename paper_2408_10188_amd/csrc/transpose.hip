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

__global__ __launch_bounds__(256) void bwd_stats_kernel(const float* __restrict__ lse, const float* __restrict__ delta,
                                                        int64_t lse_hs, int row0, int n_rows, int padded,
                                                        float* __restrict__ nl2, float* __restrict__ dl) {
  const int i = blockIdx.x * 256 + threadIdx.x, h = blockIdx.y;
  if (i >= padded) return;
  float n = -INFINITY, d = 0.f;
  if (i < n_rows) {
    const float L = lse[(int64_t)h * lse_hs + row0 + i];
    n = L == -INFINITY ? -INFINITY : -L * kLog2e;      // a row that saw nothing: P = exp2(-inf) = 0
    d = delta[(int64_t)h * lse_hs + row0 + i];
  }
  nl2[(int64_t)h * padded + i] = n;
  dl[(int64_t)h * padded + i] = d;
}

}  // namespace

hipError_t launch_bwd_stats(const float* lse, const float* delta, int64_t lse_hs, int Hq, int row0, int n_rows,
                            float* nl2, float* dl, hipStream_t stream) {
  const int padded = (int)tiles_of(n_rows) * 64;
  if (padded == 0) return hipSuccess;
  bwd_stats_kernel<<<dim3((padded + 255) / 256, Hq), dim3(256), 0, stream>>>(lse, delta, lse_hs, row0, n_rows, padded, nl2, dl);
  return hipGetLastError();
}

int64_t bwd_bf16_workspace_bytes(int Hq, int64_t n_q) {
  const int64_t t = tiles_of(n_q);
  return 2 * Hq * t * kImageBytes + 2 * Hq * t * 64 * (int64_t)sizeof(float) + bwd_dkdv_partial_bytes();
}

// Lays out the dK/dV kernel's part of the workspace of one backward call and fills it: Q^T /
// dO^T tile images and the padded row statistics; the partial-sum area follows them.
hipError_t bwd_bf16_prepare(const StepArgs& a, BwdWorkspace& w, hipStream_t stream) {
  const int64_t t = tiles_of(a.n_q);
  char* p = a.ws;
  char* qt = p;            p += a.Hq * t * kImageBytes;
  char* dot = p;           p += a.Hq * t * kImageBytes;
  float* nl2 = reinterpret_cast<float*>(p);  p += a.Hq * t * 64 * sizeof(float);
  float* dl = reinterpret_cast<float*>(p);   p += a.Hq * t * 64 * sizeof(float);
  w.qt = qt; w.dot = dot; w.nl2 = nl2; w.dl = dl; w.partial = reinterpret_cast<float*>(p); w.n_qtiles = (int32_t)t;
  hipError_t e = launch_transpose_tiles(a.q, a.q_ts, a.q_hs, a.Hq, a.q_row0, a.n_q, qt, stream);
  if (e != hipSuccess) return e;
  e = launch_transpose_tiles(a.d_o, (int64_t)a.Hq * 128, 128, a.Hq, a.q_row0, a.n_q, dot, stream);
  if (e != hipSuccess) return e;
  return launch_bwd_stats(a.lse_final, a.delta, a.lse_hs, a.Hq, a.q_row0, a.n_q, nl2, dl, stream);
}

hipError_t launch_transpose_tiles(const void* x, int64_t tok_stride, int64_t head_stride, int H, int row0, int n_rows,
                                  void* out, hipStream_t stream) {
  if (n_rows <= 0) return hipSuccess;
  const dim3 g((unsigned)tiles_of(n_rows), H), b(256);
  transpose_tiles_kernel<<<g, b, 0, stream>>>(reinterpret_cast<const uint16_t*>(x), tok_stride, head_stride, row0, n_rows,
                                              reinterpret_cast<char*>(out));
  return hipGetLastError();
}

}  // namespace mmsp
