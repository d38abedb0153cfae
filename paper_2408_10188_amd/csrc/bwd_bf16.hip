// Backward ring step on bf16 matrix cores, head_dim 128: dispatch of its two kernels and the
// small pre-pass they share.  No floating-point atomics, so results are bit-identical from run
// to run:
//
//  dq kernel   (query-stationary, like the forward): a wavefront owns 32 query rows, keeps Q,
//              dO (B operands) and the dQ^T accumulator in registers, streams K/V tiles:
//                S^T = K Q^T,  dP^T = V dO^T,  dS^T = P^T * (dP^T - delta),  dQ^T += K^T dS^T
//  dkdv kernel (key-stationary): a wavefront owns 32 keys of one KV head, keeps K, V (B
//              operands) and the dK^T, dV^T accumulators in registers, streams Q/dO tiles of
//              every query head of the group:
//                S = Q K^T,  dP = dO V^T,  P = exp(S - LSE),  dS = P * (dP - delta),
//                dV^T += dO^T P,  dK^T += Q^T dS
// Each recomputes S and dP (7 tile products in total instead of 5) in exchange for
// exclusive ownership of its outputs.
//
// Workspace of a backward call (dK/dV kernel only): [-LSE*log2e | delta] padded to whole
// 64-row tiles, then the area for partial dK / dV sums of split key tiles.
#include "common.h"

namespace mmsp {
namespace {

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
  return 2 * Hq * tiles_of(n_q) * 64 * (int64_t)sizeof(float) + bwd_dkdv_partial_bytes();
}

// Lays out the workspace of one backward call and fills the padded row statistics; the
// partial-sum area follows them.
hipError_t bwd_bf16_prepare(const StepArgs& a, BwdWorkspace& w, hipStream_t stream) {
  const int64_t t = tiles_of(a.n_q);
  char* p = a.ws;
  float* nl2 = reinterpret_cast<float*>(p);  p += a.Hq * t * 64 * sizeof(float);
  float* dl = reinterpret_cast<float*>(p);   p += a.Hq * t * 64 * sizeof(float);
  w.nl2 = nl2; w.dl = dl; w.partial = reinterpret_cast<float*>(p); w.n_qtiles = (int32_t)t;
  return launch_bwd_stats(a.lse_final, a.delta, a.lse_hs, a.Hq, a.q_row0, a.n_q, nl2, dl, stream);
}

hipError_t launch_bwd_bf16(const StepArgs& a, hipStream_t stream) {
  if (a.dq != nullptr) {
    hipError_t e = launch_bwd_dq_bf16(a, stream);
    if (e != hipSuccess) return e;
  }
  if (a.dk != nullptr) {
    BwdWorkspace w;
    hipError_t e = bwd_bf16_prepare(a, w, stream);
    if (e != hipSuccess) return e;
    e = launch_bwd_dkdv_bf16(a, w, stream);
    if (e != hipSuccess) return e;
  }
  return hipGetLastError();
}

}  // namespace mmsp
