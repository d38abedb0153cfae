// Backward ring step on bf16 matrix cores, head_dim 128: dispatch of its two kernels.  No
// floating-point atomics, so results are bit-identical from run to run:
//
//  dq kernel   (query-stationary, like the forward): a wavefront owns 32 query rows, keeps Q,
//              dO (B operands) and the dQ^T accumulator in registers, streams K/V tiles:
//                S^T = K Q^T,  dP^T = V dO^T,  dS^T = P^T * (dP^T - delta),  dQ^T += K^T dS^T
//  dkdv kernel (key-stationary): a wavefront pair owns 32 keys of one KV head, keeps K, V (B
//              operands) and the dK^T, dV^T accumulators in registers, streams Q/dO tiles of
//              every query head of the group:
//                S = Q K^T,  dP = dO V^T,  P = exp(S - LSE),  dS = P * (dP - delta),
//                dV^T += dO^T P,  dK^T += Q^T dS
// Each recomputes S and dP (7 tile products in total instead of 5) in exchange for
// exclusive ownership of its outputs.
//
// Workspace of a backward call: [Q^T images | dO^T images | -LSE*log2e | delta] for the dK/dV
// kernel, then the K^T images for the dQ kernel.
#include "mfma_tiles.h"

namespace mmsp {

int64_t bwd_bf16_total_workspace_bytes(int Hq, int Hkv, int64_t n_q, int64_t n_k) {
  return bwd_bf16_workspace_bytes(Hq, n_q) + bwd_dq_bf16_workspace_bytes(Hkv, n_k);
}

hipError_t launch_bwd_bf16(const StepArgs& a, hipStream_t stream) {
  if (a.dq != nullptr) {
    hipError_t e = launch_bwd_dq_bf16(a, a.ws + bwd_bf16_workspace_bytes(a.Hq, a.n_q), stream);
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
