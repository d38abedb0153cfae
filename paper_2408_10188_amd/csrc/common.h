// Shared declarations of the HIP side: kernel argument block, visibility bounds, and the
// launcher prototypes the C-ABI layer dispatches to.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mmsp {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Everything a kernel needs to know about one call.  Row counts and positions are
// validated on the host to fit in int32.
struct StepArgs {
  // tensors (device)
  const void* q;  const void* k;  const void* v;
  const void* d_o;              // backward only
  float* o;  float* lse;        // forward outputs / running state
  const float* lse_final;  const float* delta;   // backward inputs
  float* dq;  float* dk;  float* dv;             // backward outputs
  const int32_t* cu;            // cu_seqlens or nullptr
  // shape
  int32_t Hq, Hkv, group, d;
  int64_t q_ts, q_hs, kv_ts, kv_hs, lse_hs;
  float scale;
  // block
  int32_t q_row0, n_q, k_row0, n_k, q_pos0, k_pos0;
  int32_t mask;                 // 0 full, 1 causal-diag
  int32_t n_docs;
  int32_t accumulate;           // fwd: merge into running state; bwd: add to dk/dv
  char* ws;                     // caller's workspace (bf16 backward)
};

// Workspace views of one backward call (all inside the caller's workspace).
struct BwdWorkspace {
  const float* nl2;    // -LSE*log2e, [Hq][n_qtiles*64], -inf where LSE = -inf and in the padding
  const float* dl;     // delta,      [Hq][n_qtiles*64], 0 in the padding
  float* partial;      // partial dK then dV of split key tiles, bwd_dkdv_partial_bytes() in all
  int32_t n_qtiles;
};

__host__ __device__ inline int64_t tiles_of(int64_t rows) { return (rows + 63) / 64; }

// Visible key interval [lo, hi] (indices inside the block's key range, already clipped to
// [0, n_k-1]) of the query row with block-relative index i.  Empty when lo > hi.
// A pair is visible iff the key position is <= the query position (causal-diag only) and
// both positions lie in the same cu_seqlens document (when given).
__device__ __forceinline__ void key_interval_of_row(const StepArgs& a, int i, int& lo, int& hi) {
  const int p = a.q_pos0 + i;
  int lo_pos = INT32_MIN / 2, hi_pos = INT32_MAX / 2;
  if (a.mask == 1) hi_pos = p;
  if (a.cu != nullptr) {
    // largest k with cu[k] <= p
    int L = 0, R = a.n_docs;          // invariant: cu[L] <= p (if p >= 0) < cu[R] (if inside)
    // positions outside every document see nothing; the empty intervals are chosen so that
    // lo and hi stay non-decreasing in the row index
    if (p < a.cu[0]) { lo = 0; hi = -1; return; }
    if (p >= a.cu[a.n_docs]) { lo = a.n_k; hi = a.n_k - 1; return; }
    while (R - L > 1) { int m = (L + R) >> 1; if (a.cu[m] <= p) L = m; else R = m; }
    lo_pos = max(lo_pos, a.cu[L]);
    hi_pos = min(hi_pos, a.cu[L + 1] - 1);
  }
  lo = max(0, lo_pos - a.k_pos0);
  hi = min(a.n_k - 1, hi_pos - a.k_pos0);
}

// Mirror image: interval [lo, hi] of block-relative query rows that see the key with
// block-relative index j (clipped to [0, n_q-1]).
__device__ __forceinline__ void row_interval_of_key(const StepArgs& a, int j, int& lo, int& hi) {
  const int p = a.k_pos0 + j;
  int lo_pos = INT32_MIN / 2, hi_pos = INT32_MAX / 2;
  if (a.mask == 1) lo_pos = p;
  if (a.cu != nullptr) {
    int L = 0, R = a.n_docs;
    if (p < a.cu[0]) { lo = 0; hi = -1; return; }
    if (p >= a.cu[a.n_docs]) { lo = a.n_q; hi = a.n_q - 1; return; }
    while (R - L > 1) { int m = (L + R) >> 1; if (a.cu[m] <= p) L = m; else R = m; }
    lo_pos = max(lo_pos, a.cu[L]);
    hi_pos = min(hi_pos, a.cu[L + 1] - 1);
  }
  lo = max(0, lo_pos - a.q_pos0);
  hi = min(a.n_q - 1, hi_pos - a.q_pos0);
}

// ---- launchers (each enqueues on `stream` and returns hipGetLastError()) ----
hipError_t launch_fill_empty(float* o, float* lse, int64_t lse_hs, int Hq, int d,
                             int row0, int n_rows, hipStream_t stream);
hipError_t launch_zero_f32(float* p, int64_t n /* multiple of 4, p 16-byte aligned */, hipStream_t stream);
hipError_t launch_merge(float* o_acc, float* lse_acc, const float* o_part, const float* lse_part,
                        void* o_final, int io_dtype, int64_t lse_hs, int Hq, int d,
                        int row0, int n_rows, hipStream_t stream);
hipError_t launch_delta(const void* o_final, const void* d_o, float* delta, int io_dtype,
                        int64_t lse_hs, int Hq, int d, int row0, int n_rows, hipStream_t stream);

// Padded per-row statistics of the backward: nl2 = -LSE*log2e (or -inf), dl = delta.
hipError_t launch_bwd_stats(const float* lse, const float* delta, int64_t lse_hs, int Hq, int row0, int n_rows,
                            float* nl2, float* dl, hipStream_t stream);
hipError_t launch_bwd_dkdv_bf16(const StepArgs& a, const BwdWorkspace& w, hipStream_t stream);
int64_t bwd_bf16_workspace_bytes(int Hq, int64_t n_q);
int64_t bwd_dkdv_partial_bytes();
hipError_t launch_bwd_dq_bf16(const StepArgs& a, hipStream_t stream);
hipError_t bwd_bf16_prepare(const StepArgs& a, BwdWorkspace& w, hipStream_t stream);

hipError_t launch_zigzag_gather(const void* seq, void* shards, int64_t T, int N, int64_t row_bytes, hipStream_t stream);
hipError_t launch_zigzag_scatter(const void* shards, void* seq, int64_t T, int N, int64_t row_bytes, hipStream_t stream);
hipError_t launch_swap_outer(const void* src, void* dst, int64_t A, int64_t B, int64_t row_bytes, hipStream_t stream);

hipError_t launch_fwd_f32(const StepArgs& a, hipStream_t stream);
hipError_t launch_bwd_f32(const StepArgs& a, hipStream_t stream);
hipError_t launch_fwd_bf16(const StepArgs& a, hipStream_t stream);
hipError_t launch_bwd_bf16(const StepArgs& a, hipStream_t stream);

}  // namespace mmsp
