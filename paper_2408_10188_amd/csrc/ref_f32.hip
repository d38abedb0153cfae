// fp32 path (io_dtype = f32): true fp32 products and accumulation with accurate expf/logf, for
// the small full-precision configuration whose tolerance (1e-5) rules out bf16 matrix cores.
// One thread per query row (forward, dQ) or per key row (dK/dV); K/V rows are read by every
// lane of a wavefront at the same address (one broadcast fetch).  Not a throughput path.
#include "common.h"

namespace mmsp {
namespace {

template <int D>
__global__ __launch_bounds__(64) void fwd_f32_kernel(StepArgs a) {
  const int i = blockIdx.x * 64 + threadIdx.x;         // block-relative query row
  const int h = blockIdx.y;
  const int kvh = h / a.group;
  const bool live = i < a.n_q;
  const int ii = live ? i : a.n_q - 1;
  int lo, hi;
  key_interval_of_row(a, ii, lo, hi);
  if (!live) { lo = 1; hi = 0; }
  const float* qp = reinterpret_cast<const float*>(a.q) + (int64_t)(a.q_row0 + ii) * a.q_ts + (int64_t)h * a.q_hs;
  float q[D], acc[D];
#pragma unroll
  for (int c = 0; c < D; ++c) { q[c] = qp[c]; acc[c] = 0.f; }
  float m = -INFINITY, l = 0.f;
  // wavefront-uniform loop bounds so that every lane reads the same K/V row
  int wlo = lo, whi = hi;
  for (int w = 32; w > 0; w >>= 1) { wlo = min(wlo, __shfl_xor(wlo, w)); whi = max(whi, __shfl_xor(whi, w)); }
  const float* kb = reinterpret_cast<const float*>(a.k) + (int64_t)kvh * a.kv_hs;
  const float* vb = reinterpret_cast<const float*>(a.v) + (int64_t)kvh * a.kv_hs;
  for (int j = wlo; j <= whi; ++j) {
    const float* kr = kb + (int64_t)(a.k_row0 + j) * a.kv_ts;
    const float* vr = vb + (int64_t)(a.k_row0 + j) * a.kv_ts;
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < D; ++c) s = fmaf(q[c], kr[c], s);
    s *= a.scale;
    if (j >= lo && j <= hi) {
      const float mn = fmaxf(m, s);
      const float alpha = expf(m - mn);                // m = -inf on the first visible key -> 0
      const float p = expf(s - mn);
      l = l * alpha + p;
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] = acc[c] * alpha + p * vr[c];
      m = mn;
    }
  }
  if (!live) return;
  const int64_t r = a.q_row0 + i;
  float* op = a.o + (r * a.Hq + h) * (int64_t)D;
  float* lp = a.lse + (int64_t)h * a.lse_hs + r;
  const float inv = l > 0.f ? 1.f / l : 0.f;
  const float lse_part = l > 0.f ? m + logf(l) : -INFINITY;
  if (!a.accumulate) {
#pragma unroll
    for (int c = 0; c < D; ++c) op[c] = acc[c] * inv;
    *lp = lse_part;
  } else {
    const float la = *lp;
    const float mm = fmaxf(la, lse_part);
    if (mm == -INFINITY) return;                       // both empty: leave the running state
    const float ea = expf(la - mm), eb = expf(lse_part - mm);
    const float tot = ea + eb;
    const float wa = ea / tot, wb = eb / tot * inv;
#pragma unroll
    for (int c = 0; c < D; ++c) op[c] = wa * op[c] + wb * acc[c];
    *lp = mm + logf(tot);
  }
}

template <int D>
__global__ __launch_bounds__(64) void bwd_dq_f32_kernel(StepArgs a) {
  const int i = blockIdx.x * 64 + threadIdx.x;
  const int h = blockIdx.y;
  const int kvh = h / a.group;
  const bool live = i < a.n_q;
  const int ii = live ? i : a.n_q - 1;
  int lo, hi;
  key_interval_of_row(a, ii, lo, hi);
  if (!live) { lo = 1; hi = 0; }
  const int64_t r = a.q_row0 + ii;
  const float* qp = reinterpret_cast<const float*>(a.q) + r * a.q_ts + (int64_t)h * a.q_hs;
  const float* dop = reinterpret_cast<const float*>(a.d_o) + (r * a.Hq + h) * (int64_t)D;
  const float L = a.lse_final[(int64_t)h * a.lse_hs + r];
  const float Dl = a.delta[(int64_t)h * a.lse_hs + r];
  float q[D], dov[D], acc[D];
#pragma unroll
  for (int c = 0; c < D; ++c) { q[c] = qp[c]; dov[c] = dop[c]; acc[c] = 0.f; }
  int wlo = lo, whi = hi;
  for (int w = 32; w > 0; w >>= 1) { wlo = min(wlo, __shfl_xor(wlo, w)); whi = max(whi, __shfl_xor(whi, w)); }
  const float* kb = reinterpret_cast<const float*>(a.k) + (int64_t)kvh * a.kv_hs;
  const float* vb = reinterpret_cast<const float*>(a.v) + (int64_t)kvh * a.kv_hs;
  for (int j = wlo; j <= whi; ++j) {
    const float* kr = kb + (int64_t)(a.k_row0 + j) * a.kv_ts;
    const float* vr = vb + (int64_t)(a.k_row0 + j) * a.kv_ts;
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int c = 0; c < D; ++c) { s = fmaf(q[c], kr[c], s); dp = fmaf(dov[c], vr[c], dp); }
    if (j >= lo && j <= hi && L != -INFINITY) {
      const float p = expf(s * a.scale - L);
      const float ds = p * (dp - Dl);
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] = fmaf(ds, kr[c], acc[c]);
    }
  }
  if (!live) return;
  float* dq = a.dq + (r * a.Hq + h) * (int64_t)D;
#pragma unroll
  for (int c = 0; c < D; ++c) dq[c] += a.scale * acc[c];
}

// One thread per key row; loops over the query heads of its KV group and over the query rows
// that see it.  Query rows are wavefront-uniform, so Q/dO/LSE/delta reads are broadcasts.
template <int D>
__global__ __launch_bounds__(64) void bwd_dkdv_f32_kernel(StepArgs a) {
  const int j = blockIdx.x * 64 + threadIdx.x;
  const int kvh = blockIdx.y;
  const bool live = j < a.n_k;
  const int jj = live ? j : a.n_k - 1;
  int lo, hi;
  row_interval_of_key(a, jj, lo, hi);
  if (!live) { lo = 1; hi = 0; }
  const int64_t kr_off = (int64_t)(a.k_row0 + jj) * a.kv_ts + (int64_t)kvh * a.kv_hs;
  const float* kp = reinterpret_cast<const float*>(a.k) + kr_off;
  const float* vp = reinterpret_cast<const float*>(a.v) + kr_off;
  float kk[D], vv[D], dk[D], dv[D];
#pragma unroll
  for (int c = 0; c < D; ++c) { kk[c] = kp[c]; vv[c] = vp[c]; dk[c] = 0.f; dv[c] = 0.f; }
  int wlo = lo, whi = hi;
  for (int w = 32; w > 0; w >>= 1) { wlo = min(wlo, __shfl_xor(wlo, w)); whi = max(whi, __shfl_xor(whi, w)); }
  for (int hg = 0; hg < a.group; ++hg) {
    const int h = kvh * a.group + hg;
    for (int i = wlo; i <= whi; ++i) {
      const int64_t r = a.q_row0 + i;
      const float* qr = reinterpret_cast<const float*>(a.q) + r * a.q_ts + (int64_t)h * a.q_hs;
      const float* dor = reinterpret_cast<const float*>(a.d_o) + (r * a.Hq + h) * (int64_t)D;
      const float L = a.lse_final[(int64_t)h * a.lse_hs + r];
      const float Dl = a.delta[(int64_t)h * a.lse_hs + r];
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) { s = fmaf(qr[c], kk[c], s); dp = fmaf(dor[c], vv[c], dp); }
      if (i >= lo && i <= hi && L != -INFINITY) {
        const float p = expf(s * a.scale - L);
        const float ds = p * (dp - Dl);
#pragma unroll
        for (int c = 0; c < D; ++c) { dv[c] = fmaf(p, dor[c], dv[c]); dk[c] = fmaf(ds, qr[c], dk[c]); }
      }
    }
  }
  if (!live) return;
  const int64_t off = ((int64_t)(a.k_row0 + j) * a.Hkv + kvh) * (int64_t)D;
  float* dkp = a.dk + off;
  float* dvp = a.dv + off;
  if (a.accumulate) {
#pragma unroll
    for (int c = 0; c < D; ++c) { dkp[c] += a.scale * dk[c]; dvp[c] += dv[c]; }
  } else {
#pragma unroll
    for (int c = 0; c < D; ++c) { dkp[c] = a.scale * dk[c]; dvp[c] = dv[c]; }
  }
}

}  // namespace

hipError_t launch_fwd_f32(const StepArgs& a, hipStream_t stream) {
  const dim3 g((a.n_q + 63) / 64, a.Hq), b(64);
  if (a.d == 64) fwd_f32_kernel<64><<<g, b, 0, stream>>>(a);
  else fwd_f32_kernel<128><<<g, b, 0, stream>>>(a);
  return hipGetLastError();
}

hipError_t launch_bwd_f32(const StepArgs& a, hipStream_t stream) {
  const dim3 gq((a.n_q + 63) / 64, a.Hq), gk((a.n_k + 63) / 64, a.Hkv), b(64);
  if (a.d == 64) {
    if (a.dq != nullptr) bwd_dq_f32_kernel<64><<<gq, b, 0, stream>>>(a);
    if (a.dk != nullptr) bwd_dkdv_f32_kernel<64><<<gk, b, 0, stream>>>(a);
  } else {
    if (a.dq != nullptr) bwd_dq_f32_kernel<128><<<gq, b, 0, stream>>>(a);
    if (a.dk != nullptr) bwd_dkdv_f32_kernel<128><<<gk, b, 0, stream>>>(a);
  }
  return hipGetLastError();
}

}  // namespace mmsp
