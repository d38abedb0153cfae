// HBM-bound helpers: the log-sum-exp merge of a partial into the running result, the cast of
// the running O to the io dtype, the backward row term delta = rowsum(dO * O), and the
// "nothing visible" fill.  All are one pass over dense [rows, Hq, d] data with 16-byte
// accesses; the [Hq, rows] statistics are tiny beside them.
#include "common.h"

namespace mmsp {
namespace {

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  f32x2 x = {lo, hi};
  bf16x2 y = __builtin_convertvector(x, bf16x2);      // round to nearest even
  return __builtin_bit_cast(uint32_t, y);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// One thread owns 4 consecutive d-elements of one (row, head).  d/4 threads (16 or 32, a
// power of two, aligned inside a wavefront) share one LSE pair; the lane with chunk 0
// writes the merged LSE after every lane of the wavefront has read the old one.
template <bool kMerge, int kOut /*0 none, 1 bf16, 2 f32*/>
__global__ __launch_bounds__(256) void merge_kernel(float* __restrict__ o_acc, float* __restrict__ lse_acc,
                                                    const float* __restrict__ o_part,
                                                    const float* __restrict__ lse_part, void* __restrict__ o_final,
                                                    int64_t lse_hs, int Hq, int d, int row0, int64_t n_vec) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_vec) return;
  const int vec_per_head = d >> 2;
  const int c = (int)(t % vec_per_head);
  const int64_t rh = t / vec_per_head;
  const int h = (int)(rh % Hq);
  const int64_t r = rh / Hq + row0;
  const int64_t off = (r * Hq + h) * (int64_t)d + c * 4;
  float4 o = *reinterpret_cast<const float4*>(o_acc + off);
  if (kMerge) {
    const int64_t li = h * lse_hs + r;
    const float la = lse_acc[li], lp = lse_part[li];
    const float4 p = *reinterpret_cast<const float4*>(o_part + off);
    const float m = fmaxf(la, lp);
    float wa, wb, ln;
    if (m == -INFINITY) { wa = 0.f; wb = 0.f; ln = -INFINITY; }
    else {
      const float ea = __expf(la - m), eb = __expf(lp - m);   // exp(-inf) = 0 handles an empty side
      const float tot = ea + eb;
      wa = ea / tot; wb = eb / tot; ln = m + __logf(tot);
    }
    o.x = wa * o.x + wb * p.x; o.y = wa * o.y + wb * p.y;
    o.z = wa * o.z + wb * p.z; o.w = wa * o.w + wb * p.w;
    *reinterpret_cast<float4*>(o_acc + off) = o;
    if (c == 0) lse_acc[li] = ln;
  }
  if (kOut == 1) {
    uint2 w = {pack_bf16x2(o.x, o.y), pack_bf16x2(o.z, o.w)};
    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(o_final) + off) = w;
  } else if (kOut == 2) {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(o_final) + off) = o;
  }
}

// delta: kVec elements per thread (8 bf16 or 4 f32 = 16 bytes of each operand); the d/kVec
// lanes of one (row, head) reduce with xor-shuffles.
template <bool kBf16>
__global__ __launch_bounds__(256) void delta_kernel(const void* __restrict__ o_final, const void* __restrict__ d_o,
                                                    float* __restrict__ delta, int64_t lse_hs, int Hq, int d,
                                                    int row0, int64_t n_vec) {
  constexpr int kVec = kBf16 ? 8 : 4;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int vec_per_head = d / kVec;                    // 8, 16 or 32 lanes
  const bool live = t < n_vec;
  const int64_t tt = live ? t : 0;
  const int c = (int)(tt % vec_per_head);
  const int64_t rh = tt / vec_per_head;
  const int h = (int)(rh % Hq);
  const int64_t r = rh / Hq + row0;
  const int64_t off = (r * Hq + h) * (int64_t)d + c * kVec;
  float s = 0.f;
  if (live) {
    if (kBf16) {
      const uint4 a = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(o_final) + off);
      const uint4 b = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(d_o) + off);
      s = bf16_lo(a.x) * bf16_lo(b.x) + bf16_hi(a.x) * bf16_hi(b.x) + bf16_lo(a.y) * bf16_lo(b.y) +
          bf16_hi(a.y) * bf16_hi(b.y) + bf16_lo(a.z) * bf16_lo(b.z) + bf16_hi(a.z) * bf16_hi(b.z) +
          bf16_lo(a.w) * bf16_lo(b.w) + bf16_hi(a.w) * bf16_hi(b.w);
    } else {
      const float4 a = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(o_final) + off);
      const float4 b = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(d_o) + off);
      s = a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
    }
  }
  for (int w = vec_per_head >> 1; w > 0; w >>= 1) s += __shfl_xor(s, w);
  if (live && c == 0) delta[h * lse_hs + r] = s;
}

__global__ __launch_bounds__(256) void fill_empty_kernel(float* __restrict__ o, float* __restrict__ lse,
                                                         int64_t lse_hs, int Hq, int d, int row0, int64_t n_vec) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_vec) return;
  const int vec_per_head = d >> 2;
  const int c = (int)(t % vec_per_head);
  const int64_t rh = t / vec_per_head;
  const int h = (int)(rh % Hq);
  const int64_t r = rh / Hq + row0;
  *reinterpret_cast<float4*>(o + (r * Hq + h) * (int64_t)d + c * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
  if (c == 0) lse[h * lse_hs + r] = -INFINITY;
}

__global__ __launch_bounds__(256) void zero_kernel(float4* __restrict__ p, int64_t n_vec) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n_vec) p[t] = make_float4(0.f, 0.f, 0.f, 0.f);
}

inline unsigned grid_for(int64_t n, int block) { return (unsigned)((n + block - 1) / block); }

}  // namespace

hipError_t launch_zero_f32(float* p, int64_t n, hipStream_t stream) {
  const int64_t n_vec = n / 4;
  if (n_vec == 0) return hipSuccess;
  zero_kernel<<<grid_for(n_vec, 256), 256, 0, stream>>>(reinterpret_cast<float4*>(p), n_vec);
  return hipGetLastError();
}

hipError_t launch_fill_empty(float* o, float* lse, int64_t lse_hs, int Hq, int d, int row0, int n_rows,
                             hipStream_t stream) {
  const int64_t n_vec = (int64_t)n_rows * Hq * (d / 4);
  if (n_vec == 0) return hipSuccess;
  fill_empty_kernel<<<grid_for(n_vec, 256), 256, 0, stream>>>(o, lse, lse_hs, Hq, d, row0, n_vec);
  return hipGetLastError();
}

hipError_t launch_merge(float* o_acc, float* lse_acc, const float* o_part, const float* lse_part, void* o_final,
                        int io_dtype, int64_t lse_hs, int Hq, int d, int row0, int n_rows, hipStream_t stream) {
  const int64_t n_vec = (int64_t)n_rows * Hq * (d / 4);
  if (n_vec == 0) return hipSuccess;
  const dim3 g(grid_for(n_vec, 256)), b(256);
  const bool merge = o_part != nullptr;
  const int out = o_final == nullptr ? 0 : (io_dtype == 0 ? 1 : 2);
#define MMSP_MERGE(M, O) \
  merge_kernel<M, O><<<g, b, 0, stream>>>(o_acc, lse_acc, o_part, lse_part, o_final, lse_hs, Hq, d, row0, n_vec)
  if (merge) { if (out == 0) MMSP_MERGE(true, 0); else if (out == 1) MMSP_MERGE(true, 1); else MMSP_MERGE(true, 2); }
  else       { if (out == 1) MMSP_MERGE(false, 1); else if (out == 2) MMSP_MERGE(false, 2); }
#undef MMSP_MERGE
  return hipGetLastError();
}

hipError_t launch_delta(const void* o_final, const void* d_o, float* delta, int io_dtype, int64_t lse_hs, int Hq,
                        int d, int row0, int n_rows, hipStream_t stream) {
  const int vec = io_dtype == 0 ? 8 : 4;
  const int64_t n_vec = (int64_t)n_rows * Hq * (d / vec);
  if (n_vec == 0) return hipSuccess;
  const dim3 g(grid_for(n_vec, 256)), b(256);
  if (io_dtype == 0) delta_kernel<true><<<g, b, 0, stream>>>(o_final, d_o, delta, lse_hs, Hq, d, row0, n_vec);
  else delta_kernel<false><<<g, b, 0, stream>>>(o_final, d_o, delta, lse_hs, Hq, d, row0, n_vec);
  return hipGetLastError();
}

}  // namespace mmsp
