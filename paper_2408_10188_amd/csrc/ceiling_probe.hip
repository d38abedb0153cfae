// Stand-alone probe of what the matrix cores sustain on this GPU under the instruction mix of
// the attention kernels, to read the roofline fraction of bench.py against: the published
// dense bf16 peak assumes every CU issues one 32x32x16 MFMA per SIMD every 32 cycles at the
// peak clock, which the chip only does when the operands are trivial.
//
// One workgroup per CU, 8 wavefronts (two per SIMD) as in the attention kernels.  An
// "iteration" is one 64-key tile of a forward step for each wavefront: 16 MFMAs whose A
// operands come from LDS (S = K Q^T), optionally the softmax-like vector work on the 32
// results per lane, 16 more MFMAs with A operands from LDS (O += V^T P).  Modes:
//   zero     MFMA + LDS reads only, LDS filled with zeros
//   random   MFMA + LDS reads only, LDS filled with pseudo-random bf16 bits
//   softmax  random + the vector work (max, exp2, sum, bf16 pack), wavefronts free-running
//   tile     softmax + a workgroup barrier and a 32 KiB asynchronous global->LDS copy per iteration
// Prints one line per mode: time, TFLOP/s, fraction of the published peak.
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstring>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                      \
  do {                                                                                \
    hipError_t e_ = (x);                                                              \
    if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } \
  } while (0)

__device__ __forceinline__ f32x16 mfma32(const u32x4& a, const u32x4& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  f32x2 x = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

enum Mode { kZero = 0, kRandom = 1, kSoftmax = 2, kTile = 3 };

template <int MODE>
__global__ __launch_bounds__(512, 2) void probe_kernel(float* out, int iters, const char* src, int span) {
  __shared__ __attribute__((aligned(1024))) char lds[65536];
  __shared__ __attribute__((aligned(1024))) char landing[32768];
  for (int i = threadIdx.x; i < 32768; i += 512)
    reinterpret_cast<uint16_t*>(lds)[i] = MODE == kZero ? 0 : 0x3c00 + ((i * 2654435761u) >> 24);
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int base = lane * 16;
  u32x4 q[8], p[4];
  for (int ks = 0; ks < 8; ++ks) q[ks] = *reinterpret_cast<const u32x4*>(lds + ((base + ks * 1024 + wave * 8192) & 65535));
  for (int g = 0; g < 4; ++g) p[g] = q[g];
  f32x16 o[4], s[2];
  for (int a = 0; a < 4; ++a) for (int i = 0; i < 16; ++i) o[a][i] = 0.f;
  float m = 0.f, l = 0.f;
  const char* g = src + (size_t)(blockIdx.x % 32) * 4096 + wave * 4096 + lane * 16;

  for (int it = 0; it < iters; ++it) {
    if (MODE == kTile) {
      __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): last iteration's copy
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      const char* gp = g + ((size_t)it * 32768) % span;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gp + j * 1024),
                                         (__attribute__((address_space(3))) void*)(landing + (wave * 4 + j) * 1024), 16, 0, 0);
    }
    const char* t = lds + (it & 1) * 32768;
    u32x4 kop[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) kop[j] = *reinterpret_cast<const u32x4*>(t + base + j * 1024);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int a = 0; a < 2; ++a) for (int i = 0; i < 16; ++i) s[a][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) { s[0] = mfma32(kop[2 * ks], q[ks], s[0]); s[1] = mfma32(kop[2 * ks + 1], q[ks], s[1]); }
    u32x4 vop[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) vop[j] = *reinterpret_cast<const u32x4*>(t + 16384 + base + j * 1024);
    __builtin_amdgcn_sched_barrier(0);
    if (MODE >= kSoftmax) {
      float mx = m;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int i = 0; i < 16; i += 2) mx = fmaxf(mx, fmaxf(s[a][i], s[a][i + 1]));
      m = mx;
      float sum = 0.f;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          uint32_t w[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float e0 = __builtin_amdgcn_exp2f(fmaf(s[a][h * 8 + 2 * j], 0.1f, -mx));
            const float e1 = __builtin_amdgcn_exp2f(fmaf(s[a][h * 8 + 2 * j + 1], 0.1f, -mx));
            sum += e0; sum += e1;
            w[j] = pack2(e0, e1);
          }
          p[a * 2 + h] = (u32x4){w[0], w[1], w[2], w[3]};
        }
      l += sum;
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int gq = 0; gq < 4; ++gq)
#pragma unroll
      for (int db = 0; db < 4; ++db) o[db] = mfma32(vop[gq * 4 + db], p[gq], o[db]);
  }
  if (MODE == kTile) { __builtin_amdgcn_s_waitcnt(0x0F70); m += landing[lane * 4]; }
  float r = m + l;
  for (int a = 0; a < 4; ++a) for (int i = 0; i < 16; ++i) r += o[a][i];
  for (int a = 0; a < 2; ++a) for (int i = 0; i < 16; ++i) r += s[a][i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

int main() {
  int n_cu = 0;
  CHECK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, 0));
  float* out; char* src;
  CHECK(hipMalloc(&out, (size_t)n_cu * 512 * sizeof(float)));
  CHECK(hipMalloc(&src, 64 << 20));
  CHECK(hipMemset(src, 1, 64 << 20));
  const int iters = 4000, span = 48 << 20;
  const double flop = (double)n_cu * 8 * iters * 32 * 32768.0;   // 32 MFMAs of 2*32*32*16 flop per wavefront and iteration
  const double peak = 2500.0;
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
  const char* names[] = {"zero", "random", "softmax", "tile"};
  for (int mode = 0; mode < 4; ++mode) {
    float best = 1e30f;
    for (int rep = 0; rep < 4; ++rep) {
      CHECK(hipEventRecord(e0));
      if (mode == 0) probe_kernel<kZero><<<n_cu, 512>>>(out, iters, src, span);
      if (mode == 1) probe_kernel<kRandom><<<n_cu, 512>>>(out, iters, src, span);
      if (mode == 2) probe_kernel<kSoftmax><<<n_cu, 512>>>(out, iters, src, span);
      if (mode == 3) probe_kernel<kTile><<<n_cu, 512>>>(out, iters, src, span);
      CHECK(hipGetLastError());
      CHECK(hipEventRecord(e1));
      CHECK(hipEventSynchronize(e1));
      float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
      if (rep > 0 && ms < best) best = ms;
    }
    printf("{\"probe\": \"%s\", \"cus\": %d, \"ms\": %.3f, \"tflops\": %.1f, \"frac_of_published_peak\": %.3f}\n", names[mode], n_cu,
           best, flop / best / 1e9, flop / best / 1e9 / peak);
    fflush(stdout);
  }
  return 0;
}
