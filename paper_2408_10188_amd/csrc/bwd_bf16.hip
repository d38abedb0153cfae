// Backward ring step on bf16 matrix cores, head_dim 128.  Two kernels, no floating-point
// atomics, so results are bit-identical from run to run:
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
#include "mfma_tiles.h"

namespace mmsp {
namespace {

constexpr int kBM = 128;   // dq kernel: query rows per workgroup;  dkdv kernel: keys per workgroup
constexpr int kBN = 64;    // streamed tile length

// ------------------------------------------------------------------------------------ dQ
__global__ __launch_bounds__(256, 2) void bwd_dq_bf16_kernel(StepArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];   // K TileN | V TileN | K TileT
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int qt = (int)gridDim.x - 1 - (int)blockIdx.x;
  const int h = blockIdx.y, kvh = h / a.group;
  const int tile_row0 = qt * kBM;
  const int row = tile_row0 + wave * 32 + col;
  const bool live = row < a.n_q;
  const int rowc = min(row, a.n_q - 1);

  int lo, hi;
  key_interval_of_row(a, rowc, lo, hi);
  int t_lo, t_hi, dummy;
  key_interval_of_row(a, tile_row0, t_lo, dummy);
  key_interval_of_row(a, min(tile_row0 + kBM, a.n_q) - 1, dummy, t_hi);
  int w_lo_max, w_hi_min;
  {
    const int wr0 = min(tile_row0 + wave * 32, a.n_q - 1), wr1 = min(tile_row0 + wave * 32 + 31, a.n_q - 1);
    key_interval_of_row(a, wr0, dummy, w_hi_min);
    key_interval_of_row(a, wr1, w_lo_max, dummy);
  }
  const int kt0 = t_lo / kBN, kt1 = t_hi >= t_lo ? t_hi / kBN : kt0 - 1;

  const int64_t r = a.q_row0 + rowc;
  u32x4 qreg[8], doreg[8];
  {
    const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + r * a.q_ts + (int64_t)h * a.q_hs + half * 8;
    const uint16_t* dp = reinterpret_cast<const uint16_t*>(a.d_o) + (r * a.Hq + h) * 128 + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      qreg[ks] = *reinterpret_cast<const u32x4*>(qp + ks * 16);
      doreg[ks] = *reinterpret_cast<const u32x4*>(dp + ks * 16);
    }
  }
  const float L = a.lse_final[(int64_t)h * a.lse_hs + r];
  const float Dl = a.delta[(int64_t)h * a.lse_hs + r];
  const float neg_l2 = L == -INFINITY ? -INFINITY : -L * kLog2e;   // a row that saw nothing: P = 0
  const float c = a.scale * kLog2e;

  f32x16 dq[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;

  const uint16_t* kbase = reinterpret_cast<const uint16_t*>(a.k) + (int64_t)a.k_row0 * a.kv_ts + (int64_t)kvh * a.kv_hs;
  const uint16_t* vbase = reinterpret_cast<const uint16_t*>(a.v) + (int64_t)a.k_row0 * a.kv_ts + (int64_t)kvh * a.kv_hs;
  char* ktile = smem;
  char* vtile = smem + kTileBytes;
  char* kttile = smem + 2 * kTileBytes;

  TileRegs kr, vr;
  if (kt0 <= kt1) {
    tile_load(kr, kbase, a.kv_ts, kt0 * kBN, a.n_k, tid);
    tile_load(vr, vbase, a.kv_ts, kt0 * kBN, a.n_k, tid);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  /* vmcnt(0) */   // Q, dO, first tile landed: nothing stays pending across the back edge
  for (int kt = kt0; kt <= kt1; ++kt) {
    __syncthreads();                                   // every wavefront is done with the old tile
    tile_store_n(kr, ktile, tid);
    tile_store_t(kr, kttile, tid);
    tile_store_n(vr, vtile, tid);
    __syncthreads();
    if (kt < kt1) {
      tile_load(kr, kbase, a.kv_ts, (kt + 1) * kBN, a.n_k, tid);
      tile_load(vr, vbase, a.kv_ts, (kt + 1) * kBN, a.n_k, tid);
    }
    const int k0 = kt * kBN;
    const bool need_mask = k0 < w_lo_max || k0 + kBN - 1 > w_hi_min;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 s, dp;
#pragma unroll
      for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        s = mfma32(tile_n_read(ktile, kb, ks, lane), qreg[ks], s);
        dp = mfma32(tile_n_read(vtile, kb, ks, lane), doreg[ks], dp);
      }
      if (need_mask) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = k0 + kb * 32 + (i >> 2) * 8 + half * 4 + (i & 3);
          if (key < lo || key > hi) s[i] = -INFINITY;
        }
      }
      float ds[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[i], c, neg_l2));
        ds[i] = p * (dp[i] - Dl);
      }
      const u32x4 b0 = mk4(pack2(ds[0], ds[1]), pack2(ds[2], ds[3]), pack2(ds[4], ds[5]), pack2(ds[6], ds[7]));
      const u32x4 b1 = mk4(pack2(ds[8], ds[9]), pack2(ds[10], ds[11]), pack2(ds[12], ds[13]), pack2(ds[14], ds[15]));
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        dq[db] = mfma32(tile_t_read(kttile, db, kb * 2 + 0, lane), b0, dq[db]);
        dq[db] = mfma32(tile_t_read(kttile, db, kb * 2 + 1, lane), b1, dq[db]);
      }
    }
  }

  if (!live) return;
  float* out = a.dq + ((int64_t)(a.q_row0 + row) * a.Hq + h) * 128 + half * 4;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      float4* dst = reinterpret_cast<float4*>(out + db * 32 + g4 * 8);
      float4 o = *dst;
      o.x += a.scale * dq[db][g4 * 4 + 0]; o.y += a.scale * dq[db][g4 * 4 + 1];
      o.z += a.scale * dq[db][g4 * 4 + 2]; o.w += a.scale * dq[db][g4 * 4 + 3];
      *dst = o;
    }
}

}  // namespace

hipError_t launch_bwd_bf16(const StepArgs& a, hipStream_t stream) {
  if (a.dq != nullptr) {
    const dim3 g((a.n_q + kBM - 1) / kBM, a.Hq), b(256);
    const size_t smem = 3 * kTileBytes;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dq_bf16_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (attr != hipSuccess) return attr;
    bwd_dq_bf16_kernel<<<g, b, smem, stream>>>(a);
    hipError_t e = hipGetLastError();
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
