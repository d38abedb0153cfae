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

// ------------------------------------------------------------------------------------ dK, dV
__global__ __launch_bounds__(256, 1) void bwd_dkdv_bf16_kernel(StepArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];   // Q TileN | dO TileN | Q TileT | dO TileT | -LSE*log2e[64] | delta[64]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int kvh = blockIdx.y;
  const int tile_key0 = blockIdx.x * kBM;
  const int key = tile_key0 + wave * 32 + col;           // block-relative key of this lane
  const bool live = key < a.n_k;
  const int keyc = min(key, a.n_k - 1);

  int rlo, rhi;                                          // query rows that see this lane's key
  row_interval_of_key(a, keyc, rlo, rhi);
  if (!live) { rlo = a.n_q; rhi = a.n_q - 1; }
  int t_lo, t_hi, dummy;
  row_interval_of_key(a, tile_key0, t_lo, dummy);
  row_interval_of_key(a, min(tile_key0 + kBM, a.n_k) - 1, dummy, t_hi);
  int w_lo_max, w_hi_min;
  {
    const int wk0 = min(tile_key0 + wave * 32, a.n_k - 1);
    row_interval_of_key(a, wk0, dummy, w_hi_min);
    // the last lane's interval bounds lo from above; dead keys (beyond n_k) force masking
    w_lo_max = __shfl(rlo, 31);
    w_lo_max = max(w_lo_max, __shfl(rlo, 63));
  }
  const int qt0 = t_lo / kBN, qt1 = t_hi >= t_lo ? t_hi / kBN : qt0 - 1;
  const int ntiles = qt1 - qt0 + 1;
  const int niter = ntiles > 0 ? ntiles * a.group : 0;

  // K, V rows of this lane's key as B operands (k index along d)
  u32x4 kreg[8], vreg[8];
  {
    const int64_t off = (int64_t)(a.k_row0 + keyc) * a.kv_ts + (int64_t)kvh * a.kv_hs + half * 8;
    const uint16_t* kp = reinterpret_cast<const uint16_t*>(a.k) + off;
    const uint16_t* vp = reinterpret_cast<const uint16_t*>(a.v) + off;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      kreg[ks] = *reinterpret_cast<const u32x4*>(kp + ks * 16);
      vreg[ks] = *reinterpret_cast<const u32x4*>(vp + ks * 16);
    }
  }
  const float c = a.scale * kLog2e;

  f32x16 dk[4], dv[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dk[db][i] = 0.f; dv[db][i] = 0.f; }

  char* qtile = smem;
  char* dotile = smem + kTileBytes;
  char* qttile = smem + 2 * kTileBytes;
  char* dottile = smem + 3 * kTileBytes;
  float* stat = reinterpret_cast<float*>(smem + 4 * kTileBytes);   // [0..63] -LSE*log2e, [64..127] delta

  const uint16_t* qbase = reinterpret_cast<const uint16_t*>(a.q) + (int64_t)a.q_row0 * a.q_ts;
  const uint16_t* dobase = reinterpret_cast<const uint16_t*>(a.d_o) + (int64_t)a.q_row0 * a.Hq * 128;

  TileRegs qr, dor;
  float statreg = 0.f;
  auto prefetch = [&](int it) {
    const int hg = it / ntiles, qt = qt0 + it % ntiles;
    const int h = kvh * a.group + hg;
    tile_load(qr, qbase + (int64_t)h * a.q_hs, a.q_ts, qt * kBN, a.n_q, tid);
    tile_load(dor, dobase + (int64_t)h * 128, (int64_t)a.Hq * 128, qt * kBN, a.n_q, tid);
    if (tid < 128) {
      const int rr = a.q_row0 + min(qt * kBN + (tid & 63), a.n_q - 1);
      if (tid < 64) {
        const float L = a.lse_final[(int64_t)h * a.lse_hs + rr];
        statreg = L == -INFINITY ? -INFINITY : -L * kLog2e;
      } else {
        statreg = a.delta[(int64_t)h * a.lse_hs + rr];
      }
    }
  };
  if (niter > 0) prefetch(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);  /* vmcnt(0) */   // K, V, first tile landed (see the dq kernel)

  for (int it = 0; it < niter; ++it) {
    __syncthreads();
    tile_store_n(qr, qtile, tid);
    tile_store_t(qr, qttile, tid);
    tile_store_n(dor, dotile, tid);
    tile_store_t(dor, dottile, tid);
    if (tid < 128) stat[tid] = statreg;
    __syncthreads();
    const int q0 = (qt0 + it % ntiles) * kBN;
    if (it + 1 < niter) prefetch(it + 1);
    const bool need_mask = q0 < w_lo_max || q0 + kBN - 1 > w_hi_min;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 s, dp;
#pragma unroll
      for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        s = mfma32(tile_n_read(qtile, qb, ks, lane), kreg[ks], s);
        dp = mfma32(tile_n_read(dotile, qb, ks, lane), vreg[ks], dp);
      }
      float p[16], ds[16];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int qoff = qb * 32 + g4 * 8 + half * 4;    // tile-relative query of C register 4*g4
        const float4 nl = *reinterpret_cast<const float4*>(stat + qoff);
        const float4 dl = *reinterpret_cast<const float4*>(stat + 64 + qoff);
        const float nls[4] = {nl.x, nl.y, nl.z, nl.w}, dls[4] = {dl.x, dl.y, dl.z, dl.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = g4 * 4 + e;
          float sv = s[i];
          if (need_mask) {
            const int qrow = q0 + qoff + e;
            if (qrow < rlo || qrow > rhi) sv = -INFINITY;
          }
          p[i] = __builtin_amdgcn_exp2f(fmaf(sv, c, nls[e]));
          ds[i] = p[i] * (dp[i] - dls[e]);
        }
      }
      const u32x4 pb0 = mk4(pack2(p[0], p[1]), pack2(p[2], p[3]), pack2(p[4], p[5]), pack2(p[6], p[7]));
      const u32x4 pb1 = mk4(pack2(p[8], p[9]), pack2(p[10], p[11]), pack2(p[12], p[13]), pack2(p[14], p[15]));
      const u32x4 sb0 = mk4(pack2(ds[0], ds[1]), pack2(ds[2], ds[3]), pack2(ds[4], ds[5]), pack2(ds[6], ds[7]));
      const u32x4 sb1 = mk4(pack2(ds[8], ds[9]), pack2(ds[10], ds[11]), pack2(ds[12], ds[13]), pack2(ds[14], ds[15]));
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        dv[db] = mfma32(tile_t_read(dottile, db, qb * 2 + 0, lane), pb0, dv[db]);
        dv[db] = mfma32(tile_t_read(dottile, db, qb * 2 + 1, lane), pb1, dv[db]);
        dk[db] = mfma32(tile_t_read(qttile, db, qb * 2 + 0, lane), sb0, dk[db]);
        dk[db] = mfma32(tile_t_read(qttile, db, qb * 2 + 1, lane), sb1, dk[db]);
      }
    }
  }

  if (!live) return;
  const int64_t off = ((int64_t)(a.k_row0 + key) * a.Hkv + kvh) * 128 + half * 4;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      float4* pk = reinterpret_cast<float4*>(a.dk + off + db * 32 + g4 * 8);
      float4* pv = reinterpret_cast<float4*>(a.dv + off + db * 32 + g4 * 8);
      float4 xk = make_float4(a.scale * dk[db][g4 * 4 + 0], a.scale * dk[db][g4 * 4 + 1],
                              a.scale * dk[db][g4 * 4 + 2], a.scale * dk[db][g4 * 4 + 3]);
      float4 xv = make_float4(dv[db][g4 * 4 + 0], dv[db][g4 * 4 + 1], dv[db][g4 * 4 + 2], dv[db][g4 * 4 + 3]);
      if (a.accumulate) {
        const float4 ok = *pk, ov = *pv;
        xk.x += ok.x; xk.y += ok.y; xk.z += ok.z; xk.w += ok.w;
        xv.x += ov.x; xv.y += ov.y; xv.z += ov.z; xv.w += ov.w;
      }
      *pk = xk;
      *pv = xv;
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
    const dim3 g((a.n_k + kBM - 1) / kBM, a.Hkv), b(256);
    const size_t smem = 4 * kTileBytes + 128 * sizeof(float);
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dkdv_bf16_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (attr != hipSuccess) return attr;
    bwd_dkdv_bf16_kernel<<<g, b, smem, stream>>>(a);
  }
  return hipGetLastError();
}

}  // namespace mmsp
