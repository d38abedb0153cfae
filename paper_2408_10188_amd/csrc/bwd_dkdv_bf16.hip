// Backward ring step, dK/dV kernel (key-stationary) on bf16 matrix cores, head_dim 128.
//
// Workgroup = 4 wavefronts = 128 keys of one KV head; wavefront w owns 32 keys and keeps their
// K and V rows (MFMA B operands, 64 VGPRs) and the dK^T / dV^T accumulators (2 x 128 d x 32
// keys, 128 accumulator registers) for the whole call.  It streams 64-row tiles of Q and dO of
// every query head of the group through a two-stage LDS ring filled by asynchronous
// global->LDS copies: the natural tiles straight from the caller's tensors, the transposed
// ones (Q^T, dO^T) from tile images that the call pre-builds in the workspace, and the per-row
// statistics (-LSE*log2e, delta) from padded copies there.  Per 32-query block:
//   S = Q K^T, dP = dO V^T           (A = Q / dO tile from LDS, B = K / V registers)
//   P = exp2(S*c - LSE*log2e), dS = P * (dP - delta)     in S's register layout (lane = key)
//   dV^T += dO^T P,  dK^T += Q^T dS  (A = transposed tile from LDS, B = P / dS from registers)
// One wavefront per SIMD: the arithmetic of one block is written next to the matrix work of
// the neighbouring block so the scheduler can overlap them.
#include "mfma_tiles.h"

namespace mmsp {
namespace {

constexpr int kKeys = 128;          // keys per workgroup
constexpr int kBQ = 64;             // query rows per streamed tile
constexpr int kCopies = 4;          // 16 copies per tile / 4 wavefronts
constexpr int kStage = 4 * kTileBytes;

__device__ __forceinline__ void dma4(const char* gptr, char* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 4, 0, 0);
}

// kMask = false: the host has checked that every (query, key) pair of the block is visible and
// that n_q is a multiple of the tile length, so no tile needs masking.
template <bool kMask>
__global__ __launch_bounds__(256, 1) void bwd_dkdv_bf16_kernel(StepArgs a, BwdWorkspace w, int n_kt, int xcd_per_kv) {
  __shared__ __attribute__((aligned(1024))) char stage0[kStage];   // Q TileN | dO TileN | Q^T TileT | dO^T TileT
  __shared__ __attribute__((aligned(1024))) char stage1[kStage];
  __shared__ __attribute__((aligned(1024))) float stat0[256];      // [0,64) -LSE*log2e, [64,128) delta, rest unused
  __shared__ __attribute__((aligned(1024))) float stat1[256];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;

  int kvh, kt;
  if (xcd_per_kv > 0) {             // workgroups of one KV head share an XCD (its L2 then serves the Q/dO stream once)
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    kvh = xcd / xcd_per_kv;
    kt = slot * xcd_per_kv + (xcd % xcd_per_kv);
    if (kt >= n_kt) return;
  } else {
    kvh = blockIdx.x / n_kt;
    kt = blockIdx.x % n_kt;
  }
  const int tile_key0 = kt * kKeys;
  const int key = tile_key0 + wave * 32 + col;           // block-relative key of this lane
  const bool live = key < a.n_k;
  const int keyc = min(key, a.n_k - 1);

  int rlo, rhi;                                          // query rows that see this lane's key
  row_interval_of_key(a, keyc, rlo, rhi);
  if (!live) { rlo = a.n_q; rhi = a.n_q - 1; }
  int t_lo, t_hi, dummy;
  row_interval_of_key(a, tile_key0, t_lo, dummy);
  row_interval_of_key(a, min(tile_key0 + kKeys, a.n_k) - 1, dummy, t_hi);
  int w_lo_max, w_hi_min;
  {
    const int wk0 = min(tile_key0 + wave * 32, a.n_k - 1);
    row_interval_of_key(a, wk0, dummy, w_hi_min);
    w_lo_max = __shfl(rlo, 31);                          // last key of the wavefront (n_q for a dead key: always mask)
  }
  // wavefront-uniform values, pinned to scalar registers so that the loop control is scalar too
  t_lo = __builtin_amdgcn_readfirstlane(t_lo);
  t_hi = __builtin_amdgcn_readfirstlane(t_hi);
  w_lo_max = __builtin_amdgcn_readfirstlane(w_lo_max);
  w_hi_min = __builtin_amdgcn_readfirstlane(w_hi_min);
  const int qt0 = t_lo / kBQ, qt1 = t_hi >= t_lo ? t_hi / kBQ : qt0 - 1;
  const int ntiles = qt1 - qt0 + 1;
  const int niter = ntiles > 0 ? ntiles * a.group : 0;

  // ---- asynchronous tile fetch ----
  const char* qbase = reinterpret_cast<const char*>(a.q) + (int64_t)a.q_row0 * a.q_ts * 2;
  const char* dobase = reinterpret_cast<const char*>(a.d_o) + (int64_t)a.q_row0 * a.Hq * 256;
  const int64_t q_tile_bytes = (int64_t)kBQ * a.q_ts * 2, do_tile_bytes = (int64_t)kBQ * a.Hq * 256;
  const DmaOffs<kCopies> qoff_full = dma_n_offsets<kCopies>(a.q_ts, kBQ, wave, lane);
  const DmaOffs<kCopies> dooff_full = dma_n_offsets<kCopies>((int64_t)a.Hq * 128, kBQ, wave, lane);
  auto fetch = [&](int hg, int qt, char* stage, float* stat) {
    const int h = kvh * a.group + hg;
    const int left = a.n_q - qt * kBQ;
    const char* qp = qbase + (int64_t)h * a.q_hs * 2 + (int64_t)qt * q_tile_bytes;
    const char* dp = dobase + (int64_t)h * 256 + (int64_t)qt * do_tile_bytes;
    if (left >= kBQ) {
      dma_tile_n<kCopies>(qp, qoff_full, stage, wave);
      dma_tile_n<kCopies>(dp, dooff_full, stage + kTileBytes, wave);
    } else {                                             // ragged last tile: rows past the end repeat the last row
      dma_tile_n<kCopies>(qp, dma_n_offsets<kCopies>(a.q_ts, left, wave, lane), stage, wave);
      dma_tile_n<kCopies>(dp, dma_n_offsets<kCopies>((int64_t)a.Hq * 128, left, wave, lane), stage + kTileBytes, wave);
    }
    const int64_t img = ((int64_t)h * w.n_qtiles + qt) * kImageBytes;
    dma_tile_image<kCopies>(w.qt + img, stage + 2 * kTileBytes, wave, lane);
    dma_tile_image<kCopies>(w.dot + img, stage + 3 * kTileBytes, wave, lane);
    // statistics: wavefront 0 -> -LSE*log2e, 1 -> delta (2 and 3 repeat them into the unused half)
    const float* src = ((wave & 1) ? w.dl : w.nl2) + (int64_t)h * w.n_qtiles * kBQ + qt * kBQ + lane;
    dma4(reinterpret_cast<const char*>(src), reinterpret_cast<char*>(stat + wave * 64));
  };
  if (niter > 0) fetch(0, qt0, stage0, stat0);

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

  // LDS read offsets, fixed for the whole call
  int na[8], ta[4];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) na[ks] = tile_n_offset(col, ks * 2 + half);         // + qb*8192 (+ kTileBytes for dO)
#pragma unroll
  for (int x = 0; x < 4; ++x) ta[x] = 2 * kTileBytes + tile_t_offset(col, x * 2 + half);   // + db*4096 (+ kTileBytes for dO^T)

  // (head of the group, query tile) of the tile being computed and of the one being fetched
  int cur_qt = qt0, nxt_hg = 0, nxt_qt = qt0;
  auto advance = [&](int& hg, int& qt) { if (++qt > qt1) { qt = qt0; ++hg; } };
  if (niter > 0) advance(nxt_hg, nxt_qt);

  // One 64-row tile.  The two 32-query blocks are software-pipelined inside the wavefront: the
  // exp / dS arithmetic of one block is issued between the MFMAs of the other, so the vector
  // ALU works while the matrix pipe is busy (there is only one wavefront per SIMD to overlap).
  auto tile_body = [&](int it, const char* cur, const float* stat, char* nxt, float* nstat) {
    // own copies of this tile have landed; after the barrier everybody's have, and everybody
    // is done reading the other stage, which is then refilled
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): only this tile's copies are in flight here
    lds_barrier();
    if (it + 1 < niter) fetch(nxt_hg, nxt_qt, nxt, nstat);
    advance(nxt_hg, nxt_qt);
    const int q0 = cur_qt * kBQ;
    if (++cur_qt > qt1) cur_qt = qt0;
    // masked variant: rows outside [rlo, rhi] of this lane's key are hidden; tiles that lie
    // wholly inside every key's interval get an interval that hides nothing
    const bool need_mask = kMask && (q0 < w_lo_max || q0 + kBQ - 1 > w_hi_min);
    const int m_base = need_mask ? q0 - rlo : 0;               // (row - rlo) as unsigned must be <= m_span
    const unsigned m_span = need_mask ? (unsigned)(rhi - rlo) : 0x7fffffffu;   // rhi < rlo -> huge -> fix below
    const bool m_none = need_mask && rhi < rlo;                // this key sees no row at all

    f32x16 s0, dp0, s1, dp1;
    uint32_t pw0[8], sw0[8], pw1[8], sw1[8];          // packed P / dS of the two blocks (B operands)

    // operand of the j-th S/dP MFMA of block qb: even j -> Q tile (x K), odd j -> dO tile (x V)
    auto sdp_operand = [&](int qb, int j) {
      return *reinterpret_cast<const u32x4*>(cur + na[j >> 1] + qb * 8192 + (j & 1) * kTileBytes);
    };
    // operand of the j-th dV/dK MFMA of block qb: j = t*8 + db*2 + x, x = 0 -> dO^T (x P), 1 -> Q^T (x dS)
    auto dvdk_operand = [&](int qb, int j) {
      const int t = j >> 3, db = (j >> 1) & 3, x = j & 1;
      return *reinterpret_cast<const u32x4*>(cur + ta[(qb * 2 + t) ^ db] + db * 4096 + (1 - x) * kTileBytes);
    };
    // element i of a block: P = exp2(S*c - LSE*log2e), dS = P * (dP - delta); packs pairs
    float4 nl, dl;
    float p_prev = 0.f, ds_prev = 0.f;
    auto element = [&](int qb, int i, const f32x16& s, const f32x16& dp, uint32_t* pw, uint32_t* sw) {
      const int qoff = qb * 32 + (i >> 2) * 8 + half * 4;     // tile-relative query of C register 4*(i/4)
      if ((i & 3) == 0) {
        nl = *reinterpret_cast<const float4*>(stat + qoff);
        dl = *reinterpret_cast<const float4*>(stat + 64 + qoff);
      }
      const float nle = (i & 3) == 0 ? nl.x : (i & 3) == 1 ? nl.y : (i & 3) == 2 ? nl.z : nl.w;
      const float dle = (i & 3) == 0 ? dl.x : (i & 3) == 1 ? dl.y : (i & 3) == 2 ? dl.z : dl.w;
      float sv = s[i];
      if (kMask) {   // branch-free select
        const bool hidden = (unsigned)(m_base + qoff + (i & 3)) > m_span || m_none;
        sv = hidden ? -INFINITY : sv;
      }
      const float p = __builtin_amdgcn_exp2f(fmaf(sv, c, nle));
      const float ds = p * (dp[i] - dle);
      if (i & 1) { pw[i >> 1] = pack2(p_prev, p); sw[i >> 1] = pack2(ds_prev, ds); }
      else { p_prev = p; ds_prev = ds; }
    };

    u32x4 op[16];
    // ---- region A: S0, dP0 (matrix pipe only) ----
#pragma unroll
    for (int j = 0; j < 16; ++j) op[j] = sdp_operand(0, j);
#pragma unroll
    for (int i = 0; i < 16; ++i) { s0[i] = 0.f; dp0[i] = 0.f; s1[i] = 0.f; dp1[i] = 0.f; }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (j & 1) dp0 = mfma32(op[j], vreg[j >> 1], dp0); else s0 = mfma32(op[j], kreg[j >> 1], s0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- region B: S1, dP1 on the matrix pipe, element j of block 0 on the vector ALU ----
#pragma unroll
    for (int j = 0; j < 8; ++j) op[j] = sdp_operand(1, j);
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (j & 1) dp1 = mfma32(op[j], vreg[j >> 1], dp1); else s1 = mfma32(op[j], kreg[j >> 1], s1);
      if (j < 8) op[8 + j] = sdp_operand(1, 8 + j);
      element(0, j, s0, dp0, pw0, sw0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---- region C: dV, dK of block 0 on the matrix pipe, element j of block 1 on the vector ALU ----
    {
      const u32x4 pb[2] = {mk4(pw0[0], pw0[1], pw0[2], pw0[3]), mk4(pw0[4], pw0[5], pw0[6], pw0[7])};
      const u32x4 sb[2] = {mk4(sw0[0], sw0[1], sw0[2], sw0[3]), mk4(sw0[4], sw0[5], sw0[6], sw0[7])};
#pragma unroll
      for (int j = 0; j < 8; ++j) op[j] = dvdk_operand(0, j);
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int t = j >> 3, db = (j >> 1) & 3;
        if (j & 1) dk[db] = mfma32(op[j], sb[t], dk[db]); else dv[db] = mfma32(op[j], pb[t], dv[db]);
        if (j < 8) op[8 + j] = dvdk_operand(0, 8 + j);
        element(1, j, s1, dp1, pw1, sw1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // ---- region D: dV, dK of block 1 (matrix pipe only) ----
    {
      const u32x4 pb[2] = {mk4(pw1[0], pw1[1], pw1[2], pw1[3]), mk4(pw1[4], pw1[5], pw1[6], pw1[7])};
      const u32x4 sb[2] = {mk4(sw1[0], sw1[1], sw1[2], sw1[3]), mk4(sw1[4], sw1[5], sw1[6], sw1[7])};
#pragma unroll
      for (int j = 0; j < 16; ++j) op[j] = dvdk_operand(1, j);
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int t = j >> 3, db = (j >> 1) & 3;
        if (j & 1) dk[db] = mfma32(op[j], sb[t], dk[db]); else dv[db] = mfma32(op[j], pb[t], dv[db]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // Two bodies per trip so that LDS offsets are immediates; the odd last tile is peeled so
  // that no accumulator crosses a conditional inside the loop.
  int it = 0;
  for (; it + 1 < niter; it += 2) {
    tile_body(it, stage0, stat0, stage1, stat1);
    tile_body(it + 1, stage1, stat1, stage0, stat0);
  }
  if (it < niter) tile_body(it, stage0, stat0, stage1, stat1);

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

hipError_t launch_bwd_dkdv_bf16(const StepArgs& a, const BwdWorkspace& w, hipStream_t stream) {
  const int n_kt = (a.n_k + kKeys - 1) / kKeys;
  int xcd_per_kv = 0, n_blocks = n_kt * a.Hkv;
  if (8 % a.Hkv == 0) {
    xcd_per_kv = 8 / a.Hkv;
    n_blocks = 8 * ((n_kt + xcd_per_kv - 1) / xcd_per_kv);
  }
  const bool no_mask = a.mask == 0 && a.cu == nullptr && a.n_q % kBQ == 0;
  if (no_mask) bwd_dkdv_bf16_kernel<false><<<dim3(n_blocks), dim3(256), 0, stream>>>(a, w, n_kt, xcd_per_kv);
  else bwd_dkdv_bf16_kernel<true><<<dim3(n_blocks), dim3(256), 0, stream>>>(a, w, n_kt, xcd_per_kv);
  return hipGetLastError();
}

}  // namespace mmsp
