// Forward ring step on bf16 matrix cores, head_dim 128.
//
// Workgroup = 8 wavefronts = 256 query rows of one head (two wavefronts per SIMD, so one
// wavefront's softmax arithmetic overlaps the other's matrix work).  Wavefront w owns 32 rows
// and keeps their Q (MFMA B operands, 32 VGPRs), the O^T accumulator (128 d x 32 queries, 64
// VGPRs) and the softmax statistics in registers for the whole call.  K and V^T tiles of 64
// keys stream through a three-stage LDS ring filled by asynchronous global->LDS copies: K
// straight from the caller's tensor (swizzled by permuting which chunk a lane fetches), V^T
// from the pre-transposed tile images in the workspace.
//   S^T[key][query] = K . Q^T            (A = K tile from LDS, B = Q registers)
//   online softmax down the key axis, which is in-lane in S^T's register layout
//   O^T[d][query]  += V^T . P^T          (A = V^T tile from LDS, B = P^T straight from registers)
// Tiles wholly outside every row's visible key interval are skipped; only tiles that cut an
// interval boundary (the causal diagonal, a document start) pay for masking.
#include "mfma_tiles.h"

namespace mmsp {
namespace {

constexpr int kWaves = 8;
constexpr int kBM = 32 * kWaves;   // query rows per workgroup
constexpr int kBN = 64;            // keys per tile
constexpr int kCopies = 16 / kWaves;
constexpr int kStageBytes = 2 * kTileBytes;

// vmcnt(n) with expcnt / lgkmcnt left alone
__device__ __forceinline__ void wait_vmcnt_0() { __builtin_amdgcn_s_waitcnt(0x0F70); }
__device__ __forceinline__ void wait_vmcnt_tile() { __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * kCopies)); }

template <bool kAccum>
__global__ __launch_bounds__(64 * kWaves, 2) void fwd_bf16_kernel(StepArgs a, int n_qt, int xcd_per_kv) {
  __shared__ __attribute__((aligned(1024))) char stage0[kStageBytes];   // K TileN | V^T TileT
  __shared__ __attribute__((aligned(1024))) char stage1[kStageBytes];
  __shared__ __attribute__((aligned(1024))) char stage2[kStageBytes];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;

  // Workgroup -> (head, query tile).  Workgroups are dealt round-robin to the 8 XCDs; the
  // ones that land on the same XCD work on the same KV head so its K/V block stays in that
  // XCD's L2.  Later (heavier under the causal mask) query tiles go first.
  int h, qt;
  if (xcd_per_kv > 0) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int kvh0 = xcd / xcd_per_kv;
    const int item = slot * xcd_per_kv + (xcd % xcd_per_kv);
    if (item >= a.group * n_qt) return;
    h = kvh0 * a.group + item % a.group;
    qt = n_qt - 1 - item / a.group;
  } else {
    h = blockIdx.x % a.Hq;
    qt = n_qt - 1 - blockIdx.x / a.Hq;
  }
  const int kvh = h / a.group;
  const int tile_row0 = qt * kBM;
  const int row = tile_row0 + wave * 32 + col;          // block-relative query row of this lane
  const bool live = row < a.n_q;
  const int rowc = min(row, a.n_q - 1);

  // visible key interval of this lane's row, and of the workgroup / wavefront extremes
  int lo, hi;
  key_interval_of_row(a, rowc, lo, hi);
  int t_lo, t_hi, dummy;
  key_interval_of_row(a, tile_row0, t_lo, dummy);
  key_interval_of_row(a, min(tile_row0 + kBM, a.n_q) - 1, dummy, t_hi);
  int w_lo_max, w_hi_min;                               // wavefront: largest lo, smallest hi
  {
    const int wr0 = min(tile_row0 + wave * 32, a.n_q - 1), wr1 = min(tile_row0 + wave * 32 + 31, a.n_q - 1);
    key_interval_of_row(a, wr0, dummy, w_hi_min);
    key_interval_of_row(a, wr1, w_lo_max, dummy);
  }
  const int kt0 = t_lo / kBN, kt1 = t_hi >= t_lo ? t_hi / kBN : kt0 - 1;   // inclusive tile range

  // ---- asynchronous tile fetch ----
  const char* kbase = reinterpret_cast<const char*>(a.k) + ((int64_t)a.k_row0 * a.kv_ts + (int64_t)kvh * a.kv_hs) * 2;
  const char* vimg = a.ws + (int64_t)kvh * tiles_of(a.n_k) * kImageBytes;
  const int64_t tile_bytes = (int64_t)kBN * a.kv_ts * 2;
  const DmaOffs<kCopies> off_full = dma_n_offsets<kCopies>(a.kv_ts, kBN, wave, lane);
  auto fetch = [&](int kt, char* stage) {
    const int left = a.n_k - kt * kBN;
    const char* kp = kbase + (int64_t)kt * tile_bytes;
    if (left >= kBN) dma_tile_n<kCopies>(kp, off_full, stage, wave);
    else dma_tile_n<kCopies>(kp, dma_n_offsets<kCopies>(a.kv_ts, left, wave, lane), stage, wave);   // ragged last tile
    dma_tile_image<kCopies>(vimg + (int64_t)kt * kImageBytes, stage + kTileBytes, wave, lane);
  };
  if (kt0 <= kt1) fetch(kt0, stage0);
  if (kt0 + 1 <= kt1) fetch(kt0 + 1, stage1);

  // Q as B operands: k-step ks covers d = ks*16 .. +16, this lane holds 8 of them
  u32x4 qreg[8];
  {
    const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + (int64_t)(a.q_row0 + rowc) * a.q_ts +
                         (int64_t)h * a.q_hs + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qreg[ks] = *reinterpret_cast<const u32x4*>(qp + ks * 16);
  }

  f32x16 oacc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
  // Softmax state.  m_ref is the raw-score reference the exponentials are taken against; it
  // follows the running row maximum lazily: it only moves when the maximum has grown by more
  // than kLazy in the exponent (P stays <= 2^kLazy), so the O rescale is rare.
  constexpr float kLazy = 8.f;
  float m_ref = -INFINITY;
  float neg_mc = 0.f;        // -m_ref * c  (0 while m_ref = -inf, so masked scores give exp2(-inf) = 0)
  float l = 0.f;             // this lane's share of the row sum (its 32 of every 64 keys)
  const float c = a.scale * kLog2e;
  const float lazy_raw = kLazy / c;

  // LDS read offsets inside a stage, fixed for the whole call: K operand k-step ks (rows +32 ->
  // +8192 bytes), V^T operand chunk pair x = g ^ db (d block db -> +4096 bytes)
  int ka[8], va[4];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) ka[ks] = tile_n_offset(col, ks * 2 + half);
#pragma unroll
  for (int x = 0; x < 4; ++x) va[x] = kTileBytes + tile_t_offset(col, x * 2 + half);

  auto tile_body = [&](int kt, const char* cur, char* refill) {
    // Own copies of tile kt have landed (the newest tile's may still be in flight); after the
    // barrier everybody's have, and everybody is done with the stage about to be refilled.
    if (kt < kt1) wait_vmcnt_tile(); else wait_vmcnt_0();
    lds_barrier();
    if (kt + 2 <= kt1) fetch(kt + 2, refill);
    const int k0 = kt * kBN;

    // ---- S^T = K Q^T : two 32-key blocks, their accumulation chains interleaved.  All 16
    // operand reads are issued up front so the MFMAs stream behind the LDS instead of waiting
    // for it pair by pair. ----
    u32x4 kop[16];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      kop[2 * ks] = *reinterpret_cast<const u32x4*>(cur + ka[ks]);
      kop[2 * ks + 1] = *reinterpret_cast<const u32x4*>(cur + ka[ks] + 8192);
    }
    __builtin_amdgcn_sched_barrier(0);
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      s[0] = mfma32(kop[2 * ks], qreg[ks], s[0]);
      s[1] = mfma32(kop[2 * ks + 1], qreg[ks], s[1]);
    }
    // V^T operands for the second product: issued now, they land while the softmax runs
    u32x4 vop[16];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int db = 0; db < 4; ++db) vop[g * 4 + db] = *reinterpret_cast<const u32x4*>(cur + va[g ^ db] + db * 4096);
    __builtin_amdgcn_sched_barrier(0);

    // ---- mask (only tiles that cut an interval boundary) ----
    if (k0 < w_lo_max || k0 + kBN - 1 > w_hi_min) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = k0 + kb * 32 + (i >> 2) * 8 + half * 4 + (i & 3);
          if (key < lo || key > hi) s[kb][i] = -INFINITY;
        }
    }

    // ---- online softmax along keys ----
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kb][i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (__any(mx > m_ref + lazy_raw)) {                 // rare after the first tiles
      const float m_new = fmaxf(m_ref, mx);
      const float alpha = m_new == m_ref ? 1.f : __builtin_amdgcn_exp2f((m_ref - m_new) * c);   // -inf -> 0
      m_ref = m_new;
      neg_mc = m_new == -INFINITY ? 0.f : -m_new * c;
      l *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
    }
    u32x4 pb[4];
    float ps[4] = {0.f, 0.f, 0.f, 0.f};                 // fp32 sums of the unrounded P (LSE needs 1e-3)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      uint32_t w[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kb][2 * j], c, neg_mc));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kb][2 * j + 1], c, neg_mc));
        ps[(2 * j) & 3] += p0;
        ps[(2 * j + 1) & 3] += p1;
        w[j] = pack2(p0, p1);
      }
      pb[kb * 2 + 0] = mk4(w[0], w[1], w[2], w[3]);
      pb[kb * 2 + 1] = mk4(w[4], w[5], w[6], w[7]);
    }
    l += (ps[0] + ps[1]) + (ps[2] + ps[3]);

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int db = 0; db < 4; ++db)
        oacc[db] = mfma32(vop[g * 4 + db], pb[g], oacc[db]);
  };

  // Three bodies per trip so that every LDS offset is an immediate.
  for (int kt = kt0; kt <= kt1; kt += 3) {
    tile_body(kt, stage0, stage2);
    if (kt + 1 <= kt1) tile_body(kt + 1, stage1, stage0);
    if (kt + 2 <= kt1) tile_body(kt + 2, stage2, stage1);
  }
  const float m = m_ref;

  // ---- epilogue ----
  l += __shfl_xor(l, 32);
  const bool empty = !(l > 0.f);
  const float inv = empty ? 0.f : 1.f / l;
  const float lse_part = empty ? -INFINITY : (m * c + __builtin_amdgcn_logf(l)) * kLn2;   // v_log_f32 is log2
  if (!live) return;
  const int64_t r = a.q_row0 + row;
  float* op = a.o + (r * a.Hq + h) * 128 + half * 4;
  float* lp = a.lse + (int64_t)h * a.lse_hs + r;
  float wa = 0.f, wb = inv;
  if (kAccum) {
    const float la = *lp;
    const float mm = fmaxf(la, lse_part);
    if (mm == -INFINITY) return;                        // both sides empty
    const float ea = __expf(la - mm), eb = __expf(lse_part - mm);
    const float tot = ea + eb;
    wa = ea / tot;
    wb = eb / tot * inv;
    if (half == 0) *lp = mm + __logf(tot);
  } else {
    if (half == 0) *lp = lse_part;
  }
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      float4* dst = reinterpret_cast<float4*>(op + db * 32 + g4 * 8);
      float4 o = make_float4(oacc[db][g4 * 4 + 0] * wb, oacc[db][g4 * 4 + 1] * wb, oacc[db][g4 * 4 + 2] * wb,
                             oacc[db][g4 * 4 + 3] * wb);
      if (kAccum) {
        const float4 old = *dst;
        o.x += wa * old.x; o.y += wa * old.y; o.z += wa * old.z; o.w += wa * old.w;
      }
      *dst = o;
    }
}

}  // namespace

int64_t fwd_bf16_workspace_bytes(int Hkv, int64_t n_k) { return (int64_t)Hkv * tiles_of(n_k) * kImageBytes; }

hipError_t launch_fwd_bf16(const StepArgs& a, hipStream_t stream) {
  // V^T tile images of the visiting block
  hipError_t e = launch_transpose_tiles(a.v, a.kv_ts, a.kv_hs, a.Hkv, a.k_row0, a.n_k, a.ws, stream);
  if (e != hipSuccess) return e;
  const int n_qt = (a.n_q + kBM - 1) / kBM;
  int xcd_per_kv = 0, n_blocks = n_qt * a.Hq;
  if (8 % a.Hkv == 0) {
    xcd_per_kv = 8 / a.Hkv;
    n_blocks = 8 * ((a.group * n_qt + xcd_per_kv - 1) / xcd_per_kv);
  }
  const dim3 g(n_blocks), b(64 * kWaves);
  if (a.accumulate) fwd_bf16_kernel<true><<<g, b, 0, stream>>>(a, n_qt, xcd_per_kv);
  else fwd_bf16_kernel<false><<<g, b, 0, stream>>>(a, n_qt, xcd_per_kv);
  return hipGetLastError();
}

}  // namespace mmsp
