// Backward ring step, dQ kernel (query-stationary) on bf16 matrix cores, head_dim 128.
//
// Same skeleton as the forward kernel: a workgroup is 8 wavefronts = 256 query rows of one
// head, two wavefronts per SIMD; wavefront w owns 32 rows and keeps their Q and dO (MFMA B
// operands), the dQ^T accumulator (128 d x 32 queries) and the two row statistics (-LSE*log2e,
// delta) in registers for the whole call.  64-key tiles of K and V stream through a three-stage
// LDS ring filled by asynchronous global->LDS copies straight from the caller's tensors (natural
// orientation; the third product reads K back transposed with ds_read_b64_tr_b16).
//   S^T[key][query]  = K . Q^T            P^T = exp2(S^T * c - LSE*log2e)   (final LSE: no running max)
//   dP^T[key][query] = V . dO^T           dS^T = P^T * (dP^T - delta)
//   dQ^T[d][query]  += K^T . dS^T         (B operand = dS^T straight from registers)
// S and dP are recomputed here although the dK/dV kernel computes them too: that buys exclusive
// ownership of dQ, hence no floating-point atomics and bit-reproducible results.
#include "mfma_tiles.h"

namespace mmsp {
namespace {

constexpr int kWaves = 8;
constexpr int kBM = 32 * kWaves;   // query rows per workgroup
constexpr int kBN = 64;            // keys per tile
constexpr int kCopies = 16 / kWaves;

__global__ __launch_bounds__(64 * kWaves, 2) void bwd_dq_bf16_kernel(StepArgs a, int n_qt, int xcd_per_kv) {
  // LDS map: the three K slots in [0, 48 KiB), the three V slots in [48 KiB, 96 KiB); slots are
  // selected at compile time (the loop is unrolled three tiles deep).  An LDS instruction's
  // immediate offset reaches 64 KiB, so the V reads go through per-lane base registers that
  // already hold the V region's start (va below).
  constexpr int kVRegion = 3 * kTileBytes;
  __shared__ __attribute__((aligned(1024))) char lds[6 * kTileBytes];
  char* const ks0 = lds;                                // K tiles, TileS
  char* const ks1 = ks0 + kTileBytes;
  char* const ks2 = ks1 + kTileBytes;
  char* const vs0 = lds + kVRegion;                     // V tiles, TileS
  char* const vs1 = vs0 + kTileBytes;
  char* const vs2 = vs1 + kTileBytes;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);   // the same value in a scalar register (LDS targets of the copies)
  const int half = lane >> 5, col = lane & 31;

  // workgroup -> (head, query tile): the workgroups of a KV head share an XCD, later (heavier
  // under the causal mask) query tiles first
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
  const int64_t kv_off = ((int64_t)a.k_row0 * a.kv_ts + (int64_t)kvh * a.kv_hs) * 2;
  const char* kbase = reinterpret_cast<const char*>(a.k) + kv_off;
  const char* vbase = reinterpret_cast<const char*>(a.v) + kv_off;
  const int64_t tile_bytes = (int64_t)kBN * a.kv_ts * 2;
  // Source of a copy = the tile's address (wavefront-uniform, advanced by scalar additions) + a
  // per-lane offset that is the same for every whole tile.
  const DmaOffs<kCopies> off_full = dma_s_offsets<kCopies>(a.kv_ts, kBN, wave, lane);
  // the last key tile of the block may be ragged: rows past the end repeat the last row
  const int kt_ragged = a.n_k % kBN != 0 ? a.n_k / kBN : -1;
  const DmaOffs<kCopies> off_ragged = dma_s_offsets<kCopies>(a.kv_ts, kt_ragged >= 0 ? a.n_k % kBN : kBN, wave, lane);
  int f_kt = kt0;                                       // tile the next fetch takes
  int64_t f_tile = (int64_t)kt0 * tile_bytes;           // its byte offset from kbase / vbase
  auto fetch = [&](char* kdst, char* vdst) {            // past the end the last tile is fetched again
    constexpr int W = 16 / kCopies;
    const bool ragged = f_kt == kt_ragged;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) dma16(kbase + f_tile, ragged ? off_ragged.o[i] : off_full.o[i], kdst, (wave_s + i * W) * 1024);
#pragma unroll
    for (int i = 0; i < kCopies; ++i) dma16(vbase + f_tile, ragged ? off_ragged.o[i] : off_full.o[i], vdst, (wave_s + i * W) * 1024);
    if (f_kt < kt1) {
      ++f_kt;
      f_tile += tile_bytes;
    }
  };
  if (kt0 <= kt1) {
    fetch(ks0, vs0);
    fetch(ks1, vs1);
  }

  // Q and dO as B operands: k-step ks covers d = ks*16 .. +16, this lane holds 8 of them
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

  // LDS read offsets inside a tile, fixed for the whole call: K / V operand k-step ks (rows
  // +32 -> +8192 bytes); K^T operand of d block db, first / second transposing
  // read (16 keys further -> +4096 bytes)
  int ka[8], va[8], ta[4][2];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    ka[ks] = tile_s_offset(col, ks * 2 + half);
    va[ks] = ka[ks] + kVRegion;                         // same offset + start of the V region, kept opaque
    asm volatile("" : "+v"(va[ks]));
  }
#pragma unroll
  for (int db = 0; db < 4; ++db) {
    ta[db][0] = tile_s_tr_offset(lane, db, 0);
    ta[db][1] = tile_s_tr_offset(lane, db, 1);
  }

  auto tile_body = [&](int kt, const char* kcur, const char* vcur, char* krefill, char* vrefill) {
    // Own copies of tile kt have landed (the newest tile's may still be in flight); after the
    // barrier everybody's have, and everybody is done with the stage about to be refilled.  Every
    // tile issues one whole group of copies (past the end it fetches the last tile again, into a
    // stage nobody reads any more), so the wait is the same constant everywhere.
    __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * kCopies));
    lds_barrier();
    fetch(krefill, vrefill);
    const int k0 = kt * kBN;
    const bool need_mask = k0 < w_lo_max || k0 + kBN - 1 > w_hi_min;

#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 s, dp;
#pragma unroll
      for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        s = mfma32(*reinterpret_cast<const u32x4*>(kcur + ka[ks] + kb * 8192), qreg[ks], s);
        dp = mfma32(*reinterpret_cast<const u32x4*>(vcur - kVRegion + va[ks] + kb * 8192), doreg[ks], dp);
      }
      // K^T operands of the third product: issued now, they land during the exp / dS arithmetic
      u32x4 top[8];
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int tq = 0; tq < 2; ++tq) {
          const u32x2 v0 = lds_read_tr(kcur + ta[db][0] + (kb * 2 + tq) * 4096);
          const u32x2 v1 = lds_read_tr(kcur + ta[db][1] + (kb * 2 + tq) * 4096);
          top[2 * db + tq] = mk4(v0.x, v0.y, v1.x, v1.y);
        }
      __builtin_amdgcn_sched_barrier(0);
      if (need_mask) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = k0 + kb * 32 + (i >> 2) * 8 + half * 4 + (i & 3);
          s[i] = (key < lo || key > hi) ? -INFINITY : s[i];
        }
      }
      uint32_t w[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[2 * j], c, neg_l2));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[2 * j + 1], c, neg_l2));
        w[j] = pack2(p0 * (dp[2 * j] - Dl), p1 * (dp[2 * j + 1] - Dl));
      }
      const u32x4 b0 = mk4(w[0], w[1], w[2], w[3]);
      const u32x4 b1 = mk4(w[4], w[5], w[6], w[7]);
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        dq[db] = mfma32(top[2 * db], b0, dq[db]);
        dq[db] = mfma32(top[2 * db + 1], b1, dq[db]);
      }
    }
  };

  // Three bodies per trip so that every stage is a compile-time constant (the compiler then sees
  // that the reads of one stage cannot alias the copies in flight into another); the
  // steady-state loop has no conditional bodies.
  int kt = kt0;
  for (; kt + 2 <= kt1; kt += 3) {
    tile_body(kt, ks0, vs0, ks2, vs2);
    tile_body(kt + 1, ks1, vs1, ks0, vs0);
    tile_body(kt + 2, ks2, vs2, ks1, vs1);
  }
  if (kt <= kt1) {
    tile_body(kt, ks0, vs0, ks2, vs2);
    if (kt + 1 <= kt1) tile_body(kt + 1, ks1, vs1, ks0, vs0);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                    // drain the copies issued past the end

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

hipError_t launch_bwd_dq_bf16(const StepArgs& a, hipStream_t stream) {
  const int n_qt = (a.n_q + kBM - 1) / kBM;
  int xcd_per_kv = 0, n_blocks = n_qt * a.Hq;
  if (8 % a.Hkv == 0) {
    xcd_per_kv = 8 / a.Hkv;
    n_blocks = 8 * ((a.group * n_qt + xcd_per_kv - 1) / xcd_per_kv);
  }
  bwd_dq_bf16_kernel<<<dim3(n_blocks), dim3(64 * kWaves), 0, stream>>>(a, n_qt, xcd_per_kv);
  return hipGetLastError();
}

}  // namespace mmsp
