// Forward ring step on bf16 matrix cores, head_dim 128.
//
// Workgroup = 8 wavefronts = 256 query rows of one head, two wavefronts per SIMD.  Wavefront w
// owns 32 rows and keeps their Q (MFMA B operands, 32 VGPRs), the O^T accumulator (128 d x 32
// queries, 64 VGPRs) and the softmax statistics in registers for the whole call.  K and V tiles
// of 64 keys stream through two three-slot LDS rings filled by asynchronous global->LDS copies
// straight from the caller's tensors (one natural-orientation copy each; V is read back
// transposed by ds_read_b64_tr_b16).
//   S^T[key][query] = K . Q^T            (A = K tile from LDS, B = Q registers)
//   online softmax down the key axis, which is in-lane in S^T's register layout
//   O^T[d][query]  += V^T . P^T          (A = V tile read transposed, B = P^T straight from registers)
//
// One matrix instruction occupies a SIMD's matrix pipe for 32 cycles but its issue port for
// only about 8: up to five or six ordinary vector instructions fit beside it if they are
// independent and interleaved in program order.  The loop is therefore software-pipelined inside
// every wavefront: while the matrix pipe works on P.V of tile t-1 the vector units take the
// maximum and the first half of the exponentials of tile t, and while it works on S of tile t+1
// they take the second half.  The interleaving is written out step by step (one matrix
// instruction per step) and pinned with empty asm statements and scheduling barriers.
// Tiles wholly outside every row's visible key interval are skipped; only tiles that cut an
// interval boundary (the causal diagonal, a document start) pay for masking.
#include "mfma_tiles.h"

namespace mmsp {
namespace {

constexpr int kWaves = 8;
constexpr int kBM = 32 * kWaves;   // query rows per workgroup
constexpr int kBN = 64;            // keys per tile
constexpr int kCopies = 16 / kWaves;
constexpr int kSlots = 3;

template <bool kAccum>
__global__ __launch_bounds__(64 * kWaves, 2) void fwd_bf16_kernel(StepArgs a, int n_qt, int xcd_per_kv) {
  // Tile j (counted from the first visible tile) lives in slot j % 3 of its ring; slots are
  // selected at compile time (the loop is unrolled three tiles deep).  LDS map: the three V slots
  // in [0, 48 KiB), the three K slots in [48 KiB, 96 KiB).  An LDS instruction's immediate offset
  // reaches 64 KiB, so the K reads go through per-lane base registers that already hold the K
  // region's start (ka below) and no read needs an address addition of its own.
  constexpr int kKRegion = 3 * kTileBytes;
  __shared__ __attribute__((aligned(1024))) char lds[6 * kTileBytes];
  char* const vslot0 = lds;                             // V tiles, TileS
  char* const vslot1 = vslot0 + kTileBytes;
  char* const vslot2 = vslot1 + kTileBytes;
  char* const kslot0 = lds + kKRegion;                  // K tiles, TileS
  char* const kslot1 = kslot0 + kTileBytes;
  char* const kslot2 = kslot1 + kTileBytes;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);   // the same value in a scalar register (LDS targets of the copies)
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
  int kt0 = t_lo / kBN, kt1 = t_hi >= t_lo ? t_hi / kBN : kt0 - 1;   // inclusive tile range
  kt0 = __builtin_amdgcn_readfirstlane(kt0);
  kt1 = __builtin_amdgcn_readfirstlane(kt1);
  w_lo_max = __builtin_amdgcn_readfirstlane(w_lo_max);
  w_hi_min = __builtin_amdgcn_readfirstlane(w_hi_min);

  // ---- asynchronous tile fetch ----
  const char* kbase = reinterpret_cast<const char*>(a.k) + ((int64_t)a.k_row0 * a.kv_ts + (int64_t)kvh * a.kv_hs) * 2;
  const char* vbase = reinterpret_cast<const char*>(a.v) + ((int64_t)a.k_row0 * a.kv_ts + (int64_t)kvh * a.kv_hs) * 2;
  const int64_t tile_bytes = (int64_t)kBN * a.kv_ts * 2;
  // Source of a copy = the tile's address (wavefront-uniform, advanced by scalar additions) + a
  // per-lane offset that is the same for every whole tile.  K and V have a cursor each.
  const DmaOffs<kCopies> off_full = dma_s_offsets<kCopies>(a.kv_ts, kBN, wave, lane);
  // the last key tile of the block may be ragged: rows past the end repeat the last row
  const int kt_ragged = a.n_k % kBN != 0 ? a.n_k / kBN : -1;
  const DmaOffs<kCopies> off_ragged = dma_s_offsets<kCopies>(a.kv_ts, kt_ragged >= 0 ? a.n_k % kBN : kBN, wave, lane);
  struct Cursor { int64_t tile; int kt; };              // byte offset of the tile from kbase / vbase, tile index
  auto fetch = [&](Cursor& cu, const char* base, char* dst) {   // the cursor's tile -> slot dst; past the end the last tile again
    constexpr int W = 16 / kCopies;
    const bool ragged = cu.kt == kt_ragged;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) dma16(base + cu.tile, ragged ? off_ragged.o[i] : off_full.o[i], dst, (wave_s + i * W) * 1024);
    if (cu.kt < kt1) {
      ++cu.kt;
      cu.tile += tile_bytes;
    }
  };
  // Copies are issued in groups of 2 kCopies per wavefront so that "all but the newest group"
  // is one s_waitcnt value: {K(kt0), V(kt0)}, {K(kt0+1), K(kt0+2)}, then {K(t+3), V(t+1)} at the
  // top of iteration t.
  const bool any_tile = kt0 <= kt1;
  Cursor kc{(int64_t)kt0 * tile_bytes, kt0}, vc{(int64_t)kt0 * tile_bytes, kt0};
  if (any_tile) {
    fetch(kc, kbase, kslot0);
    fetch(vc, vbase, vslot0);
    fetch(kc, kbase, kslot1);
    fetch(kc, kbase, kslot2);
    // the first iteration multiplies an all-zero P with "the tile before the first": finite zeros
    *reinterpret_cast<u32x4*>(vslot2 + tid * 32) = mk4(0u, 0u, 0u, 0u);
    *reinterpret_cast<u32x4*>(vslot2 + tid * 32 + 16) = mk4(0u, 0u, 0u, 0u);
  }

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

  // LDS read offsets inside a tile, fixed for the whole call: K operand k-step ks (keys +32 ->
  // +8192 bytes); V^T operand of d block db, first / second read (16 keys further -> +4096 bytes)
  int ka[8], va[4][2];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {                       // offset inside a K tile + start of the K region, kept opaque
    ka[ks] = tile_s_offset(col, ks * 2 + half) + kKRegion;
    asm volatile("" : "+v"(ka[ks]));
  }
#pragma unroll
  for (int db = 0; db < 4; ++db) {
    va[db][0] = tile_s_tr_offset(lane, db, 0);
    va[db][1] = tile_s_tr_offset(lane, db, 1);
  }

  f32x16 s[2];               // S^T of the tile whose softmax is being taken: two 32-key blocks
  u32x4 pb[4];               // P^T of the previous tile, packed as the B operands of its four k-steps
#pragma unroll
  for (int g = 0; g < 4; ++g) pb[g] = mk4(0u, 0u, 0u, 0u);

  auto s_product = [&](const char* kt_tile, f32x16 (&out)[2]) {   // all 16 MFMAs of S^T = K Q^T, not interleaved
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) out[kb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      out[0] = mfma32(*reinterpret_cast<const u32x4*>(kt_tile - kKRegion + ka[ks]), qreg[ks], out[0]);
      out[1] = mfma32(*reinterpret_cast<const u32x4*>(kt_tile - kKRegion + ka[ks] + 8192), qreg[ks], out[1]);
    }
  };

  if (any_tile) {
    __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0), lgkmcnt(0): the first tiles have landed, the zeros are written
    lds_barrier();
    s_product(kslot0, s);
  }

  // One iteration: tile t, with V(t-1) in v_prev, K(t+1) in k_next; K(t+3) goes where K(t) was,
  // V(t+1) where V(t-2) was.
  auto iteration = [&](int t, const char* vt, const char* ktile, char* k_refill, char* v_refill) {
    // Own copies of every group but the newest have landed; after the barrier everybody's have,
    // and everybody is done with the slots about to be refilled.  Every iteration issues one
    // whole group (past the end it fetches the last tile again, into slots nobody reads any
    // more), so the wait is the same constant everywhere.
    __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * kCopies));
    lds_barrier();
    fetch(kc, kbase, k_refill);
    fetch(vc, vbase, v_refill);

    const int k0 = t * kBN;
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
    __builtin_amdgcn_sched_barrier(0);

    // Each step below is one MFMA with the reads that feed the MFMA four steps later and its share
    // of the vector work; MMSP_STEP_END pins the values so that neither the optimiser nor the
    // instruction scheduler moves work from one step to another.
#define MMSP_PIN(x) asm volatile("" : "+v"(x))
#define MMSP_STEP_END() __builtin_amdgcn_sched_barrier(0)

    // ================= phase 1: O^T += V(t-1)^T P(t-1)^T  beside  max(t) and the first exponentials of tile t =================
    // (the first iteration multiplies an all-zero P with a slot of zeros)
    float alpha = 1.f;
    bool moved = false;
    uint32_t w[16];          // P^T of tile t, two keys per word
    float ps[4] = {0.f, 0.f, 0.f, 0.f};                 // fp32 sums of the unrounded P (LSE needs 1e-3)
    float mx = -INFINITY, mx_other = -INFINITY;
    auto exp_item = [&](int j) {                        // keys 2j, 2j+1 of the lane's 32
      const f32x16& sv = s[j >> 3];
      const int e = (j & 7) * 2;
      const float p0 = __builtin_amdgcn_exp2f(fmaf(sv[e], c, neg_mc));
      const float p1 = __builtin_amdgcn_exp2f(fmaf(sv[e + 1], c, neg_mc));
      ps[e & 3] += p0;
      ps[(e + 1) & 3] += p1;
      w[j] = pack2(p0, p1);
      MMSP_PIN(ps[e & 3]); MMSP_PIN(ps[(e + 1) & 3]); MMSP_PIN(w[j]);
    };
    {
      u32x2 vq[4][2];        // transposing reads in flight, four steps deep
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        vq[i][0] = lds_read_tr(vt + va[i & 3][0] + (i >> 2) * 4096);
        vq[i][1] = lds_read_tr(vt + va[i & 3][1] + (i >> 2) * 4096);
      }
      MMSP_STEP_END();
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int g = i >> 2, db = i & 3;
        const u32x4 vop = mk4(vq[i & 3][0].x, vq[i & 3][0].y, vq[i & 3][1].x, vq[i & 3][1].y);
        oacc[db] = mfma32(vop, pb[g], oacc[db]);
        if (i + 4 < 16) {
          vq[i & 3][0] = lds_read_tr(vt + va[db][0] + (g + 1) * 4096);
          vq[i & 3][1] = lds_read_tr(vt + va[db][1] + (g + 1) * 4096);
        }
        if (i < 5) {                                    // running maximum: 32 scores in 16 three-input maxima
          const f32x16& sv = s[i >= 3 ? 1 : 0];
          if (i == 0) { mx = fmaxf(fmaxf(sv[0], sv[1]), sv[2]); mx = fmaxf(fmaxf(mx, sv[3]), sv[4]); mx = fmaxf(fmaxf(mx, sv[5]), sv[6]); }
          if (i == 1) { mx = fmaxf(fmaxf(mx, sv[7]), sv[8]); mx = fmaxf(fmaxf(mx, sv[9]), sv[10]); mx = fmaxf(fmaxf(mx, sv[11]), sv[12]); }
          if (i == 2) { mx = fmaxf(fmaxf(mx, sv[13]), sv[14]); mx = fmaxf(fmaxf(mx, sv[15]), s[1][0]); mx = fmaxf(fmaxf(mx, s[1][1]), s[1][2]); }
          if (i == 3) { mx = fmaxf(fmaxf(mx, sv[3]), sv[4]); mx = fmaxf(fmaxf(mx, sv[5]), sv[6]); mx = fmaxf(fmaxf(mx, sv[7]), sv[8]); }
          if (i == 4) { mx = fmaxf(fmaxf(mx, sv[9]), sv[10]); mx = fmaxf(fmaxf(mx, sv[11]), sv[12]); mx = fmaxf(fmaxf(mx, sv[13]), sv[14]);
                        mx = fmaxf(mx, sv[15]); mx_other = __shfl_xor(mx, 32); }
          MMSP_PIN(mx);
        }
        if (i == 6) {                                   // lazily followed reference (branch-free; only the O rescale is conditional)
          mx = fmaxf(mx, mx_other);
          moved = mx > m_ref + lazy_raw;
          const float m_new = moved ? mx : m_ref;
          alpha = moved ? __builtin_amdgcn_exp2f((m_ref - m_new) * c) : 1.f;   // m_ref = -inf -> 0
          m_ref = m_new;
          neg_mc = m_new == -INFINITY ? 0.f : -m_new * c;
          l *= alpha;
          MMSP_PIN(neg_mc); MMSP_PIN(alpha); MMSP_PIN(l);
        }
        if (i >= 8) {                                   // exponentials of keys 0..15 of the lane
          exp_item(i - 8);
        }
        MMSP_PIN(oacc[db]);
        MMSP_STEP_END();
      }
    }
    if (__any(moved)) {                                 // rare after the first tiles
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
    }
    MMSP_STEP_END();

    // ================= phase 2: S^T of tile t+1  beside  the remaining exponentials of tile t =================
    // (after the last tile the product runs on whatever the slot holds and is never used)
    f32x16 sn[2];
    {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) sn[kb][i] = 0.f;
      u32x4 kq[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) kq[i] = *reinterpret_cast<const u32x4*>(ktile - kKRegion + ka[i >> 1] + (i & 1) * 8192);
      MMSP_STEP_END();
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int ks = i >> 1, kb = i & 1;
        sn[kb] = mfma32(kq[i & 3], qreg[ks], sn[kb]);
        if (i + 4 < 16) kq[i & 3] = *reinterpret_cast<const u32x4*>(ktile - kKRegion + ka[ks + 2] + kb * 8192);
        if (i < 8) exp_item(8 + i);
        MMSP_PIN(sn[kb]);
        MMSP_STEP_END();
      }
      l += (ps[0] + ps[1]) + (ps[2] + ps[3]);
    }
    MMSP_STEP_END();
#pragma unroll
    for (int g = 0; g < 4; ++g) pb[g] = mk4(w[4 * g], w[4 * g + 1], w[4 * g + 2], w[4 * g + 3]);
    s[0] = sn[0];
    s[1] = sn[1];
  };
#undef MMSP_PIN
#undef MMSP_STEP_END

  int t = kt0;
  for (; t + 2 <= kt1; t += 3) {
    iteration(t, vslot2, kslot1, kslot0, vslot1);
    iteration(t + 1, vslot0, kslot2, kslot1, vslot2);
    iteration(t + 2, vslot1, kslot0, kslot2, vslot0);
  }
  if (t <= kt1) {
    iteration(t, vslot2, kslot1, kslot0, vslot1);
    if (t + 1 <= kt1) iteration(t + 1, vslot0, kslot2, kslot1, vslot2);
  }

  if (any_tile) {            // O^T += V^T P^T of the last tile
    __builtin_amdgcn_s_waitcnt(0x0F70);
    lds_barrier();
    auto last_product = [&](const char* vt) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const u32x2 v0 = lds_read_tr(vt + va[db][0] + g * 4096);
          const u32x2 v1 = lds_read_tr(vt + va[db][1] + g * 4096);
          oacc[db] = mfma32(mk4(v0.x, v0.y, v1.x, v1.y), pb[g], oacc[db]);
        }
    };
    const int last_slot = (kt1 - kt0) % kSlots;
    if (last_slot == 0) last_product(vslot0);
    else if (last_slot == 1) last_product(vslot1);
    else last_product(vslot2);
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

hipError_t launch_fwd_bf16(const StepArgs& a, hipStream_t stream) {
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
