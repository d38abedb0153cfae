// Backward ring step, dK/dV kernel (key-stationary) on bf16 matrix cores, head_dim 128.
//
// Workgroup = 4 wavefronts (one per SIMD, the whole 512-entry register file each) = 128 keys of
// one KV head.  A wavefront owns 32 keys and keeps their K and V rows (MFMA B operands) and the
// two accumulators dK^T, dV^T (128 d x 32 keys each) in registers for the whole call.  64-row
// tiles of Q and dO of every query head of the group stream through a four-slot LDS ring filled
// by asynchronous global->LDS copies straight from the caller's tensors (natural orientation;
// the second products read them back transposed with ds_read_b64_tr_b16), the per-row
// statistics (-LSE*log2e, delta) from padded copies in the workspace.  Per 32-row block:
//   S = Q K^T,  dP = dO V^T            (A = Q / dO rows from LDS, B = K / V registers)
//   P = exp2(S*c - LSE*log2e),  dS = P * (dP - delta)
//   dV^T += dO^T P,  dK^T += Q^T dS    (A = dO / Q read transposed, B = P / dS straight from registers)
// Nothing passes between wavefronts, so the only workgroup barrier is the one that hands a ring
// slot over, once per tile.
//
// A matrix instruction keeps the SIMD's matrix pipe busy for 32 cycles but its issue port for
// about 8, so a wavefront keeps the pipe full on its own if independent vector and LDS
// instructions are interleaved with the matrix instructions in program order.  The loop is
// software-pipelined over blocks: while the pipe computes S and dP of block b+1 the vector units
// turn dP of block b into dS; while it accumulates dV and dK of block b they take the exponentials
// of block b+1.  The operand of every matrix instruction is read from LDS four instructions ahead.
#include "mfma_tiles.h"

namespace mmsp {
namespace {

constexpr int kKeys = 128;          // keys per workgroup
constexpr int kBQ = 64;             // query rows per streamed tile
constexpr int kWaves = 4;
constexpr int kCopies = 16 / kWaves;            // 1 KiB copies per wavefront and 16 KiB tile
constexpr int kGroup = 2 * kCopies + 1;         // copies per wavefront and ring slot: Q, dO, one statistics row
constexpr int kDepth = 4;                        // LDS operand reads in flight ahead of the matrix instructions (power of two)

#define MMSP_PIN(x) asm volatile("" : "+v"(x))
#define MMSP_PIN_ACC(x) asm volatile("" : "+a"(x))     // keeps an accumulator in the AGPR half of the register file
#define MMSP_STEP_END() __builtin_amdgcn_sched_barrier(0)

// kMask = false: the host has checked that every (query, key) pair of the block is visible and
// that n_q is a multiple of the tile length, so no tile needs masking.
// nsplit > 1: the (query tile, head) sequence of every key tile is dealt out to nsplit
// workgroups, which store their partial dK / dV into w.partial for dkdv_reduce_kernel to sum
// (used when one workgroup per key tile would leave CUs idle or unevenly loaded).
template <bool kMask>
__global__ __launch_bounds__(64 * kWaves, 1) void bwd_dkdv_bf16_kernel(StepArgs a, BwdWorkspace w, int n_kt, int xcd_per_kv,
                                                                       int nsplit) {
  // LDS map: four Q tile slots in [0, 64 KiB), four dO tile slots in [64 KiB, 128 KiB), then the four
  // statistics slots.  Slots are selected at compile time (the loop is unrolled four tiles deep).
  // An LDS instruction's immediate offset reaches 64 KiB: reads of the upper regions go through
  // per-lane base registers that already hold the region's start (na_o, ta_o, so_st below), so
  // that no read needs an address addition of its own.
  constexpr int kQRegion = 0, kORegion = 4 * kTileBytes, kStRegion = 8 * kTileBytes;
  __shared__ __attribute__((aligned(1024))) char lds[kStRegion + 4 * 512];
  char* const qs0 = lds + kQRegion;                     // Q tiles, TileS
  char* const qs1 = qs0 + kTileBytes;
  char* const qs2 = qs1 + kTileBytes;
  char* const qs3 = qs2 + kTileBytes;
  char* const os0 = lds + kORegion;                     // dO tiles, TileS
  char* const os1 = os0 + kTileBytes;
  char* const os2 = os1 + kTileBytes;
  char* const os3 = os2 + kTileBytes;
  float* const st0 = reinterpret_cast<float*>(lds + kStRegion);   // [0,64) -LSE*log2e, [64,128) delta
  float* const st1 = st0 + 128;
  float* const st2 = st1 + 128;
  float* const st3 = st2 + 128;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);   // the same value in a scalar register (LDS targets of the copies)
  const int half = lane >> 5, col = lane & 31;

  int kvh, item;                    // item = key tile * nsplit + range
  if (xcd_per_kv > 0) {             // workgroups of one KV head share an XCD (its L2 then serves the Q/dO stream once)
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    kvh = xcd / xcd_per_kv;
    item = slot * xcd_per_kv + (xcd % xcd_per_kv);
    if (item >= n_kt * nsplit) return;
  } else {
    kvh = blockIdx.x / (n_kt * nsplit);
    item = blockIdx.x % (n_kt * nsplit);
  }
  const int kt = item / nsplit, split = item % nsplit;
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
  // this workgroup's share of the (query tile, head of the group) sequence: elements split,
  // split + nsplit, ...  (interleaved rather than contiguous, so that the workgroups of a key
  // tile, and of neighbouring key tiles, walk the Q / dO tiles at the same place and pace and
  // share them in L2).  Sequence order: query tiles from the last visible one downwards, the
  // heads of the group inside a tile: under a causal or document mask the key tiles that share
  // an XCD see query ranges with different starts but a common end.
  int niter = 0;
  if (ntiles > 0) {
    const int total = ntiles * a.group;
    niter = total > split ? (total - split + nsplit - 1) / nsplit : 0;
  }
  if (niter == 0 && nsplit == 1 && a.accumulate) return;   // nothing visible, nothing to add

  // K and V rows of this lane's key as B operands (k index along d)
  u32x4 kreg[8], vreg[8];
  {
    const int64_t off = (int64_t)(a.k_row0 + keyc) * a.kv_ts + (int64_t)kvh * a.kv_hs + half * 8;
    const uint16_t* pk = reinterpret_cast<const uint16_t*>(a.k) + off;
    const uint16_t* pv = reinterpret_cast<const uint16_t*>(a.v) + off;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      kreg[ks] = *reinterpret_cast<const u32x4*>(pk + ks * 16);
      vreg[ks] = *reinterpret_cast<const u32x4*>(pv + ks * 16);
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) { MMSP_PIN(kreg[ks]); MMSP_PIN(vreg[ks]); }   // landed before the tile copies are counted
  }
  const float c = a.scale * kLog2e;

  f32x16 dv[4], dk[4];                                   // dV^T, dK^T: 128 d x 32 keys
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dv[db][i] = 0.f; dk[db][i] = 0.f; }

  if (niter > 0) {
    // ---- asynchronous tile fetch: cursor over the (head of the group, query tile) sequence ----
    const char* qbase = reinterpret_cast<const char*>(a.q) + ((int64_t)a.q_row0 * a.q_ts + (int64_t)kvh * a.group * a.q_hs) * 2;
    const char* dobase = reinterpret_cast<const char*>(a.d_o) + ((int64_t)a.q_row0 * a.Hq + (int64_t)kvh * a.group) * 256;
    const int64_t q_tile_bytes = (int64_t)kBQ * a.q_ts * 2, do_tile_bytes = (int64_t)kBQ * a.Hq * 256;
    const int64_t q_head_bytes = (int64_t)a.q_hs * 2;
    const int64_t st_head_bytes = (int64_t)w.n_qtiles * kBQ * 4;
    const char* stat_src = reinterpret_cast<const char*>((wave_s & 1) ? w.dl : w.nl2) + (int64_t)kvh * a.group * st_head_bytes;
    const DmaOffs<kCopies> qoff_full = dma_s_offsets<kCopies>(a.q_ts, kBQ, wave, lane);
    const DmaOffs<kCopies> dooff_full = dma_s_offsets<kCopies>((int64_t)a.Hq * 128, kBQ, wave, lane);
    // the last query tile of the block may be ragged: rows past the end repeat the last row
    const int qt_ragged = a.n_q % kBQ != 0 ? a.n_q / kBQ : -1;
    const DmaOffs<kCopies> qoff_ragged = dma_s_offsets<kCopies>(a.q_ts, qt_ragged >= 0 ? a.n_q % kBQ : kBQ, wave, lane);
    const DmaOffs<kCopies> dooff_ragged = dma_s_offsets<kCopies>((int64_t)a.Hq * 128, qt_ragged >= 0 ? a.n_q % kBQ : kBQ, wave, lane);
    // Element the next fetch takes, and where its Q / dO / statistics rows start.  The three
    // addresses are wavefront-uniform and move by additions only.
    int f_hg = split % a.group, f_qt = qt1 - split / a.group, f_it = 0;
    const char* f_q = qbase + f_hg * q_head_bytes + f_qt * q_tile_bytes;
    const char* f_do = dobase + f_hg * 256 + f_qt * do_tile_bytes;
    const char* f_st = stat_src + f_hg * st_head_bytes + f_qt * (kBQ * 4);
    const int64_t step_q = nsplit * q_head_bytes, wrap_q = a.group * q_head_bytes + q_tile_bytes;
    const int64_t step_do = nsplit * 256, wrap_do = a.group * 256 + do_tile_bytes;
    const int64_t step_st = nsplit * st_head_bytes, wrap_st = a.group * st_head_bytes + kBQ * 4;
    // A fetch is issued in 2 kCopies + 1 pieces (one copy instruction each) so that the loop can
    // spread them between its matrix instructions: a copy holds up the issuing wavefront while
    // the memory pipeline accepts it, and with one wavefront per SIMD nobody else fills that gap.
    struct Fetch { const char* q; const char* d_o; const char* st; bool ragged; };
    auto fetch_begin = [&]() {
      Fetch f;
      f.q = f_q; f.d_o = f_do; f.st = f_st;
      f.ragged = f_qt == qt_ragged;
      if (f_it + 1 < niter) {                           // past the end the last tile is fetched again (into a free slot)
        ++f_it;
        f_hg += nsplit; f_q += step_q; f_do += step_do; f_st += step_st;
        while (f_hg >= a.group) { f_hg -= a.group; --f_qt; f_q -= wrap_q; f_do -= wrap_do; f_st -= wrap_st; }
      }
      return f;
    };
    auto fetch_piece = [&](const Fetch& f, int piece, char* qdst, char* odst, float* sdst) {
      constexpr int W = 16 / kCopies;
      if (piece < kCopies) {
        dma16(f.q, f.ragged ? qoff_ragged.o[piece] : qoff_full.o[piece], qdst, (wave_s + piece * W) * 1024);
      } else if (piece < 2 * kCopies) {
        const int p = piece - kCopies;
        dma16(f.d_o, f.ragged ? dooff_ragged.o[p] : dooff_full.o[p], odst, (wave_s + p * W) * 1024);
      } else {
        dma4(f.st, (uint32_t)lane * 4, sdst, (wave_s & 1) * 256);   // even wavefronts fetch -LSE*log2e, odd ones delta
      }
    };
    auto fetch = [&](char* qdst, char* odst, float* sdst) {
      const Fetch f = fetch_begin();
#pragma unroll
      for (int piece = 0; piece < kGroup; ++piece) fetch_piece(f, piece, qdst, odst, sdst);
    };
    fetch(qs0, os0, st0);
    fetch(qs1, os1, st1);
    fetch(qs2, os2, st2);

    // LDS read offsets inside a tile, fixed for the whole call: natural operand k-step ks (rows
    // +32 -> +8192 bytes); transposed operand of d block db, first / second read (16 rows further
    // -> +4096 bytes)
    int na[8], ta[4][2];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) na[ks] = tile_s_offset(col, ks * 2 + half);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      ta[db][0] = tile_s_tr_offset(lane, db, 0);
      ta[db][1] = tile_s_tr_offset(lane, db, 1);
    }
    const int so = half * 4;                             // statistics of rows (i/4)*8 + half*4 + i%4: float4 at so + 8 g4
    // the same per-lane offsets with the start of the dO / statistics region added, kept opaque so
    // that the compiler uses them as bases instead of rebuilding them from na / ta
    int na_o[8], ta_o[4][2], so_st = so * 4 + kStRegion;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) { na_o[ks] = na[ks] + kORegion; asm volatile("" : "+v"(na_o[ks])); }
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      ta_o[db][0] = ta[db][0] + kORegion; asm volatile("" : "+v"(ta_o[db][0]));
      ta_o[db][1] = ta[db][1] + kORegion; asm volatile("" : "+v"(ta_o[db][1]));
    }
    asm volatile("" : "+v"(so_st));
    auto stat4 = [&](const float* slot, int first_float) {   // float4 of this lane's rows, first_float = offset inside the slot
      return *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(slot) - kStRegion + so_st + first_float * 4);
    };

    // (head of the group, query tile) of the tile being computed
    int c_hg = split % a.group, c_qt = qt1 - split / a.group;

    // Software pipeline state carried from block to block.
    f32x16 s_nx, dp_nx;          // S and dP of the next block (first products, being accumulated)
    f32x16 p_cur, dp_cur;        // P (fp32) and dP of the current block
    u32x4 pb0, pb1;              // P of the current block packed as B operands (rows 0..15, 16..31)
    u32x4 oq[kDepth];            // LDS operands in flight, kDepth matrix instructions deep

    // Operand n of a tile body (one per matrix instruction), read four instructions ahead:
    //   n =  0..15  phase A of block 0: S / dP of block 1      natural rows 32..63 of this tile (Q even n, dO odd n)
    //   n = 16..31  phase B of block 0: dV / dK of block 0     transposed rows 0..31 (dO even n, Q odd n)
    //   n = 32..47  phase A of block 1: S / dP of the next tile's block 0   natural rows 0..31 of the next tile
    //   n = 48..63  phase B of block 1: dV / dK of block 1     transposed rows 32..63
    //   n = 64 ...  = the first operands of the next tile body (whose "this tile" is our next tile)
    auto operand = [&](int n, const char* cq, const char* co, const char* nq, const char* no) -> u32x4 {
      if (n >= 64) { n -= 64; cq = nq; co = no; }
      const int ph = n >> 4, i = n & 15;
      if ((ph & 1) == 0) {                               // natural: k-step i / 2, Q for S (even), dO for dP (odd)
        const int at = ph == 0 ? 8192 : 0;
        if (i & 1) return *reinterpret_cast<const u32x4*>((ph == 0 ? co : no) - kORegion + na_o[i >> 1] + at);
        return *reinterpret_cast<const u32x4*>((ph == 0 ? cq : nq) + na[i >> 1] + at);
      }
      // transposed: i = 8 t' + 2 db + (0: dO^T for dV, 1: Q^T for dK)
      const int tq = i >> 3, db = (i >> 1) & 3, g = (ph == 1 ? 0 : 2) + tq;
      u32x2 v0, v1;
      if (i & 1) {
        v0 = lds_read_tr(cq + ta[db][0] + g * 4096);
        v1 = lds_read_tr(cq + ta[db][1] + g * 4096);
      } else {
        v0 = lds_read_tr(co - kORegion + ta_o[db][0] + g * 4096);
        v1 = lds_read_tr(co - kORegion + ta_o[db][1] + g * 4096);
      }
      return mk4(v0.x, v0.y, v1.x, v1.y);
    };

    auto apply_mask = [&](f32x16& x, int q0) {           // q0: first row of the block
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int qrow = q0 + (i >> 2) * 8 + half * 4 + (i & 3);
        x[i] = (qrow < rlo || qrow > rhi) ? -INFINITY : x[i];
      }
    };
    auto needs_mask = [&](int q0) { return kMask && (q0 < w_lo_max || q0 + 31 > w_hi_min); };

    // ---- prologue: S, dP and P of the first block ----
    __builtin_amdgcn_s_waitcnt(0x0F70 | ((2 * kGroup) & 15) | (((2 * kGroup) >> 4) << 14));   // vmcnt(2 kGroup): the first tile has landed (two newer groups may be in flight)
    lds_barrier();
    {
#pragma unroll
      for (int i = 0; i < 16; ++i) { s_nx[i] = 0.f; dp_nx[i] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        s_nx = mfma32(*reinterpret_cast<const u32x4*>(qs0 + na[ks]), kreg[ks], s_nx);
        dp_nx = mfma32(*reinterpret_cast<const u32x4*>(os0 + na[ks]), vreg[ks], dp_nx);
      }
      if (needs_mask(c_qt * kBQ)) apply_mask(s_nx, c_qt * kBQ);
      uint32_t pw[8];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const float4 nl = *reinterpret_cast<const float4*>(st0 + so + g4 * 8);
        p_cur[g4 * 4 + 0] = __builtin_amdgcn_exp2f(fmaf(s_nx[g4 * 4 + 0], c, nl.x));
        p_cur[g4 * 4 + 1] = __builtin_amdgcn_exp2f(fmaf(s_nx[g4 * 4 + 1], c, nl.y));
        p_cur[g4 * 4 + 2] = __builtin_amdgcn_exp2f(fmaf(s_nx[g4 * 4 + 2], c, nl.z));
        p_cur[g4 * 4 + 3] = __builtin_amdgcn_exp2f(fmaf(s_nx[g4 * 4 + 3], c, nl.w));
        pw[g4 * 2] = pack2(p_cur[g4 * 4 + 0], p_cur[g4 * 4 + 1]);
        pw[g4 * 2 + 1] = pack2(p_cur[g4 * 4 + 2], p_cur[g4 * 4 + 3]);
      }
      pb0 = mk4(pw[0], pw[1], pw[2], pw[3]);
      pb1 = mk4(pw[4], pw[5], pw[6], pw[7]);
      dp_cur = dp_nx;
    }

    // One tile: four phases of 16 matrix instructions.  cq / co / cs: this tile's slot, nq / no / ns:
    // the next tile's, rq / ro / rs: the slot to refill (three tiles ahead).
    auto body = [&](bool first, const char* cq, const char* co, const float* cs, const char* nq, const char* no, const float* ns,
                    char* rq, char* ro, float* rs) {
      // Own copies of every group but the newest have landed; after the barrier everybody's have
      // (this tile's and the next one's), and everybody is done with the slot about to be refilled.
      __builtin_amdgcn_s_waitcnt(0x0F70 | kGroup);
      lds_barrier();
      const Fetch fx = fetch_begin();
      const int q0 = c_qt * kBQ;
      c_hg += nsplit;
      while (c_hg >= a.group) { c_hg -= a.group; --c_qt; }
      const int q0_next = c_qt * kBQ;                    // first row of the next tile (unused after the last)
      if (first) {
#pragma unroll
        for (int n = 0; n < kDepth; ++n) oq[n] = operand(n, cq, co, nq, no);
      }
      MMSP_STEP_END();

#pragma unroll
      for (int ph = 0; ph < 4; ++ph) {
        const int blk = ph >> 1;                         // block of this tile the phase works for
        if ((ph & 1) == 0) {
          // ---- phase A: S, dP of the following block beside dS of block blk ----
          float4 dl[4];
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4) dl[g4] = stat4(cs, 64 + blk * 32 + g4 * 8);
#pragma unroll
          for (int i = 0; i < 16; ++i) { s_nx[i] = 0.f; dp_nx[i] = 0.f; }
          uint32_t sw[8];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int n = ph * 16 + i, ks = i >> 1;
            u32x4 op = oq[n & (kDepth - 1)];
            MMSP_PIN(op);
            if ((i & 1) == 0) s_nx = mfma32(op, kreg[ks], s_nx);
            else dp_nx = mfma32(op, vreg[ks], dp_nx);
            oq[n & (kDepth - 1)] = operand(n + kDepth, cq, co, nq, no);
            if (n % 7 == 3 && n / 7 < kGroup) fetch_piece(fx, n / 7, rq, ro, rs);
            if (i >= 4 && i < 12) {                      // dS of rows 2j, 2j+1 of the lane's 16 (one pair per step)
              const int j = i - 4, e = 2 * j;
              const float d0 = (e & 3) == 0 ? dl[e >> 2].x : dl[e >> 2].z;
              const float d1 = (e & 3) == 0 ? dl[e >> 2].y : dl[e >> 2].w;
              sw[j] = pack2(p_cur[e] * (dp_cur[e] - d0), p_cur[e + 1] * (dp_cur[e + 1] - d1));
              MMSP_PIN(sw[j]);
            }
            if ((i & 1) == 0) MMSP_PIN_ACC(s_nx); else MMSP_PIN_ACC(dp_nx);
            MMSP_STEP_END();
          }
          // hand over: the packed dS of block blk feeds phase B; S / dP of the following block become current
          const u32x4 ds0 = mk4(sw[0], sw[1], sw[2], sw[3]), ds1 = mk4(sw[4], sw[5], sw[6], sw[7]);
          const int q0_f = blk == 0 ? q0 + 32 : q0_next;  // first row of the following block
          if (needs_mask(q0_f)) apply_mask(s_nx, q0_f);
          MMSP_STEP_END();
          // ---- phase B: dV, dK of block blk beside P of the following block ----
          const float* fs = blk == 0 ? cs + 32 : ns;     // -LSE*log2e of the following block's rows
          float4 nl[4];
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4) nl[g4] = stat4(fs, g4 * 8);
          uint32_t pw[8];
          f32x16 p_nx;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int n = (ph + 1) * 16 + i, tq = i >> 3, db = (i >> 1) & 3;
            u32x4 op = oq[n & (kDepth - 1)];
            MMSP_PIN(op);
            if ((i & 1) == 0) dv[db] = mfma32(op, tq ? pb1 : pb0, dv[db]);
            else dk[db] = mfma32(op, tq ? ds1 : ds0, dk[db]);
            oq[n & (kDepth - 1)] = operand(n + kDepth, cq, co, nq, no);
            if (n % 7 == 3 && n / 7 < kGroup) fetch_piece(fx, n / 7, rq, ro, rs);
            if (i >= 4 && i < 12) {                      // P of rows 2j, 2j+1
              const int j = i - 4, e = 2 * j;
              const float n0 = (e & 3) == 0 ? nl[e >> 2].x : nl[e >> 2].z;
              const float n1 = (e & 3) == 0 ? nl[e >> 2].y : nl[e >> 2].w;
              p_nx[e] = __builtin_amdgcn_exp2f(fmaf(s_nx[e], c, n0));
              p_nx[e + 1] = __builtin_amdgcn_exp2f(fmaf(s_nx[e + 1], c, n1));
              pw[j] = pack2(p_nx[e], p_nx[e + 1]);
              MMSP_PIN(pw[j]);
            }
            if ((i & 1) == 0) MMSP_PIN_ACC(dv[db]); else MMSP_PIN_ACC(dk[db]);
            MMSP_STEP_END();
          }
          pb0 = mk4(pw[0], pw[1], pw[2], pw[3]);
          pb1 = mk4(pw[4], pw[5], pw[6], pw[7]);
          p_cur = p_nx;
          dp_cur = dp_nx;
          MMSP_STEP_END();
        }
      }
    };

    // Four tiles per trip so that every slot is a compile-time constant; the steady-state loop
    // has no conditional bodies.
    int it = 0;
    for (; it + 3 < niter; it += 4) {
      body(it == 0, qs0, os0, st0, qs1, os1, st1, qs3, os3, st3);
      body(false, qs1, os1, st1, qs2, os2, st2, qs0, os0, st0);
      body(false, qs2, os2, st2, qs3, os3, st3, qs1, os1, st1);
      body(false, qs3, os3, st3, qs0, os0, st0, qs2, os2, st2);
    }
    if (it < niter) {
      body(it == 0, qs0, os0, st0, qs1, os1, st1, qs3, os3, st3);
      if (it + 1 < niter) body(false, qs1, os1, st1, qs2, os2, st2, qs0, os0, st0);
      if (it + 2 < niter) body(false, qs2, os2, st2, qs3, os3, st3, qs1, os1, st1);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // drain the copies issued past the end before the workgroup leaves
  }

  if (!live) return;
  if (nsplit > 1) {                                      // partial result of this range, summed by dkdv_reduce_kernel
    const int64_t slot_elems = (int64_t)n_kt * kKeys * a.Hkv * 128;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
      const float mul = which ? 1.f : a.scale;
      float* out = w.partial + ((int64_t)(which ? nsplit : 0) + split) * slot_elems + ((int64_t)key * a.Hkv + kvh) * 128 + half * 4;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const f32x16& x = which ? dv[db] : dk[db];
          *reinterpret_cast<float4*>(out + db * 32 + g4 * 8) =
              make_float4(mul * x[g4 * 4 + 0], mul * x[g4 * 4 + 1], mul * x[g4 * 4 + 2], mul * x[g4 * 4 + 3]);
        }
    }
    return;
  }
  const int64_t off = ((int64_t)(a.k_row0 + key) * a.Hkv + kvh) * 128 + half * 4;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const float mul = which ? 1.f : a.scale;
    float* out = (which ? a.dv : a.dk) + off;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const f32x16& x = which ? dv[db] : dk[db];
        float4* p = reinterpret_cast<float4*>(out + db * 32 + g4 * 8);
        float4 y = make_float4(mul * x[g4 * 4 + 0], mul * x[g4 * 4 + 1], mul * x[g4 * 4 + 2], mul * x[g4 * 4 + 3]);
        if (a.accumulate) {
          const float4 o = *p;
          y.x += o.x; y.y += o.y; y.z += o.z; y.w += o.w;
        }
        *p = y;
      }
  }
}
#undef MMSP_PIN
#undef MMSP_PIN_ACC
#undef MMSP_STEP_END

// out[i] (+)= sum over the nsplit partial slots, for the n4 float4 of dK (blockIdx.y = 0) or dV (1).
__global__ __launch_bounds__(256) void dkdv_reduce_kernel(const float* __restrict__ partial, int nsplit, int64_t slot_elems,
                                                          float* __restrict__ dk, float* __restrict__ dv, int64_t n4,
                                                          bool accumulate) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  const float* src = partial + (int64_t)blockIdx.y * nsplit * slot_elems + i * 4;
  float4* dst = reinterpret_cast<float4*>(blockIdx.y ? dv : dk) + i;
  float4 x = accumulate ? *dst : make_float4(0.f, 0.f, 0.f, 0.f);
  for (int sidx = 0; sidx < nsplit; ++sidx) {
    const float4 p = *reinterpret_cast<const float4*>(src + sidx * slot_elems);
    x.x += p.x; x.y += p.y; x.z += p.z; x.w += p.w;
  }
  *dst = x;
}

}  // namespace

// Workgroups the partial-sum area is sized for: ranges are only cut while (key tiles x KV
// heads x ranges) stays within this count.
constexpr int kSplitMaxBlocks = 512;
constexpr int kSplitMaxRanges = 8;

int64_t bwd_dkdv_partial_bytes() { return 2LL * kSplitMaxBlocks * kKeys * 128 * (int64_t)sizeof(float); }

hipError_t launch_bwd_dkdv_bf16(const StepArgs& a, const BwdWorkspace& w, hipStream_t stream) {
  const int n_kt = (a.n_k + kKeys - 1) / kKeys;
  // One workgroup per (key tile, KV head) fills the chip only if there are about as many as
  // CUs; with fewer, cut every key tile's query sequence into ranges.
  static int cu_of_device[64] = {};                     // 0 = not asked yet; the count never changes for a device
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64) n_cu = cu_of_device[dev];
  if (n_cu == 0) {
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) n_cu = kSplitMaxBlocks / 2;
    if (dev >= 0 && dev < 64) cu_of_device[dev] = n_cu;
  }
  // With every pair visible all key tiles carry the same work and one round of workgroups is
  // best; under a mask the work per key tile varies (by 2x across a causal block), so aim for
  // two rounds of shorter workgroups, which the dispatcher then balances (heavy tiles come first).
  const bool no_mask = a.mask == 0 && a.cu == nullptr && a.n_q % kBQ == 0;
  const int base_blocks = n_kt * a.Hkv;
  const int target = min(no_mask ? n_cu : 2 * n_cu, kSplitMaxBlocks);
  int nsplit = min(target / base_blocks, kSplitMaxRanges);
  if (nsplit < 2) nsplit = 1;
  const int n_items = n_kt * nsplit;
  int xcd_per_kv = 0, n_blocks = n_items * a.Hkv;
  if (8 % a.Hkv == 0) {
    xcd_per_kv = 8 / a.Hkv;
    n_blocks = 8 * ((n_items + xcd_per_kv - 1) / xcd_per_kv);
  }
  if (no_mask) bwd_dkdv_bf16_kernel<false><<<dim3(n_blocks), dim3(64 * kWaves), 0, stream>>>(a, w, n_kt, xcd_per_kv, nsplit);
  else bwd_dkdv_bf16_kernel<true><<<dim3(n_blocks), dim3(64 * kWaves), 0, stream>>>(a, w, n_kt, xcd_per_kv, nsplit);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || nsplit == 1) return e;
  const int64_t n4 = (int64_t)a.n_k * a.Hkv * 32;
  const int64_t first = (int64_t)a.k_row0 * a.Hkv * 128;
  dkdv_reduce_kernel<<<dim3((unsigned)((n4 + 255) / 256), 2), dim3(256), 0, stream>>>(
      w.partial, nsplit, (int64_t)n_kt * kKeys * a.Hkv * 128, a.dk + first, a.dv + first, n4, a.accumulate);
  return hipGetLastError();
}

}  // namespace mmsp
