// Backward ring step, dK/dV kernel (key-stationary) on bf16 matrix cores, head_dim 128.
//
// Workgroup = 8 wavefronts = 128 keys of one KV head.  The wavefronts are specialised in pairs
// that share 32 keys and, with the round-robin wavefront placement, a SIMD:
//   "P" wavefront (0..3):  S = Q K^T,  P = exp2(S*c - LSE*log2e),  dV^T += dO^T P
//   "D" wavefront (4..7):  dP = dO V^T,  dS = P * (dP - delta),    dK^T += Q^T dS
// P travels from the first to the second through LDS, already packed as an MFMA B operand (the
// two wavefronts use the same lane <-> (key, query) mapping, so it is a straight copy).  Each
// wavefront keeps one 128 d x 32 key accumulator and one of K / V in registers, which fits the
// plain VGPR file with two wavefronts per SIMD, and the two of a pair do the same number of
// MFMAs, so one's exp / dS arithmetic overlaps the other's matrix work.
//
// 64-row tiles of Q and dO of every query head of the group stream through a two-stage LDS
// ring filled by asynchronous global->LDS copies: the natural tiles straight from the caller's
// tensors, the transposed ones (Q^T, dO^T) from tile images pre-built in the workspace, the
// per-row statistics (-LSE*log2e, delta) from padded copies there.
#include "mfma_tiles.h"

namespace mmsp {
namespace {

constexpr int kKeys = 128;          // keys per workgroup
constexpr int kBQ = 64;             // query rows per streamed tile
constexpr int kWaves = 8;
constexpr int kCopies = 16 / kWaves;
constexpr int kStage = 4 * kTileBytes;   // Q TileN | dO TileN | Q^T TileT | dO^T TileT

__device__ __forceinline__ void dma4(const char* gptr, char* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 4, 0, 0);
}

// kMask = false: the host has checked that every (query, key) pair of the block is visible and
// that n_q is a multiple of the tile length, so no tile needs masking.
// nsplit > 1: the (query tile, head) sequence of every key tile is dealt out to nsplit
// workgroups, which store their partial dK / dV into w.partial for dkdv_reduce_kernel to sum
// (used when one workgroup per key tile would leave CUs idle or unevenly loaded).
template <bool kMask>
__global__ __launch_bounds__(64 * kWaves, 2) void bwd_dkdv_bf16_kernel(StepArgs a, BwdWorkspace w, int n_kt, int xcd_per_kv,
                                                                       int nsplit) {
  __shared__ __attribute__((aligned(1024))) char stage0[kStage];
  __shared__ __attribute__((aligned(1024))) char stage1[kStage];
  __shared__ __attribute__((aligned(1024))) float stat0[128];      // [0,64) -LSE*log2e, [64,128) delta
  __shared__ __attribute__((aligned(1024))) float stat1[128];
  __shared__ __attribute__((aligned(1024))) char pxch[2 * 4 * 2048];   // P of a block: [slot][pair][half of the lane's 32 B][lane * 16 B]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int pair = wave & 3;                    // which 32 keys
  const bool role_p = wave < 4;                 // true: S / P / dV,  false: dP / dS / dK

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
  const int key = tile_key0 + pair * 32 + col;           // block-relative key of this lane
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
    const int wk0 = min(tile_key0 + pair * 32, a.n_k - 1);
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
  // share them in L2)
  int it0 = split, niter = 0;
  if (ntiles > 0) {
    const int total = ntiles * a.group;
    niter = total > split ? (total - split + nsplit - 1) / nsplit : 0;
  }
  // Sequence order: query tiles from the last visible one downwards, the heads of the group
  // inside a tile.  Under a causal or document mask the key tiles that share an XCD see query
  // ranges with different starts but a common end, so walking down from the end keeps their
  // workgroups on the same Q / dO tiles (served once from HBM, then from L2) for as long as
  // their ranges overlap.
  const int hg_first = it0 % a.group, qt_first = qt1 - it0 / a.group;

  // ---- asynchronous tile fetch (all 8 wavefronts share the copies) ----
  const char* qbase = reinterpret_cast<const char*>(a.q) + (int64_t)a.q_row0 * a.q_ts * 2;
  const char* dobase = reinterpret_cast<const char*>(a.d_o) + (int64_t)a.q_row0 * a.Hq * 256;
  const int64_t q_tile_bytes = (int64_t)kBQ * a.q_ts * 2, do_tile_bytes = (int64_t)kBQ * a.Hq * 256;
  const DmaOffs<kCopies> qoff_full = dma_n_offsets<kCopies>(a.q_ts, kBQ, wave, lane);
  const DmaOffs<kCopies> dooff_full = dma_n_offsets<kCopies>((int64_t)a.Hq * 128, kBQ, wave, lane);
  // Cursor over the (head of the group, query tile) sequence: byte offsets of the tile in the
  // four sources, advanced by additions so that the loop carries no 64-bit multiplies.
  struct Cursor { int hg, qt; int64_t q, d_o, img, st; };
  const int64_t q_head_step = (int64_t)a.q_hs * 2, do_head_step = 256;
  const int64_t img_head_step = (int64_t)w.n_qtiles * kImageBytes, st_head_step = (int64_t)w.n_qtiles * kBQ * 4;
  const int gm1 = a.group - 1;
  auto advance = [&](Cursor& cu) {                       // nsplit elements further in the sequence
    for (int j = 0; j < nsplit; ++j) {
      if (++cu.hg == a.group) {                          // next (lower) query tile, first head of the group
        cu.hg = 0; --cu.qt;
        cu.q -= gm1 * q_head_step + q_tile_bytes; cu.d_o -= gm1 * do_head_step + do_tile_bytes;
        cu.img -= gm1 * img_head_step + kImageBytes; cu.st -= gm1 * st_head_step + kBQ * 4;
      } else {
        cu.q += q_head_step; cu.d_o += do_head_step; cu.img += img_head_step; cu.st += st_head_step;
      }
    }
  };
  Cursor fc;                                             // tile whose copies are being issued
  {
    const int h0 = kvh * a.group + hg_first;
    fc.hg = hg_first; fc.qt = qt_first;
    fc.q = (int64_t)h0 * a.q_hs * 2 + (int64_t)qt_first * q_tile_bytes;
    fc.d_o = (int64_t)h0 * 256 + (int64_t)qt_first * do_tile_bytes;
    fc.img = ((int64_t)h0 * w.n_qtiles + qt_first) * kImageBytes;
    fc.st = ((int64_t)h0 * w.n_qtiles + qt_first) * kBQ * 4;
  }
  // The copies of one tile are issued in four pieces (Q with the statistics, dO, Q^T image,
  // dO^T image) that the loop spreads between its MFMAs: a burst of copy instructions holds
  // up the issuing wavefronts until the texture path has taken them all.
  const char* const stat_src = reinterpret_cast<const char*>((wave & 1) ? w.dl : w.nl2) + lane * 4;
  auto fetch_piece = [&](int piece, const Cursor& cu, char* stage, float* stat) {
    if (piece < 2) {
      const int left = a.n_q - cu.qt * kBQ;              // < kBQ: ragged last tile, rows past the end repeat the last row
      if (piece == 0) {
        const char* qp = qbase + cu.q;
        if (left >= kBQ) dma_tile_n<kCopies>(qp, qoff_full, stage, wave);
        else dma_tile_n<kCopies>(qp, dma_n_offsets<kCopies>(a.q_ts, left, wave, lane), stage, wave);
        // statistics: even wavefronts fetch -LSE*log2e, odd ones delta (several fetch the same bytes)
        dma4(stat_src + cu.st, reinterpret_cast<char*>(stat + (wave & 1) * 64));
      } else {
        const char* dp = dobase + cu.d_o;
        if (left >= kBQ) dma_tile_n<kCopies>(dp, dooff_full, stage + kTileBytes, wave);
        else dma_tile_n<kCopies>(dp, dma_n_offsets<kCopies>((int64_t)a.Hq * 128, left, wave, lane), stage + kTileBytes, wave);
      }
    } else {
      dma_tile_image<kCopies>((piece == 2 ? w.qt : w.dot) + cu.img, stage + piece * kTileBytes, wave, lane);
    }
  };
  if (niter > 0) {
#pragma unroll
    for (int piece = 0; piece < 4; ++piece) fetch_piece(piece, fc, stage0, stat0);
  }

  // K (P role) or V (D role) rows of this lane's key as B operands (k index along d)
  u32x4 kvreg[8];
  {
    const int64_t off = (int64_t)(a.k_row0 + keyc) * a.kv_ts + (int64_t)kvh * a.kv_hs + half * 8;
    const uint16_t* p = reinterpret_cast<const uint16_t*>(role_p ? a.k : a.v) + off;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kvreg[ks] = *reinterpret_cast<const u32x4*>(p + ks * 16);
  }
  const float c = a.scale * kLog2e;

  f32x16 acc[4];                                         // dV^T (P role) or dK^T (D role): 128 d x 32 keys
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;

  // LDS read offsets, fixed for the whole call.  P role reads Q (natural) and dO^T; D role
  // reads dO (natural) and Q^T.
  int na[8], ta[4];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) na[ks] = tile_n_offset(col, ks * 2 + half) + (role_p ? 0 : kTileBytes);            // + qb*8192
#pragma unroll
  for (int x = 0; x < 4; ++x) ta[x] = tile_t_offset(col, x * 2 + half) + (role_p ? 3 : 2) * kTileBytes;             // + db*4096
  char* const my_px = pxch + pair * 2048 + lane * 16;    // + slot * 8192; second 16 bytes of the lane at + 1024

  // (head of the group, query tile) of the tile being computed and of the tile whose copies
  // are being issued.  While tile t is computed: the rest of tile t+1 during its first block,
  // the first piece of tile t+2 after its second barrier, which frees the stage of tile t.
  int cur_hg = hg_first, cur_qt = qt_first;
  if (niter > 0) advance(fc);
  if (niter > 1) fetch_piece(0, fc, stage1, stat1);

  // LDS operands are fetched a whole product ahead of the MFMAs that use them.  o1 feeds a
  // block's first product (S or dP); it is reloaded for the next block as soon as the MFMAs
  // that read it are issued, for the next tile's first block right after the barrier that hands
  // the stages over.  o2 feeds the second product (dV or dK) and is loaded before the exchange.
  u32x4 o1[8], o2[8];
  __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): K / V registers and both stages
  lds_barrier();
  if (niter > 0) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) o1[ks] = *reinterpret_cast<const u32x4*>(stage0 + na[ks]);
  }

  // One tile = two 32-row blocks and two workgroup barriers, one per block: before it the P
  // wavefronts have published P of the block and everybody has finished every LDS read issued
  // so far.  The second barrier of a tile therefore also retires the tile's stage, which is
  // refilled at once with the tile after next, and publishes the next tile's stage (each
  // wavefront waits for its own copies of it first).
  auto tile_body = [&](int it, char* cur, float* stat, char* oth, float* ostat) {
    const int q0 = cur_qt * kBQ;
    cur_hg += nsplit;
    while (cur_hg >= a.group) { cur_hg -= a.group; --cur_qt; }
    const bool need_mask = kMask && (q0 < w_lo_max || q0 + kBQ - 1 > w_hi_min);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      // first product of the block: S = Q K^T (P role) or dP = dO V^T (D role)
      f32x16 x;
#pragma unroll
      for (int i = 0; i < 16; ++i) x[i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        x = mfma32(o1[ks], kvreg[ks], x);
        if (qb == 0 && (ks == 2 || ks == 5)) {
          if (it + 1 < niter) fetch_piece(ks == 2 ? 1 : 2, fc, oth, ostat);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        o2[2 * db] = *reinterpret_cast<const u32x4*>(cur + ta[(qb * 2) ^ db] + db * 4096);
        o2[2 * db + 1] = *reinterpret_cast<const u32x4*>(cur + ta[(qb * 2 + 1) ^ db] + db * 4096);
      }
      if (qb == 0) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) o1[ks] = *reinterpret_cast<const u32x4*>(cur + na[ks] + 8192);
      }
      __builtin_amdgcn_sched_barrier(0);

      u32x4 b0, b1;                                      // B operands of the second product
      char* px = my_px + qb * 8192;                      // exchange slot of this block
      if (role_p) {
        if (need_mask) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int qrow = q0 + qb * 32 + (i >> 2) * 8 + half * 4 + (i & 3);
            x[i] = (qrow < rlo || qrow > rhi) ? -INFINITY : x[i];
          }
        }
        uint32_t pw[8];
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const float4 nl = *reinterpret_cast<const float4*>(stat + qb * 32 + g4 * 8 + half * 4);
          pw[g4 * 2] = pack2(__builtin_amdgcn_exp2f(fmaf(x[g4 * 4 + 0], c, nl.x)),
                             __builtin_amdgcn_exp2f(fmaf(x[g4 * 4 + 1], c, nl.y)));
          pw[g4 * 2 + 1] = pack2(__builtin_amdgcn_exp2f(fmaf(x[g4 * 4 + 2], c, nl.z)),
                                 __builtin_amdgcn_exp2f(fmaf(x[g4 * 4 + 3], c, nl.w)));
        }
        b0 = mk4(pw[0], pw[1], pw[2], pw[3]);
        b1 = mk4(pw[4], pw[5], pw[6], pw[7]);
        *reinterpret_cast<u32x4*>(px) = b0;
        *reinterpret_cast<u32x4*>(px + 1024) = b1;
      } else {
        // dP - delta before the barrier: the statistics belong to the stage being retired
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const float4 dl = *reinterpret_cast<const float4*>(stat + 64 + qb * 32 + g4 * 8 + half * 4);
          x[g4 * 4 + 0] -= dl.x; x[g4 * 4 + 1] -= dl.y; x[g4 * 4 + 2] -= dl.z; x[g4 * 4 + 3] -= dl.w;
        }
      }
      if (qb == 0) {
        lds_barrier_after_write();
      } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): own copies of the next tile
        lds_barrier_after_write();
        if (it + 1 < niter) {
#pragma unroll
          for (int ks = 0; ks < 8; ++ks) o1[ks] = *reinterpret_cast<const u32x4*>(oth + na[ks]);
        }
      }
      if (!role_p) {
        const u32x4 p0 = *reinterpret_cast<const u32x4*>(px);
        const u32x4 p1 = *reinterpret_cast<const u32x4*>(px + 1024);
        const uint32_t pw[8] = {p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
        uint32_t sw[8];
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const float pa = __uint_as_float(pw[g4 * 2] << 16), pb_ = __uint_as_float(pw[g4 * 2] & 0xffff0000u);
          const float pc = __uint_as_float(pw[g4 * 2 + 1] << 16), pd = __uint_as_float(pw[g4 * 2 + 1] & 0xffff0000u);
          sw[g4 * 2] = pack2(pa * x[g4 * 4 + 0], pb_ * x[g4 * 4 + 1]);
          sw[g4 * 2 + 1] = pack2(pc * x[g4 * 4 + 2], pd * x[g4 * 4 + 3]);
        }
        b0 = mk4(sw[0], sw[1], sw[2], sw[3]);
        b1 = mk4(sw[4], sw[5], sw[6], sw[7]);
      }
      __builtin_amdgcn_sched_barrier(0);
      // second product: dV^T += dO^T P (P role) or dK^T += Q^T dS (D role)
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        acc[db] = mfma32(o2[2 * db], b0, acc[db]);
        acc[db] = mfma32(o2[2 * db + 1], b1, acc[db]);
        if (db == 1) {
          if (qb == 0) {
            if (it + 1 < niter) fetch_piece(3, fc, oth, ostat);
            advance(fc);
          } else if (it + 2 < niter) {
            fetch_piece(0, fc, cur, stat);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
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
  const float mul = role_p ? 1.f : a.scale;
  if (nsplit > 1) {                                      // partial result of this range, summed by dkdv_reduce_kernel
    const int64_t slot_elems = (int64_t)n_kt * kKeys * a.Hkv * 128;
    float* out = w.partial + ((int64_t)(role_p ? nsplit : 0) + split) * slot_elems + ((int64_t)key * a.Hkv + kvh) * 128 + half * 4;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4)
        *reinterpret_cast<float4*>(out + db * 32 + g4 * 8) =
            make_float4(mul * acc[db][g4 * 4 + 0], mul * acc[db][g4 * 4 + 1], mul * acc[db][g4 * 4 + 2], mul * acc[db][g4 * 4 + 3]);
    return;
  }
  const int64_t off = ((int64_t)(a.k_row0 + key) * a.Hkv + kvh) * 128 + half * 4;
  float* out = (role_p ? a.dv : a.dk) + off;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      float4* p = reinterpret_cast<float4*>(out + db * 32 + g4 * 8);
      float4 x = make_float4(mul * acc[db][g4 * 4 + 0], mul * acc[db][g4 * 4 + 1], mul * acc[db][g4 * 4 + 2],
                             mul * acc[db][g4 * 4 + 3]);
      if (a.accumulate) {
        const float4 o = *p;
        x.x += o.x; x.y += o.y; x.z += o.z; x.w += o.w;
      }
      *p = x;
    }
}

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
