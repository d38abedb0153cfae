// C-ABI layer: argument checks, host-side zigzag layout / ring plan, dispatch to the kernels.
// No device memory is allocated here and nothing synchronises.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "../../include/mmsp.h"
#include "common.h"

namespace {

thread_local char g_err[512] = "";

mmsp_status fail(mmsp_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

constexpr int64_t kMaxExtent = (int64_t)1 << 30;   // rows and positions are int32 inside the kernels

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

mmsp_status check_shape(const mmsp_shape* s) {
  if (s == nullptr) return fail(MMSP_ERR_INVALID_ARG, "shape is NULL");
  if (s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->n_q_heads % s->n_kv_heads != 0)
    return fail(MMSP_ERR_INVALID_ARG, "n_q_heads=%d must be a positive multiple of n_kv_heads=%d", s->n_q_heads,
                s->n_kv_heads);
  if (s->io_dtype != MMSP_BF16 && s->io_dtype != MMSP_F32)
    return fail(MMSP_ERR_INVALID_ARG, "io_dtype=%d is not MMSP_BF16 or MMSP_F32", s->io_dtype);
  if (!(s->softmax_scale > 0.f) || !std::isfinite(s->softmax_scale))
    return fail(MMSP_ERR_INVALID_ARG, "softmax_scale must be positive and finite");
  if (s->head_dim != 64 && s->head_dim != 128)
    return fail(MMSP_ERR_UNSUPPORTED, "head_dim=%d: only 64 and 128 have kernels", s->head_dim);
  if (s->io_dtype == MMSP_BF16 && s->head_dim != 128)
    return fail(MMSP_ERR_UNSUPPORTED, "bf16 needs head_dim 128 (got %d)", s->head_dim);
  const int64_t d = s->head_dim;
  if (s->q_tok_stride < d || s->q_head_stride < d || s->kv_tok_stride < d || s->kv_head_stride < d ||
      s->q_tok_stride % 8 || s->q_head_stride % 8 || s->kv_tok_stride % 8 || s->kv_head_stride % 8)
    return fail(MMSP_ERR_INVALID_ARG, "Q/KV strides must be >= head_dim and multiples of 8 elements");
  if (s->q_tok_stride > (1 << 23) || s->kv_tok_stride > (1 << 23))
    return fail(MMSP_ERR_INVALID_ARG, "token strides above 2^23 elements are not supported");
  if (s->lse_head_stride < 0) return fail(MMSP_ERR_INVALID_ARG, "lse_head_stride is negative");
  return MMSP_OK;
}

mmsp_status check_rows(const mmsp_shape* s, int64_t row0, int64_t n_rows) {
  if (row0 < 0 || n_rows < 0 || row0 + n_rows > kMaxExtent)
    return fail(MMSP_ERR_INVALID_ARG, "row range [%lld, +%lld) is negative or exceeds 2^30", (long long)row0,
                (long long)n_rows);
  if (s->lse_head_stride < row0 + n_rows)
    return fail(MMSP_ERR_INVALID_ARG, "lse_head_stride=%lld is smaller than the last row %lld",
                (long long)s->lse_head_stride, (long long)(row0 + n_rows));
  return MMSP_OK;
}

mmsp_status check_block(const mmsp_shape* s, const mmsp_block* b) {
  if (b == nullptr) return fail(MMSP_ERR_INVALID_ARG, "block is NULL");
  mmsp_status st = check_rows(s, b->q_row0, b->n_q);
  if (st != MMSP_OK) return st;
  if (b->k_row0 < 0 || b->n_k < 0 || b->k_row0 + b->n_k > kMaxExtent)
    return fail(MMSP_ERR_INVALID_ARG, "key range [%lld, +%lld) is negative or exceeds 2^30", (long long)b->k_row0,
                (long long)b->n_k);
  // positions are int32 inside the kernels: the last position of either side must fit too
  if (b->q_pos0 < -kMaxExtent || b->q_pos0 + b->n_q > kMaxExtent || b->k_pos0 < -kMaxExtent || b->k_pos0 + b->n_k > kMaxExtent)
    return fail(MMSP_ERR_INVALID_ARG, "positions [q_pos0, q_pos0 + n_q) and [k_pos0, k_pos0 + n_k) must lie in [-2^30, 2^30]");
  if (b->mask != MMSP_MASK_FULL && b->mask != MMSP_MASK_CAUSAL_DIAG && b->mask != MMSP_MASK_NONE)
    return fail(MMSP_ERR_INVALID_ARG, "mask=%d is not a mmsp_mask", b->mask);
  if ((b->cu_seqlens == nullptr) != (b->n_docs == 0) || b->n_docs < 0)
    return fail(MMSP_ERR_INVALID_ARG, "cu_seqlens and n_docs must be given together (n_docs >= 1)");
  return MMSP_OK;
}

mmsp::StepArgs make_args(const mmsp_shape* s, const mmsp_block* b) {
  mmsp::StepArgs a;
  memset(&a, 0, sizeof(a));
  a.Hq = s->n_q_heads; a.Hkv = s->n_kv_heads; a.group = s->n_q_heads / s->n_kv_heads; a.d = s->head_dim;
  a.q_ts = s->q_tok_stride; a.q_hs = s->q_head_stride; a.kv_ts = s->kv_tok_stride; a.kv_hs = s->kv_head_stride;
  a.lse_hs = s->lse_head_stride; a.scale = s->softmax_scale;
  a.q_row0 = (int32_t)b->q_row0; a.n_q = (int32_t)b->n_q; a.k_row0 = (int32_t)b->k_row0; a.n_k = (int32_t)b->n_k;
  a.q_pos0 = (int32_t)b->q_pos0; a.k_pos0 = (int32_t)b->k_pos0;
  a.mask = b->mask; a.n_docs = b->n_docs; a.cu = b->cu_seqlens;
  return a;
}

mmsp_status device_result(hipError_t e, const char* what) {
  if (e == hipSuccess) return MMSP_OK;
  return fail(MMSP_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

// Only the bf16 backward needs scratch: padded row statistics and the partial dK / dV sums of
// split key tiles (dK/dV kernel).
size_t needed_workspace(const mmsp_shape* s, int64_t n_q, int64_t n_k, bool backward) {
  (void)n_k;
  if (backward) return (size_t)mmsp::bwd_bf16_workspace_bytes(s->n_q_heads, n_q);
  return 0;
}

mmsp_status check_workspace(const mmsp_shape* s, const mmsp_block* b, bool backward, const void* ws, size_t ws_bytes) {
  if (s->io_dtype != MMSP_BF16) return MMSP_OK;
  const size_t need = needed_workspace(s, b->n_q, b->n_k, backward);
  if (need == 0) return MMSP_OK;
  if (ws == nullptr || ws_bytes < need)
    return fail(MMSP_ERR_WORKSPACE_TOO_SMALL, "workspace of %zu bytes given, %zu needed (mmsp_workspace_bytes)", ws_bytes, need);
  if (!aligned16(ws)) return fail(MMSP_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
  return MMSP_OK;
}

mmsp_status check_zigzag(int64_t T, int32_t N, int32_t rank) {
  if (T <= 0 || N <= 0 || T % (2 * (int64_t)N) != 0)
    return fail(MMSP_ERR_INVALID_ARG, "T=%lld must be a positive multiple of 2N (N=%d)", (long long)T, N);
  if (rank < 0 || rank >= N) return fail(MMSP_ERR_INVALID_ARG, "rank=%d is not in [0, %d)", rank, N);
  return MMSP_OK;
}

mmsp_status check_rows_copy(int64_t row_bytes, const void* a, const void* b) {
  if (row_bytes <= 0 || row_bytes % 16 != 0) return fail(MMSP_ERR_INVALID_ARG, "row size %lld must be a positive multiple of 16 bytes", (long long)row_bytes);
  if (a == nullptr || b == nullptr || a == b) return fail(MMSP_ERR_INVALID_ARG, "source and destination must be distinct non-NULL buffers");
  if (!aligned16(a) || !aligned16(b)) return fail(MMSP_ERR_INVALID_ARG, "buffers must be 16-byte aligned");
  return MMSP_OK;
}

}  // namespace

// Scratch of mmsp_attn_step_bwd_static: lives in the library's device image, so every GPU the
// library runs on holds its own copy from load to process end.  Host code never uses the
// array's name as an address (on the host it is only a handle for the symbol lookup): the
// device address is asked for once per device and kept.
constexpr size_t kStaticScratchBytes = 72u << 20;
static __device__ __align__(256) char scratch[kStaticScratchBytes];

static hipError_t static_scratch(char** out) {
  static std::mutex mu;
  static char* address_on_device[64] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (address_on_device[dev] == nullptr) {
    char* ptr = nullptr;
    e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));   // of the current device's copy
    if (e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    address_on_device[dev] = ptr;
  }
  *out = address_on_device[dev];
  return hipSuccess;
}

extern "C" {

const char* mmsp_last_error(void) { return g_err; }

mmsp_status mmsp_zigzag_layout(int64_t T, int32_t N, int32_t rank, int32_t chunk_ids[2], int64_t* local_to_global) {
  mmsp_status st = check_zigzag(T, N, rank);
  if (st != MMSP_OK) return st;
  if (chunk_ids == nullptr) return fail(MMSP_ERR_INVALID_ARG, "chunk_ids is NULL");
  const int64_t C = T / (2 * (int64_t)N);
  chunk_ids[0] = rank;
  chunk_ids[1] = 2 * N - 1 - rank;
  if (local_to_global != nullptr) {
    for (int64_t i = 0; i < C; ++i) {
      local_to_global[i] = (int64_t)chunk_ids[0] * C + i;
      local_to_global[C + i] = (int64_t)chunk_ids[1] * C + i;
    }
  }
  return MMSP_OK;
}

mmsp_status mmsp_contiguous_plan(int64_t T, int32_t N, int32_t rank, int32_t step, int32_t* src_rank, mmsp_block* blk) {
  if (T <= 0 || N <= 0 || T % N != 0) return fail(MMSP_ERR_INVALID_ARG, "T=%lld must be a positive multiple of N=%d", (long long)T, N);
  if (rank < 0 || rank >= N || step < 0 || step >= N)
    return fail(MMSP_ERR_INVALID_ARG, "rank=%d and step=%d must be in [0, %d)", rank, step, N);
  if (src_rank == nullptr || blk == nullptr) return fail(MMSP_ERR_INVALID_ARG, "src_rank or blk is NULL");
  const int32_t src = ((rank - step) % N + N) % N;
  *src_rank = src;
  memset(blk, 0, sizeof(*blk));
  blk->n_q = T / N; blk->n_k = T / N;
  blk->mask = src == rank ? MMSP_MASK_CAUSAL_DIAG : (src < rank ? MMSP_MASK_FULL : MMSP_MASK_NONE);
  return MMSP_OK;
}

mmsp_status mmsp_zigzag_plan_packed(int64_t T, int32_t N, int32_t rank, int32_t step, const int32_t* cu_seqlens_host,
                                    int32_t n_docs, int32_t* src_rank, mmsp_block blks[4], int32_t* n_blocks) {
  mmsp_status st = check_zigzag(T, N, rank);
  if (st != MMSP_OK) return st;
  if (step < 0 || step >= N) return fail(MMSP_ERR_INVALID_ARG, "step=%d is not in [0, %d)", step, N);
  if (src_rank == nullptr || blks == nullptr || n_blocks == nullptr)
    return fail(MMSP_ERR_INVALID_ARG, "src_rank, blks or n_blocks is NULL");
  if (cu_seqlens_host != nullptr && n_docs <= 0) return fail(MMSP_ERR_INVALID_ARG, "cu_seqlens_host given with n_docs=%d", n_docs);
  const int64_t C = T / (2 * (int64_t)N);
  const int32_t src = ((rank - step) % N + N) % N;
  *src_rank = src;
  const int32_t q_chunk[2] = {rank, 2 * N - 1 - rank}, k_chunk[2] = {src, 2 * N - 1 - src};
  int32_t n = 0;
  for (int qi = 0; qi < 2; ++qi)
    for (int ki = 0; ki < 2; ++ki) {
      if (k_chunk[ki] > q_chunk[qi]) continue;          // every key of the segment follows every query
      if (cu_seqlens_host != nullptr && k_chunk[ki] < q_chunk[qi]) {
        // A document is contiguous: one that holds a key of the earlier chunk and a query of the
        // later chunk holds the later chunk's first position, so it must start before the
        // earlier chunk ends.  Positions outside every document see nothing.
        const int64_t p = q_chunk[qi] * C;
        if (p >= cu_seqlens_host[n_docs] || p < cu_seqlens_host[0]) continue;
        int32_t lo = 0, hi = n_docs;                    // cu[lo] <= p < cu[hi]
        while (hi - lo > 1) { const int32_t m = (lo + hi) / 2; if (cu_seqlens_host[m] <= p) lo = m; else hi = m; }
        if (cu_seqlens_host[lo] >= (k_chunk[ki] + 1) * C) continue;
      }
      mmsp_block* b = &blks[n++];
      memset(b, 0, sizeof(*b));
      b->q_row0 = qi * C; b->n_q = C; b->k_row0 = ki * C; b->n_k = C;
      b->q_pos0 = q_chunk[qi] * C; b->k_pos0 = k_chunk[ki] * C;
      b->mask = MMSP_MASK_CAUSAL_DIAG;
    }
  *n_blocks = n;
  return MMSP_OK;
}

mmsp_status mmsp_2d_layout(int64_t T, int32_t U, int32_t R, int32_t gpu, int32_t n_q_heads, int32_t n_kv_heads,
                           mmsp_2d_share* share) {
  if (share == nullptr) return fail(MMSP_ERR_INVALID_ARG, "share is NULL");
  if (U <= 0 || R <= 0) return fail(MMSP_ERR_INVALID_ARG, "U=%d and R=%d must be positive", U, R);
  if (gpu < 0 || (int64_t)gpu >= (int64_t)U * R) return fail(MMSP_ERR_INVALID_ARG, "gpu=%d is not in [0, U*R=%lld)", gpu, (long long)U * R);
  if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0)
    return fail(MMSP_ERR_INVALID_ARG, "n_kv_heads=%d must divide n_q_heads=%d", n_kv_heads, n_q_heads);
  if (n_q_heads % U != 0) return fail(MMSP_ERR_INVALID_ARG, "U=%d must divide n_q_heads=%d", U, n_q_heads);
  if (n_kv_heads % U != 0 && U % n_kv_heads != 0)
    return fail(MMSP_ERR_INVALID_ARG, "U=%d must divide n_kv_heads=%d or be a multiple of it", U, n_kv_heads);
  const int32_t u = gpu % U, r = gpu / U;
  mmsp_status st = check_zigzag(T, R, r);
  if (st != MMSP_OK) return st;
  share->head_rank = u; share->ring_rank = r;
  share->n_q_heads = n_q_heads / U;
  share->q_head0 = u * share->n_q_heads;
  if (n_kv_heads % U == 0) {
    share->n_kv_heads = n_kv_heads / U;
    share->kv_head0 = u * share->n_kv_heads;
  } else {                       // more head ranks than KV heads: U / n_kv_heads GPUs share one KV head
    share->n_kv_heads = 1;
    share->kv_head0 = u / (U / n_kv_heads);
  }
  share->chunk_ids[0] = r; share->chunk_ids[1] = 2 * R - 1 - r;
  share->chunk_len = T / (2 * (int64_t)R);
  return MMSP_OK;
}

mmsp_status mmsp_zigzag_plan(int64_t T, int32_t N, int32_t rank, int32_t step, int32_t* src_rank, mmsp_block* blk) {
  mmsp_status st = check_zigzag(T, N, rank);
  if (st != MMSP_OK) return st;
  if (step < 0 || step >= N) return fail(MMSP_ERR_INVALID_ARG, "step=%d is not in [0, %d)", step, N);
  if (src_rank == nullptr || blk == nullptr) return fail(MMSP_ERR_INVALID_ARG, "src_rank or blk is NULL");
  const int64_t C = T / (2 * (int64_t)N);
  const int32_t src = ((rank - step) % N + N) % N;
  *src_rank = src;
  memset(blk, 0, sizeof(*blk));
  if (src == rank) {            // own block: chunk r precedes chunk 2N-1-r, so local order is causal order
    blk->q_row0 = 0; blk->n_q = 2 * C; blk->k_row0 = 0; blk->n_k = 2 * C; blk->mask = MMSP_MASK_CAUSAL_DIAG;
  } else if (src < rank) {      // chunk src precedes both local chunks, chunk 2N-1-src follows both
    blk->q_row0 = 0; blk->n_q = 2 * C; blk->k_row0 = 0; blk->n_k = C; blk->mask = MMSP_MASK_FULL;
  } else {                      // both visiting chunks lie between the two local chunks
    blk->q_row0 = C; blk->n_q = C; blk->k_row0 = 0; blk->n_k = 2 * C; blk->mask = MMSP_MASK_FULL;
  }
  return MMSP_OK;
}

size_t mmsp_workspace_bytes(const mmsp_shape* shape, int64_t n_q_max, int64_t n_k_max, int backward) {
  if (shape == nullptr || shape->io_dtype != MMSP_BF16 || n_q_max < 0 || n_k_max < 0) return 0;
  return needed_workspace(shape, n_q_max, n_k_max, backward != 0);
}

mmsp_status mmsp_attn_step_fwd(const mmsp_shape* shape, const mmsp_block* blk, const void* q, const void* k,
                               const void* v, float* o, float* lse, int accumulate, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
  mmsp_status st = check_shape(shape);
  if (st != MMSP_OK) return st;
  st = check_block(shape, blk);
  if (st != MMSP_OK) return st;
  if (q == nullptr || k == nullptr || v == nullptr || o == nullptr || lse == nullptr)
    return fail(MMSP_ERR_INVALID_ARG, "q, k, v, o and lse must be non-NULL");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o))
    return fail(MMSP_ERR_INVALID_ARG, "q, k, v and o must be 16-byte aligned");
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  if (blk->n_q == 0) return MMSP_OK;
  if (blk->mask != MMSP_MASK_NONE && blk->n_k > 0) {
    st = check_workspace(shape, blk, false, workspace, workspace_bytes);
    if (st != MMSP_OK) return st;
  }
  if (blk->mask == MMSP_MASK_NONE || blk->n_k == 0) {
    if (accumulate) return MMSP_OK;
    return device_result(mmsp::launch_fill_empty(o, lse, shape->lse_head_stride, shape->n_q_heads, shape->head_dim,
                                                 (int)blk->q_row0, (int)blk->n_q, stream),
                         "fill_empty");
  }
  mmsp::StepArgs a = make_args(shape, blk);
  a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse; a.accumulate = accumulate != 0;
  a.ws = reinterpret_cast<char*>(workspace);
  if (shape->io_dtype == MMSP_BF16) return device_result(mmsp::launch_fwd_bf16(a, stream), "step_fwd (bf16)");
  return device_result(mmsp::launch_fwd_f32(a, stream), "step_fwd (f32)");
}

mmsp_status mmsp_attn_merge(const mmsp_shape* shape, int64_t row0, int64_t n_rows, float* o_acc, float* lse_acc,
                            const float* o_part, const float* lse_part, void* o_final, void* hip_stream) {
  mmsp_status st = check_shape(shape);
  if (st != MMSP_OK) return st;
  st = check_rows(shape, row0, n_rows);
  if (st != MMSP_OK) return st;
  if (o_acc == nullptr || lse_acc == nullptr) return fail(MMSP_ERR_INVALID_ARG, "o_acc and lse_acc must be non-NULL");
  if ((o_part == nullptr) != (lse_part == nullptr))
    return fail(MMSP_ERR_INVALID_ARG, "o_part and lse_part must both be given or both be NULL");
  if (o_part == nullptr && o_final == nullptr)
    return fail(MMSP_ERR_INVALID_ARG, "nothing to do: no partial to merge and no o_final to write");
  if (!aligned16(o_acc) || !aligned16(o_part) || !aligned16(o_final))
    return fail(MMSP_ERR_INVALID_ARG, "o_acc, o_part and o_final must be 16-byte aligned");
  return device_result(mmsp::launch_merge(o_acc, lse_acc, o_part, lse_part, o_final, shape->io_dtype,
                                          shape->lse_head_stride, shape->n_q_heads, shape->head_dim, (int)row0,
                                          (int)n_rows, reinterpret_cast<hipStream_t>(hip_stream)),
                       "merge");
}

mmsp_status mmsp_zigzag_gather(int64_t T, int32_t N, int64_t row_bytes, const void* seq, void* shards, void* hip_stream) {
  mmsp_status st = check_zigzag(T, N, 0);
  if (st != MMSP_OK) return st;
  st = check_rows_copy(row_bytes, seq, shards);
  if (st != MMSP_OK) return st;
  return device_result(mmsp::launch_zigzag_gather(seq, shards, T, N, row_bytes, reinterpret_cast<hipStream_t>(hip_stream)), "zigzag_gather");
}

mmsp_status mmsp_zigzag_scatter(int64_t T, int32_t N, int64_t row_bytes, const void* shards, void* seq, void* hip_stream) {
  mmsp_status st = check_zigzag(T, N, 0);
  if (st != MMSP_OK) return st;
  st = check_rows_copy(row_bytes, shards, seq);
  if (st != MMSP_OK) return st;
  return device_result(mmsp::launch_zigzag_scatter(shards, seq, T, N, row_bytes, reinterpret_cast<hipStream_t>(hip_stream)), "zigzag_scatter");
}

mmsp_status mmsp_a2a_pack_heads(int64_t n_tokens, int32_t U, int64_t slice_bytes, const void* x, void* y, void* hip_stream) {
  if (n_tokens < 0 || U <= 0) return fail(MMSP_ERR_INVALID_ARG, "n_tokens=%lld must be >= 0 and U=%d > 0", (long long)n_tokens, U);
  mmsp_status st = check_rows_copy(slice_bytes, x, y);
  if (st != MMSP_OK) return st;
  return device_result(mmsp::launch_swap_outer(x, y, n_tokens, U, slice_bytes, reinterpret_cast<hipStream_t>(hip_stream)), "a2a_pack_heads");
}

mmsp_status mmsp_a2a_unpack_heads(int64_t n_tokens, int32_t U, int64_t slice_bytes, const void* y, void* x, void* hip_stream) {
  if (n_tokens < 0 || U <= 0) return fail(MMSP_ERR_INVALID_ARG, "n_tokens=%lld must be >= 0 and U=%d > 0", (long long)n_tokens, U);
  mmsp_status st = check_rows_copy(slice_bytes, y, x);
  if (st != MMSP_OK) return st;
  return device_result(mmsp::launch_swap_outer(y, x, U, n_tokens, slice_bytes, reinterpret_cast<hipStream_t>(hip_stream)), "a2a_unpack_heads");
}

mmsp_status mmsp_attn_delta(const mmsp_shape* shape, int64_t row0, int64_t n_rows, const void* o_final,
                            const void* d_o, float* delta, void* hip_stream) {
  mmsp_status st = check_shape(shape);
  if (st != MMSP_OK) return st;
  st = check_rows(shape, row0, n_rows);
  if (st != MMSP_OK) return st;
  if (o_final == nullptr || d_o == nullptr || delta == nullptr)
    return fail(MMSP_ERR_INVALID_ARG, "o_final, d_o and delta must be non-NULL");
  if (!aligned16(o_final) || !aligned16(d_o)) return fail(MMSP_ERR_INVALID_ARG, "o_final and d_o must be 16-byte aligned");
  return device_result(mmsp::launch_delta(o_final, d_o, delta, shape->io_dtype, shape->lse_head_stride,
                                          shape->n_q_heads, shape->head_dim, (int)row0, (int)n_rows,
                                          reinterpret_cast<hipStream_t>(hip_stream)),
                       "delta");
}

mmsp_status mmsp_attn_step_bwd(const mmsp_shape* shape, const mmsp_block* blk, const void* q, const void* k,
                               const void* v, const void* o_final, const void* d_o, const float* lse_final,
                               float* delta, int compute_delta, float* dq_acc, float* dk, float* dv,
                               int accumulate_dkdv, void* workspace, size_t workspace_bytes, void* hip_stream) {
  mmsp_status st = check_shape(shape);
  if (st != MMSP_OK) return st;
  st = check_block(shape, blk);
  if (st != MMSP_OK) return st;
  if (q == nullptr || k == nullptr || v == nullptr || d_o == nullptr || lse_final == nullptr || delta == nullptr)
    return fail(MMSP_ERR_INVALID_ARG, "q, k, v, d_o, lse_final and delta must be non-NULL");
  if ((dk == nullptr) != (dv == nullptr)) return fail(MMSP_ERR_INVALID_ARG, "dk and dv must both be given or both be NULL");
  if (dq_acc == nullptr && dk == nullptr) return fail(MMSP_ERR_INVALID_ARG, "nothing to do: dq_acc, dk and dv are all NULL");
  if (compute_delta && o_final == nullptr) return fail(MMSP_ERR_INVALID_ARG, "compute_delta needs o_final");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(o_final) ||
      !aligned16(dq_acc) || !aligned16(dk) || !aligned16(dv))
    return fail(MMSP_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  // every check comes before the first launch: a failing call enqueues nothing
  const bool has_pairs = blk->n_k > 0 && blk->n_q > 0 && blk->mask != MMSP_MASK_NONE;
  if (has_pairs) {
    st = check_workspace(shape, blk, true, workspace, workspace_bytes);
    if (st != MMSP_OK) return st;
  }
  if (compute_delta && blk->n_q > 0) {
    hipError_t e = mmsp::launch_delta(o_final, d_o, delta, shape->io_dtype, shape->lse_head_stride, shape->n_q_heads,
                                      shape->head_dim, (int)blk->q_row0, (int)blk->n_q, stream);
    if (e != hipSuccess) return device_result(e, "delta");
  }
  if (blk->n_k == 0) return MMSP_OK;
  if (blk->mask == MMSP_MASK_NONE || blk->n_q == 0) {
    if (accumulate_dkdv || dk == nullptr) return MMSP_OK;
    const int64_t first = blk->k_row0 * shape->n_kv_heads * shape->head_dim;
    const int64_t count = blk->n_k * shape->n_kv_heads * shape->head_dim;
    hipError_t e = mmsp::launch_zero_f32(dk + first, count, stream);
    if (e == hipSuccess) e = mmsp::launch_zero_f32(dv + first, count, stream);
    return device_result(e, "zero dk/dv");
  }
  mmsp::StepArgs a = make_args(shape, blk);
  a.ws = reinterpret_cast<char*>(workspace);
  a.q = q; a.k = k; a.v = v; a.d_o = d_o; a.lse_final = lse_final; a.delta = delta;
  a.dq = dq_acc; a.dk = dk; a.dv = dv; a.accumulate = accumulate_dkdv != 0;
  if (shape->io_dtype == MMSP_BF16) return device_result(mmsp::launch_bwd_bf16(a, stream), "step_bwd (bf16)");
  return device_result(mmsp::launch_bwd_f32(a, stream), "step_bwd (f32)");
}

mmsp_status mmsp_attn_step_bwd_static(const mmsp_shape* shape, const mmsp_block* blk, const void* q, const void* k,
                                      const void* v, const void* o_final, const void* d_o, const float* lse_final,
                                      float* delta, int compute_delta, float* dq_acc, float* dk, float* dv,
                                      int accumulate_dkdv, void* hip_stream) {
  mmsp_status st = check_shape(shape);
  if (st != MMSP_OK) return st;
  st = check_block(shape, blk);
  if (st != MMSP_OK) return st;
  const size_t need = shape->io_dtype == MMSP_BF16 ? needed_workspace(shape, blk->n_q, blk->n_k, true) : 0;
  if (need > kStaticScratchBytes)
    return fail(MMSP_ERR_WORKSPACE_TOO_SMALL,
                "block of %lld query rows x %d heads needs %zu bytes of scratch, the built-in area holds %zu "
                "(use mmsp_attn_step_bwd with a workspace)",
                (long long)blk->n_q, shape->n_q_heads, need, kStaticScratchBytes);
  char* ptr = nullptr;
  if (need > 0) {
    hipError_t e = static_scratch(&ptr);
    if (e != hipSuccess) return device_result(e, "address of the built-in scratch");
  }
  return mmsp_attn_step_bwd(shape, blk, q, k, v, o_final, d_o, lse_final, delta, compute_delta, dq_acc, dk, dv,
                            accumulate_dkdv, ptr, need > 0 ? kStaticScratchBytes : 0, hip_stream);
}

}  // extern "C"
