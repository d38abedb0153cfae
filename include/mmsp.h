/* mmsp.h -- C ABI of the MI355X (gfx950) attention library for one rank of Multi-Modal
 * Sequence Parallelism (MM-SP; paper Sec. 4.2 "Multi-Modal Sequence Parallelism Training
 * Mode" and the figure comparing RingAttention, ZigZag-RingAttn and 2D-Attention).
 *
 * One rank of a zigzag ring holds query chunks r and 2N-1-r of a packed sequence and,
 * over N ring steps, attends them against the K/V block of every rank.  Each step is a
 * flash-style partial attention that yields (O_part, LSE_part); partials are combined by a
 * log-sum-exp merge; the backward of each step yields dQ (accumulated over steps) and the
 * step's dK/dV.  The Ulysses (head-sharded) mode is the same calls on the whole packed
 * sequence for a subset of heads, with a document-causal mask given by cu_seqlens.
 *
 * General rules
 *   - C99 types only.  Pointers are DEVICE pointers unless marked "host".
 *   - The caller owns every buffer and the HIP stream.  The library allocates, frees and
 *     retains nothing.  Work is enqueued on `hip_stream` (a hipStream_t; NULL = the null
 *     stream) and the call returns without synchronising.  Calls on one stream run in order.
 *   - Every call returns an mmsp_status.  On any status other than MMSP_OK nothing has been
 *     enqueued.  The library never aborts and never throws.  mmsp_last_error() returns a
 *     thread-local, statically stored message for the last failing call on this thread.
 *   - Tensor layouts (d = head_dim, contiguous, always the fastest axis):
 *       Q                       [rows, n_q_heads, d], element strides q_tok_stride / q_head_stride
 *       K, V                    [rows, n_kv_heads, d], element strides kv_tok_stride / kv_head_stride
 *       O (partial, running, final), dO, dQ   dense [rows, n_q_heads, d]
 *       dK, dV                  dense [rows, n_kv_heads, d]
 *       LSE, delta              [n_q_heads, rows], head stride lse_head_stride (elements)
 *     Q, K, V, dO and the final O are in io_dtype (bf16 or f32).  Partial / running O,
 *     LSE, delta, dQ, dK and dV are always f32.
 *   - Row indices in mmsp_block are relative to the base pointers: query-side buffers
 *     (Q, O, dO, dQ, LSE, delta) are indexed by the rank-local row, key-side buffers
 *     (K, V, dK, dV) by the row inside the visiting K/V block.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - Supported: head_dim 64 or 128; bf16 needs head_dim 128 for the matrix-core path.
 */
#ifndef MMSP_H
#define MMSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MMSP_OK = 0,
  MMSP_ERR_INVALID_ARG = 1,        /* null pointer, bad range, bad divisibility            */
  MMSP_ERR_UNSUPPORTED = 2,        /* head_dim / dtype combination with no kernel          */
  MMSP_ERR_WORKSPACE_TOO_SMALL = 3,
  MMSP_ERR_DEVICE = 4              /* launch failed; text in mmsp_last_error()             */
} mmsp_status;

/* Which (query row, key row) pairs of a block are visible.  "Position" is the index of a
 * row in the coordinate system named by q_pos0 / k_pos0 (see mmsp_block). */
typedef enum {
  MMSP_MASK_FULL = 0,        /* every query row sees every key row of the block           */
  MMSP_MASK_CAUSAL_DIAG = 1, /* query at position p sees keys at positions <= p           */
  MMSP_MASK_NONE = 2         /* nothing is visible: O_part = 0, LSE_part = -inf, grads 0  */
} mmsp_mask;

typedef enum { MMSP_BF16 = 0, MMSP_F32 = 1 } mmsp_dtype;

/* Problem shape.  Plain data, read during the call only. */
typedef struct {
  int32_t n_q_heads;
  int32_t n_kv_heads;        /* must divide n_q_heads                                     */
  int32_t head_dim;          /* 64 or 128                                                 */
  int32_t io_dtype;          /* mmsp_dtype of Q, K, V, dO and the final O                 */
  float   softmax_scale;     /* multiplies Q.K before the softmax; callers pass 1/sqrt(d) */
  int64_t q_tok_stride, q_head_stride;     /* element strides of Q                        */
  int64_t kv_tok_stride, kv_head_stride;   /* element strides of K and of V               */
  int64_t lse_head_stride;   /* elements between consecutive heads of LSE / delta arrays  */
} mmsp_shape;

/* The sub-block of (local queries) x (visiting keys) that one call works on. */
typedef struct {
  int64_t q_row0, n_q;       /* query rows [q_row0, q_row0 + n_q)                          */
  int64_t k_row0, n_k;       /* key rows   [k_row0, k_row0 + n_k) of the visiting block    */
  int64_t q_pos0, k_pos0;    /* position of row q_row0 / k_row0; consecutive rows have
                                consecutive positions.  Used by CAUSAL_DIAG and cu_seqlens */
  int32_t mask;              /* mmsp_mask                                                  */
  int32_t n_docs;            /* number of documents in cu_seqlens (0 when it is NULL)      */
  const int32_t* cu_seqlens; /* device, [n_docs + 1], ascending, [0] >= 0; NULL = one
                                document.  A pair is visible only if both positions fall
                                in the same document [cu[k], cu[k+1]) (packed variable-
                                length inputs); positions below cu[0] or from cu[n_docs]
                                on belong to no document and see nothing.                  */
} mmsp_block;

/* Zigzag sharding (chunks dealt from the two ends of the sequence) -- Sec. 4.2, MM-SP
 * workflow: the sequence is cut into 2N equal chunks and rank r takes chunk r and chunk 2N-1-r, so every rank owns the same
 * number of causal pairs.  chunk_ids (host, 2 ints) receives {r, 2N-1-r}.
 * local_to_global (host, T/N int64, may be NULL) receives the global token index of each
 * local row (ascending).  INVALID_ARG if T <= 0, N <= 0, T % (2N) != 0 or rank not in [0,N). */
mmsp_status mmsp_zigzag_layout(int64_t T, int32_t N, int32_t rank,
                               int32_t chunk_ids[2], int64_t* local_to_global);

/* Ring plan for the same sharding (the per-round schedule drawn in the ZigZag row of the
 * comparison figure).  At step s rank r is visited by the K/V block of rank
 * src = (r - s) mod N.  *blk (host) receives the only sub-block with visible pairs:
 *   src == r: all 2C rows x all 2C keys, CAUSAL_DIAG on local positions;
 *   src <  r: all 2C rows x the first C keys, FULL;
 *   src >  r: the last C rows x all 2C keys, FULL.
 * cu_seqlens is left NULL.  INVALID_ARG as above or if step not in [0,N). */
mmsp_status mmsp_zigzag_plan(int64_t T, int32_t N, int32_t rank, int32_t step,
                             int32_t* src_rank, mmsp_block* blk);

/* The ring step of the plain (contiguous) RingAttention layout, the comparison figure's first
 * row and the baseline the zigzag rule is measured against: rank r holds chunk r of N equal
 * chunks; the block of rank src = (rank - step) mod N visits.  src == rank: all T/N rows,
 * CAUSAL_DIAG; src < rank: FULL; src > rank: MMSP_MASK_NONE (the rank has nothing to do, which
 * is the imbalance the paper describes: rank 0 idles after the first round).  INVALID_ARG if
 * T <= 0, N <= 0, T % N != 0, or rank / step not in [0,N). */
mmsp_status mmsp_contiguous_plan(int64_t T, int32_t N, int32_t rank, int32_t step,
                                 int32_t* src_rank, mmsp_block* blk);

/* The same ring step for a packed (variable-length) sequence whose document mask is given by
 * cu_seqlens on global positions -- Sec. 4.2, MM-SP workflow (token-level sharding of the
 * packed vision + text inputs from both ends).  A rank's local rows are two segments with
 * different global positions, and so is the visiting block, so the step is cut into
 * sub-blocks of one query segment x one key segment, inside which positions are consecutive:
 * blks[0 .. *n_blocks) (at most 4, 3 for the own block, 2 otherwise) are MMSP_MASK_CAUSAL_DIAG
 * blocks of C x C rows with q_pos0 / k_pos0 set to global positions; segment pairs in which no
 * key can precede a query are left out, and so are, when the host copy cu_seqlens_host
 * ([n_docs + 1], may be NULL) is given, segment pairs that no document spans (*n_blocks can
 * then be 0).  The blocks' cu_seqlens / n_docs are left NULL / 0 for the caller to fill in with
 * the device copy (with NULL the sub-blocks reproduce the plain causal plan).  The forward
 * calls accumulate in order; in the backward a key segment touched by two sub-blocks of a step
 * needs accumulate_dkdv on the second, and key rows of the visiting block that no sub-block
 * touches receive no gradient from this step.  Errors as mmsp_zigzag_plan, and INVALID_ARG if
 * cu_seqlens_host is given with n_docs <= 0. */
mmsp_status mmsp_zigzag_plan_packed(int64_t T, int32_t N, int32_t rank, int32_t step,
                                    const int32_t* cu_seqlens_host, int32_t n_docs,
                                    int32_t* src_rank, mmsp_block blks[4], int32_t* n_blocks);

/* One GPU's share under 2D-attention -- Sec. 4.2 (the U x R communication mesh) and the
 * comparison figure's 2D-Attention row: a sequence-parallel group of U * R GPUs computes
 * attention with the heads split U ways (inside the all-to-all group, which is U consecutive
 * GPUs) and the sequence split R ways by the zigzag rule (ring group).  GPU g = r * U + u works
 * on query heads [q_head0, q_head0 + n_q_heads), their KV heads [kv_head0, kv_head0 +
 * n_kv_heads) (a KV head is replicated on several GPUs when U > n_kv_heads), and runs the R
 * ring steps of mmsp_zigzag_plan(T, R, ring_rank, step) on chunks chunk_ids[] of length
 * chunk_len = T / (2R).  Host integers only. */
typedef struct {
  int32_t head_rank, ring_rank;      /* u in [0,U), r in [0,R)                              */
  int32_t q_head0, n_q_heads;
  int32_t kv_head0, n_kv_heads;
  int32_t chunk_ids[2];              /* {r, 2R-1-r}                                         */
  int64_t chunk_len;
} mmsp_2d_share;

/* INVALID_ARG unless U, R > 0, gpu in [0, U*R), T a positive multiple of 2R, U divides
 * n_q_heads, n_kv_heads divides n_q_heads, and U divides n_kv_heads or n_kv_heads divides U. */
mmsp_status mmsp_2d_layout(int64_t T, int32_t U, int32_t R, int32_t gpu, int32_t n_q_heads, int32_t n_kv_heads,
                           mmsp_2d_share* share);

/* Token-level zigzag sharding of a whole sequence -- Sec. 4.2, MM-SP workflow (the
 * second stage of the two-stage sharding).  seq (device) holds T rows of row_bytes bytes in
 * sequence order (a row is one token's heads x d elements, any dtype); shards (device) holds
 * the N ranks' local rows back to back, [N][2C] rows with C = T / (2N), rank r = chunk r then
 * chunk 2N-1-r -- the order mmsp_zigzag_layout describes and the ring steps expect.  gather
 * writes shards from seq, scatter writes seq from shards (e.g. O or dQ back in sequence order).
 * One pass, 1 byte read + 1 byte written per byte.  row_bytes must be a positive multiple of
 * 16, both pointers 16-byte aligned and the buffers must not overlap.  INVALID_ARG otherwise,
 * or if T is not a positive multiple of 2N. */
mmsp_status mmsp_zigzag_gather(int64_t T, int32_t N, int64_t row_bytes, const void* seq, void* shards, void* hip_stream);
mmsp_status mmsp_zigzag_scatter(int64_t T, int32_t N, int64_t row_bytes, const void* shards, void* seq, void* hip_stream);

/* Local re-grouping around the all-to-all of the head-sharded mode -- Sec. 4.2 (the all-to-all
 * group distributes QKV by head and re-partitions along the sequence).  Before the exchange a
 * GPU holds [n_tokens][U][slice_bytes] (its tokens, all heads as U head groups) and must send
 * group u to peer u: pack writes y = [U][n_tokens][slice_bytes], one contiguous message per
 * peer.  After the return exchange it holds [U][n_tokens][slice_bytes] (one message per head
 * group) and unpack restores x = [n_tokens][U][slice_bytes].  slice_bytes = heads per group x
 * d x element size, a positive multiple of 16; pointers 16-byte aligned, no overlap. */
mmsp_status mmsp_a2a_pack_heads(int64_t n_tokens, int32_t U, int64_t slice_bytes, const void* x, void* y, void* hip_stream);
mmsp_status mmsp_a2a_unpack_heads(int64_t n_tokens, int32_t U, int64_t slice_bytes, const void* y, void* x, void* hip_stream);

/* Bytes of device workspace the step calls need for blocks of at most n_q_max x n_k_max rows.
 * The forward needs none (0; its kernels read the caller's tensors in place), neither does
 * f32.  The bf16 backward (`backward` != 0) uses the workspace for the block's row statistics
 * (-LSE and delta, padded to whole tiles: 8 bytes per query row and head) and for partial
 * dK/dV sums of key tiles whose query range was cut into several workgroups (a fixed 64 MiB);
 * nothing in it outlives the kernels of a call.  The workspace must be 16-byte aligned; a call
 * given less returns MMSP_ERR_WORKSPACE_TOO_SMALL.  Two calls that may overlap in time
 * (different streams) need separate workspaces. */
size_t mmsp_workspace_bytes(const mmsp_shape* shape, int64_t n_q_max, int64_t n_k_max, int backward);

/* One ring step, forward (the per-rank attention of one ring round; comparison figure,
 * Sec. 4.2):  for each query head h and query row i of the block,
 *   S_j = softmax_scale * Q[i,h,:] . K[j,kv(h),:]  over the visible keys j of the block,
 *   LSE_part = ln sum_j exp(S_j),  O_part = sum_j exp(S_j - LSE_part) V[j,kv(h),:].
 * accumulate == 0: o and lse are overwritten with (O_part, LSE_part) for rows of the block.
 * accumulate != 0: o and lse hold the running result and the log-sum-exp merge with the
 *   partial is applied in the kernel's epilogue (same arithmetic as mmsp_attn_merge).
 * Rows outside [q_row0, q_row0+n_q) are not touched.  A row that sees nothing gets
 * O_part = 0, LSE_part = -inf (and leaves a running result unchanged).
 * workspace: at least mmsp_workspace_bytes(shape, n_q, n_k, 0) bytes (may be NULL when 0). */
mmsp_status mmsp_attn_step_fwd(const mmsp_shape* shape, const mmsp_block* blk,
                               const void* q, const void* k, const void* v,
                               float* o, float* lse, int accumulate,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* Log-sum-exp merge of a partial into the running result on rows [row0, row0+n_rows)
 * (how the per-round results of ring attention are combined; the paper leaves the formula
 * implicit):  L' = ln(e^L + e^Lp),  O' = e^(L-L') O + e^(Lp-L') Op,  with a side whose LSE
 * is -inf contributing nothing.  o_acc / lse_acc are updated in place.
 * If o_final != NULL it also receives O' cast to io_dtype (dense [rows, n_q_heads, d]).
 * With o_part == NULL and lse_part == NULL nothing is merged and only the cast is done
 * (o_final must then be non-NULL). */
mmsp_status mmsp_attn_merge(const mmsp_shape* shape, int64_t row0, int64_t n_rows,
                            float* o_acc, float* lse_acc,
                            const float* o_part, const float* lse_part,
                            void* o_final, void* hip_stream);

/* delta[h,i] = sum_c dO[i,h,c] * O_final[i,h,c] on rows [row0, row0+n_rows): the
 * softmax-backward row term, computed once per rank from the final merged O. */
mmsp_status mmsp_attn_delta(const mmsp_shape* shape, int64_t row0, int64_t n_rows,
                            const void* o_final, const void* d_o, float* delta, void* hip_stream);

/* One ring step, backward.  With P = exp(S - lse_final) on visible pairs (0 elsewhere):
 *   dV[j,kv] (+)= sum_{h in group} sum_i P dO[i,h,:]
 *   dS = P * (dO[i,h,:] . V[j,kv,:] - delta[h,i])
 *   dK[j,kv] (+)= softmax_scale * sum_{h in group} sum_i dS Q[i,h,:]
 *   dQ[i,h]   += softmax_scale * sum_j dS K[j,kv,:]
 * lse_final / delta are those of the completed forward (all steps merged).
 * compute_delta != 0: delta for the block's query rows is first computed from o_final and
 *   d_o (as mmsp_attn_delta) and stored in `delta`; otherwise o_final may be NULL.
 * dq_acc is always accumulated into (the caller zeroes it before the first step).
 * accumulate_dkdv == 0 overwrites dk/dv rows [k_row0, k_row0+n_k); != 0 adds to them.
 * dq_acc may be NULL to skip dQ; dk and dv may both be NULL to skip dK/dV (in a ring the
 * two travel differently: dQ stays with the rank, dK/dV follow the K/V block).
 * Results are bit-identical from run to run (no floating-point atomics). */
mmsp_status mmsp_attn_step_bwd(const mmsp_shape* shape, const mmsp_block* blk,
                               const void* q, const void* k, const void* v,
                               const void* o_final, const void* d_o,
                               const float* lse_final, float* delta, int compute_delta,
                               float* dq_acc, float* dk, float* dv, int accumulate_dkdv,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* mmsp_attn_step_bwd for callers that cannot allocate device memory or pass a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * same kernels, with their scratch (padded row statistics, partial dK/dV sums) in a 72 MiB
 * area built into the library's device image instead of a caller workspace.  Each GPU the
 * library runs on holds that area until the process ends.  The call allocates and frees
 * nothing.  A block whose scratch need exceeds the area (n_q_heads x n_q rows, padded to 64,
 * above 1,048,576) is rejected with MMSP_ERR_WORKSPACE_TOO_SMALL before anything is enqueued.
 * Nothing in the area has to start at zero and nothing in it outlives the call's kernels, but
 * all calls on one GPU share it: calls that may overlap in time (different streams, or
 * threads) race; keep them on one stream.  Arguments and results as mmsp_attn_step_bwd. */
mmsp_status mmsp_attn_step_bwd_static(const mmsp_shape* shape, const mmsp_block* blk,
                                      const void* q, const void* k, const void* v,
                                      const void* o_final, const void* d_o,
                                      const float* lse_final, float* delta, int compute_delta,
                                      float* dq_acc, float* dk, float* dv, int accumulate_dkdv,
                                      void* hip_stream);

/* Message for the last non-OK status returned on the calling thread ("" if none). */
const char* mmsp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MMSP_H */
