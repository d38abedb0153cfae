/* Plain C99 caller of the step kernels: links against the library through the prototypes of
 * the public header and runs one forward and one backward step on device pointers it is
 * handed (tests/test_gpu_parity.py builds this file as a small shared object, loads it into
 * the test process and passes the addresses of its device buffers).  The backward goes
 * through the entry point that needs no workspace, so this caller allocates nothing. */
#include <stddef.h>

#include "mmsp.h"

static void describe(mmsp_shape* shape, mmsp_block* blk, int n_q, int n_k, int hq, int hkv, int d, float scale) {
  shape->n_q_heads = hq; shape->n_kv_heads = hkv; shape->head_dim = d; shape->io_dtype = MMSP_BF16;
  shape->softmax_scale = scale;
  shape->q_tok_stride = (int64_t)hq * d; shape->q_head_stride = d;
  shape->kv_tok_stride = (int64_t)hkv * d; shape->kv_head_stride = d;
  shape->lse_head_stride = n_q;
  blk->q_row0 = 0; blk->n_q = n_q; blk->k_row0 = 0; blk->n_k = n_k; blk->q_pos0 = n_k - n_q; blk->k_pos0 = 0;
  blk->mask = MMSP_MASK_CAUSAL_DIAG; blk->n_docs = 0; blk->cu_seqlens = NULL;
}

/* O and LSE of the block; then, with o_final = the caller's cast of O, delta, dQ += ..., dK, dV. */
int c_client_step_fwd(const void* q, const void* k, const void* v, float* o, float* lse, int n_q, int n_k, int hq,
                      int hkv, int d, float scale) {
  mmsp_shape shape; mmsp_block blk;
  describe(&shape, &blk, n_q, n_k, hq, hkv, d, scale);
  return (int)mmsp_attn_step_fwd(&shape, &blk, q, k, v, o, lse, 0, NULL, 0, NULL);
}

int c_client_step_bwd(const void* q, const void* k, const void* v, const void* o_final, const void* d_o,
                      const float* lse, float* delta, float* dq, float* dk, float* dv, int n_q, int n_k, int hq,
                      int hkv, int d, float scale) {
  mmsp_shape shape; mmsp_block blk;
  describe(&shape, &blk, n_q, n_k, hq, hkv, d, scale);
  return (int)mmsp_attn_step_bwd_static(&shape, &blk, q, k, v, o_final, d_o, lse, delta, 1, dq, dk, dv, 0, NULL);
}

const char* c_client_last_error(void) { return mmsp_last_error(); }
