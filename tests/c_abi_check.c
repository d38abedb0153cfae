/* Plain C99 client of the boundary: includes the public header, loads the shared library and
 * calls host-side entry points through the declared prototypes.  Built and run by
 * tests/test_host_api.py; proves that the header is C (no C++ or framework types) and that
 * the symbols have C linkage. */
#include <dlfcn.h>
#include <stdio.h>
#include <string.h>

#include "mmsp.h"

#define LOAD(name) do { *(void**)(&p_##name) = dlsym(lib, #name); if (!p_##name) { printf("missing %s\n", #name); return 2; } } while (0)

int main(int argc, char** argv) {
  if (argc < 2) return 2;
  void* lib = dlopen(argv[1], RTLD_NOW);
  if (!lib) { printf("dlopen: %s\n", dlerror()); return 2; }
  mmsp_status (*p_mmsp_zigzag_layout)(int64_t, int32_t, int32_t, int32_t*, int64_t*);
  mmsp_status (*p_mmsp_zigzag_plan)(int64_t, int32_t, int32_t, int32_t, int32_t*, mmsp_block*);
  mmsp_status (*p_mmsp_2d_layout)(int64_t, int32_t, int32_t, int32_t, int32_t, int32_t, mmsp_2d_share*);
  size_t (*p_mmsp_workspace_bytes)(const mmsp_shape*, int64_t, int64_t, int);
  const char* (*p_mmsp_last_error)(void);
  LOAD(mmsp_zigzag_layout); LOAD(mmsp_zigzag_plan); LOAD(mmsp_2d_layout); LOAD(mmsp_workspace_bytes); LOAD(mmsp_last_error);

  int32_t ids[2]; int64_t l2g[2];
  if (p_mmsp_zigzag_layout(8, 4, 1, ids, l2g) != MMSP_OK) return 1;
  printf("layout %d %d %lld %lld\n", ids[0], ids[1], (long long)l2g[0], (long long)l2g[1]);
  int32_t src; mmsp_block blk;
  if (p_mmsp_zigzag_plan(262144, 32, 0, 1, &src, &blk) != MMSP_OK) return 1;
  printf("plan %d %lld %lld %lld %lld %d\n", src, (long long)blk.q_row0, (long long)blk.n_q, (long long)blk.k_row0, (long long)blk.n_k, blk.mask);
  mmsp_2d_share sh;
  if (p_mmsp_2d_layout(262144, 4, 8, 13, 28, 4, &sh) != MMSP_OK) return 1;
  printf("2d %d %d %d %d %d %d %lld\n", sh.head_rank, sh.ring_rank, sh.q_head0, sh.n_q_heads, sh.kv_head0, sh.n_kv_heads, (long long)sh.chunk_len);
  mmsp_shape shape;
  memset(&shape, 0, sizeof shape);
  shape.n_q_heads = 28; shape.n_kv_heads = 4; shape.head_dim = 128; shape.io_dtype = MMSP_BF16; shape.softmax_scale = 0.0883883f;
  shape.q_tok_stride = 28 * 128; shape.q_head_stride = 128; shape.kv_tok_stride = 4 * 128; shape.kv_head_stride = 128; shape.lse_head_stride = 8192;
  printf("ws %zu\n", p_mmsp_workspace_bytes(&shape, 8192, 8192, 1));
  mmsp_status st = p_mmsp_zigzag_layout(10, 4, 0, ids, l2g);
  printf("bad %d %s\n", (int)st, strlen(p_mmsp_last_error()) > 0 ? "message" : "empty");
  return 0;
}
