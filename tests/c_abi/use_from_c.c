/* A plain C99 caller of the library: checks that include/magicpig.h is valid C, that the entry
 * points link by their C names, and that argument validation needs no GPU.  Built and run by
 * tests/test_host_logic.py. */
#include "magicpig.h"
#include <stdio.h>
int main(void) {
  magicpig_params p = {0};
  p.batch = 1; p.n_q_heads = 32; p.n_kv_heads = 8; p.head_dim = 128; p.K = 10; p.L = 150; p.min_hits = 2;
  p.n_sink = 4; p.n_local = 64; p.dtype = MAGICPIG_BF16; p.n_ctx = 1000; p.n_cap = 1000;
  p.k_stride_b = p.v_stride_b = 8 * 1000 * 128; p.k_stride_h = p.v_stride_h = 1000 * 128; p.k_stride_n = p.v_stride_n = 128;
  printf("%zu %zu %s\n", magicpig_code_words_per_key(&p), magicpig_workspace_bytes(&p), magicpig_status_string(MAGICPIG_UNSUPPORTED));
  return magicpig_hash_query(&p, 0, 0, 0, 0, 0, 0) == MAGICPIG_INVALID_ARG ? 0 : 1;
}
