/* Plain C caller of the library's host-side entry points (no GPU work): shows that the boundary is
 * usable without C++ or Python.  Built and run by tests/test_abi_host.py. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "speckv.h"

int main(void) {
  speckv_params p;
  memset(&p, 0, sizeof(p));
  p.n_seqs = 1; p.n_layers = 32; p.n_q_heads = 32; p.n_kv_heads = 8; p.head_dim = 128;
  p.n_window = 64; p.n_lookahead = 64; p.pool_k = 7; p.c_max = 2048;
  p.sm_scale = 0.08838834764831845f; p.dtype = SPECKV_BF16; p.cu_seqlens = NULL; p.n_in = 131072;
  p.q_stride_head = 128; p.q_stride_row = 32 * 128; p.q_stride_seq = 128 * 32 * 128; p.q_stride_layer = p.q_stride_seq;
  p.kv_stride_head = 128; p.kv_stride_token = 8 * 128; p.kv_stride_layer = p.n_in * p.kv_stride_token;
  p.reduce_op = SPECKV_REDUCE_SUM; p.pool_op = SPECKV_POOL_MAX;

  int64_t info[SPECKV_PLAN_INFO_WORDS];
  if (speckv_plan_info(&p, info) != SPECKV_OK) return 1;
  if (speckv_n_keep(&p, 0) != 2048 + 64 || speckv_total_keep(&p) != 2112) return 2;
  if (speckv_workspace_bytes(&p) == 0) return 3;
  p.head_dim = 96;                                   /* unsupported head dimension */
  if (speckv_plan_info(&p, info) != SPECKV_ERR_UNSUPPORTED) return 4;
  if (speckv_workspace_bytes(&p) != 0) return 5;
  p.head_dim = 128; p.pool_k = 0;                    /* no pooling kernel */
  if (speckv_compress(&p, (void *)256, (void *)256, (void *)256, (int32_t *)256, (void *)256, (void *)256,
                      (void *)256, (size_t)1 << 40, NULL) != SPECKV_ERR_INVALID_ARG) return 6;
  printf("%s\n", speckv_status_string(SPECKV_ERR_WORKSPACE));
  return 0;
}
