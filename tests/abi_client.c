/* A plain C client of the library's C ABI, built and run by tests/test_abi.py on a machine without a GPU:
 * it only calls entry points that do host work or that return before any launch. */
#include <stdio.h>
#include <string.h>

#include "la2.h"

int main(void) {
  la2_desc d;
  la2_desc_dense(&d, 2, 3, 100, 64, LA2_BF16);
  if (d.stride_n != 64 || d.stride_h != 6400 || d.stride_b != 19200) return 1;
  if (la2_block_size(&d) != 32) return 2;
  if (la2_fwd(&d, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) != LA2_ERR_NULL) return 3;
  d.head_dim = 100;
  if (la2_fwd(&d, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) != LA2_ERR_SHAPE) return 4;
  la2_desc_dense(&d, 0, 3, 100, 64, LA2_F16);
  if (la2_bwd(&d, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) != LA2_OK) return 5;
  if (la2_fwd_norm(&d, NULL, NULL, NULL, NULL, -1.0f, NULL, NULL, NULL, 0, NULL) != LA2_ERR_VALUE) return 6;
  if (strcmp(la2_status_string(LA2_OK), "ok") != 0) return 7;
  la2_set_chunk_tokens(256);
  la2_desc_dense(&d, 1, 2, 1024, 128, LA2_BF16);
  if (la2_workspace_bytes(&d, LA2_OP_FWD) != (size_t)2 * 4 * 128 * 128 * 4) return 8;
  la2_set_chunk_tokens(0);
  /* packed batches: a negative total, a missing offset array; states over packed batches take the 16-bit types */
  la2_desc_dense(&d, 4, 2, 300, 128, LA2_BF16);
  d.stride_b = 0; d.stride_h = 128; d.stride_n = 256;
  if (la2_fwd_varlen(&d, NULL, -1, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) != LA2_ERR_SHAPE) return 9;
  if (la2_fwd_varlen_state(&d, NULL, 0, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) != LA2_ERR_NULL) return 10;
  d.dtype = LA2_F32;
  {
    float state[4];
    if (la2_fwd_varlen_state(&d, NULL, 0, NULL, NULL, NULL, NULL, state, NULL, NULL, NULL, 0, NULL) != LA2_ERR_DTYPE) return 11;
    if (la2_bwd_varlen_state(&d, NULL, 0, NULL, NULL, NULL, NULL, NULL, NULL, state, NULL, NULL, NULL, NULL, NULL, 0, NULL) !=
        LA2_ERR_DTYPE)
      return 12;
  }
  if (la2_varlen_workspace_bytes(&d, 0, LA2_OP_FWD) != la2_workspace_bytes(&d, LA2_OP_FWD)) return 13;
  printf("abi client ok\n");
  return 0;
}
