/* Plain C99 client of libmixkv: includes the public header, fills the params struct and calls the
 * entry points that touch no GPU.  Built and run by tests/test_abi.py; prints one line per check. */
#include <stdio.h>
#include <string.h>
#include "mixkv.h"

int main(void) {
  mixkv_params p;
  size_t one = 0, two = 0, sim = 0;
  int32_t budgets[8] = {64, 64, 64, 64, 32, 96, 64, 64};
  memset(&p, 0, sizeof p);
  p.dtype = MIXKV_BF16; p.batch = 1; p.n_q_heads = 28; p.n_kv_heads = 4; p.head_dim = 128;
  p.seq_len = 8192; p.window = 32; p.budget = 64; p.pool = MIXKV_POOL_MAX; p.pool_kernel = 7;
  p.causal_window = 1; p.softmax_scale = 1.0f; p.eps = 1e-6f; p.intrinsic = MIXKV_INTRINSIC_VNORM;
  p.mix = MIXKV_MIX_HEAD_ADAPTIVE; p.budget_mode = MIXKV_BUDGET_FIXED; p.budget_floor = 0; p.head_budgets = NULL;
  if (mixkv_version() != MIXKV_VERSION) { printf("version mismatch\n"); return 1; }
  if (mixkv_workspace_size(&p, 1, &one) != MIXKV_OK || mixkv_workspace_size(&p, 2, &two) != MIXKV_OK) return 2;
  if (!(one > 0 && two > one)) return 3;
  p.budget_mode = MIXKV_BUDGET_PER_HEAD; p.head_budgets = budgets;
  if (mixkv_workspace_size(&p, 2, &two) != MIXKV_OK) return 4;
  if (mixkv_similarity_workspace_size(&p, 2, 64, &sim) != MIXKV_OK || sim == 0) return 5;
  p.head_dim = 96;
  if (mixkv_workspace_size(&p, 1, &one) != MIXKV_ERR_UNSUPPORTED) return 6;
  /* NULL arguments are rejected before anything touches a GPU */
  p.head_dim = 128;
  if (mixkv_compress(&p, NULL, NULL, 1, NULL, 0, NULL) != MIXKV_ERR_INVALID_ARG) return 7;
  if (mixkv_decode_attention(&p, NULL, 1, 0, 0, NULL, 0, NULL) != MIXKV_ERR_INVALID_ARG) return 8;
  if (mixkv_decode_workspace_size(&p, 1, 0, &sim) != MIXKV_OK || sim != 0) return 10;      /* 64 rows: no split */
  p.budget = 2048;
  if (mixkv_decode_workspace_size(&p, 1, 16, &sim) != MIXKV_OK || sim == 0) return 11;
  p.budget = 64;
  if (mixkv_similarity(&p, NULL, NULL, 1, 64, NULL, 0, NULL) != MIXKV_ERR_INVALID_ARG) return 9;
  printf("ok %s %zu %zu\n", mixkv_status_string(MIXKV_OK), one, sim);
  return 0;
}
