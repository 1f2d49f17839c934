// Host-side sanitizer run of libbct's argument validation and launch planning: no call reaches the GPU.
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include "bct.h"
#include "bct_model.h"
int main() {
  int bad = 0;
  bct_cache_desc d;
  memset(&d, 0, sizeof d);
  d.capacity_M = 4096; d.batch = 32; d.n_q_heads = 32; d.n_kv_heads = 32; d.head_dim = 128; d.dtype = BCT_BF16;
  d.read_scale = 0.088f; d.write_scale = 0.088f;
  size_t cb = 0, wb = 0;
  bad |= bct_cache_query(&d, 512, &cb, &wb) != BCT_OK;
  bad |= cb == 0 || wb == 0;
  bct_plan_info pi;
  bad |= bct_plan_query(&d, &pi) != BCT_OK;
  bad |= bct_cache_query(NULL, 0, &cb, &wb) != BCT_ERR_INVALID_ARG;
  d.head_dim = 96;
  bad |= bct_cache_query(&d, 0, &cb, &wb) != BCT_ERR_UNSUPPORTED;
  d.head_dim = 128; d.capacity_M = 100;
  bad |= bct_cache_query(&d, 0, &cb, &wb) != BCT_ERR_UNSUPPORTED;
  d.capacity_M = 64;
  bct_cache* c = NULL;
  bad |= bct_cache_init(&d, 0, NULL, 0, NULL, 0, NULL, &c) == BCT_OK;
  bad |= bct_decode_step(NULL, NULL, NULL, NULL, NULL, NULL) == BCT_OK;
  bad |= bct_prefill(NULL, NULL, NULL, NULL, 4, NULL, NULL) == BCT_OK;
  bad |= bct_decode_step_static(NULL, NULL, NULL, NULL, NULL, NULL) != BCT_ERR_INVALID_ARG;
  bad |= bct_decode_step_keyed(NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) != BCT_ERR_INVALID_ARG;
  bad |= bct_static_scratch_bytes() != ((size_t)8 << 20);
  bad |= bct_cache_steps(NULL, NULL) == BCT_OK;
  bct_cache_destroy(NULL);
  bad |= strlen(bct_strerror(BCT_ERR_MISALIGNED)) == 0;
  bad |= strlen(bct_last_error()) == 0;
  uint32_t k = 99;
  bad |= bctm_linear_plan(16384, 4096, 12288, 0, &k) != BCT_OK || k != BCTM_KERNEL_TILE256;
  bad |= bctm_linear_plan(32, 4096, 12288, 0, &k) != BCT_OK || k != BCTM_KERNEL_STREAMING_TRIPLE;
  bad |= bctm_linear_plan(32, 4096, 4096, 0, &k) != BCT_OK || k != BCTM_KERNEL_STREAMING;
  bad |= bctm_linear((void*)0x10000, (void*)0x20000, NULL, (void*)0x30000, 4, 72, 32, 0, NULL) != BCT_ERR_UNSUPPORTED;
  bad |= bctm_rmsnorm((void*)0x10000, (void*)0x20000, (void*)0x30000, 4, 12, 1e-5f, 0, NULL) != BCT_ERR_UNSUPPORTED;
  bad |= strlen(bctm_last_error()) == 0;
  printf(bad ? "host sanitizer drive: FAILED\n" : "host sanitizer drive: ok\n");
  return bad;
}
