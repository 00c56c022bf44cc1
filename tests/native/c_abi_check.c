/* The public header must be plain C and the library must link and run without a GPU for everything that
 * touches no device: logical contexts (allocator, block tables, slot mapping) and the host-side policy. */
#include <stdio.h>
#include <string.h>

#include "lkv.h"

#define CHECK(x)                                                      \
  do {                                                                \
    if (!(x)) {                                                       \
      fprintf(stderr, "c_abi_check: %s failed (line %d)\n", #x, __LINE__); \
      return 1;                                                       \
    }                                                                 \
  } while (0)

int main(void) {
  lkv_config cfg;
  lkv_ctx *c = NULL;
  int32_t table[8], res = -1, mask[8], x = -1;
  int64_t slots[20], n = 0;
  lkv_cost_model cm;
  memset(&cfg, 0, sizeof cfg);
  cfg.num_layers = 8;
  cfg.num_q_heads = 4;
  cfg.num_kv_heads = 2;
  cfg.head_dim = 128;
  cfg.block_size = 16;
  cfg.dtype = LKV_BF16;
  cfg.num_pool_blocks = 32;
  CHECK(lkv_create_logical(&cfg, &c) == LKV_OK && c != NULL);
  CHECK(lkv_num_free_blocks(c) == 32);
  CHECK(lkv_alloc_layer_blocks(c, 7, 3, 40) == LKV_OK);                 /* 40 tokens: 3 blocks */
  CHECK(lkv_num_free_blocks(c) == 29);
  CHECK(lkv_get_block_table(c, 7, 3, table, 8, &n) == LKV_OK && n == 3);
  CHECK(table[0] == 0 && table[1] == 1 && table[2] == 2);               /* ascending ids first */
  CHECK(lkv_build_slot_mapping(c, 7, 3, 15, 3, slots) == LKV_OK);       /* tokens 15, 16, 17 */
  CHECK(slots[0] == 15 && slots[1] == 16 && slots[2] == 17);
  CHECK(lkv_layer_residency(c, 7, 3, &res) == LKV_OK && res == LKV_RES_GPU);
  CHECK(lkv_alloc_layer_blocks(c, 7, 4, 16 * 40) == LKV_ERR_NO_BLOCKS); /* 40 blocks do not fit */
  CHECK(lkv_num_free_blocks(c) == 29);
  CHECK(lkv_write_kv(c, 3, NULL, NULL, NULL, 0, NULL) == LKV_ERR_DEVICE); /* no device behind this context */
  CHECK(lkv_reserve_decode_workspace(c, 4, 64) == LKV_ERR_DEVICE);
  CHECK(lkv_paged_decode_attention_static(c, 3, NULL, NULL, NULL, 0, NULL, 0, NULL) == LKV_ERR_DEVICE);
  CHECK(LKV_RES_IN_FLIGHT == 3);                                        /* never reported without a device */
  CHECK(strlen(lkv_last_error(c)) > 0);
  CHECK(lkv_free_layer_blocks(c, 7, 3, 1) == LKV_OK);
  CHECK(lkv_layer_residency(c, 7, 3, &res) == LKV_OK && res == LKV_RES_HOST);
  CHECK(lkv_num_free_blocks(c) == 32);
  lkv_destroy(c);

  /* Section 3.2.2: with 8 layers and 4 retained, layers 1, 3, 5, 7 stay */
  CHECK(lkv_plan_retained_layers(8, 4, mask) == LKV_OK);
  CHECK(!mask[0] && mask[1] && !mask[2] && mask[3] && !mask[4] && mask[5] && !mask[6] && mask[7]);

  /* Section 3.2.1: a link ten times too slow for the prefill keeps nine tenths of the layers */
  memset(&cm, 0, sizeof cm);
  cm.alpha = 1.0;
  cm.n_param = 1e9;
  cm.n_hidden = 0.0;
  cm.device_flops = 1e12;           /* prefill of s tokens: 2e9 s / 1e12 = 2 ms per token */
  cm.beta = 1.0;
  cm.num_layers = 10;
  cm.head_dim = 100;
  cm.num_heads = 10;
  cm.bytes_per_elem = 1.0;
  cm.link_bytes_per_s = 1e5;        /* one layer of one token: 2*100*10 bytes / 1e5 = 20 ms */
  CHECK(lkv_plan_offload(&cm, 1000, &x, NULL) == LKV_OK);
  CHECK(x == 10);                   /* not even one layer (20 ms/token) fits behind 2 ms/token */
  cm.link_bytes_per_s = 1e7;        /* 0.2 ms per layer and token: all ten layers fit exactly */
  CHECK(lkv_plan_offload(&cm, 1000, &x, NULL) == LKV_OK && x == 0);
  puts("c_abi_check: ok");
  return 0;
}
