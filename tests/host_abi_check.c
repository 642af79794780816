/* Host-only walk through the C ABI of include/bsr.h, for the sanitizer leg (tests/test_sanitizers.py links it
 * against the library's objects built with AddressSanitizer + UndefinedBehaviorSanitizer in their host code).
 * It calls what needs no GPU: the token schedule (Sec. 4.1, Sec. 4.3), workspace size, saved-activation report
 * (Table 1), configuration checks, NULL-argument and no-context error paths, the tile-shape list.  Exit status 0
 * when every check holds; a sanitizer report ends the program with its own status. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "bsr.h"

static int failures = 0;
#define CHECK(c) do { if (!(c)) { printf("FAILED line %d: %s\n", __LINE__, #c); failures++; } } while (0)

static bsr_config vit_b(float keep, int first_trainable, int max_batch) {
  bsr_config c;
  memset(&c, 0, sizeof c);
  c.image_size = 224; c.patch_size = 16; c.in_chans = 3;
  c.dim = 768; c.heads = 12; c.mlp_hidden = 3072; c.depth = 12; c.num_classes = 100;
  c.max_batch = max_batch;
  c.n_drop = 3; c.drop_blocks[0] = 3; c.drop_blocks[1] = 6; c.drop_blocks[2] = 9;
  c.keep_ratio = keep;
  c.first_trainable_block = first_trainable;
  c.dtype = BSR_BF16; c.loss = BSR_LOSS_CE;
  return c;
}

int main(void) {
  /* token schedule: N/2, N/4, N/8 at drop rate 0.5 */
  int32_t kk[BSR_MAX_BLOCKS], ta[BSR_MAX_BLOCKS], tm[BSR_MAX_BLOCKS];
  bsr_config c = vit_b(0.5f, 8, 32);
  CHECK(bsr_token_schedule(&c, kk, ta, tm) == BSR_OK);
  CHECK(kk[0] == 98 && kk[1] == 49 && kk[2] == 24);
  CHECK(ta[0] == 197 && tm[3] == 99 && ta[4] == 99 && tm[11] == 25);
  c = vit_b(0.7f, 8, 32);
  CHECK(bsr_token_schedule(&c, kk, NULL, NULL) == BSR_OK && kk[0] == 137 && kk[1] == 95 && kk[2] == 66);
  CHECK(bsr_token_schedule(NULL, kk, ta, tm) == BSR_ERR_INVALID_ARG);
  c.fuse_dropped = 1;
  CHECK(bsr_token_schedule(&c, kk, ta, tm) == BSR_OK && tm[3] == kk[0] + 2);

  /* workspace size grows with batch and with the number of blocks that keep activations */
  size_t a = 0, b = 0, d = 0;
  c = vit_b(0.7f, 8, 32);  CHECK(bsr_workspace_bytes(&c, &a) == BSR_OK);
  c = vit_b(0.7f, 8, 64);  CHECK(bsr_workspace_bytes(&c, &b) == BSR_OK);
  c = vit_b(0.7f, 0, 32);  CHECK(bsr_workspace_bytes(&c, &d) == BSR_OK);
  CHECK(a > 0 && a < b && a < d);
  CHECK(bsr_workspace_bytes(&c, NULL) == BSR_ERR_INVALID_ARG);
  CHECK(bsr_workspace_bytes(NULL, &a) == BSR_ERR_INVALID_ARG);

  /* saved activations: frozen blocks keep nothing, the sum is the sum */
  bsr_saved_bytes per[BSR_MAX_BLOCKS], sum;
  c = vit_b(0.7f, 8, 32);
  CHECK(bsr_saved_activation_bytes(&c, 32, per, &sum) == BSR_OK);
  uint64_t tot = 0;
  for (int l = 0; l < 12; l++) {
    CHECK((l < 8) == (per[l].total == 0));
    CHECK(per[l].total == per[l].qkv + per[l].softmax + per[l].attn_out + per[l].gelu_in + per[l].linear_in +
                              per[l].residual + per[l].stats + per[l].moe);
    tot += per[l].total;
  }
  CHECK(tot == sum.total && tot > 0);
  CHECK(bsr_saved_activation_bytes(&c, 33, per, &sum) == BSR_ERR_INVALID_ARG);
  CHECK(bsr_saved_activation_bytes(&c, 0, per, &sum) == BSR_ERR_INVALID_ARG);
  CHECK(bsr_saved_activation_bytes(&c, 8, NULL, NULL) == BSR_OK);

  /* configurations that must be refused, each with a message */
  for (int k = 0; k < 14; k++) {
    c = vit_b(0.7f, 8, 8);
    switch (k) {
      case 0: c.dim = 770; break;
      case 1: c.heads = 5; break;
      case 2: c.depth = BSR_MAX_BLOCKS + 1; break;
      case 3: c.drop_blocks[0] = 6; c.drop_blocks[1] = 3; break;
      case 4: c.drop_blocks[2] = 12; break;
      case 5: c.keep_ratio = 0.0f; break;
      case 6: c.keep_ratio = 1.5f; break;
      case 7: c.first_trainable_block = 13; break;
      case 8: c.num_classes = 0; break;
      case 9: c.image_size = 225; break;
      case 10: c.keep_k[0] = 300; c.keep_k[1] = 10; c.keep_k[2] = 5; break;
      case 11: c.max_batch = 0; break;
      case 12: c.n_drop = BSR_MAX_BLOCKS + 1; break;
      case 13: c.n_experts = 33; c.n_moe = 1; c.moe_blocks[0] = 9; c.moe_top_k = 2; break;
    }
    size_t w = 0;
    int32_t rc = bsr_workspace_bytes(&c, &w);
    CHECK(rc != BSR_OK);
    CHECK(strlen(bsr_last_error(NULL)) > 10);
    if (rc == BSR_OK) printf("  case %d was accepted\n", k);
  }
  /* lists longer than the struct holds must be refused before they are walked */
  c = vit_b(0.7f, 8, 8);
  c.n_trainable = BSR_MAX_BLOCKS + 3;
  CHECK(bsr_token_schedule(&c, kk, ta, tm) != BSR_OK);
  c = vit_b(0.7f, 8, 8);
  c.n_moe = BSR_MAX_BLOCKS + 3; c.n_experts = 4; c.moe_top_k = 2;
  CHECK(bsr_token_schedule(&c, kk, ta, tm) != BSR_OK);
  c = vit_b(0.7f, 8, 8);
  c.n_drop = -1;
  CHECK(bsr_token_schedule(&c, kk, ta, tm) != BSR_OK);

  /* calls without a context fail with a status, never by touching memory */
  CHECK(bsr_tile_choices(NULL, 0, NULL, 0) == 0);
  CHECK(bsr_refresh_weights(NULL, NULL) == BSR_ERR_INVALID_ARG);
  CHECK(bsr_profile_begin(NULL) == BSR_ERR_INVALID_ARG);
  CHECK(bsr_destroy(NULL) == BSR_OK || bsr_destroy(NULL) == BSR_ERR_INVALID_ARG);
  CHECK(bsr_last_error(NULL) != NULL);
  bsr_ctx* ctx = NULL;
  bsr_params p;
  memset(&p, 0, sizeof p);
  c = vit_b(0.7f, 8, 8);
  CHECK(bsr_init(&c, &p, NULL, 0, NULL, &ctx) != BSR_OK && ctx == NULL);   /* no workspace */
  CHECK(bsr_init(&c, NULL, NULL, 0, NULL, &ctx) == BSR_ERR_INVALID_ARG);
  CHECK(bsr_init(&c, &p, NULL, 0, NULL, NULL) == BSR_ERR_INVALID_ARG);

  /* the tile-shape list: count first, then a short and a full read */
  int32_t n = bsr_gemm_tile_shapes(NULL, 0);
  CHECK(n > 8 && n < 64);
  int32_t ids[64];
  memset(ids, 0, sizeof ids);
  CHECK(bsr_gemm_tile_shapes(ids, 3) == n && ids[2] != 0 && ids[3] == 0);
  CHECK(bsr_gemm_tile_shapes(ids, 64) == n && ids[n - 1] != 0 && ids[n] == 0);

  printf(failures ? "host_abi_check: %d checks failed\n" : "host_abi_check: all checks passed\n", failures);
  return failures ? 1 : 0;
}
