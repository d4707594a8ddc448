/* Host-side exercise of the C ABI for the sanitizer build (tests/test_host_sanitizers.py links this
 * file with the library's objects compiled with AddressSanitizer and UBSan on the host side).  It makes
 * only calls that the argument validation must turn down, plus the size queries: nothing here reaches a
 * kernel launch, so it needs no GPU and never hands a made-up pointer to one. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../include/dlayer.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)
#define EXPECT_INVALID(call)                                                \
  do {                                                                      \
    int rc_ = (call);                                                       \
    if (rc_ != DLAYER_ERR_INVALID || strlen(dlayer_last_error()) == 0) {    \
      printf("FAILED line %d: %s returned %d (%s)\n", __LINE__, #call, rc_, dlayer_last_error()); \
      ++failures;                                                           \
    }                                                                       \
  } while (0)

int main(void) {
  static char arena[4096] __attribute__((aligned(256)));
  void* ok = arena;            /* aligned, never dereferenced: every call below is rejected first */
  void* odd = arena + 2;       /* misaligned */
  dlayer_cfg good = {2, 8192, 4096, 32, 8, 128, 14336, 1e-5f, 500000.0f, 0};
  dlayer_cfg bad = good;
  EXPECT(dlayer_version() == 1);
  EXPECT(dlayer_saved_bytes(&good) > 0 && dlayer_workspace_bytes(&good) > 0);
  EXPECT(dlayer_saved_bytes(NULL) == 0);
  bad.head_dim = 96;  EXPECT(dlayer_saved_bytes(&bad) == 0 && dlayer_workspace_bytes(&bad) == 0);
  bad = good; bad.seq = 100;  EXPECT(dlayer_saved_bytes(&bad) == 0);
  bad = good; bad.n_kv_heads = 5;  EXPECT(dlayer_saved_bytes(&bad) == 0);
  bad = good; bad.batch = 1; bad.seq = 128; bad.d_model = 16384; bad.d_ff = 131072; bad.n_q_heads = 8; bad.n_kv_heads = 8;
  EXPECT(dlayer_saved_bytes(&bad) == 0);   /* a weight tensor of 4 GiB */
  bad = good; bad.batch = 1 << 20;  EXPECT(dlayer_workspace_bytes(&bad) == 0);   /* activations past 4 GiB */

  dlayer_weights w = {ok, ok, ok, ok, ok, ok, ok, ok, ok};
  dlayer_wgrads dw = {ok, ok, ok, ok, ok, ok, ok, ok, ok};
  bad = good; bad.head_dim = 48;
  EXPECT_INVALID(dlayer_forward(&bad, ok, &w, arena + 256, ok, ok, NULL));
  EXPECT_INVALID(dlayer_forward(&good, NULL, &w, ok, ok, ok, NULL));
  EXPECT_INVALID(dlayer_forward(&good, ok, &w, ok, ok, ok, NULL));            /* x == y */
  EXPECT_INVALID(dlayer_forward(&good, odd, &w, ok, ok, ok, NULL));
  EXPECT_INVALID(dlayer_forward(&good, ok, NULL, arena + 256, ok, ok, NULL));
  w.wq = NULL;
  EXPECT_INVALID(dlayer_forward(&good, ok, &w, arena + 256, ok, ok, NULL));
  w.wq = ok;
  EXPECT_INVALID(dlayer_backward(&good, ok, &w, ok, ok, ok, &dw, 64, ok, NULL));   /* unknown flag */
  EXPECT_INVALID(dlayer_backward(&good, ok, &w, ok, ok, ok, NULL, 0, ok, NULL));
  dw.w_down = odd;
  EXPECT_INVALID(dlayer_backward(&good, ok, &w, ok, ok, ok, &dw, 0, ok, NULL));

  float loss = 0.f;
  int64_t tg[4] = {0, 1, 2, 3};
  EXPECT(ce_loss_workspace_bytes(8192, 128256) == 8192 * 4 && ce_loss_workspace_bytes(0, 8) == 0);
  EXPECT_INVALID(ce_loss_fwd_bwd(ok, tg, 4, 12, 1.f, &loss, ok, ok, NULL));       /* V % 8 */
  EXPECT_INVALID(ce_loss_fwd_bwd(ok, NULL, 4, 16, 1.f, &loss, ok, ok, NULL));
  EXPECT_INVALID(ce_loss_fwd_bwd_static(ok, tg, CE_LOSS_STATIC_MAX_ROWS + 1, 16, 1.f, &loss, ok, NULL));
  EXPECT(lm_head_ce_workspace_bytes(8192, 4096, 128256, 100) == 0);
  EXPECT_INVALID(lm_head_ce_fwd_bwd(ok, ok, tg, 100, 4096, 128256, 1.f, 0, &loss, ok, ok, 0, ok, NULL));
  EXPECT_INVALID(rmsnorm_forward(ok, ok, 16, 20, 1e-5f, ok, &loss, NULL));
  EXPECT_INVALID(rmsnorm_backward(ok, ok, &loss, ok, odd, 16, 64, ok, ok, 0, ok, NULL));
  EXPECT_INVALID(linear_forward(ok, ok, NULL, 128, 100, 128, ok, NULL));
  EXPECT_INVALID(linear_forward(ok, ok, NULL, 1 << 20, 4096, 128, ok, NULL));     /* operand past 4 GiB */
  EXPECT_INVALID(qkv_rope_forward(ok, ok, ok, ok, 1, 128, 128, 4, 4, 40, 1e4f, 0, ok, ok, ok, ok, NULL));
  EXPECT(qkv_rope_workspace_bytes(128, 40) == 0 && qkv_rope_workspace_bytes(8192, 128) >= 2u * 8192 * 64 * 4);
  EXPECT_INVALID(linear_swiglu_forward(ok, ok, ok, 128, 64, 12, ok, ok, ok, NULL));
  EXPECT_INVALID(linear_swiglu_backward(ok, ok, ok, ok, 100, 64, 64, ok, ok, ok, NULL));
  EXPECT_INVALID(linear_backward(ok, ok, ok, 128, 64, 100, ok, ok, 0, ok, NULL));
  {
    const void* ps[9] = {ok, ok, ok, ok, ok, ok, ok, ok, ok};
    void* outs[9] = {ok, ok, ok, ok, ok, ok, ok, ok, ok};
    int64_t n[9] = {64, 64, 64, 64, 64, 64, 64, 64, 64}, k[9] = {64, 64, 64, 64, 64, 64, 64, 64, 100};
    EXPECT_INVALID(linear_wgrad_group(9, ps, ps, n, k, 128, outs, 0, NULL));       /* more than 8 products */
    EXPECT_INVALID(linear_wgrad_group(0, ps, ps, n, k, 128, outs, 0, NULL));
    EXPECT_INVALID(linear_wgrad_group(2, ps, ps, n, k + 7, 128, outs, 0, NULL));   /* K[1] = 100 */
  }
  EXPECT_INVALID(rope_apply(ok, 1, 128, 4, 32, 1e4f, 3, 0, NULL));
  EXPECT_INVALID(attention_forward(ok, ok, ok, 1, 128, 3, 2, 32, ok, &loss, NULL));
  EXPECT_INVALID(attention_backward(ok, ok, ok, ok, ok, &loss, 1, 64, 2, 2, 32, ok, ok, ok, ok, NULL));
  EXPECT(attention_backward_workspace_bytes(0, 128, 4, 4, 32) == 0);
  EXPECT_INVALID(swiglu_forward(ok, ok, 12, ok, NULL));
  EXPECT_INVALID(swiglu_backward(ok, ok, ok, 0, ok, ok, NULL));
  EXPECT_INVALID(embed_forward(ok, NULL, 4, 16, 64, ok, NULL));
  EXPECT_INVALID(embed_backward(ok, tg, 4, 16, 60, ok, ok, NULL));
  EXPECT(embed_backward_workspace_bytes(8192, 128256) >= (3u * 128256 + 2u * 8192) * 4);
  {
    const void* gs[17]; void* prm[17]; float* mom[17]; int64_t ne[17];
    for (int i = 0; i < 17; ++i) { gs[i] = ok; prm[i] = ok; mom[i] = (float*)ok; ne[i] = 64; }
    EXPECT(grad_sq_norm_workspace_bytes(17, ne) == 0 && grad_sq_norm_workspace_bytes(3, ne) > 0);
    EXPECT_INVALID(grad_sq_norm(17, gs, ne, &loss, 0, ok, NULL));
    ne[1] = 12;
    EXPECT_INVALID(grad_sq_norm(2, gs, ne, &loss, 0, ok, NULL));
    ne[1] = 64;
    EXPECT_INVALID(adamw_step(2, prm, gs, mom, mom, ne, 0, 1e-3f, 0.9f, 0.95f, 1e-8f, 0.f, 1.f, NULL, NULL));
    EXPECT_INVALID(adamw_step(2, prm, gs, mom, mom, ne, 1, 1e-3f, 1.0f, 0.95f, 1e-8f, 0.f, 1.f, NULL, NULL));
    gs[1] = odd;
    EXPECT_INVALID(adamw_step(2, prm, gs, mom, mom, ne, 1, 1e-3f, 0.9f, 0.95f, 1e-8f, 0.f, 1.f, NULL, NULL));
  }
  printf(failures ? "sanitize driver: %d FAILED\n" : "sanitize driver: all calls rejected as expected (%d failures)\n", failures);
  return failures ? 1 : 0;
}
