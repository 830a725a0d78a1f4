// Host-only walk through the C ABI for a build whose host code is instrumented with AddressSanitizer and
// UndefinedBehaviorSanitizer (tests/test_host_sanitizers.py): sizes, layouts and network plans of every model,
// rejected configurations, rejected arguments.  Nothing here reaches the GPU.
#include <stdio.h>
#include <string.h>

#include "../include/parle.h"

static int failures = 0;
#define EXPECT(cond)                                      \
  do {                                                    \
    if (!(cond)) {                                        \
      printf("FAILED line %d: %s\n", __LINE__, #cond);    \
      ++failures;                                         \
    }                                                     \
  } while (0)

static parle_config base(int model) {
  parle_config c;
  memset(&c, 0, sizeof(c));
  c.model = model, c.n_replicas = 3, c.batch = 128, c.L = 25;
  c.eta_inner = c.eta_outer = 0.1f, c.momentum = 0.9f, c.alpha = 0.75f;
  c.gamma0 = 0.03f, c.rho0 = 1.f, c.gamma_max = 1.f, c.rho_max = 10.f, c.reset_flags = 3;
  return c;
}

int main() {
  long long checksum = 0;
  for (int model = 0; model <= 4; ++model)
    for (int variant = 0; variant < 4; ++variant) {
      parle_config c = base(model);
      if (model == 0) c.n_params = variant == 0 ? 1 : 36500000LL + variant;
      if (variant == 1) c.compute_bf16 = 1;
      if (variant == 2) {  // odd sizes: scalar paths, ragged tiles
        c.in_h = 12, c.in_w = 10, c.in_c = 3, c.n_classes = 5, c.batch = 7, c.n_replicas = 2;
        c.arch[0] = 5, c.arch[1] = 7, c.arch[2] = model == 2 ? 3 : 1, c.arch[3] = 9;
        c.dropout = 0.3f, c.lenet_bn = model == 2;
      }
      if (variant == 3 && model == 4) c.arch[0] = 16, c.arch[1] = 10, c.arch[2] = 4, c.compute_bf16 = 1;  // WRN-28-10
      parle_sizes s;
      const parle_status st = parle_query_sizes(&c, &s);
      EXPECT(st == PARLE_OK);
      if (st != PARLE_OK) {
        printf("model %d variant %d: %s\n", model, variant, parle_last_error(NULL));
        continue;
      }
      EXPECT(s.n_pad % 1024 == 0 && s.n_pad >= s.n_params && s.workspace_bytes > 0);
      for (int i = 0; i < s.n_segments; ++i) {
        parle_segment seg;
        EXPECT(parle_query_layout(&c, i, &seg) == PARLE_OK);
        EXPECT(seg.offset + seg.size <= s.n_params && seg.size > 0);
        checksum += seg.offset ^ seg.size;
      }
      parle_segment seg;
      EXPECT(parle_query_layout(&c, s.n_segments, &seg) != PARLE_OK);
      EXPECT(parle_query_layout(&c, -1, &seg) != PARLE_OK);
      checksum += s.n_params + s.workspace_bytes + s.bn_bytes;
    }
  // rejected configurations
  {
    parle_sizes s;
    parle_config c = base(1);
    c.n_replicas = 0;
    EXPECT(parle_query_sizes(&c, &s) == PARLE_EINVAL);
    c = base(1), c.alpha = 2.f;
    EXPECT(parle_query_sizes(&c, &s) == PARLE_EINVAL);
    c = base(0), c.n_params = 1LL << 36, c.n_replicas = 65535;
    EXPECT(parle_query_sizes(&c, &s) == PARLE_ESIZE);
    c = base(7);
    EXPECT(parle_query_sizes(&c, &s) == PARLE_EINVAL);
    c = base(2), c.in_h = 4, c.in_w = 4, c.in_c = 1;   // smaller than the 5x5 filter
    EXPECT(parle_query_sizes(&c, &s) != PARLE_OK);
    EXPECT(parle_query_sizes(NULL, &s) == PARLE_EINVAL && parle_query_sizes(&c, NULL) == PARLE_EINVAL);
    EXPECT(strlen(parle_last_error(NULL)) > 0);
  }
  // rejected arguments of the calls that would reach the device
  {
    parle_config c = base(0);
    c.n_params = 100;
    parle_ctx *ctx = NULL;
    parle_buffers b;
    memset(&b, 0, sizeof(b));
    EXPECT(parle_init(&c, &b, NULL, &ctx) == PARLE_EINVAL && ctx == NULL);
    EXPECT(parle_init(&c, NULL, NULL, &ctx) == PARLE_EINVAL);
    EXPECT(parle_inner_step(NULL, NULL, NULL, NULL) == PARLE_EINVAL);
    EXPECT(parle_outer_step(NULL) == PARLE_EINVAL);
    EXPECT(parle_eval(NULL, -1, NULL, NULL, 0, NULL, NULL, NULL) == PARLE_EINVAL);
    parle_destroy(NULL);
    float *fake = (float *)4096;
    EXPECT(parle_k_inner_update(NULL, 0, 8, fake, fake, fake, fake, fake, NULL, 0.1f, 0.9f, 0.75f, 0.f, 0.03f) == PARLE_EINVAL);
    EXPECT(parle_k_inner_update(NULL, 2, 6, fake, fake, fake, fake, fake, NULL, 0.1f, 0.9f, 0.75f, 0.f, 0.03f) == PARLE_EINVAL);
    EXPECT(parle_k_replica_mean(NULL, 2, 8, NULL, fake) == PARLE_EINVAL);
    EXPECT(parle_k_spread_static(NULL, 2, (1LL << 33) + 4, fake, fake, fake) == PARLE_ESIZE);
    parle_conv_desc d = {1, 2, 4, 8, 8, 16, 32, 3, 3, 1};   /* stride 3 */
    EXPECT(parle_k_conv_forward(NULL, &d, fake, fake, NULL, NULL, 0, fake) == PARLE_EINVAL);
    EXPECT(parle_k_conv_scratch_bytes(&d) == -1);
    d.stride = 1;
    EXPECT(parle_k_conv_scratch_bytes(&d) >= 0);
    parle_act_desc a = {1, 2, 4, 8, 8, 0};
    EXPECT(parle_k_layer_scratch_bytes(&a) == -1);
    a.c = 16;
    EXPECT(parle_k_layer_scratch_bytes(&a) > 0);
    EXPECT(parle_k_bn_forward(NULL, &a, fake, fake, fake, fake, 8, fake, NULL, fake) == PARLE_ESIZE);
    EXPECT(parle_k_maxpool_forward(NULL, &a, NULL, fake) == PARLE_EINVAL);
  }
  printf("checksum %lld\n", checksum);
  printf(failures ? "%d expectation(s) failed\n" : "host walk ok%.0d\n", failures);
  return failures ? 1 : 0;
}
