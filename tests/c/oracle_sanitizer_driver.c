/* Exercises the oracle's whole-step interface under AddressSanitizer / UndefinedBehaviorSanitizer (CPU only): two
   label models of a small conditional pair, ragged batches, a model without samples, three steps in plain and in
   bf16-storage-emulation mode, every query, the row next to the step (sampling, ANOVA).  Prints nothing but "ok". */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "gan_oracle.h"

static unsigned long long rng_state = 88172645463325252ull;
static double uniform01(void) {              /* xorshift64: inputs only, no part of the method */
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return (double)(rng_state >> 11) * (1.0 / 9007199254740992.0);
}
static double normal01(void) { return sqrt(-2.0 * log(uniform01() + 1e-300)) * cos(6.283185307179586 * uniform01()); }

#define CHECK(x) do { if (!(x)) { fprintf(stderr, "check failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

int main(void) {
  oracle_config c;
  memset(&c, 0, sizeof(c));
  c.struct_size = sizeof(c);
  c.n_models = 3; c.n_labels = 3; c.cond_g = 3; c.cond_d = 3; c.z_dim = 5;
  c.img_c = 1; c.img_hw = 8; c.g_h0 = 2; c.n_g = 2; c.g_ch[0] = 6; c.g_ch[1] = 4; c.n_d = 2; c.d_ch[0] = 4; c.d_ch[1] = 6;
  c.lr = 2e-4; c.beta1 = 0.5; c.beta2 = 0.999; c.adam_eps = 1e-8; c.bn_eps = 1e-5; c.bn_momentum = 0.1; c.leaky_slope = 0.2;
  c.d_loss_scale = 0.5; c.g_loss_scale = 0.5;
  for (int emul = 0; emul < 2; ++emul) {
    oracle_ctx* o = NULL;
    CHECK(oracle_create(&c, &o) == 0 && o);
    CHECK(oracle_set_bf16_emulation(o, emul) == 0);
    for (int which = 0; which < 2; ++which) {
      const int64_t P = oracle_param_count(o, which);
      CHECK(P > 0);
      oreal* p = (oreal*)malloc(sizeof(oreal) * (size_t)P);
      for (int l = 0; l < c.n_models; ++l) {
        for (int64_t i = 0; i < P; ++i) p[i] = (oreal)(0.02 * normal01());
        CHECK(oracle_set_params(o, which, l, p) == 0);
      }
      free(p);
    }
    enum { N = 11 };
    int32_t lab[N] = {0, 2, 2, 0, 2, 0, 2, 2, 0, 2, 2};      /* model 1 has no samples */
    const int img = c.img_c * c.img_hw * c.img_hw;
    oreal* z = (oreal*)malloc(sizeof(oreal) * N * c.z_dim);
    oreal* x = (oreal*)malloc(sizeof(oreal) * N * img);
    oreal* out = (oreal*)malloc(sizeof(oreal) * N * img);
    for (int step = 0; step < 3; ++step) {
      for (int i = 0; i < N * c.z_dim; ++i) z[i] = (oreal)normal01();
      for (int i = 0; i < N * img; ++i) x[i] = (oreal)tanh(normal01());
      CHECK(oracle_train_step(o, lab, z, x, N, -1) == 0);
      oreal jd[3], jg[3];
      int32_t cnt[3], perm[N], offs[4];
      CHECK(oracle_get_losses(o, jd, jg, cnt) == 0);
      CHECK(cnt[0] == 4 && cnt[1] == 0 && cnt[2] == 7);
      CHECK(isfinite((double)jd[0]) && isfinite((double)jg[2]));
      CHECK(oracle_get_routing(o, perm, offs) == 0 && offs[3] == N);
    }
    CHECK(oracle_generate(o, lab, z, N, out, 1, -1) == 0);
    CHECK(oracle_generate(o, lab, z, N, out, 0, 2) == 0);
    for (int which = 0; which < 2; ++which) {
      const int64_t P = oracle_param_count(o, which), B = oracle_bn_count(o, which);
      oreal* a = (oreal*)malloc(sizeof(oreal) * (size_t)P * 3);
      oreal* b = (oreal*)malloc(sizeof(oreal) * (size_t)(B > 0 ? B : 1) * 2);
      int64_t t = -1;
      CHECK(oracle_get_params(o, which, 2, a) == 0 && oracle_get_grads(o, which, 2, a) == 0);
      CHECK(oracle_get_opt_state(o, which, 2, a + P, a + 2 * P, &t) == 0 && t == 3);
      CHECK(oracle_set_opt_state(o, which, 2, a + P, a + 2 * P, t) == 0);
      CHECK(oracle_get_opt_state(o, which, 1, a + P, a + 2 * P, &t) == 0 && t == 0);
      if (B > 0) CHECK(oracle_get_bn_running(o, which, 0, b, b + B) == 0 && oracle_set_bn_running(o, which, 0, b, b + B) == 0);
      free(a); free(b);
    }
    {
      const double prior[3] = {0.5, 0.0, 0.5};
      float u[N];
      int32_t drawn[N];
      for (int i = 0; i < N; ++i) u[i] = (float)uniform01();
      CHECK(oracle_sample(o, prior, u, z, N, out, drawn, 1) == 0);
      for (int i = 0; i < N; ++i) CHECK(drawn[i] == 0 || drawn[i] == 2);
      float* xf = (float*)malloc(sizeof(float) * N * img);
      double F[1];
      for (int i = 0; i < N * img; ++i) xf[i] = (float)x[i];
      CHECK(oracle_anova_f(lab, xf, N, 3, c.img_c, c.img_hw * c.img_hw, F) == 0);
      free(xf);
    }
    free(z); free(x); free(out);
    oracle_destroy(o);
  }
  printf("ok\n");
  return 0;
}
