/* Driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the column-wise CPU
 * sampler (baselines/columnwise/cw_sampler.c, included below so that this is one translation
 * unit): a few decode steps on a small batch with every feature on, a batch size that is not a
 * multiple of the column block, both logit types, histories set and pushed.  Exit code 0 and
 * no sanitizer report is the test; tests/test_sanitizers_cpu.py builds and runs it. */
#include "../../baselines/columnwise/cw_sampler.c"

#include <stdio.h>

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) {
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return (uint32_t)(rng_state >> 32);
}
static float rndf(void) { return (float)(rnd() >> 8) * (1.0f / 16777216.0f); }

int main(void) {
  const int B = 21, V = 5003, n_lp = 4, steps = 3;
  float* z = (float*)malloc(sizeof(float) * (size_t)B * V);
  uint16_t* zb = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)B * V);
  float tau[21], top_p[21], min_p[21], theta[21], phi[21], psi[21];
  int32_t top_k[21], ids[21], lp_ids[21 * 5];
  int64_t row_id[21];
  float lp[21 * 5];
  for (int b = 0; b < B; ++b) {
    tau[b] = b % 5 == 0 ? 0.0f : 0.3f + rndf();
    top_k[b] = (int32_t[]){0, 1, 7, 300}[b % 4];
    top_p[b] = b % 3 == 0 ? 1.0f : 0.6f + 0.4f * rndf();
    min_p[b] = b % 2 ? 0.05f : 0.0f;
    theta[b] = b % 4 == 1 ? 1.0f : 1.2f;
    phi[b] = 0.3f; psi[b] = b % 2 ? -0.2f : 0.4f;
    row_id[b] = 1000 + 7 * b;
  }
  cw_params P = {tau, top_k, top_p, min_p, theta, phi, psi, row_id};
  for (int dt = 0; dt < 2; ++dt) {
    cw_state* st = cw_create(B, V, 3);
    if (!st) return 2;
    for (int b = 0; b < B; ++b) {
      int32_t h[64];
      const int n = (b * 5) % 64;
      for (int i = 0; i < n; ++i) h[i] = (int32_t)(rnd() % (uint32_t)(V + 10)) - 5;   /* some ids out of range: padding */
      cw_set_history(st, b, h, n);
    }
    for (int s = 0; s < steps; ++s) {
      for (size_t i = 0; i < (size_t)B * V; ++i) {
        z[i] = 5.0f * (rndf() - 0.5f) + (rnd() % 97 == 0 ? 6.0f : 0.0f);
        union { float f; uint32_t u; } x; x.f = z[i];
        zb[i] = (uint16_t)(x.u >> 16);
      }
      if (dt == 0) cw_load_f32(st, z, V, 0, V);
      else { cw_load_bf16(st, zb, V, 0, V / 2); cw_load_bf16(st, zb + V / 2, V, V / 2, V - V / 2); }
      if (cw_sample(st, &P, 42, (uint64_t)s, n_lp, ids, lp_ids, lp) != 0) return 3;
      for (int b = 0; b < B; ++b)
        if (ids[b] < 0 || ids[b] >= V) { fprintf(stderr, "row %d: id %d out of range\n", b, ids[b]); return 4; }
      cw_push_tokens(st, ids);
    }
    cw_destroy(st);
  }
  free(z); free(zb);
  puts("ok");
  return 0;
}
