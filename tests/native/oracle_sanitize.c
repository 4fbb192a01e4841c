/* Runs every entry point of the CPU oracle (oracle/coat_ref.c, compiled INTO this program) on small
 * ragged inputs held in heap blocks of exactly the documented sizes, so that a build with
 * -fsanitize=address,undefined turns an out-of-bounds access, a signed overflow, a bad shift or a
 * misaligned access inside the oracle into a failure.  Test infrastructure; no GPU.
 * Prints "oracle_sanitize ok" and exits 0 when every call returns. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "coat_ref.h"

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) {
  rng_state = rng_state * 1664525u + 1013904223u;
  return rng_state >> 8;
}
static float rnd_float(float scale) { return scale * ((float)(rnd() & 0xffff) / 32768.0f - 1.0f); }
static uint16_t bf16_of(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
static void* block(size_t bytes) {
  void* p = malloc(bytes ? bytes : 1);     /* exact size: the red zone starts right behind it */
  if (!p) exit(3);
  memset(p, 0, bytes);
  return p;
}

static int one_size(uint64_t n, int32_t G, uint32_t flags) {
  const uint64_t ng = (n + (uint64_t)G - 1) / (uint64_t)G;
  float* x = block(n * 4);
  float* w = block(n * 4);
  uint16_t* g = block(n * 2);
  uint16_t* wb = block(n * 2);
  uint8_t *mq = block(n), *vq = block(n), *q = block(n);
  float *ms = block(ng * 4), *mk = block(ng * 4), *vs = block(ng * 4), *vk = block(ng * 4);
  float *s = block(ng * 4), *k = block(ng * 4), *amax = block(ng * 4);
  double* x64 = block(n * 8);
  float tensor_scale = 0.0f;
  coat_ref_hparams hp = {3e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 1, G, flags, 0.0f, 0.0f};
  uint64_t i;
  int rc = 0, t;
  for (i = 0; i < n; ++i) {
    x[i] = (rnd() % 7 == 0) ? 0.0f : rnd_float(1e-3f);
    w[i] = rnd_float(0.05f);
  }
  for (i = 0; i < ng; ++i) mk[i] = vk[i] = 1.0f;
  coat_ref_quant_group(x, n, G, flags & (COAT_REF_FLAG_EXPAND | COAT_REF_FLAG_E5M2 | COAT_REF_FLAG_BF16_SCALE | COAT_REF_FLAG_BF16_K), 0.0f, 0.0f, q, s, k);
  coat_ref_dequant_group(q, s, k, n, G, flags & COAT_REF_FLAG_E5M2, x);
  coat_ref_dequant_group_f64(q, s, k, n, G, flags & COAT_REF_FLAG_E5M2, x64);
  for (t = 1; t <= 3; ++t) {
    hp.step = t;
    for (i = 0; i < n; ++i) g[i] = bf16_of((rnd() % 11 == 0) ? 0.0f : rnd_float(2e-3f));
    rc |= coat_ref_fp8_adamw_step(w, g, mq, ms, mk, vq, vs, vk, n, &hp);
    rc |= coat_ref_fp8_adamw_step_bf16w(w, wb, g, mq, ms, mk, vq, vs, vk, n, &hp);
  }
  coat_ref_act_quant_group(g, n, G, q, s);
  coat_ref_act_quant_tensor(g, n, G, amax, &tensor_scale, q);
  for (i = 0; i < n; ++i)
    if (!isfinite(w[i])) rc |= 64;
  free(x); free(w); free(g); free(wb); free(mq); free(vq); free(q); free(ms); free(mk); free(vs); free(vk);
  free(s); free(k); free(amax); free(x64);
  return rc;
}

int main(void) {
  static const uint64_t sizes[] = {0, 1, 15, 16, 17, 31, 32, 33, 127, 128, 129, 1000, 1023, 1024, 1025, 4099};
  static const int32_t groups[] = {1, 16, 32, 128, 512};
  static const uint32_t flag_sets[] = {
      COAT_REF_FLAG_EXPAND, 0u, COAT_REF_FLAG_EXPAND | COAT_REF_FLAG_M_E5M2 | COAT_REF_FLAG_V_E5M2,
      COAT_REF_FLAG_EXPAND | COAT_REF_FLAG_M_PLAIN, COAT_REF_FLAG_EXPAND | COAT_REF_FLAG_V_PLAIN | COAT_REF_FLAG_V_E5M2,
      COAT_REF_FLAG_EXPAND | COAT_REF_FLAG_BF16_SCALE, COAT_REF_FLAG_EXPAND | COAT_REF_FLAG_BF16_SCALE | COAT_REF_FLAG_BF16_K};
  size_t a, b, c;
  int code;
  for (code = 0; code < 256; ++code) {
    const double d4 = coat_ref_e4m3_decode((uint8_t)code), d5 = coat_ref_e5m2_decode((uint8_t)code);
    if (isfinite(d4) && (coat_ref_e4m3_encode(d4) & 0x7f) != (code & 0x7f)) return 4;
    if (isfinite(d5) && (coat_ref_e5m2_encode(d5) & 0x7f) != (code & 0x7f)) return 5;
  }
  (void)coat_ref_e4m3_encode(1e300); (void)coat_ref_e4m3_encode(-1e-300); (void)coat_ref_e4m3_encode(NAN);
  (void)coat_ref_e5m2_encode(1e300); (void)coat_ref_e5m2_encode(-1e-300); (void)coat_ref_e5m2_encode(INFINITY);
  for (a = 0; a < sizeof sizes / sizeof sizes[0]; ++a)
    for (b = 0; b < sizeof groups / sizeof groups[0]; ++b)
      for (c = 0; c < sizeof flag_sets / sizeof flag_sets[0]; ++c) {
        const int rc = one_size(sizes[a], groups[b], flag_sets[c]);
        if (rc) {
          printf("n=%llu G=%d flags=%u: rc %d\n", (unsigned long long)sizes[a], groups[b], flag_sets[c], rc);
          return 1;
        }
      }
  printf("oracle_sanitize ok (%d threads)\n", coat_ref_num_threads());
  return 0;
}
