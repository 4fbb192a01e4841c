/*
 * coat_ref.c -- CPU oracle for COAT's FP8-state AdamW step (arxiv 2410.19313).
 *
 * TEST INFRASTRUCTURE ONLY: called by tests/, the smoke check and the bench's
 * cpu_baseline leg.  Plain C, fp64 inner math, one loop nest per definition, no blocking
 * or fusion beyond "one group at a time".  Nothing here is shared with the HIP path.
 *
 * Parity pins: every function below is pinned by tests that need no GPU (E4M3 codec by
 * brute force over all 256 codes and by a library cast; the quantizer by the k == 1
 * special case, the range identity R_f(X) = R_X^k, oddness and scale invariance; the step
 * by its G == 1 reduction to a library AdamW and by a hand-worked two-element case).
 */
#include "coat_ref.h"

#include <math.h>
#include <stddef.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Sec. 3: largest finite E4M3 magnitude.  Sec. 4.1: R_E4M3 = 448 * 512. */
#define E4M3_MAX 448.0
#define LOG2_R_E4M3 17.807354922057606 /* log2(229376) */
/* Sec. 3: E5M2 spans 2^-16 .. 57344, so R_E5M2 = 57344 * 65536. */
#define E5M2_MAX 57344.0
#define LOG2_R_E5M2 31.807354922057606 /* log2(3758096384) */

typedef struct { double fmax, log2_range; int e5m2; } fmt_t;
static fmt_t fmt_of(int e5m2) {
  fmt_t f;
  f.e5m2 = e5m2;
  f.fmax = e5m2 ? E5M2_MAX : E4M3_MAX;
  f.log2_range = e5m2 ? LOG2_R_E5M2 : LOG2_R_E4M3;
  return f;
}

int coat_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- E4M3 codec (OCP 8-bit floating point, E4M3 variant; Sec. 3 cites it) ---------- */

double coat_ref_e4m3_decode(uint8_t code) {
  int s = code >> 7, e = (code >> 3) & 15, m = code & 7;
  double v;
  if (e == 15 && m == 7) return NAN;             /* the only non-finite pattern */
  if (e == 0) v = ldexp((double)m / 8.0, -6);    /* subnormal: 2^-6 * m/8 */
  else        v = ldexp(1.0 + (double)m / 8.0, e - 7);
  return s ? -v : v;
}

uint8_t coat_ref_e4m3_encode(double q) {
  uint8_t sign = signbit(q) ? 0x80 : 0x00;
  double a = fabs(q);
  int e, mant, code;
  if (isnan(q)) return 0x7F;
  if (a > E4M3_MAX) a = E4M3_MAX;                /* saturate, never emit NaN for a number */
  if (a < ldexp(1.0, -6)) {
    /* subnormal spacing is 2^-9; rint() is round-half-even in the default mode.  A
     * result of 8 is the code of the smallest normal number, 2^-6. */
    code = (int)rint(a * 512.0);
  } else {
    int ex;
    (void)frexp(a, &ex);                         /* a = f * 2^ex, f in [0.5, 1) */
    e = ex - 1;                                  /* a = (1 + frac) * 2^e */
    mant = (int)rint((ldexp(a, -e) - 1.0) * 8.0);
    if (mant == 8) { mant = 0; e += 1; }         /* mantissa carry */
    code = ((e + 7) << 3) | mant;
    if (code > 0x7E) code = 0x7E;
  }
  return (uint8_t)(sign | code);
}

/* ---- E5M2 codec (OCP 8-bit floating point, E5M2 variant: IEEE-like, with infinities) -- */

double coat_ref_e5m2_decode(uint8_t code) {
  int s = code >> 7, e = (code >> 2) & 31, m = code & 3;
  double v;
  if (e == 31) v = m ? NAN : INFINITY;
  else if (e == 0) v = ldexp((double)m / 4.0, -14);  /* subnormal: 2^-14 * m/4 */
  else v = ldexp(1.0 + (double)m / 4.0, e - 15);
  return s ? -v : v;
}

uint8_t coat_ref_e5m2_encode(double q) {
  uint8_t sign = signbit(q) ? 0x80 : 0x00;
  double a = fabs(q);
  int e, mant, code;
  if (isnan(q)) return 0x7F;
  if (a > E5M2_MAX) a = E5M2_MAX;                /* saturate to the largest finite value */
  if (a < ldexp(1.0, -14)) {
    code = (int)rint(a * 65536.0);               /* subnormal spacing 2^-16; 4 = smallest normal */
  } else {
    int ex;
    (void)frexp(a, &ex);
    e = ex - 1;
    mant = (int)rint((ldexp(a, -e) - 1.0) * 4.0);
    if (mant == 4) { mant = 0; e += 1; }
    code = ((e + 15) << 2) | mant;
    if (code > 0x7B) code = 0x7B;
  }
  return (uint8_t)(sign | code);
}

static double fmt_decode(fmt_t f, uint8_t c) { return f.e5m2 ? coat_ref_e5m2_decode(c) : coat_ref_e4m3_decode(c); }
static uint8_t fmt_encode(fmt_t f, double q) { return f.e5m2 ? coat_ref_e5m2_encode(q) : coat_ref_e4m3_encode(q); }

/* ---- per-group quantizer with dynamic range expansion (Sec. 3, Sec. 4) ------------- */

static void resolve_k_bounds(float* k_min, float* k_max) {
  if (*k_min == 0.0f && *k_max == 0.0f) { *k_min = 0.0625f; *k_max = 1024.0f; }
}

/* Smallest bf16 value that is not below s (s > 0 and finite): the scale "stored in BF16" of Sec. 3.
 * Rounding UP keeps every |x| / (fmax * scale) at or below 1, so no code saturates. */
static float bf16_ceil(float s) {
  union { uint32_t u; float f; } cvt;
  cvt.f = s;
  cvt.u = (cvt.u + 0xFFFFu) & 0xFFFF0000u;
  return cvt.f;
}

/* The bf16 value nearest to k, ties to the even one (k > 0 and finite): the exponent "stored in BF16"
 * like the scale, by the conversion that a cast to bf16 performs.  The stored exponent is within
 * 2^-8 of the exact one (half a bf16 step), so R_X^k exceeds R_format by at most R_format^(2^-8): the
 * group's smallest element lands at 0.95 (E4M3; E5M2 0.92) of the smallest subnormal or above and still rounds to it.
 * A group that receives no gradient reproduces the range its stored exponent made, computes that
 * exponent again and keeps it: rounding to nearest makes the stored value a fixed point (rounding
 * down does too in exact arithmetic, but any evaluation that lands one rounding short of the bf16
 * value then steps a notch down per idle step, and with a BF16 scale beside it the exact value is
 * not a bf16 number and every idle step loses a notch). */
static float bf16_nearest(float k) {
  /* bf16 keeps 8 significant bits: for k = m * 2^e with 1/2 <= m < 1 its values are the multiples of 2^(e-8) */
  int e;
  double quantum;
  (void)frexp((double)k, &e);
  quantum = ldexp(1.0, e - 8);
  return (float)(rint((double)k / quantum) * quantum);   /* rint: to nearest, ties to even (default rounding mode) */
}

static void quant_one_group(const float* x, uint64_t len, int expand, fmt_t f, int scale16, int k16,
                            float k_min, float k_max,
                            uint8_t* q, float* scale_out, float* k_out) {
  double amax = 0.0, amin = INFINITY, top;
  float scale, k = 1.0f;
  double a, kd;
  uint64_t i;

  /* Definition 1, with the minimum taken over the non-zero magnitudes. */
  for (i = 0; i < len; ++i) {
    double ax = fabs((double)x[i]);
    if (ax > amax) amax = ax;
    if (ax > 0.0 && ax < amin) amin = ax;
  }
  if (amax == 0.0) {                             /* nothing but zeros (or NaNs) */
    for (i = 0; i < len; ++i)
      q[i] = isnan(x[i]) ? 0x7F : (signbit(x[i]) ? 0x80 : 0x00);
    *scale_out = 0.0f;
    *k_out = 1.0f;
    return;
  }
  scale = (float)(amax / f.fmax);                /* S_X of Sec. 3, kept in fp32 */
  top = amax;
  if (scale16) {
    /* BF16 scale: the group is normalized by fmax * scale >= amax, so the range that has to fit
     * the format is (fmax * scale) / amin: k from that ratio keeps the smallest element
     * representable (with amax / amin the whole group would shrink by (amax / (fmax scale))^k) */
    scale = bf16_ceil(scale);
    top = f.fmax * (double)scale;
  }
  if (expand && amax != amin) {
    /* optimal k of Sec. 4.2: R_X^k = R_format */
    kd = f.log2_range / log2(top / amin);
    if (kd < (double)k_min) kd = (double)k_min;
    if (kd > (double)k_max) kd = (double)k_max;
    k = (float)kd;
    if (k16) k = bf16_nearest(k);                  /* after the clamp; the quantizer below uses the stored value */
  }
  /* Quantize with the STORED scale and k so that Q and DQ agree.  The expanded group is
   * f(x / a) with a = fmax * scale ~= amax, whose largest element is 1, so the plain
   * quantizer's scale is 1/fmax and the value to round is fmax * (|x|/a)^k. */
  a = f.fmax * (double)scale;
  kd = (double)k;
  for (i = 0; i < len; ++i) {
    double xv = (double)x[i], mag;
    if (xv == 0.0) { q[i] = signbit(x[i]) ? 0x80 : 0x00; continue; }
    /* Appendix A keeps the optimizer arithmetic in FP32: the number handed to the E4M3
     * rounding is an fp32 value (with k == 1 it is the fp32 quotient x / S_X of Sec. 3). */
    mag = (double)(float)(f.fmax * pow(fabs(xv) / a, kd));
    if (mag > f.fmax) mag = f.fmax;
    q[i] = fmt_encode(f, copysign(mag, xv));
  }
  *scale_out = scale;
  *k_out = k;
}

static void dequant_one_group(const uint8_t* q, float scale, float k, fmt_t f, uint64_t len,
                              double* x) {
  double a = f.fmax * (double)scale, inv_k = 1.0 / (double)k;
  uint64_t i;
  for (i = 0; i < len; ++i) {
    double c = fmt_decode(f, q[i]);
    if (c == 0.0) { x[i] = c; continue; }        /* f(0) = 0, sign of zero kept */
    x[i] = copysign(a * pow(fabs(c) / f.fmax, inv_k), c);
  }
}

void coat_ref_quant_group(const float* x, uint64_t n, int32_t G, uint32_t flags,
                          float k_min, float k_max,
                          uint8_t* q, float* scale, float* k) {
  int64_t ng, gi;
  if (!x || !q || !scale || !k || G < 1 || n == 0) return;
  resolve_k_bounds(&k_min, &k_max);
  ng = (int64_t)((n + (uint64_t)G - 1) / (uint64_t)G);
#pragma omp parallel for schedule(static)
  for (gi = 0; gi < ng; ++gi) {
    uint64_t lo = (uint64_t)gi * (uint64_t)G;
    uint64_t len = (n - lo < (uint64_t)G) ? n - lo : (uint64_t)G;
    quant_one_group(x + lo, len, (flags & COAT_REF_FLAG_EXPAND) != 0, fmt_of((flags & COAT_REF_FLAG_E5M2) != 0),
                    (flags & COAT_REF_FLAG_BF16_SCALE) != 0, (flags & COAT_REF_FLAG_BF16_K) != 0, k_min, k_max,
                    q + lo, scale + gi, k + gi);
  }
}

void coat_ref_dequant_group_f64(const uint8_t* q, const float* scale, const float* k,
                                uint64_t n, int32_t G, uint32_t flags, double* x) {
  int64_t ng, gi;
  if (!x || !q || !scale || !k || G < 1 || n == 0) return;
  ng = (int64_t)((n + (uint64_t)G - 1) / (uint64_t)G);
#pragma omp parallel for schedule(static)
  for (gi = 0; gi < ng; ++gi) {
    uint64_t lo = (uint64_t)gi * (uint64_t)G;
    uint64_t len = (n - lo < (uint64_t)G) ? n - lo : (uint64_t)G;
    dequant_one_group(q + lo, scale[gi], k[gi], fmt_of((flags & COAT_REF_FLAG_E5M2) != 0), len, x + lo);
  }
}

void coat_ref_dequant_group(const uint8_t* q, const float* scale, const float* k,
                            uint64_t n, int32_t G, uint32_t flags, float* x) {
  int64_t ng, gi;
  if (!x || !q || !scale || !k || G < 1 || n == 0) return;
  ng = (int64_t)((n + (uint64_t)G - 1) / (uint64_t)G);
#pragma omp parallel for schedule(static)
  for (gi = 0; gi < ng; ++gi) {
    uint64_t lo = (uint64_t)gi * (uint64_t)G, i;
    uint64_t len = (n - lo < (uint64_t)G) ? n - lo : (uint64_t)G;
    double* tmp = (double*)malloc(len * sizeof(double));
    if (!tmp) continue;
    dequant_one_group(q + lo, scale[gi], k[gi], fmt_of((flags & COAT_REF_FLAG_E5M2) != 0), len, tmp);
    for (i = 0; i < len; ++i) x[lo + i] = (float)tmp[i];
    free(tmp);
  }
}

/* ---- activation quantizers (Sec. 5.2): bf16 in, E4M3 out, no expansion ---------------- */

static float bf16_to_float(uint16_t bits) {
  union { uint32_t u; float f; } cvt;
  cvt.u = (uint32_t)bits << 16;
  return cvt.f;
}

/* 1xG per-group quantization of activations (the fine-grained flow of the non-linear layers;
 * G = 16 in the paper's experiments): per group S = max|X| / 448, X_fp8 = round(X / S), the
 * quotient formed in fp32 (the activation arithmetic is not wider than that). */
void coat_ref_act_quant_group(const uint16_t* x_bf16, uint64_t n, int32_t G,
                              uint8_t* q, float* scale) {
  int64_t ng, gi;
  if (!x_bf16 || !q || !scale || G < 1 || n == 0) return;
  ng = (int64_t)((n + (uint64_t)G - 1) / (uint64_t)G);
#pragma omp parallel for schedule(static)
  for (gi = 0; gi < ng; ++gi) {
    uint64_t lo = (uint64_t)gi * (uint64_t)G, i;
    uint64_t len = (n - lo < (uint64_t)G) ? n - lo : (uint64_t)G;
    float amax = 0.0f, s;
    for (i = 0; i < len; ++i) {
      float ax = fabsf(bf16_to_float(x_bf16[lo + i]));
      if (ax > amax) amax = ax;
    }
    s = amax / 448.0f;
    scale[gi] = s;
    for (i = 0; i < len; ++i) {
      float x = bf16_to_float(x_bf16[lo + i]);
      q[lo + i] = (s > 0.0f) ? coat_ref_e4m3_encode((double)(x / s)) : (uint8_t)(signbit(x) ? 0x80 : 0x00);
    }
  }
}

/* Group Scaling (Sec. 5.2): per-tensor quantization whose max reduction is split in two stages,
 * (1) the maximum of every 1xG group, kept as an intermediate tensor, (2) the maximum of that
 * G-times smaller tensor.  Then S = max|X| / 448 for the whole tensor and X_fp8 = round(X / S).
 * group_amax [ceil(n/G)] and tensor_scale [1] are outputs. */
void coat_ref_act_quant_tensor(const uint16_t* x_bf16, uint64_t n, int32_t G,
                               float* group_amax, float* tensor_scale, uint8_t* q) {
  int64_t ng, gi, i;
  float tmax = 0.0f, s;
  if (!x_bf16 || !q || !group_amax || !tensor_scale || G < 1 || n == 0) return;
  ng = (int64_t)((n + (uint64_t)G - 1) / (uint64_t)G);
  for (gi = 0; gi < ng; ++gi) {                  /* stage 1 */
    uint64_t lo = (uint64_t)gi * (uint64_t)G, j;
    uint64_t len = (n - lo < (uint64_t)G) ? n - lo : (uint64_t)G;
    float amax = 0.0f;
    for (j = 0; j < len; ++j) {
      float ax = fabsf(bf16_to_float(x_bf16[lo + j]));
      if (ax > amax) amax = ax;
    }
    group_amax[gi] = amax;
  }
  for (gi = 0; gi < ng; ++gi)                    /* stage 2 */
    if (group_amax[gi] > tmax) tmax = group_amax[gi];
  s = tmax / 448.0f;
  *tensor_scale = s;
#pragma omp parallel for schedule(static)
  for (i = 0; i < (int64_t)n; ++i) {
    float x = bf16_to_float(x_bf16[i]);
    q[i] = (s > 0.0f) ? coat_ref_e4m3_encode((double)(x / s)) : (uint8_t)(signbit(x) ? 0x80 : 0x00);
  }
}

/* ---- the fused step (Appendix A; update rule of Sec. 3, Eq. 1) ---------------------- */

static double bf16_to_double(uint16_t bits) {
  union { uint32_t u; float f; } cvt;
  cvt.u = (uint32_t)bits << 16;                  /* bf16 is the top half of an fp32 */
  return (double)cvt.f;
}

/* fp32 -> bf16, round to nearest even (bf16 is the upper half of an fp32) */
static uint16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } cvt;
  cvt.f = f;
  if (f != f) return (uint16_t)((cvt.u >> 16) | 0x0040);      /* keep NaN a NaN */
  return (uint16_t)((cvt.u + 0x7FFFu + ((cvt.u >> 16) & 1u)) >> 16);
}

int coat_ref_fp8_adamw_step(float* w, const uint16_t* grad_bf16,
                            uint8_t* m_q, float* m_scale, float* m_k,
                            uint8_t* v_q, float* v_scale, float* v_k,
                            uint64_t n, const coat_ref_hparams* hp) {
  return coat_ref_fp8_adamw_step_bf16w(w, NULL, grad_bf16, m_q, m_scale, m_k, v_q, v_scale, v_k, n, hp);
}

int coat_ref_fp8_adamw_step_bf16w(float* w, uint16_t* w_bf16, const uint16_t* grad_bf16,
                                  uint8_t* m_q, float* m_scale, float* m_k,
                                  uint8_t* v_q, float* v_scale, float* v_k,
                                  uint64_t n, const coat_ref_hparams* hp) {
  double lr, b1, b2, eps, wd, bc1, bc2;
  float k_min, k_max;
  int32_t G;
  int64_t ng, gi;
  int failed = 0, expand_m, expand_v, scale16, k16;
  fmt_t fm, fv;

  if (!hp) return -1;
  if (n == 0) return 0;
  if (!w || !grad_bf16 || !m_q || !m_scale || !m_k || !v_q || !v_scale || !v_k) return -1;
  G = hp->group_size;
  if (G < 1 || hp->step < 1) return -1;

  lr = hp->lr; b1 = hp->beta1; b2 = hp->beta2; eps = hp->eps; wd = hp->weight_decay;
  bc1 = 1.0 - pow(b1, (double)hp->step);         /* 1 - beta1^t */
  bc2 = 1.0 - pow(b2, (double)hp->step);         /* 1 - beta2^t */
  k_min = hp->k_min; k_max = hp->k_max;
  resolve_k_bounds(&k_min, &k_max);
  ng = (int64_t)((n + (uint64_t)G - 1) / (uint64_t)G);
  /* per-moment format and expansion switch: the 4 x 4 grid of Table 1 */
  fm = fmt_of((hp->flags & COAT_REF_FLAG_M_E5M2) != 0);
  fv = fmt_of((hp->flags & COAT_REF_FLAG_V_E5M2) != 0);
  expand_m = (hp->flags & COAT_REF_FLAG_EXPAND) && !(hp->flags & COAT_REF_FLAG_M_PLAIN);
  expand_v = (hp->flags & COAT_REF_FLAG_EXPAND) && !(hp->flags & COAT_REF_FLAG_V_PLAIN);
  scale16 = (hp->flags & COAT_REF_FLAG_BF16_SCALE) != 0;
  k16 = (hp->flags & COAT_REF_FLAG_BF16_K) != 0;

#pragma omp parallel for schedule(static)
  for (gi = 0; gi < ng; ++gi) {
    uint64_t lo = (uint64_t)gi * (uint64_t)G, i;
    uint64_t len = (n - lo < (uint64_t)G) ? n - lo : (uint64_t)G;
    double* m = (double*)malloc(2 * len * sizeof(double));
    float* mt = (float*)malloc(2 * len * sizeof(float));
    double* v;
    float* vt;
    if (!m || !mt) {
      free(m); free(mt);
#pragma omp atomic write
      failed = 1;
      continue;
    }
    v = m + len; vt = mt + len;

    /* m_{t-1} = DQ(m^q), v_{t-1} = DQ(v^q), each followed by the inverse expansion */
    dequant_one_group(m_q + lo, m_scale[gi], m_k[gi], fm, len, m);
    dequant_one_group(v_q + lo, v_scale[gi], v_k[gi], fv, len, v);

    if (hp->flags & COAT_REF_FLAG_DQ_FP32)        /* the other reading of "dequantize to FP32" (see the header) */
      for (i = 0; i < len; ++i) { m[i] = (double)(float)m[i]; v[i] = (double)(float)v[i]; }

    for (i = 0; i < len; ++i) {
      double g = bf16_to_double(grad_bf16[lo + i]);
      double wi = (double)w[lo + i];
      double m_t = b1 * m[i] + (1.0 - b1) * g;
      double v_t = b2 * v[i] + (1.0 - b2) * g * g;
      double m_hat = m_t / bc1;
      double v_hat = v_t / bc2;
      /* the weight sees the new moments BEFORE they are quantized */
      w[lo + i] = (float)(wi - lr * (m_hat / (sqrt(v_hat) + eps) + wd * wi));
      if (w_bf16) w_bf16[lo + i] = f32_to_bf16(w[lo + i]);   /* the model's copy of the new weight */
      mt[i] = (float)m_t;                        /* moments live in fp32 before Q */
      vt[i] = (float)v_t;
    }

    /* m^q_t, S = Q(m_t);  v^q_t, S = Q(v_t) */
    quant_one_group(mt, len, expand_m, fm, scale16, k16, k_min, k_max, m_q + lo, m_scale + gi, m_k + gi);
    quant_one_group(vt, len, expand_v, fv, scale16, k16, k_min, k_max, v_q + lo, v_scale + gi, v_k + gi);
    free(m); free(mt);
  }
  return failed ? -1 : 0;
}
