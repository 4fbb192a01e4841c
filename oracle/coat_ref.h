/*
 * coat_ref.h -- CPU oracle for the FP8-state AdamW step of COAT (arxiv 2410.19313).
 *
 * TEST INFRASTRUCTURE ONLY.  This library is the slow, plain definition the GPU path is
 * checked against.  Only tests, the smoke check and the bench's cpu_baseline leg may call
 * it; the product path never does.  It shares no code, header, table or constant
 * generator with the HIP implementation.
 *
 * All pointers are HOST pointers.  Inner arithmetic is fp64 (libm); values are rounded
 * to fp32 exactly where the state the method keeps is fp32 (w, scale, k, and the new
 * moments just before they are quantized).
 *
 * Parity pins (tests/, run without a GPU) cover every function here; none is unpinned.
 */
#ifndef COAT_REF_H
#define COAT_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Hyper-parameters of one AdamW step (paper Sec. 3, Eq. 1 and the symbols below it). */
typedef struct {
  float    lr;            /* eta */
  float    beta1, beta2;  /* betas */
  float    eps;           /* epsilon, added to sqrt(v_hat) */
  float    weight_decay;  /* lambda, decoupled: enters as eta*lambda*w */
  int32_t  step;          /* t >= 1; bias corrections are 1 - beta^t */
  int32_t  group_size;    /* G >= 1: every G consecutive elements form a group (Sec. 3) */
  uint32_t flags;         /* COAT_REF_FLAG_*: expansion and, per moment, format / plain */
  float    k_min, k_max;  /* clamp applied to k; both 0 => defaults 2^-4 and 2^10 */
} coat_ref_hparams;

#define COAT_REF_FLAG_EXPAND  1u   /* dynamic range expansion on (off => k == 1) */
#define COAT_REF_FLAG_M_E5M2  2u   /* first moment stored as E5M2 instead of E4M3 */
#define COAT_REF_FLAG_E5M2    2u   /* the same bit for the standalone quantizer / dequantizer */
#define COAT_REF_FLAG_V_E5M2  4u   /* second moment stored as E5M2 */
#define COAT_REF_FLAG_M_PLAIN 8u   /* first moment: plain quantizer even when EXPAND is set */
#define COAT_REF_FLAG_V_PLAIN 16u  /* second moment: plain quantizer even when EXPAND is set */
#define COAT_REF_FLAG_BF16_SCALE 32u /* scales are stored in BF16 (Sec. 3): rounded UP to a bf16 value, which
                                        the quantizer then uses; k from (fmax * scale) / amin.  The arrays
                                        stay float here; every value in them is a bf16. */
#define COAT_REF_FLAG_BF16_K 64u     /* the exponents k are stored in BF16 as well (Sec. 4.2 computes k per group
                                        and step and keeps it beside the scale, whose storage Sec. 3 gives as BF16):
                                        rounded to the NEAREST bf16 value (ties to even, as a cast does) after the clamp;
                                        R_X^k then exceeds R_format by at most R_format^(2^-8) and the smallest element
                                        still rounds to the smallest subnormal; the quantizer uses the stored value.  The arrays stay float here; every value in them is a bf16. */

#define COAT_REF_FLAG_DQ_FP32 128u   /* step only, NOT the default: round the dequantized moments to fp32 before the
                                        update.  Appendix A says "dequantize to FP32"; the default reading takes the
                                        dequantizer as the real function a * (|c| / fmax)^(1/k) and rounds to fp32 only
                                        what the method stores or decides on (new moments before Q, scale, k, the value
                                        handed to the FP8 rounding).  This flag exists to MEASURE what the other reading
                                        would change (tests/test_oracle_step.py); nothing else uses it. */

/* OCP FP8 E4M3 ("FN"): 1-4-3 bits, bias 7, no infinity, 0x7F/0xFF are NaN, largest
 * finite 448 and smallest positive 2^-9 (the two constants Sec. 3 prints). */
double  coat_ref_e4m3_decode(uint8_t code);
/* Round-to-nearest, ties to even mantissa; |q| > 448 saturates to +-448; NaN -> 0x7F. */
uint8_t coat_ref_e4m3_encode(double q);

/* OCP FP8 E5M2: 1-5-2 bits, bias 15, IEEE-like (0x7C is infinity, 0x7D..0x7F NaN), largest
 * finite 57344 and smallest positive 2^-16 (Sec. 3).  Encode saturates to +-57344. */
double  coat_ref_e5m2_decode(uint8_t code);
uint8_t coat_ref_e5m2_encode(double q);

/* Quantize n fp32 values in groups of G (last group may be short).
 * Per group (Sec. 3 quantizer, Sec. 4.1 Definition 1, Sec. 4.2):
 *   amax = max|x|, amin = min over NON-ZERO |x|, scale = fl32(amax/448),
 *   k = fl32(clamp(log2(448*512) / log2(amax/amin))) if expansion is on and amax != amin,
 *   else 1;  code = E4M3(sign(x) * 448 * (|x| / (448*scale))^k).
 * All-zero group: scale 0, k 1, codes 0.  scale and k have ceil(n/G) entries.
 * With COAT_REF_FLAG_E5M2 the format constants are 57344 and 57344*65536 (Table 1's E5M2 rows). */
void coat_ref_quant_group(const float* x, uint64_t n, int32_t G, uint32_t flags,
                          float k_min, float k_max,
                          uint8_t* q, float* scale, float* k);

/* Inverse: x = sign(c) * (448*scale) * (|c|/448)^(1/k), c = decode(code)  (Sec. 4.2,
 * inverse expansion applied after the plain dequantizer of Sec. 3).  flags: only
 * COAT_REF_FLAG_E5M2 is read (57344 then replaces 448). */
void coat_ref_dequant_group(const uint8_t* q, const float* scale, const float* k,
                            uint64_t n, int32_t G, uint32_t flags, float* x);

/* Same as coat_ref_dequant_group but keeps the fp64 result (used inside the step). */
void coat_ref_dequant_group_f64(const uint8_t* q, const float* scale, const float* k,
                                uint64_t n, int32_t G, uint32_t flags, double* x);

/* 1xG per-group activation quantizer (Sec. 5.2: the fine-grained side of the mixed-granularity
 * flow; G = 16 in the paper's experiments).  x_bf16: raw bf16 patterns.  Per group
 * scale = fl32(max|x| / 448), code = E4M3(fl32(x / scale)); all-zero group: scale 0, codes 0.
 * No expansion: that is an optimizer-state technique. */
void coat_ref_act_quant_group(const uint16_t* x_bf16, uint64_t n, int32_t G,
                              uint8_t* q, float* scale);

/* Group Scaling (Sec. 5.2): per-tensor quantization with the two-stage max reduction.
 * Outputs: group_amax [ceil(n/G)] (stage 1), tensor_scale [1] = max(group_amax) / 448 (stage 2),
 * q [n] = E4M3(fl32(x / tensor_scale)). */
void coat_ref_act_quant_tensor(const uint16_t* x_bf16, uint64_t n, int32_t G,
                               float* group_amax, float* tensor_scale, uint8_t* q);

/* One fused optimizer step (Appendix A): dequantize m, v; update m, v, w; requantize.
 * w: fp32 master weights (in place).  grad_bf16: raw bf16 bit patterns.
 * m_q/v_q: E4M3 codes (in place).  *_scale, *_k: per-group metadata (in place).
 * Returns 0, or -1 on an invalid argument (NULL, G < 1, step < 1). */
int coat_ref_fp8_adamw_step(float* w, const uint16_t* grad_bf16,
                            uint8_t* m_q, float* m_scale, float* m_k,
                            uint8_t* v_q, float* v_scale, float* v_k,
                            uint64_t n, const coat_ref_hparams* hp);

/* The same step that also writes the new weights rounded to bf16 (nearest even) into w_bf16 [n]:
 * the copy a mixed-precision trainer hands to its BF16 model (the paper trains BF16/FP8 models
 * from FP32 master weights, Sec. 2 and Appendix A).  w_bf16 == NULL: no copy. */
int coat_ref_fp8_adamw_step_bf16w(float* w, uint16_t* w_bf16, const uint16_t* grad_bf16,
                                  uint8_t* m_q, float* m_scale, float* m_k,
                                  uint8_t* v_q, float* v_scale, float* v_k,
                                  uint64_t n, const coat_ref_hparams* hp);

/* Number of threads the step will use (OpenMP max threads; 1 when built without it). */
int coat_ref_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
