// coat_kernels.hip -- gfx950 kernels and C ABI of the FP8-state AdamW step of COAT
// (arxiv 2410.19313: Sec. 3 quantizer and update rule, Sec. 4.2 dynamic range expansion,
// Appendix A step order, Table 1 format grid) and of the activation quantizers of Sec. 5.2.
// Hand-written for CDNA4:
//   * 64-wide wavefronts; every lane owns 16 consecutive elements, a quantization group of G
//     elements is G/16 adjacent lanes and its max/min are DPP butterflies inside the wavefront;
//   * every global load/store instruction of a wavefront covers one contiguous 1 KiB row and is
//     issued as a streaming access; per-wavefront LDS tiles convert between those rows and the
//     16-elements-per-lane layout the arithmetic wants;
//   * one 1024-element chunk per wavefront, three resident workgroups per CU, and an admission
//     gate that lines up the bulk loads of neighbouring wavefronts (gate_on_neighbourhood);
//   * no atomics, no inter-wave communication: each group is owned by exactly one wavefront.
// Sections: storage modes, helpers, LDS staging, (de)quantizer arithmetic, the fused step,
// the multi-tensor step, standalone quantizer / dequantizer, activation quantizers, host side.
//
// Arithmetic (fp32 throughout; transcendentals are the hardware log2/exp2/rcp/sqrt), with fmax
// the largest finite value of the moment's FP8 format (448 for E4M3, 57344 for E5M2):
//   inverse expansion  |c/fmax|^(1/k) = exp2( log2|c/fmax| * (1/k) ), the logarithm from a table
//                      of the 127 code magnitudes (compensated for the first moment);
//   expansion          fmax * (|x|/a)^k = exp2( k * log2(|x| * (1/a)) + log2 fmax ), the logarithm
//                      taken of the RATIO so that its magnitude stays below log2(range)/k;
//   conversion         native fp32 -> OCP FP8 pack instructions (round to nearest even).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "coat.h"

namespace {

constexpr int kWave = 64;                 // lanes per wavefront
constexpr int kEPL = 16;                  // consecutive elements owned by one lane
#ifndef COAT_WPB
#define COAT_WPB 4
#endif
constexpr int kWavesPerBlock = COAT_WPB;
constexpr int kBlock = kWave * kWavesPerBlock;
constexpr int kChunk = kWave * kEPL;      // elements one wavefront handles per iteration

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

#include "coat_tables.inc"

// ---------------------------------------------------------------------------------------
// Storage mode of one moment: FP8 format and whether the dynamic range expansion is applied
// (the rows / columns of Table 1).  StaticMode folds at compile time (the default E4M3 + expansion
// fast path); RuntimeMode carries the two switches as wavefront-uniform values, so one kernel per
// group size serves the other fifteen combinations.
// ---------------------------------------------------------------------------------------
template <bool E5M2, bool EXPAND>
struct StaticMode {
  __device__ __forceinline__ bool e5m2() const { return E5M2; }
  __device__ __forceinline__ bool expand() const { return EXPAND; }
  __device__ __forceinline__ bool scale16() const { return false; }
};
struct RuntimeMode {
  bool e5, ex;
  bool s16;   // the per-group scales are stored as bf16 (Sec. 3) instead of fp32
  __device__ __forceinline__ bool e5m2() const { return e5; }
  __device__ __forceinline__ bool expand() const { return ex; }
  __device__ __forceinline__ bool scale16() const { return s16; }
};
typedef StaticMode<false, true> DefaultMode;

template <class Mode> __device__ __forceinline__ float fmt_max(const Mode& md) { return md.e5m2() ? 57344.0f : 448.0f; }
template <class Mode> __device__ __forceinline__ float fmt_inv_max(const Mode& md) {
  return md.e5m2() ? 1.0f / 57344.0f : 1.0f / 448.0f;
}
// log2(fmax) and log2(fmax / smallest subnormal): 448 * 2^9 (Sec. 4.1) and 57344 * 2^16
template <class Mode> __device__ __forceinline__ float fmt_log2_max(const Mode& md) {
  return md.e5m2() ? 15.807354922057604f : 8.807354922057604f;
}
template <class Mode> __device__ __forceinline__ float fmt_log2_range(const Mode& md) {
  return md.e5m2() ? 31.807354922057604f : 17.807354922057606f;
}

struct StepArgs {
  float* w;
  uint16_t* wb;          // optional bf16 copy of the new weights (nullptr: none)
  const uint16_t* g;
  uint8_t* mq; float* ms; float* mk;
  uint8_t* vq; float* vs; float* vk;
  uint64_t n;            // elements
  uint64_t n_full;       // number of full kChunk-sized chunks
  uint64_t n_groups;     // ceil(n / G)
  // The kernel carries the new moments divided by (1 - beta): m' = m_t / (1 - beta1) =
  // (beta1/(1-beta1)) m + g is ONE fma (rounded once, which matters where the two terms cancel),
  // v' = v_t / (1 - beta2) = (beta2/(1-beta2)) v + g*g one mul and one fma.  The factors are
  // folded into the constants below and into the per-group scale.
  float beta1_ratio, beta2_ratio;        // beta / (1 - beta)
  float one_minus_beta1, one_minus_beta2;
  float neg_lr_m;        // -lr * (1 - beta1) / (1 - beta1^t)
  float neg_lr_wd;       // -lr * weight_decay
  float denom_scale;     // sqrt((1 - beta2) / (1 - beta2^t))
  float eps;
  float k_min, k_max;
  RuntimeMode mode_m, mode_v;
};

struct QuantArgs {
  const float* x; uint8_t* q; float* scale; float* k;
  uint64_t n, n_full, n_groups;
  float k_min, k_max;
  RuntimeMode mode;
};

struct DequantArgs {
  const uint8_t* q; const float* scale; const float* k; float* x;
  uint64_t n, n_full, n_groups;
  RuntimeMode mode;
};

// ---------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// Per-group scale i of an array that holds fp32 or, with scale16, bf16 values (the pointer is typed
// float* either way).  A stored bf16 scale is exact: the quantizer rounded it before using it.
template <class Mode>
__device__ __forceinline__ float load_scale(const Mode& md, const float* p, uint64_t i) {
  if (md.scale16()) return as_f32(static_cast<uint32_t>(reinterpret_cast<const uint16_t*>(p)[i]) << 16);
  return p[i];
}
// The same for group gl of a FULL chunk whose first group is gb, without control flow: one dword
// load serves both layouts (a branch here costs the kernel its overlap of loads: the compiler
// drains the load counter where the two sides meet; measured 17.3 ms against 15.9).  A chunk holds
// an even number of groups starting at an even index, so the dword is inside the chunk's scales.
template <class Mode>
__device__ __forceinline__ float load_scale_full_chunk(const Mode& md, const float* p, uint64_t gb, int gl) {
  const bool s16 = md.scale16();
  const uint32_t w = reinterpret_cast<const uint32_t*>(p)[s16 ? (gb + gl) >> 1 : gb + gl];
  const uint32_t half = (gl & 1) ? (w & 0xffff0000u) : (w << 16);
  return as_f32(s16 ? half : w);
}
template <class Mode>
__device__ __forceinline__ void store_scale(const Mode& md, float* p, uint64_t i, float s) {
  if (md.scale16()) reinterpret_cast<uint16_t*>(p)[i] = static_cast<uint16_t>(as_u32(s) >> 16);
  else p[i] = s;
}

__device__ __forceinline__ float hw_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float hw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float hw_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float hw_sqrt(float x) { return __builtin_amdgcn_sqrtf(x); }

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// Butterfly all-reduce over LPG adjacent lanes (LPG = lanes per group, a power of two <= 32).
//   xor 1 / xor 2 : quad_perm, lanes 4..7 / 8..15 : row_half_mirror / row_mirror (after the
//   previous steps every lane of the smaller block already holds that block's result),
//   xor 16 : ds_swizzle inside 32 lanes.
template <int LPG, bool IS_MAX>
__device__ __forceinline__ float group_allreduce(float x) {
  auto op = [](float a, float b) { return IS_MAX ? __builtin_fmaxf(a, b) : __builtin_fminf(a, b); };
  if constexpr (LPG >= 2) x = op(x, dpp_mov<0xB1>(x));    // quad_perm:[1,0,3,2]
  if constexpr (LPG >= 4) x = op(x, dpp_mov<0x4E>(x));    // quad_perm:[2,3,0,1]
  if constexpr (LPG >= 8) x = op(x, dpp_mov<0x141>(x));   // row_half_mirror
  if constexpr (LPG >= 16) x = op(x, dpp_mov<0x140>(x));  // row_mirror
  if constexpr (LPG >= 32)
    x = op(x, __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, x), 0x401F)));
  return x;
}

// Compile-time streaming hints (bit mask): 1 load codes, 2 store codes, 4 load gradients,
// 8 load fp32, 16 store fp32.  A set bit issues the access as non-temporal.
#ifndef COAT_NT
#define COAT_NT 31
#endif
template <int BIT, typename T>
__device__ __forceinline__ T ldg(const T* p) {
  if constexpr ((COAT_NT & BIT) != 0) return __builtin_nontemporal_load(p);
  else return *p;
}
template <int BIT, typename T>
__device__ __forceinline__ void stg(T* p, T v) {
  if constexpr ((COAT_NT & BIT) != 0) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// Element-wise guarded accesses straight into the lane layout: only the ragged last chunk
// (n mod 1024 elements, one wavefront) uses them.
__device__ __forceinline__ void load_f32x16_guarded(const float* p, uint64_t base, uint64_t n, float (&x)[kEPL]) {
#pragma unroll
  for (int e = 0; e < kEPL; ++e) x[e] = (base + e < n) ? p[base + e] : 0.0f;
}
__device__ __forceinline__ void store_f32x16_guarded(float* p, uint64_t base, uint64_t n, const float (&x)[kEPL]) {
#pragma unroll
  for (int e = 0; e < kEPL; ++e)
    if (base + e < n) p[base + e] = x[e];
}
// a bf16 is the upper half of an fp32
__device__ __forceinline__ void load_bf16x16_guarded(const uint16_t* p, uint64_t base, uint64_t n, float (&x)[kEPL]) {
#pragma unroll
  for (int e = 0; e < kEPL; ++e)
    x[e] = (base + e < n) ? as_f32(static_cast<uint32_t>(p[base + e]) << 16) : 0.0f;
}
// 16 code bytes as four dwords, element e in byte (e & 3) of dword (e >> 2)
__device__ __forceinline__ void load_codes16_guarded(const uint8_t* p, uint64_t base, uint64_t n, uint32_t (&c)[4]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    uint32_t v = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b)
      if (base + 4 * d + b < n) v |= static_cast<uint32_t>(p[base + 4 * d + b]) << (8 * b);
    c[d] = v;
  }
}
__device__ __forceinline__ void store_codes16_guarded(uint8_t* p, uint64_t base, uint64_t n, const uint32_t (&c)[4]) {
#pragma unroll
  for (int e = 0; e < kEPL; ++e)
    if (base + e < n) p[base + e] = static_cast<uint8_t>(c[e >> 2] >> (8 * (e & 3)));
}

// ---------------------------------------------------------------------------------------
// LDS staging: HBM likes every load/store instruction of a wavefront to cover one contiguous
// span (and to be issued as a streaming access), the arithmetic wants every lane to own 16
// consecutive elements.  A per-wavefront LDS tile converts between the two: rows of 64 x 16 B on
// the memory side, 64 B (fp32) or 32 B (bf16) per lane on the register side.
// 16-byte slot s lives at s + (s >> 3) (one pad slot after every eight), which makes both access
// patterns conflict free and keeps every address of a lane a constant offset from one of two
// per-lane bases: row side 72 j + lane + (lane >> 3), lane side 4 lane + (lane >> 1) + i (fp32)
// or 2 lane + (lane >> 2) + j (bf16).  A wavefront only ever touches its own tile and LDS
// executes one wavefront's accesses in order, so no barrier is needed.
// ---------------------------------------------------------------------------------------
constexpr int kTileSlotsW = 256 + 32;   // fp32 tile: 1024 elements + padding, in 16-byte slots
constexpr int kTileSlotsG = 128 + 16;   // bf16 tile

struct StageTiles { f32x4* w; u32x4* g; };

// rows (memory side) -> 16 consecutive fp32 per lane, through the wavefront's fp32 tile
__device__ __forceinline__ void tile_rows_to_lanes(f32x4* tile, int lane, const f32x4 (&rows)[4], float (&x)[kEPL]) {
  f32x4* const row = tile + lane + (lane >> 3);            // + 72 j
  const f32x4* const own = tile + 4 * lane + (lane >> 1);  // + i
#pragma unroll
  for (int j = 0; j < 4; ++j) row[72 * j] = rows[j];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const f32x4 t = own[i];
    x[4 * i + 0] = t.x; x[4 * i + 1] = t.y; x[4 * i + 2] = t.z; x[4 * i + 3] = t.w;
  }
}

// 16 consecutive fp32 per lane -> rows, written straight to memory (p: start of the chunk)
__device__ __forceinline__ void tile_lanes_to_rows_store(f32x4* tile, int lane, const float (&x)[kEPL], float* p) {
  const f32x4* const row = tile + lane + (lane >> 3);
  f32x4* const own = tile + 4 * lane + (lane >> 1);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const f32x4 t = {x[4 * i + 0], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]};
    own[i] = t;
  }
  f32x4* q = reinterpret_cast<f32x4*>(p);
#pragma unroll
  for (int j = 0; j < 4; ++j) stg<16>(q + 64 * j + lane, row[72 * j]);
}

// rows of bf16 -> 16 consecutive gradients per lane as fp32
__device__ __forceinline__ void tile_rows_to_lanes_bf16(u32x4* tile, int lane, const u32x4 (&rows)[2], float (&g)[kEPL]) {
  u32x4* const row = tile + lane + (lane >> 3);            // + 72 j
  const u32x4* const own = tile + 2 * lane + (lane >> 2);  // + j
#pragma unroll
  for (int j = 0; j < 2; ++j) row[72 * j] = rows[j];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const u32x4 t = own[j];
    g[8 * j + 0] = as_f32(t.x << 16); g[8 * j + 1] = as_f32(t.x & 0xffff0000u);
    g[8 * j + 2] = as_f32(t.y << 16); g[8 * j + 3] = as_f32(t.y & 0xffff0000u);
    g[8 * j + 4] = as_f32(t.z << 16); g[8 * j + 5] = as_f32(t.z & 0xffff0000u);
    g[8 * j + 6] = as_f32(t.w << 16); g[8 * j + 7] = as_f32(t.w & 0xffff0000u);
  }
}

// two fp32 -> packed bf16 pair (round to nearest even: the native pack convert)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 16 consecutive fp32 per lane -> bf16 rows written straight to memory (p: start of the chunk)
__device__ __forceinline__ void tile_lanes_to_rows_store_bf16(u32x4* tile, int lane, const float (&x)[kEPL],
                                                              uint16_t* p) {
  const u32x4* const row = tile + lane + (lane >> 3);
  u32x4* const own = tile + 2 * lane + (lane >> 2);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const u32x4 t = {pack_bf16(x[8 * j + 0], x[8 * j + 1]), pack_bf16(x[8 * j + 2], x[8 * j + 3]),
                     pack_bf16(x[8 * j + 4], x[8 * j + 5]), pack_bf16(x[8 * j + 6], x[8 * j + 7])};
    own[j] = t;
  }
  u32x4* q = reinterpret_cast<u32x4*>(p);
#pragma unroll
  for (int j = 0; j < 2; ++j) stg<16>(q + 64 * j + lane, row[72 * j]);
}

// The lookup table in LDS: per format 256 entries so that the whole code byte indexes it (the sign
// bit is ignored).  TABLES = 1 loads E4M3 only, 2 loads E4M3 then E5M2.
template <int TABLES>
__device__ __forceinline__ void fill_lut(Log2Entry* lut) {
  for (int i = threadIdx.x; i < 256 * TABLES; i += blockDim.x) lut[i] = kLog2Code[i >> 8][i & 127];
  __syncthreads();
}

constexpr float kLn2 = 0.6931471805599453f;

// |c/fmax|^(1/k) for 16 codes.
//   ACCURATE = false: exp2(L * (1/k)), good to about |L/k| * 2^-22 relative;
//   ACCURATE = true : the rounding of the product and of 1/k is recovered with one fma
//     (r = L - t*k is the exact residual of t = fl(L * fl(1/k)) against L/k, times k), the
//     table's own rounding is added from its low word, and exp2(t + d) = exp2(t) * (1 + d ln2).
//     Used for the first moment, whose update beta1*m + (1-beta1)*g cancels and so amplifies
//     the error of m into the group minimum that fixes the next exponent k.
//   SIGNED: carry the code's sign bit into the result.
template <bool SIGNED, bool ACCURATE>
__device__ __forceinline__ void inverse_expand16(const Log2Entry* lut, const uint32_t (&c)[4], float k,
                                                 float inv_k, float (&y)[kEPL]) {
  const float inv_k_ln2 = inv_k * kLn2;
#pragma unroll
  for (int e = 0; e < kEPL; ++e) {
    const uint32_t d = c[e >> 2];
    const int sh = 8 * (e & 3);
    const uint32_t code = (d >> sh) & 0xffu;
    float v;
    if constexpr (ACCURATE) {
      const Log2Entry l = lut[code];
      const float t = l.hi * inv_k;
      const float r = __builtin_fmaf(-t, k, l.hi) + l.lo;
      const float p = hw_exp2(t);
      v = __builtin_fmaf(p, r * inv_k_ln2, p);
    } else {
      v = hw_exp2(lut[code].hi * inv_k);
    }
    if constexpr (SIGNED) v = as_f32(as_u32(v) | ((d << (24 - sh)) & 0x80000000u));
    y[e] = v;
  }
}

// plain dequantizer without expansion: the decoded code itself (to be multiplied by the scale)
template <bool E5M2>
__device__ __forceinline__ void decode16(const uint32_t (&c)[4], float (&y)[kEPL]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    if constexpr (E5M2) {
      y[4 * d + 0] = __builtin_amdgcn_cvt_f32_bf8(c[d], 0);
      y[4 * d + 1] = __builtin_amdgcn_cvt_f32_bf8(c[d], 1);
      y[4 * d + 2] = __builtin_amdgcn_cvt_f32_bf8(c[d], 2);
      y[4 * d + 3] = __builtin_amdgcn_cvt_f32_bf8(c[d], 3);
    } else {
      y[4 * d + 0] = __builtin_amdgcn_cvt_f32_fp8(c[d], 0);
      y[4 * d + 1] = __builtin_amdgcn_cvt_f32_fp8(c[d], 1);
      y[4 * d + 2] = __builtin_amdgcn_cvt_f32_fp8(c[d], 2);
      y[4 * d + 3] = __builtin_amdgcn_cvt_f32_fp8(c[d], 3);
    }
  }
}

// Dequantize 16 codes of one moment up to a per-group factor: the stored value is y * factor with
//   expansion on : y = +-|c/fmax|^(1/k), factor = fmax * scale      (Sec. 4.2, after the DQ of Sec. 3)
//   expansion off: y = c,               factor = scale              (k is 1 in this mode, not read)
template <bool SIGNED, bool ACCURATE, class Mode>
__device__ __forceinline__ float dequant16(const Mode& md, const Log2Entry* lut, const uint32_t (&c)[4],
                                           float scale, float k, float (&y)[kEPL]) {
  if (md.expand()) {
    inverse_expand16<SIGNED, ACCURATE>(lut + (md.e5m2() ? 256 : 0), c, k, hw_rcp(k), y);
    return fmt_max(md) * scale;
  }
  if (md.e5m2()) decode16<true>(c, y);
  else decode16<false>(c, y);
  return scale;
}

struct GroupQuant { float scale, k, inv_a; };

// Per-group scale and exponent from the group's extreme magnitudes (Definition 1, Sec. 4.2).
// amin is the minimum over NON-ZERO magnitudes (+inf when there is none).  The values reduced
// over are x / unit (unit = 1 - beta inside the step, 1 otherwise): the stored scale refers to x.
//   expansion on : inv_a = unit / (fmax * scale), so that (held value) * inv_a = |x| / (fmax*scale)
//   expansion off: k = 1; inv_a only flags an empty group (the quotient is formed exactly)
template <class Mode>
__device__ __forceinline__ GroupQuant group_quant_params(const Mode& md, float amax, float amin, float k_min,
                                                         float k_max, float unit) {
  GroupQuant r;
  // amax / fmax, correctly rounded: multiply by the rounded reciprocal, then one residual step
  const float inv_fmax = fmt_inv_max(md), fmax = fmt_max(md);
  const float ax = amax * unit;
  float s = ax * inv_fmax;
  s = __builtin_fmaf(__builtin_fmaf(-fmax, s, ax), inv_fmax, s);
  float top = amax;                                  // what the group is normalized by, in held units
  if (md.scale16()) {
    // BF16 scale: round UP to a bf16 value (every |x| / (fmax*scale) stays <= 1, nothing saturates)
    // and take the range that has to fit the format against fmax*scale rather than amax
    s = as_f32((as_u32(s) + 0xFFFFu) & 0xFFFF0000u);
    top = (fmax * s) / unit;
  }
  float k = 1.0f;
  if (md.expand()) {
    // two hardware reciprocals (1 ulp each) are enough here: k moves by ~2 ulp
    // (the max keeps a ratio that rounds below 1 from turning the huge k negative)
    const float ratio = __builtin_fmaxf(top * hw_rcp(amin), 1.0f);    // R_X
    float kk = fmt_log2_range(md) * hw_rcp(hw_log2(ratio));
    kk = __builtin_amdgcn_fmed3f(kk, k_min, k_max);
    k = (amax != amin) ? kk : 1.0f;
  }
  const float inv_a = unit * hw_rcp(md.expand() ? fmax * s : s);
  const bool empty = !(amax > 0.0f);                 // all zero: scale 0, k 1, every code 0
  r.scale = empty ? 0.0f : s;
  r.k = empty ? 1.0f : k;
  r.inv_a = empty ? 0.0f : inv_a;
  return r;
}

// max |x| and min non-zero |x| over the lane's 16 values
__device__ __forceinline__ void lane_extremes(const float (&x)[kEPL], float& amax, float& amin) {
  float hi = 0.0f, lo = __builtin_huge_valf();
#pragma unroll
  for (int e = 0; e < kEPL; ++e) {
    hi = __builtin_fmaxf(hi, __builtin_fabsf(x[e]));
    lo = __builtin_fminf(lo, __builtin_fabsf(x[e]));
  }
  if (__builtin_expect(lo == 0.0f, 0)) {             // rare: some element is exactly zero
    lo = __builtin_huge_valf();
#pragma unroll
    for (int e = 0; e < kEPL; ++e) {
      const float ax = __builtin_fabsf(x[e]);
      lo = __builtin_fminf(lo, ax > 0.0f ? ax : __builtin_huge_valf());
    }
  }
  amax = hi; amin = lo;
}

template <bool E5M2>
__device__ __forceinline__ uint32_t pack4(const float (&q)[4]) {
  if constexpr (E5M2) {
    const uint32_t p = __builtin_amdgcn_cvt_pk_bf8_f32(q[0], q[1], 0u, false);
    return __builtin_amdgcn_cvt_pk_bf8_f32(q[2], q[3], p, true);
  } else {
    const uint32_t p = __builtin_amdgcn_cvt_pk_fp8_f32(q[0], q[1], 0u, false);
    return __builtin_amdgcn_cvt_pk_fp8_f32(q[2], q[3], p, true);
  }
}

// Quantize 16 held values (x / unit) to FP8 codes.  The native converts round to nearest even and
// round magnitudes up to fmax * (1 + 2^-5) (E4M3: 464) back to fmax; the value converted never
// exceeds fmax * (1 + 2^-22)^k_max, so no clamp is needed.
//   expansion on : code = FP8( sign(x) * fmax * (|x| / (fmax*scale))^k ) as one fma in the exponent:
//                  exp2(k log2 r + log2 fmax), rounded once at magnitude <= log2(range)/2
//                  (log2 0 = -inf, so a zero stays zero)
//   expansion off: code = FP8( x / scale ) with the correctly rounded fp32 quotient (the plain
//                  quantizer of Sec. 3, kept as a baseline; it is not tuned)
// SIGNED = false (second moment, never negative) skips the sign transfer.
template <bool SIGNED, class Mode>
__device__ __forceinline__ void quantize16(const Mode& md, const float (&x)[kEPL], const GroupQuant& gq,
                                           uint32_t (&c)[4], float unit) {
  const float log2_fmax = fmt_log2_max(md);
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    float q[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const float xv = x[4 * d + b];
      if (md.expand()) {
        const float m = hw_exp2(__builtin_fmaf(hw_log2(__builtin_fabsf(xv) * gq.inv_a), gq.k, log2_fmax));
        q[b] = SIGNED ? as_f32(as_u32(m) | (as_u32(xv) & 0x80000000u)) : m;
      } else {
        q[b] = gq.inv_a != 0.0f ? (xv * unit) / gq.scale : 0.0f;   // IEEE division: correctly rounded
      }
    }
    c[d] = md.e5m2() ? pack4<true>(q) : pack4<false>(q);
  }
}

// ---------------------------------------------------------------------------------------
// the fused step
// ---------------------------------------------------------------------------------------

// Per-group metadata of one chunk as one lane sees it (its own group's words).
struct GroupMeta { float m_scale, m_k, v_scale, v_k; };

// The arithmetic of the step on one lane's 16 elements, registers in, registers out:
// w (in/out), g, codes (in/out), metadata (in/out).  Cross-lane traffic: the group reductions.
template <int G, class ModeM, class ModeV>
__device__ __forceinline__ void step_core(const StepArgs& a, const ModeM& mm, const ModeV& mv,
                                          const Log2Entry* lut, float (&w)[kEPL], const float (&g)[kEPL],
                                          uint32_t (&mc)[4], uint32_t (&vc)[4], GroupMeta& meta) {
  constexpr int LPG = G / kEPL;                      // lanes per group
  float m[kEPL], v[kEPL];
  // beta/(1-beta) * (magnitude of the decoded unit)
  const float m_fac = a.beta1_ratio * dequant16<true, true>(mm, lut, mc, meta.m_scale, meta.m_k, m);
  const float v_fac = a.beta2_ratio * dequant16<false, false>(mv, lut, vc, meta.v_scale, meta.v_k, v);

#pragma unroll
  for (int e = 0; e < kEPL; ++e) {
    const float ge = g[e];
    const float m_t = __builtin_fmaf(m[e], m_fac, ge);              // m_t / (1 - beta1), Sec. 3
    const float v_t = __builtin_fmaf(ge, ge, v[e] * v_fac);         // v_t / (1 - beta2)
    // Eq. (1) with the unquantized new moments; sqrt(v_t / bc2) = sqrt(v') * sqrt((1-beta2)/bc2)
    const float denom = __builtin_fmaf(hw_sqrt(v_t), a.denom_scale, a.eps);
    const float upd = m_t * hw_rcp(denom);
    const float wt = __builtin_fmaf(upd, a.neg_lr_m, w[e]);
    w[e] = __builtin_fmaf(w[e], a.neg_lr_wd, wt);
    m[e] = m_t;
    v[e] = v_t;
  }

  float m_max, m_min, v_max, v_min;
  lane_extremes(m, m_max, m_min);
  lane_extremes(v, v_max, v_min);
  m_max = group_allreduce<LPG, true>(m_max);
  m_min = group_allreduce<LPG, false>(m_min);
  v_max = group_allreduce<LPG, true>(v_max);
  v_min = group_allreduce<LPG, false>(v_min);
  const GroupQuant qm = group_quant_params(mm, m_max, m_min, a.k_min, a.k_max, a.one_minus_beta1);
  const GroupQuant qv = group_quant_params(mv, v_max, v_min, a.k_min, a.k_max, a.one_minus_beta2);
  quantize16<true>(mm, m, qm, mc, a.one_minus_beta1);
  quantize16<false>(mv, v, qv, vc, a.one_minus_beta2);
  meta.m_scale = qm.scale; meta.m_k = qm.k;
  meta.v_scale = qv.scale; meta.v_k = qv.k;
}

// What one lane fetches for one full chunk, still in the layout of the memory side: weight and
// gradient rows (row j of the chunk, 16 bytes at lane), its own 16 code bytes, its group's words.
struct RawChunk {
  f32x4 w[4];
  u32x4 g[2];
  u32x4 mc, vc;
  GroupMeta meta;
};

template <int G, class ModeM, class ModeV>
__device__ __forceinline__ void issue_loads(const StepArgs& a, const ModeM& mm, const ModeV& mv, uint64_t chunk,
                                            int lane, RawChunk& r) {
  constexpr int LPG = G / kEPL;
  // chunk is uniform over the wavefront: the array bases below are scalar, lanes add 32-bit offsets
  const uint64_t cb = chunk * kChunk;
  const uint64_t gb = chunk * (kChunk / G);
  const f32x4* wq = reinterpret_cast<const f32x4*>(a.w + cb);
  const u32x4* gq = reinterpret_cast<const u32x4*>(a.g + cb);
  const u32x4* mq = reinterpret_cast<const u32x4*>(a.mq + cb);
  const u32x4* vq = reinterpret_cast<const u32x4*>(a.vq + cb);
  const int gl = lane / LPG;
#pragma unroll
  for (int j = 0; j < 4; ++j) r.w[j] = ldg<8>(wq + 64 * j + lane);
#pragma unroll
  for (int j = 0; j < 2; ++j) r.g[j] = ldg<4>(gq + 64 * j + lane);
  r.mc = ldg<1>(mq + lane);
  r.vc = ldg<1>(vq + lane);
  r.meta.m_scale = load_scale_full_chunk(mm, a.ms, gb, gl);
  r.meta.v_scale = load_scale_full_chunk(mv, a.vs, gb, gl);
  r.meta.m_k = a.mk[gb + gl];          // written as 1 (and ignored) by a moment stored without expansion
  r.meta.v_k = a.vk[gb + gl];
}

// One full chunk: rows -> lane layout through the LDS tiles, the arithmetic, and back out.
template <int G, class ModeM, class ModeV>
__device__ __forceinline__ void process_chunk(const StepArgs& a, const ModeM& mm, const ModeV& mv,
                                              const Log2Entry* lut, const StageTiles& tiles, uint64_t chunk,
                                              int lane, RawChunk& r) {
  constexpr int LPG = G / kEPL;
  const uint64_t cb = chunk * kChunk;
  const uint64_t gb = chunk * (kChunk / G);

  float w[kEPL], g[kEPL];
  tile_rows_to_lanes_bf16(tiles.g, lane, r.g, g);
  tile_rows_to_lanes(tiles.w, lane, r.w, w);
  uint32_t mc[4] = {r.mc.x, r.mc.y, r.mc.z, r.mc.w};
  uint32_t vc[4] = {r.vc.x, r.vc.y, r.vc.z, r.vc.w};
  GroupMeta meta = r.meta;

  step_core<G>(a, mm, mv, lut, w, g, mc, vc, meta);

  tile_lanes_to_rows_store(tiles.w, lane, w, a.w + cb);
  if (a.wb) tile_lanes_to_rows_store_bf16(tiles.g, lane, w, a.wb + cb);   // the gradient tile is free by now
  const u32x4 mo = {mc[0], mc[1], mc[2], mc[3]}, vo = {vc[0], vc[1], vc[2], vc[3]};
  stg<2>(reinterpret_cast<u32x4*>(a.mq + cb) + lane, mo);
  stg<2>(reinterpret_cast<u32x4*>(a.vq + cb) + lane, vo);
  if ((lane % LPG) == 0) {
    const int gl = lane / LPG;
    store_scale(mm, a.ms, gb + gl, meta.m_scale); a.mk[gb + gl] = meta.m_k;
    store_scale(mv, a.vs, gb + gl, meta.v_scale); a.vk[gb + gl] = meta.v_k;
  }
}

// Admission gate.  Before a wavefront issues the loads of its chunk it reads ONE word that all
// wavefronts of its neighbourhood (kGateSpan consecutive chunks, i.e. a quarter of that many
// workgroups, which the dispatcher spreads over all eight XCDs) read as well: the first per-group
// exponent k of the neighbourhood's first chunk, a word of the tensor's own metadata that is
// fetched anyway.  The first reader misses to HBM; the others are served by the memory-side cache as soon
// as that fill lands.  The wavefronts of a neighbourhood therefore start their bulk loads at about
// the same moment and HBM sees their adjacent rows together, which keeps DRAM pages open
// (measured on the 7B set with three resident workgroups per CU: 15.85 -> 15.05 ms; spans of
// 32..128 chunks are equally good, 16 or >= 512 lose most of the gain; a probe that only its own
// wavefront reads, or one that hits in L2, gains nothing; the lighter kernels, whose wavefronts
// live too briefly to wait, gain nothing either, except the quantizer).  The empty asm emits no
// instruction: it makes the chunk index depend on the probed word so that the compiler keeps the
// loads behind it.  The probed value itself is never used, so it is harmless that the wavefront
// owning that chunk may be rewriting the word at the same moment.
#ifndef COAT_GATE_SHIFT
#define COAT_GATE_SHIFT 5
#endif
constexpr int kGateSpan = 1 << COAT_GATE_SHIFT;
// `words`: any array of the operand with a fixed number of 32-bit words per chunk.
__device__ __forceinline__ uint64_t gate_on_neighbourhood(const void* words, uint64_t chunk, int words_per_chunk) {
#ifdef COAT_NO_GATE
  return chunk;
#endif
  const uint64_t first = chunk & ~static_cast<uint64_t>(kGateSpan - 1);
  const uint32_t probe = __builtin_amdgcn_readfirstlane(static_cast<const uint32_t*>(words)[first * words_per_chunk]);
  uint32_t lo = static_cast<uint32_t>(chunk);
  asm volatile("" : "+s"(lo) : "s"(probe));
  return (chunk & 0xffffffff00000000ull) | lo;
}

template <bool GENERIC> struct ModesOf;
template <> struct ModesOf<false> {
  typedef DefaultMode M;
  __device__ static DefaultMode m(const StepArgs&) { return DefaultMode(); }
  __device__ static DefaultMode v(const StepArgs&) { return DefaultMode(); }
};
template <> struct ModesOf<true> {
  typedef RuntimeMode M;
  __device__ static RuntimeMode m(const StepArgs& a) { return a.mode_m; }
  __device__ static RuntimeMode v(const StepArgs& a) { return a.mode_v; }
};

// Main kernel: one chunk per wavefront (the loop only runs again for buffers with more chunks
// than the grid has wavefronts).  The first chunk's loads are issued before the block fills its
// lookup table, so the table's latency hides behind them.
// GENERIC = false: both moments E4M3 with expansion (the method as the paper runs it);
// GENERIC = true : per-moment format and expansion read from the arguments (Table 1's grid).
template <int G, bool GENERIC>
__global__ __launch_bounds__(kBlock) void adamw_step_kernel(StepArgs a) {
  constexpr int kTables = GENERIC ? 2 : 1;
  __shared__ Log2Entry lut[256 * kTables];
  __shared__ f32x4 tile_w[kWavesPerBlock * kTileSlotsW];
  __shared__ u32x4 tile_g[kWavesPerBlock * kTileSlotsG];
  const typename ModesOf<GENERIC>::M mm = ModesOf<GENERIC>::m(a), mv = ModesOf<GENERIC>::v(a);
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wavefront-uniform
  const StageTiles tiles = {tile_w + wv * kTileSlotsW, tile_g + wv * kTileSlotsG};
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv;

  RawChunk r;
  const bool have = chunk < a.n_full;
  if (have) chunk = gate_on_neighbourhood(a.mk, chunk, kChunk / G);
  if (have) issue_loads<G>(a, mm, mv, chunk, lane, r);
  fill_lut<kTables>(lut);                            // every wavefront of the block reaches this
  if (have) process_chunk<G>(a, mm, mv, lut, tiles, chunk, lane, r);
  for (chunk += stride; chunk < a.n_full; chunk += stride) {
    issue_loads<G>(a, mm, mv, chunk, lane, r);
    process_chunk<G>(a, mm, mv, lut, tiles, chunk, lane, r);
  }
}

// The ragged last chunk (n % 1024 elements): one wavefront, element-wise guarded accesses
// straight into the lane layout.
template <int G, class ModeM, class ModeV>
__device__ __forceinline__ void process_tail_chunk(const StepArgs& a, const ModeM& mm, const ModeV& mv,
                                                   const Log2Entry* lut, int lane) {
  constexpr int LPG = G / kEPL;
  const uint64_t chunk = a.n_full;
  const uint64_t base = chunk * kChunk + static_cast<uint64_t>(lane) * kEPL;
  const uint64_t gidx = chunk * (kChunk / G) + static_cast<uint64_t>(lane / LPG);
  const bool gvalid = gidx < a.n_groups;
  float w[kEPL], g[kEPL];
  uint32_t mc[4], vc[4];
  load_f32x16_guarded(a.w, base, a.n, w);
  load_bf16x16_guarded(a.g, base, a.n, g);
  load_codes16_guarded(a.mq, base, a.n, mc);
  load_codes16_guarded(a.vq, base, a.n, vc);
  GroupMeta meta;
  meta.m_scale = gvalid ? load_scale(mm, a.ms, gidx) : 0.0f;
  meta.v_scale = gvalid ? load_scale(mv, a.vs, gidx) : 0.0f;
  meta.m_k = gvalid ? a.mk[gidx] : 1.0f;
  meta.v_k = gvalid ? a.vk[gidx] : 1.0f;
  step_core<G>(a, mm, mv, lut, w, g, mc, vc, meta);
  store_f32x16_guarded(a.w, base, a.n, w);
  if (a.wb) {
#pragma unroll
    for (int e = 0; e < kEPL; e += 2) {
      const uint32_t pr = pack_bf16(w[e], w[e + 1]);
      if (base + e < a.n) a.wb[base + e] = static_cast<uint16_t>(pr);
      if (base + e + 1 < a.n) a.wb[base + e + 1] = static_cast<uint16_t>(pr >> 16);
    }
  }
  store_codes16_guarded(a.mq, base, a.n, mc);
  store_codes16_guarded(a.vq, base, a.n, vc);
  if (gvalid && (lane % LPG) == 0) {
    store_scale(mm, a.ms, gidx, meta.m_scale); a.mk[gidx] = meta.m_k;
    store_scale(mv, a.vs, gidx, meta.v_scale); a.vk[gidx] = meta.v_k;
  }
}

template <int G, bool GENERIC>
__global__ __launch_bounds__(kWave) void adamw_step_tail_kernel(StepArgs a) {
  constexpr int kTables = GENERIC ? 2 : 1;
  __shared__ Log2Entry lut[256 * kTables];
  fill_lut<kTables>(lut);
  const typename ModesOf<GENERIC>::M mm = ModesOf<GENERIC>::m(a), mv = ModesOf<GENERIC>::v(a);
  process_tail_chunk<G>(a, mm, mv, lut, threadIdx.x);
}

// ---------------------------------------------------------------------------------------
// Many tensors in one launch.  The plan (built once on the host, resident in device memory) holds
// one descriptor per tensor and, per 1024-element chunk of the concatenation, the index of the
// tensor it belongs to: a wavefront reads its chunk's entry, then that tensor's descriptor, and
// from there on runs exactly the single-tensor code (full chunk or a tensor's ragged last one).
// ---------------------------------------------------------------------------------------
struct TensorDesc {
  float* w; uint16_t* wb; const uint16_t* g;
  uint8_t* mq; float* ms; float* mk;
  uint8_t* vq; float* vs; float* vk;
  uint64_t n;
  uint64_t first_chunk;     // index of the tensor's first chunk in the concatenation
  float weight_decay;
  uint32_t reserved;
};
static_assert(sizeof(TensorDesc) == 96, "plan layout");

// The same record as the kernel reads it: pointers loaded from memory are generic to the compiler,
// which would cost flat_load / flat_store; typed as global memory they get the same global_load
// (scalar base + lane offset) forms as the single-tensor kernel's arguments.
#define COAT_GLOBAL_AS __attribute__((address_space(1)))
struct TensorDescDev {
  COAT_GLOBAL_AS float* w; COAT_GLOBAL_AS uint16_t* wb; COAT_GLOBAL_AS const uint16_t* g;
  COAT_GLOBAL_AS uint8_t* mq; COAT_GLOBAL_AS float* ms; COAT_GLOBAL_AS float* mk;
  COAT_GLOBAL_AS uint8_t* vq; COAT_GLOBAL_AS float* vs; COAT_GLOBAL_AS float* vk;
  uint64_t n;
  uint64_t first_chunk;
  float weight_decay;
  uint32_t reserved;
};
static_assert(sizeof(TensorDescDev) == sizeof(TensorDesc), "plan layout");

struct PlanHeader {
  uint64_t magic;
  uint32_t version, count;
  uint64_t total_chunks;
  uint64_t desc_offset, map_offset, bytes;
  uint64_t reserved[2];
};
static_assert(sizeof(PlanHeader) == 64, "plan layout");
constexpr uint64_t kPlanMagic = 0x314e4c5054414f43ull;     // "COATPLN1"

struct MultiArgs {
  StepArgs base;             // the shared hyper-parameter constants; pointers and sizes are per tensor
  const TensorDesc* descs;
  const uint32_t* chunk_tensor;
  uint64_t total_chunks;
  double neg_lr;             // -lr: the decay factor -lr * lambda is formed per tensor, in fp64 like the host does
  int32_t group_size;
};

template <int G, bool GENERIC>
__global__ __launch_bounds__(kBlock) void adamw_step_multi_kernel(MultiArgs ma) {
  constexpr int kTables = GENERIC ? 2 : 1;
  __shared__ Log2Entry lut[256 * kTables];
  __shared__ f32x4 tile_w[kWavesPerBlock * kTileSlotsW];
  __shared__ u32x4 tile_g[kWavesPerBlock * kTileSlotsG];
  const typename ModesOf<GENERIC>::M mm = ModesOf<GENERIC>::m(ma.base), mv = ModesOf<GENERIC>::v(ma.base);
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const StageTiles tiles = {tile_w + wv * kTileSlotsW, tile_g + wv * kTileSlotsG};
  // the host sizes the grid to cover every chunk
  const uint64_t gc = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv;

  StepArgs a = ma.base;
  uint64_t chunk = 0;
  // everything here is uniform over the wavefront (gc is), so the descriptor travels in scalar registers
  auto locate = [&](uint64_t c) {
    const uint32_t t = __builtin_amdgcn_readfirstlane(ma.chunk_tensor[c]);
    const TensorDescDev& d = reinterpret_cast<const TensorDescDev*>(ma.descs)[t];
    a.w = (float*)d.w; a.wb = (uint16_t*)d.wb; a.g = (const uint16_t*)d.g;
    a.mq = (uint8_t*)d.mq; a.ms = (float*)d.ms; a.mk = (float*)d.mk;
    a.vq = (uint8_t*)d.vq; a.vs = (float*)d.vs; a.vk = (float*)d.vk;
    a.n = d.n; a.n_full = d.n / kChunk;
    a.n_groups = (d.n + G - 1) / G;
    a.neg_lr_wd = static_cast<float>(ma.neg_lr * static_cast<double>(d.weight_decay));
    chunk = c - d.first_chunk;
  };

  RawChunk r;
  const bool have = gc < ma.total_chunks;
  bool full = false;
  if (have) {
    locate(gc);
    full = chunk < a.n_full;
    if (full) {
      chunk = gate_on_neighbourhood(a.mk, chunk, kChunk / G);
      issue_loads<G>(a, mm, mv, chunk, lane, r);
    }
  }
  fill_lut<kTables>(lut);                            // every wavefront of the block reaches this
  if (have) {
    if (full) process_chunk<G>(a, mm, mv, lut, tiles, chunk, lane, r);
    else process_tail_chunk<G>(a, mm, mv, lut, lane);
  }
}

// ---------------------------------------------------------------------------------------
// standalone quantizer / dequantizer (the two halves of the step), format and expansion at run time
// ---------------------------------------------------------------------------------------

// quantize one lane's 16 values (cross-lane: the group reductions) and hand back codes + metadata
template <int G>
__device__ __forceinline__ GroupQuant quant_core(const QuantArgs& a, const float (&x)[kEPL], uint32_t (&c)[4]) {
  constexpr int LPG = G / kEPL;
  float hi, lo;
  lane_extremes(x, hi, lo);
  hi = group_allreduce<LPG, true>(hi);
  lo = group_allreduce<LPG, false>(lo);
  const GroupQuant q = group_quant_params(a.mode, hi, lo, a.k_min, a.k_max, 1.0f);
  quantize16<true>(a.mode, x, q, c, 1.0f);
  return q;
}

// full chunks: coalesced streaming row loads of x staged through the LDS tile, one chunk per wavefront
template <int G>
__global__ __launch_bounds__(kBlock) void quant_kernel(QuantArgs a) {
  __shared__ f32x4 tile_x[kWavesPerBlock * kTileSlotsW];
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  for (uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv; chunk < a.n_full; chunk += stride) {
    chunk = gate_on_neighbourhood(a.x, chunk, kChunk);   // measured: 871 -> 845 us on 2^30 elements
    const uint64_t cb = chunk * kChunk, gb = chunk * (kChunk / G);
    const f32x4* xq = reinterpret_cast<const f32x4*>(a.x + cb);
    f32x4 rows[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) rows[j] = ldg<8>(xq + 64 * j + lane);
    float x[kEPL];
    uint32_t c[4];
    tile_rows_to_lanes(tile_x + wv * kTileSlotsW, lane, rows, x);
    const GroupQuant q = quant_core<G>(a, x, c);
    const u32x4 co = {c[0], c[1], c[2], c[3]};
    stg<2>(reinterpret_cast<u32x4*>(a.q + cb) + lane, co);
    if ((lane % LPG) == 0) { store_scale(a.mode, a.scale, gb + lane / LPG, q.scale); a.k[gb + lane / LPG] = q.k; }
  }
}

// the ragged last chunk: one wavefront, element-wise guarded accesses
template <int G>
__global__ __launch_bounds__(kWave) void quant_tail_kernel(QuantArgs a) {
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x;
  const uint64_t base = a.n_full * kChunk + static_cast<uint64_t>(lane) * kEPL;
  const uint64_t gidx = a.n_full * (kChunk / G) + static_cast<uint64_t>(lane / LPG);
  float x[kEPL];
  uint32_t c[4];
  load_f32x16_guarded(a.x, base, a.n, x);
  const GroupQuant q = quant_core<G>(a, x, c);
  store_codes16_guarded(a.q, base, a.n, c);
  if (gidx < a.n_groups && (lane % LPG) == 0) { store_scale(a.mode, a.scale, gidx, q.scale); a.k[gidx] = q.k; }
}

// The standalone dequantizer always honours the stored k (it is 1 for codes written without
// expansion), with the compensated exponent.
__device__ __forceinline__ void dequant_core(const DequantArgs& a, const Log2Entry* lut, const uint32_t (&c)[4],
                                             float scale, float k, float (&x)[kEPL]) {
  inverse_expand16<true, true>(lut + (a.mode.e5m2() ? 256 : 0), c, k, hw_rcp(k), x);
  const float amag = fmt_max(a.mode) * scale;
#pragma unroll
  for (int e = 0; e < kEPL; ++e) x[e] *= amag;
}

template <int G>
__global__ __launch_bounds__(kBlock) void dequant_kernel(DequantArgs a) {
  __shared__ Log2Entry lut[512];
  __shared__ f32x4 tile_x[kWavesPerBlock * kTileSlotsW];
  fill_lut<2>(lut);
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  for (uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv; chunk < a.n_full; chunk += stride) {
    const uint64_t cb = chunk * kChunk, gb = chunk * (kChunk / G);
    const u32x4 ci = ldg<1>(reinterpret_cast<const u32x4*>(a.q + cb) + lane);
    const uint32_t c[4] = {ci.x, ci.y, ci.z, ci.w};
    float x[kEPL];
    dequant_core(a, lut, c, load_scale(a.mode, a.scale, gb + lane / LPG), a.k[gb + lane / LPG], x);
    tile_lanes_to_rows_store(tile_x + wv * kTileSlotsW, lane, x, a.x + cb);
  }
}

template <int G>
__global__ __launch_bounds__(kWave) void dequant_tail_kernel(DequantArgs a) {
  __shared__ Log2Entry lut[512];
  fill_lut<2>(lut);
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x;
  const uint64_t base = a.n_full * kChunk + static_cast<uint64_t>(lane) * kEPL;
  const uint64_t gidx = a.n_full * (kChunk / G) + static_cast<uint64_t>(lane / LPG);
  const bool gvalid = gidx < a.n_groups;
  uint32_t c[4];
  float x[kEPL];
  load_codes16_guarded(a.q, base, a.n, c);
  dequant_core(a, lut, c, gvalid ? load_scale(a.mode, a.scale, gidx) : 0.0f, gvalid ? a.k[gidx] : 1.0f, x);
  store_f32x16_guarded(a.x, base, a.n, x);
}

// ---------------------------------------------------------------------------------------
// activation quantizers (Sec. 5.2): bf16 in, E4M3 codes out, no expansion.  Same lane layout as the
// optimizer kernels (16 consecutive elements per lane, rows staged through the bf16 tile), so a
// 1 x 16 group is exactly one lane and larger groups are the same DPP butterflies.
// ---------------------------------------------------------------------------------------

struct ActArgs {
  const uint16_t* x;
  uint8_t* q;
  float* per_group;        // per-group scales (1xG quantizer) or per-group maxima (Group Scaling stage 1)
  float* partial;          // Group Scaling stage 2: one partial maximum per workgroup (caller's workspace)
  int n_partial;           // how many of them the stage-2 launch writes (<= kActPartials)
  float* tensor_amax;      // max |x| of the tensor
  float* tensor_scale;
  uint64_t n, n_full, n_groups;
};

template <int G>
__device__ __forceinline__ float act_group_amax(const float (&x)[kEPL]) {
  float hi = 0.0f;
#pragma unroll
  for (int e = 0; e < kEPL; ++e) hi = __builtin_fmaxf(hi, __builtin_fabsf(x[e]));
  return group_allreduce<G / kEPL, true>(hi);
}

// codes = E4M3( fl32(x / s) ), s = fl32(amax / 448), every quotient correctly rounded.
// The sixteen quotients share the divisor, so one IEEE reciprocal r = fl(1/s) serves them all:
//   q0 = x r, e = x - s q0 (exact in an fma), q = q0 + e r
// is the correctly rounded x / s for every bf16 x and every s that comes from a bf16 maximum
// (all 2^14 significand pairs checked exhaustively on the host; the residual stays representable
// for amax >= 2^-80).  Smaller maxima take the plain division; an all-zero group keeps signed zeros.
__device__ __forceinline__ float act_quantize16(const float (&x)[kEPL], float amax, uint32_t (&c)[4]) {
  const float s = amax / 448.0f;
  if (__builtin_expect(amax >= 0x1p-80f, 1)) {
    const float r = 1.0f / s;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      float q[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const float xv = x[4 * d + b];
        const float q0 = xv * r;
        const float qc = __builtin_fmaf(__builtin_fmaf(-s, q0, xv), r, q0);
        q[b] = as_f32((as_u32(qc) & 0x7fffffffu) | (as_u32(xv) & 0x80000000u));   // -0 / s is -0 (the sum above loses it)
      }
      c[d] = pack4<false>(q);
    }
  } else {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      float q[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const float xv = x[4 * d + b];
        q[b] = s > 0.0f ? xv / s : __builtin_copysignf(0.0f, xv);
      }
      c[d] = pack4<false>(q);
    }
  }
  return s;
}

// one full chunk of bf16 rows -> the lane layout
__device__ __forceinline__ void act_load_chunk(const uint16_t* x, uint64_t cb, u32x4* tile, int lane, float (&v)[kEPL]) {
  const u32x4* xq = reinterpret_cast<const u32x4*>(x + cb);
  u32x4 rows[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) rows[j] = ldg<4>(xq + 64 * j + lane);
  tile_rows_to_lanes_bf16(tile, lane, rows, v);
}

// The end of Group Scaling's stage 2: every wavefront folds the (at most 64) per-workgroup partial
// maxima itself, one per lane; all lanes return the tensor maximum.
__device__ __forceinline__ float act_fold_partials(const ActArgs& a, int lane) {
  float hi = lane < a.n_partial ? a.partial[lane] : 0.0f;
  hi = group_allreduce<32, true>(hi);
  return __builtin_fmaxf(hi, __shfl_xor(hi, 32));
}

// PER_TENSOR = false: the 1xG quantizer (per-group scale).  PER_TENSOR = true: the last step of
// Group Scaling, every element divided by the one scale derived from the reduced maximum.
template <int G, bool PER_TENSOR>
__global__ __launch_bounds__(kBlock) void act_quant_kernel(ActArgs a) {
  __shared__ u32x4 tile_x[kWavesPerBlock * kTileSlotsG];
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  float tmax = 0.0f;
  if constexpr (PER_TENSOR) {
    tmax = act_fold_partials(a, lane);
    if (blockIdx.x == 0 && threadIdx.x == 0) { *a.tensor_amax = tmax; *a.tensor_scale = tmax / 448.0f; }
  }
  for (uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv; chunk < a.n_full; chunk += stride) {
    const uint64_t cb = chunk * kChunk;
    float x[kEPL];
    uint32_t c[4];
    act_load_chunk(a.x, cb, tile_x + wv * kTileSlotsG, lane, x);
    const float amax = PER_TENSOR ? tmax : act_group_amax<G>(x);
    const float s = act_quantize16(x, amax, c);
    const u32x4 co = {c[0], c[1], c[2], c[3]};
    stg<2>(reinterpret_cast<u32x4*>(a.q + cb) + lane, co);
    if constexpr (!PER_TENSOR)
      if ((lane % LPG) == 0) a.per_group[chunk * (kChunk / G) + lane / LPG] = s;
  }
}

template <int G, bool PER_TENSOR>
__global__ __launch_bounds__(kWave) void act_quant_tail_kernel(ActArgs a) {
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x;
  const uint64_t base = a.n_full * kChunk + static_cast<uint64_t>(lane) * kEPL;
  const uint64_t gidx = a.n_full * (kChunk / G) + static_cast<uint64_t>(lane / LPG);
  float x[kEPL];
  uint32_t c[4];
  load_bf16x16_guarded(a.x, base, a.n, x);
  float amax;
  if constexpr (PER_TENSOR) {
    amax = act_fold_partials(a, lane);
    if (lane == 0) { *a.tensor_amax = amax; *a.tensor_scale = amax / 448.0f; }
  } else {
    amax = act_group_amax<G>(x);
  }
  const float s = act_quantize16(x, amax, c);
  store_codes16_guarded(a.q, base, a.n, c);
  if constexpr (!PER_TENSOR)
    if (gidx < a.n_groups && (lane % LPG) == 0) a.per_group[gidx] = s;
}

// Group Scaling stage 1: the maximum of every 1xG group, kept as an intermediate tensor.
template <int G>
__global__ __launch_bounds__(kBlock) void act_group_amax_kernel(ActArgs a) {
  __shared__ u32x4 tile_x[kWavesPerBlock * kTileSlotsG];
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  for (uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv; chunk < a.n_full; chunk += stride) {
    float x[kEPL];
    act_load_chunk(a.x, chunk * kChunk, tile_x + wv * kTileSlotsG, lane, x);
    const float amax = act_group_amax<G>(x);
    if ((lane % LPG) == 0) a.per_group[chunk * (kChunk / G) + lane / LPG] = amax;
  }
}

template <int G>
__global__ __launch_bounds__(kWave) void act_group_amax_tail_kernel(ActArgs a) {
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x;
  const uint64_t base = a.n_full * kChunk + static_cast<uint64_t>(lane) * kEPL;
  const uint64_t gidx = a.n_full * (kChunk / G) + static_cast<uint64_t>(lane / LPG);
  float x[kEPL];
  load_bf16x16_guarded(a.x, base, a.n, x);
  const float amax = act_group_amax<G>(x);
  if (gidx < a.n_groups && (lane % LPG) == 0) a.per_group[gidx] = amax;
}

// Group Scaling stage 2: the maximum of the G-times smaller tensor of group maxima.  At most 64
// large workgroups each fold a strided share and store one partial maximum; the quantizing kernel
// that follows folds those in every wavefront.  No atomics (same-address atomic maxima serialize
// at about 11 ns each here, which cost more than the whole reduction), nothing to clear, and the
// result does not depend on the order in which workgroups finish.
template <int BLOCK, int UNROLL>
__global__ __launch_bounds__(BLOCK) void act_tensor_amax_kernel(ActArgs a) {
  __shared__ float part[BLOCK / kWave];
  const uint64_t n4 = a.n_groups / 4;
  const f32x4* p4 = reinterpret_cast<const f32x4*>(a.per_group);
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * BLOCK;
  float hi = 0.0f;
  uint64_t i = static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x;
  for (; i + (UNROLL - 1) * stride < n4; i += UNROLL * stride) {     // UNROLL independent loads in flight
    f32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = p4[i + u * stride];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      hi = __builtin_fmaxf(__builtin_fmaxf(hi, __builtin_fmaxf(v[u].x, v[u].y)), __builtin_fmaxf(v[u].z, v[u].w));
  }
  for (; i < n4; i += stride) {
    const f32x4 v = p4[i];
    hi = __builtin_fmaxf(__builtin_fmaxf(hi, __builtin_fmaxf(v.x, v.y)), __builtin_fmaxf(v.z, v.w));
  }
  if (blockIdx.x == 0 && threadIdx.x < (a.n_groups & 3)) hi = __builtin_fmaxf(hi, a.per_group[4 * n4 + threadIdx.x]);
  hi = group_allreduce<32, true>(hi);
  hi = __builtin_fmaxf(hi, __shfl_xor(hi, 32));
  if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x >> 6] = hi;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < BLOCK / kWave; ++w) hi = __builtin_fmaxf(hi, part[w]);
    a.partial[blockIdx.x] = hi;
  }
}


// ---------------------------------------------------------------------------------------
// host side: validation and launch
// ---------------------------------------------------------------------------------------

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool finite_f(float x) { return x == x && x - x == 0.0f; }
constexpr uint64_t kMaxElements = 1ull << 46;
bool group_ok(int32_t G) { return G == 32 || G == 64 || G == 128 || G == 256 || G == 512; }

#ifdef COAT_TUNING
int g_tune_cap_mult = 0;      // blocks per CU cap; 0 = one wavefront per chunk (no loop)
int g_tune_lds_pad = -1;      // dynamic LDS bytes per block (limits occupancy); -1 = the default
#endif

// Blocks of the main launch.  One chunk per wavefront measured best (the hardware dispatcher then
// walks memory in address order and few bytes are in flight per CU); the kernels still loop,
// which covers buffers with more chunks than a grid can hold blocks.
unsigned grid_for(uint64_t n_full) {
  const uint64_t need = (n_full + kWavesPerBlock - 1) / kWavesPerBlock;
  uint64_t cap = 1ull << 30;
#ifdef COAT_TUNING
  if (g_tune_cap_mult > 0) cap = 256ull * static_cast<uint64_t>(g_tune_cap_mult);
#endif
  return static_cast<unsigned>(need < cap ? need : cap);
}

// k bounds: 0,0 selects the defaults; the kernels assume 2^-6 <= k <= 2^16 (finite table
// sentinel for zero codes, no overflow of the value handed to the FP8 convert)
constexpr float kKLowest = 0.015625f, kKHighest = 65536.0f;
bool resolve_k_bounds(float& k_min, float& k_max) {
  if (!finite_f(k_min) || !finite_f(k_max)) return false;
  if (k_min == 0.0f && k_max == 0.0f) { k_min = 0.0625f; k_max = 1024.0f; }
  return k_min >= kKLowest && k_max <= kKHighest && k_min <= k_max;
}

int launch_status() { return hipGetLastError() == hipSuccess ? COAT_OK : COAT_ERR_LAUNCH; }

// The step kernel asks for this much dynamic LDS on top of its ~30 KiB of tiles and table, for no
// other purpose than to hold a CU to three resident blocks (12 wavefronts).  With fewer bytes in
// flight per CU the HBM controllers see longer same-page runs; three blocks rather than two cover
// the wait at the admission gate (measured on the 7B set, with the gate: 2 blocks 15.6 ms,
// 3 blocks 15.05, 4 blocks 15.3, 5 blocks 15.35; without it: 15.85, 16.1, 16.3, 16.3).
constexpr size_t kStepLdsPad = 16 * 1024;
constexpr size_t kMultiLdsPad = 16 * 1024;

template <int G, bool GENERIC>
int launch_step(const StepArgs& a, hipStream_t s) {
  if (a.n_full) {
    const unsigned grid = grid_for(a.n_full);
    size_t lds = kStepLdsPad;
#ifdef COAT_TUNING
    if (g_tune_lds_pad >= 0) lds = static_cast<size_t>(g_tune_lds_pad);
    if (lds > 32 * 1024)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&adamw_step_kernel<G, GENERIC>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
#endif
    hipLaunchKernelGGL((adamw_step_kernel<G, GENERIC>), dim3(grid), dim3(kBlock), lds, s, a);
    if (int rc = launch_status()) return rc;
  }
  if (a.n > a.n_full * kChunk) {
    hipLaunchKernelGGL((adamw_step_tail_kernel<G, GENERIC>), dim3(1), dim3(kWave), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  return COAT_OK;
}

template <int G>
int launch_quant(const QuantArgs& a, hipStream_t s) {
  if (a.n_full) {
    hipLaunchKernelGGL((quant_kernel<G>), dim3(grid_for(a.n_full)), dim3(kBlock), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  if (a.n > a.n_full * kChunk) {
    hipLaunchKernelGGL((quant_tail_kernel<G>), dim3(1), dim3(kWave), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  return COAT_OK;
}

template <int G>
int launch_dequant(const DequantArgs& a, hipStream_t s) {
  if (a.n_full) {
    hipLaunchKernelGGL((dequant_kernel<G>), dim3(grid_for(a.n_full)), dim3(kBlock), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  if (a.n > a.n_full * kChunk) {
    hipLaunchKernelGGL((dequant_tail_kernel<G>), dim3(1), dim3(kWave), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  return COAT_OK;
}

#define COAT_DISPATCH_G(G, CALL)            \
  switch (G) {                              \
    case 32: { constexpr int kG = 32; return CALL; }    \
    case 64: { constexpr int kG = 64; return CALL; }    \
    case 128: { constexpr int kG = 128; return CALL; }  \
    case 256: { constexpr int kG = 256; return CALL; }  \
    case 512: { constexpr int kG = 512; return CALL; }  \
  }                                         \
  return COAT_ERR_GROUP

int dispatch_step(const StepArgs& a, int32_t G, bool generic, hipStream_t s) {
  if (!generic) { COAT_DISPATCH_G(G, (launch_step<kG, false>(a, s))); }
  COAT_DISPATCH_G(G, (launch_step<kG, true>(a, s)));
}

int dispatch_quant(const QuantArgs& a, int32_t G, hipStream_t s) { COAT_DISPATCH_G(G, (launch_quant<kG>(a, s))); }

int dispatch_dequant(const DequantArgs& a, int32_t G, hipStream_t s) {
  COAT_DISPATCH_G(G, (launch_dequant<kG>(a, s)));
}

bool act_group_ok(int32_t G) { return G == 16 || group_ok(G); }

#define COAT_DISPATCH_ACT_G(G, CALL)                  \
  switch (G) {                                        \
    case 16: { constexpr int kG = 16; return CALL; }  \
  }                                                   \
  COAT_DISPATCH_G(G, CALL)

template <int G, bool PER_TENSOR>
int launch_act_quant(const ActArgs& a, hipStream_t s) {
  if (a.n_full) {
    hipLaunchKernelGGL((act_quant_kernel<G, PER_TENSOR>), dim3(grid_for(a.n_full)), dim3(kBlock), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  if (a.n > a.n_full * kChunk) {
    hipLaunchKernelGGL((act_quant_tail_kernel<G, PER_TENSOR>), dim3(1), dim3(kWave), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  return COAT_OK;
}

template <int G>
int launch_act_group_amax(const ActArgs& a, hipStream_t s) {
  if (a.n_full) {
    hipLaunchKernelGGL((act_group_amax_kernel<G>), dim3(grid_for(a.n_full)), dim3(kBlock), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  if (a.n > a.n_full * kChunk) {
    hipLaunchKernelGGL((act_group_amax_tail_kernel<G>), dim3(1), dim3(kWave), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  return COAT_OK;
}

int dispatch_act_quant_group(const ActArgs& a, int32_t G, hipStream_t s) {
  COAT_DISPATCH_ACT_G(G, (launch_act_quant<kG, false>(a, s)));
}
int dispatch_act_group_amax(const ActArgs& a, int32_t G, hipStream_t s) {
  COAT_DISPATCH_ACT_G(G, (launch_act_group_amax<kG>(a, s)));
}

// stages 2 and 3 of Group Scaling: reduce the group maxima, then quantize with the one scale
constexpr int kStage2Block = 1024, kStage2Unroll = 4, kStage2MaxGrid = COAT_ACT_WORKSPACE_FLOATS;
static_assert(kStage2MaxGrid <= kWave, "one partial maximum per lane");
int launch_act_tensor_rest(ActArgs a, hipStream_t s) {
  const uint64_t need = (a.n_groups / 4 + kStage2Block * kStage2Unroll - 1) / (kStage2Block * kStage2Unroll);
  const unsigned grid = static_cast<unsigned>(need < 1 ? 1 : (need > kStage2MaxGrid ? kStage2MaxGrid : need));
  a.n_partial = static_cast<int>(grid);
  hipLaunchKernelGGL((act_tensor_amax_kernel<kStage2Block, kStage2Unroll>), dim3(grid), dim3(kStage2Block), 0, s, a);
  if (int rc = launch_status()) return rc;
  return launch_act_quant<16, true>(a, s);   // the group size plays no part once the scale is per tensor
}

int act_quant_tensor_impl(const uint16_t* x, uint64_t n, int32_t G, float* group_amax, bool have_group_amax,
                          float* workspace, float* tensor_amax, float* tensor_scale, uint8_t* q, void* hip_stream) {
  if (!act_group_ok(G)) return COAT_ERR_GROUP;
  if (n == 0) return COAT_OK;
  if (!x || !q || !group_amax || !workspace || !tensor_amax || !tensor_scale) return COAT_ERR_NULL;
  if (!aligned16(x) || !aligned16(q) || !aligned16(group_amax) || !aligned16(workspace)) return COAT_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(tensor_amax) | reinterpret_cast<uintptr_t>(tensor_scale)) & 3u) return COAT_ERR_ALIGN;
  if (n > kMaxElements) return COAT_ERR_SIZE;
  ActArgs a;
  a.x = x; a.q = q; a.per_group = group_amax;
  a.partial = workspace; a.n_partial = 0; a.tensor_amax = tensor_amax; a.tensor_scale = tensor_scale;
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(G) - 1) / static_cast<uint64_t>(G);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (!have_group_amax)
    if (int rc = dispatch_act_group_amax(a, G, s)) return rc;
  return launch_act_tensor_rest(a, s);
}

template <int G, bool GENERIC>
int launch_step_multi(const MultiArgs& ma, hipStream_t s) {
  const uint64_t blocks = (ma.total_chunks + kWavesPerBlock - 1) / kWavesPerBlock;
  size_t lds = kMultiLdsPad;
#ifdef COAT_TUNING
  if (g_tune_lds_pad >= 0) lds = static_cast<size_t>(g_tune_lds_pad);
#endif
  hipLaunchKernelGGL((adamw_step_multi_kernel<G, GENERIC>), dim3(static_cast<unsigned>(blocks)), dim3(kBlock), lds, s, ma);
  return launch_status();
}

int dispatch_step_multi(const MultiArgs& ma, int32_t G, bool generic, hipStream_t s) {
  if (!generic) { COAT_DISPATCH_G(G, (launch_step_multi<kG, false>(ma, s))); }
  COAT_DISPATCH_G(G, (launch_step_multi<kG, true>(ma, s)));
}

constexpr uint32_t kStepFlags = COAT_FLAG_EXPAND | COAT_FLAG_M_E5M2 | COAT_FLAG_V_E5M2 | COAT_FLAG_M_PLAIN |
                                COAT_FLAG_V_PLAIN | COAT_FLAG_BF16_SCALE;

constexpr uint64_t kMaxPlanChunks = 1ull << 32;     // one launch covers them all (4 per workgroup)

size_t plan_map_offset(uint32_t count) {
  return sizeof(PlanHeader) + ((static_cast<size_t>(count) * sizeof(TensorDesc) + 63) / 64) * 64;
}

// Validates the hyper-parameters and fills every field of StepArgs that does not depend on the
// tensor (the pointers, sizes and the decay factor are set by the caller).
int step_constants(const coat_adamw_hparams* hp, StepArgs& a, bool& generic) {
  if (!hp) return COAT_ERR_NULL;
  if (!group_ok(hp->group_size)) return COAT_ERR_GROUP;
  if (hp->step < 1) return COAT_ERR_STEP;
  if (!finite_f(hp->lr) || !finite_f(hp->beta1) || !finite_f(hp->beta2) || !finite_f(hp->eps) ||
      !finite_f(hp->weight_decay))
    return COAT_ERR_HPARAM;
  if (hp->lr < 0.0f || hp->beta1 < 0.0f || hp->beta1 >= 1.0f || hp->beta2 < 0.0f || hp->beta2 >= 1.0f ||
      hp->eps < 0.0f)
    return COAT_ERR_HPARAM;
  if (hp->flags & ~kStepFlags) return COAT_ERR_HPARAM;
  float k_min = hp->k_min, k_max = hp->k_max;
  if (!resolve_k_bounds(k_min, k_max)) return COAT_ERR_HPARAM;

  // bias corrections in fp64 on the host (Sec. 3: 1 - beta^t)
  const double b1 = hp->beta1, b2 = hp->beta2;
  double p1 = 1.0, p2 = 1.0;
  {
    double x1 = b1, x2 = b2;
    for (uint32_t e = static_cast<uint32_t>(hp->step); e; e >>= 1) {
      if (e & 1u) { p1 *= x1; p2 *= x2; }
      x1 *= x1; x2 *= x2;
    }
  }
  const double bc1 = 1.0 - p1, bc2 = 1.0 - p2;
  if (!(bc1 > 0.0) || !(bc2 > 0.0)) return COAT_ERR_HPARAM;   // beta == 0 gives bc == 1, fine

  a.one_minus_beta1 = 1.0f - hp->beta1;               // exact (Sterbenz) for beta >= 0.5
  a.one_minus_beta2 = 1.0f - hp->beta2;
  const double omb1 = a.one_minus_beta1, omb2 = a.one_minus_beta2;
  a.beta1_ratio = static_cast<float>(b1 / omb1);
  a.beta2_ratio = static_cast<float>(b2 / omb2);
  a.neg_lr_m = static_cast<float>(-static_cast<double>(hp->lr) * omb1 / bc1);
  a.denom_scale = static_cast<float>(__builtin_sqrt(omb2 / bc2));
  a.eps = hp->eps;
  a.k_min = k_min; a.k_max = k_max;
  const bool expand = (hp->flags & COAT_FLAG_EXPAND) != 0;
  a.mode_m.e5 = (hp->flags & COAT_FLAG_M_E5M2) != 0;
  a.mode_v.e5 = (hp->flags & COAT_FLAG_V_E5M2) != 0;
  a.mode_m.ex = expand && !(hp->flags & COAT_FLAG_M_PLAIN);
  a.mode_v.ex = expand && !(hp->flags & COAT_FLAG_V_PLAIN);
  a.mode_m.s16 = a.mode_v.s16 = (hp->flags & COAT_FLAG_BF16_SCALE) != 0;
  generic = a.mode_m.e5 || a.mode_v.e5 || !a.mode_m.ex || !a.mode_v.ex || a.mode_m.s16;
  return COAT_OK;
}

}  // namespace

extern "C" {

int coat_fp8_adamw_step(float* w, const uint16_t* grad_bf16, uint8_t* m_q, void* m_scale, float* m_k,
                        uint8_t* v_q, void* v_scale, float* v_k, uint64_t n,
                        const coat_adamw_hparams* hp, void* hip_stream) {
  return coat_fp8_adamw_step_bf16w(w, nullptr, grad_bf16, m_q, m_scale, m_k, v_q, v_scale, v_k, n, hp, hip_stream);
}

int coat_fp8_adamw_step_bf16w(float* w, uint16_t* w_bf16, const uint16_t* grad_bf16, uint8_t* m_q,
                              void* m_scale, float* m_k, uint8_t* v_q, void* v_scale, float* v_k,
                              uint64_t n, const coat_adamw_hparams* hp, void* hip_stream) {
  StepArgs a;
  bool generic = false;
  if (int rc = step_constants(hp, a, generic)) return rc;
  if (n == 0) return COAT_OK;
  if (!w || !grad_bf16 || !m_q || !m_scale || !m_k || !v_q || !v_scale || !v_k) return COAT_ERR_NULL;
  if (!aligned16(w) || !aligned16(grad_bf16) || !aligned16(m_q) || !aligned16(v_q) ||
      !aligned16(m_scale) || !aligned16(m_k) || !aligned16(v_scale) || !aligned16(v_k) || !aligned16(w_bf16))
    return COAT_ERR_ALIGN;
  if (n > kMaxElements) return COAT_ERR_SIZE;
  a.w = w; a.wb = w_bf16; a.g = grad_bf16; a.mq = m_q; a.ms = static_cast<float*>(m_scale); a.mk = m_k; a.vq = v_q; a.vs = static_cast<float*>(v_scale); a.vk = v_k;
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(hp->group_size) - 1) / static_cast<uint64_t>(hp->group_size);
  a.neg_lr_wd = static_cast<float>(-static_cast<double>(hp->lr) * static_cast<double>(hp->weight_decay));
  return dispatch_step(a, hp->group_size, generic, static_cast<hipStream_t>(hip_stream));
}

size_t coat_multi_plan_bytes(const coat_tensor_desc* descs, uint32_t count) {
  if (count && !descs) return 0;
  uint64_t chunks = 0;
  for (uint32_t t = 0; t < count; ++t) {
    if (descs[t].n > kMaxElements) return 0;
    chunks += (descs[t].n + kChunk - 1) / kChunk;
  }
  if (chunks > kMaxPlanChunks) return 0;
  return plan_map_offset(count) + static_cast<size_t>(chunks) * sizeof(uint32_t);
}

int coat_multi_plan_build(const coat_tensor_desc* descs, uint32_t count, void* plan_host, size_t plan_bytes) {
  if (!plan_host || (count && !descs)) return COAT_ERR_NULL;
  const size_t need = coat_multi_plan_bytes(descs, count);
  if (need == 0 || plan_bytes < need) return COAT_ERR_SIZE;
  for (uint32_t t = 0; t < count; ++t) {
    const coat_tensor_desc& d = descs[t];
    if (d.n == 0) continue;
    if (!d.w || !d.grad_bf16 || !d.m_q || !d.m_scale || !d.m_k || !d.v_q || !d.v_scale || !d.v_k) return COAT_ERR_NULL;
    if (!aligned16(d.w) || !aligned16(d.grad_bf16) || !aligned16(d.m_q) || !aligned16(d.v_q) || !aligned16(d.m_scale) ||
        !aligned16(d.m_k) || !aligned16(d.v_scale) || !aligned16(d.v_k) || !aligned16(d.w_bf16))
      return COAT_ERR_ALIGN;
    if (!finite_f(d.weight_decay)) return COAT_ERR_HPARAM;
  }
  unsigned char* blob = static_cast<unsigned char*>(plan_host);
  PlanHeader h = {};
  h.magic = kPlanMagic; h.version = 1; h.count = count;
  h.desc_offset = sizeof(PlanHeader); h.map_offset = plan_map_offset(count); h.bytes = need;
  TensorDesc* dd = reinterpret_cast<TensorDesc*>(blob + h.desc_offset);
  uint32_t* map = reinterpret_cast<uint32_t*>(blob + h.map_offset);
  uint64_t chunk = 0;
  for (uint32_t t = 0; t < count; ++t) {
    const coat_tensor_desc& d = descs[t];
    TensorDesc o = {};
    o.w = d.w; o.wb = d.w_bf16; o.g = d.grad_bf16; o.mq = d.m_q; o.ms = static_cast<float*>(d.m_scale); o.mk = d.m_k;
    o.vq = d.v_q; o.vs = static_cast<float*>(d.v_scale); o.vk = d.v_k; o.n = d.n; o.first_chunk = chunk; o.weight_decay = d.weight_decay;
    __builtin_memcpy(dd + t, &o, sizeof o);
    const uint64_t c = (d.n + kChunk - 1) / kChunk;
    for (uint64_t i = 0; i < c; ++i) map[chunk + i] = t;
    chunk += c;
  }
  h.total_chunks = chunk;
  __builtin_memcpy(blob, &h, sizeof h);
  return COAT_OK;
}

int coat_fp8_adamw_step_multi(const void* plan_host, const void* plan_device, const coat_adamw_hparams* hp,
                              void* hip_stream) {
  MultiArgs ma;
  bool generic = false;
  if (int rc = step_constants(hp, ma.base, generic)) return rc;
  if (!plan_host) return COAT_ERR_NULL;
  PlanHeader h;
  __builtin_memcpy(&h, plan_host, sizeof h);
  if (h.magic != kPlanMagic || h.version != 1 || h.desc_offset != sizeof(PlanHeader) ||
      h.map_offset != plan_map_offset(h.count) || h.total_chunks > kMaxPlanChunks)
    return COAT_ERR_PLAN;
  if (h.total_chunks == 0) return COAT_OK;
  if (!plan_device) return COAT_ERR_NULL;
  if (!aligned16(plan_device)) return COAT_ERR_ALIGN;
  const unsigned char* dev = static_cast<const unsigned char*>(plan_device);
  ma.base.w = nullptr; ma.base.wb = nullptr; ma.base.g = nullptr; ma.base.mq = nullptr; ma.base.ms = nullptr;
  ma.base.mk = nullptr; ma.base.vq = nullptr; ma.base.vs = nullptr; ma.base.vk = nullptr;
  ma.base.n = 0; ma.base.n_full = 0; ma.base.n_groups = 0; ma.base.neg_lr_wd = 0.0f;
  ma.descs = reinterpret_cast<const TensorDesc*>(dev + h.desc_offset);
  ma.chunk_tensor = reinterpret_cast<const uint32_t*>(dev + h.map_offset);
  ma.total_chunks = h.total_chunks;
  ma.neg_lr = -static_cast<double>(hp->lr);
  ma.group_size = hp->group_size;
  return dispatch_step_multi(ma, hp->group_size, generic, static_cast<hipStream_t>(hip_stream));
}

int coat_shard_range(uint64_t n, int32_t G, uint32_t rank, uint32_t world, uint64_t* begin, uint64_t* end) {
  if (!begin || !end) return COAT_ERR_NULL;
  if (G < 1) return COAT_ERR_GROUP;
  if (world == 0 || rank >= world) return COAT_ERR_HPARAM;
  const uint64_t g = static_cast<uint64_t>(G);
  const uint64_t groups = n / g + (n % g != 0);
  const uint64_t base = groups / world, extra = groups % world;           // the first `extra` ranks own one more
  const uint64_t g0 = rank * base + (rank < extra ? rank : extra);
  const uint64_t g1 = g0 + base + (rank < extra ? 1 : 0);
  *begin = g0 * g < n ? g0 * g : n;
  *end = g1 * g < n ? g1 * g : n;
  return COAT_OK;
}

int coat_quant_group(const float* x, uint64_t n, int32_t G, uint32_t flags, float k_min, float k_max,
                     uint8_t* q, void* scale, float* k, void* hip_stream) {
  if (!group_ok(G)) return COAT_ERR_GROUP;
  if (flags & ~(COAT_FLAG_EXPAND | COAT_FLAG_E5M2 | COAT_FLAG_BF16_SCALE)) return COAT_ERR_HPARAM;
  if (!resolve_k_bounds(k_min, k_max)) return COAT_ERR_HPARAM;
  if (n == 0) return COAT_OK;
  if (!x || !q || !scale || !k) return COAT_ERR_NULL;
  if (!aligned16(x) || !aligned16(q) || !aligned16(scale) || !aligned16(k)) return COAT_ERR_ALIGN;
  if (n > kMaxElements) return COAT_ERR_SIZE;
  QuantArgs a;
  a.x = x; a.q = q; a.scale = static_cast<float*>(scale); a.k = k;
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(G) - 1) / static_cast<uint64_t>(G);
  a.k_min = k_min; a.k_max = k_max;
  a.mode.ex = (flags & COAT_FLAG_EXPAND) != 0;
  a.mode.e5 = (flags & COAT_FLAG_E5M2) != 0;
  a.mode.s16 = (flags & COAT_FLAG_BF16_SCALE) != 0;
  return dispatch_quant(a, G, static_cast<hipStream_t>(hip_stream));
}

int coat_dequant_group(const uint8_t* q, const void* scale, const float* k, uint64_t n, int32_t G,
                       uint32_t flags, float* x, void* hip_stream) {
  if (!group_ok(G)) return COAT_ERR_GROUP;
  if (flags & ~(COAT_FLAG_EXPAND | COAT_FLAG_E5M2 | COAT_FLAG_BF16_SCALE)) return COAT_ERR_HPARAM;
  if (n == 0) return COAT_OK;
  if (!x || !q || !scale || !k) return COAT_ERR_NULL;
  if (!aligned16(x) || !aligned16(q) || !aligned16(scale) || !aligned16(k)) return COAT_ERR_ALIGN;
  if (n > kMaxElements) return COAT_ERR_SIZE;
  DequantArgs a;
  a.q = q; a.scale = static_cast<const float*>(scale); a.k = k; a.x = x;
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(G) - 1) / static_cast<uint64_t>(G);
  a.mode.ex = true;
  a.mode.e5 = (flags & COAT_FLAG_E5M2) != 0;
  a.mode.s16 = (flags & COAT_FLAG_BF16_SCALE) != 0;
  return dispatch_dequant(a, G, static_cast<hipStream_t>(hip_stream));
}

int coat_act_quant_group(const uint16_t* x_bf16, uint64_t n, int32_t G, uint8_t* q, float* scale,
                         void* hip_stream) {
  if (!act_group_ok(G)) return COAT_ERR_GROUP;
  if (n == 0) return COAT_OK;
  if (!x_bf16 || !q || !scale) return COAT_ERR_NULL;
  if (!aligned16(x_bf16) || !aligned16(q) || !aligned16(scale)) return COAT_ERR_ALIGN;
  if (n > kMaxElements) return COAT_ERR_SIZE;
  ActArgs a;
  a.x = x_bf16; a.q = q; a.per_group = scale; a.partial = nullptr; a.n_partial = 0; a.tensor_amax = nullptr; a.tensor_scale = nullptr;
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(G) - 1) / static_cast<uint64_t>(G);
  return dispatch_act_quant_group(a, G, static_cast<hipStream_t>(hip_stream));
}

int coat_act_quant_tensor(const uint16_t* x_bf16, uint64_t n, int32_t G, float* group_amax, float* workspace,
                          float* tensor_amax, float* tensor_scale, uint8_t* q, void* hip_stream) {
  return act_quant_tensor_impl(x_bf16, n, G, group_amax, false, workspace, tensor_amax, tensor_scale, q, hip_stream);
}

int coat_act_quant_tensor_from_group_amax(const uint16_t* x_bf16, uint64_t n, int32_t G,
                                          const float* group_amax, float* workspace, float* tensor_amax,
                                          float* tensor_scale, uint8_t* q, void* hip_stream) {
  return act_quant_tensor_impl(x_bf16, n, G, const_cast<float*>(group_amax), true, workspace, tensor_amax,
                               tensor_scale, q, hip_stream);
}

const char* coat_strerror(int code) {
  switch (code) {
    case COAT_OK: return "ok";
    case COAT_ERR_NULL: return "a required pointer is NULL";
    case COAT_ERR_ALIGN: return "a base pointer is not 16-byte aligned";
    case COAT_ERR_GROUP: return "group size must be one of 32, 64, 128, 256, 512 (activation quantizers: also 16)";
    case COAT_ERR_STEP: return "step must be >= 1";
    case COAT_ERR_HPARAM: return "hyper-parameter or flag is non-finite, unsupported or out of its domain";
    case COAT_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    case COAT_ERR_SIZE: return "n is too large, or the plan buffer is too small";
    case COAT_ERR_PLAN: return "the plan blob is not one that coat_multi_plan_build wrote";
  }
  return "unknown error code";
}

int coat_version(void) { return 220; }

#ifdef COAT_TUNING
// development builds only: launch-shape knobs for sweeps
void coat_tune_set(int cap_mult, int lds_pad, int unused) {
  g_tune_cap_mult = cap_mult; g_tune_lds_pad = lds_pad; (void)unused;
}
#endif

}  // extern "C"
