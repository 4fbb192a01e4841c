// coat_kernels.hip -- gfx950 kernels and C ABI of the FP8-state AdamW step of COAT
// (arxiv 2410.19313: Sec. 3 quantizer and update rule, Sec. 4.2 dynamic range expansion,
// Appendix A step order).  Hand-written for CDNA4: 64-wide wavefronts, every lane owns 16
// consecutive elements (16-byte loads of the code bytes, 32 B of bf16 gradient, 64 B of fp32
// weight), a quantization group of G elements is G/16 adjacent lanes and its max/min are
// DPP butterflies inside the wavefront.  No LDS traffic except a 1 KiB lookup table, no
// atomics, no inter-wave communication: each group is owned by exactly one wavefront.
//
// Arithmetic layout (fp32 throughout; transcendental ops are the hardware log2/exp2):
//   inverse expansion  |c/448|^(1/k) = exp2( log2|c/448| * (1/k) ), log2|c/448| from a table
//                      of the 127 code magnitudes;
//   expansion          448 * (|x|/a)^k = 448 * exp2( k * log2(|x| * (1/a)) ), the logarithm
//                      is taken of the RATIO so that its magnitude stays below 17.81;
//   conversion         native fp32 -> OCP E4M3 pack instruction (round to nearest even).
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

constexpr float kE4M3Max = 448.0f;
constexpr float kLog2Range = 17.807354922057606f;   // log2(448 * 512), Sec. 4.1
constexpr float kLog2E4M3Max = 8.807354922057604f;  // log2(448)

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// log2(|decode(c)| / 448) for the 128 magnitude codes of OCP E4M3 as an unevaluated sum
// hi + lo of two fp32 numbers (hi = the fp32 nearest to the logarithm, lo = what is left).
// Code 0 is zero: a huge negative finite logarithm makes exp2 return exactly 0 for every
// admissible exponent k while keeping the correction terms finite.  Code 0x7F is NaN.
struct Log2Entry { float hi, lo; };
__device__ const Log2Entry kLog2CodeOverMax[128] = {
    {-1.0e30f, 0.0f}, {-0x1.1ceaecp+4f, -0x1.fd501p-21f},
    {-0x1.0ceaecp+4f, -0x1.fd501p-21f}, {-0x1.038eecp+4f, 0x1.49ef6ap-21f},
    {-0x1.f9d5dap+3f, 0x1.57f7a6p-28f}, {-0x1.ef889ep+3f, 0x1.44b3e8p-24f},
    {-0x1.e71dd6p+3f, -0x1.6c212cp-22f}, {-0x1.ep+3f, 0x0.0p+0f},
    {-0x1.d9d5dap+3f, 0x1.57f7a6p-28f}, {-0x1.d465d4p+3f, 0x1.225dcap-22f},
    {-0x1.cf889ep+3f, 0x1.44b3e8p-24f}, {-0x1.cb223p+3f, -0x1.a6d376p-26f},
    {-0x1.c71dd6p+3f, -0x1.6c212cp-22f}, {-0x1.c36bdap+3f, 0x1.21eefp-22f},
    {-0x1.cp+3f, 0x0.0p+0f}, {-0x1.bcd09ap+3f, -0x1.20541p-22f},
    {-0x1.b9d5dap+3f, 0x1.57f7a6p-28f}, {-0x1.b465d4p+3f, 0x1.225dcap-22f},
    {-0x1.af889ep+3f, 0x1.44b3e8p-24f}, {-0x1.ab223p+3f, -0x1.a6d376p-26f},
    {-0x1.a71dd6p+3f, -0x1.6c212cp-22f}, {-0x1.a36bdap+3f, 0x1.21eefp-22f},
    {-0x1.ap+3f, 0x0.0p+0f}, {-0x1.9cd09ap+3f, -0x1.20541p-22f},
    {-0x1.99d5dap+3f, 0x1.57f7a6p-28f}, {-0x1.9465d4p+3f, 0x1.225dcap-22f},
    {-0x1.8f889ep+3f, 0x1.44b3e8p-24f}, {-0x1.8b223p+3f, -0x1.a6d376p-26f},
    {-0x1.871dd6p+3f, -0x1.6c212cp-22f}, {-0x1.836bdap+3f, 0x1.21eefp-22f},
    {-0x1.8p+3f, 0x0.0p+0f}, {-0x1.7cd09ap+3f, -0x1.20541p-22f},
    {-0x1.79d5dap+3f, 0x1.57f7a6p-28f}, {-0x1.7465d4p+3f, 0x1.225dcap-22f},
    {-0x1.6f889ep+3f, 0x1.44b3e8p-24f}, {-0x1.6b223p+3f, -0x1.a6d376p-26f},
    {-0x1.671dd6p+3f, -0x1.6c212cp-22f}, {-0x1.636bdap+3f, 0x1.21eefp-22f},
    {-0x1.6p+3f, 0x0.0p+0f}, {-0x1.5cd09ap+3f, -0x1.20541p-22f},
    {-0x1.59d5dap+3f, 0x1.57f7a6p-28f}, {-0x1.5465d4p+3f, 0x1.225dcap-22f},
    {-0x1.4f889ep+3f, 0x1.44b3e8p-24f}, {-0x1.4b223p+3f, -0x1.a6d376p-26f},
    {-0x1.471dd6p+3f, -0x1.6c212cp-22f}, {-0x1.436bdap+3f, 0x1.21eefp-22f},
    {-0x1.4p+3f, 0x0.0p+0f}, {-0x1.3cd09ap+3f, -0x1.20541p-22f},
    {-0x1.39d5dap+3f, 0x1.57f7a6p-28f}, {-0x1.3465d4p+3f, 0x1.225dcap-22f},
    {-0x1.2f889ep+3f, 0x1.44b3e8p-24f}, {-0x1.2b223p+3f, -0x1.a6d376p-26f},
    {-0x1.271dd6p+3f, -0x1.6c212cp-22f}, {-0x1.236bdap+3f, 0x1.21eefp-22f},
    {-0x1.2p+3f, 0x0.0p+0f}, {-0x1.1cd09ap+3f, -0x1.20541p-22f},
    {-0x1.19d5dap+3f, 0x1.57f7a6p-28f}, {-0x1.1465d4p+3f, 0x1.225dcap-22f},
    {-0x1.0f889ep+3f, 0x1.44b3e8p-24f}, {-0x1.0b223p+3f, -0x1.a6d376p-26f},
    {-0x1.071dd6p+3f, -0x1.6c212cp-22f}, {-0x1.036bdap+3f, 0x1.21eefp-22f},
    {-0x1.0p+3f, 0x0.0p+0f}, {-0x1.f9a136p+2f, 0x1.bf57ep-23f},
    {-0x1.f3abb4p+2f, 0x1.57f7a6p-28f}, {-0x1.e8cba6p+2f, -0x1.bb446cp-23f},
    {-0x1.df113cp+2f, 0x1.44b3e8p-24f}, {-0x1.d6446p+2f, -0x1.a6d376p-26f},
    {-0x1.ce3baep+2f, 0x1.27bda8p-23f}, {-0x1.c6d7b2p+2f, -0x1.bc222p-23f},
    {-0x1.cp+2f, 0x0.0p+0f}, {-0x1.b9a136p+2f, 0x1.bf57ep-23f},
    {-0x1.b3abb4p+2f, 0x1.57f7a6p-28f}, {-0x1.a8cba6p+2f, -0x1.bb446cp-23f},
    {-0x1.9f113cp+2f, 0x1.44b3e8p-24f}, {-0x1.96446p+2f, -0x1.a6d376p-26f},
    {-0x1.8e3baep+2f, 0x1.27bda8p-23f}, {-0x1.86d7b2p+2f, -0x1.bc222p-23f},
    {-0x1.8p+2f, 0x0.0p+0f}, {-0x1.79a136p+2f, 0x1.bf57ep-23f},
    {-0x1.73abb4p+2f, 0x1.57f7a6p-28f}, {-0x1.68cba6p+2f, -0x1.bb446cp-23f},
    {-0x1.5f113cp+2f, 0x1.44b3e8p-24f}, {-0x1.56446p+2f, -0x1.a6d376p-26f},
    {-0x1.4e3baep+2f, 0x1.27bda8p-23f}, {-0x1.46d7b2p+2f, -0x1.bc222p-23f},
    {-0x1.4p+2f, 0x0.0p+0f}, {-0x1.39a136p+2f, 0x1.bf57ep-23f},
    {-0x1.33abb4p+2f, 0x1.57f7a6p-28f}, {-0x1.28cba6p+2f, -0x1.bb446cp-23f},
    {-0x1.1f113cp+2f, 0x1.44b3e8p-24f}, {-0x1.16446p+2f, -0x1.a6d376p-26f},
    {-0x1.0e3baep+2f, 0x1.27bda8p-23f}, {-0x1.06d7b2p+2f, -0x1.bc222p-23f},
    {-0x1.0p+2f, 0x0.0p+0f}, {-0x1.f3426ap+1f, -0x1.02a082p-25f},
    {-0x1.e75768p+1f, 0x1.57f7a6p-28f}, {-0x1.d1974ep+1f, 0x1.12ee4ep-25f},
    {-0x1.be2278p+1f, 0x1.44b3e8p-24f}, {-0x1.ac88cp+1f, -0x1.a6d376p-26f},
    {-0x1.9c775ap+1f, -0x1.b084bp-24f}, {-0x1.8daf66p+1f, 0x1.0f7782p-25f},
    {-0x1.8p+1f, 0x0.0p+0f}, {-0x1.73426ap+1f, -0x1.02a082p-25f},
    {-0x1.675768p+1f, 0x1.57f7a6p-28f}, {-0x1.51974ep+1f, 0x1.12ee4ep-25f},
    {-0x1.3e2278p+1f, 0x1.44b3e8p-24f}, {-0x1.2c88cp+1f, -0x1.a6d376p-26f},
    {-0x1.1c775ap+1f, -0x1.b084bp-24f}, {-0x1.0daf66p+1f, 0x1.0f7782p-25f},
    {-0x1.0p+1f, 0x0.0p+0f}, {-0x1.e684d4p+0f, -0x1.02a082p-25f},
    {-0x1.ceaedp+0f, 0x1.57f7a6p-28f}, {-0x1.a32e9cp+0f, 0x1.12ee4ep-25f},
    {-0x1.7c44eep+0f, -0x1.76982ep-25f}, {-0x1.59118p+0f, -0x1.a6d376p-26f},
    {-0x1.38eeb6p+0f, 0x1.3ded44p-26f}, {-0x1.1b5eccp+0f, 0x1.0f7782p-25f},
    {-0x1.0p+0f, 0x0.0p+0f}, {-0x1.cd09aap-1f, 0x1.fabefcp-26f},
    {-0x1.9d5dap-1f, 0x1.57f7a6p-28f}, {-0x1.465d36p-1f, -0x1.da2362p-26f},
    {-0x1.f113bap-2f, -0x1.da60bcp-27f}, {-0x1.644602p-2f, 0x1.64b22ap-28f},
    {-0x1.c775aep-3f, 0x1.ef6a1ep-29f}, {-0x1.b5ecb8p-4f, 0x1.eef03p-30f},
    {0x0.0p+0f, 0x0.0p+0f}, {__builtin_nanf(""), 0.0f},
};

struct StepArgs {
  float* w;
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
  uint32_t expand;
};

struct QuantArgs {
  const float* x; uint8_t* q; float* scale; float* k;
  uint64_t n, n_full, n_groups;
  float k_min, k_max;
  uint32_t expand;
};

struct DequantArgs {
  const uint8_t* q; const float* scale; const float* k; float* x;
  uint64_t n, n_full, n_groups;
};

// ---------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

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
// 8 load weights, 16 store weights.  A set bit issues the access as non-temporal.
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

template <bool GUARD>
__device__ __forceinline__ void load_f32x16(const float* p, uint64_t base, uint64_t n, float (&x)[kEPL]) {
  if constexpr (!GUARD) {
    const f32x4* q = reinterpret_cast<const f32x4*>(p + base);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      f32x4 t = ldg<8>(q + j);
      x[4 * j + 0] = t.x; x[4 * j + 1] = t.y; x[4 * j + 2] = t.z; x[4 * j + 3] = t.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < kEPL; ++e) x[e] = (base + e < n) ? p[base + e] : 0.0f;
  }
}

template <bool GUARD>
__device__ __forceinline__ void store_f32x16(float* p, uint64_t base, uint64_t n, const float (&x)[kEPL]) {
  if constexpr (!GUARD) {
    f32x4* q = reinterpret_cast<f32x4*>(p + base);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      f32x4 t = {x[4 * j + 0], x[4 * j + 1], x[4 * j + 2], x[4 * j + 3]};
      stg<16>(q + j, t);
    }
  } else {
#pragma unroll
    for (int e = 0; e < kEPL; ++e)
      if (base + e < n) p[base + e] = x[e];
  }
}

// 16 bf16 gradients -> fp32 (a bf16 is the upper half of an fp32)
template <bool GUARD>
__device__ __forceinline__ void load_bf16x16(const uint16_t* p, uint64_t base, uint64_t n, float (&x)[kEPL]) {
  if constexpr (!GUARD) {
    const u32x4* q = reinterpret_cast<const u32x4*>(p + base);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      u32x4 t = ldg<4>(q + j);
      x[8 * j + 0] = as_f32(t.x << 16); x[8 * j + 1] = as_f32(t.x & 0xffff0000u);
      x[8 * j + 2] = as_f32(t.y << 16); x[8 * j + 3] = as_f32(t.y & 0xffff0000u);
      x[8 * j + 4] = as_f32(t.z << 16); x[8 * j + 5] = as_f32(t.z & 0xffff0000u);
      x[8 * j + 6] = as_f32(t.w << 16); x[8 * j + 7] = as_f32(t.w & 0xffff0000u);
    }
  } else {
#pragma unroll
    for (int e = 0; e < kEPL; ++e)
      x[e] = (base + e < n) ? as_f32(static_cast<uint32_t>(p[base + e]) << 16) : 0.0f;
  }
}

// 16 code bytes as four dwords, element e in byte (e & 3) of dword (e >> 2)
template <bool GUARD>
__device__ __forceinline__ void load_codes16(const uint8_t* p, uint64_t base, uint64_t n, uint32_t (&c)[4]) {
  if constexpr (!GUARD) {
    u32x4 t = ldg<1>(reinterpret_cast<const u32x4*>(p + base));
    c[0] = t.x; c[1] = t.y; c[2] = t.z; c[3] = t.w;
  } else {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      uint32_t v = 0;
#pragma unroll
      for (int b = 0; b < 4; ++b)
        if (base + 4 * d + b < n) v |= static_cast<uint32_t>(p[base + 4 * d + b]) << (8 * b);
      c[d] = v;
    }
  }
}

template <bool GUARD>
__device__ __forceinline__ void store_codes16(uint8_t* p, uint64_t base, uint64_t n, const uint32_t (&c)[4]) {
  if constexpr (!GUARD) {
    u32x4 t = {c[0], c[1], c[2], c[3]};
    stg<2>(reinterpret_cast<u32x4*>(p + base), t);
  } else {
#pragma unroll
    for (int e = 0; e < kEPL; ++e)
      if (base + e < n) p[base + e] = static_cast<uint8_t>(c[e >> 2] >> (8 * (e & 3)));
  }
}

// ---------------------------------------------------------------------------------------
// LDS staging: HBM likes every load/store instruction of a wavefront to cover one contiguous
// span (and to be issued as a streaming access), the arithmetic wants every lane to own 16
// consecutive elements.  A 4 KiB (fp32) / 2 KiB (bf16) per-wavefront LDS tile converts between
// the two: rows of 64 x 16 B on the memory side, 64 B (32 B) per lane on the register side.
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
  f32x4* const row = tile + lane + (lane >> 3);          // + 72 j
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
template <int NT_BIT>
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
  for (int j = 0; j < 4; ++j) stg<NT_BIT>(q + 64 * j + lane, row[72 * j]);
}

__device__ __forceinline__ void fill_lut(Log2Entry* lut) {
  // 256 entries so that the whole code byte indexes it (the sign bit is ignored)
  for (int i = threadIdx.x; i < 256; i += blockDim.x) lut[i] = kLog2CodeOverMax[i & 127];
  __syncthreads();
}

constexpr float kLn2 = 0.6931471805599453f;

// |c/448|^(1/k) for 16 codes.
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
template <bool SIGNED>
__device__ __forceinline__ void decode16(const uint32_t (&c)[4], float (&y)[kEPL]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    y[4 * d + 0] = __builtin_amdgcn_cvt_f32_fp8(c[d], 0);
    y[4 * d + 1] = __builtin_amdgcn_cvt_f32_fp8(c[d], 1);
    y[4 * d + 2] = __builtin_amdgcn_cvt_f32_fp8(c[d], 2);
    y[4 * d + 3] = __builtin_amdgcn_cvt_f32_fp8(c[d], 3);
  }
}

struct GroupQuant { float scale, k, inv_a; };

// Per-group scale and exponent from the group's extreme magnitudes (Definition 1, Sec. 4.2).
// amin is the minimum over NON-ZERO magnitudes (+inf when there is none).
// EXPAND: inv_a = 1/(448 scale), the reciprocal of the magnitude the top code stands for.
// !EXPAND: k = 1 and inv_a = 1/scale, so that the value to round is simply x / scale (Sec. 3).
template <bool EXPAND>
__device__ __forceinline__ GroupQuant group_quant_params(float amax, float amin, float k_min, float k_max,
                                                         float unit = 1.0f) {
  // The values reduced over are x / unit (unit = 1 - beta inside the step, 1 otherwise): the
  // stored scale refers to x, the reciprocal returned refers to the values as they are held.
  GroupQuant r;
  // amax / 448, correctly rounded: multiply by the rounded reciprocal, then one residual step
  constexpr float inv448 = 1.0f / 448.0f;
  const float ax = amax * unit;
  float s = ax * inv448;
  s = __builtin_fmaf(__builtin_fmaf(-kE4M3Max, s, ax), inv448, s);
  float k = 1.0f;
  if constexpr (EXPAND) {
    // two hardware reciprocals (1 ulp each) are enough here: k moves by ~2 ulp
    // (the max keeps a ratio that rounds below 1 from turning the huge k negative)
    const float ratio = __builtin_fmaxf(amax * hw_rcp(amin), 1.0f);   // R_X
    float kk = kLog2Range * hw_rcp(hw_log2(ratio));
    kk = __builtin_amdgcn_fmed3f(kk, k_min, k_max);
    k = (amax != amin) ? kk : 1.0f;
  }
  const float inv_a = unit * hw_rcp(EXPAND ? kE4M3Max * s : s);
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

// Quantize 16 values to E4M3 codes (native convert: round to nearest even; magnitudes up to 464
// round to 448, and the value to convert never exceeds 448 * (1 + 2^-22)^k_max).
//   EXPAND : code = E4M3( sign(x) * 448 * (|x| * inv_a)^k ),  inv_a = 1/(448 scale)
//   !EXPAND: code = E4M3( x / scale ) with the correctly rounded fp32 quotient (this mode is the
//            plain quantizer of Sec. 3 kept as a baseline; it is not tuned)
// SIGNED = false (second moment, never negative) skips the sign transfer.
template <bool EXPAND, bool SIGNED>
__device__ __forceinline__ void quantize16(const float (&x)[kEPL], const GroupQuant& gq, uint32_t (&c)[4],
                                           float unit = 1.0f) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    float q[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const float xv = x[4 * d + b];
      if constexpr (EXPAND) {
        // 448 r^k = exp2(k log2 r + log2 448): one fma, rounded once at magnitude <= 9
        // (log2 0 = -inf, so a zero stays zero)
        const float m = hw_exp2(__builtin_fmaf(hw_log2(__builtin_fabsf(xv) * gq.inv_a), gq.k, kLog2E4M3Max));
        q[b] = SIGNED ? as_f32(as_u32(m) | (as_u32(xv) & 0x80000000u)) : m;
      } else {
        q[b] = gq.inv_a != 0.0f ? (xv * unit) / gq.scale : 0.0f;   // IEEE division: correctly rounded
      }
    }
    uint32_t p = __builtin_amdgcn_cvt_pk_fp8_f32(q[0], q[1], 0u, false);
    c[d] = __builtin_amdgcn_cvt_pk_fp8_f32(q[2], q[3], p, true);
  }
}

// ---------------------------------------------------------------------------------------
// the fused step: one chunk of 1024 elements per wavefront iteration
// ---------------------------------------------------------------------------------------

// Per-group metadata of one chunk as one lane sees it (its own group's words).
struct GroupMeta { float m_scale, m_k, v_scale, v_k; };

// The arithmetic of the step on one lane's 16 elements, registers in, registers out:
// w (in/out), g, codes (in/out), metadata (in/out).  Cross-lane traffic: the group reductions.
template <int G, bool EXPAND>
__device__ __forceinline__ void step_core(const StepArgs& a, const Log2Entry* lut, float (&w)[kEPL],
                                          const float (&g)[kEPL], uint32_t (&mc)[4], uint32_t (&vc)[4],
                                          GroupMeta& meta) {
  constexpr int LPG = G / kEPL;                      // lanes per group
  float m[kEPL], v[kEPL];
  float m_fac, v_fac;                                // beta/(1-beta) * (magnitude of the decoded unit)
  if constexpr (EXPAND) {
    // m = (448 scale) * |c/448|^(1/k).  A plain hardware reciprocal of k is enough: the
    // compensated path recovers its error, the other one is modelled with it.
    inverse_expand16<true, true>(lut, mc, meta.m_k, hw_rcp(meta.m_k), m);
    inverse_expand16<false, false>(lut, vc, meta.v_k, hw_rcp(meta.v_k), v);
    m_fac = a.beta1_ratio * (kE4M3Max * meta.m_scale);
    v_fac = a.beta2_ratio * (kE4M3Max * meta.v_scale);
  } else {
    // plain dequantizer: m = scale * c (k is 1 in this mode and is not read)
    decode16<true>(mc, m);
    decode16<false>(vc, v);
    m_fac = a.beta1_ratio * meta.m_scale;
    v_fac = a.beta2_ratio * meta.v_scale;
  }

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
  const GroupQuant qm = group_quant_params<EXPAND>(m_max, m_min, a.k_min, a.k_max, a.one_minus_beta1);
  const GroupQuant qv = group_quant_params<EXPAND>(v_max, v_min, a.k_min, a.k_max, a.one_minus_beta2);
  quantize16<EXPAND, true>(m, qm, mc, a.one_minus_beta1);
  quantize16<EXPAND, false>(v, qv, vc, a.one_minus_beta2);
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

template <int G, bool EXPAND>
__device__ __forceinline__ void issue_loads(const StepArgs& a, uint64_t chunk, int lane, RawChunk& r) {
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
  r.meta.m_scale = a.ms[gb + gl];
  r.meta.v_scale = a.vs[gb + gl];
  if constexpr (EXPAND) { r.meta.m_k = a.mk[gb + gl]; r.meta.v_k = a.vk[gb + gl]; }
  else { r.meta.m_k = 1.0f; r.meta.v_k = 1.0f; }
}

// One full chunk: rows -> lane layout through the LDS tiles, the arithmetic, and back out.
template <int G, bool EXPAND>
__device__ __forceinline__ void process_chunk(const StepArgs& a, const Log2Entry* lut, const StageTiles& tiles,
                                              uint64_t chunk, int lane, RawChunk& r) {
  constexpr int LPG = G / kEPL;
  const uint64_t cb = chunk * kChunk;
  const uint64_t gb = chunk * (kChunk / G);
  u32x4* const g_row = tiles.g + lane + (lane >> 3);          // + 72 j
  u32x4* const g_own = tiles.g + 2 * lane + (lane >> 2);      // + j

  float w[kEPL], g[kEPL];
#pragma unroll
  for (int j = 0; j < 2; ++j) g_row[72 * j] = r.g[j];
  tile_rows_to_lanes(tiles.w, lane, r.w, w);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const u32x4 t = g_own[j];
    g[8 * j + 0] = as_f32(t.x << 16); g[8 * j + 1] = as_f32(t.x & 0xffff0000u);
    g[8 * j + 2] = as_f32(t.y << 16); g[8 * j + 3] = as_f32(t.y & 0xffff0000u);
    g[8 * j + 4] = as_f32(t.z << 16); g[8 * j + 5] = as_f32(t.z & 0xffff0000u);
    g[8 * j + 6] = as_f32(t.w << 16); g[8 * j + 7] = as_f32(t.w & 0xffff0000u);
  }
  uint32_t mc[4] = {r.mc.x, r.mc.y, r.mc.z, r.mc.w};
  uint32_t vc[4] = {r.vc.x, r.vc.y, r.vc.z, r.vc.w};
  GroupMeta meta = r.meta;

  step_core<G, EXPAND>(a, lut, w, g, mc, vc, meta);

  tile_lanes_to_rows_store<16>(tiles.w, lane, w, a.w + cb);
  const u32x4 mo = {mc[0], mc[1], mc[2], mc[3]}, vo = {vc[0], vc[1], vc[2], vc[3]};
  stg<2>(reinterpret_cast<u32x4*>(a.mq + cb) + lane, mo);
  stg<2>(reinterpret_cast<u32x4*>(a.vq + cb) + lane, vo);
  if ((lane % LPG) == 0) {
    const int gl = lane / LPG;
    a.ms[gb + gl] = meta.m_scale; a.mk[gb + gl] = meta.m_k;
    a.vs[gb + gl] = meta.v_scale; a.vk[gb + gl] = meta.v_k;
  }
}

// Main kernel: one chunk per wavefront (the loop only runs again for buffers with more chunks
// than the grid has wavefronts).  The first chunk's loads are issued before the block fills its
// lookup table, so the table's latency hides behind them.
template <int G, bool EXPAND>
__global__ __launch_bounds__(kBlock) void adamw_step_kernel(StepArgs a) {
  __shared__ Log2Entry lut[256];
  __shared__ f32x4 tile_w[kWavesPerBlock * kTileSlotsW];
  __shared__ u32x4 tile_g[kWavesPerBlock * kTileSlotsG];
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wavefront-uniform
  const StageTiles tiles = {tile_w + wv * kTileSlotsW, tile_g + wv * kTileSlotsG};
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv;

  RawChunk r;
  const bool have = chunk < a.n_full;
  if (have) issue_loads<G, EXPAND>(a, chunk, lane, r);
  fill_lut(lut);                                     // every wavefront of the block reaches this
  if (have) process_chunk<G, EXPAND>(a, lut, tiles, chunk, lane, r);
  for (chunk += stride; chunk < a.n_full; chunk += stride) {
    issue_loads<G, EXPAND>(a, chunk, lane, r);
    process_chunk<G, EXPAND>(a, lut, tiles, chunk, lane, r);
  }
}

// The ragged last chunk (n % 1024 elements): one wavefront, element-wise guarded accesses
// straight into the lane layout.
template <int G, bool EXPAND>
__global__ __launch_bounds__(kWave) void adamw_step_tail_kernel(StepArgs a) {
  __shared__ Log2Entry lut[256];
  fill_lut(lut);
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x;
  const uint64_t chunk = a.n_full;
  const uint64_t base = chunk * kChunk + static_cast<uint64_t>(lane) * kEPL;
  const uint64_t gidx = chunk * (kChunk / G) + static_cast<uint64_t>(lane / LPG);
  const bool gvalid = gidx < a.n_groups;
  float w[kEPL], g[kEPL];
  uint32_t mc[4], vc[4];
  load_f32x16<true>(a.w, base, a.n, w);
  load_bf16x16<true>(a.g, base, a.n, g);
  load_codes16<true>(a.mq, base, a.n, mc);
  load_codes16<true>(a.vq, base, a.n, vc);
  GroupMeta meta;
  meta.m_scale = gvalid ? a.ms[gidx] : 0.0f;
  meta.v_scale = gvalid ? a.vs[gidx] : 0.0f;
  meta.m_k = (EXPAND && gvalid) ? a.mk[gidx] : 1.0f;
  meta.v_k = (EXPAND && gvalid) ? a.vk[gidx] : 1.0f;
  step_core<G, EXPAND>(a, lut, w, g, mc, vc, meta);
  store_f32x16<true>(a.w, base, a.n, w);
  store_codes16<true>(a.mq, base, a.n, mc);
  store_codes16<true>(a.vq, base, a.n, vc);
  if (gvalid && (lane % LPG) == 0) {
    a.ms[gidx] = meta.m_scale; a.mk[gidx] = meta.m_k;
    a.vs[gidx] = meta.v_scale; a.vk[gidx] = meta.v_k;
  }
}

// ---------------------------------------------------------------------------------------
// standalone quantizer / dequantizer (the two halves of the step)
// ---------------------------------------------------------------------------------------

// quantize one lane's 16 values (cross-lane: the group reductions) and hand back codes + metadata
template <int G, bool EXPAND>
__device__ __forceinline__ GroupQuant quant_core(const QuantArgs& a, const float (&x)[kEPL], uint32_t (&c)[4]) {
  constexpr int LPG = G / kEPL;
  float hi, lo;
  lane_extremes(x, hi, lo);
  hi = group_allreduce<LPG, true>(hi);
  lo = group_allreduce<LPG, false>(lo);
  const GroupQuant q = group_quant_params<EXPAND>(hi, lo, a.k_min, a.k_max);
  quantize16<EXPAND, true>(x, q, c);
  return q;
}

// full chunks: coalesced streaming row loads of x staged through the LDS tile, one chunk per wavefront
template <int G, bool EXPAND>
__global__ __launch_bounds__(kBlock) void quant_kernel(QuantArgs a) {
  __shared__ f32x4 tile_x[kWavesPerBlock * kTileSlotsW];
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  for (uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv; chunk < a.n_full; chunk += stride) {
    const uint64_t cb = chunk * kChunk, gb = chunk * (kChunk / G);
    const f32x4* xq = reinterpret_cast<const f32x4*>(a.x + cb);
    f32x4 rows[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) rows[j] = ldg<8>(xq + 64 * j + lane);
    float x[kEPL];
    uint32_t c[4];
    tile_rows_to_lanes(tile_x + wv * kTileSlotsW, lane, rows, x);
    const GroupQuant q = quant_core<G, EXPAND>(a, x, c);
    const u32x4 co = {c[0], c[1], c[2], c[3]};
    stg<2>(reinterpret_cast<u32x4*>(a.q + cb) + lane, co);
    if ((lane % LPG) == 0) { a.scale[gb + lane / LPG] = q.scale; a.k[gb + lane / LPG] = q.k; }
  }
}

// the ragged last chunk: one wavefront, element-wise guarded accesses
template <int G, bool EXPAND>
__global__ __launch_bounds__(kWave) void quant_tail_kernel(QuantArgs a) {
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x;
  const uint64_t base = a.n_full * kChunk + static_cast<uint64_t>(lane) * kEPL;
  const uint64_t gidx = a.n_full * (kChunk / G) + static_cast<uint64_t>(lane / LPG);
  float x[kEPL];
  uint32_t c[4];
  load_f32x16<true>(a.x, base, a.n, x);
  const GroupQuant q = quant_core<G, EXPAND>(a, x, c);
  store_codes16<true>(a.q, base, a.n, c);
  if (gidx < a.n_groups && (lane % LPG) == 0) { a.scale[gidx] = q.scale; a.k[gidx] = q.k; }
}

template <int G>
__global__ __launch_bounds__(kBlock) void dequant_kernel(DequantArgs a) {
  __shared__ Log2Entry lut[256];
  __shared__ f32x4 tile_x[kWavesPerBlock * kTileSlotsW];
  fill_lut(lut);
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  for (uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv; chunk < a.n_full; chunk += stride) {
    const uint64_t cb = chunk * kChunk, gb = chunk * (kChunk / G);
    const u32x4 ci = ldg<1>(reinterpret_cast<const u32x4*>(a.q + cb) + lane);
    const float amag = kE4M3Max * a.scale[gb + lane / LPG];
    const float k = a.k[gb + lane / LPG];
    const uint32_t c[4] = {ci.x, ci.y, ci.z, ci.w};
    float x[kEPL];
    inverse_expand16<true, true>(lut, c, k, hw_rcp(k), x);
#pragma unroll
    for (int e = 0; e < kEPL; ++e) x[e] *= amag;
    tile_lanes_to_rows_store<16>(tile_x + wv * kTileSlotsW, lane, x, a.x + cb);
  }
}

template <int G>
__global__ __launch_bounds__(kWave) void dequant_tail_kernel(DequantArgs a) {
  __shared__ Log2Entry lut[256];
  fill_lut(lut);
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x;
  const uint64_t base = a.n_full * kChunk + static_cast<uint64_t>(lane) * kEPL;
  const uint64_t gidx = a.n_full * (kChunk / G) + static_cast<uint64_t>(lane / LPG);
  const bool gvalid = gidx < a.n_groups;
  uint32_t c[4];
  float x[kEPL];
  load_codes16<true>(a.q, base, a.n, c);
  const float amag = kE4M3Max * (gvalid ? a.scale[gidx] : 0.0f);
  const float k = gvalid ? a.k[gidx] : 1.0f;
  inverse_expand16<true, true>(lut, c, k, hw_rcp(k), x);
#pragma unroll
  for (int e = 0; e < kEPL; ++e) x[e] *= amag;
  store_f32x16<true>(a.x, base, a.n, x);
}

// ---------------------------------------------------------------------------------------
// host side: validation and launch
// ---------------------------------------------------------------------------------------

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool finite_f(float x) { return x == x && x - x == 0.0f; }
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
// sentinel for zero codes, no overflow of the value handed to the E4M3 convert)
constexpr float kKLowest = 0.015625f, kKHighest = 65536.0f;
bool resolve_k_bounds(float& k_min, float& k_max) {
  if (!finite_f(k_min) || !finite_f(k_max)) return false;
  if (k_min == 0.0f && k_max == 0.0f) { k_min = 0.0625f; k_max = 1024.0f; }
  return k_min >= kKLowest && k_max <= kKHighest && k_min <= k_max;
}

int launch_status() { return hipGetLastError() == hipSuccess ? COAT_OK : COAT_ERR_LAUNCH; }

// The step kernel asks for this much dynamic LDS on top of its ~29 KiB of tiles and table, for no
// other purpose than to hold a CU to two resident blocks (8 wavefronts): with fewer bytes in
// flight per CU the HBM controllers see longer same-page runs, and two wavefronts per SIMD are
// enough to overlap one's arithmetic with the other's loads (measured on the 7B set: 2 blocks
// 6.04 TB/s, 3 blocks 5.91, 4 blocks 5.81, 1 block 3.66).
constexpr size_t kStepLdsPad = 24 * 1024;

template <int G, bool EXPAND>
int launch_step(const StepArgs& a, hipStream_t s) {
  if (a.n_full) {
    const unsigned grid = grid_for(a.n_full);
    size_t lds = kStepLdsPad;
#ifdef COAT_TUNING
    if (g_tune_lds_pad >= 0) lds = static_cast<size_t>(g_tune_lds_pad);
    if (lds > 32 * 1024)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&adamw_step_kernel<G, EXPAND>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
#endif
    hipLaunchKernelGGL((adamw_step_kernel<G, EXPAND>), dim3(grid), dim3(kBlock), lds, s, a);
    if (int rc = launch_status()) return rc;
  }
  if (a.n > a.n_full * kChunk) {
    hipLaunchKernelGGL((adamw_step_tail_kernel<G, EXPAND>), dim3(1), dim3(kWave), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  return COAT_OK;
}

template <int G, bool EXPAND>
int launch_quant(const QuantArgs& a, hipStream_t s) {
  if (a.n_full) {
    hipLaunchKernelGGL((quant_kernel<G, EXPAND>), dim3(grid_for(a.n_full)), dim3(kBlock), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  if (a.n > a.n_full * kChunk) {
    hipLaunchKernelGGL((quant_tail_kernel<G, EXPAND>), dim3(1), dim3(kWave), 0, s, a);
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

int dispatch_step(const StepArgs& a, int32_t G, hipStream_t s) {
  if (a.expand) { COAT_DISPATCH_G(G, (launch_step<kG, true>(a, s))); }
  COAT_DISPATCH_G(G, (launch_step<kG, false>(a, s)));
}

int dispatch_quant(const QuantArgs& a, int32_t G, hipStream_t s) {
  if (a.expand) { COAT_DISPATCH_G(G, (launch_quant<kG, true>(a, s))); }
  COAT_DISPATCH_G(G, (launch_quant<kG, false>(a, s)));
}

int dispatch_dequant(const DequantArgs& a, int32_t G, hipStream_t s) {
  COAT_DISPATCH_G(G, (launch_dequant<kG>(a, s)));
}

}  // namespace

extern "C" {

int coat_fp8_adamw_step(float* w, const uint16_t* grad_bf16, uint8_t* m_q, float* m_scale, float* m_k,
                        uint8_t* v_q, float* v_scale, float* v_k, uint64_t n,
                        const coat_adamw_hparams* hp, void* hip_stream) {
  if (!hp) return COAT_ERR_NULL;
  if (!group_ok(hp->group_size)) return COAT_ERR_GROUP;
  if (hp->step < 1) return COAT_ERR_STEP;
  if (!finite_f(hp->lr) || !finite_f(hp->beta1) || !finite_f(hp->beta2) || !finite_f(hp->eps) ||
      !finite_f(hp->weight_decay))
    return COAT_ERR_HPARAM;
  if (hp->lr < 0.0f || hp->beta1 < 0.0f || hp->beta1 >= 1.0f || hp->beta2 < 0.0f || hp->beta2 >= 1.0f ||
      hp->eps < 0.0f)
    return COAT_ERR_HPARAM;
  float k_min = hp->k_min, k_max = hp->k_max;
  if (!resolve_k_bounds(k_min, k_max)) return COAT_ERR_HPARAM;
  if (n == 0) return COAT_OK;
  if (!w || !grad_bf16 || !m_q || !m_scale || !m_k || !v_q || !v_scale || !v_k) return COAT_ERR_NULL;
  if (!aligned16(w) || !aligned16(grad_bf16) || !aligned16(m_q) || !aligned16(v_q) ||
      !aligned16(m_scale) || !aligned16(m_k) || !aligned16(v_scale) || !aligned16(v_k))
    return COAT_ERR_ALIGN;
  if (n > (1ull << 46)) return COAT_ERR_SIZE;

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

  StepArgs a;
  a.w = w; a.g = grad_bf16; a.mq = m_q; a.ms = m_scale; a.mk = m_k; a.vq = v_q; a.vs = v_scale; a.vk = v_k;
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(hp->group_size) - 1) / static_cast<uint64_t>(hp->group_size);
  a.one_minus_beta1 = 1.0f - hp->beta1;               // exact (Sterbenz) for beta >= 0.5
  a.one_minus_beta2 = 1.0f - hp->beta2;
  const double omb1 = a.one_minus_beta1, omb2 = a.one_minus_beta2;
  a.beta1_ratio = static_cast<float>(b1 / omb1);
  a.beta2_ratio = static_cast<float>(b2 / omb2);
  a.neg_lr_m = static_cast<float>(-static_cast<double>(hp->lr) * omb1 / bc1);
  a.neg_lr_wd = static_cast<float>(-static_cast<double>(hp->lr) * static_cast<double>(hp->weight_decay));
  a.denom_scale = static_cast<float>(__builtin_sqrt(omb2 / bc2));
  a.eps = hp->eps;
  a.k_min = k_min; a.k_max = k_max;
  a.expand = (hp->flags & COAT_FLAG_EXPAND) ? 1u : 0u;
  return dispatch_step(a, hp->group_size, static_cast<hipStream_t>(hip_stream));
}

int coat_quant_group(const float* x, uint64_t n, int32_t G, uint32_t flags, float k_min, float k_max,
                     uint8_t* q, float* scale, float* k, void* hip_stream) {
  if (!group_ok(G)) return COAT_ERR_GROUP;
  if (!resolve_k_bounds(k_min, k_max)) return COAT_ERR_HPARAM;
  if (n == 0) return COAT_OK;
  if (!x || !q || !scale || !k) return COAT_ERR_NULL;
  if (!aligned16(x) || !aligned16(q) || !aligned16(scale) || !aligned16(k)) return COAT_ERR_ALIGN;
  if (n > (1ull << 46)) return COAT_ERR_SIZE;
  QuantArgs a;
  a.x = x; a.q = q; a.scale = scale; a.k = k;
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(G) - 1) / static_cast<uint64_t>(G);
  a.k_min = k_min; a.k_max = k_max;
  a.expand = (flags & COAT_FLAG_EXPAND) ? 1u : 0u;
  return dispatch_quant(a, G, static_cast<hipStream_t>(hip_stream));
}

int coat_dequant_group(const uint8_t* q, const float* scale, const float* k, uint64_t n, int32_t G,
                       float* x, void* hip_stream) {
  if (!group_ok(G)) return COAT_ERR_GROUP;
  if (n == 0) return COAT_OK;
  if (!x || !q || !scale || !k) return COAT_ERR_NULL;
  if (!aligned16(x) || !aligned16(q) || !aligned16(scale) || !aligned16(k)) return COAT_ERR_ALIGN;
  if (n > (1ull << 46)) return COAT_ERR_SIZE;
  DequantArgs a;
  a.q = q; a.scale = scale; a.k = k; a.x = x;
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(G) - 1) / static_cast<uint64_t>(G);
  return dispatch_dequant(a, G, static_cast<hipStream_t>(hip_stream));
}

const char* coat_strerror(int code) {
  switch (code) {
    case COAT_OK: return "ok";
    case COAT_ERR_NULL: return "a required pointer is NULL";
    case COAT_ERR_ALIGN: return "a base pointer is not 16-byte aligned";
    case COAT_ERR_GROUP: return "group size must be one of 32, 64, 128, 256, 512";
    case COAT_ERR_STEP: return "step must be >= 1";
    case COAT_ERR_HPARAM: return "hyper-parameter is non-finite or out of its domain";
    case COAT_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    case COAT_ERR_SIZE: return "n is too large";
  }
  return "unknown error code";
}

int coat_version(void) { return 100; }

#ifdef COAT_TUNING
// development builds only: launch-shape knobs for sweeps
void coat_tune_set(int cap_mult, int lds_pad, int unused) {
  g_tune_cap_mult = cap_mult; g_tune_lds_pad = lds_pad; (void)unused;
}
#endif

}  // extern "C"
