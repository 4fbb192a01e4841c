// coat_device.hpp -- types, storage modes, cross-lane and memory helpers, LDS staging and the (de)quantizer arithmetic shared by every kernel
// Part of the one translation unit coat_kernels.hip (included from there, in this order).
#pragma once

#include <type_traits>

namespace {

constexpr int kWave = 64;                 // lanes per wavefront
constexpr int kEPL = 16;                  // consecutive elements owned by one lane
constexpr int kWavesPerBlock = 4;
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
// kDq: which inverse expansion the fused step uses for this moment (see inverse_expand16): 0 the
// plain one, 1 with the rounding of the exponent recovered.
template <bool E5M2, bool EXPAND, int DQ = 0>
struct StaticMode {
  static constexpr int kDq = DQ;
  __device__ __forceinline__ bool e5m2() const { return E5M2; }
  __device__ __forceinline__ bool expand() const { return EXPAND; }
  __device__ __forceinline__ bool scale16() const { return false; }
  __device__ __forceinline__ bool k16() const { return false; }
};
// Format and expansion folded at compile time, the storage of the per-group scales and exponents
// (fp32 or bf16) as run-time values: only the few per-group operations depend on those, the
// per-element code folds as in StaticMode.  Bf16MetaMode is the default cell with bf16 metadata.
template <bool E5M2, bool EXPAND>
struct FoldedMode {
  static constexpr int kDq = 0;
  bool s16, kh;
  __device__ __forceinline__ bool e5m2() const { return E5M2; }
  __device__ __forceinline__ bool expand() const { return EXPAND; }
  __device__ __forceinline__ bool scale16() const { return s16; }
  __device__ __forceinline__ bool k16() const { return kh; }
};
typedef FoldedMode<false, true> Bf16MetaMode;
struct RuntimeMode {
  static constexpr int kDq = 1;   // the generic kernel always takes the more accurate inverse expansion
  bool e5, ex;
  bool s16;   // the per-group scales are stored as bf16 (Sec. 3) instead of fp32
  bool kh;    // the per-group exponents k are stored as bf16 as well
  __device__ __forceinline__ bool e5m2() const { return e5; }
  __device__ __forceinline__ bool expand() const { return ex; }
  __device__ __forceinline__ bool scale16() const { return s16; }
  __device__ __forceinline__ bool k16() const { return kh; }
};
// The expansion switch folded at compile time, format and metadata storage at run time: what the
// generic kernel runs once it has picked one of its four (first moment, second moment) variants.
// The switch decides between two different per-element programs (logarithm / exponential, or an
// exact division), which as run-time branches inside the unrolled element loops compile to several
// hundred basic blocks; the format only selects constants, a table half and a convert.
template <bool EXPAND>
struct FormatMode {
  static constexpr int kDq = 1;
  bool e5, s16, kh;
  __device__ __forceinline__ explicit FormatMode(const RuntimeMode& r) : e5(r.e5), s16(r.s16), kh(r.kh) {}
  __device__ __forceinline__ bool e5m2() const { return e5; }
  __device__ __forceinline__ bool expand() const { return EXPAND; }
  __device__ __forceinline__ bool scale16() const { return s16; }
  __device__ __forceinline__ bool k16() const { return kh; }
};
typedef StaticMode<false, true> DefaultMode;
typedef StaticMode<false, true, 1> PreciseMode;   // the default cell for callers who set COAT_FLAG_PRECISE_DQ

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
  // Eq. (1) as  w <- w_keep * w + m' / (denom_mul * sqrt(v') + denom_add)  with the step size folded
  // into the denominator: with c = -lr (1 - beta1) / (1 - beta1^t) (the factor that turns m' / D into
  // the update), denom_mul = sqrt((1 - beta2) / (1 - beta2^t)) / c and denom_add = eps / c; lr == 0
  // gives denom_mul = 0 and denom_add = +inf, i.e. no update.  w_keep = 1 - lr * weight_decay.
  float denom_mul, denom_add;
  float w_keep;
  float k_min, k_max;
  RuntimeMode mode_m, mode_v;
  // the same first-moment update in fp64, for the one element per lane that is recomputed exactly
  // (ExactChain): m_t / (1 - beta1) = m_ratio64 * m + g_coef64 * g, with beta1 the fp32
  // hyper-parameter taken as a double; g_coef64 = (1 - beta1) / one_minus_beta1 is 1 whenever the
  // fp32 difference 1 - beta1 is exact (beta1 >= 0.5)
  double m_ratio64, g_coef64;
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

// Per-group word i of an array that holds fp32 or, with `half16`, bf16 values (the pointer is typed
// float* either way): the scales and the exponents k.  A stored bf16 value is exact: the quantizer
// rounded it before using it.
__device__ __forceinline__ float load_meta(bool half16, const float* p, uint64_t i) {
  if (half16) return as_f32(static_cast<uint32_t>(reinterpret_cast<const uint16_t*>(p)[i]) << 16);
  return p[i];
}
// The same for group gl of a FULL chunk whose first group is gb, without control flow: one dword
// load serves both layouts (a branch here costs the kernel its overlap of loads: the compiler
// drains the load counter where the two sides meet; measured 17.3 ms against 15.9).  A chunk holds
// an even number of groups starting at an even index, so the dword is inside the chunk's words.
__device__ __forceinline__ float load_meta_full_chunk(bool half16, const float* p, uint64_t gb, int gl) {
  const uint32_t w = reinterpret_cast<const uint32_t*>(p)[half16 ? (gb + gl) >> 1 : gb + gl];
  const uint32_t half = (gl & 1) ? (w & 0xffff0000u) : (w << 16);
  return as_f32(half16 ? half : w);
}
__device__ __forceinline__ void store_meta(bool half16, float* p, uint64_t i, float s) {
  if (half16) reinterpret_cast<uint16_t*>(p)[i] = static_cast<uint16_t>(as_u32(s) >> 16);
  else p[i] = s;
}
template <class Mode>
__device__ __forceinline__ float load_scale(const Mode& md, const float* p, uint64_t i) { return load_meta(md.scale16(), p, i); }
template <class Mode>
__device__ __forceinline__ float load_scale_full_chunk(const Mode& md, const float* p, uint64_t gb, int gl) {
  return load_meta_full_chunk(md.scale16(), p, gb, gl);
}
template <class Mode>
__device__ __forceinline__ void store_scale(const Mode& md, float* p, uint64_t i, float s) { store_meta(md.scale16(), p, i, s); }
template <class Mode>
__device__ __forceinline__ float load_k(const Mode& md, const float* p, uint64_t i) { return load_meta(md.k16(), p, i); }
template <class Mode>
__device__ __forceinline__ float load_k_full_chunk(const Mode& md, const float* p, uint64_t gb, int gl) {
  return load_meta_full_chunk(md.k16(), p, gb, gl);
}
template <class Mode>
__device__ __forceinline__ void store_k(const Mode& md, float* p, uint64_t i, float k) { store_meta(md.k16(), p, i, k); }

__device__ __forceinline__ float hw_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float hw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float hw_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float hw_sqrt(float x) { return __builtin_amdgcn_sqrtf(x); }

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t x) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), CTRL, 0xf, 0xf, true));
}

// Butterfly all-reduce over LPG adjacent lanes (LPG = lanes per group, a power of two <= 32).
//   xor 1 / xor 2 : quad_perm, lanes 4..7 / 8..15 : row_half_mirror / row_mirror (after the
//   previous steps every lane of the smaller block already holds that block's result),
//   xor 16 : ds_swizzle inside 32 lanes.
// The values reduced are magnitudes (non-negative, +inf for "none"), so their bit patterns order
// like the numbers and the reduction runs on unsigned integers: no canonicalization of the
// cross-lane operand before every floating-point min/max.  A NaN (pattern above +inf) wins a
// maximum and loses a minimum.
template <int LPG, bool IS_MAX>
__device__ __forceinline__ float group_allreduce(float xf) {
  auto op = [](uint32_t a, uint32_t b) { return IS_MAX ? (a > b ? a : b) : (a < b ? a : b); };
  uint32_t x = as_u32(xf);
  if constexpr (LPG >= 2) x = op(x, dpp_mov<0xB1>(x));    // quad_perm:[1,0,3,2]
  if constexpr (LPG >= 4) x = op(x, dpp_mov<0x4E>(x));    // quad_perm:[2,3,0,1]
  if constexpr (LPG >= 8) x = op(x, dpp_mov<0x141>(x));   // row_half_mirror
  if constexpr (LPG >= 16) x = op(x, dpp_mov<0x140>(x));  // row_mirror
  if constexpr (LPG >= 32) x = op(x, static_cast<uint32_t>(__builtin_amdgcn_ds_swizzle(static_cast<int>(x), 0x401F)));
  return as_f32(x);
}

// Bulk accesses: every array is streamed through once per step, so every bulk load and store is
// issued as non-temporal (measured best for all five kinds of access).  KIND only names the access
// at the call site: 1 load codes, 2 store codes, 4 load gradients, 8 load fp32, 16 store fp32.
template <int KIND, typename T>
__device__ __forceinline__ T ldg(const T* p) { return __builtin_nontemporal_load(p); }
template <int KIND, typename T>
__device__ __forceinline__ void stg(T* p, T v) { __builtin_nontemporal_store(v, p); }

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

struct StageTiles { f32x4* w; u32x4* g; u32x4* codes; };   // codes: 16 bytes per lane (see LaneScratch)

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

// The tables a step kernel keeps in LDS: the logarithms of the code magnitudes (per format 256
// entries so that the whole code byte indexes it; the sign bit is ignored) and the fractional
// powers 2^(j/512) that ExactChain looks up.  TABLES = 1 loads E4M3 only, 2 loads E4M3 then E5M2.
constexpr int kExp2Frac = kExp2FracSize;
struct StepTables { const Log2Entry* lut; const double* frac; };

// The fill in two halves.  THREADS: the (compile-time) size of the block.
//   fill_issue : every thread's table entries are requested (all loads before any LDS write, so
//                the fill costs ONE trip to memory; a loop that waits per iteration adds a full
//                memory latency to the wavefront's life each time, about +0.6 ms per extra trip on
//                the 7B set);
//   fill_commit: the entries go to LDS and the block synchronizes.
// A step kernel calls fill_issue FIRST, then its admission gate and its chunk's loads, then
// fill_commit: loads return in order, so the table entries arrive before the bulk data and the
// block's one barrier is over while the bulk data is still in flight; each wavefront then starts
// on its own data as soon as that arrives.  With the table requested after the bulk loads every
// wavefront of the block waited at the barrier for the slowest one's data (7B set: 15.2 -> 14.9 ms).
template <int TABLES, int THREADS>
struct FillRegs {
  static constexpr int kLutIters = (256 * TABLES + THREADS - 1) / THREADS, kFracIters = (kExp2Frac + THREADS - 1) / THREADS;
  Log2Entry e[kLutIters];
  double f[kFracIters];
};
template <int TABLES, int THREADS>
__device__ __forceinline__ void fill_issue(FillRegs<TABLES, THREADS>& fr) {
#pragma unroll
  for (int r = 0; r < FillRegs<TABLES, THREADS>::kLutIters; ++r) {
    const int i = threadIdx.x + r * THREADS;
    fr.e[r] = kLog2Code[(i >> 8) & 1][i & 127];
  }
#pragma unroll
  for (int r = 0; r < FillRegs<TABLES, THREADS>::kFracIters; ++r)
    fr.f[r] = kExp2Frac512[(threadIdx.x + r * THREADS) & (kExp2Frac - 1)];
  __builtin_amdgcn_sched_barrier(0);                 // the requests stay ahead of what follows
}
template <int TABLES, int THREADS>
__device__ __forceinline__ void fill_commit(const FillRegs<TABLES, THREADS>& fr, Log2Entry* lut, double* frac) {
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int r = 0; r < FillRegs<TABLES, THREADS>::kLutIters; ++r)
    if (threadIdx.x + r * THREADS < 256 * TABLES) lut[threadIdx.x + r * THREADS] = fr.e[r];
#pragma unroll
  for (int r = 0; r < FillRegs<TABLES, THREADS>::kFracIters; ++r)
    if (threadIdx.x + r * THREADS < kExp2Frac) frac[threadIdx.x + r * THREADS] = fr.f[r];
  __syncthreads();
}

constexpr float kLn2 = 0.6931471805599453f;

// |c/fmax|^(1/k) for 16 codes.
//   ACCURATE = 0: exp2(L * (1/k)), good to about |L/k| * 2^-22 relative;
//   ACCURATE = 1: the rounding of the product and of 1/k is recovered with one fma
//     (r = L - t*k is the exact residual of t = fl(L * fl(1/k)) against L/k, times k) and
//     exp2(t + d) = exp2(t) * (1 + d ln2): three more instructions per element, error about
//     |L/k| * 2^-24 + 1 ulp.  The fused step uses it on request (COAT_FLAG_PRECISE_DQ): the
//     weight update m / (sqrt(v) + eps) inherits the moments' relative error, which matters when
//     the update is a large fraction of the weight (large lr, beta2 close to 1, heavy-tailed
//     gradients);
//   ACCURATE = 2: also the table's own rounding, from its low word: within a few ulp of the fp64
//     value.  The standalone dequantizer uses it.
// What decides a group's exponent in the fused step is recomputed exactly either way (ExactChain).
template <bool SIGNED, int ACCURATE>
__device__ __forceinline__ void inverse_expand16(const Log2Entry* lut, const uint32_t (&c)[4], float k,
                                                 float inv_k, float (&y)[kEPL]) {
  const float inv_k_ln2 = inv_k * kLn2;
#pragma unroll
  for (int e = 0; e < kEPL; ++e) {
    const uint32_t d = c[e >> 2];
    const int sh = 8 * (e & 3);
    const uint32_t code = (d >> sh) & 0xffu;
    float v;
    if constexpr (ACCURATE == 2) {
      const Log2Entry l = lut[code];
      const float t = l.hi * inv_k;
      const float r = __builtin_fmaf(-t, k, l.hi) + l.lo;
      const float p = hw_exp2(t);
      v = __builtin_fmaf(p, r * inv_k_ln2, p);
    } else if constexpr (ACCURATE == 1) {
      const float hi = lut[code].hi;
      const float t = hi * inv_k;
      const float r = __builtin_fmaf(-t, k, hi);
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
template <bool SIGNED, int ACCURATE, class Mode>
__device__ __forceinline__ float dequant16(const Mode& md, const Log2Entry* lut, const uint32_t (&c)[4],
                                           float scale, float k, float inv_k, float (&y)[kEPL]) {
  if (md.expand()) {
    inverse_expand16<SIGNED, ACCURATE>(lut + (md.e5m2() ? 256 : 0), c, k, inv_k, y);
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
  // BF16 scale: round UP to a bf16 value (every |x| / (fmax*scale) stays <= 1, nothing saturates)
  // and take the range that has to fit the format against fmax*scale rather than amax.  Written
  // with selects: a branch here, even a uniform one, cuts the straight-line code that the exact
  // chain is interleaved with.  (The reciprocal's ulp moves k by 1e-7 / ln R at most.)
  const float s_up = as_f32((as_u32(s) + 0xFFFFu) & 0xFFFF0000u);
  const float top_up = (fmax * s_up) * hw_rcp(unit);
  const bool s16 = md.scale16();
  s = s16 ? s_up : s;
  const float top = s16 ? top_up : amax;             // what the group is normalized by, in held units
  float k = 1.0f;
  if (md.expand()) {
    // two hardware reciprocals (1 ulp each) are enough here: k moves by ~2 ulp
    // (the max keeps a ratio that rounds below 1 from turning the huge k negative)
    const float ratio = __builtin_fmaxf(top * hw_rcp(amin), 1.0f);    // R_X
    float kk = fmt_log2_range(md) * hw_rcp(hw_log2(ratio));
    kk = __builtin_amdgcn_fmed3f(kk, k_min, k_max);
    // BF16-stored exponent: the clamped value rounded to the nearest bf16, ties to even (what a cast
    // does); the codes below are computed with the stored value.  A group that received no gradient
    // reproduces the range its stored k made, computes that bf16 value again to a few 1e-7 and keeps
    // it.  (R_X^k may exceed the format's range by a factor range^(2^-8): the smallest element still
    // rounds to the smallest subnormal.)
    const uint32_t kb = as_u32(kk);
    if (md.k16()) kk = as_f32((kb + 0x7FFFu + ((kb >> 16) & 1u)) & 0xFFFF0000u);
    k = (amax != amin) ? kk : 1.0f;
  }
  const float inv_a = unit * hw_rcp(md.expand() ? fmax * s : s);
  // all zero, or so small that amax / fmax is no normal fp32 number (the hardware reciprocal of a
  // subnormal is infinite and every code would be NaN): stored as the zero state, scale 0, k 1, codes 0
  const bool empty = !(s >= 0x1.0p-126f);
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

// max |x| over the lane's 16 new first moments and, in one word, the smallest magnitude that may
// be the lane's non-zero minimum together with the index of the element that holds it:
// key = (bits of |x|, low four mantissa bits cleared) | index, so that one unsigned minimum finds
// both.  ~0 when the lane has no candidate.  An fp32 zero is a candidate too (magnitude 0, so it
// wins) when its gradient is not zero: then beta1 m and (1 - beta1) g cancelled to the last bit
// in fp32 while the exact value need not be zero; a zero with a zero gradient is a true zero
// (the old moment is zero as well) and leaves the minimum, as Definition 1 is read here.
__device__ __forceinline__ void lane_extremes_keyed(const float (&x)[kEPL], const float (&g)[kEPL], float& amax,
                                                    uint32_t& min_key) {
  float hi = 0.0f;
  uint32_t lo = 0xffffffffu;
  uint32_t mask;                                     // in a scalar register: one v_and_or_b32 per key
  asm("s_mov_b32 %0, 0x7ffffff0" : "=s"(mask));
#pragma unroll
  for (int e = 0; e < kEPL; ++e) {
    hi = __builtin_fmaxf(hi, __builtin_fabsf(x[e]));
    const uint32_t key = (as_u32(x[e]) & mask) | static_cast<uint32_t>(e);
    lo = key < lo ? key : lo;
  }
  if (__builtin_expect(lo < 16u, 0)) {               // rare: some element is exactly zero in fp32
    lo = 0xffffffffu;
#pragma unroll
    for (int e = 0; e < kEPL; ++e) {
      const uint32_t mag = as_u32(x[e]) & 0x7ffffff0u;   // (the literal, not `mask`: no sharing with the fast path's and_or)
      const bool cancelled = (as_u32(g[e]) & 0x7fffffffu) != 0u;
      const uint32_t key = (mag || cancelled) ? (mag | static_cast<uint32_t>(e)) : 0xffffffffu;
      lo = key < lo ? key : lo;
    }
  }
  amax = hi; min_key = lo;
}

// Where the lane keeps, in LDS, what the refinement below looks up by a run-time index: the 16
// first-moment codes the step started from and the 16 bf16 gradients.
typedef uint16_t __attribute__((may_alias)) lds_u16;
struct LaneScratch { const uint8_t* codes; const lds_u16* g; };

// The lane's smallest |m_t| recomputed in fp64 (with or without the expansion; without it k is 1
// and only the replacement in apply_exact_min matters).
// m_t = beta1 m + (1 - beta1) g cancels; the element where it cancels most is the group minimum,
// which fixes the exponent k = log2(range) / log2(amax / amin) (Sec. 4.2) and through k every code
// of the group.  In fp32 that element keeps the absolute error of the dequantized m but not its
// size, so the fp32 pass only NAMES the candidate (min_key, from lane_extremes_keyed) and this
// chain recomputes that one element exactly: the table logarithm as hi + lo, 1/k by a Newton
// step, 2^(L/k) by the table-based exponential (see exp2 steps below), the update as one fp64 fma,
// rounded to fp32 at the end.  About fifty instructions per lane (three per element), every one
// depending on the one before and three of them LDS look-ups, so it is cut into seventeen STEPS:
// the caller puts independent work (the second moment's quantization, one element per step) between
// them and fences every step with a scheduling barrier; left to itself the compiler runs the chain
// back to back and each wavefront lives longer by its whole latency, which costs the 7B step about
// 4 % (measured).
//   exp2 for t <= 0:  512 t = i + r with i an integer and |r| <= 1/2, so that
//   2^t = 2^(i >> 9) * 2^((i & 511) / 512) * 2^(r / 512): the middle factor from the table in LDS,
//   the last one as 1 + x + x^2/2 + x^3/6 in x = r ln2 / 512 (|x| < 6.8e-4, remainder below 1e-14);
//   below -1100 the result is 0 either way.
template <class Mode>
struct ExactChain {
  static constexpr int kSteps = 16;                  // step<0> .. step<16>
  const StepArgs& a; const Mode& md; const StepTables& tb; const LaneScratch& ls;
  uint32_t idx, code;
  float g32, scale, k, inv_k, exact;
  Log2Entry l;
  double r, amag, gd, t, u, ni, x, p, fr, q;
  int i;

  __device__ __forceinline__ ExactChain(const StepArgs& a_, const Mode& md_, const StepTables& tb_, const LaneScratch& ls_,
                                        uint32_t min_key, float scale_, float k_, float inv_k_)
      : a(a_), md(md_), tb(tb_), ls(ls_), idx(min_key & 15u), scale(scale_), k(k_), inv_k(inv_k_) {}
  // (idx is in range also when there is no candidate, min_key == ~0)

  template <int S>
  __device__ __forceinline__ void step() {
    if (md.expand()) {
      if constexpr (S == 0) {                        // the two look-ups by index go out first; 1/k meanwhile
        code = ls.codes[idx];
        g32 = as_f32(static_cast<uint32_t>(ls.g[idx]) << 16);
        const double kd = static_cast<double>(k);
        const double r0 = static_cast<double>(inv_k);
        r = __builtin_fma(r0, __builtin_fma(-kd, r0, 1.0), r0);
        amag = static_cast<double>(fmt_max(md)) * static_cast<double>(scale);
      }
      if constexpr (S == 1) l = tb.lut[(md.e5m2() ? 256u : 0u) + code];
      if constexpr (S == 2) gd = a.g_coef64 * static_cast<double>(g32);
      if constexpr (S == 3) t = (static_cast<double>(l.hi) + static_cast<double>(l.lo)) * r;
      if constexpr (S == 4) u = __builtin_fmax(t, -1100.0) * static_cast<double>(kExp2Frac);
      if constexpr (S == 5) ni = __builtin_rint(u);
      if constexpr (S == 6) {
        x = (u - ni) * (0x1.62e42fefa39efp-1 / kExp2Frac);
        i = static_cast<int>(ni);
        fr = tb.frac[i & (kExp2Frac - 1)];
      }
      if constexpr (S == 7) p = __builtin_fma(x, 1.0 / 6.0, 0.5);
      if constexpr (S == 8) p = __builtin_fma(x, p, 1.0);
      if constexpr (S == 9) p = __builtin_fma(x, p, 1.0);
      if constexpr (S == 11) q = fr * p;
      if constexpr (S == 12) q = __builtin_ldexp(q, i >> 9);
      if constexpr (S == 13) {                       // the code's sign bit goes onto the (non-negative) magnitude
        const double mag = q * amag;
        q = __builtin_bit_cast(double, __builtin_bit_cast(uint64_t, mag) | (static_cast<uint64_t>(code & 0x80u) << 56));
      }
      if constexpr (S == 14) q = __builtin_fma(a.m_ratio64, q, gd);
      if constexpr (S == 15) exact = static_cast<float>(q);
    } else {
      // stored without expansion: the decoded code times the scale, exact in fp64
      if constexpr (S == 0) {
        code = ls.codes[idx];
        g32 = as_f32(static_cast<uint32_t>(ls.g[idx]) << 16);
      }
      if constexpr (S == 2) {
        const float c = md.e5m2() ? __builtin_amdgcn_cvt_f32_bf8(code, 0) : __builtin_amdgcn_cvt_f32_fp8(code, 0);
        q = static_cast<double>(c) * static_cast<double>(scale);
        gd = a.g_coef64 * static_cast<double>(g32);
      }
      if constexpr (S == 4) q = __builtin_fma(a.m_ratio64, q, gd);
      if constexpr (S == 6) exact = static_cast<float>(q);
    }
  }
};

template <int S, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (S < N) {
    f(std::integral_constant<int, S>{});
    static_for<S + 1, N>(f);
  }
}

// The lane's smallest non-zero |m_t| given the exact value of its candidate.  Where the fp32 value
// of that element is off by more than 2^-9 of its size (deep cancellation: a few lanes in 10^4)
// `replace` is set: the minimum is then taken again with the exact value in the element's place
// (an exact zero leaves it; another element may now be the smallest) and the caller re-encodes that
// one element from the exact value (requantize_one), so that its code comes out right, sign
// included.  x itself is never written: a conditional write to the register array would cost the
// straight-line path a copy of all sixteen.  amax: the lane's maximum from the fp32 pass (in/out);
// g_named: the gradient of the candidate.
__device__ __forceinline__ float apply_exact_min(float exact, float g_named, uint32_t min_key, const float (&x)[kEPL],
                                                 float& amax, bool& replace) {
  float res = __builtin_fabsf(exact);
  const bool have = min_key != 0xffffffffu;          // false: nothing but true zeros in this lane
  const uint32_t seen_bits = min_key & 0x7ffffff0u;  // what the fp32 pass had (low mantissa bits cleared)
  // (the second condition: below 2^-20 of its gradient the fp32 value need not even have the right
  // sign, and its magnitude can still agree by chance -- seen once in 3e10 elements)
  replace = have && (!(__builtin_fabsf(res - as_f32(seen_bits)) <= 0x1p-9f * res) || res < 0x1p-20f * __builtin_fabsf(g_named));
  if (__builtin_expect(replace, 0)) {
    uint32_t idx = min_key & 15u;
    asm volatile("" : "+v"(idx));                    // keeps the loop's arithmetic inside this rare block
    res = res > 0.0f ? res : __builtin_huge_valf();
#pragma unroll
    for (int e = 0; e < kEPL; ++e) {
      const float ax = __builtin_fabsf(x[e]);
      res = __builtin_fminf(res, (static_cast<uint32_t>(e) != idx && ax > 0.0f) ? ax : __builtin_huge_valf());
    }
  }
  // a lane whose magnitudes are all the same (one element, or +-c throughout): the exact value is
  // its maximum as well, so that a group of equal magnitudes has amax == amin on this side too
  if (have && (as_u32(amax) & 0x7ffffff0u) == seen_bits && seen_bits != 0u) amax = res;
  return have ? res : __builtin_huge_valf();
}

// A first moment stored in E5M2 WITHOUT expansion: every element that cancelled deeply is recomputed
// exactly, not only the lane's smallest.  The plain E5M2 code line reaches 2^-32 of the group
// maximum, so a value that cancelled to 1e-8 of its terms is still a normal code, while the fp32
// value of m_t = beta1 m + (1 - beta1) g keeps the rounding of beta1 / (1 - beta1) * scale, 6e-8 of
// the terms.  Such values are not rare right after the start state: there m / (1 - beta1) is a
// decoded code times a bf16 maximum, the gradients are bf16 as well, and for a code of significand
// 1.75 (= fmax's) and a maximum whose significand is a multiple of ten the next gradient can equal
// -beta1 m / (1 - beta1) to the last bit (measured: 1.5e-4 of the elements at step 2, two of them in
// one lane a few times in 10^7 lanes).  Without expansion the decoded code times the scale is exact
// in fp64, so the recomputation is three operations.  (Plain E4M3 reaches 2^-17.8 only: there the
// fp32 error is 1.4 % of the smallest code step and nothing is done.)
template <class Mode>
__device__ __forceinline__ void recompute_cancelled_plain(const StepArgs& a, const Mode& md, const LaneScratch& ls,
                                                          float scale, const float (&g)[kEPL], float (&x)[kEPL]) {
  bool any = false;
#pragma unroll
  for (int e = 0; e < kEPL; ++e) any |= __builtin_fabsf(x[e]) < 0x1p-14f * __builtin_fabsf(g[e]);
  if (__builtin_expect(any, 0)) {
#pragma unroll
    for (int e = 0; e < kEPL; ++e) {
      const uint32_t code = ls.codes[e];
      const float c = md.e5m2() ? __builtin_amdgcn_cvt_f32_bf8(code, 0) : __builtin_amdgcn_cvt_f32_fp8(code, 0);
      const double ex = __builtin_fma(a.m_ratio64, static_cast<double>(c) * static_cast<double>(scale),
                                      a.g_coef64 * static_cast<double>(g[e]));
      x[e] = __builtin_fabsf(x[e]) < 0x1p-14f * __builtin_fabsf(g[e]) ? static_cast<float>(ex) : x[e];
    }
  }
}

// The lane's largest |m_t| from exact values, for the groups whose maximum FELL: rare path, the
// chain run back to back.  The fp32 value of m_t = beta1 m + (1 - beta1) g carries the error of the
// dequantized m, at most about 2.1e-7 of beta1 * (old group maximum) whichever element it is (the
// inverse expansion's error grows with |log2(c/fmax) / k| while the element shrinks as 2 to minus
// that).  Against a new maximum of at least 3/8 of beta1 * (old maximum) that is below 6e-7 and the
// scale amax / fmax keeps six digits; only a group whose largest elements all cancelled (a few in
// 10^4 under heavy-tailed gradients), or whose codes were all small to begin with, falls below, and
// for those the maximum is taken from exact values: of EVERY element whose fp32 magnitude is within
// 2^-20 of beta1 * (old maximum) (m_fac) of the lane's largest -- more than twice the error above,
// so the exactly largest one is among them whichever of them fp32 happens to rank first.
template <class Mode>
__device__ __forceinline__ float exact_lane_max(const StepArgs& a, const Mode& md, const StepTables& tb,
                                                const LaneScratch& ls, const float (&x)[kEPL], float scale, float k,
                                                float inv_k, float m_fac) {
  float hi = 0.0f;
#pragma unroll
  for (int e = 0; e < kEPL; ++e) hi = __builtin_fmaxf(hi, __builtin_fabsf(x[e]));
  const float cut = __builtin_fmaf(-0x1p-20f, m_fac, hi);
  uint32_t candidates = 0u;
#pragma unroll
  for (int e = 0; e < kEPL; ++e) candidates |= __builtin_fabsf(x[e]) >= cut ? 1u << e : 0u;
  float best = 0.0f;
  while (candidates != 0u) {                         // one trip for nearly every lane
    const uint32_t idx = static_cast<uint32_t>(__builtin_ctz(candidates));
    candidates &= candidates - 1u;
    ExactChain<Mode> chain(a, md, tb, ls, idx, scale, k, inv_k);
    static_for<0, ExactChain<Mode>::kSteps + 1>([&](auto s) { chain.template step<s.value>(); });
    best = __builtin_fmaxf(best, __builtin_fabsf(chain.exact));
  }
  return best;
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
__device__ __forceinline__ float quantize_value(const Mode& md, float xv, const GroupQuant& gq, float unit) {
  if (md.expand()) {
    const float m = hw_exp2(__builtin_fmaf(hw_log2(__builtin_fabsf(xv) * gq.inv_a), gq.k, fmt_log2_max(md)));
    return SIGNED ? as_f32(as_u32(m) | (as_u32(xv) & 0x80000000u)) : m;
  }
  return gq.inv_a != 0.0f ? (xv * unit) / gq.scale : 0.0f;      // IEEE division: correctly rounded
}
template <bool SIGNED, class Mode>
__device__ __forceinline__ void quantize16(const Mode& md, const float (&x)[kEPL], const GroupQuant& gq,
                                           uint32_t (&c)[4], float unit) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    float q[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) q[b] = quantize_value<SIGNED>(md, x[4 * d + b], gq, unit);
    c[d] = md.e5m2() ? pack4<true>(q) : pack4<false>(q);
  }
}

// BF16-stored exponents only: a group whose stored exponent came out as exactly 1 is quantized
// linearly, code = FP8(x / scale), and its codes are re-made here with the correctly rounded
// quotient (the plain quantizer's arithmetic) in place of exp2(k log2 r + log2 fmax).  The two agree
// to 2^-22, which is all the other exponents need, but a linear map sends short-significand inputs
// onto exact rounding ties: at the first step from the zero state the inputs are bf16 gradients over
// a bf16 maximum, and 8 % of such a group's elements then sit exactly half way between two codes
// (measured), where only the exact quotient rounds the way the definition does.  About one group
// in 128 of those whose exponent is near 1; a lane-local rare branch.
template <bool SIGNED, class Mode>
__device__ __forceinline__ void requantize_linear_group(const Mode& md, const float (&x)[kEPL], const GroupQuant& gq,
                                                        uint32_t (&c)[4], float unit) {
  if (!(md.expand() && md.k16())) return;
  if (__builtin_expect(gq.k == 1.0f && gq.inv_a != 0.0f, 0)) {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      float q[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) q[b] = (x[4 * d + b] * unit) / gq.scale;     // IEEE division: correctly rounded
      c[d] = md.e5m2() ? pack4<true>(q) : pack4<false>(q);
    }
  }
}

// Re-encode element idx of the lane from the value xv (the exact one, see apply_exact_min) and put
// its code in place among the sixteen.  Rare path; same arithmetic as quantize16.
template <class Mode>
__device__ __forceinline__ void requantize_one(const Mode& md, float xv, const GroupQuant& gq, uint32_t idx,
                                               uint32_t (&c)[4], float unit) {
  float q;
  if (md.expand()) {
    const float m = hw_exp2(__builtin_fmaf(hw_log2(__builtin_fabsf(xv) * gq.inv_a), gq.k, fmt_log2_max(md)));
    q = as_f32(as_u32(m) | (as_u32(xv) & 0x80000000u));
  } else {
    q = gq.inv_a != 0.0f ? (xv * unit) / gq.scale : 0.0f;
  }
  const uint32_t code = (md.e5m2() ? __builtin_amdgcn_cvt_pk_bf8_f32(q, q, 0u, false)
                                   : __builtin_amdgcn_cvt_pk_fp8_f32(q, q, 0u, false)) & 0xffu;
  const uint32_t sh = 8u * (idx & 3u);
#pragma unroll
  for (int d = 0; d < 4; ++d)
    c[d] = (idx >> 2) == static_cast<uint32_t>(d) ? ((c[d] & ~(0xffu << sh)) | (code << sh)) : c[d];
}

// Two elements of one lane that both cancelled deeply: the smaller one is the lane's candidate and
// is exact (ExactChain); the other keeps its fp32 value, whose error at a depth of 2^-19 and more is
// a whole code step of the expanded group.  The pair is rare (a few in 10^11 elements) and costs
// nothing to look for: when the candidate itself came out below 2^-16 of its gradient (one lane in
// 10^4), the lane's other elements are tested the same way against the gradients kept in LDS, and
// any that qualifies is recomputed and re-encoded like the candidate.  It does not take part in the
// group's extremes any more (they are fixed by now): if it was the true minimum the group is one of
// those whose exponent is off, a case the candidate scheme already has.
template <class Mode>
__device__ __forceinline__ void requantize_other_cancelled(const StepArgs& a, const Mode& md, const StepTables& tb,
                                                           const LaneScratch& ls, const float (&x)[kEPL],
                                                           const GroupQuant& gq, uint32_t named, float scale, float k,
                                                           float inv_k, uint32_t (&c)[4], float unit) {
  uint32_t others = 0u;
#pragma unroll
  for (int e = 0; e < kEPL; ++e) {
    const float ge = as_f32(static_cast<uint32_t>(ls.g[e]) << 16);
    others |= __builtin_fabsf(x[e]) < 0x1p-16f * __builtin_fabsf(ge) ? 1u << e : 0u;
  }
  others &= ~(1u << named);
  while (others != 0u) {
    const uint32_t idx = static_cast<uint32_t>(__builtin_ctz(others));
    others &= others - 1u;
    ExactChain<Mode> chain(a, md, tb, ls, idx, scale, k, inv_k);
    static_for<0, ExactChain<Mode>::kSteps + 1>([&](auto s) { chain.template step<s.value>(); });
    requantize_one(md, chain.exact, gq, idx, c, unit);
  }
}

}  // namespace
