// coat_quant.hpp -- the standalone per-group quantizer and dequantizer (the two halves of the step)
// Part of the one translation unit coat_kernels.hip (included from there, in this order).
#pragma once

namespace {

// ---------------------------------------------------------------------------------------
// standalone quantizer / dequantizer (the two halves of the step), format and expansion at run time
// ---------------------------------------------------------------------------------------

// quantize one lane's 16 values (cross-lane: the group reductions) and hand back codes + metadata
template <int G, class Mode>
__device__ __forceinline__ GroupQuant quant_core_as(const Mode& md, const QuantArgs& a, const float (&x)[kEPL], uint32_t (&c)[4]) {
  constexpr int LPG = G / kEPL;
  float hi, lo;
  lane_extremes(x, hi, lo);
  hi = group_allreduce<LPG, true>(hi);
  lo = group_allreduce<LPG, false>(lo);
  const GroupQuant q = group_quant_params(md, hi, lo, a.k_min, a.k_max, 1.0f);
  quantize16<true>(md, x, q, c, 1.0f);
  requantize_linear_group<true>(md, x, q, c, 1.0f);
  return q;
}
// Format and expansion are wavefront-uniform run-time values; one branch per chunk picks the code
// with both folded (left as per-element selects they compile to a hundred short basic blocks).
template <int G>
__device__ __forceinline__ GroupQuant quant_core(const QuantArgs& a, const float (&x)[kEPL], uint32_t (&c)[4]) {
  const bool s16 = a.mode.scale16(), kh = a.mode.k16();
  if (a.mode.expand()) {
    if (a.mode.e5m2()) return quant_core_as<G>(FoldedMode<true, true>{s16, kh}, a, x, c);
    return quant_core_as<G>(FoldedMode<false, true>{s16, kh}, a, x, c);
  }
  if (a.mode.e5m2()) return quant_core_as<G>(FoldedMode<true, false>{s16, kh}, a, x, c);
  return quant_core_as<G>(FoldedMode<false, false>{s16, kh}, a, x, c);
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
    // (measured: 871 -> 845 us on 2^30 elements with the gate; spans of 16 / 32 / 64 / 128 chunks alike)
    chunk = gate_on_neighbourhood(a.x, chunk, kChunk);
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
    if ((lane % LPG) == 0) { store_scale(a.mode, a.scale, gb + lane / LPG, q.scale); store_k(a.mode, a.k, gb + lane / LPG, q.k); }
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
  if (gidx < a.n_groups && (lane % LPG) == 0) { store_scale(a.mode, a.scale, gidx, q.scale); store_k(a.mode, a.k, gidx, q.k); }
}

// The standalone dequantizer always honours the stored k (it is 1 for codes written without
// expansion), with the compensated exponent.
// The dequantizer needs one format's table only; it sits at the front of the LDS array.
__device__ __forceinline__ void fill_lut_one(Log2Entry* lut, bool e5m2) {
  for (int i = threadIdx.x; i < 256; i += blockDim.x) lut[i] = kLog2Code[e5m2 ? 1 : 0][i & 127];
  __syncthreads();
}

__device__ __forceinline__ void dequant_core(const DequantArgs& a, const Log2Entry* lut, const u32x4& ci, float scale,
                                             float k, float (&x)[kEPL]) {
  const uint32_t c[4] = {ci.x, ci.y, ci.z, ci.w};
  inverse_expand16<true, 2>(lut, c, k, hw_rcp(k), x);
  const float amag = fmt_max(a.mode) * scale;
#pragma unroll
  for (int e = 0; e < kEPL; ++e) x[e] *= amag;
}

// One chunk per wavefront; the first chunk's codes and metadata are requested before the block
// fills its table, so the table's latency hides behind them.
template <int G>
__global__ __launch_bounds__(kBlock) void dequant_kernel(DequantArgs a) {
  __shared__ Log2Entry lut[256];
  __shared__ f32x4 tile_x[kWavesPerBlock * kTileSlotsW];
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv;
  const bool have = chunk < a.n_full;
  u32x4 ci = {0u, 0u, 0u, 0u};
  float scale = 0.0f, k = 1.0f;
  // the admission gate of the step kernel, keyed on the exponents, over 64 chunks (measured on 6.7e9
  // elements: no gate 6.03 ms, spans of 16 / 32 / 64 / 128 chunks 5.66 / 5.49 / 5.44 / 5.43 ms; two chunks
  // per wavefront 6.15 ms; the table requested ahead of the gate, as the step kernel does, 6.2 ms)
  if (have) chunk = gate_on_neighbourhood<64>(a.k, chunk, a.mode.k16() ? kChunk / G / 2 : kChunk / G);
  if (have) {
    ci = ldg<1>(reinterpret_cast<const u32x4*>(a.q + chunk * kChunk) + lane);
    scale = load_scale_full_chunk(a.mode, a.scale, chunk * (kChunk / G), lane / LPG);
    k = load_k_full_chunk(a.mode, a.k, chunk * (kChunk / G), lane / LPG);
  }
  fill_lut_one(lut, a.mode.e5m2());                  // every wavefront of the block reaches this
  float x[kEPL];
  if (have) {
    dequant_core(a, lut, ci, scale, k, x);
    tile_lanes_to_rows_store(tile_x + wv * kTileSlotsW, lane, x, a.x + chunk * kChunk);
  }
  for (chunk += stride; chunk < a.n_full; chunk += stride) {
    const uint64_t gb = chunk * (kChunk / G);
    ci = ldg<1>(reinterpret_cast<const u32x4*>(a.q + chunk * kChunk) + lane);
    dequant_core(a, lut, ci, load_scale_full_chunk(a.mode, a.scale, gb, lane / LPG), load_k_full_chunk(a.mode, a.k, gb, lane / LPG), x);
    tile_lanes_to_rows_store(tile_x + wv * kTileSlotsW, lane, x, a.x + chunk * kChunk);
  }
}

template <int G>
__global__ __launch_bounds__(kWave) void dequant_tail_kernel(DequantArgs a) {
  __shared__ Log2Entry lut[256];
  fill_lut_one(lut, a.mode.e5m2());
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x;
  const uint64_t base = a.n_full * kChunk + static_cast<uint64_t>(lane) * kEPL;
  const uint64_t gidx = a.n_full * (kChunk / G) + static_cast<uint64_t>(lane / LPG);
  const bool gvalid = gidx < a.n_groups;
  uint32_t c[4];
  float x[kEPL];
  load_codes16_guarded(a.q, base, a.n, c);
  const u32x4 ci = {c[0], c[1], c[2], c[3]};
  dequant_core(a, lut, ci, gvalid ? load_scale(a.mode, a.scale, gidx) : 0.0f, gvalid ? load_k(a.mode, a.k, gidx) : 1.0f, x);
  store_f32x16_guarded(a.x, base, a.n, x);
}

}  // namespace
