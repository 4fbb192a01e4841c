// coat_step.hpp -- the fused FP8-state AdamW step: per-lane arithmetic, chunk load/store, admission gate, kernels
// Part of the one translation unit coat_kernels.hip (included from there, in this order).
#pragma once

namespace {

// ---------------------------------------------------------------------------------------
// the fused step
// ---------------------------------------------------------------------------------------

// Per-group metadata of one chunk as one lane sees it (its own group's words).
struct GroupMeta { float m_scale, m_k, v_scale, v_k; };

// The arithmetic of the step on one lane's 16 elements, registers in, registers out:
// w (in/out), g, codes (in/out), metadata (in/out).  Cross-lane traffic: the group reductions.
// ls: the lane's old first-moment codes and its gradients once more, in LDS, for the one element
// per lane that is looked up by a run-time index (exact_candidate).
template <int G, class ModeM, class ModeV>
__device__ __forceinline__ void step_core(const StepArgs& a, const ModeM& mm, const ModeV& mv,
                                          const StepTables& tb, const LaneScratch& ls, float (&w)[kEPL],
                                          const float (&g)[kEPL], uint32_t (&mc)[4], uint32_t (&vc)[4],
                                          GroupMeta& meta) {
  constexpr int LPG = G / kEPL;                      // lanes per group
  float m[kEPL], v[kEPL];
  const float m_inv_k = hw_rcp(meta.m_k);
  // beta/(1-beta) * (magnitude of the decoded unit)
  const float m_fac = a.beta1_ratio * dequant16<true, false>(mm, tb.lut, mc, meta.m_scale, meta.m_k, m_inv_k, m);
  const float v_fac = a.beta2_ratio * dequant16<false, false>(mv, tb.lut, vc, meta.v_scale, meta.v_k, hw_rcp(meta.v_k), v);

#pragma unroll
  for (int e = 0; e < kEPL; ++e) {
    const float ge = g[e];
    const float m_t = __builtin_fmaf(m[e], m_fac, ge);              // m_t / (1 - beta1), Sec. 3
    const float v_t = __builtin_fmaf(ge, ge, v[e] * v_fac);         // v_t / (1 - beta2)
    // Eq. (1) with the unquantized new moments, step size and bias corrections inside the denominator
    const float denom = __builtin_fmaf(hw_sqrt(v_t), a.denom_mul, a.denom_add);
    w[e] = __builtin_fmaf(w[e], a.w_keep, m_t * hw_rcp(denom));
    m[e] = m_t;
    v[e] = v_t;
  }

  // Extremes.  The first moment's minimum fixes k and is where the update cancels: its element is
  // recomputed exactly (exact_candidate), a long dependent chain beside which the second moment
  // is quantized; the rare branches stay outside that stretch of straight-line code.
  float m_max, v_max, v_min;
  uint32_t m_key;
  lane_extremes_keyed(m, g, m_max, m_key);
  lane_extremes(v, v_max, v_min);
  float m_exact = exact_candidate(a, mm, tb, ls, m_key, meta.m_scale, meta.m_k, m_inv_k);
  v_max = group_allreduce<LPG, true>(v_max);
  v_min = group_allreduce<LPG, false>(v_min);
  const GroupQuant qv = group_quant_params(mv, v_max, v_min, a.k_min, a.k_max, a.one_minus_beta2);
  quantize16<false>(mv, v, qv, vc, a.one_minus_beta2);
  // (empty asm: holds the second moment's codes and the exact value at one point of the program, so
  // that the compiler does not sink the quantization above past the rare branch that follows)
  asm volatile("" : "+v"(vc[0]), "+v"(vc[1]), "+v"(vc[2]), "+v"(vc[3]), "+v"(m_exact));
  bool m_replace;
  float m_min = apply_exact_min(m_exact, m_key, m, m_max, m_replace);
  m_max = group_allreduce<LPG, true>(m_max);
  m_min = group_allreduce<LPG, false>(m_min);
  const GroupQuant qm = group_quant_params(mm, m_max, m_min, a.k_min, a.k_max, a.one_minus_beta1);
  quantize16<true>(mm, m, qm, mc, a.one_minus_beta1);
  if (__builtin_expect(m_replace, 0)) requantize_one(mm, m_exact, qm, m_key & 15u, mc, a.one_minus_beta1);
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
                                              const StepTables& tb, const StageTiles& tiles, uint64_t chunk,
                                              int lane, RawChunk& r) {
  constexpr int LPG = G / kEPL;
  const uint64_t cb = chunk * kChunk;
  const uint64_t gb = chunk * (kChunk / G);

  float w[kEPL], g[kEPL];
  tile_rows_to_lanes_bf16(tiles.g, lane, r.g, g);
  tile_rows_to_lanes(tiles.w, lane, r.w, w);
  // The weights are in registers now and the fp32 tile is free until they are staged back: the
  // first of this lane's own slots keeps the old first-moment codes; the gradient tile still holds
  // the lane's 16 gradients as consecutive bf16.
  f32x4* const own_w = tiles.w + 4 * lane + (lane >> 1);
  *own_w = __builtin_bit_cast(f32x4, r.mc);          // same type as the tile's other accesses: kept in order
  const LaneScratch ls = {reinterpret_cast<const uint8_t*>(own_w),
                          reinterpret_cast<const lds_u16*>(tiles.g + 2 * lane + (lane >> 2))};
  uint32_t mc[4] = {r.mc.x, r.mc.y, r.mc.z, r.mc.w};
  uint32_t vc[4] = {r.vc.x, r.vc.y, r.vc.z, r.vc.w};
  GroupMeta meta = r.meta;

  step_core<G>(a, mm, mv, tb, ls, w, g, mc, vc, meta);

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
  __shared__ double frac[kExp2Frac];
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
  fill_lut<kTables, kBlock>(lut, frac);              // every wavefront of the block reaches this
  const StepTables tb = {lut, frac};
  if (have) process_chunk<G>(a, mm, mv, tb, tiles, chunk, lane, r);
  for (chunk += stride; chunk < a.n_full; chunk += stride) {
    issue_loads<G>(a, mm, mv, chunk, lane, r);
    process_chunk<G>(a, mm, mv, tb, tiles, chunk, lane, r);
  }
}

// The ragged last chunk (n % 1024 elements): one wavefront, element-wise guarded accesses
// straight into the lane layout.  slots: three 16-byte LDS slots of this lane's own (old codes,
// gradients as bf16) for step_core's indexed lookup.
template <int G, class ModeM, class ModeV>
__device__ __forceinline__ void process_tail_chunk(const StepArgs& a, const ModeM& mm, const ModeV& mv,
                                                   const StepTables& tb, u32x4* slots, int lane) {
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
  {
    const u32x4 c = {mc[0], mc[1], mc[2], mc[3]};
    slots[0] = c;
    uint32_t gb[8];                                  // a bf16 gradient is the upper half of its fp32
#pragma unroll
    for (int i = 0; i < 8; ++i) gb[i] = (as_u32(g[2 * i + 1]) & 0xffff0000u) | (as_u32(g[2 * i]) >> 16);
    const u32x4 g0 = {gb[0], gb[1], gb[2], gb[3]}, g1 = {gb[4], gb[5], gb[6], gb[7]};
    slots[1] = g0; slots[2] = g1;
  }
  const LaneScratch ls = {reinterpret_cast<const uint8_t*>(slots), reinterpret_cast<const lds_u16*>(slots + 1)};
  step_core<G>(a, mm, mv, tb, ls, w, g, mc, vc, meta);
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
  __shared__ double frac[kExp2Frac];
  __shared__ u32x4 slots[3 * kWave];
  fill_lut<kTables, kWave>(lut, frac);
  const StepTables tb = {lut, frac};
  const typename ModesOf<GENERIC>::M mm = ModesOf<GENERIC>::m(a), mv = ModesOf<GENERIC>::v(a);
  process_tail_chunk<G>(a, mm, mv, tb, slots + 3 * threadIdx.x, threadIdx.x);
}

}  // namespace
