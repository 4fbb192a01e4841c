// coat_step.hpp -- the fused FP8-state AdamW step: per-lane arithmetic, chunk load/store, admission gate, kernels
// Part of the one translation unit coat_kernels.hip (included from there, in this order).
#pragma once

namespace {

// ---------------------------------------------------------------------------------------
// the fused step
// ---------------------------------------------------------------------------------------

// Per-group metadata of one chunk as one lane sees it (its own group's words).
struct GroupMeta { float m_scale, m_k, v_scale, v_k; };

// The arithmetic of the step on one lane's 16 elements.  Codes and metadata come in registers;
// everything else goes through `io`, in the order in which the data is needed and produced, so
// that a wavefront works on what has arrived and sends off what is final while the rest is still
// in flight or being computed (the loads are issued in that order too: codes, metadata,
// weights, gradients):
//   the moments are dequantized from codes and metadata alone;
//   io.gradients(g), io.old_weights(w) then hand over the lane's 16 gradients and weights;
//   io.weights(w) takes the new weights right after the update, before the moments are requantized;
//   io.second(codes, scale, k) after the second moment's quantization, io.first(...) at the end.
// (With all stores issued at the end, behind the rare branches of the requantization, the 7B step
// took 3 % longer.)  Cross-lane traffic: the group reductions.
// ls: the lane's old first-moment codes and its gradients once more, in LDS, for the one element
// per lane that is looked up by a run-time index (ExactChain).
template <int G, class ModeM, class ModeV, class IO>
__device__ __forceinline__ void step_core(const StepArgs& a, const ModeM& mm, const ModeV& mv,
                                          const StepTables& tb, const LaneScratch& ls, uint32_t (&mc)[4],
                                          uint32_t (&vc)[4], const GroupMeta& meta, IO&& io) {
  constexpr int LPG = G / kEPL;                      // lanes per group
  float m[kEPL], v[kEPL];
  const float m_inv_k = hw_rcp(meta.m_k);
  // beta/(1-beta) * (magnitude of the decoded unit)
  const float m_fac = a.beta1_ratio * dequant16<true, ModeM::kDq>(mm, tb.lut, mc, meta.m_scale, meta.m_k, m_inv_k, m);
  const float v_fac = a.beta2_ratio * dequant16<false, ModeV::kDq>(mv, tb.lut, vc, meta.v_scale, meta.v_k, hw_rcp(meta.v_k), v);
  __builtin_amdgcn_sched_barrier(0);
  float w[kEPL], g[kEPL];
  io.gradients(g);
  io.old_weights(w);

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
  io.weights(w);
  __builtin_amdgcn_sched_barrier(0);

  // Extremes.  The first moment's minimum fixes k and is where the update cancels: its element is
  // recomputed exactly (ExactChain), a long chain of dependent steps; the second moment's
  // quantization, which does not depend on it, is dealt out between the steps, one element each,
  // and a scheduling barrier after every step keeps the compiler from undoing the interleave.
  // The rare branches stay outside this stretch of straight-line code.
  float m_max, v_max, v_min;
  uint32_t m_key;
  if (!mm.expand() && mm.e5m2()) recompute_cancelled_plain(a, mm, ls, meta.m_scale, g, m);
  lane_extremes_keyed(m, g, m_max, m_key);
  lane_extremes(v, v_max, v_min);
  ExactChain<ModeM> chain(a, mm, tb, ls, m_key, meta.m_scale, meta.m_k, m_inv_k);
  chain.template step<0>();
  v_max = group_allreduce<LPG, true>(v_max);
  v_min = group_allreduce<LPG, false>(v_min);
  const GroupQuant qv = group_quant_params(mv, v_max, v_min, a.k_min, a.k_max, a.one_minus_beta2);
  __builtin_amdgcn_sched_barrier(0);
  float vq[kEPL];
  static_for<0, kEPL>([&](auto e) {
    chain.template step<e.value + 1>();
    vq[e.value] = quantize_value<false>(mv, v[e.value], qv, a.one_minus_beta2);
    __builtin_amdgcn_sched_barrier(0);
  });
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const float q4[4] = {vq[4 * d], vq[4 * d + 1], vq[4 * d + 2], vq[4 * d + 3]};
    vc[d] = mv.e5m2() ? pack4<true>(q4) : pack4<false>(q4);
  }
  requantize_linear_group<false>(mv, v, qv, vc, a.one_minus_beta2);
  float m_exact = chain.exact;
  // (empty asm: holds the second moment's codes and the exact value at one point of the program, so
  // that the compiler does not sink the quantization above past the rare branch that follows)
  asm volatile("" : "+v"(vc[0]), "+v"(vc[1]), "+v"(vc[2]), "+v"(vc[3]), "+v"(m_exact));
  io.second(vc, qv.scale, qv.k);
  __builtin_amdgcn_sched_barrier(0);
  bool m_replace;
  float m_min = apply_exact_min(m_exact, chain.g32, m_key, m, m_max, m_replace);
  m_max = group_allreduce<LPG, true>(m_max);
  m_min = group_allreduce<LPG, false>(m_min);
  if (mm.expand()) {
    // a group whose maximum fell below 3/8 of beta1 * (its old maximum): see exact_lane_max.  The
    // branch is taken by whole wavefronts (the butterflies inside need every lane); only the groups
    // concerned adopt the result, so a group's outcome does not depend on its neighbours.
    const bool fell = m_max < 0.375f * m_fac;
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(fell) != 0ull, 0)) {
      const float ex = group_allreduce<LPG, true>(exact_lane_max(a, mm, tb, ls, m, meta.m_scale, meta.m_k, m_inv_k, m_fac));
      m_max = fell ? ex : m_max;
    }
  }
  const GroupQuant qm = group_quant_params(mm, m_max, m_min, a.k_min, a.k_max, a.one_minus_beta1);
  quantize16<true>(mm, m, qm, mc, a.one_minus_beta1);
  requantize_linear_group<true>(mm, m, qm, mc, a.one_minus_beta1);
  if (__builtin_expect(m_replace, 0)) requantize_one(mm, m_exact, qm, m_key & 15u, mc, a.one_minus_beta1);
  if (mm.expand()) {
    const bool deep = m_key != 0xffffffffu && __builtin_fabsf(m_exact) < 0x1p-16f * __builtin_fabsf(chain.g32);
    if (__builtin_expect(deep, 0))
      requantize_other_cancelled(a, mm, tb, ls, m, qm, m_key & 15u, meta.m_scale, meta.m_k, m_inv_k, mc, a.one_minus_beta1);
  }
  io.first(mc, qm.scale, qm.k);
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
  // in the order of use (loads return in order): codes and metadata feed the dequantization,
  // which runs while the weights and the gradients are still on their way (measured on the 7B set,
  // same run: this order 14.84 ms; metadata, codes, gradients, weights 14.94; weights first 14.91)
  r.mc = ldg<1>(mq + lane);
  r.vc = ldg<1>(vq + lane);
  r.meta.m_scale = load_scale_full_chunk(mm, a.ms, gb, gl);
  r.meta.v_scale = load_scale_full_chunk(mv, a.vs, gb, gl);
  r.meta.m_k = load_k_full_chunk(mm, a.mk, gb, gl);          // written as 1 (and ignored) by a moment stored without expansion
  r.meta.v_k = load_k_full_chunk(mv, a.vk, gb, gl);
#pragma unroll
  for (int j = 0; j < 4; ++j) r.w[j] = ldg<8>(wq + 64 * j + lane);
#pragma unroll
  for (int j = 0; j < 2; ++j) r.g[j] = ldg<4>(gq + 64 * j + lane);
}

// One full chunk: rows -> lane layout through the LDS tiles, the arithmetic, and back out.
template <int G, class ModeM, class ModeV>
__device__ __forceinline__ void process_chunk(const StepArgs& a, const ModeM& mm, const ModeV& mv,
                                              const StepTables& tb, const StageTiles& tiles, uint64_t chunk,
                                              int lane, RawChunk& r) {
  constexpr int LPG = G / kEPL;
  const uint64_t cb = chunk * kChunk;
  const uint64_t gb = chunk * (kChunk / G);

  // For the look-up by index: the old first-moment codes go into the lane's slot of the code
  // scratch; the gradient tile will hold the lane's 16 gradients as consecutive bf16.
  tiles.codes[lane] = r.mc;
  const LaneScratch ls = {reinterpret_cast<const uint8_t*>(tiles.codes + lane),
                          reinterpret_cast<const lds_u16*>(tiles.g + 2 * lane + (lane >> 2))};
  uint32_t mc[4] = {r.mc.x, r.mc.y, r.mc.z, r.mc.w};
  uint32_t vc[4] = {r.vc.x, r.vc.y, r.vc.z, r.vc.w};

  struct IO {
    const StepArgs& a; const ModeM& mm; const ModeV& mv; const StageTiles& tiles; const RawChunk& r;
    uint64_t cb, gb; int lane;
    __device__ __forceinline__ void gradients(float (&g)[kEPL]) const { tile_rows_to_lanes_bf16(tiles.g, lane, r.g, g); }
    __device__ __forceinline__ void old_weights(float (&w)[kEPL]) const { tile_rows_to_lanes(tiles.w, lane, r.w, w); }
    __device__ __forceinline__ void weights(const float (&wn)[kEPL]) const {
      tile_lanes_to_rows_store(tiles.w, lane, wn, a.w + cb);
      // (the bf16 copy is staged through the fp32 tile too: its rows are in registers by now, and the
      // gradient tile is still needed)
      if (a.wb) tile_lanes_to_rows_store_bf16(reinterpret_cast<u32x4*>(tiles.w), lane, wn, a.wb + cb);
    }
    __device__ __forceinline__ void second(const uint32_t (&c)[4], float scale, float k) const {
      const u32x4 o = {c[0], c[1], c[2], c[3]};
      stg<2>(reinterpret_cast<u32x4*>(a.vq + cb) + lane, o);
      if ((lane % LPG) == 0) { store_scale(mv, a.vs, gb + lane / LPG, scale); store_k(mv, a.vk, gb + lane / LPG, k); }
    }
    __device__ __forceinline__ void first(const uint32_t (&c)[4], float scale, float k) const {
      const u32x4 o = {c[0], c[1], c[2], c[3]};
      stg<2>(reinterpret_cast<u32x4*>(a.mq + cb) + lane, o);
      if ((lane % LPG) == 0) { store_scale(mm, a.ms, gb + lane / LPG, scale); store_k(mm, a.mk, gb + lane / LPG, k); }
    }
  };
  step_core<G>(a, mm, mv, tb, ls, mc, vc, r.meta, IO{a, mm, mv, tiles, r, cb, gb, lane});
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
constexpr int kGateSpan = 32;
// `words`: any array of the operand with a fixed number of 32-bit words per chunk.
template <int SPAN = kGateSpan>
__device__ __forceinline__ uint64_t gate_on_neighbourhood(const void* words, uint64_t chunk, int words_per_chunk) {
  const uint64_t first = chunk & ~static_cast<uint64_t>(SPAN - 1);
  const uint32_t probe = __builtin_amdgcn_readfirstlane(static_cast<const uint32_t*>(words)[first * words_per_chunk]);
  uint32_t lo = static_cast<uint32_t>(chunk);
  asm volatile("" : "+s"(lo) : "s"(probe));
  return (chunk & 0xffffffff00000000ull) | lo;
}

// Which kernel serves a call: the default cell folded at compile time, the default cell with bf16
// metadata, or everything else with the storage modes as run-time values.
constexpr int kKindDefault = 0, kKindGeneric = 1, kKindBf16Meta = 2, kKindPrecise = 3;
template <int KIND> struct ModesOf;
template <> struct ModesOf<kKindDefault> {
  typedef DefaultMode M;
  __device__ static DefaultMode m(const StepArgs&) { return DefaultMode(); }
  __device__ static DefaultMode v(const StepArgs&) { return DefaultMode(); }
};
template <> struct ModesOf<kKindGeneric> {
  typedef RuntimeMode M;
  __device__ static RuntimeMode m(const StepArgs& a) { return a.mode_m; }
  __device__ static RuntimeMode v(const StepArgs& a) { return a.mode_v; }
};
template <> struct ModesOf<kKindPrecise> {
  typedef PreciseMode M;
  __device__ static PreciseMode m(const StepArgs&) { return PreciseMode(); }
  __device__ static PreciseMode v(const StepArgs&) { return PreciseMode(); }
};
template <> struct ModesOf<kKindBf16Meta> {
  typedef Bf16MetaMode M;
  __device__ static Bf16MetaMode m(const StepArgs& a) { return Bf16MetaMode{a.mode_m.s16, a.mode_m.kh}; }
  __device__ static Bf16MetaMode v(const StepArgs& a) { return Bf16MetaMode{a.mode_v.s16, a.mode_v.kh}; }
};

// Calls f(first-moment mode, second-moment mode) with the modes as far folded as the kind allows.
// The generic kind branches ONCE here, on the two expansion switches (wavefront-uniform), into one
// of four instantiations of f.
template <int KIND, class F>
__device__ __forceinline__ void with_folded_modes(const StepArgs& a, F&& f) {
  if constexpr (KIND == kKindGeneric) {
    if (a.mode_m.ex) {
      if (a.mode_v.ex) f(FormatMode<true>(a.mode_m), FormatMode<true>(a.mode_v));
      else f(FormatMode<true>(a.mode_m), FormatMode<false>(a.mode_v));
    } else {
      if (a.mode_v.ex) f(FormatMode<false>(a.mode_m), FormatMode<true>(a.mode_v));
      else f(FormatMode<false>(a.mode_m), FormatMode<false>(a.mode_v));
    }
  } else {
    f(ModesOf<KIND>::m(a), ModesOf<KIND>::v(a));
  }
}

// Main kernel: one chunk per wavefront (the loop only runs again for buffers with more chunks
// than the grid has wavefronts).  Order of the memory requests: the block's table entries, the
// gate's probe, the chunk's loads (see fill_issue).
// KIND = default : both moments E4M3 with expansion (the method as the paper runs it);
// KIND = bf16 meta: the same with scales and / or exponents stored as bf16;
// KIND = precise : the default cell with the more accurate inverse expansion;
// KIND = generic : per-moment format and expansion read from the arguments (Table 1's grid).
template <int G, int KIND>
__device__ __forceinline__ void adamw_step_body(const StepArgs& a) {
  constexpr int kTables = KIND == kKindGeneric ? 2 : 1;
  __shared__ Log2Entry lut[256 * kTables];
  __shared__ double frac[kExp2Frac];
  __shared__ f32x4 tile_w[kWavesPerBlock * kTileSlotsW];
  __shared__ u32x4 tile_g[kWavesPerBlock * kTileSlotsG];
  __shared__ u32x4 code_scratch[kBlock];
  const typename ModesOf<KIND>::M mm = ModesOf<KIND>::m(a), mv = ModesOf<KIND>::v(a);
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wavefront-uniform
  const StageTiles tiles = {tile_w + wv * kTileSlotsW, tile_g + wv * kTileSlotsG, code_scratch + wv * kWave};
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv;

  RawChunk r;
  bool have = chunk < a.n_full;                      // (only the generic kind's loop updates it)
  FillRegs<kTables, kBlock> fill;
  fill_issue(fill);
  if (have) chunk = gate_on_neighbourhood(a.mk, chunk, mm.k16() ? kChunk / G / 2 : kChunk / G);
  if (have) issue_loads<G>(a, mm, mv, chunk, lane, r);
  fill_commit(fill, lut, frac);                      // every wavefront of the block reaches this
  const StepTables tb = {lut, frac};
  if constexpr (KIND == kKindGeneric) {
    // one call site, so that the four variants exist once
    while (have) {
      with_folded_modes<KIND>(a, [&](const auto& fm, const auto& fv) { process_chunk<G>(a, fm, fv, tb, tiles, chunk, lane, r); });
      chunk += stride;
      have = chunk < a.n_full;
      if (have) issue_loads<G>(a, mm, mv, chunk, lane, r);
    }
  } else {
    // (this shape of the loop, with the first chunk outside it, measured 1.8 % faster on the 7B set
    // than the single-call-site form above: 14.89 against 15.16 ms, one process)
    if (have) process_chunk<G>(a, mm, mv, tb, tiles, chunk, lane, r);
    for (chunk += stride; chunk < a.n_full; chunk += stride) {
      issue_loads<G>(a, mm, mv, chunk, lane, r);
      process_chunk<G>(a, mm, mv, tb, tiles, chunk, lane, r);
    }
  }
}
template <int G, int KIND>
__global__ __launch_bounds__(kBlock) void adamw_step_kernel(StepArgs a) {
  static_assert(KIND != kKindGeneric, "the generic kind has its own entry");
  adamw_step_body<G, KIND>(a);
}
// The generic kind needs 170 to 177 vector registers when the allocator is left alone, a few more
// than the 168 that let three wavefronts share a SIMD -- and with two the CU holds two workgroups
// instead of the three the kernel is tuned for (17.7 ms against 15.9 on the 7B set).  Asked for
// three, the allocator fits it into 168 without spilling a vector register.
template <int G>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(3))) void adamw_step_generic_kernel(StepArgs a) {
  adamw_step_body<G, kKindGeneric>(a);
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
  meta.m_k = gvalid ? load_k(mm, a.mk, gidx) : 1.0f;
  meta.v_k = gvalid ? load_k(mv, a.vk, gidx) : 1.0f;
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
  struct IO {
    const StepArgs& a; const ModeM& mm; const ModeV& mv; const float (&w0)[kEPL]; const float (&g0)[kEPL];
    uint64_t base, gidx; bool store_meta;
    __device__ __forceinline__ void gradients(float (&g)[kEPL]) const {
#pragma unroll
      for (int e = 0; e < kEPL; ++e) g[e] = g0[e];
    }
    __device__ __forceinline__ void old_weights(float (&w)[kEPL]) const {
#pragma unroll
      for (int e = 0; e < kEPL; ++e) w[e] = w0[e];
    }
    __device__ __forceinline__ void weights(const float (&wn)[kEPL]) const {
      store_f32x16_guarded(a.w, base, a.n, wn);
      if (a.wb) {
#pragma unroll
        for (int e = 0; e < kEPL; e += 2) {
          const uint32_t pr = pack_bf16(wn[e], wn[e + 1]);
          if (base + e < a.n) a.wb[base + e] = static_cast<uint16_t>(pr);
          if (base + e + 1 < a.n) a.wb[base + e + 1] = static_cast<uint16_t>(pr >> 16);
        }
      }
    }
    __device__ __forceinline__ void second(const uint32_t (&c)[4], float scale, float k) const {
      store_codes16_guarded(a.vq, base, a.n, c);
      if (store_meta) { store_scale(mv, a.vs, gidx, scale); store_k(mv, a.vk, gidx, k); }
    }
    __device__ __forceinline__ void first(const uint32_t (&c)[4], float scale, float k) const {
      store_codes16_guarded(a.mq, base, a.n, c);
      if (store_meta) { store_scale(mm, a.ms, gidx, scale); store_k(mm, a.mk, gidx, k); }
    }
  };
  step_core<G>(a, mm, mv, tb, ls, mc, vc, meta, IO{a, mm, mv, w, g, base, gidx, gvalid && (lane % LPG) == 0});
}

template <int G, int KIND>
__global__ __launch_bounds__(kWave) void adamw_step_tail_kernel(StepArgs a) {
  constexpr int kTables = KIND == kKindGeneric ? 2 : 1;
  __shared__ Log2Entry lut[256 * kTables];
  __shared__ double frac[kExp2Frac];
  __shared__ u32x4 slots[3 * kWave];
  FillRegs<kTables, kWave> fill;
  fill_issue(fill);
  fill_commit(fill, lut, frac);
  const StepTables tb = {lut, frac};
  with_folded_modes<KIND>(a, [&](const auto& fm, const auto& fv) { process_tail_chunk<G>(a, fm, fv, tb, slots + 3 * threadIdx.x, threadIdx.x); });
}

}  // namespace
