// coat_act.hpp -- the activation quantizers of Sec. 5.2 (1xG per group; per tensor with Group Scaling)
// Part of the one translation unit coat_kernels.hip (included from there, in this order).
#pragma once

namespace {

// ---------------------------------------------------------------------------------------
// activation quantizers (Sec. 5.2): bf16 in, E4M3 codes out, no expansion.  Same lane layout as the
// optimizer kernels (16 consecutive elements per lane, rows staged through the bf16 tile), so a
// 1 x 16 group is exactly one lane and larger groups are the same DPP butterflies.
// ---------------------------------------------------------------------------------------

struct ActArgs {
  const uint16_t* x;
  uint8_t* q;
  float* per_group;        // per-group scales (1xG quantizer) or per-group maxima (Group Scaling stage 1)
  float* partial;          // Group Scaling: one partial maximum per workgroup of the reducing launch (caller's workspace)
  int n_partial;           // how many of them are written (<= COAT_ACT_WORKSPACE_FLOATS)
  int tail_slot;           // where the ragged last chunk's launch leaves its maximum
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

// The end of Group Scaling's reduction: every workgroup of the quantizing launch folds the partial
// maxima (at most COAT_ACT_WORKSPACE_FLOATS, a few per thread, served by the L2) itself; all threads
// return the tensor maximum.  part: one LDS word per wavefront of the workgroup.
__device__ __forceinline__ float act_wave_max(float hi) {
  hi = group_allreduce<32, true>(hi);
  return __builtin_fmaxf(hi, __shfl_xor(hi, 32));
}
__device__ __forceinline__ float act_fold_partials(const ActArgs& a, float* part) {
  float hi = 0.0f;
  for (int i = threadIdx.x; i < a.n_partial; i += blockDim.x) hi = __builtin_fmaxf(hi, a.partial[i]);
  hi = act_wave_max(hi);
  const int waves = blockDim.x / kWave;
  if (waves == 1) return hi;
  if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x >> 6] = hi;
  __syncthreads();
  hi = part[0];
  for (int w = 1; w < waves; ++w) hi = __builtin_fmaxf(hi, part[w]);
  return hi;
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
    __shared__ float part[kWavesPerBlock];
    tmax = act_fold_partials(a, part);
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
    amax = act_fold_partials(a, nullptr);            // one wavefront: no LDS needed
    if (lane == 0) { *a.tensor_amax = amax; *a.tensor_scale = amax / 448.0f; }
  } else {
    amax = act_group_amax<G>(x);
  }
  const float s = act_quantize16(x, amax, c);
  store_codes16_guarded(a.q, base, a.n, c);
  if constexpr (!PER_TENSOR)
    if (gidx < a.n_groups && (lane % LPG) == 0) a.per_group[gidx] = s;
}

// Group Scaling stage 1: the maximum of every 1xG group, kept as an intermediate tensor.  Every
// workgroup also leaves the maximum of what it saw in its slot of the workspace, so that the
// reduction over the intermediate tensor (stage 2) costs no pass and no launch of its own here: the
// quantizing launch folds the slots.  The grid is capped at the number of slots and loops.
template <int G>
__global__ __launch_bounds__(kBlock) void act_group_amax_kernel(ActArgs a) {
  __shared__ u32x4 tile_x[kWavesPerBlock * kTileSlotsG];
  __shared__ float part[kWavesPerBlock];
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kWavesPerBlock;
  float seen = 0.0f;
  for (uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv; chunk < a.n_full; chunk += stride) {
    float x[kEPL];
    act_load_chunk(a.x, chunk * kChunk, tile_x + wv * kTileSlotsG, lane, x);
    const float amax = act_group_amax<G>(x);
    if ((lane % LPG) == 0) a.per_group[chunk * (kChunk / G) + lane / LPG] = amax;
    seen = __builtin_fmaxf(seen, amax);
  }
  seen = act_wave_max(seen);
  if (lane == 0) part[wv] = seen;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kWavesPerBlock; ++w) seen = __builtin_fmaxf(seen, part[w]);
    a.partial[blockIdx.x] = seen;
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
  const float seen = act_wave_max(amax);             // lanes beyond n hold zeros
  if (lane == 0) a.partial[a.tail_slot] = seen;
}

// Group Scaling stage 2 for a caller who brings the group maxima (the producing operator wrote
// them): the maximum of the G-times smaller tensor.  At most 64 large workgroups each fold a strided
// share and store one partial maximum; the quantizing kernel that follows folds those.  No atomics (same-address atomic maxima serialize
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

}  // namespace
