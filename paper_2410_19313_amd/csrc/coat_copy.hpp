// coat_copy.hpp -- the copy control: the step's memory traffic without its arithmetic
// Part of the one translation unit coat_kernels.hip (included from there, in this order).
#pragma once

namespace {

// A measurement aid, not part of the method: a kernel that moves exactly the bytes the fused step
// moves (per element: w 4 + g 2 + two code bytes read, w 4 + two code bytes written; per group:
// four metadata words read and written) in the step's access pattern (one 1024-element chunk per
// wavefront, 16-byte rows, streaming hints, the admission gate, the same launch shape and LDS
// footprint), with next to no arithmetic: w <- w + g, the code arrays swap, the metadata is
// written back.  What it reaches is the ceiling this access pattern has on the machine; the step's
// bandwidth is reported beside it.
template <int G>
__global__ __launch_bounds__(kBlock) void copy_control_kernel(StepArgs a) {
  constexpr int LPG = G / kEPL;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint64_t chunk = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv;
  if (chunk >= a.n_full) return;
  chunk = gate_on_neighbourhood(a.mk, chunk, kChunk / G);
  RawChunk r;
  issue_loads<G>(a, DefaultMode(), DefaultMode(), chunk, lane, r);
  const uint64_t cb = chunk * kChunk, gb = chunk * (kChunk / G);
  // gradient row j covers the elements of weight rows 2j and 2j+1 only in bulk, not per lane; the
  // control adds the bf16 pairs a lane holds to the weights it holds, which is arithmetic enough
  f32x4* wq = reinterpret_cast<f32x4*>(a.w + cb);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const u32x4 gp = r.g[j >> 1];
    f32x4 t = r.w[j];
    t.x += as_f32(gp.x << 16); t.y += as_f32(gp.y << 16); t.z += as_f32(gp.z << 16); t.w += as_f32(gp.w << 16);
    stg<16>(wq + 64 * j + lane, t);
  }
  stg<2>(reinterpret_cast<u32x4*>(a.mq + cb) + lane, r.vc);
  stg<2>(reinterpret_cast<u32x4*>(a.vq + cb) + lane, r.mc);
  if ((lane % LPG) == 0) {
    const int gl = lane / LPG;
    a.ms[gb + gl] = r.meta.m_scale; a.mk[gb + gl] = r.meta.m_k;
    a.vs[gb + gl] = r.meta.v_scale; a.vk[gb + gl] = r.meta.v_k;
  }
}

}  // namespace
