// coat_multi.hpp -- the multi-tensor step: plan records and the kernel that looks a chunk's tensor up
// Part of the one translation unit coat_kernels.hip (included from there, in this order).
#pragma once

namespace {

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

}  // namespace
