// coat_multi.hpp -- the multi-tensor step: plan records and the kernel that looks a chunk's tensor up
// Part of the one translation unit coat_kernels.hip (included from there, in this order).
#pragma once

namespace {

// ---------------------------------------------------------------------------------------
// Many tensors in one launch.  The plan (built once on the host, resident in device memory) lays
// the tensors out in a VIRTUAL chunk space in which every tensor starts at a multiple of kGateSpan
// (32) chunks, and holds one 128-byte record per span of 32 virtual chunks: the tensor's pointers,
// its size and decay, and the index of the span's first chunk inside the tensor.  Wavefront gc
// reads record gc / 32 -- an address it can form by itself, so the lookup is ONE scalar load
// deep -- and from there on runs exactly the single-tensor code (full chunk, a tensor's ragged
// last chunk, or nothing for the padding at a tensor's end).  The record is read by all 32
// wavefronts of its span and by nobody else: it is at the same time the shared probe of the
// admission gate (see gate_on_neighbourhood), so this kernel needs no other.
// ---------------------------------------------------------------------------------------
struct PlanRecord {
  float* w; uint16_t* wb; const uint16_t* g;
  uint8_t* mq; float* ms; float* mk;
  uint8_t* vq; float* vs; float* vk;
  uint64_t n;               // elements of the tensor
  uint64_t chunk_base;      // index, inside the tensor, of this span's first chunk (a multiple of 32)
  float weight_decay;
  uint32_t tensor;          // index of the tensor in the caller's array (not read by the kernel)
  uint64_t reserved[4];
};
static_assert(sizeof(PlanRecord) == 128, "plan layout");

// The same record as the kernel reads it: pointers loaded from memory are generic to the compiler,
// which would cost flat_load / flat_store; typed as global memory they get the same global_load
// (scalar base + lane offset) forms as the single-tensor kernel's arguments.
#define COAT_GLOBAL_AS __attribute__((address_space(1)))
struct PlanRecordDev {
  COAT_GLOBAL_AS float* w; COAT_GLOBAL_AS uint16_t* wb; COAT_GLOBAL_AS const uint16_t* g;
  COAT_GLOBAL_AS uint8_t* mq; COAT_GLOBAL_AS float* ms; COAT_GLOBAL_AS float* mk;
  COAT_GLOBAL_AS uint8_t* vq; COAT_GLOBAL_AS float* vs; COAT_GLOBAL_AS float* vk;
  uint64_t n;
  uint64_t chunk_base;
  float weight_decay;
  uint32_t tensor;
  uint64_t reserved[4];
};
static_assert(sizeof(PlanRecordDev) == sizeof(PlanRecord), "plan layout");

struct PlanHeader {
  uint64_t magic;
  uint32_t version, count;
  uint64_t total_records;
  uint64_t record_offset, bytes;
  uint64_t reserved[3];
};
static_assert(sizeof(PlanHeader) == 64, "plan layout");
constexpr uint64_t kPlanMagic = 0x324e4c5054414f43ull;     // "COATPLN2"
constexpr int kPlanSpan = kGateSpan;                        // virtual chunks per record
static_assert(kPlanSpan % kWavesPerBlock == 0, "a workgroup never straddles two records");

// The numbers of a step that change from one step to the next (learning-rate schedule, bias
// corrections).  Normally they travel as kernel arguments; a caller that replays a captured graph
// keeps them in device memory instead and rewrites these 32 bytes between replays.
struct StepConsts {
  float denom_mul;           // sqrt((1 - beta2) / (1 - beta2^t)) / c,  c = -lr (1 - beta1) / (1 - beta1^t)
  float denom_add;           // eps / c   (lr == 0: denom_mul = 0, denom_add = +inf)
  double neg_lr;             // -lr
  uint64_t reserved[2];
};
static_assert(sizeof(StepConsts) == sizeof(coat_step_consts), "C ABI mirror");

struct MultiArgs {
  StepArgs base;             // the shared hyper-parameter constants; pointers and sizes are per tensor
  const PlanRecord* records;
  double neg_lr;             // -lr: the decay factor -lr * lambda is formed per tensor, in fp64 like the host does
  const StepConsts* consts;  // nullptr: the step's constants are the arguments above
};

template <int G, int KIND>
__global__ __launch_bounds__(kBlock) void adamw_step_multi_kernel(MultiArgs ma) {
  constexpr int kTables = KIND == kKindGeneric ? 2 : 1;
  __shared__ Log2Entry lut[256 * kTables];
  __shared__ double frac[kExp2Frac];
  __shared__ f32x4 tile_w[kWavesPerBlock * kTileSlotsW];
  __shared__ u32x4 tile_g[kWavesPerBlock * kTileSlotsG];
  __shared__ u32x4 code_scratch[kBlock];
  const typename ModesOf<KIND>::M mm = ModesOf<KIND>::m(ma.base), mv = ModesOf<KIND>::v(ma.base);
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const StageTiles tiles = {tile_w + wv * kTileSlotsW, tile_g + wv * kTileSlotsG, code_scratch + wv * kWave};
  // the grid covers the virtual chunk space exactly (kPlanSpan / kWavesPerBlock workgroups per record)
  const uint64_t gc = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wv;
  FillRegs<kTables, kBlock> fill;
  fill_issue(fill);                                  // the table entries are requested before anything else

  // everything here is uniform over the wavefront (gc is), so the record travels in scalar registers
  const PlanRecordDev& d = reinterpret_cast<const PlanRecordDev*>(ma.records)[gc / kPlanSpan];
  StepArgs a = ma.base;
  double neg_lr = ma.neg_lr;
  if (ma.consts) {                                   // uniform: three scalar loads beside the record's
    a.denom_mul = ma.consts->denom_mul;
    a.denom_add = ma.consts->denom_add;
    neg_lr = ma.consts->neg_lr;
  }
  a.w = (float*)d.w; a.wb = (uint16_t*)d.wb; a.g = (const uint16_t*)d.g;
  a.mq = (uint8_t*)d.mq; a.ms = (float*)d.ms; a.mk = (float*)d.mk;
  a.vq = (uint8_t*)d.vq; a.vs = (float*)d.vs; a.vk = (float*)d.vk;
  a.n = d.n; a.n_full = d.n / kChunk;
  a.n_groups = (d.n + G - 1) / G;
  a.w_keep = static_cast<float>(1.0 + neg_lr * static_cast<double>(d.weight_decay));
  const uint64_t chunk = d.chunk_base + (gc % kPlanSpan);
  const bool full = chunk < a.n_full;
  const bool tail = !full && chunk * kChunk < a.n;     // the tensor's ragged last chunk; beyond it: padding

  RawChunk r;
  if (full) issue_loads<G>(a, mm, mv, chunk, lane, r);
  fill_commit(fill, lut, frac);                      // every wavefront of the block reaches this
  const StepTables tb = {lut, frac};
  if (full)
    with_folded_modes<KIND>(a, [&](const auto& fm, const auto& fv) { process_chunk<G>(a, fm, fv, tb, tiles, chunk, lane, r); });
  else if (tail)
    with_folded_modes<KIND>(a, [&](const auto& fm, const auto& fv) {
      process_tail_chunk<G>(a, fm, fv, tb, reinterpret_cast<u32x4*>(tiles.w + 4 * lane + (lane >> 1)), lane);
    });
}

}  // namespace
