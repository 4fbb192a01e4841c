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
// One translation unit: coat_device.hpp (storage modes, helpers, LDS staging, (de)quantizer
// arithmetic), coat_step.hpp (the fused step), coat_multi.hpp (the multi-tensor step),
// coat_quant.hpp (standalone quantizer / dequantizer), coat_act.hpp (activation quantizers),
// coat_copy.hpp (the copy control of the measurements), and below them the host side: validation,
// launches and the extern "C" entry points.
//
// Arithmetic (fp32 throughout; transcendentals are the hardware log2/exp2/rcp/sqrt), with fmax
// the largest finite value of the moment's FP8 format (448 for E4M3, 57344 for E5M2):
//   inverse expansion  |c/fmax|^(1/k) = exp2( log2|c/fmax| * (1/k) ), the logarithm from a table
//                      of the 127 code magnitudes; the one element per lane that decides a group's
//                      exponent is recomputed in fp64 (ExactChain);
//   expansion          fmax * (|x|/a)^k = exp2( k * log2(|x| * (1/a)) + log2 fmax ), the logarithm
//                      taken of the RATIO so that its magnitude stays below log2(range)/k;
//   conversion         native fp32 -> OCP FP8 pack instructions (round to nearest even).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "coat.h"

// Scratch of coat_act_quant_tensor_static: the partial maxima of Group Scaling's second stage in a
// device array of the library's own instead of a caller workspace.  Every GPU holds its own copy
// of the array at its own address (looked up once per device, below); the name itself is only a
// host-side handle and is never passed to a kernel.
static __device__ __align__(256) float g_act_scratch[COAT_ACT_WORKSPACE_FLOATS];

#include "coat_device.hpp"
#include "coat_step.hpp"
#include "coat_multi.hpp"
#include "coat_quant.hpp"
#include "coat_act.hpp"
#include "coat_copy.hpp"

namespace {

// ---------------------------------------------------------------------------------------
// host side: validation and launch
// ---------------------------------------------------------------------------------------

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
// per-group arrays (scale, k) are read and written one 32-bit word at a time
bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }
bool finite_f(float x) { return x == x && x - x == 0.0f; }
constexpr uint64_t kMaxElements = 1ull << 46;
bool group_ok(int32_t G) { return G == 32 || G == 64 || G == 128 || G == 256 || G == 512; }


// Blocks of the main launch.  One chunk per wavefront measured best (the hardware dispatcher then
// walks memory in address order and few bytes are in flight per CU).  A dispatch counts its
// work-items in 32 bits, so a grid holds fewer than 2^32 / 256 blocks; the kernels loop, which
// covers buffers with more chunks than that (above 6.8e10 elements).
constexpr uint64_t kMaxGridBlocks = (1ull << 32) / kBlock - 1;
unsigned grid_for(uint64_t n_full) {
  const uint64_t need = (n_full + kWavesPerBlock - 1) / kWavesPerBlock;
  return static_cast<unsigned>(need < kMaxGridBlocks ? need : kMaxGridBlocks);
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

// The step kernel asks for this much dynamic LDS on top of the 37 KiB it declares (tiles, tables,
// scratch), for no other purpose than to hold a CU to three resident blocks (12 wavefronts).  With
// fewer bytes in flight per CU the HBM controllers see longer same-page runs; three blocks rather
// than two cover the wait at the admission gate (measured on the 7B set: 2 blocks 16.4 ms,
// 3 blocks 14.9, 4 blocks 16.7).
constexpr size_t kStepLdsPad = 12 * 1024;
constexpr size_t kStepStaticLds = 37 * 1024;       // what the step kernel declares itself (tiles, tables, scratch)
constexpr size_t kMultiLdsPad = 12 * 1024;
constexpr size_t kQuantLdsPad = 12 * 1024;

template <int G, int KIND>
int launch_step(const StepArgs& a, hipStream_t s) {
  if (a.n_full) {
    const unsigned grid = grid_for(a.n_full);
    size_t lds = kStepLdsPad;
    if constexpr (KIND == kKindGeneric) hipLaunchKernelGGL((adamw_step_generic_kernel<G>), dim3(grid), dim3(kBlock), lds, s, a);
    else hipLaunchKernelGGL((adamw_step_kernel<G, KIND>), dim3(grid), dim3(kBlock), lds, s, a);
    if (int rc = launch_status()) return rc;
  }
  if (a.n > a.n_full * kChunk) {
    hipLaunchKernelGGL((adamw_step_tail_kernel<G, KIND>), dim3(1), dim3(kWave), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  return COAT_OK;
}

template <int G>
int launch_quant(const QuantArgs& a, hipStream_t s) {
  if (a.n_full) {
    // 12 KiB of dynamic LDS on top of the 18 KiB tile hold a CU to five resident blocks (6.7e9
    // elements: no request, 7 blocks, 5.68 ms; 6 KiB 5.59; 9 or 12 KiB 5.50; 16 KiB 5.54; 24 KiB 5.81)
    hipLaunchKernelGGL((quant_kernel<G>), dim3(grid_for(a.n_full)), dim3(kBlock), kQuantLdsPad, s, a);
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

int dispatch_step(const StepArgs& a, int32_t G, int kind, hipStream_t s) {
  if (kind == kKindDefault) { COAT_DISPATCH_G(G, (launch_step<kG, kKindDefault>(a, s))); }
  if (kind == kKindBf16Meta) { COAT_DISPATCH_G(G, (launch_step<kG, kKindBf16Meta>(a, s))); }
  if (kind == kKindPrecise) { COAT_DISPATCH_G(G, (launch_step<kG, kKindPrecise>(a, s))); }
  COAT_DISPATCH_G(G, (launch_step<kG, kKindGeneric>(a, s)));
}

template <int G>
int launch_copy_control(const StepArgs& a, hipStream_t s) {
  if (a.n_full) {
    hipLaunchKernelGGL((copy_control_kernel<G>), dim3(grid_for(a.n_full)), dim3(kBlock), kStepLdsPad + kStepStaticLds, s, a);
    if (int rc = launch_status()) return rc;
  }
  return COAT_OK;
}
int dispatch_copy_control(const StepArgs& a, int32_t G, hipStream_t s) { COAT_DISPATCH_G(G, (launch_copy_control<kG>(a, s))); }

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

constexpr unsigned kActTensorMaxGrid = 1024;
template <int G, bool PER_TENSOR>
int launch_act_quant(const ActArgs& a, hipStream_t s) {
  if (a.n_full) {
    // with one scale per tensor every workgroup first folds the workspace slots: few, looping
    // workgroups pay that once each (8192 x 4096 elements, whole call: uncapped 35.5 us, at most
    // 4096 / 2048 / 1024 / 768 / 512 workgroups 34.9 / 33.7 / 33.1 / 32.9 / 35.1 us)
    unsigned grid = grid_for(a.n_full);
    if (PER_TENSOR && grid > kActTensorMaxGrid) grid = kActTensorMaxGrid;
    hipLaunchKernelGGL((act_quant_kernel<G, PER_TENSOR>), dim3(grid), dim3(kBlock), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  if (a.n > a.n_full * kChunk) {
    hipLaunchKernelGGL((act_quant_tail_kernel<G, PER_TENSOR>), dim3(1), dim3(kWave), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  return COAT_OK;
}

// Stage 1 of Group Scaling; also fills the workspace slots (one per workgroup, one more for the
// ragged last chunk) and says how many in a.n_partial.
constexpr unsigned kStage1MaxGrid = COAT_ACT_WORKSPACE_FLOATS - 1;
template <int G>
int launch_act_group_amax(ActArgs& a, hipStream_t s) {
  unsigned grid = 0;
  if (a.n_full) {
    const uint64_t need = (a.n_full + kWavesPerBlock - 1) / kWavesPerBlock;
    grid = static_cast<unsigned>(need < kStage1MaxGrid ? need : kStage1MaxGrid);
    hipLaunchKernelGGL((act_group_amax_kernel<G>), dim3(grid), dim3(kBlock), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  a.n_partial = static_cast<int>(grid);
  if (a.n > a.n_full * kChunk) {
    a.tail_slot = static_cast<int>(grid);
    a.n_partial = static_cast<int>(grid) + 1;
    hipLaunchKernelGGL((act_group_amax_tail_kernel<G>), dim3(1), dim3(kWave), 0, s, a);
    if (int rc = launch_status()) return rc;
  }
  return COAT_OK;
}

int dispatch_act_quant_group(const ActArgs& a, int32_t G, hipStream_t s) {
  COAT_DISPATCH_ACT_G(G, (launch_act_quant<kG, false>(a, s)));
}
int dispatch_act_group_amax(ActArgs& a, int32_t G, hipStream_t s) {
  COAT_DISPATCH_ACT_G(G, (launch_act_group_amax<kG>(a, s)));
}

// Group Scaling for a caller who brings the group maxima: reduce them (stage 2), then quantize
constexpr int kStage2Block = 1024, kStage2Unroll = 4, kStage2MaxGrid = 64;
static_assert(kStage2MaxGrid <= COAT_ACT_WORKSPACE_FLOATS, "one workspace slot per workgroup");
int launch_act_tensor_amax(ActArgs& a, hipStream_t s) {
  const uint64_t need = (a.n_groups / 4 + kStage2Block * kStage2Unroll - 1) / (kStage2Block * kStage2Unroll);
  const unsigned grid = static_cast<unsigned>(need < 1 ? 1 : (need > kStage2MaxGrid ? kStage2MaxGrid : need));
  a.n_partial = static_cast<int>(grid);
  hipLaunchKernelGGL((act_tensor_amax_kernel<kStage2Block, kStage2Unroll>), dim3(grid), dim3(kStage2Block), 0, s, a);
  return launch_status();
}

constexpr int kMaxDevices = 64;
std::atomic<float*> g_act_scratch_ptr[kMaxDevices];

// The device address of g_act_scratch on the current device (nullptr on failure).  The first call
// on a device asks the runtime for it; later calls read the cached pointer.  Nothing is allocated.
float* act_scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  float* p = g_act_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  void* sym = nullptr;
  if (hipGetSymbolAddress(&sym, HIP_SYMBOL(g_act_scratch)) != hipSuccess || !sym) return nullptr;
  g_act_scratch_ptr[dev].store(static_cast<float*>(sym), std::memory_order_release);   // same value from any thread
  return static_cast<float*>(sym);
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
  a.partial = workspace; a.n_partial = 0; a.tail_slot = 0; a.tensor_amax = tensor_amax; a.tensor_scale = tensor_scale;
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(G) - 1) / static_cast<uint64_t>(G);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  // the reduction to one maximum: from the caller's group maxima in a launch of its own, otherwise
  // as a by-product of stage 1; either way the quantizing launch folds the workspace slots
  if (int rc = have_group_amax ? launch_act_tensor_amax(a, s) : dispatch_act_group_amax(a, G, s)) return rc;
  return launch_act_quant<16, true>(a, s);   // the group size plays no part once the scale is per tensor
}

template <int G, int KIND>
int launch_step_multi(const MultiArgs& ma, uint64_t total_records, hipStream_t s) {
  const uint64_t blocks = total_records * (kPlanSpan / kWavesPerBlock);
  size_t lds = kMultiLdsPad;
  hipLaunchKernelGGL((adamw_step_multi_kernel<G, KIND>), dim3(static_cast<unsigned>(blocks)), dim3(kBlock), lds, s, ma);
  return launch_status();
}

int dispatch_step_multi(const MultiArgs& ma, uint64_t total_records, int32_t G, int kind, hipStream_t s) {
  if (kind == kKindDefault) { COAT_DISPATCH_G(G, (launch_step_multi<kG, kKindDefault>(ma, total_records, s))); }
  if (kind == kKindBf16Meta) { COAT_DISPATCH_G(G, (launch_step_multi<kG, kKindBf16Meta>(ma, total_records, s))); }
  if (kind == kKindPrecise) { COAT_DISPATCH_G(G, (launch_step_multi<kG, kKindPrecise>(ma, total_records, s))); }
  COAT_DISPATCH_G(G, (launch_step_multi<kG, kKindGeneric>(ma, total_records, s)));
}

constexpr uint32_t kStepFlags = COAT_FLAG_EXPAND | COAT_FLAG_M_E5M2 | COAT_FLAG_V_E5M2 | COAT_FLAG_M_PLAIN |
                                COAT_FLAG_V_PLAIN | COAT_FLAG_BF16_SCALE | COAT_FLAG_BF16_K | COAT_FLAG_PRECISE_DQ;

constexpr uint64_t kPlanRecordOffset = 128;          // records start one cache line into the blob
// one launch covers all records with kPlanSpan / kWavesPerBlock = 8 workgroups each, and a grid holds
// fewer than 2^24 workgroups
constexpr uint64_t kMaxPlanRecords = kMaxGridBlocks / (kPlanSpan / kWavesPerBlock);

uint64_t plan_records_of(uint64_t n) {               // spans of 32 chunks a tensor of n elements occupies
  const uint64_t chunks = (n + kChunk - 1) / kChunk;
  return (chunks + kPlanSpan - 1) / kPlanSpan;
}

// Validates the hyper-parameters and fills every field of StepArgs that does not depend on the
// tensor (the pointers, sizes and the decay factor are set by the caller).
int step_constants(const coat_adamw_hparams* hp, StepArgs& a, int& kind) {
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
  a.m_ratio64 = b1 / omb1;
  a.g_coef64 = (1.0 - b1) / omb1;
  a.beta2_ratio = static_cast<float>(b2 / omb2);
  const double c = -static_cast<double>(hp->lr) * omb1 / bc1;      // m' / D times this is the update
  if (c != 0.0) {
    a.denom_mul = static_cast<float>(__builtin_sqrt(omb2 / bc2) / c);
    a.denom_add = static_cast<float>(static_cast<double>(hp->eps) / c);
  } else {                                                          // lr == 0: 1 / (0 * sqrt(v') + inf) = 0
    a.denom_mul = 0.0f;
    a.denom_add = __builtin_huge_valf();
  }
  a.k_min = k_min; a.k_max = k_max;
  const bool expand = (hp->flags & COAT_FLAG_EXPAND) != 0;
  a.mode_m.e5 = (hp->flags & COAT_FLAG_M_E5M2) != 0;
  a.mode_v.e5 = (hp->flags & COAT_FLAG_V_E5M2) != 0;
  a.mode_m.ex = expand && !(hp->flags & COAT_FLAG_M_PLAIN);
  a.mode_v.ex = expand && !(hp->flags & COAT_FLAG_V_PLAIN);
  a.mode_m.s16 = a.mode_v.s16 = (hp->flags & COAT_FLAG_BF16_SCALE) != 0;
  a.mode_m.kh = a.mode_v.kh = (hp->flags & COAT_FLAG_BF16_K) != 0;
  const bool default_cell = !a.mode_m.e5 && !a.mode_v.e5 && a.mode_m.ex && a.mode_v.ex;
  // The more accurate inverse expansion: on request, and by itself where the step can be large against
  // the weight.  |m_hat| / sqrt(v_hat) is at most (1 - beta1) / sqrt(1 - beta2), so the update is at
  // most lr times that; its relative error without the correction (2e-6) stays below 1e-6 of a
  // weight of a few 1e-2 while that bound is below 2e-4 (lr = 3e-4 with beta = 0.9 / 0.95: 1.3e-4;
  // PyTorch's defaults lr = 1e-3, beta = 0.9 / 0.999: 3.2e-3).
  const bool large_steps = static_cast<double>(hp->lr) * omb1 >= 2e-4 * __builtin_sqrt(omb2);
  const bool precise = (hp->flags & COAT_FLAG_PRECISE_DQ) != 0 || large_steps;
  const bool bf16_meta = a.mode_m.s16 || a.mode_m.kh;
  // (the generic kernel always takes the more accurate inverse expansion, so it also serves the
  // request for it in combination with bf16 metadata)
  kind = (!default_cell || (precise && bf16_meta)) ? kKindGeneric : bf16_meta ? kKindBf16Meta : precise ? kKindPrecise : kKindDefault;
  return COAT_OK;
}


int step_multi_impl(const void* plan_host, const void* plan_device, const coat_adamw_hparams* hp,
                    const coat_step_consts* consts_device, bool want_consts, void* hip_stream) {
  MultiArgs ma;
  int kind = kKindDefault;
  if (int rc = step_constants(hp, ma.base, kind)) return rc;
  if (!plan_host) return COAT_ERR_NULL;
  PlanHeader h;
  __builtin_memcpy(&h, plan_host, sizeof h);
  if (h.magic != kPlanMagic || h.version != 2 || h.record_offset != kPlanRecordOffset ||
      h.total_records > kMaxPlanRecords || h.bytes != kPlanRecordOffset + h.total_records * sizeof(PlanRecord))
    return COAT_ERR_PLAN;
  if (want_consts && !consts_device) return COAT_ERR_NULL;
  if (want_consts && !aligned16(consts_device)) return COAT_ERR_ALIGN;
  if (h.total_records == 0) return COAT_OK;
  if (!plan_device) return COAT_ERR_NULL;
  if (!aligned16(plan_device)) return COAT_ERR_ALIGN;
  const unsigned char* dev = static_cast<const unsigned char*>(plan_device);
  ma.base.w = nullptr; ma.base.wb = nullptr; ma.base.g = nullptr; ma.base.mq = nullptr; ma.base.ms = nullptr;
  ma.base.mk = nullptr; ma.base.vq = nullptr; ma.base.vs = nullptr; ma.base.vk = nullptr;
  ma.base.n = 0; ma.base.n_full = 0; ma.base.n_groups = 0; ma.base.w_keep = 1.0f;
  ma.records = reinterpret_cast<const PlanRecord*>(dev + h.record_offset);
  ma.neg_lr = -static_cast<double>(hp->lr);
  ma.consts = reinterpret_cast<const StepConsts*>(consts_device);
  return dispatch_step_multi(ma, h.total_records, hp->group_size, kind, static_cast<hipStream_t>(hip_stream));
}

}  // namespace

extern "C" {

int coat_fp8_adamw_step(float* w, const uint16_t* grad_bf16, uint8_t* m_q, void* m_scale, void* m_k,
                        uint8_t* v_q, void* v_scale, void* v_k, uint64_t n,
                        const coat_adamw_hparams* hp, void* hip_stream) {
  return coat_fp8_adamw_step_bf16w(w, nullptr, grad_bf16, m_q, m_scale, m_k, v_q, v_scale, v_k, n, hp, hip_stream);
}

int coat_fp8_adamw_step_bf16w(float* w, uint16_t* w_bf16, const uint16_t* grad_bf16, uint8_t* m_q,
                              void* m_scale, void* m_k, uint8_t* v_q, void* v_scale, void* v_k,
                              uint64_t n, const coat_adamw_hparams* hp, void* hip_stream) {
  StepArgs a;
  int kind = kKindDefault;
  if (int rc = step_constants(hp, a, kind)) return rc;
  if (n == 0) return COAT_OK;
  if (!w || !grad_bf16 || !m_q || !m_scale || !m_k || !v_q || !v_scale || !v_k) return COAT_ERR_NULL;
  if (!aligned16(w) || !aligned16(grad_bf16) || !aligned16(m_q) || !aligned16(v_q) ||
      !aligned4(m_scale) || !aligned4(m_k) || !aligned4(v_scale) || !aligned4(v_k) || !aligned16(w_bf16))
    return COAT_ERR_ALIGN;
  if (n > kMaxElements) return COAT_ERR_SIZE;
  a.w = w; a.wb = w_bf16; a.g = grad_bf16; a.mq = m_q; a.ms = static_cast<float*>(m_scale); a.mk = static_cast<float*>(m_k); a.vq = v_q; a.vs = static_cast<float*>(v_scale); a.vk = static_cast<float*>(v_k);
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(hp->group_size) - 1) / static_cast<uint64_t>(hp->group_size);
  a.w_keep = static_cast<float>(1.0 - static_cast<double>(hp->lr) * static_cast<double>(hp->weight_decay));
  return dispatch_step(a, hp->group_size, kind, static_cast<hipStream_t>(hip_stream));
}

size_t coat_multi_plan_bytes(const coat_tensor_desc* descs, uint32_t count) {
  if (count && !descs) return 0;
  uint64_t records = 0;
  for (uint32_t t = 0; t < count; ++t) {
    if (descs[t].n > kMaxElements) return 0;
    records += plan_records_of(descs[t].n);
  }
  if (records > kMaxPlanRecords) return 0;
  return kPlanRecordOffset + static_cast<size_t>(records) * sizeof(PlanRecord);
}

int coat_multi_plan_build(const coat_tensor_desc* descs, uint32_t count, void* plan_host, size_t plan_bytes) {
  if (!plan_host || (count && !descs)) return COAT_ERR_NULL;
  const size_t need = coat_multi_plan_bytes(descs, count);
  if (need == 0 || plan_bytes < need) return COAT_ERR_SIZE;
  for (uint32_t t = 0; t < count; ++t) {
    const coat_tensor_desc& d = descs[t];
    if (d.n == 0) continue;
    if (!d.w || !d.grad_bf16 || !d.m_q || !d.m_scale || !d.m_k || !d.v_q || !d.v_scale || !d.v_k) return COAT_ERR_NULL;
    if (!aligned16(d.w) || !aligned16(d.grad_bf16) || !aligned16(d.m_q) || !aligned16(d.v_q) || !aligned4(d.m_scale) ||
        !aligned4(d.m_k) || !aligned4(d.v_scale) || !aligned4(d.v_k) || !aligned16(d.w_bf16))
      return COAT_ERR_ALIGN;
    if (!finite_f(d.weight_decay)) return COAT_ERR_HPARAM;
  }
  unsigned char* blob = static_cast<unsigned char*>(plan_host);
  PlanHeader h = {};
  h.magic = kPlanMagic; h.version = 2; h.count = count;
  h.record_offset = kPlanRecordOffset; h.bytes = need;
  uint64_t rec = 0;
  for (uint32_t t = 0; t < count; ++t) {
    const coat_tensor_desc& d = descs[t];
    const uint64_t spans = plan_records_of(d.n);
    for (uint64_t i = 0; i < spans; ++i, ++rec) {
      PlanRecord o = {};
      o.w = d.w; o.wb = d.w_bf16; o.g = d.grad_bf16; o.mq = d.m_q; o.ms = static_cast<float*>(d.m_scale); o.mk = static_cast<float*>(d.m_k);
      o.vq = d.v_q; o.vs = static_cast<float*>(d.v_scale); o.vk = static_cast<float*>(d.v_k); o.n = d.n;
      o.chunk_base = i * kPlanSpan; o.weight_decay = d.weight_decay; o.tensor = t;
      __builtin_memcpy(blob + h.record_offset + rec * sizeof(PlanRecord), &o, sizeof o);
    }
  }
  h.total_records = rec;
  __builtin_memcpy(blob, &h, sizeof h);
  return COAT_OK;
}

int coat_step_consts_compute(const coat_adamw_hparams* hp, coat_step_consts* out) {
  if (!out) return COAT_ERR_NULL;
  StepArgs a;
  int kind = kKindDefault;
  if (int rc = step_constants(hp, a, kind)) return rc;
  coat_step_consts c = {};
  c.denom_mul = a.denom_mul;
  c.denom_add = a.denom_add;
  c.neg_lr = -static_cast<double>(hp->lr);
  *out = c;
  return COAT_OK;
}

int coat_fp8_adamw_step_multi(const void* plan_host, const void* plan_device, const coat_adamw_hparams* hp,
                              void* hip_stream) {
  return step_multi_impl(plan_host, plan_device, hp, nullptr, false, hip_stream);
}

int coat_fp8_adamw_step_multi_consts(const void* plan_host, const void* plan_device, const coat_adamw_hparams* hp,
                                     const coat_step_consts* consts_device, void* hip_stream) {
  return step_multi_impl(plan_host, plan_device, hp, consts_device, true, hip_stream);
}

int coat_launch_shape(uint64_t n, uint32_t* blocks, uint32_t* threads_per_block) {
  if (!blocks || !threads_per_block) return COAT_ERR_NULL;
  if (n > kMaxElements) return COAT_ERR_SIZE;
  *blocks = grid_for(n / kChunk);
  *threads_per_block = kBlock;
  return COAT_OK;
}

int coat_shard_range(uint64_t n, int32_t G, uint32_t rank, uint32_t world, uint64_t* begin, uint64_t* end) {
  if (!begin || !end) return COAT_ERR_NULL;
  if (G < 1) return COAT_ERR_GROUP;
  if (world == 0 || rank >= world) return COAT_ERR_HPARAM;
  // cuts fall on PAIRS of groups: with scales stored as bf16 a shard's scale array then still starts
  // on a 32-bit word, which is how the kernels read it
  const uint64_t g = 2 * static_cast<uint64_t>(G);
  const uint64_t groups = n / g + (n % g != 0);
  const uint64_t base = groups / world, extra = groups % world;           // the first `extra` ranks own one more pair
  const uint64_t g0 = rank * base + (rank < extra ? rank : extra);
  const uint64_t g1 = g0 + base + (rank < extra ? 1 : 0);
  *begin = g0 * g < n ? g0 * g : n;
  *end = g1 * g < n ? g1 * g : n;
  return COAT_OK;
}

int coat_bench_copy_control(float* w, const uint16_t* grad_bf16, uint8_t* m_q, float* m_scale, float* m_k,
                            uint8_t* v_q, float* v_scale, float* v_k, uint64_t n, int32_t G, void* hip_stream) {
  if (!group_ok(G)) return COAT_ERR_GROUP;
  if (n == 0) return COAT_OK;
  if (!w || !grad_bf16 || !m_q || !m_scale || !m_k || !v_q || !v_scale || !v_k) return COAT_ERR_NULL;
  if (!aligned16(w) || !aligned16(grad_bf16) || !aligned16(m_q) || !aligned16(v_q) || !aligned4(m_scale) ||
      !aligned4(m_k) || !aligned4(v_scale) || !aligned4(v_k))
    return COAT_ERR_ALIGN;
  if (n > kMaxElements || n % kChunk != 0) return COAT_ERR_SIZE;
  StepArgs a = {};
  a.w = w; a.g = grad_bf16; a.mq = m_q; a.ms = m_scale; a.mk = m_k; a.vq = v_q; a.vs = v_scale; a.vk = v_k;
  a.n = n; a.n_full = n / kChunk; a.n_groups = n / static_cast<uint64_t>(G);
  return dispatch_copy_control(a, G, static_cast<hipStream_t>(hip_stream));
}

int coat_quant_group(const float* x, uint64_t n, int32_t G, uint32_t flags, float k_min, float k_max,
                     uint8_t* q, void* scale, void* k, void* hip_stream) {
  if (!group_ok(G)) return COAT_ERR_GROUP;
  if (flags & ~(COAT_FLAG_EXPAND | COAT_FLAG_E5M2 | COAT_FLAG_BF16_SCALE | COAT_FLAG_BF16_K)) return COAT_ERR_HPARAM;
  if (!resolve_k_bounds(k_min, k_max)) return COAT_ERR_HPARAM;
  if (n == 0) return COAT_OK;
  if (!x || !q || !scale || !k) return COAT_ERR_NULL;
  if (!aligned16(x) || !aligned16(q) || !aligned4(scale) || !aligned4(k)) return COAT_ERR_ALIGN;
  if (n > kMaxElements) return COAT_ERR_SIZE;
  QuantArgs a;
  a.x = x; a.q = q; a.scale = static_cast<float*>(scale); a.k = static_cast<float*>(k);
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(G) - 1) / static_cast<uint64_t>(G);
  a.k_min = k_min; a.k_max = k_max;
  a.mode.ex = (flags & COAT_FLAG_EXPAND) != 0;
  a.mode.e5 = (flags & COAT_FLAG_E5M2) != 0;
  a.mode.s16 = (flags & COAT_FLAG_BF16_SCALE) != 0;
  a.mode.kh = (flags & COAT_FLAG_BF16_K) != 0;
  return dispatch_quant(a, G, static_cast<hipStream_t>(hip_stream));
}

int coat_dequant_group(const uint8_t* q, const void* scale, const void* k, uint64_t n, int32_t G,
                       uint32_t flags, float* x, void* hip_stream) {
  if (!group_ok(G)) return COAT_ERR_GROUP;
  if (flags & ~(COAT_FLAG_EXPAND | COAT_FLAG_E5M2 | COAT_FLAG_BF16_SCALE | COAT_FLAG_BF16_K)) return COAT_ERR_HPARAM;
  if (n == 0) return COAT_OK;
  if (!x || !q || !scale || !k) return COAT_ERR_NULL;
  if (!aligned16(x) || !aligned16(q) || !aligned4(scale) || !aligned4(k)) return COAT_ERR_ALIGN;
  if (n > kMaxElements) return COAT_ERR_SIZE;
  DequantArgs a;
  a.q = q; a.scale = static_cast<const float*>(scale); a.k = static_cast<const float*>(k); a.x = x;
  a.n = n; a.n_full = n / kChunk;
  a.n_groups = (n + static_cast<uint64_t>(G) - 1) / static_cast<uint64_t>(G);
  a.mode.ex = true;
  a.mode.e5 = (flags & COAT_FLAG_E5M2) != 0;
  a.mode.s16 = (flags & COAT_FLAG_BF16_SCALE) != 0;
  a.mode.kh = (flags & COAT_FLAG_BF16_K) != 0;
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

int coat_act_quant_tensor_static(const uint16_t* x_bf16, uint64_t n, int32_t G, float* group_amax,
                                 float* tensor_amax, float* tensor_scale, uint8_t* q, void* hip_stream) {
  if (n > kMaxElements) return COAT_ERR_SIZE;       // before anything else: this variant's size limit
  float* scratch = act_scratch_on_current_device();
  if (!scratch) return COAT_ERR_LAUNCH;
  return act_quant_tensor_impl(x_bf16, n, G, group_amax, false, scratch, tensor_amax, tensor_scale, q, hip_stream);
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
    case COAT_ERR_ALIGN: return "a base pointer is not aligned as required (16 bytes; 4 for per-group scale and k arrays)";
    case COAT_ERR_GROUP: return "group size must be one of 32, 64, 128, 256, 512 (activation quantizers: also 16)";
    case COAT_ERR_STEP: return "step must be >= 1";
    case COAT_ERR_HPARAM: return "hyper-parameter or flag is non-finite, unsupported or out of its domain";
    case COAT_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    case COAT_ERR_SIZE: return "n is too large (above 2^46 elements), or the plan buffer is too small";
    case COAT_ERR_PLAN: return "the plan blob is not one that coat_multi_plan_build wrote";
  }
  return "unknown error code";
}

int coat_version(void) { return 240; }


}  // extern "C"
