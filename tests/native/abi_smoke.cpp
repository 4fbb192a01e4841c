// abi_smoke.cpp -- the C ABI used from a plain HIP host program: no Python, no PyTorch.
// Allocates with hipMalloc, runs two optimizer steps twice from the same start (the results must be
// bit-identical: the kernels are deterministic), a quantize -> dequantize round trip, and the
// activation quantizers; checks invariants that need no oracle.  Prints "abi_smoke ok" and exits 0.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "coat.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); return 1; } } while (0)
#define CHECK_COAT(x) do { int r_ = (x); if (r_ != COAT_OK) { printf("coat error %d (%s) at %s:%d\n", r_, coat_strerror(r_), __FILE__, __LINE__); return 1; } } while (0)
#define REQUIRE(c) do { if (!(c)) { printf("check failed: %s at %s:%d\n", #c, __FILE__, __LINE__); return 1; } } while (0)

static uint32_t lcg(uint32_t& s) { s = s * 1664525u + 1013904223u; return s; }
static float unit(uint32_t& s) { return (float)(lcg(s) >> 8) * (1.0f / 16777216.0f) - 0.5f; }
static uint16_t to_bf16(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16); }

template <typename T> struct DevBuf {
  T* p = nullptr; size_t n = 0;
  hipError_t alloc(size_t count) { n = count; return hipMalloc((void**)&p, count * sizeof(T) + 16); }
  hipError_t up(const std::vector<T>& h) { return hipMemcpy(p, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice); }
  hipError_t down(std::vector<T>& h) const { h.resize(n); return hipMemcpy(h.data(), p, n * sizeof(T), hipMemcpyDeviceToHost); }
  ~DevBuf() { if (p) (void)hipFree(p); }
};

int main() {
  const uint64_t n = 5 * 1024 + 333;
  const int G = 128;
  const uint64_t ng = (n + G - 1) / G;
  uint32_t seed = 12345u;
  std::vector<float> w0(n), x(n);
  std::vector<uint16_t> g1(n), g2(n);
  for (uint64_t i = 0; i < n; ++i) {
    w0[i] = 0.04f * unit(seed); g1[i] = to_bf16(2e-3f * unit(seed)); g2[i] = to_bf16(2e-3f * unit(seed));
    x[i] = 1e-3f * unit(seed) * (1.0f + (float)(i % 7));
  }
  printf("coat_version %d\n", coat_version());

  std::vector<float> w_run[2];
  std::vector<uint8_t> mq_run[2], vq_run[2];
  std::vector<float> ms_run[2], vk_run[2];
  for (int run = 0; run < 2; ++run) {
    DevBuf<float> w, ms, mk, vs, vk; DevBuf<uint16_t> g; DevBuf<uint8_t> mq, vq;
    CHECK_HIP(w.alloc(n)); CHECK_HIP(g.alloc(n)); CHECK_HIP(mq.alloc(n)); CHECK_HIP(vq.alloc(n));
    CHECK_HIP(ms.alloc(ng)); CHECK_HIP(mk.alloc(ng)); CHECK_HIP(vs.alloc(ng)); CHECK_HIP(vk.alloc(ng));
    CHECK_HIP(w.up(w0));
    CHECK_HIP(hipMemset(mq.p, 0, n)); CHECK_HIP(hipMemset(vq.p, 0, n));
    CHECK_HIP(ms.up(std::vector<float>(ng, 0.0f))); CHECK_HIP(vs.up(std::vector<float>(ng, 0.0f)));
    CHECK_HIP(mk.up(std::vector<float>(ng, 1.0f))); CHECK_HIP(vk.up(std::vector<float>(ng, 1.0f)));
    for (int t = 1; t <= 2; ++t) {
      CHECK_HIP(g.up(t == 1 ? g1 : g2));
      coat_adamw_hparams hp = {3e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, t, G, COAT_FLAG_EXPAND, 0.0f, 0.0f};
      CHECK_COAT(coat_fp8_adamw_step(w.p, g.p, mq.p, ms.p, mk.p, vq.p, vs.p, vk.p, n, &hp, nullptr));
    }
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(w.down(w_run[run])); CHECK_HIP(mq.down(mq_run[run])); CHECK_HIP(vq.down(vq_run[run]));
    CHECK_HIP(ms.down(ms_run[run])); CHECK_HIP(vk.down(vk_run[run]));
  }
  REQUIRE(memcmp(w_run[0].data(), w_run[1].data(), n * 4) == 0);
  REQUIRE(mq_run[0] == mq_run[1] && vq_run[0] == vq_run[1]);
  REQUIRE(memcmp(ms_run[0].data(), ms_run[1].data(), ng * 4) == 0);
  uint64_t moved = 0, signed_v = 0, nonzero_m = 0;
  for (uint64_t i = 0; i < n; ++i) {
    REQUIRE(isfinite(w_run[0][i]));
    moved += w_run[0][i] != w0[i]; signed_v += vq_run[0][i] >= 0x80; nonzero_m += (mq_run[0][i] & 0x7F) != 0;
  }
  REQUIRE(moved > n * 9 / 10 && signed_v == 0 && nonzero_m > n * 9 / 10);
  for (uint64_t gI = 0; gI < ng; ++gI) REQUIRE(ms_run[0][gI] > 0.0f && vk_run[0][gI] >= 0.0625f && vk_run[0][gI] <= 1024.0f);

  {   // quantize -> dequantize: signs kept, nothing above the largest input, all but a few elements within 7 %
    DevBuf<float> dx, dy, sc, kk; DevBuf<uint8_t> q;
    CHECK_HIP(dx.alloc(n)); CHECK_HIP(dy.alloc(n)); CHECK_HIP(sc.alloc(ng)); CHECK_HIP(kk.alloc(ng)); CHECK_HIP(q.alloc(n));
    CHECK_HIP(dx.up(x));
    CHECK_COAT(coat_quant_group(dx.p, n, G, COAT_FLAG_EXPAND, 0.0f, 0.0f, q.p, sc.p, kk.p, nullptr));
    CHECK_COAT(coat_dequant_group(q.p, sc.p, kk.p, n, G, 0, dy.p, nullptr));
    CHECK_HIP(hipDeviceSynchronize());
    std::vector<float> y; CHECK_HIP(dy.down(y));
    uint64_t coarse = 0;                       // elements that landed on subnormal codes are coarser than 7 %
    for (uint64_t i = 0; i < n; ++i) {
      REQUIRE((y[i] < 0) == (x[i] < 0) || y[i] == 0.0f);
      REQUIRE(fabsf(y[i]) <= 1.001f * 3.5e-3f);
      coarse += fabsf(y[i] - x[i]) > 0.07f * fabsf(x[i]);
    }
    REQUIRE(coarse < n / 20);
  }
  {   // activation quantizers: per group and per tensor (Group Scaling); the largest element of a group encodes to +-448
    std::vector<uint16_t> xb(n);
    for (uint64_t i = 0; i < n; ++i) xb[i] = to_bf16(x[i] * 1000.0f);
    const uint64_t ng16 = (n + 15) / 16;
    DevBuf<uint16_t> dx; DevBuf<uint8_t> q, qt; DevBuf<float> sc, gmax, ws, stats;
    CHECK_HIP(dx.alloc(n)); CHECK_HIP(q.alloc(n)); CHECK_HIP(qt.alloc(n)); CHECK_HIP(sc.alloc(ng16)); CHECK_HIP(gmax.alloc(ng16));
    CHECK_HIP(ws.alloc(COAT_ACT_WORKSPACE_FLOATS)); CHECK_HIP(stats.alloc(2));
    CHECK_HIP(dx.up(xb));
    CHECK_COAT(coat_act_quant_group(dx.p, n, 16, q.p, sc.p, nullptr));
    CHECK_COAT(coat_act_quant_tensor(dx.p, n, 16, gmax.p, ws.p, stats.p, stats.p + 1, qt.p, nullptr));
    CHECK_HIP(hipDeviceSynchronize());
    std::vector<uint8_t> hq, hqt; std::vector<float> hs, hg, hstats;
    CHECK_HIP(q.down(hq)); CHECK_HIP(qt.down(hqt)); CHECK_HIP(sc.down(hs)); CHECK_HIP(gmax.down(hg)); CHECK_HIP(stats.down(hstats));
    float tmax = 0.0f; uint64_t tops = 0;
    for (uint64_t gI = 0; gI < ng16; ++gI) {
      REQUIRE(hs[gI] == hg[gI] / 448.0f);
      tmax = fmaxf(tmax, hg[gI]);
      bool top = false;
      for (uint64_t i = gI * 16; i < n && i < gI * 16 + 16; ++i) top |= (hq[i] & 0x7F) == 0x7E;
      REQUIRE(top || hg[gI] == 0.0f);
    }
    REQUIRE(hstats[0] == tmax && hstats[1] == tmax / 448.0f);
    for (uint64_t i = 0; i < n; ++i) tops += (hqt[i] & 0x7F) == 0x7E;
    REQUIRE(tops >= 1);
  }
  // error paths answer before anything is launched
  coat_adamw_hparams bad = {3e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 0, G, COAT_FLAG_EXPAND, 0.0f, 0.0f};
  REQUIRE(coat_fp8_adamw_step(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 10, &bad, nullptr) == COAT_ERR_STEP);
  printf("abi_smoke ok\n");
  return 0;
}
