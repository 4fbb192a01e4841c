// Drives the HOST-ONLY entry points of the library (plan building, shard ranges, launch shapes,
// step constants, argument validation, error strings) from a program built, like the library it
// links, with -fsanitize=address,undefined on the host side.  Every buffer is a heap block of
// exactly the documented size, so an overrun in the host code is a failure.  Device pointers are
// made-up addresses: these entry points validate them and never dereference them.  No GPU is used.
// Prints "host_sanitize ok" and exits 0.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "coat.h"

#define REQUIRE(c) do { if (!(c)) { printf("check failed: %s at line %d\n", #c, __LINE__); return 1; } } while (0)

static coat_tensor_desc fake_tensor(uint64_t base, uint64_t n, bool with_copy) {
  coat_tensor_desc d;
  memset(&d, 0, sizeof d);
  d.w = reinterpret_cast<float*>(base);
  d.w_bf16 = with_copy ? reinterpret_cast<uint16_t*>(base + (1ull << 36)) : nullptr;
  d.grad_bf16 = reinterpret_cast<const uint16_t*>(base + (2ull << 36));
  d.m_q = reinterpret_cast<uint8_t*>(base + (3ull << 36));
  d.m_scale = reinterpret_cast<void*>(base + (4ull << 36));
  d.m_k = reinterpret_cast<float*>(base + (5ull << 36));
  d.v_q = reinterpret_cast<uint8_t*>(base + (6ull << 36));
  d.v_scale = reinterpret_cast<void*>(base + (7ull << 36));
  d.v_k = reinterpret_cast<float*>(base + (8ull << 36));
  d.n = n;
  d.weight_decay = 0.1f;
  return d;
}

int main() {
  REQUIRE(coat_version() > 0);
  for (int code = -40; code <= 2; ++code) {
    const char* s = coat_strerror(code);
    REQUIRE(s != nullptr && strlen(s) > 0);
  }

  // shard ranges: a partition of [0, n) into `world` contiguous pieces cut at multiples of 2 G
  const uint64_t sizes[] = {0, 1, 31, 32, 33, 1000, 4096, 70003, (1ull << 33) + 5, 1ull << 46};
  const int32_t groups[] = {32, 64, 128, 256, 512};
  const uint32_t worlds[] = {1, 2, 3, 8, 64, 1000};
  for (uint64_t n : sizes)
    for (int32_t G : groups)
      for (uint32_t world : worlds) {
        uint64_t covered = 0, lo_groups = ~0ull, hi_groups = 0;
        for (uint32_t r = 0; r < world; ++r) {
          uint64_t b = 1, e = 0;
          REQUIRE(coat_shard_range(n, G, r, world, &b, &e) == COAT_OK);
          REQUIRE(b == covered && e >= b && e <= n && (b % (2 * (uint64_t)G) == 0 || b == n) && (e % (2 * (uint64_t)G) == 0 || e == n));
          const uint64_t ng = (e - b + 2 * (uint64_t)G - 1) / (2 * (uint64_t)G);   // in pairs of groups
          lo_groups = ng < lo_groups ? ng : lo_groups;
          hi_groups = ng > hi_groups ? ng : hi_groups;
          covered = e;
        }
        REQUIRE(covered == n && hi_groups - lo_groups <= 1);
      }
  uint64_t b = 0, e = 0;
  REQUIRE(coat_shard_range(100, 128, 0, 0, &b, &e) != COAT_OK);
  REQUIRE(coat_shard_range(100, 128, 3, 3, &b, &e) != COAT_OK);
  REQUIRE(coat_shard_range(100, 0, 0, 1, &b, &e) == COAT_ERR_GROUP);
  REQUIRE(coat_shard_range(100, 128, 0, 1, nullptr, &e) == COAT_ERR_NULL);

  // launch shapes
  uint32_t blocks = 0, threads = 0;
  for (uint64_t n : sizes) {
    REQUIRE(coat_launch_shape(n, &blocks, &threads) == COAT_OK);
    REQUIRE(threads == 256 && (uint64_t)blocks * threads < (1ull << 32));
  }
  REQUIRE(coat_launch_shape((1ull << 46) + 1, &blocks, &threads) == COAT_ERR_SIZE);
  REQUIRE(coat_launch_shape(5, nullptr, &threads) == COAT_ERR_NULL);

  // plans: 0, 1 and many ragged tensors; the blob is exactly coat_multi_plan_bytes long
  for (uint32_t count : {0u, 1u, 7u, 300u}) {
    std::vector<coat_tensor_desc> descs;
    for (uint32_t t = 0; t < count; ++t)
      descs.push_back(fake_tensor(0x100000000ull + 0x1000000ull * t, t % 5 == 4 ? 0 : 1 + 40961ull * t, t % 3 == 0));
    const size_t need = coat_multi_plan_bytes(descs.data(), count);
    REQUIRE(need >= 128);
    unsigned char* blob = static_cast<unsigned char*>(malloc(need));
    REQUIRE(blob != nullptr);
    REQUIRE(coat_multi_plan_build(descs.data(), count, blob, need) == COAT_OK);
    REQUIRE(coat_multi_plan_build(descs.data(), count, blob, need - 1) == COAT_ERR_SIZE);
    REQUIRE(coat_multi_plan_build(descs.data(), count, nullptr, need) == COAT_ERR_NULL);
    if (count) {
      std::vector<coat_tensor_desc> bad = descs;
      bad[0].n = 77;
      bad[0].m_q = nullptr;
      REQUIRE(coat_multi_plan_build(bad.data(), count, blob, need) == COAT_ERR_NULL);
      bad = descs;
      bad[0].n = 77;
      bad[0].w = reinterpret_cast<float*>(0x100000004ull);
      REQUIRE(coat_multi_plan_build(bad.data(), count, blob, need) == COAT_ERR_ALIGN);
      bad = descs;
      bad[0].n = 77;
      bad[0].weight_decay = NAN;
      REQUIRE(coat_multi_plan_build(bad.data(), count, blob, need) == COAT_ERR_HPARAM);
      bad = descs;
      bad[0].n = (1ull << 46) + 1;
      REQUIRE(coat_multi_plan_bytes(bad.data(), count) == 0);
    }
    // a blob that is not a plan is refused before anything is launched
    memset(blob, 0, need);
    coat_adamw_hparams hp = {3e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 1, 128, COAT_FLAG_EXPAND, 0.0f, 0.0f};
    REQUIRE(coat_fp8_adamw_step_multi(blob, reinterpret_cast<void*>(0x200000000ull), &hp, nullptr) == COAT_ERR_PLAN);
    free(blob);
  }
  REQUIRE(coat_multi_plan_bytes(nullptr, 3) == 0);

  // step constants and hyper-parameter validation
  coat_step_consts* c = static_cast<coat_step_consts*>(malloc(sizeof(coat_step_consts)));
  REQUIRE(c != nullptr);
  coat_adamw_hparams hp = {3e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 1, 128, COAT_FLAG_EXPAND, 0.0f, 0.0f};
  for (int t : {1, 2, 10, 1000, 2000000000}) {
    hp.step = t;
    REQUIRE(coat_step_consts_compute(&hp, c) == COAT_OK);
    REQUIRE(isfinite(c->denom_mul) && isfinite(c->denom_add) && c->neg_lr < 0.0);
  }
  hp.lr = 0.0f;
  REQUIRE(coat_step_consts_compute(&hp, c) == COAT_OK && c->denom_mul == 0.0f && isinf(c->denom_add));
  hp.lr = 3e-4f;
  hp.step = 0;
  REQUIRE(coat_step_consts_compute(&hp, c) == COAT_ERR_STEP);
  hp.step = 1;
  hp.group_size = 100;
  REQUIRE(coat_step_consts_compute(&hp, c) == COAT_ERR_GROUP);
  hp.group_size = 128;
  hp.beta2 = 1.5f;
  REQUIRE(coat_step_consts_compute(&hp, c) == COAT_ERR_HPARAM);
  hp.beta2 = 0.95f;
  hp.flags = 1u << 30;
  REQUIRE(coat_step_consts_compute(&hp, c) == COAT_ERR_HPARAM);
  REQUIRE(coat_step_consts_compute(nullptr, c) != COAT_OK);
  REQUIRE(coat_step_consts_compute(&hp, nullptr) == COAT_ERR_NULL);
  free(c);

  // the compute entry points refuse bad arguments before they touch the device
  hp.flags = COAT_FLAG_EXPAND;
  float* fw = reinterpret_cast<float*>(0x100000000ull);
  uint16_t* fg = reinterpret_cast<uint16_t*>(0x200000000ull);
  uint8_t* fq = reinterpret_cast<uint8_t*>(0x300000000ull);
  REQUIRE(coat_fp8_adamw_step(nullptr, fg, fq, fw, fw, fq, fw, fw, 100, &hp, nullptr) == COAT_ERR_NULL);
  REQUIRE(coat_fp8_adamw_step(fw, fg, fq, fw, fw, fq, fw, fw, 100, nullptr, nullptr) == COAT_ERR_NULL);
  REQUIRE(coat_fp8_adamw_step(fw + 1, fg, fq, fw, fw, fq, fw, fw, 100, &hp, nullptr) == COAT_ERR_ALIGN);
  REQUIRE(coat_fp8_adamw_step(fw, fg, fq, fw, fw, fq, fw, fw, (1ull << 46) + 1, &hp, nullptr) == COAT_ERR_SIZE);
  REQUIRE(coat_quant_group(fw, 100, 100, COAT_FLAG_EXPAND, 0.0f, 0.0f, fq, fw, fw, nullptr) == COAT_ERR_GROUP);
  REQUIRE(coat_dequant_group(nullptr, fw, fw, 100, 128, 0, fw, nullptr) == COAT_ERR_NULL);
  printf("host_sanitize ok\n");
  return 0;
}
