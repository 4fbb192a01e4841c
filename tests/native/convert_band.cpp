// The gfx950 FP32 -> FP8 converts at and above the largest finite value, exhaustively.
//
// The kernels of the library convert without clamping first: the expanded value of a group's largest
// element is fmax * (1 + a few ulp)^k, which for every admissible k stays below the half-way point to
// the next (non-existent) value.  This program pins what the hardware does there, for every fp32 bit
// pattern from fmax up to past the half-way point, both signs:
//   E4M3 (OCP, max 448 = 1.110b * 2^8): up to and including the tie 464 the nearest-even result is
//         448 (code 0x7E); above it the code is 0x7F (NaN) -- E4M3 has no infinity (Sec. 3 of arxiv
//         2410.19313 names the format and its maximum).
//   E5M2 (OCP, max 57344 = 1.11b * 2^15): below the tie 61440 the result is 57344 (code 0x7B); the tie
//         itself rounds to the even neighbour 2^16, which the format does not have: non-finite
//         (0x7C infinity or a NaN code) from there on.
// Exit status 0 and a line "convert_band ok" when everything matches; otherwise the first mismatch.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#define CHECK(x)                                                                          \
  do {                                                                                    \
    hipError_t e_ = (x);                                                                  \
    if (e_ != hipSuccess) {                                                               \
      std::printf("%s failed: %s\n", #x, hipGetErrorString(e_));                          \
      return 2;                                                                           \
    }                                                                                     \
  } while (0)

__global__ void convert_range(uint32_t first_bits, uint32_t count, int e5m2, uint8_t* out) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const float x = __uint_as_float(first_bits + i);
  const uint32_t p = e5m2 ? __builtin_amdgcn_cvt_pk_bf8_f32(x, -x, 0u, false) : __builtin_amdgcn_cvt_pk_fp8_f32(x, -x, 0u, false);
  out[2 * i] = static_cast<uint8_t>(p & 0xffu);              // +x
  out[2 * i + 1] = static_cast<uint8_t>((p >> 8) & 0xffu);   // -x
}

static uint32_t bits_of(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  return u;
}

static int run(const char* name, int e5m2, float fmax, float tie, bool tie_stays, float end, uint8_t max_code) {
  const uint32_t first = bits_of(fmax), count = bits_of(end) - first + 1;
  uint8_t* d = nullptr;
  CHECK(hipMalloc(&d, 2ull * count));
  convert_range<<<(count + 255) / 256, 256>>>(first, count, e5m2, d);
  CHECK(hipGetLastError());
  std::vector<uint8_t> h(2ull * count);
  CHECK(hipMemcpy(h.data(), d, h.size(), hipMemcpyDeviceToHost));
  CHECK(hipFree(d));
  uint64_t finite = 0, other = 0;
  for (uint32_t i = 0; i < count; ++i) {
    uint32_t u = first + i;
    float x;
    std::memcpy(&x, &u, 4);
    const bool stays = x < tie || (x == tie && tie_stays);
    const uint8_t pos = h[2 * i], neg = h[2 * i + 1];
    bool ok;
    if (stays) {
      ok = pos == max_code && neg == (max_code | 0x80);
      ++finite;
    } else {
      ok = (pos & 0x7f) > max_code && (neg & 0x7f) > max_code && !(pos & 0x80) && (neg & 0x80);
      ++other;
    }
    if (!ok) {
      std::printf("%s: x = %.9g (bits %08x): codes %02x / %02x, expected %s\n", name, x, u, pos, neg,
                  stays ? "the largest finite code" : "a non-finite code");
      return 1;
    }
  }
  std::printf("%s: %llu patterns up to the tie give %02x, %llu above give a non-finite code (first: %02x)\n", name,
              (unsigned long long)finite, max_code, (unsigned long long)other, h[2 * finite]);
  return 0;
}

int main() {
  int rc = run("E4M3", 0, 448.0f, 464.0f, true, 480.0f, 0x7E);
  if (rc) return rc;
  rc = run("E5M2", 1, 57344.0f, 61440.0f, false, 65536.0f, 0x7B);
  if (rc) return rc;
  std::printf("convert_band ok\n");
  return 0;
}
