// Host-side check of the device index logic in common.hpp (no GPU needed): the 32-bucket scheme and the
// 4-level search must both equal the plain count of thresholds below x, for every float near a threshold
// or a bucket edge and for a dense sweep of [-1.25, 1.25].  Prints "OK <count>" or the first mismatch.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "common.hpp"

using namespace qlora;

static uint32_t plain_count(float x) {
  uint32_t n = 0;
  for (int j = 0; j < 15; ++j) n += x > nf4_threshold(j) ? 1u : 0u;
  return n;
}
static float from_bits(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }
static uint32_t to_bits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }

static long long checked = 0;
static bool check(float x) {
  ++checked;
  const uint32_t want = plain_count(x), a = nf4_index_bucket_ref(x), b = nf4_index_search(x);
  if (a != want || b != want) {
    std::printf("MISMATCH x=%.9g bits=%08x plain=%u bucket=%u search=%u\n", x, to_bits(x), want, a, b);
    return false;
  }
  return true;
}
static bool around(float c, int ulps) {
  const uint32_t u = to_bits(c);
  for (int d = -ulps; d <= ulps; ++d)
    if (!check(from_bits(u + (uint32_t)d))) return false;       // same sign neighbourhood (c is never 0 here)
  return true;
}

int main() {
  for (int j = 0; j < 15; ++j) if (!around(nf4_threshold(j), 4096)) return 1;
  for (int b = -20; b <= 20; ++b) {
    if (b == 0) continue;
    if (!around((float)b / 16.0f, 4096)) return 1;
  }
  const float specials[] = {0.0f, -0.0f, 1e-45f, -1e-45f, 1e-30f, -1e-30f, 1.0f, -1.0f, 1.0000001f, -1.0000001f,
                            2.0f, -2.0f, 3.4e38f, -3.4e38f};
  for (float x : specials) if (!check(x)) return 1;
  for (int d = -4096; d <= 4096; ++d) {                           // both sides of zero
    if (!check(from_bits((uint32_t)(d < 0 ? -d : d) | (d < 0 ? 0x80000000u : 0u)))) return 1;
  }
  // dense sweep: every 13th float of [-1.25, 1.25]
  for (uint32_t u = to_bits(1e-8f); u <= to_bits(1.25f); u += 13u) {
    if (!check(from_bits(u)) || !check(from_bits(u | 0x80000000u))) return 1;
  }
  std::printf("OK %lld\n", checked);
  return 0;
}
