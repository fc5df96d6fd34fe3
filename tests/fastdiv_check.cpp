// Host-side check of the multiply-and-shift division the streaming kernels use for row / column numbers:
// compares it with the compiler's division on edge values and on a pseudo-random sample.  Prints "ok <count>"
// or the first mismatch.  Compiled and run by tests/test_abi_host.py.
#include <cstdint>
#include <cstdio>
#include <initializer_list>

#include "sbp_fastdiv.h"

static uint64_t next(uint64_t& s) {   // xorshift64
  s ^= s << 13; s ^= s >> 7; s ^= s << 17;
  return s;
}

static bool check(const sbp::FastDiv& f, uint32_t n, long long& count) {
  uint32_t q, r;
  f.divmod(n, q, r);
  ++count;
  if (q != n / f.d || r != n % f.d) {
    std::printf("mismatch: %u / %u gives %u rem %u\n", n, f.d, q, r);
    return false;
  }
  return true;
}

int main() {
  uint64_t seed = 0x9E3779B97F4A7C15ull;
  long long count = 0;
  const uint32_t fixed[] = {1, 2, 3, 4, 5, 7, 12, 16, 49, 64, 96, 168, 192, 197, 336, 384, 641, 1000, 3072, 65535, 65536, 65537,
                            0x7FFFFFFFu, 0x80000000u, 0x80000001u, 0xFFFFFFFEu, 0xFFFFFFFFu};
  for (int i = 0; i < 27 + 2000; ++i) {
    uint32_t d = i < 27 ? fixed[i] : (uint32_t)(next(seed) >> (32 + (i % 31)));
    if (d == 0) d = 1;
    const sbp::FastDiv f(d);
    const uint32_t edges[] = {0u, 1u, d - 1, d, d + 1, 2 * d - 1, 2 * d, 0xFFFFFFFFu, 0xFFFFFFFEu, 0x80000000u, 0x7FFFFFFFu,
                              0xFFFFFFFFu / d * d, 0xFFFFFFFFu / d * d - 1, 0xFFFFFFFFu / d * d + (d > 1 ? 1u : 0u)};
    for (uint32_t n : edges)
      if (!check(f, n, count)) return 1;
    for (int k = 0; k < 2000; ++k) {
      const uint32_t q = (uint32_t)(next(seed) % (0xFFFFFFFFull / d + 1));
      for (uint32_t n : {q * d, q * d + (uint32_t)(next(seed) % d), (uint32_t)next(seed)})
        if (!check(f, n, count)) return 1;
    }
  }
  std::printf("ok %lld\n", count);
  return 0;
}
