// Division of a flat element number by a length that is fixed per launch (row length, map width).
// Plain C++: no HIP types, so host-side checks can compile it with any compiler.
#ifndef SBP_FASTDIV_H_
#define SBP_FASTDIV_H_

#include <stdint.h>

#if defined(__HIPCC__)
#define SBP_HD __host__ __device__ __forceinline__
#else
#define SBP_HD inline
#endif

namespace sbp {

// Exact unsigned 32-bit division by a divisor fixed per launch (Granlund and Montgomery's multiply-and-shift, in the
// form that needs no branch for any divisor >= 1): a handful of instructions where the 64-bit division of a flat
// element number by a run-time row length costs about a hundred.  Holds for every n < 2^32.
struct FastDiv {
  uint32_t d, m, s1, s2;
  FastDiv() = default;
  explicit FastDiv(uint32_t div) : d(div) {
    uint32_t s = 0;
    while (s < 32 && (1ull << s) < div) ++s;                               // s = ceil(log2 d)
    m = (uint32_t)((((1ull << s) - div) << 32) / div) + 1u;
    s1 = s < 1 ? s : 1;
    s2 = s < 1 ? 0 : s - 1;
  }
  SBP_HD uint32_t div(uint32_t n) const {
#ifdef __HIP_DEVICE_COMPILE__
    const uint32_t t = __umulhi(m, n);
#else
    const uint32_t t = (uint32_t)(((uint64_t)m * n) >> 32);
#endif
    return (t + ((n - t) >> s1)) >> s2;
  }
  SBP_HD void divmod(uint32_t n, uint32_t& q, uint32_t& r) const {
    q = div(n);
    r = n - q * d;
  }
};

}  // namespace sbp
#endif
