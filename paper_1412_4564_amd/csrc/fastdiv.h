// Division of a non-negative 32-bit integer by a block-wide constant as a multiplication, an addition and a
// shift (the round-up method of Granlund and Montgomery, "Division by invariant integers using multiplication"):
// with l = ceil(log2 d) and m = floor(2^32 (2^l - d) / d) + 1,
//     n / d = (floor(m n / 2^32) + n) >> l      exactly, for every 0 <= n < 2^31 and 1 <= d < 2^31.
// A hardware-less integer division is some 35 vector instructions, each of which takes issue cycles from the
// matrix core; the kernels divide by tile, plane and stride sizes that the host knows.
// The header also compiles as plain C++ so that a host program can check the identity against `/`.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define MCN_HOST_DEVICE __host__ __device__
#else
#define MCN_HOST_DEVICE
#endif

namespace mcn {

struct Div32 {
    unsigned m;
    int l;
};
inline Div32 make_div32(int d) {
    Div32 f;
    int l = 0;
    while (((int64_t)1 << l) < d) ++l;
    f.l = l;
    f.m = (unsigned)((((uint64_t)1 << 32) * (((uint64_t)1 << l) - (uint64_t)d)) / (uint64_t)d + 1);
    return f;
}
MCN_HOST_DEVICE inline int div32(int n, Div32 f) {
    const unsigned hi = (unsigned)(((uint64_t)f.m * (unsigned)n) >> 32);
    return (int)((hi + (unsigned)n) >> f.l);
}

// n / d for any 0 <= n < 2^32 and 1 <= d < 2^32:  m = ceil(2^64 / d), n / d = floor(n m / 2^64)
// (n (m d - 2^64) < n d < 2^64, so the error term never reaches the next integer; d = 1: m does not fit, n / 1 = n).
struct FastDiv64 {
    unsigned d;
    unsigned long long m;
};
inline FastDiv64 make_fastdiv64(unsigned d) {
    FastDiv64 f;
    f.d = d;
    f.m = d == 1 ? 0ull : ~0ull / d + 1;      // floor((2^64 - 1) / d) + 1 = ceil(2^64 / d) when d does not divide 2^64; powers of two: also exact
    return f;
}
MCN_HOST_DEVICE inline unsigned div64(unsigned n, FastDiv64 f) {
    // upper 64 bits of the 96-bit product n * m, taken in two 32 x 32 -> 64 products
    const uint64_t lo = (uint64_t)n * (unsigned)f.m, hi = (uint64_t)n * (unsigned)(f.m >> 32);
    return f.d == 1 ? n : (unsigned)((hi + (lo >> 32)) >> 32);
}

}  // namespace mcn
