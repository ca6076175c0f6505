// Host-side check of the reciprocal divisions the kernels use (paper_1412_4564_amd/csrc/fastdiv.h) against the
// integer division of the language.  Built and run by tests/test_host_fastdiv.py; prints OK or the first mismatch.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <initializer_list>
#include "fastdiv.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {          // xorshift64*
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return rng_state * 0x2545F4914F6CDD1Dull;
}

static long checked = 0;
static void check32(int d, int64_t n) {
    if (n < 0 || n > 0x7fffffffll) return;
    const mcn::Div32 f = mcn::make_div32(d);
    const int q = mcn::div32((int)n, f);
    ++checked;
    if (q != (int)(n / d)) { printf("MISMATCH div32 n=%lld d=%d got %d want %lld\n", (long long)n, d, q, (long long)(n / d)); exit(1); }
}
static void check64(unsigned d, uint64_t n) {
    if (n > 0xffffffffull) return;
    const mcn::FastDiv64 f = mcn::make_fastdiv64(d);
    const unsigned q = mcn::div64((unsigned)n, f);
    ++checked;
    if (q != (unsigned)(n / d)) { printf("MISMATCH div64 n=%llu d=%u got %u want %llu\n", (unsigned long long)n, d, q, (unsigned long long)(n / d)); exit(1); }
}
// the places where a wrong reciprocal shows first: around multiples of d, most of all the largest ones
static void around32(int d) {
    const int64_t top = 0x7fffffffll;
    const int64_t ks[] = {0, 1, 2, top / d, top / d - 1, top / d / 2, (int64_t)(rnd() % (uint64_t)(top / d + 1))};
    for (int64_t k : ks)
        for (int64_t e = -2; e <= 2; ++e) check32(d, k * d + e);
    check32(d, top);
    for (int i = 0; i < 4; ++i) check32(d, (int64_t)(rnd() & 0x7fffffff));
}
static void around64(unsigned d) {
    const uint64_t top = 0xffffffffull;
    const uint64_t ks[] = {0, 1, 2, top / d, top / d - 1, top / d / 2, rnd() % (top / d + 1)};
    for (uint64_t k : ks)
        for (int e = -2; e <= 2; ++e) check64(d, k * d + (uint64_t)(int64_t)e);
    check64(d, top);
    for (int i = 0; i < 4; ++i) check64(d, rnd() & 0xffffffffull);
}

int main() {
    // every divisor up to 2^17, then powers of two and their neighbours, then random ones
    for (int d = 1; d < (1 << 17); ++d) { around32(d); around64((unsigned)d); }
    for (int b = 17; b < 31; ++b)
        for (int e = -3; e <= 3; ++e) { around32((1 << b) + e); around64((1u << b) + (unsigned)e); }
    for (int e = 0; e < 4; ++e) { around32(0x7fffffff - e); around64(0xffffffffu - (unsigned)e); around64(0x80000000u + (unsigned)e); }
    for (int i = 0; i < 200000; ++i) { around32((int)(rnd() % 0x7fffffffull) + 1); around64((unsigned)(rnd() % 0xffffffffull) + 1u); }
    // planes of pooling layers: the flat index e = i + H*j of the last two columns splits into (i, j), for every plane
    // height and the widest plane the library accepts (H*W < 2^31)
    for (int H = 1; H <= 70000; ++H) {
        const int64_t W = 0x7fffffffll / H;
        const mcn::Div32 f = mcn::make_div32(H);
        for (int64_t j = (W > 2 ? W - 2 : 0); j < W; ++j)
            for (int64_t i : {(int64_t)0, (int64_t)1, (int64_t)H / 2, (int64_t)H - 2, (int64_t)H - 1}) {
                if (i < 0 || i >= H) continue;
                const int64_t e = i + (int64_t)H * j;
                const int q = mcn::div32((int)e, f);
                ++checked;
                if (q != j || e - (int64_t)q * H != i) { printf("MISMATCH plane H=%d W=%lld e=%lld got j=%d\n", H, (long long)W, (long long)e, q); return 1; }
            }
    }
    // sizes at which a reciprocal exact only for n*d < 2^32 fails: 2240 x 2240, 3000 x 3000, 1500 x 6000
    const int HW[][2] = {{2240, 2240}, {3000, 3000}, {1500, 6000}, {32767, 32767}, {46340, 46340}};
    for (auto &hw : HW) {
        const mcn::Div32 f = mcn::make_div32(hw[0]);
        for (int64_t e = (int64_t)hw[0] * hw[1] - 3 * hw[0]; e < (int64_t)hw[0] * hw[1]; ++e) {
            ++checked;
            if (mcn::div32((int)e, f) != (int)(e / hw[0])) { printf("MISMATCH plane %dx%d e=%lld\n", hw[0], hw[1], (long long)e); return 1; }
        }
    }
    printf("OK %ld\n", checked);
    return 0;
}
