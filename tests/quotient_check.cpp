// CPU check of the five-operation quotient (granq_quotient.h, the product's own
// source) against the correctly rounded division `/`, on random and on
// adversarial operand pairs.  Prints the number of mismatches of
//   (a) the quotient itself where the theorem applies (|x| in [2^-100, 2^90] and
//       |x/s| >= 2^-40: no underflow anywhere),
//   (b) the derived code u = rint(q + z) everywhere else.
// Build: g++ -O2 -ffp-contract=off [-mfma] quotient_check.cpp -o quotient_check
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>
#include "granq_quotient.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static inline uint64_t next() {               // xorshift64*
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return rng_state * 0x2545F4914F6CDD1Dull;
}
static inline float from_bits(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
static inline uint32_t bits_of(float f) { uint32_t b; memcpy(&b, &f, 4); return b; }

static long bad_q = 0, bad_u = 0, checked = 0;

static void check(float x, float s, float z) {
    if (!granq::quotient_fast_ok(s, z)) return;
    if (!(x == x) || std::fabs(x) > 3.0e38f) return;
    ++checked;
    const float r = 1.0f / s;
    const float want = x / s;
    const float got = granq::quotient_fast(granq::quotient_clamp(x), s, r);
    const float ax = std::fabs(x);
    if (ax >= 0x1p-100f && ax <= 0x1p90f && std::fabs(want) >= 0x1p-40f) {
        if (bits_of(want) != bits_of(got) && !(want == 0.0f && got == 0.0f)) {
            if (bad_q < 10) std::printf("quotient mismatch x=%a s=%a want=%a got=%a\n", x, s, want, got);
            ++bad_q;
        }
    }
    for (int bits = 1; bits <= 8; bits += 7) {
        const float qmax = (float)((1 << bits) - 1);
        float uw = rintf(want + z), ug = rintf(got + z);
        float cw = fminf(fmaxf(uw, 0.0f), qmax), cg = fminf(fmaxf(ug, 0.0f), qmax);
        bool iw = uw >= 0.0f && uw <= qmax, ig = ug >= 0.0f && ug <= qmax;
        if (cw != cg || iw != ig) {
            if (bad_u < 10) std::printf("code mismatch x=%a s=%a z=%a want u=%a got u=%a\n", x, s, z, uw, ug);
            ++bad_u;
        }
    }
}

int main(int argc, char **argv) {
    long n = argc > 1 ? atol(argv[1]) : 20000000;
    // 1. random bit patterns for x, s across the whole admissible window
    for (long i = 0; i < n; ++i) {
        uint64_t a = next(), b = next();
        float x = from_bits((uint32_t)a);
        float s = from_bits(((uint32_t)b & 0x007FFFFFu) | ((uint32_t)(97 + (b >> 40) % 91) << 23));  // 2^-30..2^60
        float z = (float)((int)((a >> 32) % 513) - 256);
        check(x, s, z);
    }
    // 2. activations-like magnitudes, small integer zero-points
    for (long i = 0; i < n; ++i) {
        uint64_t a = next(), b = next();
        float x = from_bits(((uint32_t)a & 0x807FFFFFu) | ((uint32_t)(110 + (a >> 40) % 30) << 23));
        float s = from_bits(((uint32_t)b & 0x007FFFFFu) | ((uint32_t)(110 + (b >> 40) % 30) << 23));
        check(x, s, (float)((b >> 52) % 16));
    }
    // 3. near ties of the code: x ~ s * (k + 1/2), and its neighbours
    for (long i = 0; i < n / 4; ++i) {
        uint64_t a = next(), b = next();
        float s = from_bits(((uint32_t)b & 0x007FFFFFu) | ((uint32_t)(117 + (b >> 40) % 20) << 23));
        float k = (float)(a % 256);
        float x = s * (k + 0.5f);
        for (int d = -2; d <= 2; ++d) check(from_bits(bits_of(x) + d), s, (float)((a >> 20) % 5));
    }
    // 4. awkward significands: all ones, one, one plus an ulp, for both operands
    const uint32_t sig[] = {0x000000u, 0x000001u, 0x7FFFFFu, 0x7FFFFEu, 0x400000u, 0x3FFFFFu, 0x400001u, 0x555555u, 0x2AAAAAu};
    for (uint32_t sx : sig) for (uint32_t ss : sig)
        for (int ex = 1; ex < 255; ++ex) for (int es = 97; es <= 187; ++es)
            for (int neg = 0; neg < 2; ++neg)
                check(from_bits(sx | ((uint32_t)ex << 23) | ((uint32_t)neg << 31)), from_bits(ss | ((uint32_t)es << 23)), 3.0f);
    // 5. zeros, subnormals, the largest finite values
    const float xs[] = {0.0f, -0.0f, 0x1p-149f, -0x1p-149f, 0x1p-127f, 0x1p-126f, 0x1.fffffep127f, -0x1.fffffep127f, 0x1p-101f, 0x1p-100f, 0x1p90f, 0x1.000002p90f};
    for (float x : xs) for (int es = 97; es <= 187; ++es) for (uint32_t ss : sig)
        for (float z : {0.0f, 1.0f, -7.0f, 0.3f, 0.49999997f, 67108864.0f, -67108864.0f})
            check(x, from_bits(ss | ((uint32_t)es << 23)), z);
    std::printf("checked %ld pairs: %ld quotient mismatches, %ld code mismatches\n", checked, bad_q, bad_u);
    return (bad_q || bad_u) ? 1 : 0;
}
