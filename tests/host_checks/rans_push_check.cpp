// Host check of the row coder's exact division (paper_2212_01185_amd/csrc/rans_arith.h): the very source the
// HIP kernels compile, built here with the host compiler, against 64-bit integer division.
//
// For every frequency f = 1 .. 65536 (65536 is the padding symbol's) and a set of states x in [2^31, f * 2^47)
// -- the lower and upper ends, multiples of f and their neighbours, powers of two and their neighbours, states
// just below the renormalisation threshold, and seeded random ones -- rans_push must return exactly
// ((x / f) << 16) + (x % f) + start.  The reciprocal is built from seeds off by up to +-2^-23 relative (the
// accuracy class of a hardware fp64 reciprocal estimate) and in both host rounding modes that the GPU's loader
// waves could be in; the push itself runs with rounding toward zero, as the coding wave does.
// Prints one line "checked <n> failures <m>" and exits 0 iff m == 0.
#include <cfenv>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>

static double g_seed_scale = 1.0;
static inline double seed_rcp(double fd) { return (1.0 / fd) * g_seed_scale; }

#define PCC_RANS_HD static inline
#define PCC_RANS_RCP_SEED(fd) seed_rcp(fd)
#include "rans_arith.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static inline uint64_t rnd() {   // splitmix64
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

int main() {
    const uint64_t L = 1ull << 31;
    unsigned long long checked = 0, failures = 0, recip_bad = 0;
    const double scales[3] = {1.0, 1.0 + 0x1p-23, 1.0 - 0x1p-23};
    for (int si = 0; si < 3; ++si) {
        g_seed_scale = scales[si];
        for (uint32_t f = 1; f <= 65536; ++f) {
            std::fesetround(FE_TONEAREST);
            const double rf = pcc::rans_recip_below(f);
            // strictly below 1/f, and by no more than 2^-49 relative: the residual rf * f - 1 is computed exactly by one fma
            const double resid = std::fma(rf, (double)f, -1.0);
            if (!(resid < 0.0) || resid < -0x1p-49) ++recip_bad;
            const uint64_t top = (uint64_t)f << 47;     // states are below this when they are pushed
            uint64_t xs[48];
            int nx = 0;
            xs[nx++] = L; xs[nx++] = L + 1; xs[nx++] = top - 1; xs[nx++] = top - 2;
            xs[nx++] = top - f; xs[nx++] = top - f - 1; xs[nx++] = top - f + 1;
            for (int b = 32; b < 63; b += 5) {
                const uint64_t p = 1ull << b;
                if (p < top) { xs[nx++] = p; xs[nx++] = p - 1; }
            }
            for (int i = 0; i < 8; ++i) {
                const uint64_t k = rnd() % ((top - L) / f) + (L + f - 1) / f;   // a multiple of f in range and its neighbours
                xs[nx++] = k * f; xs[nx++] = k * f - 1; if (k * f + 1 < top) xs[nx++] = k * f + 1;
            }
            while (nx < 48) xs[nx++] = L + rnd() % (top - L);
            std::fesetround(FE_TOWARDZERO);
            for (int i = 0; i < nx; ++i) {
                const uint64_t x = xs[i];
                if (x < L || x >= top) continue;
                const uint32_t start = f == 65536 ? 0u : (uint32_t)(rnd() % (65536u - f + 1u));
                uint32_t xl = (uint32_t)x, xh = (uint32_t)(x >> 32);
                pcc::rans_push(xl, xh, f, start, rf);
                const uint64_t got = ((uint64_t)xh << 32) | xl;
                const uint64_t want = ((x / f) << 16) + (x % f) + start;
                ++checked;
                if (got != want) {
                    if (failures < 10) std::printf("MISMATCH f=%u x=%llu start=%u got=%llu want=%llu\n", f, (unsigned long long)x, start,
                                                   (unsigned long long)got, (unsigned long long)want);
                    ++failures;
                }
            }
        }
    }
    std::fesetround(FE_TONEAREST);
    std::printf("checked %llu failures %llu recip_out_of_bounds %llu\n", checked, failures, recip_bad);
    return (failures == 0 && recip_bad == 0) ? 0 : 1;
}
