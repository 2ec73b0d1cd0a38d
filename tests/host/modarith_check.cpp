// Host-side check of the device arithmetic header: the FP64 routines are plain
// IEEE-754 double operations with explicit fma, so they behave identically on
// the CPU.  Compared against 128-bit integer arithmetic.
#include <cstdio>
#include <cstdlib>
#include <cmath>
#include <cstdint>
#include "../../paper_2602_08798_amd/csrc/modarith.hpp"

typedef unsigned __int128 u128;
typedef __int128 i128;
static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd()
{
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static int64_t pmod(i128 x, int64_t p) { i128 r = x % p; if (r < 0) r += p; return (int64_t)r; }

int main()
{
    const uint64_t primes[] = {(1ull << 50) - 16383, (1ull << 50) - 212991, (1ull << 50) - 5177343,
                               (1ull << 49) + 1 + 2 * 8192ull * 3 /* not prime: arithmetic still must hold */,
                               1099511922689ull /* ~2^40 */};
    long bad = 0;
    for (uint64_t p : primes) {
        cg::ModD m{(double)p, 1.0 / (double)p};
        cg::ModI mi{p, (uint64_t)((((u128)1) << 100) / p)};
        // lazy factors: |a| <= A p, |b| <= B p with A*B <= 16
        const double As[] = {1, 2.64, 7.9, 0.5, 4, 2};
        const double Bs[] = {1, 2.64, 0.5, 0.5, 4, 7.9};
        for (int cfg = 0; cfg < 6; cfg++) {
            for (long it = 0; it < 400000; it++) {
                int64_t amax = (int64_t)(As[cfg] * (double)p), bmax = (int64_t)(Bs[cfg] * (double)p);
                int64_t a = (int64_t)(rnd() % (2 * (uint64_t)amax + 1)) - amax;
                int64_t b = (int64_t)(rnd() % (2 * (uint64_t)bmax + 1)) - bmax;
                if (it < 64) {  // extremes
                    a = (it & 1) ? amax : -amax; b = (it & 2) ? bmax : -bmax;
                    if (it & 4) a -= (it >> 3); if (it & 8) b += (it >> 4);
                    if (a > amax) a = amax; if (b > bmax) b = bmax;
                }
                double r = cg::mulmod((double)a, (double)b, m);
                double bound = (0.5 + 3.0 * As[cfg] * Bs[cfg] / 8.0) * (double)p + 1.0;
                if (r != std::floor(r) || std::fabs(r) > bound) { bad++; continue; }
                if (pmod((i128)(int64_t)r, (int64_t)p) != pmod((i128)a * b, (int64_t)p)) bad++;
                double c = cg::canon((double)a, m);
                if (c < 0 || c >= (double)p || (int64_t)c != pmod(a, (int64_t)p)) bad++;
                double rr = cg::red((double)a, m);
                if (std::fabs(rr) > 0.5 * (double)p + 1.0 || pmod((i128)(int64_t)rr, (int64_t)p) != pmod(a, (int64_t)p)) bad++;
            }
        }
        for (long it = 0; it < 400000; it++) {
            uint64_t a = rnd() % p, b = rnd() % p;
            if (it < 4) { a = p - 1 - (it & 1); b = p - 1 - (it >> 1); }
            if (cg::f64_to_u64(cg::u64_to_f64(a)) != a) bad++;
            if (p > (1ull << 49) && cg::mulmod_barrett(a, b, mi) != (uint64_t)((u128)a * b % p)) bad++;
            double s = cg::addmod_canon((double)a, (double)b, m);
            if ((uint64_t)s != (a + b) % p) bad++;
        }
    }
    std::printf("modarith_check mismatches: %ld\n", bad);
    return bad ? 1 : 0;
}
