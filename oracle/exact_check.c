/*
 * Exact-integer pin for the CPU oracle (test infrastructure, never on the
 * product path; shares nothing with the HIP sources).
 *
 * Every finite binary16 value is an integer multiple of 2^-24 with
 * |v| * 2^24 < 2^40, so the reduction R(X) = sum x_i (Section 4 of the paper)
 * can be carried out with no rounding at all in 128-bit integers.  The result
 * is the mathematically exact sum in units of 2^-24; the Kahan oracle must
 * agree with it to within a couple of binary64 ulps.  The decoder here works
 * on integers only and is written independently of the oracle's floating
 * decoder, so a mistake in either shows up as a disagreement.
 */
#include <stddef.h>
#include <stdint.h>

/* out[0..1] = low, high 64 bits of the signed exact sum   (units of 2^-24)
 * out[2..3] = low, high 64 bits of the exact sum of |x_i| (units of 2^-24)
 * returns the number of non-finite inputs (those are skipped). */
size_t exact_sum_f16(const uint16_t *x, size_t n, uint64_t out[4])
{
    __int128 s = 0;
    unsigned __int128 a = 0;
    size_t nonfinite = 0;
    for (size_t i = 0; i < n; ++i) {
        const uint16_t h = x[i];
        const unsigned e = (h >> 10) & 0x1fu;
        const uint64_t f = h & 0x3ffu;
        if (e == 31u) { ++nonfinite; continue; }
        const uint64_t k = e ? ((1024u + f) << (e - 1u)) : f;
        a += k;
        if (h & 0x8000u) s -= (__int128)k; else s += (__int128)k;
    }
    out[0] = (uint64_t)(unsigned __int128)s;
    out[1] = (uint64_t)((unsigned __int128)s >> 64);
    out[2] = (uint64_t)a;
    out[3] = (uint64_t)(a >> 64);
    return nonfinite;
}
