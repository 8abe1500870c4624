/* Oracle: fp32 -> bf16 narrowing, round-to-nearest-even (IEEE-754
 * roundTiesToEven), written from the definition: of the two bf16 values that
 * bracket x, return the nearer one; on a tie the one whose last mantissa bit is
 * even.  Distances are compared in double, where every fp32 and bf16 value and
 * their differences are exact.  Overflow follows IEEE: the upper neighbour of
 * the largest finite bf16 is taken at its unbounded-exponent value 2^128 and
 * maps to infinity.  Subnormals are not flushed.
 *
 * NaN (a reading; IEEE leaves the payload open): keep the sign and the top 7
 * payload bits and force the quiet bit, so a NaN never turns into infinity.
 *
 * Test infrastructure only; shares nothing with the GPU library. */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

static double f32_magnitude(uint32_t mag) /* mag: bits 30..0 of a finite fp32 */
{
    int e = (int)(mag >> 23);
    uint32_t m = mag & 0x7FFFFFu;
    if (e == 0) return ldexp((double)m, -149);
    return ldexp((double)(0x800000u + m), e - 150);
}

static double bf16_magnitude(uint32_t mag) /* mag: bits 14..0 of a bf16, exponent 255 read as a normal binade */
{
    int e = (int)(mag >> 7);
    uint32_t m = mag & 0x7Fu;
    if (e == 0) return ldexp((double)m, -133);
    return ldexp((double)(0x80u + m), e - 134);
}

uint16_t oracle_narrow_one(uint32_t u)
{
    uint32_t sign = (u >> 31) << 15;
    uint32_t mag = u & 0x7FFFFFFFu;
    if (mag > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN */
    if (mag == 0x7F800000u) return (uint16_t)(sign | 0x7F80u);      /* Inf */
    double x = f32_magnitude(mag);
    uint32_t lo = mag >> 16;  /* largest bf16 magnitude <= x (same exponent field layout) */
    uint32_t hi = lo + 1;     /* next bf16 magnitude */
    double dl = x - bf16_magnitude(lo);
    double dh = bf16_magnitude(hi) - x;
    uint32_t pick;
    if (dl < dh) pick = lo;
    else if (dl > dh) pick = hi;
    else pick = (lo & 1u) ? hi : lo;
    return (uint16_t)(sign | pick);
}

void oracle_narrow_rne(const uint32_t* in, uint16_t* out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = oracle_narrow_one(in[i]);
}
