/*
 * IEEE binary16 bit pattern -> double, by fields  --  TEST INFRASTRUCTURE (part of the CPU oracle).
 */
#ifndef ORACLE_HALF_BITS_H
#define ORACLE_HALF_BITS_H
#include <math.h>
#include <stdint.h>

/* no half arithmetic anywhere: sign, exponent and fraction fields are read out */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);              /* zero and subnormals: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

#endif
