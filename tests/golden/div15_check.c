/* x / 15 == x * fl(1/15) followed by one fused correction step, for every float mantissa.
 * The encoder's kernels use the right-hand side for (max - min) / 15 (paper Sec. 2, the
 * scale of the asymmetric 4-bit quantiser); the CPU oracle divides.  Exit code 0: equal
 * for all 2^23 mantissas at each exponent given on the command line. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float shortcut(float a)
{
    const float y = 0x1.111112p-4f;
    float q = a * y;
    float r = fmaf(-15.0f, q, a);
    return fmaf(r, y, q);
}

int main(int argc, char **argv)
{
    long bad = 0;
    for (int k = 1; k < argc; ++k) {
        const uint32_t e = (uint32_t)atoi(argv[k]);  /* biased exponent, 1..254 */
        for (uint32_t m = 0; m < (1u << 23); ++m) {
            const uint32_t b = (e << 23) | m;
            float a, ref, got;
            memcpy(&a, &b, 4);
            volatile float d = a / 15.0f;
            ref = d;
            got = shortcut(a);
            bad += memcmp(&ref, &got, 4) != 0;
        }
    }
    printf("%ld\n", bad);
    return bad != 0;
}
