"""The LayerNorm kernel replaces the division d/i of the running-mean update (Eq. 5) by
    q0 = RN(d * rk),  r = d - q0*i (one FMA, exact),  q = RN(q0 + r*rk),   rk = RN(1/i),
which is only legitimate if it returns the bits of the IEEE division.  That was established by
exhaustion over all 2^23 significands for every i <= 16384; this test re-checks a slice of that
space on every run (all divisors the kernel's table holds, a few thousand significands each,
the extreme ones included) with a small C program, so a change of the scheme cannot go unnoticed.
The check is arithmetic on the host: it shares nothing with the kernel but the formula."""
import os
import subprocess
import tempfile

SRC = r"""
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
int main(void) {
    long long bad = 0, n = 0;
    uint32_t lcg = 12345u;
    for (int k = 1; k <= 4096; ++k) {
        const float kf = (float)k, rk = 1.0f / kf;
        for (int s = 0; s < 6000; ++s) {
            uint32_t m;
            if (s < 64) m = (uint32_t)s;                          /* smallest significands   */
            else if (s < 128) m = (1u << 23) - 1u - (uint32_t)(s - 64);   /* largest           */
            else { lcg = lcg * 1664525u + 1013904223u; m = lcg >> 9; }
            uint32_t bits = 0x3F800000u | m;
            float a; memcpy(&a, &bits, 4);
            for (int e = -60; e <= 60; e += 60) {                 /* the exponent only scales */
                const float d = ldexpf(a, e);
                const float want = d / kf;
                const float q0 = d * rk;
                const float r = fmaf(-q0, kf, d);
                const float q = fmaf(r, rk, q0);
                bad += (q != want); ++n;
            }
        }
    }
    printf("%lld %lld\n", n, bad);
    return bad != 0;
}
"""


def test_corrected_reciprocal_multiply_equals_ieee_division():
    with tempfile.TemporaryDirectory() as d:
        src, exe = os.path.join(d, "chk.c"), os.path.join(d, "chk")
        with open(src, "w") as f:
            f.write(SRC)
        subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-march=native", src, "-o", exe, "-lm"], check=True)
        out = subprocess.run([exe], capture_output=True, text=True)
        n, bad = (int(v) for v in out.stdout.split())
        assert out.returncode == 0 and bad == 0 and n == 4096 * 6000 * 3
