/* Exhaustive check (host, no GPU) of the centroid update of the resident matrix-core kernel, which
 * computes the mean S / n of a cluster knob as
 *     r = fl(1 / n);  q0 = fl(S r);  rem = fma(-q0, n, S);  q = fma(rem, r, q0)
 * (one division per cluster instead of one per knob).  The kernel's domain is small enough to try
 * every case: counts 1 <= n <= 4096 (a resident task has at most 4096 rows) and integer sums
 * 0 <= S <= 255 n (byte knobs): about 2.1e9 pairs.  q must equal the correctly rounded quotient
 * fl(S / n), which is what the other kernels and the CPU reference compute (Sec. 3.3: a centroid is the mean
 * of its cluster; bit-equal centroids are what make the labels of the next pass comparable).
 * Needs hardware fused multiply-add on the host (gcc -O2 -mfma -fopenmp -ffp-contract=off).
 * Prints the number of mismatches; exit status 0 iff there is none. */
#include <math.h>
#include <stdio.h>

int main(void)
{
    long bad = 0, uncorrected = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : bad, uncorrected)
    for (int n = 1; n <= 4096; ++n) {
        const double dn = (double)n, r = 1.0 / dn;
        const long smax = 255L * n;
        for (long S = 0; S <= smax; ++S) {
            const double a = (double)S;
            const double q0 = a * r;
            const double rem = fma(-q0, dn, a);
            const double q = fma(rem, r, q0);
            const double ref = a / dn;
            if (q != ref) ++bad;
            if (q0 != ref) ++uncorrected;
        }
    }
    printf("quotient_check: %ld mismatches (the uncorrected product S * fl(1/n) differs in %ld cases)\n", bad,
           uncorrected);
    return bad != 0;
}
