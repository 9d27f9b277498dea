/*
 * CPU oracle for fused-tile-partitioned CNN training (forward + back-propagation of
 * convolution / leaky-ReLU / 2x2 max-pool layers).
 *
 * TEST INFRASTRUCTURE ONLY.  Imported by the tests, the smoke check and the benchmark's
 * cpu_baseline leg; the GPU library neither links nor calls it, and it shares no code,
 * headers or tables with the GPU path.
 *
 * The method reproduces the untiled network exactly (tiling must not change accuracy,
 * Sec. 1 and Sec. 4.1), so the oracle is the untiled definition written out.
 * Build: gcc -O2 -fopenmp -shared -fPIC ftp_oracle.c -o libftp_oracle.so
 */
#include <stdlib.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#include <omp.h>

#define REAL float
#define NAME(f) oracle_f32_##f
#include "ftp_oracle_impl.inc"
#undef REAL
#undef NAME

#define REAL double
#define NAME(f) oracle_f64_##f
#include "ftp_oracle_impl.inc"
#undef REAL
#undef NAME

/* fp32 -> nearest bf16 (ties to even), returned as the fp32 value it represents. */
void oracle_round_bf16(float* a, size_t count)
{
    #pragma omp parallel for
    for (long i = 0; i < (long)count; ++i) {
        uint32_t u;
        memcpy(&u, &a[i], 4);
        if ((u & 0x7F800000u) != 0x7F800000u) {
            u += 0x7FFFu + ((u >> 16) & 1u);
            u &= 0xFFFF0000u;
        }
        memcpy(&a[i], &u, 4);
    }
}

int oracle_num_threads(void)
{
    int n = 1;
    #pragma omp parallel
    {
        #pragma omp single
        n = omp_get_num_threads();
    }
    return n;
}
