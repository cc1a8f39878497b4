/*
 * TEST INFRASTRUCTURE -- NOT part of the product path.
 *
 * Plain, slow CPU oracle for one worker's hot path of the training method of
 * "One weird trick for parallelizing convolutional neural networks":
 * convolution forward / backward-data / backward-filter, the worker's column
 * shard of the fully-connected layers, and the max-pooling that joins the
 * layers (Section 4, forward steps 1-3 and backward steps 1-2; Section 5 for
 * the model), plus the weight update rule and the logistic output layer of
 * Section 5.  Only tests, the smoke check and the benchmark's cpu_baseline
 * leg may call it; the HIP library shares no code with it.
 *
 * Build: gcc -O3 -march=native -fopenmp -shared -fPIC owt_oracle.c -o liboracle.so
 *
 * Parity status: every function here is pinned by the CPU tests
 * (1x1 conv == matmul, delta filters, adjoint identities, finite differences,
 * closed forms for pooling and padding, hand-picked bf16 bit patterns;
 * the update rule by its closed forms and the weight-decay example the paper
 * prints, the logistic output layer by the textbook formula and finite
 * differences).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define REAL float
#define SUFFIX f32
#include "owt_oracle_impl.inc"
#undef REAL
#undef SUFFIX

#define REAL double
#define SUFFIX f64
#include "owt_oracle_impl.inc"
#undef REAL
#undef SUFFIX

/* fp32 -> bf16 -> fp32, round-to-nearest-even on the 16 dropped mantissa bits.
 * bf16 keeps the sign, the 8 exponent bits and the top 7 mantissa bits of an
 * IEEE-754 binary32.  NaN stays NaN (quiet bit forced), +-inf and +-0 are exact. */
void oracle_round_bf16(const float *in, float *out, size_t n)
{
    for (size_t i = 0; i < n; i++) {
        uint32_t u;
        memcpy(&u, &in[i], 4);
        if ((u & 0x7f800000u) == 0x7f800000u && (u & 0x007fffffu)) {
            u = (u | 0x00400000u) & 0xffff0000u;
        } else {
            const uint32_t lsb = (u >> 16) & 1u;
            u += 0x7fffu + lsb;
            u &= 0xffff0000u;
        }
        memcpy(&out[i], &u, 4);
    }
}

/* Hyperparameters for a batch k times larger (Section 5): the learning rate
 * grows by sqrt(k); the weight decay is chosen so that one application at the
 * new batch size shrinks a weight as much as k applications did before:
 * (1 - eps*omega)^k = 1 - eps2*omega2. */
void oracle_scale_hyperparameters(double k, double eps, double omega, double *eps2, double *omega2)
{
    *eps2 = sqrt(k) * eps;
    *omega2 = (1.0 - pow(1.0 - eps * omega, k)) / *eps2;
}

int oracle_abi_version(void) { return 2; }

/* Threads the OpenMP loops above run on. */
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
