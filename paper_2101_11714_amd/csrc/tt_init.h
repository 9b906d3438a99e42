// Sampled Gaussian initialisation of the cores on the device (Section 3.2, Alg. 3 of the paper):
// every entry is drawn from N(0,1) and redrawn while |x| <= 2, then scaled so that an entry of
// the reconstructed table has variance 1 / (3 num_rows).
//
// The random numbers come from a counter-based generator (SplitMix64's finaliser applied to seed,
// core, element and attempt), so every entry is independent of the launch shape and can be
// reproduced anywhere: for core c, element e, attempt t,
//   h = mix(mix(seed + GOLD (c + 1)) ^ e),  a = mix(h + T_MUL t),  b = mix(a ^ B_XOR),
//   u1 = ((a >> 11) + 0.5) 2^-53,  u2 = (b >> 11) 2^-53,  z = sqrt(-2 ln u1) cos(2 pi u2).
// The transform and the accept test run in fp64, so that the decision |z| > 2 is the same on
// every implementation up to an event of probability ~1e-15 per attempt.
#pragma once

#include "tt_common.h"

namespace tt {

__device__ __forceinline__ uint64_t init_mix64(uint64_t x)
{
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

__global__ __launch_bounds__(WG) void init_sampled_gaussian_kernel(float *__restrict__ core, int64_t count, int core_id,
                                                                   uint64_t seed, double scale)
{
    const uint64_t base = init_mix64(seed + 0x9E3779B97F4A7C15ull * (uint64_t)(core_id + 1));
    for (int64_t e = (int64_t)blockIdx.x * WG + threadIdx.x; e < count; e += (int64_t)gridDim.x * WG) {
        const uint64_t h = init_mix64(base ^ (uint64_t)e);
        double z;
        for (uint64_t t = 0;; ++t) {                               // ends: every attempt succeeds with probability 0.0455
            const uint64_t a = init_mix64(h + 0xD1342543DE82EF95ull * t);
            const uint64_t b = init_mix64(a ^ 0xA0761D6478BD642Full);
            const double u1 = ((double)(a >> 11) + 0.5) * (1.0 / 9007199254740992.0);
            const double u2 = (double)(b >> 11) * (1.0 / 9007199254740992.0);
            z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
            if (fabs(z) > 2.0) break;
        }
        core[e] = (float)(z * scale);
    }
}

// (1 / (3 num_rows R1 R2 v^3))^(1/6), v = E[z^2 | |z| > 2] = 1 + 2 phi(2) / P(z > 2): an entry of the
// table is a sum of R1 R2 products of three core entries of second moment v scale^2 each
static inline double sampled_gaussian_scale(int64_t num_rows, int R1, int R2)
{
    const double two_pi = 6.283185307179586476925286766559;
    const double phi2 = exp(-2.0) / sqrt(two_pi);
    const double tail = 0.5 * erfc(2.0 / sqrt(2.0));
    const double v = 1.0 + 2.0 * phi2 / tail;
    return pow(1.0 / (3.0 * (double)num_rows * (double)R1 * (double)R2 * v * v * v), 1.0 / 6.0);
}

}  // namespace tt
