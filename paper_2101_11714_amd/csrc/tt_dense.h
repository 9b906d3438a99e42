// Uncompressed EmbeddingBag on the same GPU: the in-box comparison for the pooling-factor and
// hit-rate microbenchmarks (the role PyTorch's EmbeddingBag plays in Section 6.6 / 6.7 of the
// paper).  table is fp32 [num_rows][N], N a multiple of 4.  Not part of the TT path.
#pragma once

#include "tt_common.h"

namespace tt {

// out[bag] = sum_k alpha[k] table[indices[k]]: one wave per bag, lane l owns float4 (l % (N/4)) of the
// row and the lanes of a wave take the bag's positions 64 / (N/4) at a time.
__global__ __launch_bounds__(WG) void dense_fwd_kernel(const float *__restrict__ table, int N,
                                                       const int64_t *__restrict__ indices,
                                                       const int64_t *__restrict__ offsets, int n_bags,
                                                       const float *__restrict__ alpha, float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int bag = blockIdx.x * NWAVE + (threadIdx.x >> 6);
    if (bag >= n_bags) return;
    const int nq = N / 4;                        // float4 per row: 4 or 16 here, a power of two <= 64
    const int per = WAVE / nq;                   // positions in flight per wave
    const int f = lane % nq, sub = lane / nq;
    const int k0 = offsets ? (int)offsets[bag] : bag, k1 = offsets ? (int)offsets[bag + 1] : bag + 1;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k = k0 + sub; k < k1; k += per) {
        const float w = alpha ? alpha[k] : 1.f;
        const float4 v = *reinterpret_cast<const float4 *>(table + (size_t)indices[k] * N + 4 * f);
        acc.x = fmaf(w, v.x, acc.x); acc.y = fmaf(w, v.y, acc.y); acc.z = fmaf(w, v.z, acc.z); acc.w = fmaf(w, v.w, acc.w);
    }
    for (int d = nq; d < WAVE; d <<= 1) {        // add the partial sums of the position groups
        acc.x += __shfl_xor(acc.x, d); acc.y += __shfl_xor(acc.y, d);
        acc.z += __shfl_xor(acc.z, d); acc.w += __shfl_xor(acc.w, d);
    }
    if (sub == 0) *reinterpret_cast<float4 *>(out + (size_t)bag * N + 4 * f) = acc;
}

// table[indices[k]] -= lr alpha[k] grad_out[bag(k)] for every position (sparse SGD; floating-point
// atomics, so rows that occur more than once are updated in no fixed order).
__global__ __launch_bounds__(WG) void dense_bwd_sgd_kernel(float *__restrict__ table, int N,
                                                           const int64_t *__restrict__ indices,
                                                           const int64_t *__restrict__ offsets, int n_bags,
                                                           const float *__restrict__ alpha,
                                                           const float *__restrict__ grad_out, float lr)
{
    const int lane = threadIdx.x & 63;
    const int bag = blockIdx.x * NWAVE + (threadIdx.x >> 6);
    if (bag >= n_bags) return;
    const int per = WAVE / N > 0 ? WAVE / N : 1; // positions in flight per wave (N <= 64), else columns in turns
    const int k0 = offsets ? (int)offsets[bag] : bag, k1 = offsets ? (int)offsets[bag + 1] : bag + 1;
    for (int c0 = 0; c0 < N; c0 += WAVE) {
        const int c = c0 + lane % (N < WAVE ? N : WAVE), sub = N < WAVE ? lane / N : 0;
        if (c >= N) continue;
        const float g = grad_out[(size_t)bag * N + c];
        for (int k = k0 + sub; k < k1; k += per) {
            const float w = alpha ? alpha[k] : 1.f;
            unsafeAtomicAdd(table + (size_t)indices[k] * N + c, -lr * w * g);
        }
    }
}

}  // namespace tt
