// Access-frequency tracker of the semi-dynamic cache (Section 4.2 of the paper): an
// open-addressing hash table row -> number of accesses, kept on the device and updated from the
// index stream of every step.  Integer only.
//
// An entry is one 64-bit word, (row << 32) | count, empty = all ones: inserting a row is one
// compare-and-swap, counting an access one 64-bit add of the right amount to the same word.
// Equal rows inside a wave are combined first (one add per distinct row and wave), so that a
// row that makes up a fifth of the stream does not turn into as many adds to one address.
#pragma once

#include "tt_common.h"

namespace tt {

constexpr uint64_t FREQ_EMPTY = ~0ull;

struct FreqDev {
    unsigned long long *table;
    unsigned long long *stats;      // [0] distinct rows in the table, [1] accesses dropped because it was full
    uint32_t mask;                  // capacity - 1
};

__global__ __launch_bounds__(WG) void freq_reset_kernel(FreqDev f)
{
    const uint32_t i = blockIdx.x * WG + threadIdx.x;
    if (i <= f.mask) f.table[i] = FREQ_EMPTY;
    if (i < 2) f.stats[i] = 0ull;
}

// add `n` accesses of `row`; linear probing from the same hash as the cache map
__device__ __forceinline__ void freq_add(const FreqDev &f, uint32_t row, uint32_t n)
{
    uint32_t h = cache_hash(row, f.mask);
    for (uint32_t probes = 0; probes <= f.mask; ++probes) {
        unsigned long long e = __hip_atomic_load(&f.table[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (e == FREQ_EMPTY) {
            const unsigned long long fresh = (unsigned long long)row << 32;
            e = atomicCAS(&f.table[h], (unsigned long long)FREQ_EMPTY, fresh);
            if (e == FREQ_EMPTY) {
                atomicAdd(&f.stats[0], 1ull);
                e = fresh;
            }
        }
        if ((uint32_t)(e >> 32) == row) {
            atomicAdd(&f.table[h], (unsigned long long)n);
            return;
        }
        h = (h + 1) & f.mask;
    }
    atomicAdd(&f.stats[1], (unsigned long long)n);                 // table full
}

__global__ __launch_bounds__(WG) void freq_update_kernel(FreqDev f, const int64_t *__restrict__ indices, int L)
{
    const int k = blockIdx.x * WG + threadIdx.x;
    const bool in = k < L;
    const uint32_t my = in ? (uint32_t)indices[k] : 0xFFFFFFFFu;
    const int lane = threadIdx.x & 63;
    // equal rows of the wave are combined without touching memory: the first lane of every
    // distinct row becomes its leader and learns how many lanes hold it ...
    uint64_t rem = __ballot(in);
    uint32_t mine = 0;
    while (rem) {                                                  // uniform: one step per distinct row of the wave
        const int j = __builtin_ctzll(rem);
        const uint32_t rj = (uint32_t)__builtin_amdgcn_readlane((int)my, j);
        const uint64_t m = __ballot(my == rj);
        rem &= ~m;
        if (lane == j) mine = (uint32_t)__popcll(m);
    }
    // ... then all leaders update the table at the same time
    if (mine) freq_add(f, my, mine);
}

// Long streams: a workgroup first counts its FQ_CHUNK positions in a small table in LDS (LDS
// atomics; equal rows meet there), then adds every distinct row of the chunk to the device table
// once.  The hottest row of a Zipf stream then costs one device atomic per chunk, not per wave.
constexpr int FQ_PER = 4;                       // positions per thread
constexpr int FQ_CHUNK = FQ_PER * WG;           // positions per workgroup
constexpr int FQ_T = 2 * FQ_CHUNK;              // LDS table entries (never full)

__global__ __launch_bounds__(WG) void freq_update_chunk_kernel(FreqDev f, const int64_t *__restrict__ indices, int L)
{
    __shared__ uint32_t lkey[FQ_T], lcnt[FQ_T];
    const int t = threadIdx.x;
    for (int i = t; i < FQ_T; i += WG) { lkey[i] = 0xFFFFFFFFu; lcnt[i] = 0u; }
    __syncthreads();
    const int base = blockIdx.x * FQ_CHUNK;
    uint32_t row[FQ_PER];
#pragma unroll
    for (int q = 0; q < FQ_PER; ++q) {
        const int k = base + q * WG + t;
        row[q] = k < L ? (uint32_t)indices[k] : 0xFFFFFFFFu;
    }
#pragma unroll
    for (int q = 0; q < FQ_PER; ++q) {
        if (row[q] == 0xFFFFFFFFu) continue;
        uint32_t h = cache_hash(row[q], FQ_T - 1);
        for (;;) {                                                 // ends: at most FQ_CHUNK rows in 2 FQ_CHUNK entries
            const uint32_t old = atomicCAS(&lkey[h], 0xFFFFFFFFu, row[q]);
            if (old == 0xFFFFFFFFu || old == row[q]) { atomicAdd(&lcnt[h], 1u); break; }
            h = (h + 1) & (FQ_T - 1);
        }
    }
    __syncthreads();
    for (int i = t; i < FQ_T; i += WG)
        if (lkey[i] != 0xFFFFFFFFu) freq_add(f, lkey[i], lcnt[i]);
}

// rows / counts of the occupied entries, in no particular order; *n_out = how many
__global__ __launch_bounds__(WG) void freq_export_kernel(FreqDev f, int64_t *__restrict__ rows,
                                                         int64_t *__restrict__ counts, unsigned long long *n_out)
{
    const uint32_t i = blockIdx.x * WG + threadIdx.x;
    const unsigned long long e = i <= f.mask ? f.table[i] : FREQ_EMPTY;
    const bool used = e != FREQ_EMPTY;
    const uint64_t um = __ballot(used);
    if (!um) return;
    const int lane = threadIdx.x & 63;
    unsigned long long base = 0;
    if (lane == __builtin_ctzll(um)) base = atomicAdd(n_out, (unsigned long long)__popcll(um));
    base = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(base >> 32), __builtin_ctzll(um)) << 32) |
           (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)base, __builtin_ctzll(um));
    if (used) {
        const unsigned long long pos = base + (unsigned long long)__popcll(um & lanemask_lt());
        rows[pos] = (int64_t)(e >> 32);
        counts[pos] = (int64_t)(uint32_t)e;
    }
}

__global__ void freq_zero_kernel(unsigned long long *p) { if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0ull; }

__global__ __launch_bounds__(WG) void copy_f32_kernel(const float *__restrict__ src, float *__restrict__ dst, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < n; i += (int64_t)gridDim.x * WG) dst[i] = src[i];
}

__global__ __launch_bounds__(WG) void copy_i64_kernel(const int64_t *__restrict__ src, int64_t *__restrict__ dst, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < n; i += (int64_t)gridDim.x * WG) dst[i] = src[i];
}

}  // namespace tt
