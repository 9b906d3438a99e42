// Shared device-side definitions of the TT-EmbeddingBag kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tt {

constexpr int WG = 256;          // threads per workgroup in every kernel here
constexpr int WAVE = 64;         // CDNA wavefront width
constexpr int NWAVE = WG / WAVE;

// Shape of one table as the kernels see it (Section 2, Eq. 2 of the paper).
struct Params {
    int m1, m2, m3;
    int n1, n2, n3;
    int R1, R2;
    int N;                // n1*n2*n3
    int sA, sB, sC;       // floats per slice of core 1, 2, 3
    int cols;             // n2*R2: columns of the unfolded G2 slice (R1 x n2 R2)
    uint32_t mg3, mg2;    // ceil(2^32 / m3), ceil(2^32 / m2)
    // Set per call, not per shape: fixed bag length P = L / n_bags when every bag may have that
    // length (L divisible by n_bags), else 0; mgP = ceil(2^32 / P).  Only a guess that is checked.
    uint32_t bagP, mgP;
    // 1/m3, 0.5/m3, 1/m2, 0.5/m2 and m3, m2 as doubles, for the multiply-free decode below
    double inv3, half3, inv2, half2, m3d, m2d;
};

// floor(n / d) for n < 2^31 and 1 <= d < 2^31, with mg = ceil(2^32 / d).
// umulhi(n, mg) is floor(n/d) or one more; one compare settles it.
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t d, uint32_t mg)
{
    if (d == 1) return n;
    uint32_t q = __umulhi(n, mg);
    if (q * d > n) --q;
    return q;
}

// Row index -> digits, i = i1*m2*m3 + i2*m3 + i3 (Section 3.1).
__device__ __forceinline__ void decode(const Params &p, uint32_t row, int &i1, int &i2, int &i3)
{
    uint32_t q = fast_div(row, (uint32_t)p.m3, p.mg3);
    i3 = (int)(row - q * (uint32_t)p.m3);
    uint32_t q2 = fast_div(q, (uint32_t)p.m2, p.mg2);
    i2 = (int)(q - q2 * (uint32_t)p.m2);
    i1 = (int)q2;
}

// The same digits without integer multiplies (which run at a quarter of the fp64 FMA rate on
// CDNA): q = floor((row + 0.5) / m3) is exact in fp64 for row < 2^31 because (row + 0.5) / m3 is
// at least 0.5 / m3 away from an integer while the rounding error is below 2^-21 / m3; the
// remainders are exact integer arithmetic in fp64.
__device__ __forceinline__ void decode_f64(const Params &p, uint32_t row, int &i1, int &i2, int &i3)
{
    const double rd = (double)row;
    const double q = floor(fma(rd, p.inv3, p.half3));
    i3 = (int)fma(-q, p.m3d, rd);
    const double q2 = floor(fma(q, p.inv2, p.half2));
    i2 = (int)fma(-q2, p.m2d, q);
    i1 = (int)q2;
}

// What an owner workgroup of the backward pass tests to find its positions (Section 3.1's digit
// map, one digit at a time).  Cores 2 and 3: the digit of the row (given as a double) from the
// same multiply-free arithmetic, compared with the slice number as doubles.  Core 1: the rows
// with i1 = s are the contiguous range [s m2 m3, (s+1) m2 m3), clamped to the 31-bit row space.
__device__ __forceinline__ double select_digit_f64(const Params &p, int role, double rd)
{
    const double q = floor(fma(rd, p.inv3, p.half3));
    double d = fma(-q, p.m3d, rd);                                          // i3
    if (role == 1) {
        const double q2 = floor(fma(q, p.inv2, p.half2));
        d = fma(-q2, p.m2d, q);                                             // i2
    }
    return d;
}

struct RowRange {
    uint32_t lo, len;                                                       // rows lo <= row < lo + len
};

__device__ __forceinline__ RowRange rows_of_i1(const Params &p, int s)
{
    RowRange r{0u, 0u};
    const uint64_t m23 = (uint64_t)p.m2 * (uint64_t)p.m3;
    const uint64_t lo64 = (uint64_t)s * m23;
    if (lo64 < (1ull << 31)) {
        r.lo = (uint32_t)lo64;
        const uint64_t hi64 = lo64 + m23 < (1ull << 31) ? lo64 + m23 : (1ull << 31);
        r.len = (uint32_t)(hi64 - lo64);
    }
    return r;
}

__device__ __forceinline__ bool in_rows(const RowRange &r, uint32_t row) { return (row - r.lo) < r.len; }

// ---- cache map: open addressing, linear probing -----------------------------
// entry = (row << 32) | slot, empty = all ones.

constexpr uint64_t CACHE_EMPTY = ~0ull;

struct CacheDev {
    const float *rows;
    const uint64_t *table;
    uint32_t mask;       // capacity - 1
    int K;               // 0 = no cache
};

__device__ __forceinline__ uint32_t cache_hash(uint32_t row, uint32_t mask)
{
    uint32_t h = row * 0x9E3779B1u;
    return (h ^ (h >> 15)) & mask;
}

__device__ __forceinline__ int cache_probe(const CacheDev &c, uint32_t row)
{
    uint32_t h = cache_hash(row, c.mask);
    for (;;) {                                   // the table is never full: capacity >= 2K
        uint64_t e = c.table[h];
        if (e == CACHE_EMPTY) return -1;
        if ((uint32_t)(e >> 32) == row) return (int)(uint32_t)e;
        h = (h + 1) & c.mask;
    }
}

// ---- small wave / block helpers ----------------------------------------------

__device__ __forceinline__ uint64_t lanemask_lt()
{
    return (1ull << (threadIdx.x & 63)) - 1ull;
}

// Exclusive scan of one int per thread over the 256-thread block.
// tmp: NWAVE + 1 ints of LDS.  *total receives the block sum.
__device__ __forceinline__ int block_excl_scan(int v, int *tmp, int *total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    __syncthreads();                             // tmp may still be read from a previous call
    if (lane == 63) tmp[w] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NWAVE; ++i) {
        int x = tmp[i];
        if (i < w) base += x;
        tot += x;
    }
    *total = tot;
    return base + inc - v;
}

// Largest b with offsets[b] <= k (offsets non-decreasing, offsets[0] = 0 <= k < offsets[n_bags]).
__device__ __attribute__((noinline)) int bag_of(const int64_t *offsets, int n_bags, int k)
{
    if (!offsets) return k;
    int lo = 0, hi = n_bags;                     // answer in [lo, hi)
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (offsets[mid] <= (int64_t)k) lo = mid; else hi = mid;
    }
    return lo;
}

}  // namespace tt
