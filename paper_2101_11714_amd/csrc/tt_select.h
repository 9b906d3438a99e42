// In-workgroup selection and duplicate removal for the backward pass.
//
// The backward pass gives every core slice one owner workgroup.  The owner finds
// the lookups that touch its slice by scanning the index array (a stable
// compaction: the list keeps the order of the positions k), then sorts that list
// by row id and merges equal rows, so that each distinct row is processed once
// with the sum of its upstream gradients.  This is the grouping that the "+=" of
// Alg. 2 in the paper implies, done without atomics and in a fixed order.
#pragma once

#include "tt_common.h"

namespace tt {

// LDS scratch of one workgroup for lists of up to CH entries.
template <int CH>
struct SelectLds {
    int klist[CH];            // positions k of the matches, ascending
    uint32_t rows[CH];        // their row ids (or, for the cache role, their slots)
    int sk[CH];               // positions sorted by (row, k)
    uint32_t sr[CH];          // rows in that order
    int wcnt[NWAVE];
    int scan_tmp[NWAVE + 1];
};

// Which digit a role matches on: 0 -> i1, 1 -> i2, 2 -> i3.
__device__ __forceinline__ int role_digit(const Params &p, int role, uint32_t row)
{
    int i1, i2, i3;
    decode(p, row, i1, i2, i3);
    return role == 0 ? i1 : (role == 1 ? i2 : i3);
}

// Stable compaction of the positions k in [c0, c1) (c1 - c0 <= CH) whose key equals
// `want`.  KeyFn(k, &row) returns the key of position k (or -1 to skip it) and the
// value to remember for it.  Result in lds.klist / lds.rows; returns the count.
template <int CH, typename KeyFn>
__device__ int select_chunk(SelectLds<CH> &lds, int c0, int c1, KeyFn key_of)
{
    constexpr int SUB = CH / NWAVE;
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int lo = c0 + w * SUB;
    const int hi = min(c1, lo + SUB);
    int cnt = 0;
    for (int k0 = lo; k0 < hi; k0 += WAVE) {
        const int k = k0 + lane;
        uint32_t val = 0;
        const bool hit = (k < hi) && key_of(k, &val);
        const uint64_t mask = __ballot(hit);
        if (hit) {
            const int pos = w * SUB + cnt + __popcll(mask & lanemask_lt());
            lds.sk[pos] = k;                     // sk / sr serve as per-wave staging here
            lds.sr[pos] = val;
        }
        cnt += __popcll(mask);
    }
    if (lane == 0) lds.wcnt[w] = cnt;
    __syncthreads();
    int off[NWAVE + 1];
    off[0] = 0;
#pragma unroll
    for (int j = 0; j < NWAVE; ++j) off[j + 1] = off[j] + lds.wcnt[j];
#pragma unroll
    for (int j = 0; j < NWAVE; ++j) {
        const int c = off[j + 1] - off[j];
        for (int i = t; i < c; i += WG) {
            lds.klist[off[j] + i] = lds.sk[j * SUB + i];
            lds.rows[off[j] + i] = lds.sr[j * SUB + i];
        }
    }
    __syncthreads();
    return off[NWAVE];
}

// Sort the n selected entries by (row, k) with a rank sort.  Result in lds.sk / lds.sr.
// O(n^2 / 256) per thread: the lists of one slice are short (L / m_k on average).
template <int CH>
__device__ void sort_by_row(SelectLds<CH> &lds, int n)
{
    const int t = threadIdx.x;
    for (int i = t; i < n; i += WG) {
        const uint32_t my = lds.rows[i];
        int rank = 0;
        for (int j = 0; j < n; ++j) {
            const uint32_t r = lds.rows[j];
            rank += (r < my) || (r == my && j < i);
        }
        lds.sk[rank] = lds.klist[i];
        lds.sr[rank] = my;
    }
    __syncthreads();
}

// Sort as above, then find the runs of equal rows: ustart[0..nu] are the run boundaries
// in lds.sk / lds.sr (ustart: CH + 1 ints of LDS).  Returns nu, the number of distinct rows.
template <int CH>
__device__ int sort_dedup(SelectLds<CH> &lds, int n, int *ustart)
{
    const int t = threadIdx.x;
    sort_by_row(lds, n);
    // run heads -> ustart, via a block scan over CH / 256 consecutive entries per thread
    constexpr int PER = CH / WG;
    int heads = 0;
    uint32_t flags = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int i = t * PER + q;
        if (i < n && (i == 0 || lds.sr[i] != lds.sr[i - 1])) { flags |= 1u << q; ++heads; }
    }
    int total;
    int u = block_excl_scan(heads, lds.scan_tmp, &total);
#pragma unroll
    for (int q = 0; q < PER; ++q)
        if (flags & (1u << q)) ustart[u++] = t * PER + q;
    if (t == 0) ustart[total] = n;
    __syncthreads();
    return total;
}

}  // namespace tt
