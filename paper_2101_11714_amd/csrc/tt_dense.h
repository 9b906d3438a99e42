// Uncompressed EmbeddingBag on the same GPU: the in-box comparison for the pooling-factor and
// hit-rate microbenchmarks (the role PyTorch's EmbeddingBag plays in Section 6.6 / 6.7 of the
// paper).  table is fp32 [num_rows][N], N a multiple of 4.  Not part of the TT path.
#pragma once

#include "tt_common.h"
#include "tt_sort.h"

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

// ---- the same update with duplicates merged first: sort the positions by row, add up each row's
// gradients in position order, write every distinct row once.  No floating-point atomics: the
// result is the same in every run.

constexpr int DT = 64;                          // sorted entries per tile: one wave each, one entry per lane

__global__ __launch_bounds__(WG) void dense_keys_kernel(const int64_t *__restrict__ indices, int n, uint64_t *__restrict__ keys)
{
    const int k = blockIdx.x * WG + threadIdx.x;
    if (k < n) keys[k] = (uint64_t)indices[k];
}

// Tile t holds the sorted entries [64 t, 64 t + 64).  A run of equal rows that lies inside the tile is
// applied to the table here; the part of a run that goes on in the next tile is left in part[t][1],
// the part of a run that began in an earlier tile in part[t][0] (a tile that is one run throughout: [0]).
// Lane l owns columns l + 64 c.
template <int MAXC, int NBATCH>                  // columns per lane (N <= 64 MAXC), entries in flight
__global__ __launch_bounds__(WG) void dense_seg_kernel(float *__restrict__ table, int N, const uint64_t *__restrict__ ks,
                                                       const uint32_t *__restrict__ vs, int n,
                                                       const int64_t *__restrict__ offsets, int n_bags, int bag_len,
                                                       const float *__restrict__ alpha,
                                                       const float *__restrict__ grad_out, float lr,
                                                       float *__restrict__ part)
{
    const int lane = threadIdx.x & 63;
    const int tile = blockIdx.x * NWAVE + (threadIdx.x >> 6);
    const int i0 = tile * DT;
    if (i0 >= n) return;
    const int cnt = min(DT, n - i0);
    long long my_key = -1;
    int my_bag = 0;
    float my_w = 0.f;
    if (lane < cnt) {
        my_key = (long long)ks[i0 + lane];
        const int k = (int)vs[i0 + lane];
        my_bag = -1;
        if (offsets && bag_len > 0) {                                        // bags of one length: a guess, checked
            const int g = min(k / bag_len, n_bags - 1);
            if (offsets[g] <= (int64_t)k && (int64_t)k < offsets[g + 1]) my_bag = g;
        }
        if (my_bag < 0) my_bag = bag_of(offsets, n_bags, k);
        my_w = alpha ? alpha[k] : 1.f;
    }
    const long long key_prev = i0 > 0 ? (long long)ks[i0 - 1] : -1;
    const long long key_next = i0 + cnt < n ? (long long)ks[i0 + cnt] : -1;
    float sum[MAXC];
    float tb_last[MAXC];                                                     // the table's row of the entry last added
#pragma unroll
    for (int c = 0; c < MAXC; ++c) { sum[c] = 0.f; tb_last[c] = 0.f; }
    long long cur = __builtin_amdgcn_readfirstlane((int)(my_key >> 32));
    cur = (cur << 32) | (unsigned)__builtin_amdgcn_readfirstlane((int)my_key);
    bool first = cur == key_prev;                                            // the first run began in an earlier tile
    auto flush = [&](long long key, bool goes_on) {
        float *dst = first ? part + ((size_t)tile * 2 + 0) * N : (goes_on ? part + ((size_t)tile * 2 + 1) * N : nullptr);
#pragma unroll
        for (int c = 0; c < MAXC; ++c)
            if (lane + 64 * c < N) {
                if (dst) dst[lane + 64 * c] = sum[c];
                else table[(size_t)key * N + lane + 64 * c] = tb_last[c] - lr * sum[c];
            }
        first = false;
#pragma unroll
        for (int c = 0; c < MAXC; ++c) sum[c] = 0.f;
    };
    // the gradient rows and the table rows of NBATCH entries are in flight together (no run waits for its own row of the
    // table: nothing else writes a row whose run lies inside this tile)
    for (int e0 = 0; e0 < cnt; e0 += NBATCH) {
        float g[NBATCH][MAXC], tb[NBATCH][MAXC];
#pragma unroll
        for (int q = 0; q < NBATCH; ++q) {
            const int e = min(e0 + q, cnt - 1);
            const int bag = __builtin_amdgcn_readlane(my_bag, e);
            long long key = __builtin_amdgcn_readlane((int)(my_key >> 32), e);
            key = (key << 32) | (unsigned)__builtin_amdgcn_readlane((int)my_key, e);
#pragma unroll
            for (int c = 0; c < MAXC; ++c) {
                g[q][c] = lane + 64 * c < N ? grad_out[(size_t)bag * N + lane + 64 * c] : 0.f;
                tb[q][c] = lane + 64 * c < N ? table[(size_t)key * N + lane + 64 * c] : 0.f;
            }
        }
#pragma unroll
        for (int q = 0; q < NBATCH; ++q) {
            const int e = e0 + q;
            if (e < cnt) {                                                   // uniform
                long long key = __builtin_amdgcn_readlane((int)(my_key >> 32), e);
                key = (key << 32) | (unsigned)__builtin_amdgcn_readlane((int)my_key, e);
                const float w = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_w), e));
                if (key != cur) { flush(cur, false); cur = key; }
#pragma unroll
                for (int c = 0; c < MAXC; ++c) { sum[c] = fmaf(w, g[q][c], sum[c]); tb_last[c] = tb[q][c]; }
            }
        }
    }
    // the last run: it goes on if the next tile starts with the same row.  (If it is also the run that came in
    // from an earlier tile, `first` is still set and the sum goes to part[t][0] either way: the tile where the
    // run begins adds it up.)
    if (first || cur == key_next) flush(cur, true); else flush(cur, false);
}

// A run that crosses tile borders is applied to the table by the wave of the tile where it begins: its own
// part[t][1], then part[u][0] of the later tiles that the run reaches, in tile order.  A later tile lies
// inside the run if its last entry still has the run's row (the entries are sorted); the wave looks at
// 64 tiles at a time.
__global__ __launch_bounds__(WG) void dense_fix_kernel(float *__restrict__ table, int N, const uint64_t *__restrict__ ks, int n,
                                                       float lr, const float *__restrict__ part)
{
    constexpr int MAXC = 4, NB = 8;
    const int lane = threadIdx.x & 63;
    const int tile = blockIdx.x * NWAVE + (threadIdx.x >> 6);
    const int ntiles = (n + DT - 1) / DT;
    const int i0 = tile * DT, i1 = i0 + DT;
    if (i1 >= n) return;                                                     // no tile here, or nothing to its right
    const uint64_t key = ks[i1 - 1];
    if (ks[i1] != key) return;                                               // the last run ends with the tile
    if (ks[i0] == key && i0 > 0 && ks[i0 - 1] == key) return;                // it began in an earlier tile
    // last tile that the run reaches
    int last = tile;
    for (int base = tile + 1; base < ntiles; base += WAVE) {
        const int u = base + lane;
        bool in = false;
        if (u < ntiles) in = ks[(size_t)u * DT] == key;                      // the tile's first entry is of the run
        const unsigned long long b = __ballot(in);
        const int reach = b == ~0ull ? WAVE : __builtin_ctzll(~b);           // tiles of this group the run reaches
        last = base + reach - 1;
        if (reach < WAVE) break;
    }
    // N <= 32: 64 / N groups of lanes take every (64 / N)-th later tile, NB tiles in flight each, and their sums are
    // added in group order at the end; else every lane owns columns lane + 64 c of every tile.
    const int G = N < WAVE ? WAVE / N : 1;
    const int gi = N < WAVE ? lane / N : 0, col = N < WAVE ? lane % N : lane;
    float sum[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
        sum[c] = (gi == 0 && col + 64 * c < N) ? part[((size_t)tile * 2 + 1) * N + col + 64 * c] : 0.f;
    for (int u0 = tile + 1 + gi; u0 <= last; u0 += NB * G) {
        float x[NB][MAXC];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int u = min(u0 + j * G, last);
#pragma unroll
            for (int c = 0; c < MAXC; ++c)
                x[j][c] = col + 64 * c < N ? part[((size_t)u * 2 + 0) * N + col + 64 * c] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < NB; ++j)
            if (u0 + j * G <= last) {
#pragma unroll
                for (int c = 0; c < MAXC; ++c) sum[c] += x[j][c];
            }
    }
    for (int d = N; d < WAVE; d <<= 1)                                      // (no step if N >= 64)
        sum[0] += __shfl_xor(sum[0], d);
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
        if (gi == 0 && col + 64 * c < N) table[(size_t)key * N + col + 64 * c] -= lr * sum[c];
}

struct DenseWs {
    SortWs sort;
    float *part;                                 // [tiles][2][N]
    size_t bytes;
};

static inline DenseWs dense_ws_layout(void *ws, int64_t L, int N)
{
    DenseWs d;
    d.sort = sort_ws_layout(ws, L);
    const size_t tiles = (size_t)((L + DT - 1) / DT);
    d.part = ws ? (float *)((char *)ws + d.sort.bytes) : nullptr;
    d.bytes = d.sort.bytes + align256(tiles * 2 * (size_t)N * sizeof(float)) + 256;
    return d;
}

}  // namespace tt
