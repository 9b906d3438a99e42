// Grouping pre-pass of the backward pass for long index streams.
//
// For a few thousand lookups every slice owner of the backward kernel finds its lookups by
// scanning the whole index array; that costs nothing next to a kernel launch.  For long
// streams (multi-hot bags) the scan would dominate, so the lookups are grouped once, with
// the device radix sort: every position k contributes three items keyed by the slice it
// touches in core 1, 2 and 3, or, if its row is cached (Section 4.2 of the paper), one item
// keyed by its cache slot.  After a stable sort by key the items of one key are one
// contiguous list, in the order of k: the list a scan of the positions in order would build.
//
// Keys: [0, m1) slices of G1, [m1, m1+m2) of G2, [m1+m2, nb3) of G3 (nb3 = m1+m2+m3),
// [nb3, nb3+K) cache slots, nb3+K = unused item (sorts last).  The payload of an item is
// r * L + k with r the item's number (0..2), so a list owner recovers k without a division.
//
// The gradient of the cached rows is a segmented sum over the sorted cached items: one wave
// per tile of 64 items adds up the runs of equal slots in order; runs inside a tile are
// written at once, runs that cross tile borders leave partial sums that the wave owning the
// run's first tile adds up, tile by tile.  No atomics; the order of summation is fixed.
#pragma once

#include "tt_common.h"
#include "tt_sort.h"

namespace tt {

constexpr int GT = 64;                      // sorted items per tile of the cached-row reduction

struct GroupWs {
    SortWs sort;                            // for 3 L items
    int *off, *end;                         // [nbins + 1] list bounds per key, in the sorted arrays
    int *crange;                            // [6] sorted ranges [first, one past last): [0..1] cached items, [2..3] items of the third core, [4..5] of the first
    float *part;                            // [tiles][2][N] partial sums of runs that cross tile borders
    float *rows;                            // [L][N] rows of the positions, for the forward pass that works from the lists
    int4 *tiles;                            // [L / 32 + m2 + 1] tiles of the passes that work from the lists: {slice of G2, first item, items, 0}
    int *tile_base;                         // [m2 + 1] first tile of every slice of G2
    int4 *info;                             // [3 L] per sorted item: {position k, i1, i3, bag} (unused items: k = -1)
    size_t bytes;
};

// rowsN: N if a forward pass may work from the lists of this workspace (it then leaves one row per position there), else 0
static inline GroupWs group_ws_layout(void *ws, int64_t L, int nbins, int N, int rowsN)
{
    GroupWs g;
    const int64_t n = 3 * (L > 0 ? L : 1);
    g.sort = sort_ws_layout(ws, n);
    char *p = (char *)ws;
    size_t off = g.sort.bytes;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += align256(bytes); return q; };
    g.off = (int *)take(((size_t)nbins + 1) * 4);
    g.end = (int *)take(((size_t)nbins + 1) * 4);
    g.crange = (int *)take(32);
    const int64_t tiles = (L + GT - 1) / GT + 1;
    g.part = (float *)take((size_t)tiles * 2 * N * 4);
    g.rows = (float *)take(rowsN ? (size_t)(L > 0 ? L : 1) * rowsN * 4 : 16);
    g.tiles = (int4 *)take(((size_t)L / 32 + (size_t)nbins + 1) * sizeof(int4));
    g.tile_base = (int *)take(((size_t)nbins + 2) * 4);
    g.info = (int4 *)take((size_t)n * sizeof(int4));
    g.bytes = off + 256;
    return g;
}

// items[r * L + k]: key of item r of position k (see the file comment); the cache is probed here.
// The first threads also clear the list bounds that grp_bounds_kernel fills after the sort, and the kernel
// zeroes nzero4 float4 at `zero` (the gradient of the cached rows in the fused step; may be none).
__global__ __launch_bounds__(WG) void grp_keys_kernel(Params p, const int64_t *__restrict__ indices, int L,
                                                      CacheDev cache, uint64_t *__restrict__ keys,
                                                      int *__restrict__ off, int *__restrict__ end, int nbins,
                                                      int *__restrict__ crange, float4 *__restrict__ zero, int64_t nzero4)
{
    const int k = blockIdx.x * WG + threadIdx.x;
    if (k <= nbins) { off[k] = 0; end[k] = 0; }
    if (k < 6) crange[k] = 0;
    for (int64_t i = k; i < nzero4; i += (int64_t)gridDim.x * WG) zero[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k >= L) return;
    const int nb3 = p.m1 + p.m2 + p.m3;
    const uint64_t unused = (uint64_t)(nb3 + cache.K);
    const uint32_t row = (uint32_t)indices[k];
    const int sl = cache.K ? cache_probe(cache, row) : -1;
    if (sl >= 0) {
        keys[k] = (uint64_t)(nb3 + sl);
        keys[(size_t)L + k] = unused;
        keys[2 * (size_t)L + k] = unused;
    } else {
        int i1, i2, i3;
        decode(p, row, i1, i2, i3);
        keys[k] = (uint64_t)i1;
        keys[(size_t)L + k] = (uint64_t)(p.m1 + i2);
        keys[2 * (size_t)L + k] = (uint64_t)(p.m1 + p.m2 + i3);
    }
}

// list bounds of every key that occurs, and the range of the cached items
__global__ __launch_bounds__(WG) void grp_bounds_kernel(const uint64_t *__restrict__ ks, int n, int m1, int m12, int nb3, int nbins,
                                                        int *__restrict__ off, int *__restrict__ end,
                                                        int *__restrict__ crange)
{
    const int i = blockIdx.x * WG + threadIdx.x;
    if (i >= n) return;
    const int key = (int)ks[i];
    if (key >= nbins) return;                                    // unused items
    const int prev = i > 0 ? (int)ks[i - 1] : -1;
    const int next = i + 1 < n ? (int)ks[i + 1] : nbins;
    if (prev != key) off[key] = i;
    if (next != key) end[key] = i + 1;
    if (key >= nb3) {
        if (prev < nb3) crange[0] = i;
        if (next >= nbins) crange[1] = i + 1;
    } else if (key >= m12) {
        if (prev < m12) crange[2] = i;
        if (next >= nb3) crange[3] = i + 1;
    } else if (key < m1) {
        if (next >= m1) crange[5] = i + 1;                        // (the items of the first core start the sorted arrays)
    }
}

// Tiles of the forward pass that works from the lists: the list of every slice of the second core cut into pieces
// of tp items, numbered slice after slice.  tiles[i] = {slice, first sorted item, items, 0}; entries past the last
// tile get 0 items.  Every workgroup works the numbering out for itself (m2 <= 4 x 256 slices, four per thread)
// and its threads then look their own tiles up.
__global__ __launch_bounds__(WG) void grp_tiles_kernel(int m1, int m2, int L, int tp, const int *__restrict__ off,
                                                       const int *__restrict__ end, int4 *__restrict__ tiles, int ntiles,
                                                       int *__restrict__ tile_base)
{
    __shared__ int s_tmp[NWAVE + 1];
    __shared__ int s_base[4 * WG + 1];
    const int t = threadIdx.x;
    int cnt[4], v = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int b = 4 * t + q;
        int len = b < m2 ? end[m1 + b] - off[m1 + b] : 0;
        len = len < 0 ? 0 : (len > L ? L : len);
        cnt[q] = (len + tp - 1) / tp;
        v += cnt[q];
    }
    int total;
    int base = block_excl_scan(v, s_tmp, &total);
#pragma unroll
    for (int q = 0; q < 4; ++q) { s_base[4 * t + q] = base; base += cnt[q]; }
    if (t == WG - 1) s_base[4 * WG] = total;
    __syncthreads();
    if (blockIdx.x == 0)
        for (int b = t; b <= m2; b += WG) tile_base[b] = s_base[b < 4 * WG ? b : 4 * WG];
    const int tile = blockIdx.x * WG + t;
    if (tile >= ntiles) return;
    int4 out = make_int4(0, 0, 0, 0);
    if (tile < total) {
        int lo = 0, hi = 4 * WG;                                           // last b with s_base[b] <= tile
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s_base[mid] <= tile) lo = mid; else hi = mid;
        }
        const int first = off[m1 + lo] + (tile - s_base[lo]) * tp;
        out = make_int4(lo, first, min(tp, end[m1 + lo] - first), 0);
    }
    tiles[tile] = out;
}

// bag of position k: fixed bag length if the caller found one, else a search
__device__ __forceinline__ int grp_bag(const Params &p, const int64_t *__restrict__ offsets, int n_bags, int k);

// What the kernels that work from the sorted items need of every item, in sorted order, so that they fetch it in one
// go: the position k the item belongs to (payload r L + k), the digits of its row and its bag.
__global__ __launch_bounds__(WG) void grp_info_kernel(Params p, const int64_t *__restrict__ indices, int L,
                                                      const int64_t *__restrict__ offsets, int n_bags,
                                                      const uint64_t *__restrict__ ks, const uint32_t *__restrict__ vs, int nb3,
                                                      int4 *__restrict__ info)
{
    const int i = blockIdx.x * WG + threadIdx.x;
    if (i >= 3 * L) return;
    int4 out = make_int4(-1, 0, 0, 0);
    if ((int)ks[i] < nb3) {                                      // an item of one of the cores
        uint32_t v = vs[i];
        const int k = (int)(v >= 2u * (uint32_t)L ? v - 2u * (uint32_t)L : (v >= (uint32_t)L ? v - (uint32_t)L : v));
        if (k < L) {
            int i1, i2, i3;
            decode(p, (uint32_t)indices[k], i1, i2, i3);
            out = make_int4(k, i1, i3, grp_bag(p, offsets, n_bags, k));
        }
    }
    info[i] = out;
}


__device__ __forceinline__ int grp_bag(const Params &p, const int64_t *__restrict__ offsets, int n_bags, int k)
{
    if (!offsets) return k;
    if (p.bagP) {
        int g = (int)fast_div((uint32_t)k, p.bagP, p.mgP);
        g = g < n_bags ? g : n_bags - 1;
        if (offsets[g] <= (int64_t)k && (int64_t)k < offsets[g + 1]) return g;
    }
    return bag_of(offsets, n_bags, k);
}

// One wave per tile of GT = 64 sorted cached items.  Lane e first fetches key, position, weight
// and bag of item e (one round trip for the whole tile); then the rows of the upstream gradient
// are read 16 items at a time, lane j owning columns j, j + 64, ..., and added run by run.
// (`block` is the workgroup's number among those that do this work: the body also runs as extra workgroups
// of the backward kernel of the (4,4,4) shapes, next to the slice owners.)
template <int MAXC>                                               // columns per lane: N <= 64 MAXC
__device__ __forceinline__ void grp_cache_tile_body(const Params &p, int block, const uint64_t *__restrict__ ks,
                                                    const uint32_t *__restrict__ vs, const int *__restrict__ crange,
                                                    const int64_t *__restrict__ offsets, int n_bags,
                                                    const float *__restrict__ alpha, const float *__restrict__ grad_out,
                                                    float *__restrict__ grad_cache, float *__restrict__ part, bool fresh)
{
    static_assert(GT == WAVE, "one item per lane");
    const int N = p.N, nb3 = p.m1 + p.m2 + p.m3;
    const int lane = threadIdx.x & 63;
    const int tile = block * NWAVE + (threadIdx.x >> 6);
    const int cb = crange[0], ce = crange[1];
    const int i0 = cb + tile * GT;
    if (i0 >= ce) return;
    const int i1 = min(ce, i0 + GT);
    const int cnt = i1 - i0;
    const int key_prev = i0 > cb ? (int)ks[i0 - 1] : -1;
    const int key_next = i1 < ce ? (int)ks[i1] : -1;
    // item of this lane
    const int ie = min(i0 + lane, i1 - 1);
    const int my_key = (int)ks[ie];
    const int my_k = (int)vs[ie];                                 // cached items are item 0: payload = k
    const float my_w = alpha ? alpha[my_k] : 1.f;
    const int my_bag = grp_bag(p, offsets, n_bags, my_k);

    float sum[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) sum[c] = 0.f;
    int cur = __builtin_amdgcn_readfirstlane(my_key);
    bool first = true;
    auto flush = [&](int key, bool run_ends_here) {
        // a run that began in an earlier tile, or continues into the next one, leaves a partial sum
        const bool from_left = first && key == key_prev;
        const bool to_right = !run_ends_here;
        if (from_left || to_right) {
            float *dst = part + ((size_t)tile * 2 + (from_left ? 0 : 1)) * N;
#pragma unroll
            for (int c = 0; c < MAXC; ++c)
                if (lane + 64 * c < N) dst[lane + 64 * c] = sum[c];
        } else {
            // a run inside the tile is all there is for its slot: where the caller has just cleared the gradient
            // (`fresh`) it is stored, not added, and the waves do not wait for a load per run
            float *dst = grad_cache + (size_t)(key - nb3) * N;
            if (fresh) {
#pragma unroll
                for (int c = 0; c < MAXC; ++c)
                    if (lane + 64 * c < N) dst[lane + 64 * c] = sum[c];
            } else {
#pragma unroll
                for (int c = 0; c < MAXC; ++c)
                    if (lane + 64 * c < N) dst[lane + 64 * c] += sum[c];
            }
        }
        first = false;
#pragma unroll
        for (int c = 0; c < MAXC; ++c) sum[c] = 0.f;
    };
    for (int e0 = 0; e0 < cnt; e0 += 16) {
        float g[16][MAXC];
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int e = min(e0 + q, cnt - 1);
            const int bag = __builtin_amdgcn_readlane(my_bag, e);
#pragma unroll
            for (int c = 0; c < MAXC; ++c)
                g[q][c] = lane + 64 * c < N ? grad_out[(size_t)bag * N + lane + 64 * c] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int e = e0 + q;
            if (e < cnt) {                                         // uniform
                const int key = __builtin_amdgcn_readlane(my_key, e);
                const float w = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_w), e));
                if (key != cur) { flush(cur, true); cur = key; }
#pragma unroll
                for (int c = 0; c < MAXC; ++c) sum[c] = fmaf(w, g[q][c], sum[c]);
            }
        }
    }
    flush(cur, cur != key_next);
}

__global__ __launch_bounds__(WG) void grp_cache_tile_kernel(Params p, const uint64_t *__restrict__ ks,
                                                            const uint32_t *__restrict__ vs,
                                                            const int *__restrict__ crange,
                                                            const int64_t *__restrict__ offsets, int n_bags,
                                                            const float *__restrict__ alpha,
                                                            const float *__restrict__ grad_out,
                                                            float *__restrict__ grad_cache, float *__restrict__ part, bool fresh)
{
    grp_cache_tile_body<4>(p, blockIdx.x, ks, vs, crange, offsets, n_bags, alpha, grad_out, grad_cache, part, fresh);   // N <= 256
}

// A run that crosses tile borders is finished where it begins.  Wave w of a workgroup looks at tile
// 4 block + w; if a run begins there and goes on, its last item is known from the list bounds, so the
// partial sums of its later tiles can be loaded independently.  A run over a few tiles (nearly all of them)
// is finished by the wave alone, the four waves working side by side; a long one (the hottest slots) by the
// whole workgroup: wave w adds every fourth partial sum, NB in flight, and the four results are added in
// wave order.
template <int MAXC>
__device__ __forceinline__ void grp_cache_fix_body(const Params &p, int block, const uint64_t *__restrict__ ks,
                                                   const int *__restrict__ crange, const int *__restrict__ gend,
                                                   const float *__restrict__ part, float *__restrict__ grad_cache)
{
    constexpr int NB = 64 / MAXC;                                  // partial sums in flight per wave (long runs)
    constexpr int SHORT = 16;                                      // later tiles a wave handles alone
    __shared__ float red[NWAVE][MAXC * WAVE];
    __shared__ int info[NWAVE][2];                                 // long run that begins in the wave's tile: key, last tile
    const int N = p.N, nb3 = p.m1 + p.m2 + p.m3;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int cb = crange[0], ce = crange[1];
    {
        const int tile = block * NWAVE + w;
        const int i0 = cb + tile * GT, i1 = min(ce, i0 + GT);
        int key = -1, last_tile = 0;
        bool own = false;
        if (i0 < ce && i1 < ce) {                                  // else no tile here, or nothing to its right
            // the four keys that decide are loaded together (one round trip, not one per condition)
            const int kl = (int)ks[i1 - 1], kn = (int)ks[i1], kf = (int)ks[i0], kb = (int)ks[max(i0 - 1, cb)];
            key = kl;
            own = kn == key;                                       // the last run goes on in the next tile
            if (own && kf == key && i0 > cb && kb == key) own = false;                         // it begins elsewhere
            if (own) last_tile = (gend[key] - 1 - cb) / GT;        // tile that holds the run's last item
        }
        const bool is_long = own && last_tile - tile > SHORT;
        if (lane == 0) { info[w][0] = is_long ? key : -1; info[w][1] = last_tile; }
        if (own && !is_long) {                                     // uniform in the wave
            float x[SHORT + 1][MAXC];
#pragma unroll
            for (int j = 0; j <= SHORT; ++j) {
                const int u = min(tile + j, last_tile);
#pragma unroll
                for (int c = 0; c < MAXC; ++c)
                    x[j][c] = lane + 64 * c < N ? part[((size_t)u * 2 + (j == 0 ? 1 : 0)) * N + lane + 64 * c] : 0.f;
            }
            float *dst = grad_cache + (size_t)(key - nb3) * N;
#pragma unroll
            for (int c = 0; c < MAXC; ++c) {
                float sum = x[0][c];
#pragma unroll
                for (int j = 1; j <= SHORT; ++j)
                    if (tile + j <= last_tile) sum += x[j][c];
                if (lane + 64 * c < N) dst[lane + 64 * c] += sum;
            }
        }
    }
    __syncthreads();
    for (int q = 0; q < NWAVE; ++q) {                              // long runs: uniform in the workgroup
        const int key = info[q][0];
        if (key < 0) continue;
        const int tile = block * NWAVE + q, last_tile = info[q][1];
        float sum[MAXC];
#pragma unroll
        for (int c = 0; c < MAXC; ++c)
            sum[c] = (w == 0 && lane + 64 * c < N) ? part[((size_t)tile * 2 + 1) * N + lane + 64 * c] : 0.f;
        for (int u0 = tile + 1 + w; u0 <= last_tile; u0 += NB * NWAVE) {
            float x[NB][MAXC];
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int u = min(u0 + j * NWAVE, last_tile);
#pragma unroll
                for (int c = 0; c < MAXC; ++c)
                    x[j][c] = lane + 64 * c < N ? part[((size_t)u * 2 + 0) * N + lane + 64 * c] : 0.f;
            }
#pragma unroll
            for (int j = 0; j < NB; ++j)
                if (u0 + j * NWAVE <= last_tile) {
#pragma unroll
                    for (int c = 0; c < MAXC; ++c) sum[c] += x[j][c];
                }
        }
#pragma unroll
        for (int c = 0; c < MAXC; ++c) red[w][lane + 64 * c] = sum[c];
        __syncthreads();
        if (w == 0) {
            float *dst = grad_cache + (size_t)(key - nb3) * N;
#pragma unroll
            for (int c = 0; c < MAXC; ++c)
                if (lane + 64 * c < N) {
                    float tot = red[0][lane + 64 * c];
#pragma unroll
                    for (int j = 1; j < NWAVE; ++j) tot += red[j][lane + 64 * c];
                    dst[lane + 64 * c] += tot;
                }
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(WG) void grp_cache_fix_kernel(Params p, const uint64_t *__restrict__ ks,
                                                           const int *__restrict__ crange,
                                                           const int *__restrict__ gend,
                                                           const float *__restrict__ part,
                                                           float *__restrict__ grad_cache)
{
    grp_cache_fix_body<4>(p, blockIdx.x, ks, crange, gend, part, grad_cache);                                     // N <= 256
}

// The cached-row work of one backward call, for a kernel that runs it as extra workgroups: `blocks`
// workgroups of grp_cache_tile_body, then (in a later launch) as many of grp_cache_fix_body.
struct GrpCacheWork {
    const uint64_t *ks;
    const uint32_t *vs;
    const int *crange, *gend;
    float *part, *grad_cache;
    int blocks;                                  // 0: nothing to do
    bool fresh;                                  // grad_cache was cleared for this call (else the sums are added to it)
};

}  // namespace tt
