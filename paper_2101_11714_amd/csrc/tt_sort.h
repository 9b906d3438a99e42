// Device-wide stable LSD radix sort (64-bit keys, 32-bit payload) and run-length
// "unique" on the sorted keys.  Used by the cache population (top-K selection,
// Section 4.2 of the paper) and by the canonical dedup export.  Integer only.
#pragma once

#include "tt_common.h"

namespace tt {

constexpr int RS_TILE = 2048;                   // keys per workgroup and pass
constexpr int RS_SUB = RS_TILE / WG;            // 8 rounds of 256 keys
constexpr int SCAN_WG = 1024;

static inline int rs_blocks(int64_t n) { return (int)((n + RS_TILE - 1) / RS_TILE); }

// hist[bin * nblk + blk] = number of keys of tile blk whose digit is bin (BYBLK: hist[blk * nbins + bin], the
// layout the scatter kernel reads when it does the scan itself).
// A pass sorts by `db` <= 8 bits of the key, taken at `shift` (1 << db bins).
template <bool BYBLK>
__global__ __launch_bounds__(WG) void rs_hist_kernel(const uint64_t *__restrict__ keys, int n, int shift, int db,
                                                     uint32_t *__restrict__ hist, int nblk)
{
    __shared__ uint32_t h[256];
    const int t = threadIdx.x;
    const uint32_t mask = (1u << db) - 1u;
    h[t] = 0;
    __syncthreads();
    const int base = blockIdx.x * RS_TILE;
    uint64_t k[RS_SUB];                                             // all loads first (clamped: none is conditional)
#pragma unroll
    for (int s = 0; s < RS_SUB; ++s) k[s] = keys[min(base + s * WG + t, n - 1)];
#pragma unroll
    for (int s = 0; s < RS_SUB; ++s)
        if (base + s * WG + t < n) atomicAdd(&h[(uint32_t)(k[s] >> shift) & mask], 1u);
    __syncthreads();
    if (t <= (int)mask) hist[BYBLK ? blockIdx.x * (int)(mask + 1u) + t : t * nblk + blockIdx.x] = h[t];
}

// In-place exclusive scan of data[0..total); data[total] receives the sum.  One workgroup.
// A step covers SCAN_SUB sub-blocks of 4096 values; a thread loads one uint4 of each (coalesced,
// all loads of the step in flight together) and the sub-blocks are scanned one after the other.
// `data` must be 16-byte aligned; it is padded to a multiple of 4 values (see sort_ws_layout).
constexpr int SCAN_SUB = 4;

__global__ __launch_bounds__(SCAN_WG) void scan_kernel(uint32_t *__restrict__ data, int total)
{
    __shared__ uint32_t wsum[SCAN_WG / WAVE];
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    uint32_t carry = 0;                                            // same value in every thread
    for (int base = 0; base < total; base += SCAN_SUB * SCAN_WG * 4) {
        uint4 v[SCAN_SUB];
#pragma unroll
        for (int q = 0; q < SCAN_SUB; ++q) {
            const int i = base + q * SCAN_WG * 4 + t * 4;
            v[q] = make_uint4(0u, 0u, 0u, 0u);
            if (i + 3 < total) {
                v[q] = *reinterpret_cast<const uint4 *>(data + i);
            } else if (i < total) {
                v[q].x = data[i];
                if (i + 1 < total) v[q].y = data[i + 1];
                if (i + 2 < total) v[q].z = data[i + 2];
            }
        }
#pragma unroll
        for (int q = 0; q < SCAN_SUB; ++q) {
            const int i = base + q * SCAN_WG * 4 + t * 4;
            const uint32_t mine = v[q].x + v[q].y + v[q].z + v[q].w;
            uint32_t inc = mine;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                uint32_t o = __shfl_up(inc, d);
                if (lane >= d) inc += o;
            }
            __syncthreads();                                       // wsum of the previous sub-block has been read
            if (lane == 63) wsum[w] = inc;
            __syncthreads();
            uint32_t pre = carry, all = 0;
#pragma unroll
            for (int j = 0; j < SCAN_WG / WAVE; ++j) {
                const uint32_t x = wsum[j];
                if (j < w) pre += x;
                all += x;
            }
            carry += all;
            uint4 o;
            o.x = pre + inc - mine;
            o.y = o.x + v[q].x;
            o.z = o.y + v[q].y;
            o.w = o.z + v[q].z;
            if (i + 3 < total) {
                *reinterpret_cast<uint4 *>(data + i) = o;
            } else if (i < total) {
                data[i] = o.x;
                if (i + 1 < total) data[i + 1] = o.y;
                if (i + 2 < total) data[i + 2] = o.z;
            }
        }
    }
    if (t == 0) data[total] = carry;
}

// Stable scatter of one pass.  vin == nullptr means payload = position.
// The tile is 8 rounds of 256 keys; a wave ranks its 64 keys of a round among themselves with ballots, all rounds
// first, then thread t (= bin t) turns the 32 (round, wave) counts of its bin into starting positions, and every key
// goes to start + rank, through LDS, where the tile is put in order first: a digit's keys of one tile are neighbours in
// the output, and scattered 8-byte stores of single lanes cost several times the stores of whole runs.
// OWNSCAN: `hist` holds the raw counts by tile (rs_hist_kernel<true>) and every workgroup derives its own starting
// positions from them: the keys with smaller digits anywhere plus the keys with the same digit in earlier tiles.  That is
// nblk * nbins / 1024 16-byte loads per thread, all independent, instead of a scan kernel of one workgroup between the
// two launches; the host takes this form for up to RS_OWNSCAN_MAX tiles.
constexpr int RS_OWNSCAN_MAX = 512;

template <bool OWNSCAN>
__global__ __launch_bounds__(WG) void rs_scatter_kernel(const uint64_t *__restrict__ kin, const uint32_t *__restrict__ vin,
                                                        uint64_t *__restrict__ kout, uint32_t *__restrict__ vout,
                                                        int n, int shift, int db, const uint32_t *__restrict__ hist, int nblk)
{
    __shared__ __align__(16) uint32_t cnt[RS_SUB * NWAVE * 256];    // [round][wave][bin]; first the partial sums below
    __shared__ uint64_t sk[RS_TILE];                                // the tile in output order
    __shared__ uint32_t sv[RS_TILE];
    __shared__ uint32_t gofs[256];
    __shared__ uint32_t wtot[NWAVE], wtot2[NWAVE];
    const int t = threadIdx.x, w = t >> 6;
    const uint32_t mask = (1u << db) - 1u;
    const int tile = blockIdx.x * RS_TILE;
    // the keys and payloads of all rounds are loaded before anything else
    uint64_t keys[RS_SUB];
    uint32_t vals[RS_SUB];
#pragma unroll
    for (int s = 0; s < RS_SUB; ++s) {
        const int i = tile + s * WG + t;
        keys[s] = i < n ? kin[i] : 0ull;
        vals[s] = i < n && vin ? vin[i] : (uint32_t)i;
    }
    uint32_t start;                                                 // of bin t in the output
    if constexpr (OWNSCAN) {
        // thread t sums 4 neighbouring bins (one 16-byte load per tile) over every (256 / q4)-th tile; all loads are
        // independent and the counts were written by workgroups anywhere on the chip, so they are issued together
        const int nbins = (int)mask + 1;
        uint32_t *ptot = cnt, *ppre = cnt + 4 * WG;                 // [row group][bin]: totals, earlier tiles
        uint32_t tot = 0, pre = 0;
        if (nbins >= 4) {
            const int q4 = nbins >> 2, c = t & (q4 - 1), rg = t / q4, nrg = WG / q4;
            const uint4 *h4 = reinterpret_cast<const uint4 *>(hist);
            uint4 t4 = make_uint4(0u, 0u, 0u, 0u), p4 = t4;
            for (int b0 = rg; b0 < nblk; b0 += 16 * nrg) {         // 16 loads in flight (clamped, so none is conditional)
                uint4 v[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) v[q] = h4[min(b0 + q * nrg, nblk - 1) * q4 + c];
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int b = b0 + q * nrg;
                    const uint32_t in = b < nblk ? 0xffffffffu : 0u;
                    const uint32_t m = b < (int)blockIdx.x ? 0xffffffffu : 0u;      // blockIdx.x < nblk
                    t4.x += v[q].x & in; t4.y += v[q].y & in; t4.z += v[q].z & in; t4.w += v[q].w & in;
                    p4.x += v[q].x & m; p4.y += v[q].y & m; p4.z += v[q].z & m; p4.w += v[q].w & m;
                }
            }
            *reinterpret_cast<uint4 *>(&ptot[rg * nbins + 4 * c]) = t4;
            *reinterpret_cast<uint4 *>(&ppre[rg * nbins + 4 * c]) = p4;
            __syncthreads();
            if (t < nbins)
                for (int q = 0; q < nrg; ++q) { tot += ptot[q * nbins + t]; pre += ppre[q * nbins + t]; }
        } else {
            if (t < nbins)
                for (int b = 0; b < nblk; ++b) {
                    const uint32_t v = hist[b * nbins + t];
                    tot += v;
                    pre += b < (int)blockIdx.x ? v : 0u;
                }
        }
        // exclusive scan of the totals over the bins (thread t = bin t)
        const int lane = t & 63;
        uint32_t inc = tot;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(inc, d);
            if (lane >= d) inc += o;
        }
        if (lane == 63) wtot[w] = inc;
        __syncthreads();                                            // also: ptot / ppre have been read
        uint32_t before = inc - tot;
        for (int j = 0; j < w; ++j) before += wtot[j];
        start = before + pre;
    } else {
        start = t <= (int)mask ? hist[t * nblk + blockIdx.x] : 0u;
    }
    {   // clear the counts: 8192 values, 8 stores of 16 bytes per thread
        uint4 *c4 = reinterpret_cast<uint4 *>(cnt);
#pragma unroll
        for (int q = 0; q < RS_SUB * NWAVE * 256 / 4 / WG; ++q) c4[q * WG + t] = make_uint4(0u, 0u, 0u, 0u);
    }
    __syncthreads();
    int rank[RS_SUB];
    {   // lanes of this wave that hold the same digit, one bit at a time, the rounds side by side (independent chains)
        uint64_t same[RS_SUB];
#pragma unroll
        for (int s = 0; s < RS_SUB; ++s) same[s] = __ballot(tile + s * WG + t < n);
        for (int b = 0; b < db; ++b) {                              // uniform
#pragma unroll
            for (int s = 0; s < RS_SUB; ++s) {
                const bool bit = (keys[s] >> (shift + b)) & 1ull;
                const uint64_t bal = __ballot(bit);
                same[s] &= bit ? bal : ~bal;
            }
        }
#pragma unroll
        for (int s = 0; s < RS_SUB; ++s) {
            const uint32_t dg = (uint32_t)(keys[s] >> shift) & mask;
            rank[s] = __popcll(same[s] & lanemask_lt());
            if (tile + s * WG + t < n && rank[s] == 0) cnt[(s * NWAVE + w) * 256 + dg] = (uint32_t)__popcll(same[s]);
        }
    }
    __syncthreads();
    {   // thread t owns bin t: the counts per round and wave become positions within the tile sorted by digit
        uint32_t c[RS_SUB * NWAVE];
        uint32_t total = 0;
#pragma unroll
        for (int q = 0; q < RS_SUB * NWAVE; ++q) { c[q] = cnt[q * 256 + t]; total += c[q]; }
        const int lane = t & 63;
        uint32_t inc = total;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(inc, d);
            if (lane >= d) inc += o;
        }
        if (lane == 63) wtot2[w] = inc;
        __syncthreads();
        uint32_t r = inc - total;                                   // keys of the tile with a smaller digit
        for (int j = 0; j < w; ++j) r += wtot2[j];
        gofs[t] = start - r;                                        // output position minus position in the tile
#pragma unroll
        for (int q = 0; q < RS_SUB * NWAVE; ++q) {
            cnt[q * 256 + t] = r;
            r += c[q];
        }
    }
    __syncthreads();
    // the tile is put in order in LDS first, so that neighbouring lanes store to neighbouring addresses
#pragma unroll
    for (int s = 0; s < RS_SUB; ++s) {
        if (tile + s * WG + t < n) {
            const uint32_t dg = (uint32_t)(keys[s] >> shift) & mask;
            const uint32_t lp = cnt[(s * NWAVE + w) * 256 + dg] + (uint32_t)rank[s];
            sk[lp] = keys[s];
            sv[lp] = vals[s];
        }
    }
    __syncthreads();
    const int nv = min(RS_TILE, n - tile);
#pragma unroll
    for (int s = 0; s < RS_SUB; ++s) {
        const int lp = s * WG + t;
        if (lp < nv) {
            const uint64_t key = sk[lp];
            const uint32_t dst = (uint32_t)lp + gofs[(uint32_t)(key >> shift) & mask];
            kout[dst] = key;
            vout[dst] = sv[lp];
        }
    }
}

// ---- unique on sorted keys ------------------------------------------------------
// Keys equal to `sentinel` (sorted last) are not counted.

__global__ __launch_bounds__(WG) void uq_count_kernel(const uint64_t *__restrict__ keys, int n, uint64_t sentinel,
                                                      uint32_t *__restrict__ blkcnt)
{
    __shared__ int tmp[NWAVE + 1];
    const int t = threadIdx.x;
    const int tile = blockIdx.x * RS_TILE;
    int c = 0;
#pragma unroll
    for (int s = 0; s < RS_SUB; ++s) {
        int i = tile + s * WG + t;
        if (i < n) {
            uint64_t k = keys[i];
            if (k != sentinel && (i == 0 || keys[i - 1] != k)) ++c;
        }
    }
    int total;
    (void)block_excl_scan(c, tmp, &total);
    if (t == 0) blkcnt[blockIdx.x] = (uint32_t)total;
}

// head_pos[u] = position of the first occurrence of the u-th distinct key; uniq[u] = that key.
// n_out[0] = number of distinct keys, n_out[1] = number of non-sentinel keys.
__global__ __launch_bounds__(WG) void uq_write_kernel(const uint64_t *__restrict__ keys, int n, uint64_t sentinel,
                                                      const uint32_t *__restrict__ blkoff, int nblk,
                                                      uint32_t *__restrict__ head_pos, int64_t *__restrict__ uniq,
                                                      int64_t *__restrict__ n_out)
{
    __shared__ int tmp[NWAVE + 1];
    const int t = threadIdx.x;
    const int tile = blockIdx.x * RS_TILE;
    int running = (int)blkoff[blockIdx.x];
    for (int s = 0; s < RS_SUB; ++s) {
        const int i = tile + s * WG + t;
        uint64_t k = 0;
        bool head = false;
        if (i < n) {
            k = keys[i];
            const bool first = (i == 0) || keys[i - 1] != k;
            head = first && k != sentinel;
            if (first && k == sentinel) n_out[1] = i;          // first skipped key: only one thread can see it
        }
        int total;
        const int ex = block_excl_scan(head ? 1 : 0, tmp, &total);
        if (head) {
            head_pos[running + ex] = (uint32_t)i;
            uniq[running + ex] = (int64_t)k;
        }
        running += total;
    }
    if (blockIdx.x == 0 && t == 0) n_out[0] = (int64_t)blkoff[nblk];
}

__global__ void uq_init_kernel(int64_t *n_out, int64_t n)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) { n_out[0] = 0; n_out[1] = n; }
}

__global__ __launch_bounds__(WG) void uq_counts_kernel(const uint32_t *__restrict__ head_pos,
                                                       const int64_t *__restrict__ n_out,
                                                       int32_t *__restrict__ count, int n)
{
    const int64_t nu = n_out[0], kept = n_out[1];
    const int64_t u = (int64_t)blockIdx.x * WG + threadIdx.x;
    if (u < nu && u < n) {
        const uint32_t next = (u + 1 < nu) ? head_pos[u + 1] : (uint32_t)kept;
        count[u] = (int32_t)(next - head_pos[u]);
    }
}

// Workspace of a sort of n keys: two key buffers, two payload buffers, histogram.
struct SortWs {
    uint64_t *k0, *k1;
    uint32_t *v0, *v1;
    uint32_t *hist;          // 256*nblk + 1
    uint32_t *head_pos;      // n + 1
    uint32_t *blk;           // nblk + 1
    size_t bytes;
};

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static inline SortWs sort_ws_layout(void *ws, int64_t n)
{
    SortWs s;
    const int nblk = rs_blocks(n > 0 ? n : 1);
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += align256(bytes); return q; };
    s.k0 = (uint64_t *)take((size_t)n * 8);
    s.k1 = (uint64_t *)take((size_t)n * 8);
    s.v0 = (uint32_t *)take((size_t)n * 4);
    s.v1 = (uint32_t *)take((size_t)n * 4);
    s.hist = (uint32_t *)take(((size_t)256 * nblk + 1) * 4);
    s.head_pos = (uint32_t *)take(((size_t)n + 1) * 4);
    s.blk = (uint32_t *)take(((size_t)nblk + 1) * 4);
    s.bytes = off + 256;
    return s;
}

// The buffers that hold the result of radix_sort(s, n, bits, ...): they depend on the number of passes only.
static inline void radix_sort_result(const SortWs &s, int bits, uint64_t **kres, uint32_t **vres)
{
    const int npass = (bits + 7) / 8;
    const int db = (bits + npass - 1) / npass;
    const int count = (bits + db - 1) / db;                // passes that run
    *kres = count % 2 ? s.k1 : s.k0;
    *vres = count == 0 ? nullptr : (count % 2 ? s.v0 : s.v1);
}

// Sort keys in s.k0 (payload = original position) by their low `bits` bits.
// Returns the buffers that hold the result in *kres / *vres.
static inline hipError_t radix_sort(const SortWs &s, int n, int bits, hipStream_t st,
                                    uint64_t **kres, uint32_t **vres)
{
    uint64_t *kin = s.k0, *kout = s.k1;
    uint32_t *vin = nullptr, *vout = s.v0;
    const int nblk = rs_blocks(n);
    bool first = true;
    // as few passes as 8-bit digits allow, the bits spread evenly over them (a narrow digit means a short scan)
    const int npass = (bits + 7) / 8;
    const int db = (bits + npass - 1) / npass;
    for (int shift = 0; shift < bits; shift += db) {
        if (nblk <= RS_OWNSCAN_MAX) {
            hipLaunchKernelGGL(rs_hist_kernel<true>, dim3(nblk), dim3(WG), 0, st, kin, n, shift, db, s.hist, nblk);
            hipLaunchKernelGGL(rs_scatter_kernel<true>, dim3(nblk), dim3(WG), 0, st, kin, vin, kout, vout, n, shift, db,
                               s.hist, nblk);
        } else {
            hipLaunchKernelGGL(rs_hist_kernel<false>, dim3(nblk), dim3(WG), 0, st, kin, n, shift, db, s.hist, nblk);
            hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(SCAN_WG), 0, st, s.hist, (1 << db) * nblk);
            hipLaunchKernelGGL(rs_scatter_kernel<false>, dim3(nblk), dim3(WG), 0, st, kin, vin, kout, vout, n, shift, db,
                               s.hist, nblk);
        }
        uint64_t *tk = kin; kin = kout; kout = tk;
        if (first) { vin = s.v0; vout = s.v1; first = false; }
        else { uint32_t *tv = vin; vin = vout; vout = tv; }
    }
    *kres = kin;
    *vres = vin;          // nullptr only if bits == 0 (never asked for)
    return hipGetLastError();
}

}  // namespace tt
