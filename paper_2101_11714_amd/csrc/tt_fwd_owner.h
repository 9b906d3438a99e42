// Forward pass for long index streams: the workgroups own slices of the second core.
//
// With a wave per bag every lookup streams its whole slice G2[i2] (R x n2 R values) from the
// L2, and for hundreds of thousands of lookups that traffic is the limit.  Here the positions
// are taken from the per-slice lists of the grouping pre-pass (tt_group.h): a workgroup takes
// up to TP positions of one slice and one value of j2, stages that R x R part of G2[i2] in
// LDS once, stacks the positions' rows of G1 into a 128 x R matrix and computes the 128 x R
// block of T0 = A Bm (Eq. 3, first product) on the matrix cores (fp32 MFMA 32x32x2).  The
// block goes through LDS to the kept copy of T0 (if asked for) and to the second product
// T0 C; the weighted row of every position is written to rows[k][N].  A second kernel pools
// the rows of each bag in position order (cached rows come from the cache there), so the
// result does not depend on which workgroup computed which position.
#pragma once

#include "tt_common.h"
#include "tt_fast.h"
#include "tt_fast_bwd.h"

namespace tt {

constexpr int FO_GRID_TILES = 8192;               // tiles started per launch (measured: a tile per workgroup beats fewer, looping ones)
constexpr int FO_MAX_M2 = 4 * WG;                 // four slices per thread when the tiles are numbered

template <typename C>
struct FoCfg {
    static constexpr int ROWS = 128;                          // rows of T0 per tile: 32 per wave
    static constexpr int TP = ROWS / C::N1;                   // positions per tile
    static constexpr int CB = C::R / 32;                      // 32-column blocks of the tile's part of T0 (one j2: R columns)
    static constexpr int KH = C::R / 2;                       // k values per half of the wave
    static constexpr int LDT = C::R + 2;                      // row stride of the T0 block in LDS (the reads of step 8 then spread over the banks)
    static constexpr int LDS_FLOATS = C::R * C::R > ROWS * LDT ? C::R * C::R : ROWS * LDT;
    static constexpr int NBQ = WG / TP;                       // threads per position in the second product: a part of b each
    static constexpr bool EARLY_C = C::R / NBQ <= 8;          // fetch the third core's rows before the first product (if they fit the registers)
    static constexpr int BQ = C::R / NBQ;                     // values of b per thread: b = NBQ i + bq
    static_assert(C::R % 32 == 0 && ROWS % C::N1 == 0 && WG % TP == 0 && NBQ <= 8, "tile layout");
};

template <typename C>
static inline size_t fo_lds_bytes() { return (size_t)FoCfg<C>::LDS_FLOATS * sizeof(float); }

// Workgroup n2 * tile + j2 computes, for the tile's positions, the columns (j2, .) of T0 and the outputs (., j2, .).
// vs / tiles: the sorted payloads (r L + k) and the tile table of the grouping pre-pass; info: the records (position,
// first digit, third digit, bag) of the sorted items if the pre-pass wrote them (it does for the backward on tiles),
// else null: then the positions' rows are read and decoded here, one dependent round trip more.
template <typename C>
__global__ __launch_bounds__(WG) void fwd_owner_kernel(Params p, const float *__restrict__ G1, const float *__restrict__ G2,
                                                       const float *__restrict__ G3, const int64_t *__restrict__ indices,
                                                       int L, const float *__restrict__ alpha,
                                                       const uint32_t *__restrict__ vs, const int4 *__restrict__ info,
                                                       const int4 *__restrict__ tiles, int ntiles,
                                                       float *__restrict__ rows_out, float *__restrict__ t0_out)
{
    using F = FoCfg<C>;
    constexpr int N1 = C::N1, N2 = C::N2, R = C::R, COLS = C::COLS, TP = F::TP, LDT = F::LDT;
    extern __shared__ __align__(16) float fo_lds[];
    __shared__ int s_k[TP];
    __shared__ float s_w[TP];
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;

    // 1. the tiles of this workgroup: every (gridDim.x / n2)-th one, until the table runs out of tiles with items
    const int j2 = blockIdx.x % N2;
    for (int tile = blockIdx.x / N2; tile < ntiles; tile += gridDim.x / N2) {
    const int4 td = tiles[tile];
    const int i2 = td.x, lo = td.y;
    const int n = td.z;
    if (n <= 0) return;                                                    // uniform: the tiles in use come first
    if ((unsigned)i2 >= (unsigned)p.m2 || lo < 0 || n > TP || lo + n > 3 * L) return;   // (no pre-pass wrote this)

    // 2. this part of the slice to LDS, [R][R]: the loads first, so that the positions are fetched behind them
    constexpr int NB4 = R * R / 4 / WG;                                    // float4 per thread
    float4 bm[NB4];
    {
        const float *src = G2 + (size_t)i2 * C::sB + j2 * R;
#pragma unroll
        for (int q = 0; q < NB4; ++q) {
            const int i = q * WG + t, a = i / (R / 4), c4 = i % (R / 4);
            bm[q] = *reinterpret_cast<const float4 *>(src + a * COLS + 4 * c4);
        }
    }
    // 3. positions: lane (ln, kh) of wave w supplies row 32 w + ln of the stacked first-core rows, i.e. row j1 of
    //    position e; every lane fetches its own position (the lanes of a position fetch the same words)
    const int ln = lane & 31, kh = lane >> 5;
    const int row = 32 * w + ln, e = row / N1, j1 = row % N1;
    const bool have = e < n;
    int k = 0, i1 = 0, i3 = 0;
    if (have) {
        if (info) {
            const int4 pi = info[lo + e];
            k = (unsigned)pi.x < (unsigned)L ? pi.x : 0;
            i1 = min(max(pi.y, 0), p.m1 - 1);
            i3 = min(max(pi.z, 0), p.m3 - 1);
        } else {
            k = (int)(vs[lo + e] - (uint32_t)L);                           // item 1 of position k carries L + k
            k = (unsigned)k < (unsigned)L ? k : 0;
            int i2x;
            decode(p, (uint32_t)indices[k], i1, i2x, i3);
        }
    }
    if (j1 == 0 && kh == 0 && have) { s_k[e] = k; s_w[e] = alpha ? alpha[k] : 1.f; }
    // ... and thread (position ee, bq) of the second product fetches its part of G3[i3] now, to have it when the
    //    first product is done
    const int ee = t / F::NBQ, bq = t % F::NBQ;
    const bool on = ee < n;
    float4 cv[F::BQ];
    const float4 *Cp;
    {
        int k2 = 0, i1x, i2x, i3x = 0;
        if (on) {
            if (info) {
                i3x = min(max(info[lo + ee].z, 0), p.m3 - 1);
            } else {
                k2 = (int)(vs[lo + ee] - (uint32_t)L);
                k2 = (unsigned)k2 < (unsigned)L ? k2 : 0;
                decode(p, (uint32_t)indices[k2], i1x, i2x, i3x);
            }
        }
        // (the NBQ lanes of a position read neighbouring rows of the slice: b = NBQ i + bq)
        Cp = reinterpret_cast<const float4 *>(G3 + (size_t)i3x * C::sC) + bq;
        if constexpr (F::EARLY_C) {
#pragma unroll
            for (int i = 0; i < F::BQ; ++i) cv[i] = on ? Cp[i * F::NBQ] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    // 4. A operand: step s of the product covers k = kh KH + s (any order of k will do as long as both operands
    //    agree), so a lane reads half a row of G1[i1], contiguous
    float areg[F::KH];
    {
        const float *Ap = G1 + (size_t)i1 * C::sA + j1 * R + kh * F::KH;
#pragma unroll
        for (int q = 0; q < F::KH / 4; ++q) {
            const float4 x = have ? *reinterpret_cast<const float4 *>(Ap + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
            areg[4 * q + 0] = x.x; areg[4 * q + 1] = x.y; areg[4 * q + 2] = x.z; areg[4 * q + 3] = x.w;
        }
    }
#pragma unroll
    for (int q = 0; q < NB4; ++q) reinterpret_cast<float4 *>(fo_lds)[q * WG + t] = bm[q];
    __syncthreads();
    // 5. T0 block of this wave: rows 32 w .. 32 w + 31, the R columns of j2
    mfma16_t acc[F::CB];
#pragma unroll
    for (int cb = 0; cb < F::CB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;
#pragma unroll
    for (int s = 0; s < F::KH; ++s) {
        const float *Brow = fo_lds + (kh * F::KH + s) * R + ln;
#pragma unroll
        for (int cb = 0; cb < F::CB; ++cb)
            acc[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(areg[s], Brow[32 * cb], acc[cb], 0, 0, 0);
    }
    __syncthreads();                                                       // the slice has been read by everyone
    // 6. the block to LDS: register r of lane (kh, ln) is row 8 (r / 4) + 4 kh + r % 4, column ln of its 32 x 32 tile
#pragma unroll
    for (int cb = 0; cb < F::CB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            fo_lds[(32 * w + 8 * (r / 4) + 4 * kh + r % 4) * LDT + 32 * cb + ln] = acc[cb][r];
    __syncthreads();
    // 7. the kept copy of T0: t0[k][j1][j2][R]
    if (t0_out) {
        for (int i = t; i < F::ROWS * R / 4; i += WG) {
            const int rowl = i / (R / 4), col = 4 * (i % (R / 4)), e7 = rowl / N1;
            if (e7 < n) {
                const float2 lo2 = *reinterpret_cast<const float2 *>(fo_lds + rowl * LDT + col);
                const float2 hi2 = *reinterpret_cast<const float2 *>(fo_lds + rowl * LDT + col + 2);
                *reinterpret_cast<float4 *>(t0_out + ((size_t)s_k[e7] * N1 + rowl % N1) * COLS + j2 * R + col) =
                    make_float4(lo2.x, lo2.y, hi2.x, hi2.y);
            }
        }
    }
    // 8. second product: rows (j1, j2) of the position's T0 (R values each) against G3[i3] (R x n3), weighted.  Thread
    //    (position, bq) takes BQ values of b for all j1; the NBQ partial sums of a position sit in neighbouring lanes.
    {
        float4 o[N1];
#pragma unroll
        for (int j = 0; j < N1; ++j) o[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if constexpr (!F::EARLY_C) {
#pragma unroll
            for (int i = 0; i < F::BQ; ++i) cv[i] = on ? Cp[i * F::NBQ] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        if (on) {
#pragma unroll
            for (int i = 0; i < F::BQ; ++i) {
                const float4 c = cv[i];
#pragma unroll
                for (int j = 0; j < N1; ++j) {
                    const float tv = fo_lds[(ee * N1 + j) * LDT + i * F::NBQ + bq];
                    o[j].x = fmaf(tv, c.x, o[j].x); o[j].y = fmaf(tv, c.y, o[j].y);
                    o[j].z = fmaf(tv, c.z, o[j].z); o[j].w = fmaf(tv, c.w, o[j].w);
                }
            }
        }
#pragma unroll
        for (int d = 1; d < F::NBQ; d <<= 1)
#pragma unroll
            for (int j = 0; j < N1; ++j) {
                o[j].x += __shfl_xor(o[j].x, d); o[j].y += __shfl_xor(o[j].y, d);
                o[j].z += __shfl_xor(o[j].z, d); o[j].w += __shfl_xor(o[j].w, d);
            }
        if (on) {
            const float wgt = s_w[ee];
#pragma unroll
            for (int j = 0; j < N1; ++j)
                if (bq == j % F::NBQ)                                        // the writers of a position share out its j1
                    *reinterpret_cast<float4 *>(rows_out + (size_t)s_k[ee] * C::N + (j * N2 + j2) * 4) =
                        make_float4(wgt * o[j].x, wgt * o[j].y, wgt * o[j].z, wgt * o[j].w);
        }
    }
    __syncthreads();                                                       // LDS is reused by the next tile
    }  // tiles
}

// out[bag] = sum over the bag's positions of rows[k] (already weighted) or, for a cached row, alpha[k] times its
// line of the cache.  One wave per bag.  The wave looks at up to 64 positions at once (lane l probes the cache for
// position l); then lane (sub, f) adds float4 f of every (64 / (N/4))-th of them, four in flight, and the lanes'
// sums are added in a fixed order at the end.
__global__ __launch_bounds__(WG) void fwd_pool_kernel(int N, const float *__restrict__ rows,
                                                      const int64_t *__restrict__ indices,
                                                      const int64_t *__restrict__ offsets, int n_bags,
                                                      const float *__restrict__ alpha, CacheDev cache, float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int bag = blockIdx.x * NWAVE + (threadIdx.x >> 6);
    if (bag >= n_bags) return;
    const int nq = N / 4, per = WAVE / nq;                                  // N a power of two <= 256
    const int f = lane % nq, sub = lane / nq;
    const int k0 = offsets ? (int)offsets[bag] : bag, k1 = offsets ? (int)offsets[bag + 1] : bag + 1;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int kc = k0; kc < k1; kc += WAVE) {
        const int cnt = min(WAVE, k1 - kc);
        int myslot = -1;
        float myw = 1.f;
        if (cache.K && lane < cnt) {
            myslot = cache_probe(cache, (uint32_t)indices[kc + lane]);
            if (myslot >= 0 && alpha) myw = alpha[kc + lane];
        }
        for (int qb = 0; qb < cnt; qb += 4 * per) {                          // uniform: every lane takes part in the shuffles
            const int q0 = qb + sub;
            float4 x[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int pi = min(q0 + q * per, cnt - 1);
                const int sl = __shfl(myslot, pi);
                const float wgt = __shfl(myw, pi);
                const float *src = sl >= 0 ? cache.rows + (size_t)sl * N : rows + (size_t)(kc + pi) * N;
                const float4 y = *reinterpret_cast<const float4 *>(src + 4 * f);
                x[q] = make_float4(wgt * y.x, wgt * y.y, wgt * y.z, wgt * y.w);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (q0 + q * per < cnt) { acc.x += x[q].x; acc.y += x[q].y; acc.z += x[q].z; acc.w += x[q].w; }
        }
    }
    for (int d = nq; d < WAVE; d <<= 1) {
        acc.x += __shfl_xor(acc.x, d); acc.y += __shfl_xor(acc.y, d);
        acc.z += __shfl_xor(acc.z, d); acc.w += __shfl_xor(acc.w, d);
    }
    if (sub == 0) *reinterpret_cast<float4 *>(out + (size_t)bag * N + 4 * f) = acc;
}

// Shapes the slice-owner forward handles.
static inline bool fwd_owner_supported(const Params &p)
{
    const int cfg = fast_config(p);
    return (cfg == 2 || cfg == 3 || cfg == 4 || cfg == 5) && p.m2 <= FO_MAX_M2;
}

// positions per tile and entries of the tile table (the tiles in use come first, the rest hold no items)
static inline int fwd_owner_tp(const Params &p) { return 128 / p.n1; }
static inline int fwd_owner_tiles(const Params &p, int64_t L) { return (int)((L + fwd_owner_tp(p) - 1) / fwd_owner_tp(p)) + p.m2; }

template <typename C>
static inline hipError_t launch_fwd_owner(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx,
                                          int64_t L, const int64_t *off, int n_bags, const float *alpha, const CacheDev &cd,
                                          const uint32_t *vs, const int4 *info, const int4 *tiles, float *rows, float *out,
                                          float *t0_out, hipStream_t st)
{
    const size_t lds = fo_lds_bytes<C>();
    static bool allowed = false;                                             // (one device per process)
    if (!allowed) {
        hipError_t e = hipFuncSetAttribute((const void *)fwd_owner_kernel<C>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        allowed = true;
    }
    // How many of the table's entries are in use is only known on the device (cached positions are in no list):
    // at most FO_GRID_TILES tiles are started, each workgroup goes on to later tiles while there are any.
    const int ntiles = fwd_owner_tiles(p, L);
    const int grid_tiles = ntiles < FO_GRID_TILES ? ntiles : FO_GRID_TILES;
    hipLaunchKernelGGL((fwd_owner_kernel<C>), dim3(grid_tiles * C::N2), dim3(WG), lds, st, p, G1, G2, G3, idx, (int)L, alpha, vs,
                       info, tiles, ntiles, rows, t0_out);
    hipLaunchKernelGGL(fwd_pool_kernel, dim3((unsigned)((n_bags + NWAVE - 1) / NWAVE)), dim3(WG), 0, st, C::N, rows, idx, off, n_bags,
                       alpha, cd, out);
    return hipGetLastError();
}

static inline hipError_t fwd_owner(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx,
                                   int64_t L, const int64_t *off, int n_bags, const float *alpha, const CacheDev &cd,
                                   const uint32_t *vs, const int4 *info, const int4 *tiles, float *rows, float *out, float *t0_out,
                                   hipStream_t st)
{
    switch (fast_config(p)) {
    case 2: return launch_fwd_owner<Cfg224R32>(p, G1, G2, G3, idx, L, off, n_bags, alpha, cd, vs, info, tiles, rows, out, t0_out, st);
    case 3: return launch_fwd_owner<Cfg224R64>(p, G1, G2, G3, idx, L, off, n_bags, alpha, cd, vs, info, tiles, rows, out, t0_out, st);
    case 4: return launch_fwd_owner<Cfg444R32>(p, G1, G2, G3, idx, L, off, n_bags, alpha, cd, vs, info, tiles, rows, out, t0_out, st);
    case 5: return launch_fwd_owner<Cfg444R64>(p, G1, G2, G3, idx, L, off, n_bags, alpha, cd, vs, info, tiles, rows, out, t0_out, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tt
