// Specialised kernels for the shapes the paper uses: column factors (2,2,4) and
// (4,4,4) with equal ranks R in {8,16,32,64}.  All sizes are compile-time, the
// contraction chain of Eq. 3 / Eq. 4 runs out of registers, and one lane owns V
// consecutive columns c = (j2, b) of the unfolded middle slice G2[i2] (R x n2 R).
//
// Lane layout (wave64): lane l < LANES = n2 R / V owns columns c0 .. c0+V-1 with
// c0 = l V, j2 = c0 / R, b0 = c0 % R.  The LN = R / V lanes that share j2 are
// consecutive, so the sum over b of stage 1 is a shuffle reduction inside an
// aligned lane group.  G1[i1] is wave-uniform and is read through scalar loads.
#pragma once

#include "tt_common.h"
#include "tt_select.h"

namespace tt {

template <int N1_, int N2_, int N3_, int R_, int V_>
struct FastCfg {
    static constexpr int N1 = N1_, N2 = N2_, N3 = N3_, R = R_, V = V_;
    static constexpr int COLS = N2 * R;
    static constexpr int LANES = COLS / V;         // active lanes of a wave
    static constexpr int LN = R / V;               // lanes per j2 group
    static constexpr int N = N1 * N2 * N3;
    static constexpr int NV = N1 * N3;             // outputs per j2 group
    static constexpr int sA = N1 * R, sB = R * COLS, sC = R * N3;
    static constexpr int RQ = R / NWAVE;           // rows a of G2[i2] per wave in the backward
    static_assert(LANES <= WAVE && COLS % V == 0 && R % V == 0 && R % NWAVE == 0, "bad lane layout");
    static_assert(N3 == 4 && N % 4 == 0, "float4 paths assume n3 = 4");
};

template <int V>
__device__ __forceinline__ void load_vec(const float *__restrict__ p, float (&o)[V])
{
    if constexpr (V == 1) {
        o[0] = p[0];
    } else if constexpr (V == 2) {
        const float2 t = *reinterpret_cast<const float2 *>(p);
        o[0] = t.x; o[1] = t.y;
    } else {
        static_assert(V == 4, "V must be 1, 2 or 4");
        const float4 t = *reinterpret_cast<const float4 *>(p);
        o[0] = t.x; o[1] = t.y; o[2] = t.z; o[3] = t.w;
    }
}

template <int V>
__device__ __forceinline__ void store_vec(float *__restrict__ p, const float (&o)[V])
{
    if constexpr (V == 1) {
        p[0] = o[0];
    } else if constexpr (V == 2) {
        *reinterpret_cast<float2 *>(p) = make_float2(o[0], o[1]);
    } else {
        static_assert(V == 4, "V must be 1, 2 or 4");
        *reinterpret_cast<float4 *>(p) = make_float4(o[0], o[1], o[2], o[3]);
    }
}

// Sum NV values per lane over an aligned group of LN lanes.  While more than one value
// is left, each step halves the values a lane keeps (the lane whose bit D is set keeps
// the upper half); then plain butterfly adds.  Afterwards a lane holds KEEP =
// max(1, NV / LN) values v[0..KEEP) that belong to the indices base .. base+KEEP-1 with
// base = reduce_base<NV, LN>(lane); when LN > NV the value is replicated over the lanes
// that agree in their low log2(NV) bits.
template <int H, int D, int LN>
struct GroupReduce {
    template <int NV>
    static __device__ __forceinline__ void run(float (&v)[NV], int lane)
    {
        if constexpr (D < LN) {
            if constexpr (H >= 1) {
                const bool hi = (lane & D) != 0;
#pragma unroll
                for (int i = 0; i < H; ++i) {
                    const float send = hi ? v[i] : v[i + H];
                    const float recv = __shfl_xor(send, D);
                    v[i] = (hi ? v[i + H] : v[i]) + recv;
                }
                GroupReduce<H / 2, D * 2, LN>::run(v, lane);
            } else {
                v[0] += __shfl_xor(v[0], D);
                GroupReduce<0, D * 2, LN>::run(v, lane);
            }
        }
    }
};

template <int NV, int LN>
__device__ __forceinline__ void group_reduce(float (&v)[NV], int lane)
{
    GroupReduce<NV / 2, 1, LN>::run(v, lane);
}

template <int NV, int LN>
__device__ __forceinline__ int reduce_base(int lane)
{
    int base = 0;
#pragma unroll
    for (int d = 1, h = NV / 2; d < LN && h >= 1; d <<= 1, h >>= 1)
        if (lane & d) base += h;
    return base;
}

template <int NV, int LN>
struct ReduceKeep {
    static constexpr int value = NV > LN ? NV / LN : 1;
    static constexpr int writers = NV > LN ? LN : NV;     // lanes of a group that hold distinct results
};

// ---- forward ---------------------------------------------------------------------
constexpr int FWD_WAVE_PER_BAG = 0, FWD_WG_PER_BAG = 1, FWD_XCD_LOCAL = 2;
constexpr int FWD_SEG = 32;                       // bags per segment of the XCD-local variant (8 workgroups, a bag per wave)
// One wave per bag.  The wave reads the bag's positions 64 at a time and probes the cache
// for all of them at once; cached rows are summed 64 / (N/4) at a time as float4 pieces,
// the other positions go through the cores one after the other.  The partial products of
// stage 1 are accumulated over the bag's lookups before one shuffle reduction per bag,
// and the sum of the cached rows is added to the result at the end.
// MODE FWD_WG_PER_BAG: a whole workgroup per bag, for long bags: its four waves take a quarter of the bag's
// positions each and their results are added through LDS, in wave order.
// MODE FWD_XCD_LOCAL: still a wave per bag, but which bags a workgroup takes depends on their rows, so that each of
// the 8 XCDs reads an eighth of the second core (see the end of the kernel).
template <typename C, int MODE>
__global__ __launch_bounds__(WG) void fwd_fast_kernel(Params p, const float *__restrict__ G1,
                                                      const float *__restrict__ G2, const float *__restrict__ G3,
                                                      const int64_t *__restrict__ indices,
                                                      const int64_t *__restrict__ offsets, int n_bags,
                                                      const float *__restrict__ alpha, CacheDev cache,
                                                      float *__restrict__ out, float *__restrict__ t0_out)
{
    constexpr int N1 = C::N1, N2 = C::N2, N3 = C::N3, R = C::R, V = C::V;
    constexpr bool WGBAG = MODE == FWD_WG_PER_BAG;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool active = lane < C::LANES;
    const int c0 = active ? lane * V : 0;
    const int j2 = c0 / R, b0 = c0 % R;

    // bounds: the bag's positions [bk0, bk1) and its first row if the caller has read them already (bk0 < 0: not)
    auto do_bag = [&](const int bag, const int bk0, const int bk1, const uint32_t brow) __attribute__((always_inline)) {
    float acc[C::NV];
#pragma unroll
    for (int i = 0; i < C::NV; ++i) acc[i] = 0.f;

    // one position through the cores: T0 = A Bm (kept for the backward pass if asked for), then acc += w T0 C
    auto through_cores = [&](uint32_t row, float w, int k) __attribute__((always_inline)) {
        int i1, i2, i3;
        decode(p, row, i1, i2, i3);
        const float *A = G1 + (size_t)i1 * C::sA;
        const float *B = G2 + (size_t)i2 * C::sB + c0;
        const float *Cp = G3 + (size_t)i3 * C::sC + b0 * N3;
        float t0[N1][V];
#pragma unroll
        for (int j1 = 0; j1 < N1; ++j1)
#pragma unroll
            for (int v = 0; v < V; ++v) t0[j1][v] = 0.f;
#pragma unroll
        for (int a = 0; a < R; ++a) {
            float bv[V];
            load_vec<V>(B + a * C::COLS, bv);
#pragma unroll
            for (int j1 = 0; j1 < N1; ++j1) {
                const float av = A[j1 * R + a];
#pragma unroll
                for (int v = 0; v < V; ++v) t0[j1][v] = fmaf(av, bv[v], t0[j1][v]);
            }
        }
        if (t0_out && active) {                             // keep T0[(j1,j2)][b] of this position for the backward pass
            float *o = t0_out + (size_t)k * (N1 * C::COLS) + c0;
#pragma unroll
            for (int j1 = 0; j1 < N1; ++j1) store_vec<V>(o + j1 * C::COLS, t0[j1]);
        }
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const float4 cv = *reinterpret_cast<const float4 *>(Cp + v * N3);
#pragma unroll
            for (int j1 = 0; j1 < N1; ++j1) {
                const float tw = w * t0[j1][v];
                acc[j1 * N3 + 0] = fmaf(tw, cv.x, acc[j1 * N3 + 0]);
                acc[j1 * N3 + 1] = fmaf(tw, cv.y, acc[j1 * N3 + 1]);
                acc[j1 * N3 + 2] = fmaf(tw, cv.z, acc[j1 * N3 + 2]);
                acc[j1 * N3 + 3] = fmaf(tw, cv.w, acc[j1 * N3 + 3]);
            }
        }
    };

    int k0 = bk0 >= 0 ? bk0 : (offsets ? (int)offsets[bag] : bag);
    int k1 = bk0 >= 0 ? bk1 : (offsets ? (int)offsets[bag + 1] : bag + 1);
    if (WGBAG) {                                            // this wave's quarter of the bag
        const int per = (k1 - k0 + NWAVE - 1) / NWAVE;
        k0 = min(k1, k0 + wv * per);
        k1 = min(k1, k0 + per);
    }
    int kb = k0;
    if (k1 - k0 == 1 && !cache.K) {
        // one index per bag and no cache (the Criteo-shaped workloads): the shortest chain from index to slices
        through_cores(bk0 >= 0 ? brow : (uint32_t)__builtin_amdgcn_readfirstlane((int)indices[k0]), alpha ? alpha[k0] : 1.f, k0);
        kb = k1;
    }
    // cached rows: NG = 64 / NQ of them per step, lane (g, f) adds float4 f of the g-th one
    constexpr int NQ = C::N / 4, NG = WAVE / NQ;
    const int cg = lane / NQ, cf = lane % NQ;
    float4 cacc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (; kb < k1; kb += WAVE) {
        // The wave reads up to 64 positions of the bag at once and probes the cache for all of them, so the
        // chain index -> probe -> row data is walked once per 64 positions, not once per position.
        int pk = kb + lane;
        const bool valid = pk < k1;
        uint32_t prow = valid ? (uint32_t)indices[pk] : 0u;
        float pw = valid && alpha ? alpha[pk] : 1.f;
        int nb = k1 - kb < WAVE ? k1 - kb : WAVE, first = 0;       // positions first .. nb-1 go through the cores
        if (cache.K) {
            int pslot = valid ? cache_probe(cache, prow) : -1;
            const uint64_t hits = __ballot(pslot >= 0), lt = lanemask_lt();
            const int nhit = __popcll(hits);
            if (nhit) {
                // hits to lanes 0 .. nhit-1, the rest behind them, both in their old order
                const int dst = 4 * (pslot >= 0 ? __popcll(hits & lt) : nhit + __popcll(~hits & lt));
                pslot = __builtin_amdgcn_ds_permute(dst, pslot);
                pk = __builtin_amdgcn_ds_permute(dst, pk);
                prow = (uint32_t)__builtin_amdgcn_ds_permute(dst, (int)prow);
                pw = __int_as_float(__builtin_amdgcn_ds_permute(dst, __float_as_int(pw)));
                for (int h0 = 0; h0 < nhit; h0 += NG) {
                    const int h = h0 + cg;
                    const int sl = __shfl(pslot, h & 63);
                    const float w = __shfl(pw, h & 63);
                    if (h < nhit) {
                        const float4 t = *reinterpret_cast<const float4 *>(cache.rows + (size_t)sl * C::N + 4 * cf);
                        cacc.x = fmaf(w, t.x, cacc.x); cacc.y = fmaf(w, t.y, cacc.y);
                        cacc.z = fmaf(w, t.z, cacc.z); cacc.w = fmaf(w, t.w, cacc.w);
                    }
                }
                first = nhit;
            }
        }
        for (int j = first; j < nb; ++j)
            through_cores((uint32_t)__builtin_amdgcn_readlane((int)prow, j),
                          __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pw), j)), __builtin_amdgcn_readlane(pk, j));
    }
    group_reduce<C::NV, C::LN>(acc, lane);
    constexpr int KEEP = ReduceKeep<C::NV, C::LN>::value;
    const int lg = lane % C::LN;
    const int base = reduce_base<C::NV, C::LN>(lane);
    if (cache.K) {
        // every lane gets the sum of float4 f over the groups, then the writers fetch their elements
#pragma unroll
        for (int d = NQ; d < WAVE; d <<= 1) {
            cacc.x += __shfl_xor(cacc.x, d); cacc.y += __shfl_xor(cacc.y, d);
            cacc.z += __shfl_xor(cacc.z, d); cacc.w += __shfl_xor(cacc.w, d);
        }
#pragma unroll
        for (int i = 0; i < KEEP; ++i) {
            const int idx = base + i, j1 = idx / N3, j3 = idx % N3, q = j1 * N2 + j2;
            const float x = __shfl(cacc.x, q), y = __shfl(cacc.y, q), z = __shfl(cacc.z, q), u = __shfl(cacc.w, q);
            acc[i] += j3 == 0 ? x : (j3 == 1 ? y : (j3 == 2 ? z : u));
        }
    }
    if constexpr (WGBAG) {
        __shared__ float partial[NWAVE][C::N];
        if (active && lg < ReduceKeep<C::NV, C::LN>::writers) {
#pragma unroll
            for (int i = 0; i < KEEP; ++i) {
                const int idx = base + i, j1 = idx / N3, j3 = idx % N3;
                partial[wv][(j1 * N2 + j2) * N3 + j3] = acc[i];
            }
        }
        __syncthreads();
        for (int e = threadIdx.x; e < C::N; e += WG)
            out[(size_t)bag * C::N + e] = (partial[0][e] + partial[1][e]) + (partial[2][e] + partial[3][e]);
    } else if (active && lg < ReduceKeep<C::NV, C::LN>::writers) {
        float *o = out + (size_t)bag * C::N;
#pragma unroll
        for (int i = 0; i < KEEP; ++i) {
            const int idx = base + i;                       // = j1 * N3 + j3
            const int j1 = idx / N3, j3 = idx % N3;
            o[(j1 * N2 + j2) * N3 + j3] = acc[i];
        }
    }
    };  // do_bag

    if constexpr (MODE == FWD_XCD_LOCAL) {
        // Workgroup 8 s + x runs on XCD x (workgroups go to the XCDs in turn).  Of the FWD_SEG bags of segment s it takes
        // those whose first row has its second digit in the x-th eighth of [0, m2), so that every XCD reads an eighth
        // of the second core, which then stays in its L2 -- but at most an eighth of the segment's bags: what a
        // bucket holds beyond that (a hot row fills its bucket) goes to the workgroups with room left, in a fixed
        // order.  Every wave works the assignment out for itself (lane l looks at bag l) and takes every fourth bag
        // of its workgroup's list.  Any assignment gives the same result: a bag is computed by one wave as a whole.
        static_assert(FWD_SEG <= WAVE && FWD_SEG % 8 == 0, "one bag per lane");
        __shared__ int list[NWAVE][FWD_SEG / 8 + 1];
        const int x = blockIdx.x & 7, first = (int)(blockIdx.x >> 3) * FWD_SEG;
        const int mybag = first + lane;
        const bool valid = lane < FWD_SEG && mybag < n_bags;
        const int k0v = valid ? (offsets ? (int)offsets[mybag] : mybag) : 0;
        const int k1v = valid ? (offsets ? (int)offsets[mybag + 1] : mybag + 1) : 0;
        const uint32_t rowv = k1v > k0v ? (uint32_t)indices[k0v] : 0u;
        int bucket = lane & 7;                                             // empty bags: spread
        if (k1v > k0v) {
            int i1, i2, i3;
            decode(p, rowv, i1, i2, i3);
            bucket = min(7, (int)fast_div((uint32_t)i2 * 8u, (uint32_t)p.m2, p.mg2));
        }
        uint64_t M[8];
        int spare_before = 0, spare_mine = 0, nvalid = __popcll(__ballot(valid));
        const int cap = (nvalid + 7) / 8;
#pragma unroll
        for (int y = 0; y < 8; ++y) {
            M[y] = __ballot(valid && bucket == y);
            const int spare = cap - min(cap, (int)__popcll(M[y]));
            if (y < x) spare_before += spare;
            if (y == x) spare_mine = spare;
        }
        int cnt = 0;                                                       // bags of this workgroup
        {
            uint64_t m = 0;
#pragma unroll
            for (int y = 0; y < 8; ++y) m = y == x ? M[y] : m;
            for (int q = 0; m && q < cap; ++q) {                           // uniform: the bucket's first bags
                const int j = __builtin_ctzll(m);
                m &= m - 1;
                if (lane == 0) list[wv][cnt] = j;
                ++cnt;
            }
        }
        int r = 0;                                                         // number of the bag among those beyond the caps
#pragma unroll
        for (int y = 0; y < 8; ++y) {
            uint64_t m = M[y];
            for (int q = 0; m; ++q) {                                      // uniform
                const int j = __builtin_ctzll(m);
                m &= m - 1;
                if (q < cap) continue;
                if (r >= spare_before && r < spare_before + spare_mine) {
                    if (lane == 0) list[wv][cnt] = j;
                    ++cnt;
                }
                ++r;
            }
        }
        __builtin_amdgcn_wave_barrier();
        for (int q = wv; q < cnt; q += NWAVE) {                            // uniform
            const int j = __builtin_amdgcn_readfirstlane(list[wv][q]);    // the bag that lane j looked at
            do_bag(first + j, __builtin_amdgcn_readlane(k0v, j), __builtin_amdgcn_readlane(k1v, j),
                   (uint32_t)__builtin_amdgcn_readlane((int)rowv, j));
        }
    } else {
        const int bag = WGBAG ? (int)blockIdx.x : (int)blockIdx.x * NWAVE + wv;
        if (bag < n_bags) do_bag(bag, -1, 0, 0u);           // (uniform in the workgroup if WGBAG)
    }
}

// ---- dispatch ----------------------------------------------------------------------

// L: number of positions; a workgroup per bag from an average of 32 positions per bag on (measured: at 20 positions
// per bag, most of them cached, a wave per bag is faster; at 100 the workgroup is)
template <typename C>
static inline void launch_fwd(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx,
                              const int64_t *off, int64_t L, int n_bags, const float *alpha, const CacheDev &cd, float *out,
                              float *t0_out, hipStream_t st)
{
    static_assert(NWAVE == 4, "the workgroup-per-bag variant adds four partial results");
    // XCD-local: short bags (one index mostly), a second core too large for one XCD's L2 (4 MB) next to the rest, and
    // enough slices to read that their bandwidth matters more than the longer way to a wave's first load
    // (measured: 8,192 lookups of 64 KB slices 42.5 -> 31 us; 4,096 of 32 KB slices 11.7 -> 13.4 us)
    const bool xcd_local = L < 2 * (int64_t)n_bags && (size_t)p.m2 * C::sB * sizeof(float) > (3u << 20) &&
                           (size_t)n_bags * C::sB * sizeof(float) >= ((size_t)256 << 20);
    if (off && L >= 32 * (int64_t)n_bags)
        hipLaunchKernelGGL((fwd_fast_kernel<C, FWD_WG_PER_BAG>), dim3(n_bags), dim3(WG), 0, st, p, G1, G2, G3, idx, off, n_bags,
                           alpha, cd, out, t0_out);
    else if (xcd_local)
        hipLaunchKernelGGL((fwd_fast_kernel<C, FWD_XCD_LOCAL>), dim3(8 * ((n_bags + FWD_SEG - 1) / FWD_SEG)), dim3(WG), 0, st, p,
                           G1, G2, G3, idx, off, n_bags, alpha, cd, out, t0_out);
    else
        hipLaunchKernelGGL((fwd_fast_kernel<C, FWD_WAVE_PER_BAG>), dim3((n_bags + NWAVE - 1) / NWAVE), dim3(WG), 0, st, p, G1, G2,
                           G3, idx, off, n_bags, alpha, cd, out, t0_out);
}

// id of the specialised configuration for this shape, or -1
static inline int fast_config(const Params &p)
{
    if (p.R1 != p.R2) return -1;
    const int R = p.R1;
    if (p.n1 == 2 && p.n2 == 2 && p.n3 == 4) {
        if (R == 8) return 0;
        if (R == 16) return 1;
        if (R == 32) return 2;
        if (R == 64) return 3;
    }
    if (p.n1 == 4 && p.n2 == 4 && p.n3 == 4) {
        if (R == 32) return 4;
        if (R == 64) return 5;
    }
    return -1;
}

using Cfg224R8 = FastCfg<2, 2, 4, 8, 1>;
using Cfg224R16 = FastCfg<2, 2, 4, 16, 1>;
using Cfg224R32 = FastCfg<2, 2, 4, 32, 1>;
using Cfg224R64 = FastCfg<2, 2, 4, 64, 2>;
using Cfg444R32 = FastCfg<4, 4, 4, 32, 2>;
using Cfg444R64 = FastCfg<4, 4, 4, 64, 4>;

// Returns 0 if a specialised forward kernel was launched, -1 if the shape has none.
static inline int fast_fwd(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx,
                           const int64_t *off, int64_t L, int n_bags, const float *alpha, const CacheDev &cd, float *out,
                           float *t0_out, hipStream_t st)
{
    switch (fast_config(p)) {
    case 0: launch_fwd<Cfg224R8>(p, G1, G2, G3, idx, off, L, n_bags, alpha, cd, out, t0_out, st); return 0;
    case 1: launch_fwd<Cfg224R16>(p, G1, G2, G3, idx, off, L, n_bags, alpha, cd, out, t0_out, st); return 0;
    case 2: launch_fwd<Cfg224R32>(p, G1, G2, G3, idx, off, L, n_bags, alpha, cd, out, t0_out, st); return 0;
    case 3: launch_fwd<Cfg224R64>(p, G1, G2, G3, idx, off, L, n_bags, alpha, cd, out, t0_out, st); return 0;
    case 4: launch_fwd<Cfg444R32>(p, G1, G2, G3, idx, off, L, n_bags, alpha, cd, out, t0_out, st); return 0;
    case 5: launch_fwd<Cfg444R64>(p, G1, G2, G3, idx, off, L, n_bags, alpha, cd, out, t0_out, st); return 0;
    default: return -1;
    }
}

}  // namespace tt
