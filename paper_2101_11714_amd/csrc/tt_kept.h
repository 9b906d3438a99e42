// Backward pass for short index lists of the (2,2,4) shapes, fed by what can be prepared before it runs
// (Section 4.2, first paragraph: the recomputation of Alg. 2 can be traded for stored tensors; the grouping
// of the positions by core slice that Alg. 2's "+=" implies depends on the indices alone).
//
// The forward pass keeps T0[k] = G1[i1] G2[i2] of every position whose row is not cached (tt_fast.h), and a few
// workgroups (the "sorters": a launch of their own, or riders of the backward launch of the batch before) file
// every position under the three core slices it touches.  A slice owner of the backward pass then loads its
// list instead of scanning and decoding the whole index array, and the owner of a G3 slice reads T0 instead of
// recomputing it.
//
// Lists.  Sorter g files the positions [256 g, 256 (g+1)), one per thread.  For every slice ("bin": m1 + m2 +
// m3 of them) and sorter there is a sub-list: its length and the place of its overflow in hdr[bin][g], its first
// capg entries at fixed places in main[bin][], the rest in the sorter's overflow area.  An entry is (k, hsub,
// row): hsub is the place in the sub-list of the first entry with the same row, so that the owner sees the runs
// of equal rows without comparing rows.  A thread sets bit t of its three slices' bitmaps in LDS (an OR: the
// order does not matter) and its place in a sub-list is the number of set bits below t: the sub-lists are in
// position order whatever the order in which the threads ran, so every sum that follows has a fixed order.
#pragma once

#include "tt_fast_bwd.h"

namespace tt {

constexpr int KP_CHK = WG;                 // positions per sorter workgroup: one per thread
constexpr int KP_MAXG = 32;                // sorter workgroups (sub-lists per slice) at most
constexpr int KP_MAX_L = KP_CHK * KP_MAXG; // positions per call
constexpr int KP_MAX_BINS = 1536;          // m1 + m2 + m3
constexpr int KP_BW = KP_CHK / 32;         // words of a sorter's bitmap per slice
constexpr int KP_OV = 3 * KP_CHK;          // overflow entries per sorter
constexpr uint32_t KP_NONE = 0xFFFFFFFFu;

// where the kept data of one call lives (byte offsets into the caller's buffer)
struct KeptLayout {
    size_t t0, hdr, mainp, ov, bytes;
    int G, capg, nbins;
};

static inline KeptLayout kept_layout(const Params &p, int64_t L)
{
    KeptLayout k;
    const int64_t Lp = L > 0 ? L : 1;
    k.G = (int)((Lp + KP_CHK - 1) / KP_CHK);
    int gp = 8;                                                        // sub-lists that share the 64 fixed places of a slice
    while (gp < k.G) gp <<= 1;
    k.capg = WAVE / gp;                                                // 8, 4 or 2 fixed places per sub-list
    k.nbins = p.m1 + p.m2 + p.m3;
    size_t at = 0;
    k.t0 = at; at += align256((size_t)Lp * p.n1 * p.cols * sizeof(float));
    k.hdr = at; at += align256((size_t)k.nbins * KP_MAXG * sizeof(uint2));
    k.mainp = at; at += align256((size_t)k.nbins * WAVE * sizeof(uint4));
    k.ov = at; at += align256((size_t)k.G * KP_OV * sizeof(uint4));
    k.bytes = at;
    return k;
}

struct KeptDev {
    float *t0;
    uint2 *hdr;
    uint4 *mainp, *ov;
    int G, capg, cshift, nbins;                                       // capg = 1 << cshift
};

static inline KeptDev kept_dev(void *base, const KeptLayout &k)
{
    char *b = (char *)base;
    return KeptDev{(float *)(b + k.t0), (uint2 *)(b + k.hdr), (uint4 *)(b + k.mainp),
                   (uint4 *)(b + k.ov), k.G, k.capg, k.capg == 8 ? 3 : (k.capg == 4 ? 2 : 1), k.nbins};
}

// Does the kept path cover this call?  (Otherwise the entry points fall back to the stored-T0 kernels.)
static inline bool kept_supported(const Params &p, int64_t L)
{
    const int cfg = fast_config(p);
    return cfg >= 0 && cfg <= 2 && L > 0 && L <= KP_MAX_L && p.m1 + p.m2 + p.m3 <= KP_MAX_BINS;   // (R = 64: measured slower)
}

// ---- sorter: one workgroup files the positions [g KP_CHK, (g+1) KP_CHK), one per thread -------------
// Thread t sets bit t in the bitmap of each of its three slices (an OR: the order does not matter), so the
// place of its entry in a sub-list is the number of set bits below t: the sub-lists come out in the order
// of the positions, whatever the order in which the threads ran.

struct KpSortLds {
    uint32_t (*bm)[KP_BW];                           // [nbins]: which threads' positions touch the slice
    uint32_t *hkey;                                  // [2 KP_CHK] open-addressing table: row -> ...
    uint32_t *hmin;                                  // ... the first thread that holds it
    int *ovo;                                        // [nbins]
    int *scan_tmp;                                   // [NWAVE + 1]
};

static inline size_t kp_sort_lds_bytes(int nbins)
{
    return (size_t)nbins * KP_BW * 4 + 2 * (2 * KP_CHK) * 4 + (size_t)nbins * 4 + (NWAVE + 1) * 4 + 16;
}

__device__ __forceinline__ KpSortLds kp_sort_lds(unsigned char *base, int nbins)
{
    KpSortLds l;
    l.bm = reinterpret_cast<uint32_t (*)[KP_BW]>(base);
    l.hkey = reinterpret_cast<uint32_t *>(base) + (size_t)nbins * KP_BW;
    l.hmin = l.hkey + 2 * KP_CHK;
    l.ovo = reinterpret_cast<int *>(l.hmin + 2 * KP_CHK);
    l.scan_tmp = l.ovo + nbins;
    return l;
}

__device__ __forceinline__ int kp_bits_below(const uint32_t (&wd)[KP_BW], int t)
{
    int n = 0;
#pragma unroll
    for (int i = 0; i < KP_BW; ++i) {
        const uint32_t m = i < (t >> 5) ? 0xFFFFFFFFu : (i == (t >> 5) ? (1u << (t & 31)) - 1u : 0u);
        n += __popc(wd[i] & m);
    }
    return n;
}

__device__ __forceinline__ void kept_sort_body(const KpSortLds &lds, const Params &p, int g, const int64_t *__restrict__ indices,
                                               int L, const CacheDev &cache, const KeptDev &kd)
{
    static_assert(KP_BW == 8, "a slice's bitmap is two 16-byte pieces");
    const int t = threadIdx.x;
    const int k = g * KP_CHK + t;
    uint32_t row = k < L ? (uint32_t)indices[k] : KP_NONE;
    {
        uint4 *z = reinterpret_cast<uint4 *>(&lds.bm[0][0]);
        for (int i = t; i < kd.nbins * (KP_BW / 4); i += WG) z[i] = make_uint4(0u, 0u, 0u, 0u);
        for (int i = t; i < 2 * KP_CHK; i += WG) { lds.hkey[i] = KP_NONE; lds.hmin[i] = KP_NONE; }
    }
    if (cache.K && row != KP_NONE && cache_probe(cache, row) >= 0) row = KP_NONE;      // cached rows bypass the cores
    __syncthreads();
    int slot = 0, bins[3] = {0, 0, 0};
    if (row != KP_NONE) {
        uint32_t h = cache_hash(row, 2 * KP_CHK - 1);
        for (;;) {                                                         // ends: at most KP_CHK rows in twice as many slots
            const uint32_t old = atomicCAS(&lds.hkey[h], KP_NONE, row);
            if (old == KP_NONE || old == row) break;
            h = (h + 1) & (2 * KP_CHK - 1);
        }
        atomicMin(&lds.hmin[h], (uint32_t)t);
        slot = (int)h;
        int i1, i2, i3;
        decode(p, row, i1, i2, i3);
        bins[0] = i1; bins[1] = p.m1 + i2; bins[2] = p.m1 + p.m2 + i3;
#pragma unroll
        for (int r = 0; r < 3; ++r) atomicOr(&lds.bm[bins[r]][t >> 5], 1u << (t & 31));
    }
    __syncthreads();
    // lengths of the sub-lists, and where their entries beyond the fixed places go (running total in slice order)
    {
        constexpr int BPT = KP_MAX_BINS / WG;                               // slices per thread: t BPT .. t BPT + BPT - 1
        int cnt[BPT], sum = 0;
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            const int b = t * BPT + i;
            cnt[i] = 0;
            if (b < kd.nbins) {
                const uint4 lo4 = *reinterpret_cast<const uint4 *>(&lds.bm[b][0]), hi4 = *reinterpret_cast<const uint4 *>(&lds.bm[b][4]);
                cnt[i] = __popc(lo4.x) + __popc(lo4.y) + __popc(lo4.z) + __popc(lo4.w) + __popc(hi4.x) + __popc(hi4.y) +
                         __popc(hi4.z) + __popc(hi4.w);
            }
            sum += max(0, cnt[i] - kd.capg);
        }
        int total;
        int ex = block_excl_scan(sum, lds.scan_tmp, &total);
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            const int b = t * BPT + i;
            if (b < kd.nbins) {
                lds.ovo[b] = ex;
                kd.hdr[(size_t)b * KP_MAXG + g] = make_uint2((uint32_t)cnt[i], (uint32_t)ex);
            }
            ex += max(0, cnt[i] - kd.capg);
        }
    }
    __syncthreads();
    if (row != KP_NONE) {
        const int trep = (int)lds.hmin[slot];                              // first thread of the range with the same row
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int b = bins[r];
            const uint4 lo4 = *reinterpret_cast<const uint4 *>(&lds.bm[b][0]), hi4 = *reinterpret_cast<const uint4 *>(&lds.bm[b][4]);
            const uint32_t wd[KP_BW] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
            const int rank = kp_bits_below(wd, t);                         // my place in the sub-list
            const int hsub = kp_bits_below(wd, trep);                      // the place of the first entry with my row
            const uint4 e = make_uint4((uint32_t)k, (uint32_t)hsub, row, 0u);
            if (rank < kd.capg) kd.mainp[(size_t)b * WAVE + g * kd.capg + rank] = e;
            else kd.ov[(size_t)g * KP_OV + lds.ovo[b] + rank - kd.capg] = e;
        }
    }
}

extern __shared__ __align__(16) unsigned char kp_dyn_lds[];

__global__ __launch_bounds__(WG) void kept_sort_kernel(Params p, const int64_t *__restrict__ indices, int L, CacheDev cache, KeptDev kd)
{
    kept_sort_body(kp_sort_lds(kp_dyn_lds, kd.nbins), p, (int)blockIdx.x, indices, L, cache, kd);
}

// ---- backward: slice owners fed by the lists ----------------------------------------------------------

template <typename C>
struct KpCfg {
    static constexpr int W = 4096 / C::N;                   // list entries per window (16 KB of upstream gradients)
    static constexpr int SB = 16;                           // rows whose G1 and G3 slices sit in LDS (G2 owners)
    static constexpr int SMALL = C::sA + C::sC;
    static constexpr int BMR = C::RQ * C::V;                // registers per row for the wave's part of G2[i2]
    static constexpr int TB0 = 32 / BMR >= 4 ? 4 : (32 / BMR >= 1 ? 32 / BMR : 1);   // G1 owner: rows of G2 in flight
    static_assert(W <= FB_CAP && W % WAVE == 0, "windows hold whole pieces");
    static_assert(NWAVE * C::COLS * C::N3 <= W * C::N, "partials do not fit");
};

template <typename C>
struct __align__(16) KpLds {
    float stage[KpCfg<C>::W * C::N];                        // alpha_k * grad_out[bag(k)] of the window's entries, runs contiguous
    float small[KpCfg<C>::SB * KpCfg<C>::SMALL];            // must follow stage[]: both are written through one index
    uint32_t klist[FB_CAP], rows[FB_CAP];                   // the list (a round of it), in the order of the positions
    int epos[KpCfg<C>::W];
    int seg_start[KpCfg<C>::W + 1];
    int seg_i1[KpCfg<C>::W], seg_i2[KpCfg<C>::W], seg_i3[KpCfg<C>::W];
    uint32_t seg_k[KpCfg<C>::W];
    int pcnt[NWAVE];
};

// the next batch, whose lists the sorters that ride along with a backward launch file (n_sort = 0: none)
struct KpNext {
    const int64_t *indices;
    int L, n_sort;
    KeptDev kd;
};

template <typename C>
__global__ __launch_bounds__(WG) __attribute__((amdgpu_waves_per_eu(C::R >= 64 ? 2 : 3))) void bwd_kept_kernel(
    Params p, const float *__restrict__ G1, const float *__restrict__ G2, const float *__restrict__ G3, int L,
    const int64_t *__restrict__ offsets, int n_bags, const float *__restrict__ alpha,
    const float *__restrict__ grad_out, float *__restrict__ dG1, float *__restrict__ dG2, float *__restrict__ dG3,
    float lr, float *__restrict__ o1, float *__restrict__ o2, float *__restrict__ o3, KeptDev kd, CacheDev next_cache, KpNext nx)
{
    using F = KpCfg<C>;
    constexpr int N1 = C::N1, N2 = C::N2, N3 = C::N3, R = C::R, V = C::V, N = C::N, RQ = C::RQ;
    constexpr int W = F::W, NQ = N / 4, SB = F::SB, SMALL = F::SMALL, TB0 = F::TB0;
    constexpr int PA = C::sA / 4, PC = C::sC / 4;
    static_assert(offsetof(KpLds<C>, small) == sizeof(float) * W * N, "small[] must follow stage[]");
    if ((int)blockIdx.x >= kd.nbins) {                                       // uniform: a sorter of the next batch
        kept_sort_body(kp_sort_lds(kp_dyn_lds, nx.kd.nbins), p, (int)blockIdx.x - kd.nbins, nx.indices, nx.L, next_cache, nx.kd);
        return;
    }
    KpLds<C> &lds = *reinterpret_cast<KpLds<C> *>(kp_dyn_lds);
    float *stage = lds.stage;
    const bool fused = o1 != nullptr;
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int a0 = w * RQ;
    const bool active = lane < C::LANES;
    const int c0 = active ? lane * V : 0;
    const int j2 = c0 / R, b0 = c0 % R;

    // role and slice of this workgroup, without branches so that all kernel arguments load together
    const int bin = blockIdx.x;
    const int ge1 = bin >= p.m1, ge2 = bin >= p.m1 + p.m2;
    const int ROLE = ge1 + ge2;
    const int s = bin - (ge1 ? p.m1 : 0) - (ge2 ? p.m2 : 0);

    // the fixed-place part of the list: lane (g, i) holds entry i of sub-list g
    const int sg = lane >> kd.cshift, si = lane & (kd.capg - 1);
    const uint2 hd = kd.hdr[(size_t)bin * KP_MAXG + sg];
    const uint4 ent = kd.mainp[(size_t)bin * WAVE + lane];

    // Fused SGD step: every workgroup rewrites its slice; the old values are loaded now.
    constexpr int NACC2 = RQ * V, NACC3 = V * N3;
    constexpr int NACC1 = N1 * RQ;                                           // G1 owner: lane partials of its wave's rows a
    constexpr int KEEP1 = ReduceKeep<NACC1, WAVE>::value;
    constexpr int PF3 = (C::sC + WG - 1) / WG;
    constexpr int PFMAX = NACC2 > KEEP1 ? (NACC2 > PF3 ? NACC2 : PF3) : (KEEP1 > PF3 ? KEEP1 : PF3);
    float old[PFMAX];
    {
        const float *x1 = fused ? G1 : dG1, *x2 = fused ? G2 : dG2, *x3 = fused ? G3 : dG3;
        if (ROLE == 1) {
            const float *src = x2 + (size_t)s * C::sB + (size_t)a0 * C::COLS + c0;    // inactive lanes: c0 = 0, in range
#pragma unroll
            for (int aa = 0; aa < RQ; ++aa)
#pragma unroll
                for (int v = 0; v < V; ++v) old[aa * V + v] = src[aa * C::COLS + v];
        } else if (ROLE == 0) {
            const int base = reduce_base<NACC1, WAVE>(lane < ReduceKeep<NACC1, WAVE>::writers ? lane : 0);
#pragma unroll
            for (int i = 0; i < KEEP1; ++i) {
                const int idx = base + i;
                old[i] = x1[(size_t)s * C::sA + (idx / RQ) * R + a0 + idx % RQ];
            }
        } else {
#pragma unroll
            for (int i = 0; i < PF3; ++i) old[i] = x3[(size_t)s * C::sC + min(t + i * WG, C::sC - 1)];
        }
    }

    // accumulators: G1 owner N1 x RQ lane partials, G2 owner RQ x V elements, G3 owner V x N3 partials
    constexpr int NACC = NACC1 > NACC2 ? (NACC1 > NACC3 ? NACC1 : NACC3) : (NACC2 > NACC3 ? NACC2 : NACC3);
    float acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = 0.f;

    // ---- staging (as in fb_body): gather float4 items from global memory into LDS ----
    struct Item {
        float4 val;
        float scale;
        int dst, chk_k;
        int o0, o1;
    };
    auto grad_issue = [&](int k, int f, Item &r) __attribute__((always_inline)) {
        r.scale = alpha ? alpha[k] : 1.f;
        r.chk_k = -1;
        r.o0 = 0;
        r.o1 = 0;
        int row = k;
        if (offsets) {
            int gs = p.bagP ? (int)fast_div((uint32_t)k, p.bagP, p.mgP) : (int)((float)k * ((float)n_bags / (float)L));
            gs = gs < n_bags ? gs : n_bags - 1;
            const int *olo = reinterpret_cast<const int *>(offsets);      // little endian: low word first
            r.o0 = olo[2 * gs];
            r.o1 = olo[2 * gs + 2];
            r.chk_k = k;
            row = gs;
        }
        r.val = *reinterpret_cast<const float4 *>(grad_out + (size_t)row * N + 4 * f);
    };
    auto item_finish = [&](const Item &r) __attribute__((always_inline)) {
        float4 g = r.val;
        if (r.chk_k >= 0 && !(r.o0 <= r.chk_k && r.chk_k < r.o1)) {       // ragged bags
            const int bag = bag_of(offsets, n_bags, r.chk_k);
            g = *reinterpret_cast<const float4 *>(grad_out + (size_t)bag * N + 4 * ((r.dst / 4) % NQ));
        }
        g.x *= r.scale; g.y *= r.scale; g.z *= r.scale; g.w *= r.scale;
        return g;
    };
    // Items of a pass, up to IPT per thread, all loads in flight together: the gradients of entries [0, n_g / NQ)
    // of the window that starts at list entry i0, then (G2 owners) the G1 and G3 slices of runs [sb0, sb0 + nb).
    constexpr int IPT = 4;
    // `hook` runs after the loads of the first pass have been issued and before they are waited for: loads issued in it
    // return behind them and are not waited for here.
    auto stage_items = [&](int i0, int n_g, int sb0, int nb, auto &&hook) __attribute__((always_inline)) {
        const int n_a = ROLE == 1 ? nb * PA : 0;
        const int n_c = ROLE == 1 ? nb * PC : 0;
        const int total = n_g + n_a + n_c;
        for (int it0 = 0; it0 < total; it0 += IPT * WG) {                 // uniform
            Item r[IPT];
#pragma unroll
            for (int q = 0; q < IPT; ++q) {
                const int item = min(it0 + q * WG + t, total - 1);        // past the end: repeat the last item
                if (item < n_g) {
                    const int e = item / NQ, f = item % NQ;
                    grad_issue((int)lds.klist[i0 + e], f, r[q]);
                    r[q].dst = 4 * (NQ * lds.epos[e] + f);                // = stage[position * N + 4 f]
                } else {
                    const float *src;
                    if (item < n_g + n_a) {
                        const int x = item - n_g, u = x / PA, f = x % PA;
                        src = G1 + (size_t)lds.seg_i1[sb0 + u] * C::sA + 4 * f;
                        r[q].dst = W * N + u * SMALL + 4 * f;             // small[] follows stage[] in LDS
                    } else {
                        const int x = item - n_g - n_a, u = x / PC, f = x % PC;
                        src = G3 + (size_t)lds.seg_i3[sb0 + u] * C::sC + 4 * f;
                        r[q].dst = W * N + u * SMALL + C::sA + 4 * f;
                    }
                    r[q].scale = 1.f;
                    r[q].chk_k = -1;
                    r[q].o0 = 0;
                    r[q].o1 = 0;
                    r[q].val = *reinterpret_cast<const float4 *>(src);
                }
                if (it0 + (q + 1) * WG >= total) break;                   // uniform: the pass ends here
            }
            if (it0 == 0) hook();
#pragma unroll
            for (int q = 0; q < IPT; ++q) {
                if (it0 + q * WG >= total) break;                         // uniform
                const float4 g = item_finish(r[q]);
                if (it0 + q * WG + t < total) *reinterpret_cast<float4 *>(&stage[r[q].dst]) = g;
            }
        }
    };

    constexpr int ACH = RQ % 4 == 0 ? 4 : RQ;
    auto load_a = [&](const float *src, float (&ax)[ACH]) __attribute__((always_inline)) {
        if constexpr (ACH == 4) {
            const float4 av = *reinterpret_cast<const float4 *>(src);
            ax[0] = av.x; ax[1] = av.y; ax[2] = av.z; ax[3] = av.w;
        } else {
#pragma unroll
            for (int aa = 0; aa < ACH; ++aa) ax[aa] = src[aa];
        }
    };
    // G2 owner, the runs [sb0, sb0 + nb) whose G1 and G3 slices sit in small[]: dT0'[j1][c] = sum_j3 dY[(j1,j2)][j3] C[b][j3]
    // (every wave for its own columns: cheaper than sharing it through LDS and a barrier), then
    // dG2[a][c] += sum_j1 A[j1][a] dT0'[j1][c] for the wave's rows a.  Two runs at a time, their LDS reads in flight together.
    auto consume_g2 = [&](int sb0, int nb) __attribute__((always_inline)) {
        constexpr int UH = 2;                                              // (as many as the registers allow)
        for (int u0 = 0; u0 < nb; u0 += UH) {                              // uniform
            float4 q4[UH][N1], cv[UH][V];
            const float *sm[UH];
            float keep[UH];
#pragma unroll
            for (int u = 0; u < UH; ++u) {
                const int uu = min(u0 + u, nb - 1);                        // past the end: the last run again, weight 0
                keep[u] = u0 + u < nb ? 1.f : 0.f;
                sm[u] = lds.small + uu * SMALL;
                const float *dy = stage + lds.seg_start[sb0 + uu] * N + j2 * N3;
#pragma unroll
                for (int j1 = 0; j1 < N1; ++j1) q4[u][j1] = *reinterpret_cast<const float4 *>(dy + j1 * N2 * N3);
#pragma unroll
                for (int v = 0; v < V; ++v) cv[u][v] = *reinterpret_cast<const float4 *>(&sm[u][C::sA + (b0 + v) * N3]);
            }
#pragma unroll
            for (int j1 = 0; j1 < N1; ++j1) {
                float ax[UH][RQ / ACH][ACH];
#pragma unroll
                for (int u = 0; u < UH; ++u)
#pragma unroll
                    for (int a4 = 0; a4 < RQ / ACH; ++a4) load_a(&sm[u][j1 * R + a0 + a4 * ACH], ax[u][a4]);
#pragma unroll
                for (int u = 0; u < UH; ++u)
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const float dt = keep[u] * fmaf(q4[u][j1].x, cv[u][v].x, fmaf(q4[u][j1].y, cv[u][v].y,
                                                   fmaf(q4[u][j1].z, cv[u][v].z, q4[u][j1].w * cv[u][v].w)));
#pragma unroll
                        for (int a4 = 0; a4 < RQ / ACH; ++a4)
#pragma unroll
                            for (int q = 0; q < ACH; ++q)
                                acc[(a4 * ACH + q) * V + v] = fmaf(ax[u][a4][q], dt, acc[(a4 * ACH + q) * V + v]);
                    }
            }
        }
    };
    // G1 and G3 owners: the operands of a batch of runs are loaded by ops_issue and used by ops_use, so that the first batch
    // can be in flight while the upstream gradients are staged.
    //   G3 owner: dG3[b][j3]  += sum_{(j1,j2)} T0[(j1,j2)][b] dY[(j1,j2)][j3] with the T0 that the forward pass kept (of the
    //             run's first position); lane = columns c = (j2, b); wave w takes the runs w, w + 4, ..., TB at a time.
    //   G1 owner: dG1[j1][a] += sum_c dT0'[j1][c] Bm[a][c], dT0'[j1][c] = sum_j3 dY[(j1,j2)][j3] C[b][j3]: all waves take the
    //             same runs, TB0 at a time; wave w streams the rows a in [w RQ, (w+1) RQ) of Bm = G2[i2] through registers,
    //             lane = columns c; the sum over c stays a lane partial until the end.
    constexpr int TB = 4;
    constexpr int PF0 = TB0 * (RQ * V + V * N3), PF2 = TB * N1 * V;
    constexpr int PFN = PF0 > PF2 ? PF0 : PF2;
    auto ops_issue = [&](int sg0, int nsegs, float (&pf)[PFN]) __attribute__((always_inline)) {
        if (ROLE == 0) {
            int i2q[TB0], i3q[TB0];
#pragma unroll
            for (int q = 0; q < TB0; ++q) {                                 // past the end: the last run again, not used
                i2q[q] = lds.seg_i2[min(sg0 + q, nsegs - 1)];
                i3q[q] = lds.seg_i3[min(sg0 + q, nsegs - 1)];
            }
#pragma unroll
            for (int q = 0; q < TB0; ++q) {
                const float *B = G2 + (size_t)__builtin_amdgcn_readfirstlane(i2q[q]) * C::sB + (size_t)a0 * C::COLS + c0;
                const float *Cp = G3 + (size_t)__builtin_amdgcn_readfirstlane(i3q[q]) * C::sC + b0 * N3;
#pragma unroll
                for (int aa = 0; aa < RQ; ++aa) {
                    float tmp[V];
                    load_vec<V>(B + aa * C::COLS, tmp);
#pragma unroll
                    for (int v = 0; v < V; ++v) pf[(q * RQ + aa) * V + v] = tmp[v];
                }
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const float4 cv = *reinterpret_cast<const float4 *>(Cp + v * N3);
                    float *d = &pf[TB0 * RQ * V + (q * V + v) * N3];
                    d[0] = cv.x; d[1] = cv.y; d[2] = cv.z; d[3] = cv.w;
                }
            }
        } else {
            size_t kq[TB];
#pragma unroll
            for (int q = 0; q < TB; ++q) kq[q] = lds.seg_k[min(sg0 + q * NWAVE, nsegs - 1)];
#pragma unroll
            for (int q = 0; q < TB; ++q)
#pragma unroll
                for (int j1 = 0; j1 < N1; ++j1) {
                    float tmp[V];
                    load_vec<V>(kd.t0 + kq[q] * (N1 * C::COLS) + c0 + j1 * C::COLS, tmp);
#pragma unroll
                    for (int v = 0; v < V; ++v) pf[(q * N1 + j1) * V + v] = tmp[v];
                }
        }
    };
    auto ops_use = [&](int sg0, int nsegs, const float (&pf)[PFN]) __attribute__((always_inline)) {
        if (ROLE == 0) {
            float4 g[TB0][N1];
            float keep[TB0];
#pragma unroll
            for (int q = 0; q < TB0; ++q) {
                const float *dy = stage + lds.seg_start[min(sg0 + q, nsegs - 1)] * N + j2 * N3;
                keep[q] = sg0 + q < nsegs ? 1.f : 0.f;
#pragma unroll
                for (int j1 = 0; j1 < N1; ++j1) g[q][j1] = *reinterpret_cast<const float4 *>(dy + j1 * N2 * N3);
            }
#pragma unroll
            for (int q = 0; q < TB0; ++q)
#pragma unroll
                for (int j1 = 0; j1 < N1; ++j1)
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const float *cv = &pf[TB0 * RQ * V + (q * V + v) * N3];
                        const float dt = keep[q] * fmaf(g[q][j1].x, cv[0], fmaf(g[q][j1].y, cv[1], fmaf(g[q][j1].z, cv[2], g[q][j1].w * cv[3])));
#pragma unroll
                        for (int aa = 0; aa < RQ; ++aa) acc[j1 * RQ + aa] = fmaf(dt, pf[(q * RQ + aa) * V + v], acc[j1 * RQ + aa]);
                    }
        } else {
            const float *dy[TB];
            float keep[TB];
#pragma unroll
            for (int q = 0; q < TB; ++q) {
                dy[q] = stage + lds.seg_start[min(sg0 + q * NWAVE, nsegs - 1)] * N;
                keep[q] = sg0 + q * NWAVE < nsegs ? 1.f : 0.f;
            }
            float4 g[TB][N1];
#pragma unroll
            for (int q = 0; q < TB; ++q)
#pragma unroll
                for (int j1 = 0; j1 < N1; ++j1) g[q][j1] = *reinterpret_cast<const float4 *>(dy[q] + j2 * N3 + j1 * N2 * N3);
#pragma unroll
            for (int q = 0; q < TB; ++q)
#pragma unroll
                for (int j1 = 0; j1 < N1; ++j1)
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const float tk = pf[(q * N1 + j1) * V + v] * keep[q];
                        acc[v * N3 + 0] = fmaf(tk, g[q][j1].x, acc[v * N3 + 0]);
                        acc[v * N3 + 1] = fmaf(tk, g[q][j1].y, acc[v * N3 + 1]);
                        acc[v * N3 + 2] = fmaf(tk, g[q][j1].z, acc[v * N3 + 2]);
                        acc[v * N3 + 3] = fmaf(tk, g[q][j1].w, acc[v * N3 + 3]);
                    }
        }
    };

    // One window: nw entries (lds.klist[i0 ..], staged positions lds.epos[], runs in lds.seg_*[0 .. nsegs)).
    auto window = [&](int i0, int nw, int nsegs) __attribute__((always_inline)) {
        float pf[PFN];
        stage_items(i0, nw * NQ, 0, min(SB, nsegs), [&]() __attribute__((always_inline)) {
            if (ROLE == 0 || (ROLE == 2 && w < nsegs)) ops_issue(ROLE == 0 ? 0 : w, nsegs, pf);   // in flight behind the gradients
        });
        __syncthreads();
        if (nsegs < nw) {                                                  // uniform: some row occurs more than once
            // Every run is summed into its first entry; items (run, column) touch disjoint floats.  Runs of up to
            // LONGRUN entries: one thread per item, the entries in list order, eight loads in flight.  Longer
            // runs (a hot row), one after the other: thread (part q, float4 f) adds every (WG / NQ)-th entry, the
            // parts are added within the wave by a fixed butterfly and across the waves through LDS.
            constexpr int LONGRUN = 16;
            static_assert(WG % NQ == 0 && WAVE % NQ == 0, "float4 columns divide a wave");
            for (int item = t; item < nsegs * N; item += WG) {
                const int sgq = item / N, j = item % N;
                const int e0 = lds.seg_start[sgq], e1 = lds.seg_start[sgq + 1];
                if (e1 - e0 > 1 && e1 - e0 <= LONGRUN) {
                    float x[LONGRUN];
#pragma unroll
                    for (int q = 0; q < LONGRUN; ++q) x[q] = stage[min(e0 + q, e1 - 1) * N + j];
                    float sum = x[0];
#pragma unroll
                    for (int q = 1; q < LONGRUN; ++q) sum += e0 + q < e1 ? x[q] : 0.f;
                    stage[e0 * N + j] = sum;
                }
            }
            if (nw > LONGRUN) {                                            // uniform
                // Wave w sums the long runs number w, w + 4, ... on its own (they are disjoint from the short runs above): lane
                // (part q of WAVE / NQ, float4 f) adds every (WAVE / NQ)-th entry, four loads in flight, then a fixed butterfly
                // over the parts.  The runs' bounds are read into the lanes once; a ballot finds the long ones.
                constexpr int WP = WAVE / NQ;
                int nlong = 0;
                for (int r0 = 0; r0 < nsegs; r0 += WAVE) {                 // uniform
                    const int r = r0 + lane;
                    const int s0 = r < nsegs ? lds.seg_start[r] : 0, s1 = r < nsegs ? lds.seg_start[r + 1] : 0;
                    uint64_t lm = __ballot(s1 - s0 > LONGRUN);
                    while (lm) {                                           // uniform
                        const int jl = __builtin_ctzll(lm);
                        lm &= lm - 1;
                        if ((nlong++ & (NWAVE - 1)) != w) continue;        // uniform per wave
                        const int e0 = __builtin_amdgcn_readlane(s0, jl), e1 = __builtin_amdgcn_readlane(s1, jl);
                        const int f = lane % NQ, q = lane / NQ;
                        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
                        for (int e = e0 + q; e < e1; e += 4 * WP) {
                            float4 x[4];
#pragma unroll
                            for (int i = 0; i < 4; ++i) x[i] = *reinterpret_cast<const float4 *>(&stage[min(e + i * WP, e1 - 1) * N + 4 * f]);
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (e + i * WP < e1) { sum.x += x[i].x; sum.y += x[i].y; sum.z += x[i].z; sum.w += x[i].w; }
                        }
#pragma unroll
                        for (int d = NQ; d < WAVE; d <<= 1) {
                            sum.x += __shfl_xor(sum.x, d); sum.y += __shfl_xor(sum.y, d);
                            sum.z += __shfl_xor(sum.z, d); sum.w += __shfl_xor(sum.w, d);
                        }
                        if (lane < NQ) *reinterpret_cast<float4 *>(&stage[e0 * N + 4 * lane]) = sum;
                    }
                }
            }
            __syncthreads();
        }
        if (ROLE == 0) {
            for (int sg0 = 0; sg0 < nsegs; sg0 += TB0) {                   // uniform
                if (sg0 > 0) ops_issue(sg0, nsegs, pf);
                ops_use(sg0, nsegs, pf);
            }
        } else if (ROLE == 2) {
            for (int sg0 = w; sg0 < nsegs; sg0 += NWAVE * TB) {            // uniform per wave
                if (sg0 > w) ops_issue(sg0, nsegs, pf);
                ops_use(sg0, nsegs, pf);
            }
        } else {
            for (int sb0 = 0; sb0 < nsegs; sb0 += SB) {                    // uniform
                const int nb = min(SB, nsegs - sb0);
                if (sb0 > 0) {
                    __syncthreads();
                    stage_items(i0, 0, sb0, nb, []() {});
                    __syncthreads();
                }
                consume_g2(sb0, nb);
            }
        }
        __syncthreads();                                                   // before the LDS lists are reused
    };

    // ---- the list of this slice ----
    const int ng = sg < kd.G ? (int)hd.x : 0;
    const uint64_t lt = lanemask_lt();
    const bool longlist = __ballot(ng > kd.capg) != 0ull;
    const bool anyentry = __ballot(ng > 0) != 0ull;
    if (anyentry && !longlist) {
        // Short list (the usual case): all of it sits at the fixed places, lane order is position order.  Every wave
        // analyses it by itself, in registers; no barrier.  ent.y = place in its sub-list of the first entry with the
        // same row: the runs of equal rows without comparing rows.
        const bool valid = si < ng;
        const uint64_t vm = __ballot(valid);
        const int n = __popcll(vm), e = __popcll(vm & lt);                 // this lane's entry is entry e of the list
        const bool head = valid && (int)ent.y == si;
        const int hl = lane - si + (int)ent.y;                             // lane of the first entry of my run
        const uint64_t hm = __ballot(head);
        const int nsegs = __popcll(hm);
        const int runidx = __popcll(hm & ((1ull << (hl & 63)) - 1ull));    // number of the run = heads before its head
        int extra = 0, rin = 0;
        uint64_t rem = __ballot(valid && !head);
        while (rem) {                                                      // uniform: one step per run of more than one entry
            const int jl = __builtin_ctzll(rem);
            const int h = __builtin_amdgcn_readlane(hl, jl);
            const uint64_t m = __ballot(valid && hl == h);
            const int hidx = __popcll(hm & ((1ull << h) - 1ull));
            if (valid && hl == h) rin = __popcll(m & lt);
            if (runidx > hidx) extra += __popcll(m) - 1;
            rem &= ~m;
        }
        if (valid) {
            lds.klist[e] = ent.x;
            lds.epos[e] = runidx + extra + rin;
        }
        if (head) {
            int i1, i2, i3;
            decode(p, ent.z, i1, i2, i3);
            lds.seg_start[runidx] = runidx + extra;
            lds.seg_i1[runidx] = i1;
            lds.seg_i2[runidx] = i2;
            lds.seg_i3[runidx] = i3;
            lds.seg_k[runidx] = ent.x;
        }
        if (lane == 0) lds.seg_start[nsegs] = n;
        __builtin_amdgcn_wave_barrier();
        window(0, n, nsegs);
    } else if (anyentry) {
        // Long list (a hot row's slices): some sub-list continues in its sorter's overflow area.  The sub-lists one after
        // the other are the list in position order; the workgroup goes through it in rounds of FB_CAP entries,
        // windows of W, pieces of 64 (one wave each; runs found by comparing rows).
        const int ngroups = WAVE >> kd.cshift;
        int ntot = 0;
        for (int g = 0; g < ngroups; ++g) ntot += __builtin_amdgcn_readlane(ng, g << kd.cshift);   // uniform
        for (int r0 = 0; r0 < ntot; r0 += FB_CAP) {                        // uniform
            const int nr = min(FB_CAP, ntot - r0);
            {
                constexpr int NL = FB_CAP / WG;
                uint4 ev[NL];
                // entry i of the list lies in the last sub-list whose first entry is at or before i
                int ii[NL], gsel[NL], gbase[NL], gov[NL];
#pragma unroll
                for (int q = 0; q < NL; ++q) {
                    ii[q] = r0 + min(q * WG + t, nr - 1);                  // (clamped: no load is conditional)
                    gsel[q] = 0; gbase[q] = 0; gov[q] = 0;
                }
                int run = 0;
                for (int g = 0; g < ngroups; ++g) {                        // uniform
                    const int n_g = __builtin_amdgcn_readlane(ng, g << kd.cshift);
                    const int ov_g = __builtin_amdgcn_readlane((int)hd.y, g << kd.cshift);
#pragma unroll
                    for (int q = 0; q < NL; ++q) {
                        const bool in = run <= ii[q];
                        gsel[q] = in ? g : gsel[q];
                        gbase[q] = in ? run : gbase[q];
                        gov[q] = in ? ov_g : gov[q];
                    }
                    run += n_g;
                }
#pragma unroll
                for (int q = 0; q < NL; ++q) {
                    const int j = ii[q] - gbase[q];
                    ev[q] = j < kd.capg ? kd.mainp[(size_t)bin * WAVE + (gsel[q] << kd.cshift) + j]
                                        : kd.ov[(size_t)gsel[q] * KP_OV + gov[q] + j - kd.capg];
                }
#pragma unroll
                for (int q = 0; q < NL; ++q)
                    if (q * WG + t < nr) { lds.klist[q * WG + t] = ev[q].x; lds.rows[q * WG + t] = ev[q].z; }
            }
            __syncthreads();
            for (int i0 = 0; i0 < nr; i0 += W) {                           // uniform
                const int nw = min(W, nr - i0);
                // wave w analyses the pieces w, w + 4, ... of the window, one after the other (W / 64 pieces)
                int nsegs = 0;
                for (int pc0 = 0; pc0 < (nw + WAVE - 1) / WAVE; pc0 += NWAVE) {   // uniform
                    const int pc = pc0 + w;
                    const int len = min(WAVE, nw - pc * WAVE);             // <= 0: no piece for this wave
                    const uint32_t my = lane < len ? lds.rows[i0 + pc * WAVE + lane] : KP_NONE;
                    const uint32_t myk = lane < len ? lds.klist[i0 + pc * WAVE + lane] : 0u;
                    uint64_t rem = __ballot(lane < len);
                    int pos = 0, cnt = 0, mysg = -1, mypos = 0;
                    while (rem) {                                          // uniform: one step per distinct row
                        const int jl = __builtin_ctzll(rem);
                        const uint32_t rj = (uint32_t)__builtin_amdgcn_readlane((int)my, jl);
                        const uint64_t m = __ballot(my == rj);
                        rem &= ~m;
                        if (my == rj) mypos = pos + __popcll(m & lt);
                        if (lane == jl) mysg = cnt;
                        pos += __popcll(m);
                        ++cnt;
                    }
                    if (lane == 0) lds.pcnt[w] = cnt;
                    __syncthreads();
                    int base = nsegs;
#pragma unroll
                    for (int jw = 0; jw < NWAVE; ++jw) {
                        const int c = lds.pcnt[jw];
                        if (jw < w) base += c;
                        nsegs += c;
                    }
                    if (lane < len) lds.epos[pc * WAVE + lane] = pc * WAVE + mypos;
                    if (mysg >= 0) {
                        int i1, i2, i3;
                        decode(p, my, i1, i2, i3);
                        lds.seg_start[base + mysg] = pc * WAVE + mypos;
                        lds.seg_i1[base + mysg] = i1;
                        lds.seg_i2[base + mysg] = i2;
                        lds.seg_i3[base + mysg] = i3;
                        lds.seg_k[base + mysg] = myk;
                    }
                    __syncthreads();                                       // pcnt is reused by the next group of pieces
                }
                if (t == 0) lds.seg_start[nsegs] = nw;
                __syncthreads();
                window(i0, nw, nsegs);
            }
        }
    }
    if (!anyentry && !fused) return;                                       // nothing to add

    // ---- last phase: the slice gradient is added to dG (old = dG) or the slice after its SGD step is written (old = G) ----
    const float mul = fused ? -lr : 1.f;
    if (ROLE == 1) {
        if (active) {
            float *dst = (fused ? o2 : dG2) + (size_t)s * C::sB + (size_t)a0 * C::COLS + c0;
#pragma unroll
            for (int aa = 0; aa < RQ; ++aa)
#pragma unroll
                for (int v = 0; v < V; ++v) dst[aa * C::COLS + v] = fmaf(mul, acc[aa * V + v], old[aa * V + v]);
        }
    } else if (ROLE == 0) {
        float red[NACC1];
#pragma unroll
        for (int i = 0; i < NACC1; ++i) red[i] = active ? acc[i] : 0.f;
        group_reduce<NACC1, WAVE>(red, lane);
        if (lane < ReduceKeep<NACC1, WAVE>::writers) {
            const int base = reduce_base<NACC1, WAVE>(lane);
#pragma unroll
            for (int i = 0; i < KEEP1; ++i) {
                const int idx = base + i;                                  // = j1 * RQ + aa
                (fused ? o1 : dG1)[(size_t)s * C::sA + (idx / RQ) * R + a0 + idx % RQ] = fmaf(mul, red[i], old[i]);
            }
        }
    } else {
        float *part = lds.stage;                                           // [wave][column][j3]
        if (active) {
#pragma unroll
            for (int v = 0; v < V; ++v)
#pragma unroll
                for (int j3 = 0; j3 < N3; ++j3) part[(w * C::COLS + c0 + v) * N3 + j3] = acc[v * N3 + j3];
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PF3; ++i) {
            const int e = t + i * WG;
            if (e < C::sC) {
                const int b = e / N3, j3 = e - b * N3;
                float sum = 0.f;
#pragma unroll
                for (int ww = 0; ww < NWAVE; ++ww)
#pragma unroll
                    for (int jj = 0; jj < N2; ++jj) sum += part[(ww * C::COLS + jj * R + b) * N3 + j3];
                (fused ? o3 : dG3)[(size_t)s * C::sC + e] = fmaf(mul, sum, old[i]);
            }
        }
    }
}

// ---- test export: what the lists say about every position --------------------------------------------------
// For role r (0..2) and every position k: slice[r][k] = the slice of core r+1 whose list holds k, rep[r][k] = the rep of
// that entry, times[r][k] = in how many lists of that core k was found (1, or 0 for a cached position).
__global__ __launch_bounds__(WG) void kept_lists_export_kernel(Params p, KeptDev kd, int L, int32_t *__restrict__ slice,
                                                               int32_t *__restrict__ rep, int32_t *__restrict__ times)
{
    const int bin = blockIdx.x, t = threadIdx.x;
    const int ge1 = bin >= p.m1, ge2 = bin >= p.m1 + p.m2;
    const int role = ge1 + ge2, s = bin - (ge1 ? p.m1 : 0) - (ge2 ? p.m2 : 0);
    auto entry = [&](int g, const uint2 &hd, int i) {
        return i < kd.capg ? kd.mainp[(size_t)bin * WAVE + g * kd.capg + i] : kd.ov[(size_t)g * KP_OV + hd.y + i - kd.capg];
    };
    for (int g = 0; g < kd.G; ++g) {
        const uint2 hd = kd.hdr[(size_t)bin * KP_MAXG + g];
        for (int i = t; i < (int)hd.x; i += WG) {
            const uint4 e = entry(g, hd, i);
            if (e.x < (uint32_t)L) {
                slice[(size_t)role * L + e.x] = s;
                rep[(size_t)role * L + e.x] = e.y < hd.x ? (int32_t)entry(g, hd, (int)e.y).x : -2;   // position of the run's first entry
                atomicAdd(&times[(size_t)role * L + e.x], 1);
            }
        }
    }
}

static inline void kept_sort(const Params &p, const int64_t *idx, int L, const CacheDev &cd, const KeptDev &kd, hipStream_t st)
{
    hipLaunchKernelGGL(kept_sort_kernel, dim3(kd.G), dim3(WG), kp_sort_lds_bytes(kd.nbins), st, p, idx, L, cd, kd);
}

// ---- launchers -----------------------------------------------------------------------------------------

template <typename C>
static inline void launch_bwd_kept(const Params &p, const float *G1, const float *G2, const float *G3, int L, const int64_t *off,
                                   int n_bags, const float *alpha, const float *go, float *dG1, float *dG2, float *dG3, float lr,
                                   float *o1, float *o2, float *o3, const KeptDev &kd, const CacheDev &next_cache,
                                   const KpNext &nx, hipStream_t st)
{
    const size_t own = sizeof(KpLds<C>), srt = nx.n_sort ? kp_sort_lds_bytes(nx.kd.nbins) : 0;
    hipLaunchKernelGGL(bwd_kept_kernel<C>, dim3(kd.nbins + nx.n_sort), dim3(WG), own > srt ? own : srt, st, p, G1, G2, G3, L, off,
                       n_bags, alpha, go, dG1, dG2, dG3, lr, o1, o2, o3, kd, next_cache, nx);
}

static inline void kept_bwd(const Params &p, const float *G1, const float *G2, const float *G3, int L, const int64_t *off,
                            int n_bags, const float *alpha, const float *go, float *dG1, float *dG2, float *dG3, float lr,
                            float *o1, float *o2, float *o3, const KeptDev &kd, const CacheDev &next_cache, const KpNext &nx,
                            hipStream_t st)
{
    switch (fast_config(p)) {
    case 0: launch_bwd_kept<Cfg224R8>(p, G1, G2, G3, L, off, n_bags, alpha, go, dG1, dG2, dG3, lr, o1, o2, o3, kd, next_cache, nx, st); break;
    case 1: launch_bwd_kept<Cfg224R16>(p, G1, G2, G3, L, off, n_bags, alpha, go, dG1, dG2, dG3, lr, o1, o2, o3, kd, next_cache, nx, st); break;
    case 2: launch_bwd_kept<Cfg224R32>(p, G1, G2, G3, L, off, n_bags, alpha, go, dG1, dG2, dG3, lr, o1, o2, o3, kd, next_cache, nx, st); break;
    default: break;
    }
}

}  // namespace tt
