// Specialised backward kernel (Eq. 4 / Alg. 2 of the paper) for the shapes of tt_fast.h.
//
// One workgroup owns one core slice: workgroups [0, m1) own G1[s], the next m2 own G2[s],
// the last m3 own G3[s].  The owner
//   1. scans the index array and keeps, in order, the positions whose digit selects its
//      slice (ballots; every wave appends to its own sub-list, no atomics),
//   2. finds the runs of equal rows in pieces of 64 entries, lane e holding entry e, with one
//      ballot per distinct row, and lays the runs out one after the other (a row that shows up
//      in two pieces is simply handled twice: the gradient is linear in dY),
//   3. stages alpha_k * grad_out[bag(k)] of every entry in LDS at its position in that layout
//      and sums each run into its first entry: one dY per distinct row,
//   4. stages the small operands of every distinct row (its G1 and/or G3 slice) in LDS, all
//      loads in flight together, and streams the large one (the G2 slice, for the G1 and G3
//      owners) through registers several rows at a time,
//   5. accumulates its slice gradient in registers and either adds it to grad_cores once or
//      writes the slice after its SGD step to a second set of cores.
// All four waves walk over the same rows; wave w owns rows a in [w RQ, (w+1) RQ) of the
// unfolded G2 slice (R x n2 R), lane l owns columns c0 .. c0+V-1:
//   G2 owner: dG2[a][c]  += sum_j1 A[j1][a] dT0'[j1][c]              (reads no G2 at all)
//   G1 owner: dG1[j1][a] += sum_c dT0'[j1][c] Bm[a][c]              (lane partials, reduced once at the end)
//   G3 owner: dG3[b][j3] += sum_{j1,j2} T0[(j1,j2)][b] dY[(j1,j2)][j3], T0 partial over the wave's rows a
// with dT0'[j1][c] = sum_j3 dY[(j1,j2)][j3] C[b][j3].  Everything is summed in a fixed order.
//
// The kernel is bound by instruction and memory latency, not by bandwidth: the code keeps the
// dependent chain short (kernel arguments -> indices -> operands -> result), issues the loads
// of a phase together, avoids integer multiplies, and keeps the role a run-time value so that
// the three owners share one copy of the code in the instruction cache.
//
// The (4,4,4) shapes (lists of hundreds of entries, rows that cost 16-64 KB of G2 each) differ:
// the owners are separate copies of the body, the G2 owner works on the matrix cores in batches
// of rows and, after the grouping pre-pass, also produces the G1 gradient of every row
// (g1_from_p_kernel then finishes the G1 slices), long lists are shared by several workgroups
// whose partial slice gradients bwd_split_finish_kernel adds up, and the cached-row reduction
// of tt_group.h runs as extra workgroups of these launches.  See FbSplit and the comment above
// consume_g2_mfma.
#pragma once

#include <stddef.h>

#include "tt_fast.h"
#include "tt_group.h"

namespace tt {

constexpr int FB_CAP = 512;                 // list entries a workgroup handles at once
constexpr int FB_SCAN = 2048;               // positions scanned per round
constexpr int FB_ITER = FB_SCAN / WG;       // positions per lane and round
constexpr int FB_PIECE = WAVE;              // entries sorted together
constexpr int FB_WCAP = FB_CAP / NWAVE;     // entries one wave may select per round
constexpr uint32_t FB_NONE = 0xFFFFFFFFu;


typedef float mfma16_t __attribute__((ext_vector_type(16)));
typedef float mfma4_t __attribute__((ext_vector_type(4)));

// *dst += x where no other thread touches *dst.  (An add performed by the memory system, without
// a returned value, was measured and is slower here than load, add, store.)
__device__ __forceinline__ void add_to(float *dst, float x) { *dst += x; }

// Several workgroups may share one slice (from 4096 positions on: the lists get long, and one hot row can
// fill a list): ns[r] workgroups per slice of core r, each takes one part of the positions and, where
// ns[r] > 1, stores its partial slice gradient at part[r] + (slice ns[r] + part) * slice size instead of
// finishing the slice; bwd_split_finish_kernel adds the parts up.
struct FbSplit {
    int ns[3];
    float *part[3];
    float *pbuf;        // (4,4,4) shapes: G1 gradient of every row, [L][n1 R], written by the G2 owners
    int *pflag;         // [L]: is this position the first of its row's run in its G2 owner's list
    GrpCacheWork cw;    // cached-row tiles that run as extra workgroups behind the n_owner slice owners
    int n_owner;
};

struct FbNoSplit {};                                        // kernel argument of the shapes that never split
template <bool SPLITS> struct FbSplitArg { typedef FbSplit type; };
template <> struct FbSplitArg<false> { typedef FbNoSplit type; };

// Part `part` of `nparts` of the positions (scan, gran = FB_CAP) or list entries (grouped, gran = 16)
// [lo, end), in whole pieces of `gran`.
__device__ __forceinline__ void fb_part_range(int part, int nparts, int gran, int &lo, int &end)
{
    if (nparts > 1) {
        const int per = (((end - lo + nparts - 1) / nparts + gran - 1) / gran) * gran;
        lo = min(end, lo + part * per);
        end = min(end, lo + per);
    }
}

template <typename C>
struct FbCfg {
    // sorted entries per window: 16 KB of upstream gradients; 32 KB for (4,4,4) at R = 64, whose kernel time is the
    // time of the longest lists and whose other LDS needs leave the room
    static constexpr int W = (C::N1 == 4 && C::R == 64 ? 8192 : 4096) / C::N;
    static constexpr int NB = (W + WAVE - 1) / WAVE;        // ballots that cover a window
    static constexpr int SB = 16;                           // distinct rows whose small operands sit in LDS
    static constexpr int SMALL = C::sA + C::sC;             // floats per row: G1 slice | G3 slice
    static constexpr int BMR = C::RQ * C::V;                // registers per row for the wave's part of G2[i2]
    // register budget: three workgroups per CU (one wave each per SIMD) for the small slices, fewer for the large
    static constexpr int WAVES_PER_SIMD = BMR <= 32 ? 3 : 2;
    // rows of G2 in flight per wave: up to 4, within 32 registers (8 rows / 64 registers was measured: slower,
    // the extra loads and the idle row slots of short lists cost more than the saved round trip)
    static constexpr int BUDGET = 32;
    static constexpr int UB = BUDGET / BMR >= 4 ? 4 : (BUDGET / BMR >= 1 ? BUDGET / BMR : 1);
    // (4,4,4) shapes: the G2 owner multiplies on the matrix cores, wave w owning the columns with j2 = w
    static constexpr bool MFMA = C::N1 == 4 && C::N2 == NWAVE && C::R % 32 == 0;
    // there the G2 owner works on batches of GB rows: dT0' of the batch as a 4 GB x n2 R matrix (odd row
    // stride: its columns are read as well as its rows)
    static constexpr int GB = 8;
    static constexpr int DTS = C::COLS + 1;
    static constexpr int SMALL_FLOATS = MFMA ? (4 * GB * DTS + 3) / 4 * 4 : 0;
    static_assert(W <= FB_CAP && (W % FB_PIECE == 0 || W < FB_PIECE), "windows hold whole pieces");
    static_assert(SB % UB == 0, "register batches must not straddle LDS batches");
};

template <typename C>
struct __align__(16) FbLds {
    float stage[FbCfg<C>::W * C::N];                        // alpha_k * grad_out[bag(k)] of the window's entries (16 KB)
    float small[FbCfg<C>::SMALL_FLOATS > FbCfg<C>::SB * FbCfg<C>::SMALL ? FbCfg<C>::SMALL_FLOATS
                                                                       : FbCfg<C>::SB * FbCfg<C>::SMALL];   // must follow stage[]: both are written through one index
    uint32_t rows[FB_CAP];                                  // selected row ids: four sub-lists, see fb_select
    uint32_t klist[FB_CAP];                                 // positions k of the selected entries
    int epos[FbCfg<C>::W];                                  // staged position of each entry of the window (runs contiguous)
    int seg_start[FbCfg<C>::W + 1];                         // staged position of the first entry of each run of equal rows
    int seg_i1[FbCfg<C>::W], seg_i2[FbCfg<C>::W], seg_i3[FbCfg<C>::W];   // its digits
    uint32_t seg_k[FbCfg<C>::W];                            // position k of the run's first entry (for the stored T0)
    int pcnt[NWAVE];                                        // runs per piece of a long window
    int wcnt[2][NWAVE];
};

// Row ids of the positions [lo, hi), hi - lo <= FB_SCAN, FB_ITER per lane: wave w covers a
// contiguous quarter.  Positions past hi, and cached positions (slot >= 0), give FB_NONE.
__device__ __forceinline__ void fb_load_rows(const int64_t *__restrict__ indices, const int32_t *__restrict__ slot,
                                             int lo, int hi, uint32_t (&rowv)[FB_ITER])
{
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int span = ((hi - lo + WG - 1) / WG) * WAVE;      // positions per wave
    const int wlo = lo + w * span;
#pragma unroll
    for (int it = 0; it < FB_ITER; ++it) {
        const int k = wlo + it * WAVE + lane;
        const bool ok = (it * WAVE < span) && (k < hi);
        rowv[it] = ok ? (uint32_t)indices[k] : FB_NONE;
    }
    if (slot) {
        // all loads first: the compiler would test each value where it is loaded, one round trip per value
        // (the empty asm statements keep the eight loads ahead of the eight tests)
        int32_t sl[FB_ITER];
#pragma unroll
        for (int it = 0; it < FB_ITER; ++it) {
            const int k = wlo + it * WAVE + lane;
            const bool ok = (it * WAVE < span) && (k < hi);
            sl[it] = ok ? slot[k] : -1;
        }
#pragma unroll
        for (int it = 0; it < FB_ITER; ++it) asm volatile("" : "+v"(sl[it]));
#pragma unroll
        for (int it = 0; it < FB_ITER; ++it)
            if (sl[it] >= 0) rowv[it] = FB_NONE;
    }
}

// Stable selection of the positions in [lo, hi) (rows in rowv, see fb_load_rows) that select
// slice s of the role's core.  Wave w appends its matches, in order, to its own sub-list
// lds.klist / lds.rows [w * FB_WCAP ...), which already holds fill[w] entries of earlier rounds:
// the list of the workgroup is the concatenation of the four sub-lists (fb_slot), so one barrier
// is enough.  wc[] receives the number of matches of every wave in this round.  If one of the
// sub-lists would overflow, the entries written are to be ignored (they lie behind fill[]).
// `round` alternates the counters between calls.
template <typename C>
__device__ __forceinline__ int fb_select(FbLds<C> &lds, const Params &p, int role, int s,
                                         const uint32_t (&rowv)[FB_ITER], int lo, int hi, int round,
                                         const int (&fill)[NWAVE], int (&wc)[NWAVE]
                                         )
{
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int span = ((hi - lo + WG - 1) / WG) * WAVE;      // positions per wave
    const int wlo = lo + w * span;
    // Which rows select slice s?  Role 0 (digit i1): a contiguous range of rows, clamped to the
    // 31-bit row space.  Role 2 (i3) and role 1 (i2): the digit from the multiply-free fp64 decode.
    uint64_t masks[FB_ITER];
    int cnt = 0;
    if (role == 0) {
        const RowRange rr = rows_of_i1(p, s);
#pragma unroll
        for (int it = 0; it < FB_ITER; ++it) {
            const bool hit = rowv[it] != FB_NONE && in_rows(rr, rowv[it]);
            masks[it] = __ballot(hit);
            cnt += __popcll(masks[it]);
        }
    } else {
        const double sd = (double)s;
#pragma unroll
        for (int it = 0; it < FB_ITER; ++it) {
            const bool hit = rowv[it] != FB_NONE && select_digit_f64(p, role, (double)rowv[it]) == sd;
            masks[it] = __ballot(hit);
            cnt += __popcll(masks[it]);
        }
    }
    int myfill = 0;
#pragma unroll
    for (int j = 0; j < NWAVE; ++j) myfill = j == w ? fill[j] : myfill;
    if (cnt > 0 && myfill + cnt <= FB_WCAP) {                               // uniform in the wave
        const uint64_t lt = lanemask_lt();
        int off = w * FB_WCAP + myfill;
#pragma unroll
        for (int it = 0; it < FB_ITER; ++it) {
            if (masks[it] == 0) continue;                                   // uniform: most are empty
            if ((masks[it] >> lane) & 1ull) {
                const int pos = off + __popcll(masks[it] & lt);
                lds.klist[pos] = (uint32_t)(wlo + it * WAVE + lane);
                lds.rows[pos] = rowv[it];
            }
            off += __popcll(masks[it]);
        }
    }
    int *wcnt = lds.wcnt[round & 1];
    if (lane == 0) wcnt[w] = cnt;
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int j = 0; j < NWAVE; ++j) {
        wc[j] = wcnt[j];
        total += wc[j];
    }
    return total;
}

// LDS position of entry e of the workgroup's list, given the sub-list lengths (see fb_select)
__device__ __forceinline__ int fb_slot(const int (&wc)[NWAVE], int e)
{
    int sl = e, pre = 0;
#pragma unroll
    for (int j = 0; j + 1 < NWAVE; ++j) {
        pre += wc[j];
        if (e >= pre) sl = e - pre + (j + 1) * FB_WCAP;
    }
    return sl;
}

template <typename C>
__device__ __forceinline__ void fb_body(FbLds<C> &lds, const Params &p, const int ROLE, int s,
                                        const float *__restrict__ G1, const float *__restrict__ G2,
                                        const float *__restrict__ G3, const int64_t *__restrict__ indices, int L,
                                        const int64_t *__restrict__ offsets, int n_bags,
                                        const float *__restrict__ alpha, const int32_t *__restrict__ slot,
                                        const float *__restrict__ grad_out, float *__restrict__ dG1,
                                        float *__restrict__ dG2, float *__restrict__ dG3,
                                        const uint32_t *__restrict__ gvals, const int *__restrict__ goff,
                                        const int *__restrict__ gend, float lr, float *__restrict__ o1,
                                        float *__restrict__ o2, float *__restrict__ o3, const float *__restrict__ t0,
                                        uint32_t (&rowv)[FB_ITER], int part, int nparts, float *__restrict__ pout,
                                        float *__restrict__ pbuf, int *__restrict__ pflag, int rh)
{
    using F = FbCfg<C>;
    const bool t0mode = ROLE == 2 && t0 != nullptr;                    // the G3 owner uses the stored T0
    const bool needk = t0mode || (F::MFMA && ROLE == 1);               // the positions of the list entries are needed
    // Two ways to finish: add the slice gradient to dG1/dG2/dG3 (o1 == nullptr), or write the
    // slice after its SGD step, x - lr * gradient, to o1/o2/o3 (every slice is written then, also
    // one that no lookup touches).
    const bool fused = o1 != nullptr;
    constexpr int N1 = C::N1, N2 = C::N2, N3 = C::N3, R = C::R, V = C::V, N = C::N, RQ = C::RQ;
    constexpr bool MFMA = F::MFMA;
    constexpr int W = F::W, NQ = N / 4, SB = F::SB, UB = F::UB, SMALL = F::SMALL;
    // float4 of small operands per row: G1 slice (needed by the G2 and G3 owners) and G3 slice (G1, G2 owners)
    constexpr int PA = C::sA / 4, PC = C::sC / 4;
    static_assert((PA & (PA - 1)) == 0 && (PC & (PC - 1)) == 0 && (NQ & (NQ - 1)) == 0, "item counts must be powers of two");
    static_assert(offsetof(FbLds<C>, small) == sizeof(float) * W * N, "small[] must follow stage[]");

    float *stage = lds.stage;
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int a0 = w * RQ;
    const bool active = lane < C::LANES;
    const int c0 = active ? lane * V : 0;
    const int j2 = c0 / R, b0 = c0 % R;

    // accumulators: G1 owner N1*RQ lane partials, G2 owner RQ*V elements, G3 owner V*N3 partials
    constexpr int NACC1 = N1 * RQ, NACC2 = RQ * V, NACC3 = V * N3;
    // (on the matrix cores the G2 owner keeps its 32 x 32 result tiles in accm instead)
    constexpr int NACC = MFMA ? (NACC1 > NACC3 ? NACC1 : NACC3) : (NACC1 > NACC2 ? (NACC1 > NACC3 ? NACC1 : NACC3) : (NACC2 > NACC3 ? NACC2 : NACC3));
    float acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = 0.f;
    constexpr int NTILE = MFMA ? R / 32 : 1;                              // a G2 owner there has one row tile of 32 rows (rh)
    mfma16_t accm[NTILE];
#pragma unroll
    for (int i = 0; i < NTILE; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) accm[i][r] = 0.f;
    bool any = false;
    // Fused SGD step: every workgroup rewrites its slice, so the old values are loaded now and the
    // last phase does not wait for them (where that takes few registers).
    constexpr int KEEP1 = ReduceKeep<NACC1, WAVE>::value;
    constexpr int PF3 = (C::sC + WG - 1) / WG;
    constexpr int PFMAX = NACC2 > KEEP1 ? (NACC2 > PF3 ? NACC2 : PF3) : (KEEP1 > PF3 ? KEEP1 : PF3);
    constexpr bool PREFETCH = PFMAX <= 8;
    float old[PREFETCH ? PFMAX : 1];
    if (PREFETCH && fused && !pout) {
        if (ROLE == 1) {
            const float *src = G2 + (size_t)s * C::sB + (size_t)a0 * C::COLS + c0;    // inactive lanes: c0 = 0, in range
#pragma unroll
            for (int aa = 0; aa < RQ; ++aa)
#pragma unroll
                for (int v = 0; v < V; ++v) old[aa * V + v] = src[aa * C::COLS + v];
        } else if (ROLE == 0) {
            const int base = reduce_base<NACC1, WAVE>(lane < ReduceKeep<NACC1, WAVE>::writers ? lane : 0);
#pragma unroll
            for (int i = 0; i < KEEP1; ++i) {
                const int idx = base + i;
                old[i] = G1[(size_t)s * C::sA + (idx / RQ) * R + a0 + idx % RQ];
            }
        } else {
#pragma unroll
            for (int i = 0; i < PF3; ++i) old[i] = G3[(size_t)s * C::sC + min(t + i * WG, C::sC - 1)];
        }
    }

    // ---- staging: gather float4 items from global memory into LDS ----
    // One item in flight: its value, and for a gradient item what is needed to confirm the bag.
    struct Item {
        float4 val;
        float scale;
        int dst, chk_k;                                                   // dst = 4 (NQ position + f)
        int o0, o1;                                                       // offsets are < 2^31: the low words suffice
    };
    // float4 f of alpha_k * grad_out[bag(k)]: the bag is guessed (exact for fixed-length bags) and
    // its row is loaded while the two offsets that confirm the guess are in flight
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
        r.val = *reinterpret_cast<const float4 *>(grad_out + (uint32_t)row * (uint32_t)N + 4u * (uint32_t)f);
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
    // Item list of a pass, up to IPT items per thread, all loads of a pass in flight together: the
    // gradients of entries [0, n_g / NQ) of the window that starts at list entry i0 (entry e goes
    // to its staged position lds.epos[e]), then the G1 slices of rows [sb0, sb0 + nb) (unless the
    // G1 owner), then their G3 slices (unless the G3 owner).
    constexpr int IPT = N <= 16 ? 4 : (MFMA ? (R == 64 ? 8 : 4) : 2);           // (as many as the registers allow)
    auto stage_items = [&](int i0, int n_g, int sb0, int nb, const int (&wc)[NWAVE]) __attribute__((always_inline)) {
        const int n_a = ROLE != 0 ? nb * PA : 0;
        const int n_c = ROLE != 2 ? nb * PC : 0;
        const int total = n_g + n_a + n_c;
        for (int it0 = 0; it0 < total; it0 += IPT * WG) {                 // uniform
            Item r[IPT];
#pragma unroll
            for (int q = 0; q < IPT; ++q) {
                const int item = min(it0 + q * WG + t, total - 1);        // past the end: repeat the last item
                if (item < n_g) {
                    const int e = item / NQ, f = item % NQ;
                    grad_issue((int)lds.klist[fb_slot(wc, i0 + e)], f, r[q]);
                    r[q].dst = 4 * (NQ * lds.epos[e] + f);                // = stage[position * N + 4 f]
                } else {
                    const float *src;
                    if (item < n_g + n_a) {
                        const int x = item - n_g, u = x / PA, f = x % PA;
                        src = G1 + (uint32_t)lds.seg_i1[sb0 + u] * (uint32_t)C::sA + 4u * (uint32_t)f;
                        r[q].dst = W * N + u * SMALL + 4 * f;             // small[] follows stage[] in LDS
                    } else {
                        const int x = item - n_g - n_a, u = x / PC, f = x % PC;
                        src = G3 + (uint32_t)lds.seg_i3[sb0 + u] * (uint32_t)C::sC + 4u * (uint32_t)f;
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
#pragma unroll
            for (int q = 0; q < IPT; ++q) {
                if (it0 + q * WG >= total) break;                         // uniform
                const float4 g = item_finish(r[q]);
                if (it0 + q * WG + t < total) *reinterpret_cast<float4 *>(&stage[r[q].dst]) = g;
            }
        }
    };

    // this wave's rows of G2[i2] for rows [ub0, ub0 + UB) of the window -> registers
    auto bm_load = [&](int ub0, int nsegs, float (&bm)[UB][RQ][V]) __attribute__((always_inline)) {
        int i2v[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) i2v[u] = lds.seg_i2[min(ub0 + u, nsegs - 1)];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int i2 = __builtin_amdgcn_readfirstlane(i2v[u]);
            const float *B = G2 + (size_t)i2 * C::sB + (size_t)a0 * C::COLS + c0;
#pragma unroll
            for (int aa = 0; aa < RQ; ++aa) load_vec<V>(B + aa * C::COLS, bm[u][aa]);
        }
    };

    // ACH consecutive values of a row of A from LDS: four at a time where the wave's part of the row allows it
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

    // dT0'[j1][c] = sum_j3 dY[(j1,j2)][j3] C[b][j3] is the same in all four waves: where it is exactly as large
    // as the G3 slice it is made from (n1 n2 R = R n3), wave w computes it once for the rows w, w + 4, ... of
    // the batch of small operands and puts it in the place of that slice, which nobody needs afterwards.
    constexpr bool DTPRE = N1 * C::COLS == C::sC;
    auto load_lds_vec = [&](const float *src, float (&x)[V]) __attribute__((always_inline)) {
#pragma unroll
        for (int v = 0; v < V; ++v) x[v] = src[v];
    };
    auto dt_prepare = [&](int sb0, int nb) __attribute__((always_inline)) {
        if (!DTPRE || ROLE == 2) return;
        for (int u = w; u < nb; u += NWAVE) {                              // uniform per wave
            float *smu = lds.small + u * SMALL;
            const float *dy = stage + lds.seg_start[sb0 + u] * N + j2 * N3;
            float d[N1][V];
#pragma unroll
            for (int j1 = 0; j1 < N1; ++j1) {
                const float4 q = *reinterpret_cast<const float4 *>(dy + j1 * N2 * N3);
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const float4 cv = *reinterpret_cast<const float4 *>(&smu[C::sA + (b0 + v) * N3]);
                    d[j1][v] = fmaf(q.x, cv.x, fmaf(q.y, cv.y, fmaf(q.z, cv.z, q.w * cv.w)));
                }
            }
            // all lanes of the wave have read the slice before any of them overwrites it
            __builtin_amdgcn_wave_barrier();
            if (active) {
#pragma unroll
                for (int j1 = 0; j1 < N1; ++j1)
#pragma unroll
                    for (int v = 0; v < V; ++v) smu[C::sA + j1 * C::COLS + c0 + v] = d[j1][v];
            }
        }
        __syncthreads();
    };

    // Rows [ub0, ub0 + UB) of the window.  Every run has been summed into its first staged entry,
    // so each row reads exactly one dY.  No branches on the row count: rows past the end repeat
    // the last one with a zero weight, so the LDS reads of the batch can be in flight together.
    auto consume = [&](int ub0, int sb0, int nsegs, const float (&bm)[UB][RQ][V]) __attribute__((always_inline)) {
        constexpr int UH = UB < 4 ? UB : 4;                             // rows whose LDS reads are in flight together
#pragma unroll
        for (int h = 0; h < UB; h += UH) {
            const float *sm[UH];
            const float *dyp[UH];
            float keep[UH];
#pragma unroll
            for (int u = 0; u < UH; ++u) {
                const int sg = min(ub0 + h + u, nsegs - 1);
                keep[u] = ub0 + h + u < nsegs ? 1.f : 0.f;
                sm[u] = lds.small + (sg - sb0) * SMALL;
                dyp[u] = stage + lds.seg_start[sg] * N + j2 * N3;
            }
            if (ROLE == 2) {
                // T0 partial over this wave's rows a, then dG3 partial
                float t0[UH][N1][V];
#pragma unroll
                for (int u = 0; u < UH; ++u) {
#pragma unroll
                    for (int j1 = 0; j1 < N1; ++j1)
#pragma unroll
                        for (int v = 0; v < V; ++v) t0[u][j1][v] = 0.f;
#pragma unroll
                    for (int j1 = 0; j1 < N1; ++j1)
#pragma unroll
                        for (int a4 = 0; a4 < RQ; a4 += ACH) {
                            float ax[ACH];
                            load_a(&sm[u][j1 * R + a0 + a4], ax);
#pragma unroll
                            for (int q = 0; q < ACH; ++q)
#pragma unroll
                                for (int v = 0; v < V; ++v)
                                    t0[u][j1][v] = fmaf(ax[q], bm[h + u][a4 + q][v], t0[u][j1][v]);
                        }
                }
#pragma unroll
                for (int u = 0; u < UH; ++u)
#pragma unroll
                    for (int j1 = 0; j1 < N1; ++j1) {
                        const float4 q = *reinterpret_cast<const float4 *>(dyp[u] + j1 * N2 * N3);
#pragma unroll
                        for (int v = 0; v < V; ++v) {
                            const float tk = t0[u][j1][v] * keep[u];
                            acc[v * N3 + 0] = fmaf(tk, q.x, acc[v * N3 + 0]);
                            acc[v * N3 + 1] = fmaf(tk, q.y, acc[v * N3 + 1]);
                            acc[v * N3 + 2] = fmaf(tk, q.z, acc[v * N3 + 2]);
                            acc[v * N3 + 3] = fmaf(tk, q.w, acc[v * N3 + 3]);
                        }
                    }
            } else {
                // dT0'[j1][c0+v] = sum_j3 dY[(j1,j2)][j3] C[b0+v][j3]
                float dt[UH][N1][V];
#pragma unroll
                for (int u = 0; u < UH; ++u)
#pragma unroll
                    for (int j1 = 0; j1 < N1; ++j1) {
                        if constexpr (DTPRE) {                     // computed once per row by dt_prepare
                            float x[V];
                            load_lds_vec(&sm[u][C::sA + j1 * C::COLS + c0], x);
#pragma unroll
                            for (int v = 0; v < V; ++v) dt[u][j1][v] = keep[u] * x[v];
                        } else {
                            const float4 q = *reinterpret_cast<const float4 *>(dyp[u] + j1 * N2 * N3);
#pragma unroll
                            for (int v = 0; v < V; ++v) {
                                const float4 cv = *reinterpret_cast<const float4 *>(&sm[u][C::sA + (b0 + v) * N3]);
                                dt[u][j1][v] = keep[u] * fmaf(q.x, cv.x, fmaf(q.y, cv.y, fmaf(q.z, cv.z, q.w * cv.w)));
                            }
                        }
                    }
                if (!MFMA && ROLE == 1) {
#pragma unroll
                    for (int u = 0; u < UH; ++u)
#pragma unroll
                        for (int j1 = 0; j1 < N1; ++j1)
#pragma unroll
                            for (int a4 = 0; a4 < RQ; a4 += ACH) {
                                float ax[ACH];
                                load_a(&sm[u][j1 * R + a0 + a4], ax);
#pragma unroll
                                for (int q = 0; q < ACH; ++q)
#pragma unroll
                                    for (int v = 0; v < V; ++v)
                                        acc[(a4 + q) * V + v] = fmaf(ax[q], dt[u][j1][v], acc[(a4 + q) * V + v]);
                            }
                } else if (ROLE == 0) {
#pragma unroll
                    for (int u = 0; u < UH; ++u)
#pragma unroll
                        for (int aa = 0; aa < RQ; ++aa)
#pragma unroll
                            for (int j1 = 0; j1 < N1; ++j1)
#pragma unroll
                                for (int v = 0; v < V; ++v)
                                    acc[j1 * RQ + aa] = fmaf(dt[u][j1][v], bm[h + u][aa][v], acc[j1 * RQ + aa]);
                }
            }
        }
    };

    // G3 owner with the T0 that the forward pass kept (Section 4.2's alternative to recomputing):
    // dG3[b][j3] += sum_{(j1,j2)} T0[(j1,j2)][b] dY[(j1,j2)][j3] needs no G1 or G2 at all.  Wave w
    // takes the rows w, w + 4, ...; lane c = (j2, b) reads T0[k][j1][c] of the row's first position k.
    auto consume_t0 = [&](int nsegs) __attribute__((always_inline)) {
        constexpr int TB = 4;                                              // rows in flight per wave
        for (int sg0 = w; sg0 < nsegs; sg0 += NWAVE * TB) {
            float tv[TB][N1][V];
            const float *dyp[TB];
            float keep[TB];
#pragma unroll
            for (int q = 0; q < TB; ++q) {
                const int sg = min(sg0 + q * NWAVE, nsegs - 1);
                keep[q] = sg0 + q * NWAVE < nsegs ? 1.f : 0.f;
                const float *src = t0 + (size_t)lds.seg_k[sg] * (N1 * C::COLS) + c0;
#pragma unroll
                for (int j1 = 0; j1 < N1; ++j1) load_vec<V>(src + j1 * C::COLS, tv[q][j1]);
                dyp[q] = stage + lds.seg_start[sg] * N + j2 * N3;
            }
#pragma unroll
            for (int q = 0; q < TB; ++q)
#pragma unroll
                for (int j1 = 0; j1 < N1; ++j1) {
                    const float4 g = *reinterpret_cast<const float4 *>(dyp[q] + j1 * N2 * N3);
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const float tk = tv[q][j1][v] * keep[q];
                        acc[v * N3 + 0] = fmaf(tk, g.x, acc[v * N3 + 0]);
                        acc[v * N3 + 1] = fmaf(tk, g.y, acc[v * N3 + 1]);
                        acc[v * N3 + 2] = fmaf(tk, g.z, acc[v * N3 + 2]);
                        acc[v * N3 + 3] = fmaf(tk, g.w, acc[v * N3 + 3]);
                    }
                }
        }
    };

    // ---- (4,4,4) shapes: the G2 owner works on the matrix cores and also serves the G1 owner ----
    // All rows of a G2 owner's list share Bm = G2[s].  The owner therefore computes, besides its own
    //   dG2[a][c] += sum_j1 A[j1][a] dT0'[j1][c]             D(32x32) += A(32x2) B(2x32), two steps per row,
    // the G1 gradient of every row of its list,
    //   P[(row,j1)][a] = sum_c dT0'[(row,j1)][c] Bm[a][c]     D(16x16) += A(16x4) B(4x16) over GB = 8 rows at a
    //                                                          time (32 lines (row,j1) of dT0' = two tiles of 16),
    // with Bm held in registers as the B operand, and writes P to pbuf[k] (k = first position of the
    // row's run; pflag[k'] says for every position whether it is such a first one).  A small kernel
    // (g1_from_p_kernel) then sums P over the list of every G1 slice: no workgroup streams a G2 slice
    // per row any more.  dT0' itself is a product of the same kind,
    //   dT0'[(j1,j2)][b] = sum_j3 dY[(j1,j2)][j3] C[b][j3]    D(16x16) += A(16x4) B(4x16), R / 16 per row,
    // whose result goes to lds.small as the 4 GB x n2 R matrix (line (row,j1), column c = (j2,b)) that
    // the other two products read their operands from.  A workgroup owns 32 rows a of the slice (rh);
    // wave w takes the columns with j2 = w in dG2, rows 2w, 2w+1 of the batch in dT0', and tile
    // (w / 2, w % 2) of P.  The G1 / G3 slices come from global memory (L2) straight in the operand
    // layout, one batch ahead.  Two barriers per batch.
    constexpr int RT = R / 32;                                            // 32-column tiles of a wave's R columns
    constexpr int GB = F::GB, DTS = F::DTS;
    constexpr int NKP = MFMA ? C::COLS / 4 : 1;                           // steps of P (four columns each)
    const int ln = lane & 31, kh = lane >> 5;
    const int l16 = lane & 15, q16 = lane >> 4;
    // Bm^T as B operand of P: step i multiplies columns c = 4 i + q16 with rows a = 32 rh + 16 (w % 2) + l16
    const bool with_p = pbuf != nullptr;                                  // else the G1 owners do their own work (see launch_bwd)
    float bmt[NKP];
    if (MFMA && ROLE == 1 && with_p) {
#pragma unroll
        for (int i = 0; i < NKP; ++i)
            bmt[i] = G2[(size_t)s * C::sB + (size_t)(32 * rh + 16 * (w % 2) + l16) * C::COLS + 4 * i + q16];
    }
    constexpr int NCB = R / 16;                                           // 16-wide pieces of b
    constexpr int SPW = GB / NWAVE;                                       // rows per wave in the dT0' product
    struct G2Ops {
        float a[MFMA ? GB : 1][2];                                        // A[2 h + kh][32 rh + ln] of every row of the batch
        float c[MFMA ? SPW : 1][MFMA ? NCB : 1];                          // C[16 x + l16][q16] of this wave's rows
    };
    // operands of the batch of rows that starts at row sb0 of the window (rows past the end repeat the last one)
    auto g2_fetch = [&](int sb0, int nsegs, G2Ops &o) __attribute__((always_inline)) {
        if constexpr (MFMA) {
            int i1v[GB], i3v[SPW];
#pragma unroll
            for (int u = 0; u < GB; ++u) i1v[u] = lds.seg_i1[min(sb0 + u, nsegs - 1)];
#pragma unroll
            for (int u = 0; u < SPW; ++u) i3v[u] = lds.seg_i3[min(sb0 + SPW * w + u, nsegs - 1)];
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                const float *A = G1 + (size_t)__builtin_amdgcn_readfirstlane(i1v[u]) * C::sA + kh * R + 32 * rh + ln;
                o.a[u][0] = A[0];
                o.a[u][1] = A[2 * R];
            }
#pragma unroll
            for (int u = 0; u < SPW; ++u) {
                const float *Cs = G3 + (size_t)__builtin_amdgcn_readfirstlane(i3v[u]) * C::sC + l16 * N3 + q16;
#pragma unroll
                for (int x = 0; x < NCB; ++x) o.c[u][x] = Cs[16 * x * N3];
            }
        }
    };
    G2Ops g2cur;                                                          // first batch of a window: fetched before the staging
    auto consume_g2_mfma = [&](int nsegs) __attribute__((always_inline)) {
        if constexpr (MFMA) {
            float *dt = lds.small;                                        // [4 GB][DTS]
            G2Ops cur = g2cur, nxt;
            for (int sb0 = 0; sb0 < nsegs; sb0 += GB) {                   // uniform
                const int nb = min(GB, nsegs - sb0);
                // 1. dT0' of this wave's rows -> LDS (rows past the end: zeros).  Lane (l16, q16) supplies
                //    dY[(j1,j2) = l16][j3 = q16] and C[b = 16 x + l16][j3 = q16]; register r of the result is
                //    (j1 = q16, j2 = r), column b = 16 x + l16.
#pragma unroll
                for (int u = 0; u < SPW; ++u) {
                    const int ub = SPW * w + u;
                    const float keep = ub < nb ? 1.f : 0.f;
                    const float dy = keep * stage[lds.seg_start[min(sb0 + ub, nsegs - 1)] * N + l16 * N3 + q16];
#pragma unroll
                    for (int x = 0; x < NCB; ++x) {
                        mfma4_t d = {0.f, 0.f, 0.f, 0.f};
                        d = __builtin_amdgcn_mfma_f32_16x16x4f32(dy, cur.c[u][x], d, 0, 0, 0);
#pragma unroll
                        for (int r = 0; r < 4; ++r) dt[(ub * N1 + q16) * DTS + r * R + 16 * x + l16] = d[r];
                    }
                }
                __syncthreads();
                if (sb0 + GB < nsegs) g2_fetch(sb0 + GB, nsegs, nxt);     // uniform
                // 2. dG2: per row two steps, j1 = 2 h + kh;  3. tile (tm, tn) = (w / 2, w % 2) of P: lines 16 tm + l16 of
                //    dT0' against Bm^T, four columns per step (register r of the result is row u = 4 tm + q16 of the
                //    batch, j1 = r, a = 32 rh + 16 tn + l16).  Both as groups of 16 multiplications whose operands are
                //    read from LDS while the group before is multiplied (the sched_barriers keep that order).
                constexpr int HB = GB / RT;                               // rows per group of dG2
                constexpr int NGP = NKP / 16;                             // groups of P
                const float *dline = dt + (16 * (w / 2) + l16) * DTS + q16;
                auto read_bv = [&](int u0, float (&r)[16]) __attribute__((always_inline)) {
#pragma unroll
                    for (int u = 0; u < HB; ++u)
#pragma unroll
                        for (int h = 0; h < 2; ++h)
#pragma unroll
                            for (int x = 0; x < RT; ++x)
                                r[(u * 2 + h) * RT + x] = dt[((u0 + u) * N1 + 2 * h + kh) * DTS + w * R + 32 * x + ln];
                };
                auto mul_bv = [&](int u0, const float (&r)[16]) __attribute__((always_inline)) {
#pragma unroll
                    for (int u = 0; u < HB; ++u) {
                        if (u0 + u >= nb) break;                          // uniform: the rest of the batch is empty
#pragma unroll
                        for (int h = 0; h < 2; ++h)
#pragma unroll
                            for (int tc = 0; tc < RT; ++tc)
                                accm[tc] = __builtin_amdgcn_mfma_f32_32x32x2f32(cur.a[u0 + u][h], r[(u * 2 + h) * RT + tc], accm[tc], 0, 0, 0);
                    }
                };
                auto read_dv = [&](int g, float (&r)[16]) __attribute__((always_inline)) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) r[i] = dline[4 * (16 * g + i)];
                };
                mfma4_t pa = {0.f, 0.f, 0.f, 0.f};
                float ra[16], rb[16];
                static_assert(HB * 2 * RT == 16 && (RT == 1 || RT == 2) && NGP % 2 == 0, "groups of 16");
                read_bv(0, ra);
                if (RT == 2) read_bv(HB, rb);
                else if (with_p) read_dv(0, rb);
                __builtin_amdgcn_sched_barrier(0);
                mul_bv(0, ra);
                if (RT == 2) {
                    if (with_p) read_dv(0, ra);
                    __builtin_amdgcn_sched_barrier(0);
                    mul_bv(HB, rb);
                    if (with_p) read_dv(1, rb);
                    __builtin_amdgcn_sched_barrier(0);
                } else {
                    if (with_p) read_dv(1, ra);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // now the first two groups of P are in flight: group 0 in ra (rb if RT == 1), group 1 in the other
                if (with_p) {
#pragma unroll
                    for (int g = 0; g < NGP; g += 2) {
                        float (&r0)[16] = RT == 2 ? ra : rb;
                        float (&r1)[16] = RT == 2 ? rb : ra;
#pragma unroll
                        for (int i = 0; i < 16; ++i) pa = __builtin_amdgcn_mfma_f32_16x16x4f32(r0[i], bmt[16 * g + i], pa, 0, 0, 0);
                        if (g + 2 < NGP) read_dv(g + 2, r0);
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int i = 0; i < 16; ++i) pa = __builtin_amdgcn_mfma_f32_16x16x4f32(r1[i], bmt[16 * (g + 1) + i], pa, 0, 0, 0);
                        if (g + 3 < NGP) read_dv(g + 3, r1);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                {
                    const int u = 4 * (w / 2) + q16;
                    if (with_p && u < nb) {
                        float *dst = pbuf + (size_t)lds.seg_k[sb0 + u] * C::sA + 32 * rh + 16 * (w % 2) + l16;
#pragma unroll
                        for (int r = 0; r < 4; ++r) dst[r * R] = pa[r];
                    }
                }
                cur = nxt;
                __syncthreads();                                          // dT0' has been read by everyone
            }
        }
    };

    // Runs of equal rows among the entries [e0, e0 + len) of the list, len <= 64, lane e holding
    // entry e0 + e: one ballot per distinct row gives the lanes of its run.  The runs are laid out
    // one after the other in the order of their first entries, each in list order: mypos is the
    // lane's position in that layout, mysg the number of the run if the lane is its first entry
    // (else -1).  Returns the number of runs.
    auto analyse = [&](const int (&wc)[NWAVE], int e0, int len, int &mysg, int &mypos, int &i1, int &i2, int &i3,
                       uint32_t &myk) __attribute__((always_inline)) {
        const uint32_t my = lane < len ? lds.rows[fb_slot(wc, e0 + lane)] : FB_NONE;
        myk = (needk && lane < len) ? lds.klist[fb_slot(wc, e0 + lane)] : 0u;
        decode_f64(p, my, i1, i2, i3);
        uint64_t rem = __ballot(lane < len);
        int pos = 0, cnt = 0;
        mysg = -1;
        mypos = 0;
        while (rem) {                                                      // uniform: one step per distinct row
            const int j = __builtin_ctzll(rem);
            const uint32_t rj = (uint32_t)__builtin_amdgcn_readlane((int)my, j);
            const uint64_t m = __ballot(my == rj);                         // the run of this row, in list order
            rem &= ~m;
            if (my == rj) mypos = pos + __popcll(m & lanemask_lt());
            if (lane == j) mysg = cnt;
            pos += __popcll(m);
            ++cnt;
        }
        return cnt;
    };

    // One round: the n selected entries, entry e at fb_slot(wc, e) of lds.klist / lds.rows.
    auto process = [&](int n, const int (&wc)[NWAVE]) __attribute__((always_inline)) {
        for (int i0 = 0; i0 < n; i0 += W) {
            const int nw = min(W, n - i0);
            // A short window's gradients are loaded while it is analysed (one float4 per thread).
            constexpr bool EARLY = FB_PIECE * NQ <= WG;
            const bool early_done = EARLY && nw <= FB_PIECE;
            Item early;
            if (early_done) {
                const int e = min(t / NQ, nw - 1), f = t % NQ;
                grad_issue((int)lds.klist[fb_slot(wc, i0 + e)], f, early);
                early.dst = 4 * f;
            }
            int nsegs, mysg, mypos, i1, i2, i3;
            uint32_t myk;
            if (W <= FB_PIECE || nw <= FB_PIECE) {
                // one piece: every wave analyses it by itself (same result everywhere, no barrier)
                nsegs = analyse(wc, i0, nw, mysg, mypos, i1, i2, i3, myk);
                if (MFMA && ROLE == 1 && with_p && w == 0 && lane < nw) pflag[myk] = mysg >= 0;
                if (lane < nw) lds.epos[lane] = mypos;
                if (mysg >= 0) {                                           // first entry of its run
                    lds.seg_start[mysg] = mypos;
                    lds.seg_i1[mysg] = i1; lds.seg_i2[mysg] = i2; lds.seg_i3[mysg] = i3;
                    if (needk) lds.seg_k[mysg] = myk;
                }
                if (lane == 0) lds.seg_start[nsegs] = nw;
            } else {
                // several pieces of 64 entries: wave w analyses piece w; equal rows of different pieces
                // stay separate runs (the gradient is linear in dY)
                const int len = min(FB_PIECE, nw - w * FB_PIECE);          // <= 0: no piece for this wave
                const int cnt = analyse(wc, i0 + w * FB_PIECE, len, mysg, mypos, i1, i2, i3, myk);
                if (MFMA && ROLE == 1 && with_p && lane < len) pflag[myk] = mysg >= 0;
                if (lane == 0) lds.pcnt[w] = cnt;
                __syncthreads();
                int base = 0;
                nsegs = 0;
#pragma unroll
                for (int j = 0; j < NWAVE; ++j) {
                    const int c = lds.pcnt[j];
                    if (j < w) base += c;
                    nsegs += c;
                }
                if (lane < len) lds.epos[w * FB_PIECE + lane] = w * FB_PIECE + mypos;
                if (mysg >= 0) {
                    lds.seg_start[base + mysg] = w * FB_PIECE + mypos;
                    lds.seg_i1[base + mysg] = i1; lds.seg_i2[base + mysg] = i2; lds.seg_i3[base + mysg] = i3;
                    if (needk) lds.seg_k[base + mysg] = myk;
                }
                if (t == 0) lds.seg_start[nsegs] = nw;
                __syncthreads();
            }
            // All global loads of the window's first phase are issued together: first G2 rows,
            // upstream gradients, small operands of the first rows.
            const bool mm = MFMA && ROLE == 1;                            // this owner multiplies on the matrix cores
            if (mm) g2_fetch(0, nsegs, g2cur);
            float bm[UB][RQ][V];
            if (ROLE != 1 && !t0mode && !mm) bm_load(0, nsegs, bm);
            stage_items(i0, early_done ? 0 : nw * NQ, 0, t0mode || mm ? 0 : min(SB, nsegs), wc);
            if (early_done) {
                const float4 g = item_finish(early);
                if (t < nw * NQ) *reinterpret_cast<float4 *>(&stage[4 * (NQ * lds.epos[t / NQ] + t % NQ)]) = g;
            }
            __syncthreads();
            if (nsegs < nw) {                                              // uniform: some row occurs more than once
                // sum each run into its first entry, in list order (a run has at most 64 entries)
                for (int item = t; item < nsegs * N; item += WG) {
                    const int sg = item / N, j = item % N;
                    const int e0 = lds.seg_start[sg], e1 = lds.seg_start[sg + 1];
                    if (e1 - e0 > 1) {
                        float sum = stage[e0 * N + j];
                        int e = e0 + 1;
                        for (; e + 8 <= e1; e += 8) {
                            float x[8];
#pragma unroll
                            for (int q = 0; q < 8; ++q) x[q] = stage[(e + q) * N + j];
#pragma unroll
                            for (int q = 0; q < 8; ++q) sum += x[q];
                        }
                        for (; e < e1; ++e) sum += stage[e * N + j];
                        stage[e0 * N + j] = sum;
                    }
                }
                __syncthreads();
            }
            if (!mm) dt_prepare(0, min(SB, nsegs));
            if (t0mode) consume_t0(nsegs);
            if (mm) consume_g2_mfma(nsegs);
            for (int ub0 = 0; ub0 < (t0mode || mm ? 0 : nsegs); ub0 += UB) {
                const int sb0 = (ub0 / SB) * SB;
                if (ub0 > 0) {
                    if (ROLE != 1) bm_load(ub0, nsegs, bm);
                    if (ub0 == sb0) {                                    // next batch of small operands
                        __syncthreads();
                        stage_items(i0, 0, sb0, min(SB, nsegs - sb0), wc);
                        __syncthreads();
                        dt_prepare(sb0, min(SB, nsegs - sb0));
                    }
                }
                consume(ub0, sb0, nsegs, bm);
            }
            __syncthreads();                                             // before the LDS lists are reused
        }
    };

    // The list comes from the workgroup's own scan of the index array, FB_SCAN positions per round,
    // or, if the lookups were grouped by a pre-pass (tt_group.h), from this slice's list
    // gvals[goff[bin] .. gend[bin]) (payload = item number * L + k, in the order of k), FB_CAP entries
    // at a time.  A scan keeps appending the matches of its rounds to the list and processes it
    // when the next round no longer fits (and once at the end): the cost of a list is paid per
    // list, not per round.  A round that alone selects too many entries (an adversarial index
    // stream) is redone in pieces of FB_CAP positions, which always fit.  The caller has already
    // loaded the rows of the first scan round into rowv.  One loop for both sources, so that the
    // body exists once.
    const int bin = (ROLE == 0 ? 0 : (ROLE == 1 ? p.m1 : p.m1 + p.m2)) + s;
    const uint32_t sub = (uint32_t)ROLE * (uint32_t)L;
    int lo = gvals ? goff[bin] : 0;
    int end = gvals ? gend[bin] : L;
    fb_part_range(part, nparts, gvals ? 16 : FB_CAP, lo, end);
    const int lo0 = lo;
    int span = gvals ? FB_CAP : FB_SCAN, round = 0;
    int fill[NWAVE] = {0, 0, 0, 0};                                    // entries of the sub-lists (scan only)
    while (lo < end) {
        const int hi = min(end, lo + span);
        int pw[NWAVE] = {0, 0, 0, 0}, pn = 0;                              // the list to process in this turn, if any
        if (gvals) {
            pn = hi - lo;
            {   // two round trips for the whole list: all payloads, then all rows (clamped indices: no load is conditional)
                constexpr int NL = FB_CAP / WG;
                uint32_t kk[NL], rr[NL];
#pragma unroll
                for (int q = 0; q < NL; ++q) kk[q] = gvals[lo + min(q * WG + t, pn - 1)] - sub;
#pragma unroll
                for (int q = 0; q < NL; ++q) rr[q] = (uint32_t)indices[kk[q]];
#pragma unroll
                for (int q = 0; q < NL; ++q)
                    if (q * WG + t < pn) { lds.klist[q * WG + t] = kk[q]; lds.rows[q * WG + t] = rr[q]; }
            }
            __syncthreads();
            pw[0] = pn;                                                    // one contiguous list
            lo = hi;
        } else {
            if (lo > lo0 || span != FB_SCAN || round > 0) fb_load_rows(indices, slot, lo, hi, rowv);
            int wc[NWAVE];
            fb_select<C>(lds, p, ROLE, s, rowv, lo, hi, round++, fill, wc);
            bool too_big = false, over = false;
#pragma unroll
            for (int j = 0; j < NWAVE; ++j) {
                too_big = too_big || wc[j] > FB_WCAP;
                over = over || fill[j] + wc[j] > FB_WCAP;
            }
            if (too_big) {
                span = FB_CAP;                                             // redo the round in pieces
            } else {
                if (!over) {                                               // the round's matches join the list
#pragma unroll
                    for (int j = 0; j < NWAVE; ++j) fill[j] += wc[j];
                    lo = hi;
                    if (span == FB_CAP && ((lo - lo0) % FB_SCAN) == 0) span = FB_SCAN;
                }
                if (over || lo >= end) {                                   // process what has been collected
#pragma unroll                                                             // (after "over" the round is redone)
                    for (int j = 0; j < NWAVE; ++j) { pw[j] = fill[j]; pn += fill[j]; fill[j] = 0; }
                }
            }
        }
        if (pn > 0) {
            any = true;
            process(pn, pw);
        }
    }
    if (!any && !fused && !pout) return;

    // The G2 owner's last phase: all old values are loaded before the first store (one round trip, not one per element).
    const float *src2 = fused ? G2 : dG2;                              // x - lr * g to the second set of cores, or dG += g
    float *dst2 = fused ? o2 : dG2;
    const float mul2 = fused ? -lr : 1.f;
    if (MFMA && ROLE == 1) {
        // result registers of the 32 x 32 tiles: register r of lane (kh, ln) is row 32 rh + 8 (r / 4) + 4 kh + r % 4, column ln
        constexpr int NR = MFMA ? RT * 16 : 1;
        float prev[NR];
        if (!pout) {
#pragma unroll
            for (int j = 0; j < NR; ++j) {
                const int tc = j / 16, r = j % 16, a = 32 * rh + 8 * (r / 4) + 4 * kh + r % 4, c = w * R + 32 * tc + ln;
                prev[j] = src2[(size_t)s * C::sB + (size_t)a * C::COLS + c];
            }
        }
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const int tc = j / 16, r = j % 16, a = 32 * rh + 8 * (r / 4) + 4 * kh + r % 4, c = w * R + 32 * tc + ln;
            const float g = accm[MFMA ? tc : 0][r];
            if (pout) pout[a * C::COLS + c] = g;
            else dst2[(size_t)s * C::sB + (size_t)a * C::COLS + c] = fmaf(mul2, g, prev[j]);
        }
    } else if (!MFMA && ROLE == 1) {
        if (active) {
            const size_t at = (size_t)s * C::sB + (size_t)a0 * C::COLS + c0;
            float prev[NACC2];
            if (pout) {
                // a partial slice gradient: nothing to read
            } else if (PREFETCH && fused) {
#pragma unroll
                for (int j = 0; j < NACC2; ++j) prev[j] = old[j];
            } else {
#pragma unroll
                for (int aa = 0; aa < RQ; ++aa)
#pragma unroll
                    for (int v = 0; v < V; ++v) prev[aa * V + v] = src2[at + aa * C::COLS + v];
            }
            if (pout) {
#pragma unroll
                for (int aa = 0; aa < RQ; ++aa)
#pragma unroll
                    for (int v = 0; v < V; ++v) pout[(a0 + aa) * C::COLS + c0 + v] = acc[aa * V + v];
            } else {
#pragma unroll
                for (int aa = 0; aa < RQ; ++aa)
#pragma unroll
                    for (int v = 0; v < V; ++v) dst2[at + aa * C::COLS + v] = fmaf(mul2, acc[aa * V + v], prev[aa * V + v]);
            }
        }
    } else if (ROLE == 0) {
        float red[NACC1];
#pragma unroll
        for (int i = 0; i < NACC1; ++i) red[i] = active ? acc[i] : 0.f;
        group_reduce<NACC1, WAVE>(red, lane);
        if (lane < ReduceKeep<NACC1, WAVE>::writers) {
            const int base = reduce_base<NACC1, WAVE>(lane);
#pragma unroll
            for (int i = 0; i < ReduceKeep<NACC1, WAVE>::value; ++i) {
                const int idx = base + i;                                  // = j1 * RQ + aa
                const int j1 = idx / RQ, aa = idx % RQ;
                const size_t at = (size_t)s * C::sA + j1 * R + a0 + aa;
                if (pout) pout[j1 * R + a0 + aa] = red[i];
                else if (fused) o1[at] = fmaf(-lr, red[i], PREFETCH ? old[i] : G1[at]);
                else add_to(&dG1[at], red[i]);
            }
        }
    } else {
        // partials [wave][column][j3] -> LDS, then a fixed-order sum over (wave, j2)
        float *part = lds.stage;
        static_assert(NWAVE * C::COLS * N3 <= W * N, "partials do not fit");
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
                const size_t at = (size_t)s * C::sC + e;
                if (pout) pout[e] = sum;
                else if (fused) o3[at] = fmaf(-lr, sum, PREFETCH ? old[i] : G3[at]);
                else add_to(&dG3[at], sum);
            }
        }
    }
}

// SPLIT: the launch may share slices between workgroups (FbSplit); without it the kernel takes no such argument
// and its workgroups are the slice owners, nothing else (the small batches of the Criteo-shaped workloads).
template <typename C, bool SPLIT>
__global__ __launch_bounds__(WG) __attribute__((amdgpu_waves_per_eu(FbCfg<C>::WAVES_PER_SIMD))) void bwd_fast_kernel(
    Params p, const float *__restrict__ G1, const float *__restrict__ G2, const float *__restrict__ G3,
    const int64_t *__restrict__ indices, int L, const int64_t *__restrict__ offsets, int n_bags,
    const float *__restrict__ alpha, const int32_t *__restrict__ slot, const float *__restrict__ grad_out,
    float *__restrict__ dG1, float *__restrict__ dG2, float *__restrict__ dG3,
    const uint32_t *__restrict__ gvals, const int *__restrict__ goff, const int *__restrict__ gend,
    float lr, float *__restrict__ o1, float *__restrict__ o2, float *__restrict__ o3, const float *__restrict__ t0,
    typename FbSplitArg<SPLIT>::type sp)
{
    static_assert(SPLIT || !FbCfg<C>::MFMA, "the (4,4,4) shapes always take the split descriptor");
    __shared__ FbLds<C> lds;
    uint32_t rowv[FB_ITER];
    if constexpr (FbCfg<C>::MFMA) {
        if (sp.cw.blocks && (int)blockIdx.x >= sp.n_owner) {             // uniform: this workgroup sums cached-row gradients
            grp_cache_tile_body<(C::N + 63) / 64>(p, (int)blockIdx.x - sp.n_owner, sp.cw.ks, sp.cw.vs, sp.cw.crange, offsets, n_bags, alpha,
                                grad_out, sp.cw.grad_cache, sp.cw.part, sp.cw.fresh);
            return;
        }
        // Role, slice and part of this workgroup (see FbSplit); with sp.pbuf there are no G1 owners here (the G2
        // owners compute the G1 gradient of every row and g1_from_p_kernel finishes the G1 slices).  The role is
        // a constant in each copy of the body: the owners differ too much to share registers.  A G2 slice has
        // R / 32 owners of 32 rows each (they go through the same list).
        constexpr int RTW = C::R / 32;
        const int g = blockIdx.x, n0 = sp.pbuf ? 0 : p.m1 * sp.ns[0], n1 = p.m2 * sp.ns[1] * RTW;
        const int role = (g >= n0) + (g >= n0 + n1);
        int q = g - (role == 0 ? 0 : (role == 1 ? n0 : n0 + n1)), rh = 0;
        if (role == 1) { rh = q % RTW; q /= RTW; }
        const int S = sp.ns[role], sl = q / S, part = q - sl * S;
        float *pout = nullptr;
        if (S > 1) pout = sp.part[role] + (size_t)q * (role == 0 ? C::sA : (role == 1 ? C::sB : C::sC));
        if (!gvals) {
            int lo = 0, end = L;
            fb_part_range(part, S, FB_CAP, lo, end);
            fb_load_rows(indices, slot, lo, min(end, lo + FB_SCAN), rowv);
        }
        if (role == 0) fb_body<C>(lds, p, 0, sl, G1, G2, G3, indices, L, offsets, n_bags, alpha, slot, grad_out, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, rowv, part, S, pout, sp.pbuf, sp.pflag, rh);
        else
        if (role == 1) fb_body<C>(lds, p, 1, sl, G1, G2, G3, indices, L, offsets, n_bags, alpha, slot, grad_out, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, rowv, part, S, pout, sp.pbuf, sp.pflag, rh);
        else fb_body<C>(lds, p, 2, sl, G1, G2, G3, indices, L, offsets, n_bags, alpha, slot, grad_out, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, rowv, part, S, pout, sp.pbuf, sp.pflag, rh);
    } else if constexpr (SPLIT) {
        // run-time role as below, but ns[role] workgroups share a slice, each with a part of the positions
        const int g = blockIdx.x, n0 = p.m1 * sp.ns[0], n1 = p.m2 * sp.ns[1];
        const int role = (g >= n0) + (g >= n0 + n1);
        const int q = g - (role == 0 ? 0 : (role == 1 ? n0 : n0 + n1));
        const int S = sp.ns[role], sl = q / S, part = q - sl * S;
        float *pout = nullptr;
        if (S > 1) pout = sp.part[role] + (size_t)q * (role == 0 ? C::sA : (role == 1 ? C::sB : C::sC));
        if (!gvals) {
            int lo = 0, end = L;
            fb_part_range(part, S, FB_CAP, lo, end);
            fb_load_rows(indices, slot, lo, min(end, lo + FB_SCAN), rowv);
        }
        fb_body<C>(lds, p, role, sl, G1, G2, G3, indices, L, offsets, n_bags, alpha, slot, grad_out, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, rowv, part, S, pout, nullptr, nullptr, 0);
    } else {
        // The index loads do not depend on the role: issue them before anything else.
        if (!gvals) fb_load_rows(indices, slot, 0, min(L, FB_SCAN), rowv);
        __builtin_amdgcn_sched_barrier(0);
        // role and slice of this workgroup, without branches so that all kernel arguments load together
        const int g = blockIdx.x;
        const int ge1 = g >= p.m1, ge2 = g >= p.m1 + p.m2;
        const int role = ge1 + ge2;
        const int sl = g - (ge1 ? p.m1 : 0) - (ge2 ? p.m2 : 0);
        fb_body<C>(lds, p, role, sl, G1, G2, G3, indices, L, offsets, n_bags, alpha, slot, grad_out, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, rowv, 0, 1, nullptr, nullptr, nullptr, 0);
    }
}

// Sums the partial slice gradients of the split roles (FbSplit) and finishes their slices: adds the sum to dG
// (out == nullptr) or writes x - lr * sum to out.  One thread per float4 of the split cores, all of them in one launch.
constexpr int FB_MAX_PARTS = 8;                             // workgroups that may share one slice
struct FbFinish {
    const float *part[4], *x[4];
    float *dG[4], *out[4];
    int ns[4], slice4[4];                                   // parts per slice, float4 per slice
    int64_t end4[4];                                        // running total of float4 over the (up to four) arrays:
    int n;                                                  // split cores, and the cache lines (one "part": their gradient)
};

__global__ __launch_bounds__(WG) void bwd_split_finish_kernel(FbFinish a, float lr)
{
    for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < a.end4[a.n - 1]; i += (int64_t)gridDim.x * WG) {
        const int r = (i >= a.end4[0]) + (i >= a.end4[1]) + (i >= a.end4[2]);
        // One copy of the body per array, so that its descriptor sits in scalar registers: an argument array indexed
        // by a run-time number is read from memory, one more round trip before the first useful load.
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            if (r != rr) continue;
            const int ns = a.ns[rr], slice4 = a.slice4[rr];
            float *out = a.out[rr];
            const int64_t j = i - (rr ? a.end4[rr ? rr - 1 : 0] : 0);
            const int64_t sl = j / slice4, e = j - sl * slice4;
            const float4 *src = reinterpret_cast<const float4 *>(a.part[rr]) + sl * ns * slice4 + e;
            // the old value and all parts (at most FB_MAX_PARTS) are loaded together
            const float4 x = reinterpret_cast<const float4 *>(out ? a.x[rr] : a.dG[rr])[j];
            float4 v[FB_MAX_PARTS];
#pragma unroll
            for (int h = 0; h < FB_MAX_PARTS; ++h)
                v[h] = h < ns ? src[(int64_t)h * slice4] : make_float4(0.f, 0.f, 0.f, 0.f);
            float4 sum = v[0];
#pragma unroll
            for (int h = 1; h < FB_MAX_PARTS; ++h)
                if (h < ns) { sum.x += v[h].x; sum.y += v[h].y; sum.z += v[h].z; sum.w += v[h].w; }
            if (out) {
                reinterpret_cast<float4 *>(out)[j] =
                    make_float4(fmaf(-lr, sum.x, x.x), fmaf(-lr, sum.y, x.y), fmaf(-lr, sum.z, x.z), fmaf(-lr, sum.w, x.w));
            } else {
                reinterpret_cast<float4 *>(a.dG[rr])[j] = make_float4(x.x + sum.x, x.y + sum.y, x.z + sum.z, x.w + sum.w);
            }
        }
    }
}

// (4,4,4) shapes: finishes the G1 slices from the per-row gradients P that the G2 owners wrote (see fb_body).
// Workgroup s collects the flagged positions whose first digit is s, 8192 candidates per round (all positions,
// or the slice's list from the grouping pre-pass), every wave appending to its own list, and adds their rows
// of P: a row is n1 R floats, PA threads read it as float4, WG / PA rows side by side, UN in flight each.
// Fixed order, no atomics.  out == nullptr: dG1 += sum; else out = G1 - lr * sum.
template <typename C>
__global__ __launch_bounds__(WG) void g1_from_p_kernel(Params p, const int64_t *__restrict__ indices, int L,
                                                       const int32_t *__restrict__ slot, const uint32_t *__restrict__ gvals,
                                                       const int *__restrict__ goff, const int *__restrict__ gend,
                                                       const float *__restrict__ pbuf, const int *__restrict__ pflag,
                                                       const float *__restrict__ G1, float *__restrict__ dG1,
                                                       float *__restrict__ out, float lr, GrpCacheWork cw)
{
    if ((int)blockIdx.x >= p.m1) {                                        // extra workgroups: runs of cached rows that cross tiles
        grp_cache_fix_body<(C::N + 63) / 64>(p, (int)blockIdx.x - p.m1, cw.ks, cw.crange, cw.gend, cw.part, cw.grad_cache);
        return;
    }
    constexpr int PA = C::sA / 4, NG = WG / PA, UN = 16;                  // UN rows of P in flight per thread: a slice's list is one or two passes
    constexpr int ITER = 32, PER = ITER * WAVE;                           // candidates per lane / per wave and round
    __shared__ uint32_t list[NWAVE][PER];
    __shared__ int wcnt[NWAVE];
    __shared__ float4 part[NG][PA];
    const int s = blockIdx.x, t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int f = t % PA, g = t / PA;
    const float4 *p4 = reinterpret_cast<const float4 *>(pbuf);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    const int lo = gvals ? goff[s] : 0, end = gvals ? gend[s] : L;
    for (int base = lo; base < end; base += NWAVE * PER) {               // uniform
        // candidates base + w PER + it 64 + lane, ITER per lane, all loads of a round together
        int n = 0;
#pragma unroll
        for (int i0 = 0; i0 < ITER; i0 += 8) {
            if (base + w * PER + i0 * WAVE >= end) break;                 // uniform per wave
            uint32_t kk[8];
            bool take[8];
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int c = base + w * PER + (i0 + it) * WAVE + lane;
                const bool ok = c < end;
                if (gvals) {
                    kk[it] = ok ? gvals[c] : 0u;                          // the G1 items carry the position itself
                    take[it] = ok;
                } else {
                    kk[it] = (uint32_t)c;
                    int i1 = -1, i2, i3;
                    if (ok) decode(p, (uint32_t)indices[c], i1, i2, i3);
                    take[it] = ok && i1 == s && !(slot && slot[c] >= 0);
                }
            }
            // (index 0 for the candidates that are out already: a load behind a condition would be waited for on the spot)
            int pf[8];
#pragma unroll
            for (int it = 0; it < 8; ++it) pf[it] = pflag[take[it] ? kk[it] : 0u];
#pragma unroll
            for (int it = 0; it < 8; ++it) take[it] = take[it] && pf[it] != 0;
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const uint64_t m = __ballot(take[it]);
                if (take[it]) list[w][n + __popcll(m & lanemask_lt())] = kk[it];
                n += __popcll(m);
            }
        }
        if (lane == 0) wcnt[w] = n;
        __syncthreads();
        int wc[NWAVE], total = 0;
#pragma unroll
        for (int j = 0; j < NWAVE; ++j) { wc[j] = wcnt[j]; total += wc[j]; }
        for (int j0 = g; j0 < total; j0 += NG * UN) {
            float4 v[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int j = min(j0 + u * NG, total - 1);                // past the end: the last row again, not added
                int e = j, ww = 0;
#pragma unroll
                for (int x = 0; x + 1 < NWAVE; ++x)
                    if (e >= wc[x] && ww == x) { e -= wc[x]; ww = x + 1; }
                v[u] = p4[(size_t)list[ww][e] * PA + f];
            }
#pragma unroll
            for (int u = 0; u < UN; ++u)
                if (j0 + u * NG < total) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
        }
        __syncthreads();                                                  // before the lists are reused
    }
    part[g][f] = acc;
    __syncthreads();
    if (t < PA) {
        float4 sum = part[0][t];
#pragma unroll
        for (int x = 1; x < NG; ++x) {
            const float4 v = part[x][t];
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        const size_t at = (size_t)s * PA + t;
        if (out) {
            const float4 x = reinterpret_cast<const float4 *>(G1)[at];
            reinterpret_cast<float4 *>(out)[at] =
                make_float4(fmaf(-lr, sum.x, x.x), fmaf(-lr, sum.y, x.y), fmaf(-lr, sum.z, x.z), fmaf(-lr, sum.w, x.w));
        } else {
            float4 *d = reinterpret_cast<float4 *>(dG1) + at;
            const float4 o = *d;
            *d = make_float4(o.x + sum.x, o.y + sum.y, o.z + sum.z, o.w + sum.w);
        }
    }
}

// Split factors for a call: from 4096 or 8192 positions on (below that the extra pass does not pay).  Two or four
// workgroups share a slice: the longest lists decide the kernel time (without a cache one hot row can fill a
// list), and a scan of a part of the positions takes fewer rounds.  With the grouping pre-pass the G2 owners also compute the G1 gradients (fb_with_p), so
// there are no G1 owners; without it they exist and four of them share a slice (each streams a G2 slice per row).
template <typename C>
static inline void fb_choose_split(int L, int (&ns)[3])
{
    ns[0] = ns[1] = ns[2] = 1;
    if (FbCfg<C>::MFMA) {
        if (L >= 4096) {
            ns[0] = 4;
            ns[1] = ns[2] = 2;
        }
    } else if (L >= (C::R >= 64 ? 4096 : 8192)) {
        // (2,2,4): at 4096 positions twice the workgroups no longer fit the chip at once and the extra pass costs
        // more than the shorter lists save, except at R = 64 where a G1 owner has one G2 row in flight at a time
        ns[0] = ns[1] = ns[2] = L >= 131072 ? 8 : (L >= 16384 ? 4 : 2);
    }
}

// Do the G2 owners compute the G1 gradients of their rows (and g1_from_p_kernel finish the G1 slices)?  With the
// grouping pre-pass: the lists are long and full batches of rows amortise the extra product; for the shorter
// lists of a scan the G1 owners' own pass was measured to be faster.
template <typename C>
static inline bool fb_with_p(bool grouped) { return FbCfg<C>::MFMA && grouped; }

// With the grouping pre-pass, the backward of the (4,4,4) shapes runs the cached-row reduction as extra workgroups of
// its own launches (and the SGD step of the cache lines in its finishing kernel) instead of three launches of their own.
static inline bool fast_bwd_takes_cache_work(const Params &p, int L)
{
    const int cfg = fast_config(p);
    return (cfg == 4 || cfg == 5) && L >= 4096;
}

static inline void fast_bwd_split(const Params &p, int L, int (&ns)[3])
{
    ns[0] = ns[1] = ns[2] = 1;
    switch (fast_config(p)) {
    case 0: fb_choose_split<Cfg224R8>(L, ns); break;
    case 1: fb_choose_split<Cfg224R16>(L, ns); break;
    case 2: fb_choose_split<Cfg224R32>(L, ns); break;
    case 3: fb_choose_split<Cfg224R64>(L, ns); break;
    case 4: fb_choose_split<Cfg444R32>(L, ns); break;
    case 5: fb_choose_split<Cfg444R64>(L, ns); break;
    default: break;
    }
}

// floats of workspace the specialised kernel may need beyond the lists: partial slices of the split roles, and for
// the (4,4,4) shapes with the grouping pre-pass the per-row G1 gradients (L n1 R floats) and the flags (L ints)
static inline size_t fast_bwd_extra_floats(const Params &p, int L, bool grouped)
{
    int ns[3];
    fast_bwd_split(p, L, ns);
    const int cfg = fast_config(p);
    const bool with_p = (cfg == 4 || cfg == 5) && grouped;
    size_t n = 0;
    if (ns[0] > 1 && !with_p) n += (size_t)ns[0] * p.m1 * p.sA;
    if (ns[1] > 1) n += (size_t)ns[1] * p.m2 * p.sB;
    if (ns[2] > 1) n += (size_t)ns[2] * p.m3 * p.sC;
    if (with_p) n += (size_t)(L > 0 ? L : 1) * p.sA + (size_t)((L > 0 ? L : 1) + 3) / 4 * 4;
    return n;
}

template <typename C>
static inline void launch_bwd(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx,
                              int L, const int64_t *off, int n_bags, const float *alpha, const int32_t *slot,
                              const float *go, float *dG1, float *dG2, float *dG3, const uint32_t *gvals,
                              const int *goff, const int *gend, float lr, float *o1, float *o2, float *o3,
                              const float *t0, float *extra_ws, const GrpCacheWork *cw, float *cache_rows,
                              int64_t cache_floats, hipStream_t st)
{
    constexpr bool MFMA = FbCfg<C>::MFMA;
    const bool with_p = fb_with_p<C>(gvals != nullptr);
    FbSplit sp;
    fb_choose_split<C>(L, sp.ns);
    const int m[3] = {p.m1, p.m2, p.m3}, slice[3] = {p.sA, p.sB, p.sC};
    float *q = extra_ws;
    int grid = 0;
    for (int r = 0; r < 3; ++r) {
        sp.part[r] = nullptr;
        if (with_p && r == 0) continue;                                    // no G1 owners in the main kernel
        if (sp.ns[r] > 1) {
            sp.part[r] = q;
            q += (size_t)sp.ns[r] * m[r] * slice[r];
        }
        grid += sp.ns[r] * m[r] * (MFMA && r == 1 ? C::R / 32 : 1);
    }
    sp.pbuf = nullptr;
    sp.pflag = nullptr;
    if (with_p) {
        sp.pbuf = q;
        q += (size_t)(L > 0 ? L : 1) * p.sA;
        sp.pflag = reinterpret_cast<int *>(q);
    }
    // the caller's cached-row work rides along (fast_bwd_takes_cache_work): tiles behind the owners, the runs that cross
    // tiles behind g1_from_p_kernel's workgroups, the SGD step of the cache lines in the finishing kernel
    const bool with_cw = cw != nullptr && cw->blocks > 0;
    sp.cw = GrpCacheWork{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, false};
    sp.n_owner = grid;
    if (with_cw) {
        sp.cw = *cw;
        grid += cw->blocks;
    }
    if (MFMA || sp.ns[0] > 1 || sp.ns[1] > 1 || sp.ns[2] > 1)
        hipLaunchKernelGGL((bwd_fast_kernel<C, true>), dim3(grid), dim3(WG), 0, st, p, G1, G2, G3, idx, L, off,
                           n_bags, alpha, slot, go, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, sp);
    else if constexpr (!MFMA)
        hipLaunchKernelGGL((bwd_fast_kernel<C, false>), dim3(grid), dim3(WG), 0, st, p, G1, G2, G3, idx, L, off,
                           n_bags, alpha, slot, go, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, FbNoSplit());
    if (with_p)
        hipLaunchKernelGGL(g1_from_p_kernel<C>, dim3(p.m1 + sp.cw.blocks), dim3(WG), 0, st, p, idx, L, slot, gvals, goff, gend,
                           sp.pbuf, sp.pflag, G1, dG1, o1, lr, sp.cw);
    const float *x[3] = {G1, G2, G3};
    float *dG[3] = {dG1, dG2, dG3}, *out[3] = {o1, o2, o3};
    FbFinish f;
    f.n = 0;
    int64_t total4 = 0;
    for (int r = 0; r < 3; ++r) {
        if (sp.part[r] == nullptr) continue;
        const int i = f.n++;
        f.part[i] = sp.part[r]; f.x[i] = x[r]; f.dG[i] = dG[r]; f.out[i] = out[r];
        f.ns[i] = sp.ns[r]; f.slice4[i] = slice[r] / 4;
        total4 += (int64_t)m[r] * (slice[r] / 4);
        f.end4[i] = total4;
    }
    if (with_cw && cache_rows) {                                           // fused step: lines <- lines - lr * gradient
        const int i = f.n++;
        f.part[i] = sp.cw.grad_cache; f.x[i] = cache_rows; f.dG[i] = nullptr; f.out[i] = cache_rows;
        f.ns[i] = 1; f.slice4[i] = 1;
        total4 += cache_floats / 4;
        f.end4[i] = total4;
    }
    if (f.n) {
        for (int i = f.n; i < 4; ++i) {                                    // unused entries: harmless values
            f.part[i] = f.part[0]; f.x[i] = f.x[0]; f.dG[i] = f.dG[0]; f.out[i] = f.out[0];
            f.ns[i] = 1; f.slice4[i] = 1; f.end4[i] = total4;
        }
        const int64_t blocks = (total4 + WG - 1) / WG;
        hipLaunchKernelGGL(bwd_split_finish_kernel, dim3((int)(blocks < 4096 ? blocks : 4096)), dim3(WG), 0, st, f, lr);
    }
}

static inline bool fast_bwd_supported(const Params &p) { return fast_config(p) >= 0; }

static inline void fast_bwd(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx, int L,
                            const int64_t *off, int n_bags, const float *alpha, const int32_t *slot, const float *go,
                            float *dG1, float *dG2, float *dG3, const uint32_t *gvals, const int *goff,
                            const int *gend, float lr, float *o1, float *o2, float *o3, const float *t0,
                            float *extra_ws, const GrpCacheWork *cw, float *cache_rows, int64_t cache_floats,
                            hipStream_t st)
{
    switch (fast_config(p)) {
    case 0: launch_bwd<Cfg224R8>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, extra_ws, cw, cache_rows, cache_floats, st); break;
    case 1: launch_bwd<Cfg224R16>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, extra_ws, cw, cache_rows, cache_floats, st); break;
    case 2: launch_bwd<Cfg224R32>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, extra_ws, cw, cache_rows, cache_floats, st); break;
    case 3: launch_bwd<Cfg224R64>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, extra_ws, cw, cache_rows, cache_floats, st); break;
    case 4: launch_bwd<Cfg444R32>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, extra_ws, cw, cache_rows, cache_floats, st); break;
    case 5: launch_bwd<Cfg444R64>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, gvals, goff, gend, lr, o1, o2, o3, t0, extra_ws, cw, cache_rows, cache_floats, st); break;
    default: break;
    }
}

}  // namespace tt
