// Backward pass for long index streams on the matrix cores (Eq. 4 / Alg. 2), after the grouping
// pre-pass of tt_group.h and with the intermediate T0 kept by the forward pass.
//
// The positions that share a slice of the second core share the operand Bm = G2[i2], so the
// two large products of Eq. 4 become matrix products over a tile of such positions.  With
// dT0'[(e,j1)][(j2,b)] = sum_j3 dY_e[(j1,j2)][j3] C_e[b][j3] (the rows (e,j1) of up to TP
// positions stacked: 128 rows):
//     dG2[i2][a][(j2,b)] += sum_rows A[(e,j1)][a] dT0'[(e,j1)][(j2,b)]        (A = stacked rows of G1)
//     P[(e,j1)][a]        = sum_(j2,b) dT0'[(e,j1)][(j2,b)] Bm[a][(j2,b)]     (the G1 gradient of position e)
// both as fp32 MFMA 32x32x2 products with operands in LDS, one j2 at a time.  A workgroup works
// through consecutive tiles, leaves the part of a slice gradient that it has added up in
// part2[first tile of the stretch] and the rows P in pbuf[k]; two more launches finish the
// cores in a fixed order of summation (no atomics):
//   * the parts of every G2 slice are added in tile order,
//   * the G1 gradient is a segmented sum of the rows P over the sorted items of the first
//     core (one wave per 8 to 64 items; runs over the borders of such pieces are finished, in
//     the second of the two launches, by the wave where the run begins, as in the cached-row
//     reduction of tt_group.h),
//   * the G3 gradient dG3[i3][b][j3] += sum_(j1,j2) T0_k[(j1,j2)][b] dY_k[(j1,j2)][j3] is the same
//     kind of segmented sum over the sorted items of the third core, the row of an item being
//     computed from the kept T0 on the way.
// Every finish either adds to the gradient arrays or writes x - lr * gradient to the second
// set of cores (slices that no position touches are copied).
#pragma once

#include "tt_common.h"
#include "tt_fast.h"
#include "tt_fast_bwd.h"
#include "tt_group.h"

namespace tt {

constexpr int BO_MAX_CHUNK = 64;                    // tiles that one workgroup takes at most (their descriptors sit in LDS)

template <typename C, int ROWS_ = 128>
struct BoCfg {
    static constexpr int ROWS = ROWS_, TP = ROWS / C::N1;      // stacked rows / positions of a tile
    static constexpr int RB = C::R / 32;                       // 32-wide blocks of a rank index
    static constexpr int NB = RB * RB;                         // 32 x 32 blocks of the R x R slice gradient of one j2
    static constexpr int KS = NWAVE / NB;                      // waves that share a block: each takes ROWS / KS of the stacked rows
    static constexpr int RBK = ROWS / 32;                      // 32-row blocks of P
    static constexpr int WPR = NWAVE / RBK;                    // waves that share a row block of P: each takes RB / WPR of its 32-wide column blocks
    static constexpr int ABW = RB / WPR;
    // row strides in LDS: As and Bm rows are written and (Bm) read as float4 (stride a multiple of 4; four K-steps of the
    // second product per read), dT0' is read in pairs (even stride)
    static constexpr int LDA = C::R + 4, LDT = C::R + 2, LDB = C::R + 4;
    static constexpr int NBQ = WG / TP, BQ = C::R / NBQ;       // threads per position / values of b per thread in dT0'
    static constexpr int DY_FLOATS = TP * C::N;
    static constexpr int LDS_FLOATS = DY_FLOATS + ROWS * LDA + ROWS * LDT + C::R * LDB;
    static constexpr int NDY = TP * C::N / 4 / WG;             // float4 of dY per thread and tile
    static constexpr int NA4 = ROWS * C::R / 4 / WG;           // float4 of the stacked G1 rows per thread and tile
    static constexpr int WGS_PER_CU = C::R >= 64 ? 1 : 2;      // what the LDS and the registers of a tile leave room for
    static_assert(C::R % 32 == 0 && NB <= NWAVE && NWAVE % NB == 0 && WG % TP == 0 && NBQ <= 16 && BQ >= 1, "tile layout");
    static_assert(ROWS % 32 == 0 && RBK <= NWAVE && NWAVE % RBK == 0 && RB % WPR == 0 && ABW >= 1, "the waves share out the blocks of P");
    static_assert(TP * C::N % (4 * WG) == 0 && ROWS * C::R % (4 * WG) == 0, "whole float4 per thread");
    static_assert(KS == 1 || NWAVE * 1024 <= ROWS * LDT, "the partial blocks of a slice gradient fit the dT0' area");
    static_assert((ROWS / KS) % 2 == 0, "pairs of rows per product step");
};

template <typename C, int ROWS_>
static inline size_t bo_lds_bytes() { return (size_t)BoCfg<C, ROWS_>::LDS_FLOATS * sizeof(float); }

// tiles per workgroup: the tiles in use (the first `used` of the table) shared out evenly among the workgroups
__host__ __device__ static inline int bo_chunk(int used, int nwg) { return used > 0 ? (used + nwg - 1) / nwg : 1; }

// One workgroup takes ch = bo_chunk(tiles in use, workgroups) consecutive tiles of the tile table (tt_group.h) and
// works through them as a pipeline: while the products of a tile run on the matrix cores, the operands of the next
// one (its upstream gradients, stacked G1 rows and G3 rows, looked up through the position records that were fetched
// a tile earlier) are on their way into registers, and they are written to LDS when the tile is done, so that the
// chain record -> operands -> products of a tile is not waited for.  The part of a slice gradient that the workgroup
// has added up goes to part2[first tile of that stretch]: a stretch begins with the workgroup's first tile and
// wherever the slice changes.  Where the R x R block structure leaves waves without a block of their own (R = 32),
// the waves split the stacked rows of a block among them and their partial blocks are added, in wave order, when
// the stretch is written.
// A barrier for data exchanged through LDS only.  __syncthreads() also waits for the workgroup's global stores, and on
// this hardware stores and loads share a counter, so it would drain the global loads that are fetched ahead; nothing
// that the tile kernel stores to global memory is read again by it.
__device__ __forceinline__ void bo_lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <typename C, int ROWS_>
__global__ __launch_bounds__(WG) __attribute__((amdgpu_waves_per_eu(BoCfg<C, ROWS_>::WGS_PER_CU, BoCfg<C, ROWS_>::WGS_PER_CU))) void bo_tile_kernel(
    Params p, const float *__restrict__ G1, const float *__restrict__ G2, const float *__restrict__ G3, int L, int n_bags,
    const float *__restrict__ alpha, const float *__restrict__ grad_out, const int4 *__restrict__ info,
    const int4 *__restrict__ tiles, int ntiles, const int *__restrict__ tile_base, float *__restrict__ part2,
    float *__restrict__ pbuf, float4 *__restrict__ o1, float4 *__restrict__ o3)
{
    using F = BoCfg<C, ROWS_>;
    if (o1) {
        // the fused step: the first and the third core are copied to the second set here, all workgroups together; the
        // kernels that follow overwrite the slices that the batch touches
        const int64_t n1 = (int64_t)p.m1 * C::sA / 4, n3 = (int64_t)p.m3 * C::sC / 4;
        const float4 *a1 = reinterpret_cast<const float4 *>(G1), *a3 = reinterpret_cast<const float4 *>(G3);
        for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < n1 + n3; i += (int64_t)gridDim.x * WG) {
            if (i < n1) o1[i] = a1[i];
            else o3[i - n1] = a3[i - n1];
        }
    }
    constexpr int N1 = C::N1, N2 = C::N2, R = C::R, N = C::N, COLS = C::COLS, TP = F::TP;
    constexpr int LDA = F::LDA, LDT = F::LDT, LDB = F::LDB, NQ = N / 4;
    extern __shared__ __align__(16) float bo_lds[];
    float *dyl = bo_lds;                              // [TP][N]      alpha_k dY of the positions
    float *As = dyl + F::DY_FLOATS;                   // [128][LDA]   stacked rows of G1
    float *dT = As + F::ROWS * LDA;                   // [128][LDT]   dT0' for the current j2
    float *Bl = dT + F::ROWS * LDT;                   // [R][LDB]     Bm[a][(j2, .)]
    __shared__ int s_ti2[BO_MAX_CHUNK], s_tlo[BO_MAX_CHUNK], s_tn[BO_MAX_CHUNK];   // the workgroup's tiles: slice, first item, items
    __shared__ int s_k[2][TP], s_i1[2][TP], s_i3[2][TP], s_bag[2][TP];   // the positions of this tile and of the next one
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int ln = lane & 31, kh = lane >> 5;
    const int blk = w % F::NB, ks = w / F::NB;        // this wave adds rows [ks ROWS / KS, (ks + 1) ROWS / KS) into block blk
    const int ab1 = blk / F::RB, bb1 = blk % F::RB;
    const int rb = w % F::RBK, ab0 = (w / F::RBK) * F::ABW;   // this wave's block of P: rows 32 rb .., column blocks ab0 .. ab0 + ABW - 1

    const int used = min(ntiles, tile_base[p.m2]);
    const int ch = bo_chunk(used, gridDim.x);
    const int tbeg = blockIdx.x * ch, tend = min(used, tbeg + min(ch, BO_MAX_CHUNK));
    if (tbeg >= tend) return;                         // uniform
    if (t < tend - tbeg) {
        const int4 td = tiles[tbeg + t];
        // (guards against a table that no pre-pass wrote: such a tile ends the workgroup's work)
        const bool ok = td.z > 0 && (unsigned)td.x < (unsigned)p.m2 && td.y >= 0 && td.z <= TP && td.y + td.z <= 3 * L;
        s_ti2[t] = ok ? td.x : -1; s_tlo[t] = ok ? td.y : 0; s_tn[t] = ok ? td.z : 0;
    }
    bo_lds_barrier();

    // ---- the pipeline's registers: records of the tile after next, operands of the next tile ----
    // (plain floats and ints: arrays of vector types that lambdas take by reference end up in scratch memory)
    int pin_k = 0, pin_i1 = 0, pin_i3 = 0, pin_bag = 0;
    float nxt_dy[F::NDY][4], nxt_a[F::NA4][4], nxt_cv[F::BQ][4], cv[F::BQ][4];
    float nxt_w[F::NDY];
    constexpr int NB4 = R * R / 4 / WG;
    float bm[NB4][4];
    auto ld4 = [](const float *src, float (&d)[4]) __attribute__((always_inline)) {
        const float4 v = *reinterpret_cast<const float4 *>(src);
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
    };
    const int ee = t / F::NBQ, bq = t % F::NBQ;        // thread (position ee, bq) of the dT0' product: rows b = NBQ i + bq of G3[i3]

    auto load_records = [&](int lo) __attribute__((always_inline)) {
        if (t < TP) {
            const int4 pi = info[min(lo + t, 3 * L - 1)];
            pin_k = pi.x; pin_i1 = pi.y; pin_i3 = pi.z; pin_bag = pi.w;
        }
    };
    auto publish_records = [&](int n, int set) __attribute__((always_inline)) {
        if (t < TP) {
            const bool on = t < n;
            s_k[set][t] = on && (unsigned)pin_k < (unsigned)L ? pin_k : 0;
            s_i1[set][t] = on ? min(max(pin_i1, 0), p.m1 - 1) : 0;
            s_i3[set][t] = on ? min(max(pin_i3, 0), p.m3 - 1) : 0;
            s_bag[set][t] = on ? min(max(pin_bag, 0), n_bags - 1) : 0;
        }
    };
    auto fetch_bm = [&](int i2, int j2) __attribute__((always_inline)) {
        const float *src = G2 + (size_t)i2 * C::sB + j2 * R;
#pragma unroll
        for (int q = 0; q < NB4; ++q) {
            const int i = q * WG + t, a = i / (R / 4), b4 = 4 * (i % (R / 4));
            ld4(src + a * COLS + b4, bm[q]);
        }
    };
    auto issue_operands = [&](int set) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < F::NDY; ++q) {
            const int i = q * WG + t, e = i / NQ, f = i % NQ;
            ld4(grad_out + (size_t)s_bag[set][e] * N + 4 * f, nxt_dy[q]);
            nxt_w[q] = alpha ? alpha[s_k[set][e]] : 1.f;
        }
#pragma unroll
        for (int q = 0; q < F::NA4; ++q) {
            const int i = q * WG + t, row = i / (R / 4), a4 = 4 * (i % (R / 4)), e = row / N1, j1 = row % N1;
            ld4(G1 + (size_t)s_i1[set][e] * C::sA + j1 * R + a4, nxt_a[q]);
        }
        const float *Cp = G3 + (size_t)s_i3[set][ee] * C::sC + 4 * bq;
#pragma unroll
        for (int i = 0; i < F::BQ; ++i) ld4(Cp + 4 * i * F::NBQ, nxt_cv[i]);
    };
    // the operands of a tile of n positions to LDS and to cv[] (positions past the end: zeros)
    auto commit_operands = [&](int n) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < F::NDY; ++q) {
            const int i = q * WG + t, e = i / NQ, f = i % NQ;
            const float wgt = e < n ? nxt_w[q] : 0.f;                        // (selected per component: a select of float4s goes through memory)
            *reinterpret_cast<float4 *>(dyl + e * N + 4 * f) =
                make_float4(e < n ? nxt_dy[q][0] * wgt : 0.f, e < n ? nxt_dy[q][1] * wgt : 0.f, e < n ? nxt_dy[q][2] * wgt : 0.f,
                            e < n ? nxt_dy[q][3] * wgt : 0.f);
        }
#pragma unroll
        for (int q = 0; q < F::NA4; ++q) {
            const int i = q * WG + t, row = i / (R / 4), a4 = 4 * (i % (R / 4)), e = row / N1;
            const bool on = e < n;
            *reinterpret_cast<float4 *>(As + row * LDA + a4) =
                make_float4(on ? nxt_a[q][0] : 0.f, on ? nxt_a[q][1] : 0.f, on ? nxt_a[q][2] : 0.f, on ? nxt_a[q][3] : 0.f);
        }
#pragma unroll
        for (int i = 0; i < F::BQ; ++i)
#pragma unroll
            for (int x = 0; x < 4; ++x) cv[i][x] = ee < n ? nxt_cv[i][x] : 0.f;
    };

    mfma16_t acc1[N2];
    int cur = -1, slot = 0;
    auto flush1 = [&]() __attribute__((always_inline)) {                       // (uniform)
        if (cur < 0) return;
        if constexpr (F::KS == 1) {
#pragma unroll
            for (int j2 = 0; j2 < N2; ++j2) {
                float *dst = part2 + (size_t)slot * C::sB + j2 * R + 32 * bb1 + ln;
#pragma unroll
                for (int r = 0; r < 16; ++r) dst[(size_t)(32 * ab1 + 8 * (r / 4) + 4 * kh + r % 4) * COLS] = acc1[j2][r];
            }
        } else {
            // the waves' partial blocks through the dT0' area (free between tiles): element (row, col) of wave w's block is
            // value r = 4 (row / 8) + row % 4 of lane 32 ((row / 4) % 2) + col; thread (row, four columns) adds the KS partials
            // of a block in wave order and stores a float4
#pragma unroll
            for (int j2 = 0; j2 < N2; ++j2) {
#pragma unroll
                for (int r = 0; r < 16; ++r) dT[w * 1024 + r * 64 + lane] = acc1[j2][r];
                bo_lds_barrier();
                for (int x = t; x < F::NB * 256; x += WG) {
                    const int b = x / 256, row = (x % 256) / 8, c4 = 4 * (x % 8);
                    const int at = (4 * (row / 8) + row % 4) * 64 + 32 * ((row / 4) % 2) + c4;
                    float4 sum = *reinterpret_cast<const float4 *>(&dT[b * 1024 + at]);
#pragma unroll
                    for (int q = 1; q < F::KS; ++q) {
                        const float4 v = *reinterpret_cast<const float4 *>(&dT[(b + F::NB * q) * 1024 + at]);
                        sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
                    }
                    *reinterpret_cast<float4 *>(part2 + (size_t)slot * C::sB + (size_t)(32 * (b / F::RB) + row) * COLS + j2 * R +
                                                32 * (b % F::RB) + c4) = sum;
                }
                bo_lds_barrier();
            }
        }
    };

    // ---- prologue: the first tile's operands, the second tile's records ----
    {
        load_records(s_tlo[0]);
        publish_records(s_tn[0], 0);
        bo_lds_barrier();
        issue_operands(0);
        if (s_ti2[0] >= 0) fetch_bm(s_ti2[0], 0);
        if (tbeg + 1 < tend) load_records(s_tlo[1]);
        commit_operands(s_tn[0]);
        bo_lds_barrier();
    }
    int sc = 0;
    for (int tile = tbeg; tile < tend; ++tile, sc ^= 1) {
        const int i2 = s_ti2[tile - tbeg], n = s_tn[tile - tbeg];
        if (i2 < 0) break;                                                 // uniform
        const bool has_next = tile + 1 < tend;
        const int i2n = has_next ? s_ti2[tile + 1 - tbeg] : -1, nn = has_next ? s_tn[tile + 1 - tbeg] : 0;
        if (i2 != cur) {
            flush1();
            cur = i2; slot = tile;
#pragma unroll
            for (int j2 = 0; j2 < N2; ++j2)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc1[j2][r] = 0.f;
        }
        // the next tile: its records to LDS, its operands on their way, the records of the one after it too
        if (has_next) {
            publish_records(nn, sc ^ 1);
            bo_lds_barrier();
            issue_operands(sc ^ 1);
            if (tile + 2 < tend) load_records(s_tlo[tile + 2 - tbeg]);
        }

        mfma16_t accp[F::ABW];                                             // P: rows 32 rb .. 32 rb + 31, this wave's column blocks
#pragma unroll
        for (int ab = 0; ab < F::ABW; ++ab)
#pragma unroll
            for (int r = 0; r < 16; ++r) accp[ab][r] = 0.f;

#pragma unroll
        for (int j2 = 0; j2 < N2; ++j2) {
            // Bm[a][(j2, b)] to LDS (it came through registers: the part for the next j2, or for the next tile, is fetched
            // while the products of this one run)
#pragma unroll
            for (int q = 0; q < NB4; ++q) {
                const int i = q * WG + t, a = i / (R / 4), b4 = 4 * (i % (R / 4));
                *reinterpret_cast<float4 *>(Bl + a * LDB + b4) = make_float4(bm[q][0], bm[q][1], bm[q][2], bm[q][3]);
            }
            if (j2 + 1 < N2) fetch_bm(i2, j2 + 1);
            else if (i2n >= 0) fetch_bm(i2n, 0);
            // dT0'[(ee, j1)][b] for this j2
#pragma unroll
            for (int j1 = 0; j1 < N1; ++j1) {
                const float4 dy = *reinterpret_cast<const float4 *>(dyl + ee * N + (j1 * N2 + j2) * 4);
#pragma unroll
                for (int i = 0; i < F::BQ; ++i) {
                    dT[(ee * N1 + j1) * LDT + i * F::NBQ + bq] = fmaf(dy.x, cv[i][0], fmaf(dy.y, cv[i][1], fmaf(dy.z, cv[i][2], dy.w * cv[i][3])));
                }
            }
            bo_lds_barrier();
            // the part of dG2: block blk of the R x R result for this j2, over this wave's share of the 128 rows
            {
                constexpr int RW = F::ROWS / F::KS;
#pragma unroll
                for (int s = 0; s < RW / 2; ++s) {
                    const int row = ks * RW + kh * (RW / 2) + s;
                    acc1[j2] = __builtin_amdgcn_mfma_f32_32x32x2f32(As[row * LDA + 32 * ab1 + ln], dT[row * LDT + 32 * bb1 + ln],
                                                                   acc1[j2], 0, 0, 0);
                }
            }
            // P += dT0' Bm^T over the columns of this j2
#pragma unroll
            for (int s = 0; s < R / 2; s += 4) {
                const float2 av0 = *reinterpret_cast<const float2 *>(&dT[(32 * rb + ln) * LDT + kh * (R / 2) + s]);
                const float2 av1 = *reinterpret_cast<const float2 *>(&dT[(32 * rb + ln) * LDT + kh * (R / 2) + s + 2]);
#pragma unroll
                for (int ab = 0; ab < F::ABW; ++ab) {
                    const float4 bv = *reinterpret_cast<const float4 *>(&Bl[(32 * (ab0 + ab) + ln) * LDB + kh * (R / 2) + s]);
                    accp[ab] = __builtin_amdgcn_mfma_f32_32x32x2f32(av0.x, bv.x, accp[ab], 0, 0, 0);
                    accp[ab] = __builtin_amdgcn_mfma_f32_32x32x2f32(av0.y, bv.y, accp[ab], 0, 0, 0);
                    accp[ab] = __builtin_amdgcn_mfma_f32_32x32x2f32(av1.x, bv.z, accp[ab], 0, 0, 0);
                    accp[ab] = __builtin_amdgcn_mfma_f32_32x32x2f32(av1.y, bv.w, accp[ab], 0, 0, 0);
                }
            }
            bo_lds_barrier();                                               // dT0' and Bm are rewritten for the next j2
        }
        // the rows P of the positions: pbuf[k][j1][a]
#pragma unroll
        for (int ab = 0; ab < F::ABW; ++ab)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 32 * rb + 8 * (r / 4) + 4 * kh + r % 4, e = row / N1, j1 = row % N1;
                if (e < n) pbuf[((size_t)s_k[sc][e] * N1 + j1) * R + 32 * (ab0 + ab) + ln] = accp[ab][r];
            }
        if (has_next) commit_operands(nn);
        bo_lds_barrier();                                                   // the next tile's operands are in place; this tile's records are free
    }
    flush1();
}

// dst[i2] = src[i2] + mul * (sum of the parts of slice i2, in the order of their tiles); a slice without tiles is copied
// if dst is another array.  A workgroup takes BO_FIN float4 of a slice, two per thread, and every thread adds the parts
// of its float4 one after the other, eight in flight (a workgroup of the tile kernel adds consecutive tiles of a slice
// in registers, so a slice has few parts: a twentieth of its tiles at 100 positions per bag).  tile_base[i2] ..
// tile_base[i2 + 1] are the slice's tiles; only those that begin a stretch hold a part (the slice's first tile and
// every ch-th tile of the table, ch being the tiles per workgroup of bo_tile_kernel, which ran with nwg workgroups).
constexpr int BO_FIN = 2 * WG;

struct BoFinishArgs {
    int m2, slice4, ntiles, nwg;
    const int *tile_base;
    const float4 *part2, *src;
    float4 *dst;
};

__device__ __forceinline__ void bo_g2_finish_body(int vblock, const BoFinishArgs &a, float mul)
{
    constexpr int NF = BO_FIN / WG, NP = 8;
    const int m2 = a.m2, slice4 = a.slice4;
    const int *__restrict__ tile_base = a.tile_base;
    const float4 *__restrict__ part2 = a.part2, *__restrict__ src = a.src;
    float4 *__restrict__ dst = a.dst;
    const int ch = bo_chunk(min(a.ntiles, tile_base[m2]), a.nwg);            // as in bo_tile_kernel
    const int per = (slice4 + BO_FIN - 1) / BO_FIN;                          // workgroups per slice
    const int i2 = vblock / per, e0 = (vblock % per) * BO_FIN + threadIdx.x;
    if (i2 >= m2) return;
    const int t0 = tile_base[i2], t1 = tile_base[i2 + 1];
    const size_t base = (size_t)i2 * slice4;
    if (t1 <= t0) {                                                          // uniform
        if (dst != src) {
#pragma unroll
            for (int f = 0; f < NF; ++f)
                if (e0 + f * WG < slice4) dst[base + e0 + f * WG] = src[base + e0 + f * WG];
        }
        return;
    }
    // the parts: the stretch that begins with the slice, then those that begin at multiples of ch
    const int first_u = (t0 / ch + 1) * ch;
    const int nparts = first_u < t1 ? (t1 - first_u + ch - 1) / ch : 0;      // beyond the first one
    int e[NF];
    float4 sum[NF], old[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        e[f] = min(e0 + f * WG, slice4 - 1);                                 // (clamped: no load is conditional)
        sum[f] = part2[(size_t)t0 * slice4 + e[f]];
        old[f] = src[base + e[f]];
    }
    for (int jb = 0; jb < nparts; jb += NP) {                                // uniform
        float4 x[NF][NP];
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int u = first_u + min(jb + j, nparts - 1) * ch;
#pragma unroll
            for (int f = 0; f < NF; ++f) x[f][j] = part2[(size_t)u * slice4 + e[f]];
        }
#pragma unroll
        for (int j = 0; j < NP; ++j)
            if (jb + j < nparts) {
#pragma unroll
                for (int f = 0; f < NF; ++f) { sum[f].x += x[f][j].x; sum[f].y += x[f][j].y; sum[f].z += x[f][j].z; sum[f].w += x[f][j].w; }
            }
    }
#pragma unroll
    for (int f = 0; f < NF; ++f)
        if (e0 + f * WG < slice4)
            dst[base + e[f]] = make_float4(fmaf(mul, sum[f].x, old[f].x), fmaf(mul, sum[f].y, old[f].y), fmaf(mul, sum[f].z, old[f].z),
                                           fmaf(mul, sum[f].w, old[f].w));
}

// ---- segmented sums over the sorted items of the first and of the third core ----------------------
//
// Items [range[0], range[1]) of the sorted arrays have keys klo .. klo + slices - 1; the row of an item (ROW4 float4,
// lane l < ROW4 holds float4 l) comes from the producer.  One wave per tile of st items (bo_seg_st): runs of equal keys inside
// the tile are applied at once (dst[key] = src[key] + mul * sum), the part of a run that goes on in the next tile is
// left in part[tile][1], the part of a run that began in an earlier tile in part[tile][0] (a tile that is one run
// throughout: [0]); bo_seg_fix_kernel finishes the runs that cross tile borders.
// Items per wave: fewer for shorter streams, so that there are thousands of waves and each one's chain of dependent
// loads (a round trip per batch of items) stays short.  The host sizes the partial sums for bo_seg_st(L) items per
// wave; the kernels take the smallest power of two from 8 on with which the items in the range (known on the device
// only: cached positions have no items) still fit that many waves.
// (measured: 8,192 positions of the (4,4,4) shape at rank 64, 64 -> 8 items: 77 -> 27 us; 204,800 positions: 64 is best)
static inline int bo_seg_st(int64_t L) { return L >= 131072 ? 64 : (L >= 65536 ? 32 : (L >= 32768 ? 16 : 8)); }
__device__ __forceinline__ int bo_seg_st_dev(int n, int cap)
{
    int st = 8;
    while (st < 64 && (n + st - 1) / st > cap) st <<= 1;
    return st;
}

// The row of an item comes from a producer in two steps, so that a wave can have the loads of a whole batch of items
// in flight before it uses any of them (a producer that loads and computes in one go, under a test of the lane, makes
// every item a round trip of its own: 8 dependent trips per batch): issue() only loads, for every lane (a lane past
// the row loads what the row's last lane loads), finish() only computes.
//
// row of an item of the first core: the G1 gradient of its position, from pbuf
struct BoRowP {
    const float *pbuf;
    int row_floats;
    struct Raw { float v[4]; };
    __device__ __forceinline__ Raw issue(int k, int /*bag*/, int lane_c) const
    {
        const float4 x = *reinterpret_cast<const float4 *>(pbuf + (size_t)k * row_floats + 4 * lane_c);
        return Raw{{x.x, x.y, x.z, x.w}};
    }
    __device__ __forceinline__ float4 finish(const Raw &r, float /*w*/) const { return make_float4(r.v[0], r.v[1], r.v[2], r.v[3]); }
};

// row of an item of the third core: lane b holds sum_(j1,j2) T0_k[(j1,j2)][b] w dY[bag][(j1,j2)][0..3].  The
// upstream gradient row (N <= 64 values) is loaded one value per lane and handed round with readlane.
template <typename C>
struct BoRowT0 {
    const float *t0, *grad_out;
    static constexpr int NJ = C::N1 * C::N2;
    static_assert(C::N <= WAVE && (C::N & (C::N - 1)) == 0, "the upstream gradient row fits the lanes of a wave");
    struct Raw { float tv[NJ]; float dy; };
    __device__ __forceinline__ Raw issue(int k, int bag, int lane_c) const
    {
        Raw r;
        const float *T = t0 + (size_t)k * NJ * C::R + lane_c;
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) r.tv[jj] = T[jj * C::R];
        r.dy = grad_out[(size_t)bag * C::N + (threadIdx.x & (C::N - 1))];
        return r;
    }
    __device__ __forceinline__ float4 finish(const Raw &r, float w) const
    {
        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            const float tv = w * r.tv[jj];
            const float dx = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r.dy), 4 * jj + 0));
            const float dy = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r.dy), 4 * jj + 1));
            const float dz = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r.dy), 4 * jj + 2));
            const float dw = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r.dy), 4 * jj + 3));
            o.x = fmaf(tv, dx, o.x); o.y = fmaf(tv, dy, o.y); o.z = fmaf(tv, dz, o.z); o.w = fmaf(tv, dw, o.w);
        }
        return o;
    }
};

struct BoSegArgs {
    int row4, klo, cap;                                                      // cap: waves (tiles of items) that the partial sums have room for
    const int *range;
    const float *src;
    float *dst, *part;
};

template <int NBATCH, typename Producer>
__device__ __forceinline__ void bo_seg_body(int vblock, const Producer &prod, const BoSegArgs &a, int L, const uint64_t *__restrict__ ks,
                                            const int4 *__restrict__ info, const float *__restrict__ alpha, float mul)
{
    const int row4 = a.row4, klo = a.klo;
    const int *__restrict__ range = a.range;
    const float *__restrict__ src = a.src;
    float *__restrict__ dst = a.dst, *__restrict__ part = a.part;
    const int lane = threadIdx.x & 63;
    const int tile = vblock * NWAVE + (threadIdx.x >> 6);
    const int r0 = range[0], r1 = range[1];
    const int st = bo_seg_st_dev(r1 - r0, a.cap);
    const int i0 = r0 + tile * st;
    if (i0 >= r1 || tile >= a.cap) return;
    const int cnt = min(st, r1 - i0);
    const bool active = lane < row4;
    int my_key = -1, my_k = 0, my_bag = 0;
    float my_w = 0.f;
    if (lane < cnt) {
        my_key = (int)ks[i0 + lane];
        const int4 pi = info[i0 + lane];
        my_k = (unsigned)pi.x < (unsigned)L ? pi.x : 0;
        my_bag = pi.w;
        my_w = alpha ? alpha[my_k] : 1.f;
    }
    const int key_prev = i0 > r0 ? (int)ks[i0 - 1] : -1;
    const int key_next = i0 + cnt < r1 ? (int)ks[i0 + cnt] : -1;
    // the old value of a slice is only needed where a run ends
    const int my_end = (lane + 1 >= cnt || __shfl_down(my_key, 1) != my_key) ? 1 : 0;
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f), old_last = sum;
    int cur = __builtin_amdgcn_readfirstlane(my_key);
    bool first = cur == key_prev;                                          // the first run began in an earlier tile
    auto flush = [&](int key, bool goes_on) {
        if (active) {
            if (first) *reinterpret_cast<float4 *>(part + ((size_t)tile * 2 + 0) * 256 + 4 * lane) = sum;
            else if (goes_on) *reinterpret_cast<float4 *>(part + ((size_t)tile * 2 + 1) * 256 + 4 * lane) = sum;
            else
                *reinterpret_cast<float4 *>(dst + (size_t)(key - klo) * (4 * row4) + 4 * lane) =
                    make_float4(fmaf(mul, sum.x, old_last.x), fmaf(mul, sum.y, old_last.y), fmaf(mul, sum.z, old_last.z),
                                fmaf(mul, sum.w, old_last.w));
        }
        first = false;
        sum = make_float4(0.f, 0.f, 0.f, 0.f);
    };
    const int lane_c = min(lane, row4 - 1);                                  // (a lane past the row repeats the row's last lane: no load is conditional)
    for (int e0 = 0; e0 < cnt; e0 += NBATCH) {
        typename Producer::Raw raw[NBATCH];
        float old[NBATCH][4];
        // all loads of the batch first: the items' rows and the old values of their slices (needed where a run ends; the
        // few slices stay in the caches)
#pragma unroll
        for (int q = 0; q < NBATCH; ++q) {
            const int e = min(e0 + q, cnt - 1);
            const int key = __builtin_amdgcn_readlane(my_key, e), k = __builtin_amdgcn_readlane(my_k, e);
            const int bag = __builtin_amdgcn_readlane(my_bag, e);
            raw[q] = prod.issue(k, bag, lane_c);
            const float4 o4 = *reinterpret_cast<const float4 *>(src + (size_t)(key - klo) * (4 * row4) + 4 * lane_c);
            old[q][0] = o4.x; old[q][1] = o4.y; old[q][2] = o4.z; old[q][3] = o4.w;
        }
#pragma unroll
        for (int q = 0; q < NBATCH; ++q) {
            const int e = e0 + q;
            if (e < cnt) {                                                   // uniform
                const int key = __builtin_amdgcn_readlane(my_key, e);
                const float wgt = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_w), e));
                const float4 g = prod.finish(raw[q], wgt);
                if (key != cur) { flush(cur, false); cur = key; }
                sum.x += g.x; sum.y += g.y; sum.z += g.z; sum.w += g.w;
                if (__builtin_amdgcn_readlane(my_end, e)) old_last = make_float4(old[q][0], old[q][1], old[q][2], old[q][3]);
            }
        }
    }
    if (first || cur == key_next) flush(cur, true); else flush(cur, false);
}

// A run that crosses tile borders is applied by the workgroup of the tile where it begins: its own part[t][1], then
// part[u][0] of the later tiles that the run reaches (a later tile is reached if its first item still has the run's
// key), in tile order; a wave looks at 64 later tiles at a time.  A run over up to 16 later tiles is finished by its
// wave alone; a longer one (a hot row) by the four waves together, wave w adding every fourth part, 16 in flight, and
// the four sums are added in wave order.
__device__ __forceinline__ void bo_seg_fix_body(int vblock, const BoSegArgs &a, const uint64_t *__restrict__ ks, float mul)
{
    const int row4 = a.row4, klo = a.klo;
    const int *__restrict__ range = a.range;
    const float *__restrict__ src = a.src;
    float *__restrict__ dst = a.dst;
    const float *__restrict__ part = a.part;
    constexpr int NB = 16, SHORT = 16;
    __shared__ int s_long[NWAVE][2];                                         // key (-1: none) and last tile of a long run
    __shared__ float4 s_red[NWAVE][WAVE];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int tile = vblock * NWAVE + w;
    const int r0 = range[0], r1 = range[1];
    const int st = bo_seg_st_dev(r1 - r0, a.cap);
    const int ntiles = (r1 - r0 + st - 1) / st;
    const int i0 = r0 + tile * st, i1 = i0 + st;
    const bool active = lane < row4;
    int key = -1, last = tile;
    bool own = false;
    if (i1 < r1) {                                                           // else no tile here, or nothing to its right
        key = (int)ks[i1 - 1];
        own = (int)ks[i1] == key;                                            // the last run goes on in the next tile
        if (own && (int)ks[i0] == key && i0 > r0 && (int)ks[i0 - 1] == key) own = false;   // it began in an earlier tile
    }
    if (own) {                                                               // uniform in the wave
        for (int base = tile + 1; base < ntiles; base += WAVE) {
            const int u = base + lane;
            const bool in = u < ntiles && (int)ks[r0 + (size_t)u * st] == key;
            const unsigned long long b = __ballot(in);
            const int reach = b == ~0ull ? WAVE : __builtin_ctzll(~b);
            last = base + reach - 1;
            if (reach < WAVE) break;
        }
    }
    const bool is_long = own && last - tile > SHORT;
    if (lane == 0) { s_long[w][0] = is_long ? key : -1; s_long[w][1] = last; }
    if (own && !is_long) {
        float4 sum = active ? *reinterpret_cast<const float4 *>(part + ((size_t)tile * 2 + 1) * 256 + 4 * lane) : make_float4(0.f, 0.f, 0.f, 0.f);
        float4 x[SHORT];
#pragma unroll
        for (int j = 0; j < SHORT; ++j)
            x[j] = active ? *reinterpret_cast<const float4 *>(part + ((size_t)min(tile + 1 + j, last) * 2 + 0) * 256 + 4 * lane)
                          : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int j = 0; j < SHORT; ++j)
            if (tile + 1 + j <= last) { sum.x += x[j].x; sum.y += x[j].y; sum.z += x[j].z; sum.w += x[j].w; }
        if (active) {
            const size_t at = (size_t)(key - klo) * (4 * row4) + 4 * lane;
            const float4 old = *reinterpret_cast<const float4 *>(src + at);
            *reinterpret_cast<float4 *>(dst + at) =
                make_float4(fmaf(mul, sum.x, old.x), fmaf(mul, sum.y, old.y), fmaf(mul, sum.z, old.z), fmaf(mul, sum.w, old.w));
        }
    }
    __syncthreads();
    for (int q = 0; q < NWAVE; ++q) {                                        // long runs: uniform in the workgroup
        const int lkey = s_long[q][0];
        if (lkey < 0) continue;
        const int ltile = vblock * NWAVE + q, llast = s_long[q][1];
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
        if (w == 0 && active) sum = *reinterpret_cast<const float4 *>(part + ((size_t)ltile * 2 + 1) * 256 + 4 * lane);
        for (int u0 = ltile + 1 + w; u0 <= llast; u0 += NB * NWAVE) {
            float4 x[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j)
                x[j] = active ? *reinterpret_cast<const float4 *>(part + ((size_t)min(u0 + j * NWAVE, llast) * 2 + 0) * 256 + 4 * lane)
                              : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int j = 0; j < NB; ++j)
                if (u0 + j * NWAVE <= llast) { sum.x += x[j].x; sum.y += x[j].y; sum.z += x[j].z; sum.w += x[j].w; }
        }
        s_red[w][lane] = sum;
        __syncthreads();
        if (w == 0 && active) {
            float4 tot = s_red[0][lane];
#pragma unroll
            for (int ww = 1; ww < NWAVE; ++ww) { tot.x += s_red[ww][lane].x; tot.y += s_red[ww][lane].y; tot.z += s_red[ww][lane].z; tot.w += s_red[ww][lane].w; }
            const size_t at = (size_t)(lkey - klo) * (4 * row4) + 4 * lane;
            const float4 old = *reinterpret_cast<const float4 *>(src + at);
            *reinterpret_cast<float4 *>(dst + at) =
                make_float4(fmaf(mul, tot.x, old.x), fmaf(mul, tot.y, old.y), fmaf(mul, tot.z, old.z), fmaf(mul, tot.w, old.w));
        }
        __syncthreads();                                                     // s_red is written again for the next long run
    }
}

// What follows the tile kernel, in two launches instead of seven (the parts are independent of each other, so they
// fill the chip together): first the sums of the slice parts of the second core and the segmented sums of the first
// and of the third core, then the runs of those two that cross tile borders.  Block ranges: [0, nseg) third core (the
// longest part first), [nseg, 2 nseg) first core, [2 nseg, 2 nseg + nfin) slice parts of the second core.
template <typename C>
__global__ __launch_bounds__(WG) void bo_post_kernel(BoFinishArgs fin, int nfin, BoSegArgs s1, BoSegArgs s3, int nseg, BoRowP p1,
                                                     BoRowT0<C> p3, int L, const uint64_t *__restrict__ ks,
                                                     const int4 *__restrict__ info, const float *__restrict__ alpha, float mul)
{
    const int b = blockIdx.x;
    if (b < nseg) bo_seg_body<(C::N1 * C::N2 > 4 ? 4 : 8)>(b, p3, s3, L, ks, info, alpha, mul);
    else if (b < 2 * nseg) bo_seg_body<8>(b - nseg, p1, s1, L, ks, info, alpha, mul);
    else bo_g2_finish_body(b - 2 * nseg, fin, mul);
}

__global__ __launch_bounds__(WG) void bo_fix_kernel(BoSegArgs s1, BoSegArgs s3, int nseg, const uint64_t *__restrict__ ks, float mul)
{
    if ((int)blockIdx.x < nseg) bo_seg_fix_body(blockIdx.x, s1, ks, mul);
    else bo_seg_fix_body(blockIdx.x - nseg, s3, ks, mul);
}

// ---- host side -------------------------------------------------------------------------------------

// compute units of the current device (asked once)
static inline int bo_compute_units()
{
    static int cus = 0;
    if (!cus) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) cus = n;
        else cus = 256;
    }
    return cus;
}

static inline bool bwd_owner_supported(const Params &p)
{
    const int cfg = fast_config(p);
    return (cfg == 2 || cfg == 3 || cfg == 4 || cfg == 5) && p.m2 <= 4 * WG;
}

struct BoWs {
    float *part2;        // [tiles][sB]
    float *pbuf;         // [L][sA]
    float *seg1, *seg3;  // [L / bo_seg_st(L) + 2][2][256] each
    size_t bytes;
};

// tp: positions per tile (128 / n1, or 64 / n1 for short streams of the (4,4,4) shape at rank 64: see launch_bwd_owner)
static inline int bo_tiles(const Params &p, int64_t L, int tp) { return (int)((L + tp - 1) / tp) + p.m2; }

static inline BoWs bo_ws_layout(void *ws, const Params &p, int64_t L, int tp)
{
    BoWs b;
    char *base = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = base ? base + off : nullptr; off += (bytes + 255) & ~(size_t)255; return q; };
    const int64_t Lp = L > 0 ? L : 1;
    b.part2 = (float *)take((size_t)bo_tiles(p, Lp, tp) * p.sB * 4);
    b.pbuf = (float *)take((size_t)Lp * p.sA * 4);
    const size_t seg = (size_t)(Lp / bo_seg_st(Lp) + 2) * 2 * 256 * 4;
    b.seg1 = (float *)take(seg);
    b.seg3 = (float *)take(seg);
    b.bytes = off;
    return b;
}

// dst (o1..o3, or the gradient arrays if they are null) as described at the top.  crange[2..3]: the sorted range of
// the third core's items; the first core's items start the sorted arrays.
// Positions per tile.  Tiles of 128 stacked rows, except for short streams of the (4,4,4) shape at rank 64 (the
// Terabyte-shaped table: 8,192 positions over 200 slices are 328 tiles of 32 positions, two rounds on 256 compute
// units and a fifth of the rows empty): there tiles of 64 rows, two workgroups to a compute unit.  `small_ok` is
// false where the forward pass shares the tile table (it works on tiles of 128 rows).
static inline int bo_tp(const Params &p, int64_t L, bool small_ok)
{
    const bool small = small_ok && fast_config(p) == 5 && L < 32768;
    return (small ? 64 : 128) / p.n1;
}

template <typename C, int ROWS_>
static inline hipError_t launch_bo_tiles(const Params &p, const float *G1, const float *G2, const float *G3, int64_t L, int n_bags,
                                         const float *alpha, const float *go, float *o1, float *o3, const GroupWs &g, const BoWs &b,
                                         int ntiles, int *nwg_out, hipStream_t st)
{
    const size_t lds = bo_lds_bytes<C, ROWS_>();
    static bool allowed = false;                                             // (one device per process)
    if (!allowed) {
        hipError_t e = hipFuncSetAttribute((const void *)bo_tile_kernel<C, ROWS_>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        allowed = true;
    }
    // one or two workgroups per compute unit (what the tile's LDS and registers allow), more only where a workgroup would
    // get more tiles than it can hold descriptors of (the table's size is an upper bound of the tiles in use)
    int nwg = BoCfg<C, ROWS_>::WGS_PER_CU * bo_compute_units();
    if ((ntiles + BO_MAX_CHUNK - 1) / BO_MAX_CHUNK > nwg) nwg = (ntiles + BO_MAX_CHUNK - 1) / BO_MAX_CHUNK;
    hipLaunchKernelGGL((bo_tile_kernel<C, ROWS_>), dim3(nwg), dim3(WG), lds, st, p, G1, G2, G3, (int)L, n_bags, alpha, go, g.info,
                       g.tiles, ntiles, g.tile_base, b.part2, b.pbuf, (float4 *)o1, (float4 *)o3);
    *nwg_out = nwg;
    return hipSuccess;
}

template <typename C>
static inline hipError_t launch_bwd_owner(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx,
                                          int64_t L, const int64_t *off, int n_bags, const float *alpha, const float *go,
                                          const float *t0, float *dG1, float *dG2, float *dG3, float lr, float *o1, float *o2,
                                          float *o3, const uint64_t *ks, const uint32_t *vs, const GroupWs &g, const BoWs &b, int tp,
                                          hipStream_t st)
{
    const bool fused = o1 != nullptr;
    const float mul = fused ? -lr : 1.f;
    const int ntiles = bo_tiles(p, L, tp);
    int nwg = 0;
    hipError_t et;
    if constexpr (C::N1 == 4 && C::R == 64) {
        if (tp * C::N1 == 64)
            et = launch_bo_tiles<C, 64>(p, G1, G2, G3, L, n_bags, alpha, go, fused ? o1 : nullptr, fused ? o3 : nullptr, g, b, ntiles, &nwg, st);
        else
            et = launch_bo_tiles<C, 128>(p, G1, G2, G3, L, n_bags, alpha, go, fused ? o1 : nullptr, fused ? o3 : nullptr, g, b, ntiles, &nwg, st);
    } else {
        if (tp * C::N1 != 128) return hipErrorInvalidValue;
        et = launch_bo_tiles<C, 128>(p, G1, G2, G3, L, n_bags, alpha, go, fused ? o1 : nullptr, fused ? o3 : nullptr, g, b, ntiles, &nwg, st);
    }
    if (et != hipSuccess) return et;
    const int slice4 = C::sB / 4, per = (slice4 + BO_FIN - 1) / BO_FIN;
    const int sst = bo_seg_st(L);
    const int seg_tiles = (int)(L / sst + 1), nseg = (seg_tiles + NWAVE - 1) / NWAVE, nfin = p.m2 * per;
    const BoFinishArgs fin{p.m2, slice4, ntiles, nwg, g.tile_base, (const float4 *)b.part2, (const float4 *)(fused ? G2 : dG2),
                           (float4 *)(fused ? o2 : dG2)};
    // first core: items [crange[4], crange[5]) = [0, number of items of the first core); third core: [crange[2], crange[3])
    const BoSegArgs s1{C::sA / 4, 0, seg_tiles, g.crange + 4, fused ? G1 : dG1, fused ? o1 : dG1, b.seg1};
    const BoSegArgs s3{C::sC / 4, p.m1 + p.m2, seg_tiles, g.crange + 2, fused ? G3 : dG3, fused ? o3 : dG3, b.seg3};
    hipLaunchKernelGGL((bo_post_kernel<C>), dim3(nfin + 2 * nseg), dim3(WG), 0, st, fin, nfin, s1, s3, nseg, BoRowP{b.pbuf, C::sA},
                       BoRowT0<C>{t0, go}, (int)L, ks, g.info, alpha, mul);
    hipLaunchKernelGGL(bo_fix_kernel, dim3(2 * nseg), dim3(WG), 0, st, s1, s3, nseg, ks, mul);
    return hipGetLastError();
}

static inline hipError_t bwd_owner(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx,
                                   int64_t L, const int64_t *off, int n_bags, const float *alpha, const float *go, const float *t0,
                                   float *dG1, float *dG2, float *dG3, float lr, float *o1, float *o2, float *o3,
                                   const uint64_t *ks, const uint32_t *vs, const GroupWs &g, const BoWs &b, int tp, hipStream_t st)
{
    switch (fast_config(p)) {
    case 2: return launch_bwd_owner<Cfg224R32>(p, G1, G2, G3, idx, L, off, n_bags, alpha, go, t0, dG1, dG2, dG3, lr, o1, o2, o3, ks, vs, g, b, tp, st);
    case 3: return launch_bwd_owner<Cfg224R64>(p, G1, G2, G3, idx, L, off, n_bags, alpha, go, t0, dG1, dG2, dG3, lr, o1, o2, o3, ks, vs, g, b, tp, st);
    case 4: return launch_bwd_owner<Cfg444R32>(p, G1, G2, G3, idx, L, off, n_bags, alpha, go, t0, dG1, dG2, dG3, lr, o1, o2, o3, ks, vs, g, b, tp, st);
    case 5: return launch_bwd_owner<Cfg444R64>(p, G1, G2, G3, idx, L, off, n_bags, alpha, go, t0, dG1, dG2, dG3, lr, o1, o2, o3, ks, vs, g, b, tp, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tt
