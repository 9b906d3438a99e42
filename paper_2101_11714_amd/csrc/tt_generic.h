// Shape-generic kernels: correct for any (m, n, r) with d = 3, within the LDS
// budget.  The specialised kernels in tt_fast.h replace them for the shapes the
// paper uses; these remain the fallback and the in-library cross-check.
#pragma once

#include "tt_common.h"
#include "tt_select.h"

namespace tt {

constexpr int GEN_CH = 1024;     // positions scanned per selection round in the generic backward

// ---- forward (Eq. 3, Eq. 5-6; Alg. 1) -------------------------------------------
// One workgroup per bag (grid-stride).  LDS: A [sA] | C [sC] | T0 [n1*cols].
// Thread j < N owns output column j.  Requires N <= 256.
__global__ __launch_bounds__(WG) void fwd_generic_kernel(Params p, const float *__restrict__ G1,
                                                         const float *__restrict__ G2, const float *__restrict__ G3,
                                                         const int64_t *__restrict__ indices,
                                                         const int64_t *__restrict__ offsets, int n_bags,
                                                         const float *__restrict__ alpha, CacheDev cache,
                                                         float *__restrict__ out)
{
    extern __shared__ float smem[];
    float *sA = smem, *sC = sA + p.sA, *sT = sC + p.sC;
    const int t = threadIdx.x;
    for (int b = blockIdx.x; b < n_bags; b += gridDim.x) {
        const int k0 = offsets ? (int)offsets[b] : b;
        const int k1 = offsets ? (int)offsets[b + 1] : b + 1;
        float acc = 0.f;
        for (int k = k0; k < k1; ++k) {
            const uint32_t row = (uint32_t)indices[k];
            const float w = alpha ? alpha[k] : 1.f;
            const int slot = cache.K ? cache_probe(cache, row) : -1;
            if (slot >= 0) {                                     // uniform over the workgroup
                if (t < p.N) acc += w * cache.rows[(size_t)slot * p.N + t];
                continue;
            }
            int i1, i2, i3;
            decode(p, row, i1, i2, i3);
            const float *A = G1 + (size_t)i1 * p.sA;
            const float *B = G2 + (size_t)i2 * p.sB;
            const float *C = G3 + (size_t)i3 * p.sC;
            for (int e = t; e < p.sA; e += WG) sA[e] = A[e];
            for (int e = t; e < p.sC; e += WG) sC[e] = C[e];
            __syncthreads();
            // T0[j1][c] = sum_a A[j1][a] Bm[a][c]
            for (int e = t; e < p.n1 * p.cols; e += WG) {
                const int j1 = e / p.cols, c = e - j1 * p.cols;
                float s = 0.f;
                for (int a = 0; a < p.R1; ++a) s = fmaf(sA[j1 * p.R1 + a], B[a * p.cols + c], s);
                sT[e] = s;
            }
            __syncthreads();
            if (t < p.N) {                                       // y[q][j3] = sum_b T0[q][b] C[b][j3]
                const int q = t / p.n3, j3 = t - q * p.n3;
                float s = 0.f;
                for (int bb = 0; bb < p.R2; ++bb) s = fmaf(sT[q * p.R2 + bb], sC[bb * p.n3 + j3], s);
                acc += w * s;
            }
            __syncthreads();
        }
        if (t < p.N) out[(size_t)b * p.N + t] = acc;
    }
}

// ---- backward for the cores (Eq. 4; Alg. 2) ---------------------------------------
// Workgroup g owns one slice: g < m1 -> G1[g]; g < m1+m2 -> G2[g-m1]; else G3[g-m1-m2].
// It accumulates the slice gradient in LDS (each element has one owner thread) and adds
// it to grad_cores once.  LDS: SelectLds | ustart | acc [max slice] | A | C | T [n1*cols] | dY [N].
__global__ __launch_bounds__(WG) void bwd_generic_kernel(Params p, const float *__restrict__ G1,
                                                         const float *__restrict__ G2, const float *__restrict__ G3,
                                                         const int64_t *__restrict__ indices, int L,
                                                         const int64_t *__restrict__ offsets, int n_bags,
                                                         const float *__restrict__ alpha,
                                                         const int32_t *__restrict__ slot,
                                                         const float *__restrict__ grad_out,
                                                         float *__restrict__ dG1, float *__restrict__ dG2,
                                                         float *__restrict__ dG3)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    SelectLds<GEN_CH> &lds = *reinterpret_cast<SelectLds<GEN_CH> *>(smem_raw);
    const int max_slice = max(p.sA, max(p.sB, p.sC));
    int *ustart = reinterpret_cast<int *>(smem_raw + sizeof(SelectLds<GEN_CH>));
    float *acc = reinterpret_cast<float *>(ustart + GEN_CH + 4);
    float *sA = acc + max_slice, *sC = sA + p.sA, *sT = sC + p.sC, *sY = sT + p.n1 * p.cols;

    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    int role, s;
    {
        const int g = blockIdx.x;
        if (g < p.m1) { role = 0; s = g; }
        else if (g < p.m1 + p.m2) { role = 1; s = g - p.m1; }
        else { role = 2; s = g - p.m1 - p.m2; }
    }
    const int slice = role == 0 ? p.sA : (role == 1 ? p.sB : p.sC);
    for (int e = t; e < slice; e += WG) acc[e] = 0.f;
    bool any = false;

    for (int c0 = 0; c0 < L; c0 += GEN_CH) {
        const int c1 = min(L, c0 + GEN_CH);
        const int n = select_chunk<GEN_CH>(lds, c0, c1, [&](int k, uint32_t *val) {
            if (slot && slot[k] >= 0) return false;
            const uint32_t row = (uint32_t)indices[k];
            *val = row;
            return role_digit(p, role, row) == s;
        });
        if (n == 0) continue;                                    // uniform
        any = true;
        const int nu = sort_dedup<GEN_CH>(lds, n, ustart);
        for (int u = 0; u < nu; ++u) {
            const int d0 = ustart[u], d1 = ustart[u + 1];
            int i1, i2, i3;
            decode(p, lds.sr[d0], i1, i2, i3);
            const float *A = G1 + (size_t)i1 * p.sA;
            const float *B = G2 + (size_t)i2 * p.sB;
            const float *C = G3 + (size_t)i3 * p.sC;
            // dY = sum over the duplicates of alpha_k * grad_out[bag(k)], in list order
            if (t < p.N) {
                float g = 0.f;
                for (int d = d0; d < d1; ++d) {
                    const int k = lds.sk[d];
                    const int bag = bag_of(offsets, n_bags, k);
                    g += (alpha ? alpha[k] : 1.f) * grad_out[(size_t)bag * p.N + t];
                }
                sY[t] = g;
            }
            for (int e = t; e < p.sA; e += WG) sA[e] = A[e];
            for (int e = t; e < p.sC; e += WG) sC[e] = C[e];
            __syncthreads();
            if (role == 2) {
                // T0[j1][c] = sum_a A[j1][a] Bm[a][c];  dG3[b][j3] += sum_q T0[q][b] dY[q][j3]
                for (int e = t; e < p.n1 * p.cols; e += WG) {
                    const int j1 = e / p.cols, c = e - j1 * p.cols;
                    float sum = 0.f;
                    for (int a = 0; a < p.R1; ++a) sum = fmaf(sA[j1 * p.R1 + a], B[a * p.cols + c], sum);
                    sT[e] = sum;
                }
                __syncthreads();
                for (int e = t; e < p.sC; e += WG) {
                    const int bb = e / p.n3, j3 = e - bb * p.n3;
                    float sum = 0.f;
                    for (int q = 0; q < p.n1 * p.n2; ++q) sum = fmaf(sT[q * p.R2 + bb], sY[q * p.n3 + j3], sum);
                    acc[e] += sum;
                }
            } else {
                // dT0[q][b] = sum_j3 dY[q][j3] C[b][j3], stored as dT0'[j1][c]
                for (int e = t; e < p.n1 * p.cols; e += WG) {
                    const int q = e / p.R2, bb = e - q * p.R2;
                    float sum = 0.f;
                    for (int j3 = 0; j3 < p.n3; ++j3) sum = fmaf(sY[q * p.n3 + j3], sC[bb * p.n3 + j3], sum);
                    sT[e] = sum;
                }
                __syncthreads();
                if (role == 1) {
                    // dG2[a][c] += sum_j1 A[j1][a] dT0'[j1][c]
                    for (int e = t; e < p.sB; e += WG) {
                        const int a = e / p.cols, c = e - a * p.cols;
                        float sum = 0.f;
                        for (int j1 = 0; j1 < p.n1; ++j1) sum = fmaf(sA[j1 * p.R1 + a], sT[j1 * p.cols + c], sum);
                        acc[e] += sum;
                    }
                } else {
                    // dG1[j1][a] += sum_c dT0'[j1][c] Bm[a][c]: one wave per output, lanes over c
                    for (int e = w; e < p.sA; e += NWAVE) {
                        const int j1 = e / p.R1, a = e - j1 * p.R1;
                        float sum = 0.f;
                        for (int c = lane; c < p.cols; c += WAVE) sum = fmaf(sT[j1 * p.cols + c], B[a * p.cols + c], sum);
#pragma unroll
                        for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d);
                        if (lane == 0) acc[e] += sum;
                    }
                }
            }
            __syncthreads();
        }
    }
    if (any) {
        float *dst = role == 0 ? dG1 + (size_t)s * p.sA : (role == 1 ? dG2 + (size_t)s * p.sB : dG3 + (size_t)s * p.sC);
        __syncthreads();
        for (int e = t; e < slice; e += WG) dst[e] += acc[e];
    }
}

// ---- backward for the cached rows (Section 4.2) ------------------------------------
// Workgroup g owns the slots [g*G, g*G + G), G = max(1, 256 / N).  It scans the slot of
// every position, keeps the matches in order and adds alpha_k * grad_out[bag(k)] to the
// owned line.  LDS: SelectLds | acc [G*N].
__global__ __launch_bounds__(WG) void bwd_cache_kernel(int N, int K, int G, const int32_t *__restrict__ slot, int L,
                                                       const int64_t *__restrict__ offsets, int n_bags,
                                                       const float *__restrict__ alpha,
                                                       const float *__restrict__ grad_out,
                                                       float *__restrict__ grad_cache)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    SelectLds<GEN_CH> &lds = *reinterpret_cast<SelectLds<GEN_CH> *>(smem_raw);
    float *acc = reinterpret_cast<float *>(smem_raw + sizeof(SelectLds<GEN_CH>));
    const int t = threadIdx.x;
    const int g0 = blockIdx.x * G;
    const int g1 = min(K, g0 + G);
    for (int e = t; e < G * N; e += WG) acc[e] = 0.f;
    bool any = false;
    for (int c0 = 0; c0 < L; c0 += GEN_CH) {
        const int c1 = min(L, c0 + GEN_CH);
        const int n = select_chunk<GEN_CH>(lds, c0, c1, [&](int k, uint32_t *val) {
            const int sl = slot[k];
            *val = (uint32_t)(sl - g0);
            return sl >= g0 && sl < g1;
        });
        if (n == 0) continue;
        any = true;
        // lds.sk is free here: keep the bag of every match in it
        for (int i = t; i < n; i += WG) lds.sk[i] = bag_of(offsets, n_bags, lds.klist[i]);
        __syncthreads();
        for (int e = t; e < G * N; e += WG) {
            const int sl = e / N, j = e - sl * N;
            float sum = acc[e];
            for (int i = 0; i < n; ++i) {
                if ((int)lds.rows[i] == sl) {
                    const int k = lds.klist[i];
                    sum += (alpha ? alpha[k] : 1.f) * grad_out[(size_t)lds.sk[i] * N + j];
                }
            }
            acc[e] = sum;
        }
        __syncthreads();
    }
    if (any) {
        for (int e = t; e < (g1 - g0) * N; e += WG) grad_cache[(size_t)g0 * N + e] += acc[e];
    }
}

// ---- SGD (Section 5) ------------------------------------------------------------------
// x <- x - lr * g over up to four arrays in one launch (three cores and the cache lines).
// Work is split in float4 items (arrays are 16-byte aligned); the last count % 4 elements of
// an array are handled as scalars by the threads that follow the float4 items.
struct SgdArgs {
    float *x[4];
    float *g[4];
    int64_t count[4];
    int64_t start4[5];    // prefix sums of count / 4
    int64_t tail[5];      // prefix sums of count % 4
};

__global__ __launch_bounds__(WG) void sgd_kernel(SgdArgs a, float lr, int zero_grad)
{
    const int64_t total4 = a.start4[4], total = total4 + a.tail[4];
    for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < total; i += (int64_t)gridDim.x * WG) {
        if (i < total4) {
            int k = 0;
#pragma unroll
            for (int q = 1; q < 4; ++q) k += (i >= a.start4[q]);
            const int64_t e = i - a.start4[k];
            float4 *x = reinterpret_cast<float4 *>(a.x[k]) + e;
            float4 *g = reinterpret_cast<float4 *>(a.g[k]) + e;
            float4 xv = *x;
            const float4 gv = *g;
            xv.x = fmaf(-lr, gv.x, xv.x); xv.y = fmaf(-lr, gv.y, xv.y);
            xv.z = fmaf(-lr, gv.z, xv.z); xv.w = fmaf(-lr, gv.w, xv.w);
            *x = xv;
            if (zero_grad) *g = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
            const int64_t j = i - total4;
            int k = 0;
#pragma unroll
            for (int q = 1; q < 4; ++q) k += (j >= a.tail[q]);
            const int64_t e = (a.count[k] & ~(int64_t)3) + (j - a.tail[k]);
            a.x[k][e] = fmaf(-lr, a.g[k][e], a.x[k][e]);
            if (zero_grad) a.g[k][e] = 0.f;
        }
    }
}

__global__ __launch_bounds__(WG) void fill_i32_kernel(int32_t *__restrict__ p, int64_t n, int32_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < n; i += (int64_t)gridDim.x * WG) p[i] = v;
}

// Checks of the lookup arguments (Section 4.1): every index in [0, num_rows), offsets[0] == 0, offsets
// non-decreasing, offsets[n_bags] == L.  The bits of what fails are OR-ed into *flag (cleared before the launch).
__global__ __launch_bounds__(WG) void validate_kernel(int64_t num_rows, const int64_t *__restrict__ indices, int64_t L,
                                                      const int64_t *__restrict__ offsets, int64_t n_bags,
                                                      int32_t *__restrict__ flag)
{
    int bad = 0;
    const int64_t n = L > n_bags + 1 ? L : n_bags + 1;
    for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < n; i += (int64_t)gridDim.x * WG) {
        if (i < L) {
            const int64_t row = indices[i];
            if (row < 0 || row >= num_rows) bad |= 1;
        }
        if (offsets && i <= n_bags) {
            const int64_t o = offsets[i];
            if (i == 0 ? o != 0 : o < offsets[i - 1]) bad |= 2;
            if (o < 0 || o > L || (i == n_bags && o != L)) bad |= 4;
        }
    }
    // one atomic per wave that found something
    int wave_bad = 0;
    for (int b = 1; b <= 4; b <<= 1)
        if (__ballot((bad & b) != 0) != 0) wave_bad |= b;
    if (wave_bad && (threadIdx.x & (WAVE - 1)) == 0) atomicOr(flag, wave_bad);
}

// A launch that does nothing (one store by one thread if sink is given): what a kernel costs before it computes.
__global__ __launch_bounds__(WG) void launch_probe_kernel(int32_t *__restrict__ sink)
{
    if (sink && blockIdx.x == 0 && threadIdx.x == 0) *sink = 1;
}

__global__ __launch_bounds__(WG) void fill_f32_kernel(float *__restrict__ p, int64_t n, float v)
{
    for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < n; i += (int64_t)gridDim.x * WG) p[i] = v;
}

// out = x - lr * g (out may be x itself)
__global__ __launch_bounds__(WG) void sgd_out_kernel(const float *x, const float *__restrict__ g, float *out, int64_t n,
                                                     float lr)
{
    for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < n; i += (int64_t)gridDim.x * WG)
        out[i] = fmaf(-lr, g[i], x[i]);
}

// w[k] = alpha[k] / (length of the bag of k): the weights that turn sum pooling into mean pooling.
// One wave per bag.
__global__ __launch_bounds__(WG) void mean_weights_kernel(const int64_t *__restrict__ offsets, int n_bags,
                                                          const float *__restrict__ alpha, float *__restrict__ w)
{
    const int lane = threadIdx.x & 63;
    const int bag = blockIdx.x * NWAVE + (threadIdx.x >> 6);
    if (bag >= n_bags) return;
    const int64_t k0 = offsets[bag], k1 = offsets[bag + 1];
    const float len = (float)(k1 - k0);
    for (int64_t k = k0 + lane; k < k1; k += WAVE) w[k] = (alpha ? alpha[k] : 1.f) / len;
}

// ---- cache map --------------------------------------------------------------------------

__global__ __launch_bounds__(WG) void fill_u64_kernel(uint64_t *__restrict__ p, int64_t n, uint64_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < n; i += (int64_t)gridDim.x * WG) p[i] = v;
}

// table[h(row)] = (row << 32 | slot) with linear probing; rows are distinct.
__global__ __launch_bounds__(WG) void cache_insert_kernel(const int64_t *__restrict__ keys, int K,
                                                          uint64_t *__restrict__ table, uint32_t mask)
{
    const int s = blockIdx.x * WG + threadIdx.x;
    if (s >= K) return;
    const uint32_t row = (uint32_t)keys[s];
    const uint64_t entry = ((uint64_t)row << 32) | (uint32_t)s;
    uint32_t h = cache_hash(row, mask);
    for (;;) {                                    // ends: capacity >= 2K, so an empty entry exists
        const unsigned long long old = atomicCAS((unsigned long long *)&table[h], (unsigned long long)CACHE_EMPTY,
                                                 (unsigned long long)entry);
        if (old == (unsigned long long)CACHE_EMPTY) return;
        h = (h + 1) & mask;
    }
}

__global__ __launch_bounds__(WG) void cache_lookup_kernel(CacheDev c, const int64_t *__restrict__ indices, int L,
                                                          int32_t *__restrict__ slot)
{
    const int k = blockIdx.x * WG + threadIdx.x;
    if (k < L) slot[k] = c.K ? cache_probe(c, (uint32_t)indices[k]) : -1;
}

// ---- integer exports ------------------------------------------------------------------------

__global__ __launch_bounds__(WG) void decode_kernel(Params p, const int64_t *__restrict__ indices, int L,
                                                    int32_t *__restrict__ o1, int32_t *__restrict__ o2,
                                                    int32_t *__restrict__ o3)
{
    const int k = blockIdx.x * WG + threadIdx.x;
    if (k >= L) return;
    int i1, i2, i3;
    decode(p, (uint32_t)indices[k], i1, i2, i3);
    o1[k] = i1; o2[k] = i2; o3[k] = i3;
}

// The digits as the other decoders of the library produce them, for the bit-exact tests:
// mode 1: decode_f64 (run detection of the backward's owners);  mode 2: what an owner's
// selection decides: i2 and i3 from select_digit_f64, i1 = the slice s among (integer i1) - 1,
// i1, i1 + 1 whose row range holds the row (-1: none does, -2: more than one does).
__global__ __launch_bounds__(WG) void decode_as_kernel(Params p, const int64_t *__restrict__ indices, int L, int mode,
                                                       int32_t *__restrict__ o1, int32_t *__restrict__ o2,
                                                       int32_t *__restrict__ o3)
{
    const int k = blockIdx.x * WG + threadIdx.x;
    if (k >= L) return;
    const uint32_t row = (uint32_t)indices[k];
    int i1, i2, i3;
    if (mode == 1) {
        decode_f64(p, row, i1, i2, i3);
    } else {
        int g1, g2, g3;
        decode(p, row, g1, g2, g3);
        i1 = -1;
        for (int s = g1 - 1; s <= g1 + 1; ++s)
            if (s >= 0 && s < p.m1 && in_rows(rows_of_i1(p, s), row)) i1 = i1 == -1 ? s : -2;
        i2 = (int)select_digit_f64(p, 1, (double)row);
        i3 = (int)select_digit_f64(p, 2, (double)row);
    }
    o1[k] = i1; o2[k] = i2; o3[k] = i3;
}

// keys[k] = row id (which = 0) or digit (which = 1..3) of indices[k]; skipped positions get `sentinel`.
__global__ __launch_bounds__(WG) void dedup_keys_kernel(Params p, const int64_t *__restrict__ indices, int L,
                                                        const int32_t *__restrict__ slot, int which,
                                                        uint64_t sentinel, uint64_t *__restrict__ keys)
{
    const int k = blockIdx.x * WG + threadIdx.x;
    if (k >= L) return;
    const uint32_t row = (uint32_t)indices[k];
    uint64_t key = row;
    if (which > 0) {
        int i1, i2, i3;
        decode(p, row, i1, i2, i3);
        key = (uint64_t)(which == 1 ? i1 : (which == 2 ? i2 : i3));
    }
    if (slot && slot[k] >= 0) key = sentinel;
    keys[k] = key;
}

__global__ __launch_bounds__(WG) void copy_perm_kernel(const uint32_t *__restrict__ v, int n, int32_t *__restrict__ perm)
{
    const int i = blockIdx.x * WG + threadIdx.x;
    if (i < n) perm[i] = (int32_t)v[i];
}

// Candidate (row, count) -> sort key: most used first, then lower row id (Section 4.2, ties by row).
__global__ __launch_bounds__(WG) void cand_keys_kernel(const int64_t *__restrict__ rows, const int64_t *__restrict__ counts,
                                                       int n, uint64_t *__restrict__ keys)
{
    const int i = blockIdx.x * WG + threadIdx.x;
    if (i >= n) return;
    const uint64_t c = (uint64_t)counts[i];
    const uint32_t inv = 0xFFFFFFFFu - (uint32_t)(c > 0xFFFFFFFFull ? 0xFFFFFFFFull : c);
    keys[i] = ((uint64_t)inv << 32) | (uint32_t)rows[i];
}

__global__ __launch_bounds__(WG) void take_keys_kernel(const uint64_t *__restrict__ sorted, int K, int64_t *__restrict__ keys)
{
    const int s = blockIdx.x * WG + threadIdx.x;
    if (s < K) keys[s] = (int64_t)(uint32_t)sorted[s];
}

}  // namespace tt
