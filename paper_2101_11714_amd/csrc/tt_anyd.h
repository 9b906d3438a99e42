// TT-EmbeddingBag for any number of cores d in {2, 3, 4} (Section 4.1 of the paper: Alg. 1 and 2
// are written for three cores and generalise by extending the chain of products).  Plain
// kernels: correct and deterministic, not tuned; the three-core shapes of the paper's workloads
// have their own kernels.  No cache.
//
// Core k (k = 0..d-1) is stored [m_k][r_k][n_k][r_{k+1}], r_0 = r_d = 1; row digits are mixed
// radix with i_0 most significant; the product of the first k slices is kept as a matrix
// (n_0 .. n_{k-1}) x r_k, reshaped row-major before the next multiply (Eq. 3).
#pragma once

#include "tt_common.h"

namespace tt {

constexpr int DMAX = 4;
constexpr int DBUF = 4096;                      // floats per LDS buffer: bounds every intermediate

struct ShapeD {
    int d;
    int m[DMAX], n[DMAX], r[DMAX + 1];
    int slice[DMAX];                            // r_k n_k r_{k+1}
    int N;
};

__device__ __forceinline__ void digits_d(const ShapeD &s, uint32_t row, int (&dig)[DMAX])
{
#pragma unroll
    for (int k = DMAX - 1; k >= 0; --k) {
        if (k < s.d) {
            dig[k] = (int)(row % (uint32_t)s.m[k]);
            row /= (uint32_t)s.m[k];
        } else {
            dig[k] = 0;
        }
    }
}

// dst ((np n_k) x r_{k+1}) = src (np x r_k) . slice (r_k x n_k r_{k+1}); src, dst in LDS, slice in global memory
__device__ __forceinline__ void chain_right(const float *src, float *dst, const float *__restrict__ g, int np, int rk,
                                            int nk, int rk1)
{
    const int cols = nk * rk1;
    for (int e = threadIdx.x; e < np * cols; e += WG) {
        const int jp = e / cols, c = e - jp * cols;
        float sum = 0.f;
        for (int a = 0; a < rk; ++a) sum = fmaf(src[jp * rk + a], g[a * cols + c], sum);
        dst[e] = sum;                            // e = (jp * n_k + j_k) * r_{k+1} + b
    }
}

// dst (r_k x (n_k nr)) = slice (r_k n_k x r_{k+1}) . src (r_{k+1} x nr)
__device__ __forceinline__ void chain_left(const float *src, float *dst, const float *__restrict__ g, int rk, int nk,
                                           int rk1, int nr)
{
    for (int e = threadIdx.x; e < rk * nk * nr; e += WG) {
        const int aj = e / nr, jr = e - aj * nr;         // aj = a * n_k + j_k
        float sum = 0.f;
        for (int b = 0; b < rk1; ++b) sum = fmaf(g[aj * rk1 + b], src[b * nr + jr], sum);
        dst[e] = sum;                            // e = a * (n_k nr) + j_k * nr + jr
    }
}

__global__ __launch_bounds__(WG) void fwd_anyd_kernel(ShapeD s, const float *__restrict__ g0, const float *__restrict__ g1,
                                                      const float *__restrict__ g2, const float *__restrict__ g3,
                                                      const int64_t *__restrict__ indices,
                                                      const int64_t *__restrict__ offsets, int n_bags,
                                                      const float *__restrict__ alpha, float *__restrict__ out)
{
    __shared__ float buf[2][DBUF];
    const float *g[DMAX] = {g0, g1, g2, g3};
    const int t = threadIdx.x;
    constexpr int NACC = DBUF / WG;              // N <= DBUF
    for (int bag = blockIdx.x; bag < n_bags; bag += gridDim.x) {
        float acc[NACC];
#pragma unroll
        for (int i = 0; i < NACC; ++i) acc[i] = 0.f;
        const int k0 = offsets ? (int)offsets[bag] : bag, k1 = offsets ? (int)offsets[bag + 1] : bag + 1;
        for (int k = k0; k < k1; ++k) {
            int dig[DMAX];
            digits_d(s, (uint32_t)indices[k], dig);
            const float w = alpha ? alpha[k] : 1.f;
            __syncthreads();                     // the buffers are free again
            for (int e = t; e < s.slice[0]; e += WG) buf[0][e] = g[0][(size_t)dig[0] * s.slice[0] + e];
            int cur = 0, np = s.n[0];
#pragma unroll
            for (int q = 1; q < DMAX; ++q) {
                if (q < s.d) {
                    __syncthreads();
                    chain_right(buf[cur], buf[cur ^ 1], g[q] + (size_t)dig[q] * s.slice[q], np, s.r[q], s.n[q], s.r[q + 1]);
                    cur ^= 1;
                    np *= s.n[q];
                }
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NACC; ++i)
                if (t + i * WG < s.N) acc[i] = fmaf(w, buf[cur][t + i * WG], acc[i]);
        }
#pragma unroll
        for (int i = 0; i < NACC; ++i)
            if (t + i * WG < s.N) out[(size_t)bag * s.N + t + i * WG] = acc[i];
    }
}

// One workgroup per slice of every core.  It scans the positions WG at a time, keeps those whose
// digit selects its slice (in order), and handles them one after the other:
//   left  = product of the slices before core k      ((n_<k) x r_k)
//   right = product of the slices after core k       (r_{k+1} x (n_>k))
//   T[a][j_k][j_>] = sum_{j_<} left[j_<][a] dY[j_<, j_k, j_>]
//   dG_k[a][j_k][b] += sum_{j_>} T[a][j_k][j_>] right[b][j_>]
// The slice gradient is accumulated in LDS and added to grad once.
__global__ __launch_bounds__(WG) void bwd_anyd_kernel(ShapeD s, const float *__restrict__ g0, const float *__restrict__ g1,
                                                      const float *__restrict__ g2, const float *__restrict__ g3,
                                                      const int64_t *__restrict__ indices, int L,
                                                      const int64_t *__restrict__ offsets, int n_bags,
                                                      const float *__restrict__ alpha, const float *__restrict__ grad_out,
                                                      float *__restrict__ d0, float *__restrict__ d1,
                                                      float *__restrict__ d2, float *__restrict__ d3)
{
    __shared__ float bl[2][DBUF], br[2][DBUF], bt[DBUF], accum[DBUF];
    __shared__ int list[WG];
    __shared__ int tmp[NWAVE + 1];
    const float *g[DMAX] = {g0, g1, g2, g3};
    float *dg[DMAX] = {d0, d1, d2, d3};
    const int t = threadIdx.x;
    // which core and slice
    int core = 0, sl = blockIdx.x;
#pragma unroll
    for (int k = 0; k < DMAX - 1; ++k)
        if (core == k && k + 1 < s.d && sl >= s.m[k]) { sl -= s.m[k]; core = k + 1; }
    const int ssz = s.slice[core];
    for (int e = t; e < ssz; e += WG) accum[e] = 0.f;
    bool any = false;
    for (int base = 0; base < L; base += WG) {
        const int k = base + t;
        int dig[DMAX];
        bool hit = false;
        if (k < L) {
            digits_d(s, (uint32_t)indices[k], dig);
            int mine = 0;
#pragma unroll
            for (int q = 0; q < DMAX; ++q) mine = q == core ? dig[q] : mine;
            hit = mine == sl;
        }
        int total;
        const int pos = block_excl_scan(hit ? 1 : 0, tmp, &total);
        if (hit) list[pos] = k;
        __syncthreads();
        for (int i = 0; i < total; ++i) {                          // uniform
            any = true;
            const int kk = list[i];
            int dg2[DMAX];
            digits_d(s, (uint32_t)indices[kk], dg2);
            const int bag = bag_of(offsets, n_bags, kk);
            const float w = alpha ? alpha[kk] : 1.f;
            // left
            int lcur = 0, nl = 1;
            if (t == 0) bl[0][0] = 1.f;
#pragma unroll
            for (int q = 0; q < DMAX; ++q) {
                if (q < core) {
                    __syncthreads();
                    chain_right(bl[lcur], bl[lcur ^ 1], g[q] + (size_t)dg2[q] * s.slice[q], nl, s.r[q], s.n[q], s.r[q + 1]);
                    lcur ^= 1;
                    nl *= s.n[q];
                }
            }
            // right
            int rcur = 0, nr = 1;
            if (t == 0) br[0][0] = 1.f;
#pragma unroll
            for (int q = DMAX - 1; q >= 1; --q) {
                if (q < s.d && q > core) {
                    __syncthreads();
                    chain_left(br[rcur], br[rcur ^ 1], g[q] + (size_t)dg2[q] * s.slice[q], s.r[q], s.n[q], s.r[q + 1], nr);
                    rcur ^= 1;
                    nr *= s.n[q];
                }
            }
            __syncthreads();
            const int rk = s.r[core], nk = s.n[core], rk1 = s.r[core + 1];
            const float *dy = grad_out + (size_t)bag * s.N;
            // T[a][j_k][j_>]
            for (int e = t; e < rk * nk * nr; e += WG) {
                const int a = e / (nk * nr), rest = e - a * (nk * nr);   // rest = j_k * nr + j_>
                float sum = 0.f;
                for (int jl = 0; jl < nl; ++jl) sum = fmaf(bl[lcur][jl * rk + a], dy[jl * (nk * nr) + rest], sum);
                bt[e] = w * sum;
            }
            __syncthreads();
            for (int e = t; e < ssz; e += WG) {                    // e = (a * n_k + j_k) * r_{k+1} + b
                const int aj = e / rk1, b = e - aj * rk1;
                float sum = 0.f;
                for (int jr = 0; jr < nr; ++jr) sum = fmaf(bt[aj * nr + jr], br[rcur][b * nr + jr], sum);
                accum[e] += sum;
            }
            __syncthreads();
        }
        __syncthreads();                                           // before the list is rebuilt
    }
    if (any) {
        float *dst = dg[core] + (size_t)sl * ssz;
        for (int e = t; e < ssz; e += WG) dst[e] += accum[e];
    }
}

__global__ __launch_bounds__(WG) void sgd_plain_kernel(float *__restrict__ x, float *__restrict__ gr, int64_t n, float lr,
                                                       int zero_grad)
{
    for (int64_t i = (int64_t)blockIdx.x * WG + threadIdx.x; i < n; i += (int64_t)gridDim.x * WG) {
        x[i] = fmaf(-lr, gr[i], x[i]);
        if (zero_grad) gr[i] = 0.f;
    }
}

}  // namespace tt
