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
// One wave per bag.  The partial products of stage 1 are accumulated over the bag's
// lookups (and cached rows are added on the lane with b0 = 0) before one shuffle
// reduction per bag.
template <typename C>
__global__ __launch_bounds__(WG) void fwd_fast_kernel(Params p, const float *__restrict__ G1,
                                                      const float *__restrict__ G2, const float *__restrict__ G3,
                                                      const int64_t *__restrict__ indices,
                                                      const int64_t *__restrict__ offsets, int n_bags,
                                                      const float *__restrict__ alpha, CacheDev cache,
                                                      float *__restrict__ out)
{
    constexpr int N1 = C::N1, N2 = C::N2, N3 = C::N3, R = C::R, V = C::V;
    const int lane = threadIdx.x & 63;
    const int bag = __builtin_amdgcn_readfirstlane(blockIdx.x * NWAVE + (threadIdx.x >> 6));
    if (bag >= n_bags) return;
    const bool active = lane < C::LANES;
    const int c0 = active ? lane * V : 0;
    const int j2 = c0 / R, b0 = c0 % R;
    float acc[C::NV];
#pragma unroll
    for (int i = 0; i < C::NV; ++i) acc[i] = 0.f;

    const int k0 = offsets ? (int)offsets[bag] : bag;
    const int k1 = offsets ? (int)offsets[bag + 1] : bag + 1;
    for (int k = k0; k < k1; ++k) {
        const uint32_t row = (uint32_t)__builtin_amdgcn_readfirstlane((int)indices[k]);
        const float w = alpha ? alpha[k] : 1.f;
        if (cache.K) {
            const int slot = __builtin_amdgcn_readfirstlane(cache_probe(cache, row));
            if (slot >= 0) {
                if (active && b0 == 0) {
                    const float *cr = cache.rows + (size_t)slot * C::N + j2 * N3;
#pragma unroll
                    for (int j1 = 0; j1 < N1; ++j1) {
                        const float4 t = *reinterpret_cast<const float4 *>(cr + j1 * N2 * N3);
                        acc[j1 * N3 + 0] = fmaf(w, t.x, acc[j1 * N3 + 0]);
                        acc[j1 * N3 + 1] = fmaf(w, t.y, acc[j1 * N3 + 1]);
                        acc[j1 * N3 + 2] = fmaf(w, t.z, acc[j1 * N3 + 2]);
                        acc[j1 * N3 + 3] = fmaf(w, t.w, acc[j1 * N3 + 3]);
                    }
                }
                continue;
            }
        }
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
    }
    group_reduce<C::NV, C::LN>(acc, lane);
    constexpr int KEEP = ReduceKeep<C::NV, C::LN>::value;
    const int lg = lane % C::LN;
    if (active && lg < ReduceKeep<C::NV, C::LN>::writers) {
        const int base = reduce_base<C::NV, C::LN>(lane);
        float *o = out + (size_t)bag * C::N;
#pragma unroll
        for (int i = 0; i < KEEP; ++i) {
            const int idx = base + i;                       // = j1 * N3 + j3
            const int j1 = idx / N3, j3 = idx % N3;
            o[(j1 * N2 + j2) * N3 + j3] = acc[i];
        }
    }
}

// ---- backward --------------------------------------------------------------------
// One workgroup owns one core slice (see bwd_generic_kernel).  After the selection
// and the sort by row, the sorted list is cut into windows of W entries.  For each
// window the workgroup stages alpha_k * grad_out[bag(k)] of every entry in LDS, sums
// the runs of equal rows (a run cut by a window border is simply handled as two rows,
// the gradient being linear in dY), and then all four waves walk over the runs; wave w
// owns the rows a in [w RQ, (w+1) RQ) of the unfolded G2 slice, so that
//   G2 owner: dG2[a][c]  += sum_j1 A[j1][a] dT0'[j1][c]            (no G2 read at all)
//   G1 owner: dG1[j1][a] += sum_c dT0'[j1][c] Bm[a][c]            (lane partials, one reduction at the end)
//   G3 owner: dG3[b][j3] += sum_{j1,j2} T0[(j1,j2)][b] dY[..][j3]  (T0 partial over the wave's rows a)
// with dT0'[j1][c] = sum_j3 dY[(j1,j2)][j3] C[b][j3].
constexpr int FAST_CH = 2048;

template <typename C>
struct FastBwdLds {
    static constexpr int W = 4096 / C::N;           // entries per window: 16 KB of staged gradients
    SelectLds<FAST_CH> sel;                          // sel.klist / sel.rows double as the staging area
    float dys[W * C::N];                             // summed dY of every run of the window
    int seg_start[W + 1];
    static_assert(sizeof(int) * FAST_CH * 2 >= sizeof(float) * W * C::N, "staging area too small");
};

// bag of position k: try the evenly-spaced guess first, fall back to a binary search.
__device__ __forceinline__ int bag_guess(const int64_t *__restrict__ offsets, int n_bags, int L, int k)
{
    if (!offsets) return k;
    int g = (int)(((int64_t)k * n_bags) / L);
    if (g >= n_bags) g = n_bags - 1;
    if (offsets[g] <= (int64_t)k && (int64_t)k < offsets[g + 1]) return g;
    return bag_of(offsets, n_bags, k);
}

template <typename C>
__global__ __launch_bounds__(WG) void bwd_fast_kernel(Params p, const float *__restrict__ G1,
                                                      const float *__restrict__ G2, const float *__restrict__ G3,
                                                      const int64_t *__restrict__ indices, int L,
                                                      const int64_t *__restrict__ offsets, int n_bags,
                                                      const float *__restrict__ alpha,
                                                      const int32_t *__restrict__ slot,
                                                      const float *__restrict__ grad_out,
                                                      float *__restrict__ dG1, float *__restrict__ dG2,
                                                      float *__restrict__ dG3)
{
    constexpr int N1 = C::N1, N2 = C::N2, N3 = C::N3, R = C::R, V = C::V, N = C::N, RQ = C::RQ;
    constexpr int W = FastBwdLds<C>::W, NQ = N / 4;
    __shared__ FastBwdLds<C> lds;
    float *stage = reinterpret_cast<float *>(lds.sel.klist);

    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int a0 = w * RQ;
    int role, s;
    {
        const int g = blockIdx.x;
        if (g < p.m1) { role = 0; s = g; }
        else if (g < p.m1 + p.m2) { role = 1; s = g - p.m1; }
        else { role = 2; s = g - p.m1 - p.m2; }
    }
    const bool active = lane < C::LANES;
    const int c0 = active ? lane * V : 0;
    const int j2 = c0 / R, b0 = c0 % R;

    // accumulators of the three roles (only one set is live in a given workgroup)
    float acc2[RQ][V];           // G2 owner: dG2[a0+aa][c0+v]
    float acc1[N1 * RQ];         // G1 owner: lane partial of dG1[j1][a0+aa], index j1*RQ+aa
    float acc3[V][N3];           // G3 owner: partial of dG3[b0+v][j3] over (this j2, this wave's a)
#pragma unroll
    for (int aa = 0; aa < RQ; ++aa)
#pragma unroll
        for (int v = 0; v < V; ++v) acc2[aa][v] = 0.f;
#pragma unroll
    for (int i = 0; i < N1 * RQ; ++i) acc1[i] = 0.f;
#pragma unroll
    for (int v = 0; v < V; ++v)
#pragma unroll
        for (int j3 = 0; j3 < N3; ++j3) acc3[v][j3] = 0.f;
    bool any = false;

    for (int ch0 = 0; ch0 < L; ch0 += FAST_CH) {
        const int ch1 = min(L, ch0 + FAST_CH);
        const int n = select_chunk<FAST_CH>(lds.sel, ch0, ch1, [&](int k, uint32_t *val) {
            if (slot && slot[k] >= 0) return false;
            const uint32_t row = (uint32_t)indices[k];
            *val = row;
            return role_digit(p, role, row) == s;
        });
        if (n == 0) continue;
        any = true;
        sort_by_row(lds.sel, n);

        for (int i0 = 0; i0 < n; i0 += W) {
            const int nw = min(W, n - i0);
            // 1. runs of equal rows inside the window (W <= 256: one thread per entry)
            int nsegs;
            {
                bool head = false;
                if (t < nw) head = (t == 0) || lds.sel.sr[i0 + t] != lds.sel.sr[i0 + t - 1];
                const int ex = block_excl_scan(head ? 1 : 0, lds.sel.scan_tmp, &nsegs);
                if (head) lds.seg_start[ex] = t;
                if (t == 0) lds.seg_start[nsegs] = nw;
            }
            // 2. stage alpha_k * grad_out[bag(k)] of every entry (float4 per thread and step)
            for (int item = t; item < nw * NQ; item += WG) {
                const int e = item / NQ, q = item - e * NQ;
                const int k = lds.sel.sk[i0 + e];
                const int bag = bag_guess(offsets, n_bags, L, k);
                const float wk = alpha ? alpha[k] : 1.f;
                float4 g = *reinterpret_cast<const float4 *>(grad_out + (size_t)bag * N + 4 * q);
                g.x *= wk; g.y *= wk; g.z *= wk; g.w *= wk;
                *reinterpret_cast<float4 *>(stage + e * N + 4 * q) = g;
            }
            __syncthreads();
            // 3. sum the runs, in list order
            for (int item = t; item < nsegs * N; item += WG) {
                const int sg = item / N, j = item - sg * N;
                const int e0 = lds.seg_start[sg], e1 = lds.seg_start[sg + 1];
                float sum = 0.f;
                for (int e = e0; e < e1; ++e) sum += stage[e * N + j];
                lds.dys[item] = sum;
            }
            __syncthreads();
            // 4. the waves walk over the runs
            for (int sg = 0; sg < nsegs; ++sg) {
                const uint32_t row = lds.sel.sr[i0 + lds.seg_start[sg]];
                int i1, i2, i3;
                decode(p, (uint32_t)__builtin_amdgcn_readfirstlane((int)row), i1, i2, i3);
                const float *dyp = lds.dys + sg * N + j2 * N3;
                float dy[N1][N3];
#pragma unroll
                for (int j1 = 0; j1 < N1; ++j1) {
                    const float4 q = *reinterpret_cast<const float4 *>(dyp + j1 * N2 * N3);
                    dy[j1][0] = q.x; dy[j1][1] = q.y; dy[j1][2] = q.z; dy[j1][3] = q.w;
                }
                const float *A = G1 + (size_t)i1 * C::sA;
                const float *B = G2 + (size_t)i2 * C::sB + (size_t)a0 * C::COLS + c0;
                const float *Cp = G3 + (size_t)i3 * C::sC + b0 * N3;
                if (role == 2) {
                    // T0 partial over this wave's rows a, then dG3 partial
                    float t0[N1][V];
#pragma unroll
                    for (int j1 = 0; j1 < N1; ++j1)
#pragma unroll
                        for (int v = 0; v < V; ++v) t0[j1][v] = 0.f;
#pragma unroll
                    for (int aa = 0; aa < RQ; ++aa) {
                        float bv[V];
                        load_vec<V>(B + aa * C::COLS, bv);
#pragma unroll
                        for (int j1 = 0; j1 < N1; ++j1) {
                            const float av = A[j1 * R + a0 + aa];
#pragma unroll
                            for (int v = 0; v < V; ++v) t0[j1][v] = fmaf(av, bv[v], t0[j1][v]);
                        }
                    }
#pragma unroll
                    for (int v = 0; v < V; ++v)
#pragma unroll
                        for (int j3 = 0; j3 < N3; ++j3)
#pragma unroll
                            for (int j1 = 0; j1 < N1; ++j1) acc3[v][j3] = fmaf(t0[j1][v], dy[j1][j3], acc3[v][j3]);
                } else {
                    // dT0'[j1][c0+v] = sum_j3 dY[(j1,j2)][j3] C[b0+v][j3]
                    float dt[N1][V];
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const float4 cv = *reinterpret_cast<const float4 *>(Cp + v * N3);
#pragma unroll
                        for (int j1 = 0; j1 < N1; ++j1)
                            dt[j1][v] = fmaf(dy[j1][0], cv.x, fmaf(dy[j1][1], cv.y, fmaf(dy[j1][2], cv.z, dy[j1][3] * cv.w)));
                    }
                    if (role == 1) {
#pragma unroll
                        for (int aa = 0; aa < RQ; ++aa)
#pragma unroll
                            for (int j1 = 0; j1 < N1; ++j1) {
                                const float av = A[j1 * R + a0 + aa];
#pragma unroll
                                for (int v = 0; v < V; ++v) acc2[aa][v] = fmaf(av, dt[j1][v], acc2[aa][v]);
                            }
                    } else {
#pragma unroll
                        for (int aa = 0; aa < RQ; ++aa) {
                            float bv[V];
                            load_vec<V>(B + aa * C::COLS, bv);
#pragma unroll
                            for (int j1 = 0; j1 < N1; ++j1)
#pragma unroll
                                for (int v = 0; v < V; ++v) acc1[j1 * RQ + aa] = fmaf(dt[j1][v], bv[v], acc1[j1 * RQ + aa]);
                        }
                    }
                }
            }
            __syncthreads();             // the next window overwrites stage / dys / seg_start
        }
    }
    if (!any) return;

    if (role == 1) {
        if (active) {
            float *dst = dG2 + (size_t)s * C::sB + (size_t)a0 * C::COLS + c0;
#pragma unroll
            for (int aa = 0; aa < RQ; ++aa)
#pragma unroll
                for (int v = 0; v < V; ++v) dst[aa * C::COLS + v] += acc2[aa][v];
        }
    } else if (role == 0) {
        if (!active) {
#pragma unroll
            for (int i = 0; i < N1 * RQ; ++i) acc1[i] = 0.f;
        }
        group_reduce<N1 * RQ, WAVE>(acc1, lane);
        constexpr int NVV = N1 * RQ;
        if (lane < ReduceKeep<NVV, WAVE>::writers) {
            const int base = reduce_base<NVV, WAVE>(lane);
            float *dst = dG1 + (size_t)s * C::sA;
#pragma unroll
            for (int i = 0; i < ReduceKeep<NVV, WAVE>::value; ++i) {
                const int idx = base + i;                     // = j1 * RQ + aa
                const int j1 = idx / RQ, aa = idx % RQ;
                dst[j1 * R + a0 + aa] += acc1[i];
            }
        }
    } else {
        // partials [wave][column c][j3] -> LDS, then a fixed-order sum over (wave, j2)
        float *part = lds.dys;                                // NWAVE * COLS * N3 floats
        static_assert(NWAVE * C::COLS * N3 <= FastBwdLds<C>::W * C::N, "partials do not fit");
        __syncthreads();
        if (active) {
#pragma unroll
            for (int v = 0; v < V; ++v)
#pragma unroll
                for (int j3 = 0; j3 < N3; ++j3) part[(w * C::COLS + c0 + v) * N3 + j3] = acc3[v][j3];
        }
        __syncthreads();
        float *dst = dG3 + (size_t)s * C::sC;
        for (int e = t; e < C::sC; e += WG) {
            const int b = e / N3, j3 = e - b * N3;
            float sum = 0.f;
#pragma unroll
            for (int ww = 0; ww < NWAVE; ++ww)
#pragma unroll
                for (int jj = 0; jj < N2; ++jj) sum += part[(ww * C::COLS + jj * R + b) * N3 + j3];
            dst[e] += sum;
        }
    }
}

// ---- dispatch ----------------------------------------------------------------------

template <typename C>
static inline void launch_fwd(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx,
                              const int64_t *off, int n_bags, const float *alpha, const CacheDev &cd, float *out,
                              hipStream_t st)
{
    hipLaunchKernelGGL(fwd_fast_kernel<C>, dim3((n_bags + NWAVE - 1) / NWAVE), dim3(WG), 0, st, p, G1, G2, G3, idx, off,
                       n_bags, alpha, cd, out);
}

template <typename C>
static inline void launch_bwd(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx,
                              int L, const int64_t *off, int n_bags, const float *alpha, const int32_t *slot,
                              const float *go, float *dG1, float *dG2, float *dG3, hipStream_t st)
{
    hipLaunchKernelGGL(bwd_fast_kernel<C>, dim3(p.m1 + p.m2 + p.m3), dim3(WG), 0, st, p, G1, G2, G3, idx, L, off,
                       n_bags, alpha, slot, go, dG1, dG2, dG3);
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
                           const int64_t *off, int n_bags, const float *alpha, const CacheDev &cd, float *out,
                           hipStream_t st)
{
    switch (fast_config(p)) {
    case 0: launch_fwd<Cfg224R8>(p, G1, G2, G3, idx, off, n_bags, alpha, cd, out, st); return 0;
    case 1: launch_fwd<Cfg224R16>(p, G1, G2, G3, idx, off, n_bags, alpha, cd, out, st); return 0;
    case 2: launch_fwd<Cfg224R32>(p, G1, G2, G3, idx, off, n_bags, alpha, cd, out, st); return 0;
    case 3: launch_fwd<Cfg224R64>(p, G1, G2, G3, idx, off, n_bags, alpha, cd, out, st); return 0;
    case 4: launch_fwd<Cfg444R32>(p, G1, G2, G3, idx, off, n_bags, alpha, cd, out, st); return 0;
    case 5: launch_fwd<Cfg444R64>(p, G1, G2, G3, idx, off, n_bags, alpha, cd, out, st); return 0;
    default: return -1;
    }
}

static inline bool fast_bwd_supported(const Params &p) { return fast_config(p) >= 0; }

static inline void fast_bwd(const Params &p, const float *G1, const float *G2, const float *G3, const int64_t *idx, int L,
                            const int64_t *off, int n_bags, const float *alpha, const int32_t *slot, const float *go,
                            float *dG1, float *dG2, float *dG3, hipStream_t st)
{
    switch (fast_config(p)) {
    case 0: launch_bwd<Cfg224R8>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, st); break;
    case 1: launch_bwd<Cfg224R16>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, st); break;
    case 2: launch_bwd<Cfg224R32>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, st); break;
    case 3: launch_bwd<Cfg224R64>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, st); break;
    case 4: launch_bwd<Cfg444R32>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, st); break;
    case 5: launch_bwd<Cfg444R64>(p, G1, G2, G3, idx, L, off, n_bags, alpha, slot, go, dG1, dG2, dG3, st); break;
    default: break;
    }
}

}  // namespace tt
