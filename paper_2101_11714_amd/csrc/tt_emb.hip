// C-ABI entry points of the TT-EmbeddingBag library (declared in include/tt_emb.h):
// argument checks, workspace layout, kernel selection and launches.  Nothing here
// allocates device memory or waits for the stream.

#include "../../include/tt_emb.h"

#include <stdarg.h>
#include <initializer_list>
#include <mutex>
#include <stdio.h>
#include <string.h>

#include "tt_common.h"
#include "tt_sort.h"
#include "tt_select.h"
#include "tt_generic.h"
#include "tt_fast.h"
#include "tt_fast_bwd.h"
#include "tt_kept.h"
#include "tt_group.h"
#include "tt_fwd_owner.h"
#include "tt_bwd_owner.h"
#include "tt_freq.h"
#include "tt_dense.h"
#include "tt_init.h"
#include "tt_anyd.h"

using namespace tt;

// Scratch memory of tt_emb_bwd_sgd_static, the entry point for callers that cannot allocate: every GPU
// the library runs on holds its own copy of this array until the process ends.  In host code the name
// is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";
// Kernel selection of the calling thread (tests only; no other thread's calls change with it):
// 0: generic kernels, 1: specialised, 2: specialised + grouping pre-pass always + list owners always
thread_local int g_fast_path = 1;
thread_local int g_bwd_tiles = 0;          // 1: the grouped backward with a kept T0 runs the tile kernels of tt_bwd_owner.h even under selection 2
// The grouped backward with a kept T0 runs on tiles of positions (tt_bwd_owner.h) wherever that path covers the
// shape: measured ahead of the list owners for every shape it covers (rank 64, 204,800 positions: 276 against 444 us;
// Terabyte-shaped, 8,192 positions: 83 against 101 us).  Selection 2 (tests) keeps the list owners.
bool bwd_tiles_wanted(const Params &p, int64_t L)
{
    (void)L;
    return bwd_owner_supported(p) && (g_bwd_tiles || g_fast_path == 1);
}
// from this many positions on the backward groups them first (tt_group.h)
constexpr int64_t GROUP_MIN_L = 32768;          // without a cache
constexpr int64_t GROUP_MIN_L_CACHE = 16384;    // with a cache (the grouped path also has the faster cached-row reduction)
// With a kept T0 and no cache the grouped backward runs on tiles (tt_bwd_owner.h), which are ahead of the scanning
// owners much earlier, but only if the pre-pass (about 30 us of small kernels) does not count: so these limits hold
// for the two-call form, whose first call can run beside other work (Terabyte-shaped, 8,192 positions: 84 against
// 101 us; (2,2,4) at rank 32 / 64, 20,480 positions: 38 against 59 / 64 against 90 us).
constexpr int64_t GROUP_MIN_L_TILES_444 = 8192, GROUP_MIN_L_TILES_224 = 16384;

int64_t group_min_l(const Params &p, int64_t K, bool kept_t0, bool two_calls)
{
    if (two_calls && kept_t0 && !K && g_fast_path == 1 && bwd_owner_supported(p))
        return p.n1 == 4 ? GROUP_MIN_L_TILES_444 : GROUP_MIN_L_TILES_224;
    return K ? GROUP_MIN_L_CACHE : GROUP_MIN_L;
}

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_shape(const tt_shape_t *s, Params *p)
{
    if (!s) return fail(TT_ERR_NULL, "shape is NULL");
    if (s->d != 3) return fail(TT_ERR_BAD_SHAPE, "d = %d, only d = 3 is supported", s->d);
    if (s->r[0] != 1 || s->r[3] != 1) return fail(TT_ERR_BAD_SHAPE, "boundary ranks must be 1");
    for (int k = 0; k < 3; ++k)
        if (s->m[k] <= 0 || s->n[k] <= 0 || s->r[k + 1] <= 0)
            return fail(TT_ERR_BAD_SHAPE, "non-positive factor or rank at core %d", k);
    const __int128 prod = (__int128)s->m[0] * s->m[1] * s->m[2];
    if (s->num_rows <= 0 || (__int128)s->num_rows > prod)
        return fail(TT_ERR_BAD_SHAPE, "num_rows must be in [1, m1*m2*m3]");
    if (s->num_rows >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "num_rows >= 2^31");
    const int64_t N = (int64_t)s->n[0] * s->n[1] * s->n[2];
    const int64_t sB = (int64_t)s->r[1] * s->n[1] * s->r[2];
    if (N > WG) return fail(TT_ERR_UNSUPPORTED, "embedding dimension %lld > %d", (long long)N, WG);
    if (sB > (1 << 16) || (int64_t)s->n[0] * s->r[1] > (1 << 14) || (int64_t)s->r[2] * s->n[2] > (1 << 14))
        return fail(TT_ERR_UNSUPPORTED, "core slice too large for the on-chip accumulators");
    if (p) {
        p->m1 = s->m[0]; p->m2 = s->m[1]; p->m3 = s->m[2];
        p->n1 = s->n[0]; p->n2 = s->n[1]; p->n3 = s->n[2];
        p->R1 = s->r[1]; p->R2 = s->r[2];
        p->N = (int)N;
        p->sA = p->n1 * p->R1; p->sB = (int)sB; p->sC = p->R2 * p->n3;
        p->cols = p->n2 * p->R2;
        p->mg3 = p->m3 > 1 ? (uint32_t)(((1ull << 32) + p->m3 - 1) / (uint64_t)p->m3) : 0u;
        p->mg2 = p->m2 > 1 ? (uint32_t)(((1ull << 32) + p->m2 - 1) / (uint64_t)p->m2) : 0u;
        p->bagP = 0; p->mgP = 0;
        p->m3d = (double)p->m3; p->m2d = (double)p->m2;
        p->inv3 = 1.0 / p->m3d; p->half3 = 0.5 * p->inv3;
        p->inv2 = 1.0 / p->m2d; p->half2 = 0.5 * p->inv2;
    }
    return TT_OK;
}

int check_lookup_args(const int64_t *indices, int64_t L, int64_t n_bags, const int64_t *offsets, int64_t N)
{
    if (L < 0 || n_bags < 0) return fail(TT_ERR_BAD_ARG, "negative L or n_bags");
    if (L >= (1ll << 31) || n_bags >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "L or n_bags >= 2^31");
    // (some kernels form element offsets into the [n_bags][N] arrays in 32 bits)
    if (n_bags * N >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "n_bags * N >= 2^31");
    if (L > 0 && !indices) return fail(TT_ERR_NULL, "indices is NULL");
    if (!offsets && n_bags != L) return fail(TT_ERR_BAD_ARG, "offsets == NULL requires n_bags == L");
    return TT_OK;
}

int check_cache(const tt_cache_t *c, CacheDev *dev, bool need_rows)
{
    dev->rows = nullptr; dev->table = nullptr; dev->mask = 0; dev->K = 0;
    if (!c) return TT_OK;
    if (c->K < 0 || c->K > (1 << 24)) return fail(TT_ERR_BAD_ARG, "cache K out of range [0, 2^24]");
    if (c->K == 0) return TT_OK;
    if (c->capacity < tt_cache_table_capacity(c->K) || (c->capacity & (c->capacity - 1)) || c->capacity > (1ll << 31))
        return fail(TT_ERR_BAD_ARG, "cache capacity must be a power of two >= tt_cache_table_capacity(K)");
    if (!c->table || !c->keys || (need_rows && !c->rows)) return fail(TT_ERR_NULL, "cache array is NULL");
    dev->rows = c->rows; dev->table = c->table; dev->mask = (uint32_t)(c->capacity - 1); dev->K = (int)c->K;
    return TT_OK;
}

// The kernels move fp32 data in 16-byte pieces: true if any of the given arrays does not start on one.
bool misaligned(std::initializer_list<const void *> ptrs)
{
    uintptr_t bits = 0;
    for (const void *q : ptrs) bits |= (uintptr_t)q;
    return (bits & 15) != 0;
}

int hip_fail(hipError_t e, const char *what)
{
    return fail(TT_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

size_t lds_limit()
{
    static size_t lim = 0;
    if (!lim) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0)
            lim = (size_t)v;
        else
            lim = 64 * 1024;
    }
    return lim;
}

template <typename K>
int allow_lds(K kernel, size_t bytes)
{
    if (bytes > lds_limit()) return fail(TT_ERR_UNSUPPORTED, "kernel needs %zu bytes of LDS, device offers %zu", bytes, lds_limit());
    if (bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute");
    }
    return TT_OK;
}

inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// workspace of tt_emb_bwd: slot of every position (with a cache) | grouping pre-pass
size_t slot_ws_bytes(int64_t L, int with_cache) { return with_cache ? align256((size_t)(L > 0 ? L : 1) * 4) : 0; }

// Does the forward pass that works from the pre-pass's lists pay for such a table (tt_fwd_owner.h)?  (Measured: with a
// cache that takes most positions the wave-per-bag kernel is as fast at rank 32: 49 against 51 us for 163,840 positions
// of which a fifth go through the cores.)  If so the workspace has room for one row per position.
static inline bool fwd_lists_pay(const Params &p, int64_t K) { return fwd_owner_supported(p) && (K == 0 || p.R1 >= 64); }
static inline int fwd_rows_n(const Params &p, int64_t K) { return fwd_lists_pay(p, K) ? p.N : 0; }

size_t fwd_bwd_ws_bytes(const Params &p, int64_t L, int64_t K)
{
    return 256 + slot_ws_bytes(L, K != 0) + group_ws_layout(nullptr, L, p.m1 + p.m2 + p.m3 + (int)K, p.N, fwd_rows_n(p, K)).bytes;
}

// what the specialised backward kernel needs beyond the lists: partial slice gradients of the roles it splits over
// several workgroups and, for the (4,4,4) shapes, the per-row G1 gradients
size_t split_ws_bytes(const Params &p, int64_t L, bool grouped, bool tiles_possible = true);

// enough for either way of running the backward
size_t split_ws_bytes_max(const Params &p, int64_t L)
{
    const size_t a = split_ws_bytes(p, L, false), b = split_ws_bytes(p, L, true);
    return a > b ? a : b;
}

// tiles_possible: false for a call that brings no kept T0 (the tiled backward needs one) or that has a cache
size_t split_ws_bytes(const Params &p, int64_t L, bool grouped, bool tiles_possible)
{
    const size_t n = fast_bwd_supported(p) ? fast_bwd_extra_floats(p, (int)L, grouped) : 0;
    size_t bytes = n ? align256(n * sizeof(float)) : 0;
    if (grouped && tiles_possible && bwd_tiles_wanted(p, L)) {          // the tiled backward's buffers instead
        // (room for either size of tile)
        const size_t b1 = align256(bo_ws_layout(nullptr, p, L, bo_tp(p, L, false)).bytes), b2 = align256(bo_ws_layout(nullptr, p, L, bo_tp(p, L, true)).bytes);
        const size_t b = b1 > b2 ? b1 : b2;
        bytes = b > bytes ? b : bytes;
    }
    return bytes;
}

}  // namespace

extern "C" {

const char *tt_last_error(void) { return g_err; }

int tt_emb_debug_set_fast_path(int mode)
{
    int old = g_bwd_tiles ? 3 : g_fast_path;
    g_bwd_tiles = mode == 3;
    g_fast_path = mode < 0 ? 0 : (mode > 2 ? 2 : mode);
    return old;
}

int64_t tt_cache_table_capacity(int64_t K)
{
    int64_t cap = 16;
    while (cap < 2 * K) cap <<= 1;
    return cap;
}

size_t tt_emb_workspace_bytes(const tt_shape_t *shape, int64_t L, int64_t n_bags, int64_t cache_rows)
{
    (void)n_bags;
    Params p;
    if (check_shape(shape, &p) != TT_OK || L < 0) return 0;
    if (cache_rows < 0 || cache_rows > (1 << 24)) return 0;
    return fwd_bwd_ws_bytes(p, L, cache_rows) + split_ws_bytes_max(p, L);
}

size_t tt_emb_dedup_workspace_bytes(int64_t L)
{
    if (L < 0) return 0;
    return sort_ws_layout(nullptr, L > 0 ? L : 1).bytes;
}

size_t tt_cache_build_workspace_bytes(const tt_shape_t *shape, int64_t n_cand, int64_t K)
{
    (void)K;
    if (check_shape(shape, nullptr) != TT_OK || n_cand < 0) return 0;
    return sort_ws_layout(nullptr, n_cand > 0 ? n_cand : 1).bytes;
}

static int fwd_common(const tt_shape_t *shape, const float *const cores[3],
                      const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                      const float *alpha, const tt_cache_t *cache, float *output, float *t0_out, bool keep_t0,
                      void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if ((rc = check_lookup_args(indices, L, n_bags, offsets, p.N))) return rc;
    if (!cores || !cores[0] || !cores[1] || !cores[2]) return fail(TT_ERR_NULL, "cores is NULL");
    if (n_bags > 0 && !output) return fail(TT_ERR_NULL, "output is NULL");
    CacheDev cd;
    if ((rc = check_cache(cache, &cd, true))) return rc;
    if (keep_t0) {
        if (L > 0 && !t0_out) return fail(TT_ERR_NULL, "t0 is NULL");
        if (fast_config(p) < 0) return fail(TT_ERR_UNSUPPORTED, "no kernel keeps T0 for this shape");
    }
    if (misaligned({cores[0], cores[1], cores[2], output, t0_out, cd.rows}))
        return fail(TT_ERR_BAD_ARG, "cores, output, t0 and cache rows must be 16-byte aligned");
    if (n_bags == 0) return TT_OK;
    hipStream_t st = (hipStream_t)stream;

    if (g_fast_path || keep_t0) {
        int frc = fast_fwd(p, cores[0], cores[1], cores[2], indices, offsets, L, (int)n_bags, alpha, cd, output,
                           keep_t0 ? t0_out : nullptr, st);
        if (frc == 0) {
            hipError_t e = hipGetLastError();
            return e == hipSuccess ? TT_OK : hip_fail(e, "forward launch");
        }
    }
    const size_t lds = (size_t)(p.sA + p.sC + p.n1 * p.cols) * sizeof(float);
    if ((rc = allow_lds(fwd_generic_kernel, lds))) return rc;
    const int grid = (int)(n_bags < 65536 ? n_bags : 65536);
    hipLaunchKernelGGL(fwd_generic_kernel, dim3(grid), dim3(WG), lds, st, p, cores[0], cores[1], cores[2],
                       indices, offsets, (int)n_bags, alpha, cd, output);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "forward launch");
}

int tt_emb_fwd(const tt_shape_t *shape, const float *const cores[3],
               const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
               const float *alpha, const tt_cache_t *cache,
               float *output, void *workspace, size_t workspace_bytes, void *stream)
{
    (void)workspace; (void)workspace_bytes;
    return fwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, output, nullptr, false, stream);
}

int tt_emb_fwd_keep_t0(const tt_shape_t *shape, const float *const cores[3],
                       const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                       const float *alpha, const tt_cache_t *cache,
                       float *output, float *t0, void *stream)
{
    return fwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, output, t0, true, stream);
}

// does the backward of such a call group the positions first (tt_group.h)?
static bool bwd_groups(const Params &p, int64_t L, int64_t K, bool kept_t0)
{
    const bool fast = (g_fast_path || kept_t0) && fast_bwd_supported(p);
    return fast && (g_fast_path == 2 || L >= group_min_l(p, K, kept_t0, false));
}

// does tt_emb_fwd_prepared work from the pre-pass's lists for such a call?
static bool fwd_from_lists(const Params &p, int64_t L, int64_t K, bool kept_t0)
{
    // (only for the long streams: at 8,192 positions, where the (4,4,4) backward already groups, the wave per bag is ahead: 31 against 36 us)
    return L > 0 && fwd_lists_pay(p, K) && bwd_groups(p, L, K, kept_t0) && (g_fast_path == 2 || L >= (K ? GROUP_MIN_L_CACHE : GROUP_MIN_L)) &&
           3 * L < (1ll << 31);
}

int tt_emb_fwd_uses_lists(const tt_shape_t *shape, int64_t L, int64_t cache_rows, int kept_t0)
{
    Params p;
    if (check_shape(shape, &p) != TT_OK || L <= 0 || cache_rows < 0) return 0;
    return fwd_from_lists(p, L, cache_rows, kept_t0 != 0) ? 1 : 0;
}

int tt_emb_fwd_prepared(const tt_shape_t *shape, const float *const cores[3],
                        const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                        const float *alpha, const tt_cache_t *cache,
                        float *output, float *t0, void *workspace, size_t workspace_bytes, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if ((rc = check_lookup_args(indices, L, n_bags, offsets, p.N))) return rc;
    CacheDev cd;
    if ((rc = check_cache(cache, &cd, true))) return rc;
    if (t0 && fast_config(p) < 0) return fail(TT_ERR_UNSUPPORTED, "no kernel keeps T0 for this shape");
    // the lists exist if the backward of this call groups its positions; else the forward needs none
    if (!(n_bags > 0 && fwd_from_lists(p, L, cd.K, t0 != nullptr)))
        return fwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, output, t0, t0 != nullptr, stream);
    if (!cores || !cores[0] || !cores[1] || !cores[2]) return fail(TT_ERR_NULL, "cores is NULL");
    if (!output) return fail(TT_ERR_NULL, "output is NULL");
    const size_t need = fwd_bwd_ws_bytes(p, L, cd.K);
    if (!workspace || workspace_bytes < need)
        return fail(TT_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    if (misaligned({cores[0], cores[1], cores[2], output, t0, cd.rows, workspace}))
        return fail(TT_ERR_BAD_ARG, "cores, output, t0, cache rows and workspace must be 16-byte aligned");
    const int nbins = p.m1 + p.m2 + p.m3 + cd.K;
    GroupWs g = group_ws_layout((char *)workspace + slot_ws_bytes(L, cd.K != 0), L, nbins, p.N, fwd_rows_n(p, cd.K));
    int bits = 1;
    while ((1 << bits) <= nbins) ++bits;
    uint64_t *ks; uint32_t *vs;
    radix_sort_result(g.sort, bits, &ks, &vs);
    // the pre-pass wrote the items' records if the backward that follows runs on tiles (the same test as there)
    const bool have_info = t0 != nullptr && (!cd.K || g_bwd_tiles) && bwd_tiles_wanted(p, L);
    hipError_t e = fwd_owner(p, cores[0], cores[1], cores[2], indices, L, offsets, (int)n_bags, alpha, cd, vs, have_info ? g.info : nullptr, g.tiles,
                             g.rows, output, t0, (hipStream_t)stream);
    return e == hipSuccess ? TT_OK : hip_fail(e, "forward launch");
}

enum BwdPhase { BWD_ALL, BWD_PREPARE, BWD_REST };

// Backward pass behind tt_emb_bwd (cores_out == nullptr: gradients are added to grad_cores /
// grad_cache) and tt_emb_bwd_sgd (cores_out != nullptr: the cores after the SGD step are written
// to cores_out, the cached rows are updated in place; grad_cores / grad_cache are unused).
static int bwd_common(const tt_shape_t *shape, const float *const cores[3],
                      const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                      const float *alpha, const tt_cache_t *cache, const float *grad_output,
                      float *const grad_cores[3], float *grad_cache, float lr, float *const cores_out[3],
                      const float *t0, void *workspace, size_t workspace_bytes, void *stream, BwdPhase phase = BWD_ALL)
{
    // BWD_PREPARE (fused step only): the part that needs the indices and the cache's row map alone, into the
    // workspace; t0 != nullptr then only says that the later call will bring a kept T0.  BWD_REST: everything else.
    const bool prep = phase == BWD_PREPARE;
    const bool fused = cores_out != nullptr || prep;
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if ((rc = check_lookup_args(indices, L, n_bags, offsets, p.N))) return rc;
    if (!prep && (!cores || !cores[0] || !cores[1] || !cores[2])) return fail(TT_ERR_NULL, "cores is NULL");
    if (prep) {
    } else if (fused) {
        if (!cores_out[0] || !cores_out[1] || !cores_out[2]) return fail(TT_ERR_NULL, "cores_out is NULL");
        for (int k = 0; k < 3; ++k)
            if (cores_out[k] == cores[k]) return fail(TT_ERR_BAD_ARG, "cores_out must not alias cores");
    } else if (!grad_cores || !grad_cores[0] || !grad_cores[1] || !grad_cores[2]) {
        return fail(TT_ERR_NULL, "grad_cores is NULL");
    }
    if (!prep && n_bags > 0 && !grad_output) return fail(TT_ERR_NULL, "grad_output is NULL");
    CacheDev cd;
    if ((rc = check_cache(cache, &cd, fused))) return rc;
    if (!fused && cd.K && !grad_cache) return fail(TT_ERR_NULL, "grad_cache is NULL but a cache is given");
    if (t0 && !fast_bwd_supported(p)) return fail(TT_ERR_UNSUPPORTED, "no kernel uses a kept T0 for this shape");
    if (prep ? misaligned({cd.rows, workspace})
             : (misaligned({cores[0], cores[1], cores[2], grad_output, t0, cd.rows, workspace}) ||
                (fused ? misaligned({cores_out[0], cores_out[1], cores_out[2]})
                       : misaligned({grad_cores[0], grad_cores[1], grad_cores[2], grad_cache}))))
        return fail(TT_ERR_BAD_ARG, "cores, gradients, t0, cache rows and workspace must be 16-byte aligned");
    const bool fast = (g_fast_path || t0) && fast_bwd_supported(p);
    const bool grouped = fast && (g_fast_path == 2 || L >= group_min_l(p, cd.K, t0 != nullptr, phase != BWD_ALL));
    if (grouped && 3 * L >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "3 L >= 2^31");
    const size_t need_bwd = grouped ? fwd_bwd_ws_bytes(p, L, cd.K) : 256 + slot_ws_bytes(L, cd.K != 0);
    const int64_t core_floats[3] = {(int64_t)p.m1 * p.sA, (int64_t)p.m2 * p.sB, (int64_t)p.m3 * p.sC};
    // the fused step keeps the gradient of the cached rows, and without a specialised kernel the
    // gradients of the cores, in the workspace
    const size_t gc_bytes = fused && cd.K ? align256((size_t)cd.K * p.N * 4) : 0;
    size_t g_bytes[3] = {0, 0, 0};
    if (fused && !fast)
        for (int k = 0; k < 3; ++k) g_bytes[k] = align256((size_t)core_floats[k] * 4);
    // long streams with a kept T0: the products of Eq. 4 over tiles of positions, on the matrix cores (tt_bwd_owner.h)
    // (with a cache the list owners stay: the cached rows' sums ride along in their launches, multi-hot table 0: 113 against 140 us)
    const bool tiled = grouped && t0 && (!cd.K || g_bwd_tiles) && bwd_tiles_wanted(p, L);
    // positions per tile of the tile table: 128 / n1 where the forward pass works from it too; the smaller tiles of the
    // tiled backward only where the table has room for them (tt_group.h: L / 32 + slices + 1 entries)
    int tile_tp = bo_tp(p, L, tiled && !fwd_from_lists(p, L, cd.K, t0 != nullptr));
    if (bo_tiles(p, L, tile_tp) > L / 32 + p.m1 + p.m2 + p.m3 + cd.K + 1) tile_tp = 128 / p.n1;
    const size_t sp_bytes = fast ? split_ws_bytes(p, L, grouped, t0 != nullptr && (!cd.K || g_bwd_tiles)) : 0;
    const size_t need = need_bwd + gc_bytes + g_bytes[0] + g_bytes[1] + g_bytes[2] + sp_bytes;
    const bool wants_ws = cd.K || grouped || (fused && !fast) || sp_bytes;
    if (wants_ws && (!workspace || workspace_bytes < need))
        return fail(TT_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    if (L == 0 && !fused) return TT_OK;
    hipStream_t st = (hipStream_t)stream;

    // LDS needs of the generic kernels, checked before anything is enqueued
    const int max_slice = p.sA > p.sB ? (p.sA > p.sC ? p.sA : p.sC) : (p.sB > p.sC ? p.sB : p.sC);
    const size_t lds_core = sizeof(SelectLds<GEN_CH>) + (GEN_CH + 4) * sizeof(int) +
                            (size_t)(max_slice + p.sA + p.sC + p.n1 * p.cols + p.N) * sizeof(float);
    const int G = WG / p.N > 0 ? WG / p.N : 1;
    const size_t lds_cache = sizeof(SelectLds<GEN_CH>) + (size_t)G * p.N * sizeof(float);
    if (!fast && (rc = allow_lds(bwd_generic_kernel, lds_core))) return rc;
    if (cd.K && !grouped && (rc = allow_lds(bwd_cache_kernel, lds_cache))) return rc;

    float *split_ws = sp_bytes ? (float *)((char *)workspace + need - sp_bytes) : nullptr;
    float *gtmp[3] = {nullptr, nullptr, nullptr};
    if (fused) {
        char *q = (char *)workspace + need_bwd;
        if (cd.K) {
            grad_cache = (float *)q;
            q += gc_bytes;
            const int64_t n = (int64_t)cd.K * p.N;
            if (!(grouped && L > 0) && phase != BWD_REST)                 // the grouping pre-pass clears it itself
                hipLaunchKernelGGL(fill_f32_kernel, dim3(cdiv(n, WG) < 1024 ? cdiv(n, WG) : 1024), dim3(WG), 0, st, grad_cache, n, 0.f);
        }
        if (!fast) {
            for (int k = 0; k < 3; ++k) {
                gtmp[k] = (float *)q;
                q += g_bytes[k];
                if (phase != BWD_PREPARE)                                 // not index-only work: the pre-pass leaves it
                    hipLaunchKernelGGL(fill_f32_kernel, dim3(cdiv(core_floats[k], WG) < 1024 ? cdiv(core_floats[k], WG) : 1024),
                                       dim3(WG), 0, st, gtmp[k], core_floats[k], 0.f);
            }
            grad_cores = gtmp;
        }
    }
    const bool outs = fused && fast && !prep;                            // (the pre-pass has no cores)
    float *o1 = outs ? cores_out[0] : nullptr, *o2 = outs ? cores_out[1] : nullptr, *o3 = outs ? cores_out[2] : nullptr;
    float *d1 = grad_cores ? grad_cores[0] : nullptr, *d2 = grad_cores ? grad_cores[1] : nullptr,
          *d3 = grad_cores ? grad_cores[2] : nullptr;

    if (offsets && n_bags > 0 && L > 0 && L % n_bags == 0) {              // a guess for the bag of a position
        p.bagP = (uint32_t)(L / n_bags);
        p.mgP = p.bagP > 1 ? (uint32_t)(((1ull << 32) + p.bagP - 1) / (uint64_t)p.bagP) : 0u;
    }
    bool cache_merged = false;
    int32_t *slot = nullptr;
    if (cd.K && L > 0 && !grouped) {                                      // the grouping pre-pass probes the cache itself
        slot = (int32_t *)workspace;
        if (phase != BWD_REST)
            hipLaunchKernelGGL(cache_lookup_kernel, dim3(cdiv(L, WG)), dim3(WG), 0, st, cd, indices, (int)L, slot);
    }
    if (grouped && L > 0) {
        // group the positions by the slices / cache slots they touch, then run the owners on their lists
        const int nb3 = p.m1 + p.m2 + p.m3, nbins = nb3 + cd.K;
        GroupWs g = group_ws_layout((char *)workspace + slot_ws_bytes(L, cd.K != 0), L, nbins, p.N, fwd_rows_n(p, cd.K));
        const int n = 3 * (int)L;
        const int64_t kthreads = L > nbins + 1 ? L : nbins + 1;
        const bool clear_gc = fused && cd.K;                                // N is a multiple of 4 for these shapes
        int bits = 1;
        while ((1 << bits) <= nbins) ++bits;
        uint64_t *ks; uint32_t *vs;
        radix_sort_result(g.sort, bits, &ks, &vs);
        if (phase != BWD_REST) {
            hipLaunchKernelGGL(grp_keys_kernel, dim3(cdiv(kthreads, WG)), dim3(WG), 0, st, p, indices, (int)L, cd, g.sort.k0, g.off,
                               g.end, nbins, g.crange, clear_gc ? (float4 *)grad_cache : nullptr,
                               clear_gc ? (int64_t)cd.K * p.N / 4 : (int64_t)0);
            uint64_t *ks2; uint32_t *vs2;
            hipError_t es = radix_sort(g.sort, n, bits, st, &ks2, &vs2);
            if (es != hipSuccess) return hip_fail(es, "grouping sort");
            if (ks2 != ks || vs2 != vs) return fail(TT_ERR_BAD_ARG, "internal: the sort's result is not where it was expected");
            hipLaunchKernelGGL(grp_bounds_kernel, dim3(cdiv(n, WG)), dim3(WG), 0, st, ks, n, p.m1, p.m1 + p.m2, nb3, nbins, g.off, g.end, g.crange);
            if (tiled)
                hipLaunchKernelGGL(grp_info_kernel, dim3(cdiv(n, WG)), dim3(WG), 0, st, p, indices, (int)L, offsets, (int)n_bags, ks, vs,
                                   nb3, g.info);
            if (fwd_from_lists(p, L, cd.K, t0 != nullptr) || tiled) {       // for tt_emb_fwd_prepared and the tiled backward
                const int ntiles = bo_tiles(p, L, tile_tp);
                hipLaunchKernelGGL(grp_tiles_kernel, dim3(cdiv(ntiles, WG)), dim3(WG), 0, st, p.m1, p.m2, (int)L, tile_tp,
                                   g.off, g.end, g.tiles, ntiles, g.tile_base);
            }
        }
        if (prep) {
            hipError_t e = hipGetLastError();
            return e == hipSuccess ? TT_OK : hip_fail(e, "backward pre-pass launch");
        }
        GrpCacheWork cw{ks, vs, g.crange, g.end, g.part, grad_cache, cd.K ? cdiv(cdiv(L, GT), NWAVE) : 0, clear_gc};
        cache_merged = !tiled && cd.K && fast_bwd_takes_cache_work(p, (int)L);     // the owner kernels do the cached rows as well
        if (cd.K && !cache_merged) {
            hipLaunchKernelGGL(grp_cache_tile_kernel, dim3(cw.blocks), dim3(WG), 0, st, p, ks, vs, g.crange, offsets,
                               (int)n_bags, alpha, grad_output, grad_cache, g.part, clear_gc);
            hipLaunchKernelGGL(grp_cache_fix_kernel, dim3(cw.blocks), dim3(WG), 0, st, p, ks, g.crange, g.end, g.part,
                               grad_cache);
        }
        if (tiled) {
            const BoWs bw = bo_ws_layout(split_ws, p, L, tile_tp);
            hipError_t eb = bwd_owner(p, cores[0], cores[1], cores[2], indices, L, offsets, (int)n_bags, alpha, grad_output, t0,
                                      d1, d2, d3, lr, o1, o2, o3, ks, vs, g, bw, tile_tp, st);
            if (eb != hipSuccess) return hip_fail(eb, "backward launch");
        } else
        fast_bwd(p, cores[0], cores[1], cores[2], indices, (int)L, offsets, (int)n_bags, alpha, slot, grad_output,
                 d1, d2, d3, vs, g.off, g.end, lr, o1, o2, o3, t0, split_ws, cache_merged ? &cw : nullptr,
                 fused && cache_merged ? cache->rows : nullptr, (int64_t)cd.K * p.N, st);
    } else {
        if (prep) {
            hipError_t e = hipGetLastError();
            return e == hipSuccess ? TT_OK : hip_fail(e, "backward pre-pass launch");
        }
        if (cd.K && L > 0)
            hipLaunchKernelGGL(bwd_cache_kernel, dim3(cdiv(cd.K, G)), dim3(WG), lds_cache, st, p.N, cd.K, G, slot, (int)L,
                               offsets, (int)n_bags, alpha, grad_output, grad_cache);
        if (fast) {
            fast_bwd(p, cores[0], cores[1], cores[2], indices, (int)L, offsets, (int)n_bags, alpha, slot, grad_output,
                     d1, d2, d3, nullptr, nullptr, nullptr, lr, o1, o2, o3, t0, split_ws, nullptr, nullptr, 0, st);
        } else if (L > 0) {
            hipLaunchKernelGGL(bwd_generic_kernel, dim3(p.m1 + p.m2 + p.m3), dim3(WG), lds_core, st, p,
                               cores[0], cores[1], cores[2], indices, (int)L, offsets, (int)n_bags, alpha, slot,
                               grad_output, d1, d2, d3);
        }
    }
    if (fused) {
        if (!fast)
            for (int k = 0; k < 3; ++k)
                hipLaunchKernelGGL(sgd_out_kernel, dim3(cdiv(core_floats[k], WG) < 2048 ? cdiv(core_floats[k], WG) : 2048),
                                   dim3(WG), 0, st, cores[k], gtmp[k], cores_out[k], core_floats[k], lr);
        if (cd.K && !cache_merged) {
            const int64_t n = (int64_t)cd.K * p.N;
            hipLaunchKernelGGL(sgd_out_kernel, dim3(cdiv(n, WG) < 2048 ? cdiv(n, WG) : 2048), dim3(WG), 0, st,
                               cache->rows, grad_cache, cache->rows, n, lr);
        }
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "backward launch");
}

int tt_emb_bwd(const tt_shape_t *shape, const float *const cores[3],
               const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
               const float *alpha, const tt_cache_t *cache,
               const float *grad_output,
               float *const grad_cores[3], float *grad_cache,
               void *workspace, size_t workspace_bytes, void *stream)
{
    return bwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, grad_output, grad_cores, grad_cache,
                      0.f, nullptr, nullptr, workspace, workspace_bytes, stream);
}

int tt_emb_bwd_t0(const tt_shape_t *shape, const float *const cores[3],
                  const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                  const float *alpha, const tt_cache_t *cache,
                  const float *grad_output, const float *t0,
                  float *const grad_cores[3], float *grad_cache,
                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (L > 0 && !t0) return fail(TT_ERR_NULL, "t0 is NULL");
    return bwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, grad_output, grad_cores, grad_cache,
                      0.f, nullptr, t0, workspace, workspace_bytes, stream);
}

int tt_emb_bwd_sgd(const tt_shape_t *shape, const float *const cores[3], float *const cores_out[3],
                   const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                   const float *alpha, const tt_cache_t *cache,
                   const float *grad_output, float lr,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    if (!cores_out) return fail(TT_ERR_NULL, "cores_out is NULL");
    return bwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, grad_output, nullptr, nullptr,
                      lr, cores_out, nullptr, workspace, workspace_bytes, stream);
}

// Address of this device's copy of scratch[], looked up once per device.
static int static_scratch_ptr(void **out)
{
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static void *ptrs[MAX_DEV] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEV) return fail(TT_ERR_UNSUPPORTED, "device number %d beyond %d", dev, MAX_DEV - 1);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void *q = nullptr;
        e = hipGetSymbolAddress(&q, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!q) return fail(TT_ERR_HIP, "hipGetSymbolAddress(scratch) returned no address");
        ptrs[dev] = q;
    }
    *out = ptrs[dev];
    return TT_OK;
}

size_t tt_emb_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int tt_emb_bwd_sgd_static(const tt_shape_t *shape, const float *const cores[3], float *const cores_out[3],
                          const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                          const float *alpha, const tt_cache_t *cache,
                          const float *grad_output, float lr, void *stream)
{
    if (!cores_out) return fail(TT_ERR_NULL, "cores_out is NULL");
    void *ws = nullptr;
    int rc = static_scratch_ptr(&ws);
    if (rc) return rc;
    // (the kernels initialise every part of the workspace that they read: nothing is left to clear here)
    rc = bwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, grad_output, nullptr, nullptr,
                    lr, cores_out, nullptr, ws, STATIC_SCRATCH_BYTES, stream);
    if (rc == TT_ERR_WORKSPACE)
        return fail(TT_ERR_WORKSPACE, "this call needs more scratch memory than the %zu bytes of the static array "
                    "(%zu positions, cache of %lld rows): use tt_emb_bwd_sgd with a workspace of "
                    "tt_emb_bwd_sgd_workspace_bytes() bytes", STATIC_SCRATCH_BYTES, (size_t)L,
                    (long long)(cache ? cache->K : 0));
    return rc;
}

int tt_emb_bwd_sgd_t0(const tt_shape_t *shape, const float *const cores[3], float *const cores_out[3],
                      const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                      const float *alpha, const tt_cache_t *cache,
                      const float *grad_output, const float *t0, float lr,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    if (!cores_out) return fail(TT_ERR_NULL, "cores_out is NULL");
    if (L > 0 && !t0) return fail(TT_ERR_NULL, "t0 is NULL");
    return bwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, grad_output, nullptr, nullptr,
                      lr, cores_out, t0, workspace, workspace_bytes, stream);
}

// ---- forward and backward with the kept partial products and lists (tt_kept.h) ----

size_t tt_emb_kept_bytes(const tt_shape_t *shape, int64_t L)
{
    Params p;
    if (check_shape(shape, &p) != TT_OK || L < 0 || L >= (1ll << 31) || fast_config(p) < 0) return 0;
    if (kept_supported(p, L)) return kept_layout(p, L).bytes;
    return align256((size_t)(L > 0 ? L : 1) * p.n1 * p.cols * sizeof(float));       // T0 alone
}

int tt_emb_kept_has_lists(const tt_shape_t *shape, int64_t L)
{
    Params p;
    if (check_shape(shape, &p) != TT_OK || L < 0) return 0;
    return kept_supported(p, L) ? 1 : 0;
}

int tt_emb_fwd_keep(const tt_shape_t *shape, const float *const cores[3],
                    const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                    const float *alpha, const tt_cache_t *cache,
                    float *output, void *kept, size_t kept_bytes, int lists_ready, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (fast_config(p) < 0) return fail(TT_ERR_UNSUPPORTED, "no kernel keeps intermediates for this shape");
    if ((rc = check_lookup_args(indices, L, n_bags, offsets, p.N))) return rc;
    const size_t need = tt_emb_kept_bytes(shape, L);
    if (L > 0 && (!kept || kept_bytes < need))
        return fail(TT_ERR_WORKSPACE, "kept buffer of %zu bytes needed, %zu given", need, kept_bytes);
    // T0 at the start of the buffer, by the forward kernel that keeps it
    rc = fwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, output, (float *)kept, true, stream);
    if (rc || !kept_supported(p, L) || lists_ready) return rc;
    CacheDev cd;
    if ((rc = check_cache(cache, &cd, false))) return rc;
    kept_sort(p, indices, (int)L, cd, kept_dev(kept, kept_layout(p, L)), (hipStream_t)stream);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "list launch");
}

// Checks the description of a batch whose lists are to be filed; *kd_out gets its layout if lists exist for it
// (*has = true), else nothing is to be done for it.
static int check_next(const Params &p, const int64_t *indices, int64_t L, void *kept, size_t kept_bytes, const tt_shape_t *shape,
                      KeptDev *kd_out, bool *has)
{
    *has = false;
    if (L < 0) return fail(TT_ERR_BAD_ARG, "negative L");
    if (L >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "L >= 2^31");
    if (!kept_supported(p, L)) return TT_OK;
    if (!indices) return fail(TT_ERR_NULL, "indices is NULL");
    const size_t need = tt_emb_kept_bytes(shape, L);
    if (!kept || kept_bytes < need) return fail(TT_ERR_WORKSPACE, "kept buffer of %zu bytes needed, %zu given", need, kept_bytes);
    if (misaligned({kept})) return fail(TT_ERR_BAD_ARG, "the kept buffer must be 16-byte aligned");
    *kd_out = kept_dev(kept, kept_layout(p, L));
    *has = true;
    return TT_OK;
}

int tt_emb_kept_prepare(const tt_shape_t *shape, const int64_t *indices, int64_t L, const tt_cache_t *cache,
                        void *kept, size_t kept_bytes, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (fast_config(p) < 0) return fail(TT_ERR_UNSUPPORTED, "no kernel keeps intermediates for this shape");
    CacheDev cd;
    if ((rc = check_cache(cache, &cd, false))) return rc;
    KeptDev kd;
    bool has;
    if ((rc = check_next(p, indices, L, kept, kept_bytes, shape, &kd, &has))) return rc;
    if (!has) return TT_OK;
    kept_sort(p, indices, (int)L, cd, kd, (hipStream_t)stream);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "list launch");
}

// tt_emb_bwd_kept (cores_out == nullptr) and tt_emb_bwd_sgd_kept
static int bwd_kept_common(const tt_shape_t *shape, const float *const cores[3], const int64_t *indices, int64_t L,
                           const int64_t *offsets, int64_t n_bags, const float *alpha, const tt_cache_t *cache,
                           const float *grad_output, const void *kept, size_t kept_bytes, float *const grad_cores[3],
                           float *grad_cache, float lr, float *const cores_out[3], const tt_next_batch_t *next,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (fast_config(p) < 0) return fail(TT_ERR_UNSUPPORTED, "no kernel uses kept intermediates for this shape");
    if ((rc = check_lookup_args(indices, L, n_bags, offsets, p.N))) return rc;
    const size_t need = tt_emb_kept_bytes(shape, L);
    if (L > 0 && (!kept || kept_bytes < need))
        return fail(TT_ERR_WORKSPACE, "kept buffer of %zu bytes needed, %zu given", need, kept_bytes);
    CacheDev cd;
    if ((rc = check_cache(cache, &cd, false))) return rc;
    KpNext nx{nullptr, 0, 0, KeptDev{}};
    if (next) {
        bool has;
        if ((rc = check_next(p, next->indices, next->L, next->kept, next->kept_bytes, shape, &nx.kd, &has))) return rc;
        if (has) {
            nx.indices = next->indices;
            nx.L = (int)next->L;
            nx.n_sort = nx.kd.G;
        }
    }
    const bool fused = cores_out != nullptr;
    if (!kept_supported(p, L) || cd.K) {                                    // the kept T0 sits at the start of the buffer
        rc = bwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, grad_output, grad_cores, grad_cache, lr,
                        cores_out, L > 0 ? (const float *)kept : nullptr, workspace, workspace_bytes, stream);
        if (rc || !nx.n_sort) return rc;
        kept_sort(p, nx.indices, nx.L, cd, nx.kd, (hipStream_t)stream);     // no launch to ride along with: one of their own
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? TT_OK : hip_fail(e, "list launch");
    }
    if (!cores || !cores[0] || !cores[1] || !cores[2]) return fail(TT_ERR_NULL, "cores is NULL");
    if (fused) {
        if (!cores_out[0] || !cores_out[1] || !cores_out[2]) return fail(TT_ERR_NULL, "cores_out is NULL");
        for (int k = 0; k < 3; ++k)
            if (cores_out[k] == cores[k]) return fail(TT_ERR_BAD_ARG, "cores_out must not alias cores");
    } else if (!grad_cores || !grad_cores[0] || !grad_cores[1] || !grad_cores[2]) {
        return fail(TT_ERR_NULL, "grad_cores is NULL");
    }
    if (n_bags > 0 && !grad_output) return fail(TT_ERR_NULL, "grad_output is NULL");
    if (misaligned({cores[0], cores[1], cores[2], grad_output, kept}) ||
        (fused ? misaligned({cores_out[0], cores_out[1], cores_out[2]})
               : misaligned({grad_cores[0], grad_cores[1], grad_cores[2]})))
        return fail(TT_ERR_BAD_ARG, "cores, gradients and kept buffer must be 16-byte aligned");
    if (offsets && n_bags > 0 && L % n_bags == 0) {                         // a guess for the bag of a position
        p.bagP = (uint32_t)(L / n_bags);
        p.mgP = p.bagP > 1 ? (uint32_t)(((1ull << 32) + p.bagP - 1) / (uint64_t)p.bagP) : 0u;
    }
    const KeptDev kd = kept_dev(const_cast<void *>(kept), kept_layout(p, L));
    kept_bwd(p, cores[0], cores[1], cores[2], (int)L, offsets, (int)n_bags, alpha, grad_output,
             fused ? nullptr : grad_cores[0], fused ? nullptr : grad_cores[1], fused ? nullptr : grad_cores[2], lr,
             fused ? cores_out[0] : nullptr, fused ? cores_out[1] : nullptr, fused ? cores_out[2] : nullptr, kd, cd, nx,
             (hipStream_t)stream);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "backward launch");
}

int tt_emb_bwd_kept(const tt_shape_t *shape, const float *const cores[3],
                    const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                    const float *alpha, const tt_cache_t *cache,
                    const float *grad_output, const void *kept, size_t kept_bytes,
                    float *const grad_cores[3], float *grad_cache, const tt_next_batch_t *next,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    return bwd_kept_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, grad_output, kept, kept_bytes, grad_cores,
                           grad_cache, 0.f, nullptr, next, workspace, workspace_bytes, stream);
}

int tt_emb_bwd_sgd_kept(const tt_shape_t *shape, const float *const cores[3], float *const cores_out[3],
                        const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                        const float *alpha, const tt_cache_t *cache,
                        const float *grad_output, const void *kept, size_t kept_bytes, float lr,
                        const tt_next_batch_t *next, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!cores_out) return fail(TT_ERR_NULL, "cores_out is NULL");
    return bwd_kept_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, grad_output, kept, kept_bytes, nullptr,
                           nullptr, lr, cores_out, next, workspace, workspace_bytes, stream);
}

int tt_emb_debug_kept_lists(const tt_shape_t *shape, const void *kept, size_t kept_bytes, int64_t L,
                            int32_t *slice, int32_t *rep, int32_t *times, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (!kept_supported(p, L)) return fail(TT_ERR_UNSUPPORTED, "no lists are kept for this shape and length");
    if (!kept || !slice || !rep || !times) return fail(TT_ERR_NULL, "NULL array");
    const KeptLayout kl = kept_layout(p, L);
    if (kept_bytes < kl.bytes) return fail(TT_ERR_WORKSPACE, "kept buffer of %zu bytes needed, %zu given", kl.bytes, kept_bytes);
    hipStream_t st = (hipStream_t)stream;
    const int64_t n = 3 * L;
    hipLaunchKernelGGL(fill_i32_kernel, dim3(cdiv(n, WG) < 1024 ? cdiv(n, WG) : 1024), dim3(WG), 0, st, slice, n, -1);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(cdiv(n, WG) < 1024 ? cdiv(n, WG) : 1024), dim3(WG), 0, st, rep, n, -1);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(cdiv(n, WG) < 1024 ? cdiv(n, WG) : 1024), dim3(WG), 0, st, times, n, 0);
    hipLaunchKernelGGL(kept_lists_export_kernel, dim3(kl.nbins), dim3(WG), 0, st, p, kept_dev(const_cast<void *>(kept), kl), (int)L,
                       slice, rep, times);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "list export launch");
}

int tt_emb_bwd_prepare(const tt_shape_t *shape, const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                       const tt_cache_t *cache, int kept_t0, void *workspace, size_t workspace_bytes, void *stream)
{
    static const float marker = 0.f;                       // stands for "a kept T0 will be given": never dereferenced
    return bwd_common(shape, nullptr, indices, L, offsets, n_bags, nullptr, cache, nullptr, nullptr, nullptr, 0.f,
                      nullptr, kept_t0 ? &marker : nullptr, workspace, workspace_bytes, stream, BWD_PREPARE);
}

int tt_emb_bwd_has_prepass(const tt_shape_t *shape, int64_t L, int64_t cache_rows, int kept_t0)
{
    Params p;
    if (check_shape(shape, &p) != TT_OK || L <= 0 || cache_rows < 0) return 0;
    const bool fast = (g_fast_path || kept_t0) && fast_bwd_supported(p);
    const bool grouped = fast && (g_fast_path == 2 || L >= group_min_l(p, cache_rows, kept_t0 != 0, true));
    return cache_rows > 0 || grouped;
}

int tt_emb_bwd_two_calls_group_earlier(const tt_shape_t *shape, int64_t L, int64_t cache_rows, int kept_t0)
{
    Params p;
    if (check_shape(shape, &p) != TT_OK || L <= 0 || cache_rows < 0) return 0;
    const bool fast = (g_fast_path || kept_t0) && fast_bwd_supported(p);
    if (!fast || g_fast_path == 2) return 0;
    return L >= group_min_l(p, cache_rows, kept_t0 != 0, true) && L < group_min_l(p, cache_rows, kept_t0 != 0, false);
}

int tt_emb_bwd_sgd_prepared(const tt_shape_t *shape, const float *const cores[3], float *const cores_out[3],
                            const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                            const float *alpha, const tt_cache_t *cache,
                            const float *grad_output, const float *t0, float lr,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    if (!cores_out) return fail(TT_ERR_NULL, "cores_out is NULL");
    return bwd_common(shape, cores, indices, L, offsets, n_bags, alpha, cache, grad_output, nullptr, nullptr,
                      lr, cores_out, t0, workspace, workspace_bytes, stream, BWD_REST);
}

size_t tt_emb_bwd_sgd_workspace_bytes(const tt_shape_t *shape, int64_t L, int64_t n_bags, int64_t cache_rows)
{
    (void)n_bags;
    Params p;
    if (check_shape(shape, &p) != TT_OK || L < 0) return 0;
    if (cache_rows < 0 || cache_rows > (1 << 24)) return 0;
    size_t n = fwd_bwd_ws_bytes(p, L, cache_rows) + split_ws_bytes_max(p, L) + align256((size_t)cache_rows * p.N * 4);
    n += align256((size_t)p.m1 * p.sA * 4) + align256((size_t)p.m2 * p.sB * 4) + align256((size_t)p.m3 * p.sC * 4);
    return n;
}

int tt_emb_sgd_update(const tt_shape_t *shape, float *const cores[3], float *const grad_cores[3],
                      float lr, const tt_cache_t *cache, float *grad_cache, int zero_grad, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (!cores || !cores[0] || !cores[1] || !cores[2]) return fail(TT_ERR_NULL, "cores is NULL");
    if (!grad_cores || !grad_cores[0] || !grad_cores[1] || !grad_cores[2])
        return fail(TT_ERR_NULL, "grad_cores is NULL");
    CacheDev cd;
    if ((rc = check_cache(cache, &cd, true))) return rc;
    if (cd.K && !grad_cache) return fail(TT_ERR_NULL, "grad_cache is NULL but a cache is given");
    SgdArgs a;
    const int64_t sizes[4] = {(int64_t)p.m1 * p.sA, (int64_t)p.m2 * p.sB, (int64_t)p.m3 * p.sC,
                              cd.K ? (int64_t)cd.K * p.N : 0};
    a.start4[0] = 0;
    a.tail[0] = 0;
    for (int k = 0; k < 4; ++k) {
        a.x[k] = k < 3 ? cores[k] : (cd.K ? cache->rows : nullptr);
        a.g[k] = k < 3 ? grad_cores[k] : (cd.K ? grad_cache : nullptr);
        a.count[k] = sizes[k];
        a.start4[k + 1] = a.start4[k] + sizes[k] / 4;
        a.tail[k + 1] = a.tail[k] + sizes[k] % 4;
    }
    for (int k = 0; k < 4; ++k)
        if (sizes[k] && ((((uintptr_t)a.x[k]) | ((uintptr_t)a.g[k])) & 15))
            return fail(TT_ERR_BAD_ARG, "cores and gradients must be 16-byte aligned");
    const int64_t total = a.start4[4] + a.tail[4];
    int grid = cdiv(total, WG);
    if (grid > 4096) grid = 4096;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(sgd_kernel, dim3(grid), dim3(WG), 0, (hipStream_t)stream, a, lr, zero_grad);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "sgd launch");
}

int tt_cache_lookup(const tt_cache_t *cache, const int64_t *indices, int64_t L, int32_t *slot, void *stream)
{
    if (!cache) return fail(TT_ERR_NULL, "cache is NULL");
    if (L < 0) return fail(TT_ERR_BAD_ARG, "negative L");
    if (L >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "L >= 2^31");
    if (L > 0 && (!indices || !slot)) return fail(TT_ERR_NULL, "indices or slot is NULL");
    CacheDev cd;
    int rc = check_cache(cache, &cd, false);
    if (rc) return rc;
    if (L == 0) return TT_OK;
    hipLaunchKernelGGL(cache_lookup_kernel, dim3(cdiv(L, WG)), dim3(WG), 0, (hipStream_t)stream, cd, indices, (int)L, slot);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "cache lookup launch");
}

int tt_cache_build(const tt_shape_t *shape, const float *const cores[3],
                   const int64_t *cand_rows, const int64_t *cand_counts, int64_t n_cand,
                   const tt_cache_t *out, void *workspace, size_t workspace_bytes, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (!cores || !cores[0] || !cores[1] || !cores[2]) return fail(TT_ERR_NULL, "cores is NULL");
    if (!out) return fail(TT_ERR_NULL, "out is NULL");
    if (n_cand < 0 || n_cand >= (1ll << 31)) return fail(TT_ERR_BAD_ARG, "n_cand out of range");
    if (out->K < 0 || out->K > n_cand) return fail(TT_ERR_BAD_ARG, "K must be in [0, n_cand]");
    CacheDev cd;
    if ((rc = check_cache(out, &cd, true))) return rc;
    if (out->K == 0) return TT_OK;
    if (!cand_rows || !cand_counts) return fail(TT_ERR_NULL, "candidate arrays are NULL");
    const size_t need = sort_ws_layout(nullptr, n_cand).bytes;
    if (!workspace || workspace_bytes < need)
        return fail(TT_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    const int K = (int)out->K, n = (int)n_cand;
    SortWs ws = sort_ws_layout(workspace, n_cand);

    // 1. order the candidates: most used first, ties by row id
    hipLaunchKernelGGL(cand_keys_kernel, dim3(cdiv(n, WG)), dim3(WG), 0, st, cand_rows, cand_counts, n, ws.k0);
    uint64_t *ks; uint32_t *vs;
    hipError_t e = radix_sort(ws, n, 64, st, &ks, &vs);
    if (e != hipSuccess) return hip_fail(e, "cache sort");
    // 2. the first K become slots 0..K-1
    hipLaunchKernelGGL(take_keys_kernel, dim3(cdiv(K, WG)), dim3(WG), 0, st, ks, K, out->keys);
    // 3. row -> slot map
    hipLaunchKernelGGL(fill_u64_kernel, dim3(cdiv(out->capacity, WG)), dim3(WG), 0, st, out->table,
                       out->capacity, CACHE_EMPTY);
    hipLaunchKernelGGL(cache_insert_kernel, dim3(cdiv(K, WG)), dim3(WG), 0, st, out->keys, K, out->table,
                       (uint32_t)(out->capacity - 1));
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "cache build launch");
    // 4. lines initialised from the cores: one bag per cached row, no cache consulted
    return tt_emb_fwd(shape, cores, out->keys, K, nullptr, K, nullptr, nullptr, out->rows, nullptr, 0, stream);
}

size_t tt_cache_refill_workspace_bytes(const tt_shape_t *shape, int64_t n_cand, int64_t K)
{
    Params p;
    if (check_shape(shape, &p) != TT_OK || n_cand < 0 || K < 0 || K > (1 << 24)) return 0;
    return sort_ws_layout(nullptr, n_cand > 0 ? n_cand : 1).bytes + align256((size_t)K * 8) +
           align256((size_t)K * p.N * 4) + 256;
}

int tt_cache_refill(const tt_shape_t *shape, const float *const cores[3],
                    const int64_t *cand_rows, const int64_t *cand_counts, int64_t n_cand,
                    const tt_cache_t *cache, void *workspace, size_t workspace_bytes, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (!cores || !cores[0] || !cores[1] || !cores[2]) return fail(TT_ERR_NULL, "cores is NULL");
    if (!cache) return fail(TT_ERR_NULL, "cache is NULL");
    if (n_cand < 0 || n_cand >= (1ll << 31)) return fail(TT_ERR_BAD_ARG, "n_cand out of range");
    if (cache->K < 0 || cache->K > n_cand) return fail(TT_ERR_BAD_ARG, "K must be in [0, n_cand]");
    CacheDev cd;
    if ((rc = check_cache(cache, &cd, true))) return rc;
    if (cache->K == 0) return TT_OK;
    if (!cand_rows || !cand_counts) return fail(TT_ERR_NULL, "candidate arrays are NULL");
    const size_t need = tt_cache_refill_workspace_bytes(shape, n_cand, cache->K);
    if (!workspace || workspace_bytes < need)
        return fail(TT_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    const int K = (int)cache->K, n = (int)n_cand;
    SortWs ws = sort_ws_layout(workspace, n_cand);
    int64_t *new_keys = (int64_t *)((char *)workspace + ws.bytes);
    float *new_rows = (float *)((char *)new_keys + align256((size_t)K * 8));

    // 1. the K most used candidates, most used first, ties by row id
    hipLaunchKernelGGL(cand_keys_kernel, dim3(cdiv(n, WG)), dim3(WG), 0, st, cand_rows, cand_counts, n, ws.k0);
    uint64_t *ks; uint32_t *vs;
    hipError_t e = radix_sort(ws, n, 64, st, &ks, &vs);
    if (e != hipSuccess) return hip_fail(e, "cache sort");
    hipLaunchKernelGGL(take_keys_kernel, dim3(cdiv(K, WG)), dim3(WG), 0, st, ks, K, new_keys);
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "cache refill launch");
    // 2. their lines: a forward pass of one bag per row THROUGH THE OLD CACHE, so a row that stays
    //    cached keeps its line and a row that enters is rebuilt from the cores
    rc = tt_emb_fwd(shape, cores, new_keys, K, nullptr, K, nullptr, cache, new_rows, nullptr, 0, stream);
    if (rc) return rc;
    // 3. the new set replaces the old one
    const int64_t nr = (int64_t)K * p.N;
    hipLaunchKernelGGL(copy_i64_kernel, dim3(cdiv(K, WG)), dim3(WG), 0, st, new_keys, cache->keys, (int64_t)K);
    hipLaunchKernelGGL(copy_f32_kernel, dim3(cdiv(nr, WG) < 2048 ? cdiv(nr, WG) : 2048), dim3(WG), 0, st, new_rows,
                       cache->rows, nr);
    hipLaunchKernelGGL(fill_u64_kernel, dim3(cdiv(cache->capacity, WG)), dim3(WG), 0, st, cache->table,
                       cache->capacity, CACHE_EMPTY);
    hipLaunchKernelGGL(cache_insert_kernel, dim3(cdiv(K, WG)), dim3(WG), 0, st, cache->keys, K, cache->table,
                       (uint32_t)(cache->capacity - 1));
    e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "cache refill launch");
}

static int check_freq(const tt_freq_t *f, FreqDev *d)
{
    if (!f) return fail(TT_ERR_NULL, "tracker is NULL");
    if (f->capacity < 64 || f->capacity > (1ll << 31) || (f->capacity & (f->capacity - 1)))
        return fail(TT_ERR_BAD_ARG, "tracker capacity must be a power of two in [64, 2^31]");
    if (!f->table || !f->stats) return fail(TT_ERR_NULL, "tracker array is NULL");
    d->table = (unsigned long long *)f->table;
    d->stats = (unsigned long long *)f->stats;
    d->mask = (uint32_t)(f->capacity - 1);
    return TT_OK;
}

int tt_freq_reset(const tt_freq_t *tracker, void *stream)
{
    FreqDev f;
    int rc = check_freq(tracker, &f);
    if (rc) return rc;
    hipLaunchKernelGGL(freq_reset_kernel, dim3(cdiv(tracker->capacity, WG)), dim3(WG), 0, (hipStream_t)stream, f);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "tracker reset launch");
}

int tt_freq_update(const tt_freq_t *tracker, const int64_t *indices, int64_t L, void *stream)
{
    FreqDev f;
    int rc = check_freq(tracker, &f);
    if (rc) return rc;
    if (L < 0) return fail(TT_ERR_BAD_ARG, "negative L");
    if (L >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "L >= 2^31");
    if (L == 0) return TT_OK;
    if (!indices) return fail(TT_ERR_NULL, "indices is NULL");
    if (L >= 16384)
        hipLaunchKernelGGL(freq_update_chunk_kernel, dim3(cdiv(L, FQ_CHUNK)), dim3(WG), 0, (hipStream_t)stream, f, indices, (int)L);
    else
        hipLaunchKernelGGL(freq_update_kernel, dim3(cdiv(L, WG)), dim3(WG), 0, (hipStream_t)stream, f, indices, (int)L);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "tracker update launch");
}

int tt_freq_export(const tt_freq_t *tracker, int64_t *rows, int64_t *counts, int64_t *n_out, void *stream)
{
    FreqDev f;
    int rc = check_freq(tracker, &f);
    if (rc) return rc;
    if (!rows || !counts || !n_out) return fail(TT_ERR_NULL, "NULL array");
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(freq_zero_kernel, dim3(1), dim3(64), 0, st, (unsigned long long *)n_out);
    hipLaunchKernelGGL(freq_export_kernel, dim3(cdiv(tracker->capacity, WG)), dim3(WG), 0, st, f, rows, counts,
                       (unsigned long long *)n_out);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "tracker export launch");
}

static int check_dense(const float *table, int64_t num_rows, int32_t N, const int64_t *indices, int64_t L,
                       const int64_t *offsets, int64_t n_bags)
{
    if (num_rows <= 0 || N <= 0 || N % 4 || N > 256 || (N & (N - 1))) return fail(TT_ERR_BAD_ARG, "N must be a power of two in [4, 256]");
    int rc = check_lookup_args(indices, L, n_bags, offsets, N);
    if (rc) return rc;
    if (!table) return fail(TT_ERR_NULL, "table is NULL");
    return TT_OK;
}

int tt_dense_bag_fwd(const float *table, int64_t num_rows, int32_t N,
                     const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                     const float *alpha, float *output, void *stream)
{
    int rc = check_dense(table, num_rows, N, indices, L, offsets, n_bags);
    if (rc) return rc;
    if (n_bags > 0 && !output) return fail(TT_ERR_NULL, "output is NULL");
    if (misaligned({table, output})) return fail(TT_ERR_BAD_ARG, "table and output must be 16-byte aligned");
    if (n_bags == 0) return TT_OK;
    hipLaunchKernelGGL(dense_fwd_kernel, dim3(cdiv(n_bags, NWAVE)), dim3(WG), 0, (hipStream_t)stream, table, (int)N,
                       indices, offsets, (int)n_bags, alpha, output);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "dense forward launch");
}

int tt_dense_bag_bwd_sgd(float *table, int64_t num_rows, int32_t N,
                         const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                         const float *alpha, const float *grad_output, float lr, void *stream)
{
    int rc = check_dense(table, num_rows, N, indices, L, offsets, n_bags);
    if (rc) return rc;
    if (n_bags > 0 && !grad_output) return fail(TT_ERR_NULL, "grad_output is NULL");
    if (misaligned({table, grad_output})) return fail(TT_ERR_BAD_ARG, "table and grad_output must be 16-byte aligned");
    if (n_bags == 0 || L == 0) return TT_OK;
    hipLaunchKernelGGL(dense_bwd_sgd_kernel, dim3(cdiv(n_bags, NWAVE)), dim3(WG), 0, (hipStream_t)stream, table, (int)N,
                       indices, offsets, (int)n_bags, alpha, grad_output, lr);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "dense backward launch");
}

size_t tt_dense_bag_bwd_workspace_bytes(int64_t L, int32_t N)
{
    if (L < 0 || L >= (1ll << 31) || N <= 0 || N > 256) return 0;
    return dense_ws_layout(nullptr, L > 0 ? L : 1, N).bytes;
}

int tt_dense_bag_bwd_sgd_merged(float *table, int64_t num_rows, int32_t N,
                                const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                                const float *alpha, const float *grad_output, float lr,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_dense(table, num_rows, N, indices, L, offsets, n_bags);
    if (rc) return rc;
    if (n_bags > 0 && !grad_output) return fail(TT_ERR_NULL, "grad_output is NULL");
    if (misaligned({table, grad_output, workspace})) return fail(TT_ERR_BAD_ARG, "table, grad_output and workspace must be 16-byte aligned");
    if (n_bags == 0 || L == 0) return TT_OK;
    const size_t need = tt_dense_bag_bwd_workspace_bytes(L, N);
    if (!workspace || workspace_bytes < need)
        return fail(TT_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    DenseWs ws = dense_ws_layout(workspace, L, N);
    const int n = (int)L;
    int bits = 1;
    while (bits < 63 && (1ull << bits) <= (uint64_t)num_rows - 1) ++bits;
    hipLaunchKernelGGL(dense_keys_kernel, dim3(cdiv(n, WG)), dim3(WG), 0, st, indices, n, ws.sort.k0);
    uint64_t *ks; uint32_t *vs;
    hipError_t e = radix_sort(ws.sort, n, bits, st, &ks, &vs);
    if (e != hipSuccess) return hip_fail(e, "dense backward sort");
    const int tiles = (int)cdiv(n, DT);
    const int bag_len = offsets && L % n_bags == 0 ? (int)(L / n_bags) : 0;     // a guess that the kernel checks
    if (N <= 64)
        hipLaunchKernelGGL((dense_seg_kernel<1, 16>), dim3(cdiv(tiles, NWAVE)), dim3(WG), 0, st, table, (int)N, ks, vs, n,
                           offsets, (int)n_bags, bag_len, alpha, grad_output, lr, ws.part);
    else
        hipLaunchKernelGGL((dense_seg_kernel<4, 8>), dim3(cdiv(tiles, NWAVE)), dim3(WG), 0, st, table, (int)N, ks, vs, n,
                           offsets, (int)n_bags, bag_len, alpha, grad_output, lr, ws.part);
    hipLaunchKernelGGL(dense_fix_kernel, dim3(cdiv(tiles, NWAVE)), dim3(WG), 0, st, table, (int)N, ks, n, lr, ws.part);
    e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "dense backward launch");
}

int tt_emb_mean_weights(const int64_t *offsets, int64_t n_bags, int64_t L, const float *alpha, float *weights, void *stream)
{
    if (n_bags < 0 || L < 0) return fail(TT_ERR_BAD_ARG, "negative count");
    if (n_bags >= (1ll << 31) || L >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "count >= 2^31");
    if (L == 0 || n_bags == 0) return TT_OK;
    if (!offsets || !weights) return fail(TT_ERR_NULL, "NULL array");
    hipLaunchKernelGGL(mean_weights_kernel, dim3(cdiv(n_bags, NWAVE)), dim3(WG), 0, (hipStream_t)stream, offsets,
                       (int)n_bags, alpha, weights);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "mean weights launch");
}

int tt_init_sampled_gaussian(const tt_shape_t *shape, float *const cores[3], uint64_t seed, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (!cores || !cores[0] || !cores[1] || !cores[2]) return fail(TT_ERR_NULL, "cores is NULL");
    const double scale = sampled_gaussian_scale(shape->num_rows, p.R1, p.R2);
    const int64_t count[3] = {(int64_t)p.m1 * p.sA, (int64_t)p.m2 * p.sB, (int64_t)p.m3 * p.sC};
    for (int k = 0; k < 3; ++k) {
        const int grid = cdiv(count[k], WG) < 4096 ? cdiv(count[k], WG) : 4096;
        hipLaunchKernelGGL(init_sampled_gaussian_kernel, dim3(grid), dim3(WG), 0, (hipStream_t)stream, cores[k], count[k], k,
                           seed, scale);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "initialisation launch");
}

static int check_shape_d(const tt_shape_d_t *sh, ShapeD *out)
{
    if (!sh) return fail(TT_ERR_NULL, "shape is NULL");
    if (sh->d < 2 || sh->d > DMAX) return fail(TT_ERR_BAD_SHAPE, "d must be 2, 3 or 4");
    if (sh->r[0] != 1 || sh->r[sh->d] != 1) return fail(TT_ERR_BAD_SHAPE, "boundary ranks must be 1");
    ShapeD s;
    memset(&s, 0, sizeof(s));
    s.d = sh->d;
    int64_t rows = 1, N = 1;
    for (int k = 0; k < sh->d; ++k) {
        if (sh->m[k] <= 0 || sh->n[k] <= 0 || sh->r[k] <= 0 || sh->r[k + 1] <= 0)
            return fail(TT_ERR_BAD_SHAPE, "factors and ranks must be positive");
        s.m[k] = sh->m[k]; s.n[k] = sh->n[k]; s.r[k] = sh->r[k];
        rows *= sh->m[k];
        N *= sh->n[k];
        if (rows >= (1ll << 31) || N > DBUF) return fail(TT_ERR_UNSUPPORTED, "table too large for the general-d kernels");
        const int64_t slice = (int64_t)sh->r[k] * sh->n[k] * sh->r[k + 1];
        if (slice > DBUF) return fail(TT_ERR_UNSUPPORTED, "a core slice exceeds %d values", DBUF);
        s.slice[k] = (int)slice;
    }
    s.r[sh->d] = 1;
    s.N = (int)N;
    if (sh->num_rows <= 0 || sh->num_rows > rows) return fail(TT_ERR_BAD_SHAPE, "num_rows must be in [1, prod(m)]");
    // every intermediate of the chain has to fit one LDS buffer
    int64_t nl = 1;
    for (int k = 0; k < sh->d; ++k) {
        int64_t nr = 1;
        for (int q = k + 1; q < sh->d; ++q) nr *= sh->n[q];
        const int64_t left = nl * sh->r[k], right = (int64_t)sh->r[k + 1] * nr, tt = (int64_t)sh->r[k] * sh->n[k] * nr;
        nl *= sh->n[k];
        const int64_t part = nl * sh->r[k + 1];
        if (left > DBUF || right > DBUF || tt > DBUF || part > DBUF)
            return fail(TT_ERR_UNSUPPORTED, "an intermediate product exceeds %d values", DBUF);
    }
    if (out) *out = s;
    return TT_OK;
}

int tt_embd_fwd(const tt_shape_d_t *shape, const float *const cores[4],
                const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                const float *alpha, float *output, void *stream)
{
    ShapeD s;
    int rc = check_shape_d(shape, &s);
    if (rc) return rc;
    if ((rc = check_lookup_args(indices, L, n_bags, offsets, s.N))) return rc;
    if (!cores) return fail(TT_ERR_NULL, "cores is NULL");
    for (int k = 0; k < s.d; ++k)
        if (!cores[k]) return fail(TT_ERR_NULL, "cores is NULL");
    if (n_bags > 0 && !output) return fail(TT_ERR_NULL, "output is NULL");
    if (n_bags == 0) return TT_OK;
    const int grid = (int)(n_bags < 16384 ? n_bags : 16384);
    hipLaunchKernelGGL(fwd_anyd_kernel, dim3(grid), dim3(WG), 0, (hipStream_t)stream, s, cores[0], cores[1],
                       s.d > 2 ? cores[2] : nullptr, s.d > 3 ? cores[3] : nullptr, indices, offsets, (int)n_bags, alpha, output);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "forward launch");
}

int tt_embd_bwd(const tt_shape_d_t *shape, const float *const cores[4],
                const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                const float *alpha, const float *grad_output, float *const grad_cores[4], void *stream)
{
    ShapeD s;
    int rc = check_shape_d(shape, &s);
    if (rc) return rc;
    if ((rc = check_lookup_args(indices, L, n_bags, offsets, s.N))) return rc;
    if (!cores || !grad_cores) return fail(TT_ERR_NULL, "cores or grad_cores is NULL");
    for (int k = 0; k < s.d; ++k)
        if (!cores[k] || !grad_cores[k]) return fail(TT_ERR_NULL, "cores or grad_cores is NULL");
    if (n_bags > 0 && !grad_output) return fail(TT_ERR_NULL, "grad_output is NULL");
    if (L == 0) return TT_OK;
    int grid = 0;
    for (int k = 0; k < s.d; ++k) grid += s.m[k];
    hipLaunchKernelGGL(bwd_anyd_kernel, dim3(grid), dim3(WG), 0, (hipStream_t)stream, s, cores[0], cores[1],
                       s.d > 2 ? cores[2] : nullptr, s.d > 3 ? cores[3] : nullptr, indices, (int)L, offsets, (int)n_bags,
                       alpha, grad_output, grad_cores[0], grad_cores[1], s.d > 2 ? grad_cores[2] : nullptr,
                       s.d > 3 ? grad_cores[3] : nullptr);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "backward launch");
}

int tt_embd_sgd_update(const tt_shape_d_t *shape, float *const cores[4], float *const grad_cores[4], float lr,
                       int zero_grad, void *stream)
{
    ShapeD s;
    int rc = check_shape_d(shape, &s);
    if (rc) return rc;
    if (!cores || !grad_cores) return fail(TT_ERR_NULL, "cores or grad_cores is NULL");
    for (int k = 0; k < s.d; ++k)
        if (!cores[k] || !grad_cores[k]) return fail(TT_ERR_NULL, "cores or grad_cores is NULL");
    for (int k = 0; k < s.d; ++k) {
        const int64_t n = (int64_t)s.m[k] * s.slice[k];
        hipLaunchKernelGGL(sgd_plain_kernel, dim3(cdiv(n, WG) < 2048 ? cdiv(n, WG) : 2048), dim3(WG), 0, (hipStream_t)stream,
                           cores[k], grad_cores[k], n, lr, zero_grad);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "sgd launch");
}

int tt_emb_debug_decode(const tt_shape_t *shape, const int64_t *indices, int64_t L,
                        int32_t *i1, int32_t *i2, int32_t *i3, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (L < 0) return fail(TT_ERR_BAD_ARG, "negative L");
    if (L >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "L >= 2^31");
    if (L == 0) return TT_OK;
    if (!indices || !i1 || !i2 || !i3) return fail(TT_ERR_NULL, "NULL array");
    hipLaunchKernelGGL(decode_kernel, dim3(cdiv(L, WG)), dim3(WG), 0, (hipStream_t)stream, p, indices, (int)L, i1, i2, i3);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "decode launch");
}

int tt_emb_validate(const tt_shape_t *shape, const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                    int32_t *flag, void *stream)
{
    int rc = check_shape(shape, nullptr);
    if (rc) return rc;
    if ((rc = check_lookup_args(indices, L, n_bags, offsets, 1))) return rc;
    if (!flag) return fail(TT_ERR_NULL, "flag is NULL");
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(WG), 0, st, flag, (int64_t)1, 0);
    const int64_t n = L > n_bags + 1 ? L : n_bags + 1;
    hipLaunchKernelGGL(validate_kernel, dim3(cdiv(n, WG) < 2048 ? cdiv(n, WG) : 2048), dim3(WG), 0, st, shape->num_rows,
                       indices, L, offsets, n_bags, flag);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "validate launch");
}

int tt_emb_debug_launch_probe(int32_t blocks, int32_t *sink, void *stream)
{
    if (blocks < 1 || blocks > (1 << 20)) return fail(TT_ERR_BAD_ARG, "blocks must be in [1, 2^20]");
    hipLaunchKernelGGL(launch_probe_kernel, dim3(blocks), dim3(WG), 0, (hipStream_t)stream, sink);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "probe launch");
}

int tt_emb_debug_decode_as(const tt_shape_t *shape, const int64_t *indices, int64_t L, int mode,
                           int32_t *i1, int32_t *i2, int32_t *i3, void *stream)
{
    if (mode == 0) return tt_emb_debug_decode(shape, indices, L, i1, i2, i3, stream);
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (mode != 1 && mode != 2) return fail(TT_ERR_BAD_ARG, "mode must be 0, 1 or 2");
    if (L < 0) return fail(TT_ERR_BAD_ARG, "negative L");
    if (L >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "L >= 2^31");
    if (L == 0) return TT_OK;
    if (!indices || !i1 || !i2 || !i3) return fail(TT_ERR_NULL, "NULL array");
    hipLaunchKernelGGL(decode_as_kernel, dim3(cdiv(L, WG)), dim3(WG), 0, (hipStream_t)stream, p, indices, (int)L, mode, i1, i2, i3);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "decode launch");
}

int tt_emb_debug_dedup(const tt_shape_t *shape, const int64_t *indices, int64_t L,
                       const int32_t *slot, int which,
                       int64_t *uniq, int32_t *count, int32_t *perm, int64_t *n_out,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    Params p;
    int rc = check_shape(shape, &p);
    if (rc) return rc;
    if (L < 0) return fail(TT_ERR_BAD_ARG, "negative L");
    if (L >= (1ll << 31)) return fail(TT_ERR_UNSUPPORTED, "L >= 2^31");
    if (which < 0 || which > 3) return fail(TT_ERR_BAD_ARG, "which must be 0..3");
    if (!n_out) return fail(TT_ERR_NULL, "n_out is NULL");
    hipStream_t st = (hipStream_t)stream;
    if (L > 0) {
        if (!indices || !uniq || !count || !perm) return fail(TT_ERR_NULL, "NULL array");
        const size_t need = sort_ws_layout(nullptr, L).bytes;
        if (!workspace || workspace_bytes < need)
            return fail(TT_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    }
    hipLaunchKernelGGL(uq_init_kernel, dim3(1), dim3(64), 0, st, n_out, L);
    if (L == 0) {
        hipError_t e0 = hipGetLastError();
        return e0 == hipSuccess ? TT_OK : hip_fail(e0, "dedup launch");
    }
    SortWs ws = sort_ws_layout(workspace, L);
    const int n = (int)L;
    // number of key bits: the sentinel (all ones) must exceed every real key
    const uint64_t maxkey = which == 0 ? (uint64_t)shape->num_rows - 1
                                       : (uint64_t)(which == 1 ? p.m1 : (which == 2 ? p.m2 : p.m3)) - 1;
    int bits = 1;
    while (((1ull << bits) - 1) <= maxkey) ++bits;
    const uint64_t sentinel = (1ull << bits) - 1;
    hipLaunchKernelGGL(dedup_keys_kernel, dim3(cdiv(n, WG)), dim3(WG), 0, st, p, indices, n, slot, which, sentinel, ws.k0);
    uint64_t *ks; uint32_t *vs;
    hipError_t e = radix_sort(ws, n, bits, st, &ks, &vs);
    if (e != hipSuccess) return hip_fail(e, "dedup sort");
    const int nblk = rs_blocks(n);
    hipLaunchKernelGGL(uq_count_kernel, dim3(nblk), dim3(WG), 0, st, ks, n, sentinel, ws.blk);
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(SCAN_WG), 0, st, ws.blk, nblk);
    hipLaunchKernelGGL(uq_write_kernel, dim3(nblk), dim3(WG), 0, st, ks, n, sentinel, ws.blk, nblk, ws.head_pos, uniq, n_out);
    hipLaunchKernelGGL(uq_counts_kernel, dim3(cdiv(n, WG)), dim3(WG), 0, st, ws.head_pos, n_out, count, n);
    hipLaunchKernelGGL(copy_perm_kernel, dim3(cdiv(n, WG)), dim3(WG), 0, st, vs, n, perm);
    e = hipGetLastError();
    return e == hipSuccess ? TT_OK : hip_fail(e, "dedup launch");
}


}  // extern "C"
