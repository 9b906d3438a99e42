/*
 * tt_emb.h - C ABI of the TT-EmbeddingBag library for AMD MI355X (gfx950).
 *
 * The library computes the forward and backward pass of an embedding bag whose
 * table W (num_rows x N) is stored in TT-matrix format with d = 3 cores
 * (paper: Section 2, Eq. 2; Section 3.1, Eq. 3-4; Section 4.1, Eq. 5-6 and
 * Alg. 1-2), the SGD update of the cores (Section 5), and the uncompressed
 * cache of the most frequently used rows (Section 4.2).
 *
 * Conventions common to every entry point
 * ---------------------------------------
 *  - tt_shape_t and tt_cache_t are read from HOST memory.  Every other pointer is
 *    DEVICE memory owned by the caller, unless a comment says "host".  The
 *    library allocates nothing and frees nothing; temporary storage comes from a
 *    caller-provided workspace whose size the *_workspace_bytes queries return.
 *  - Core k (k = 0,1,2) is a contiguous fp32 array G_k[m_k][r_k][n_k][r_{k+1}]
 *    with r_0 = r_3 = 1: the paper's G_k in R^{r_{k-1} x m_k x n_k x r_k} with the
 *    row digit in front, so that the slice selected by one digit is one
 *    contiguous block.
 *  - Row index i has digits i = i1*m2*m3 + i2*m3 + i3 (i1 most significant,
 *    Section 3.1).  Only 0 <= i < num_rows <= m1*m2*m3 may be looked up; this is a
 *    precondition on `indices` that only tt_emb_validate checks on the device.
 *  - An embedding row has N = n1*n2*n3 columns; column j = (j1*n2 + j2)*n3 + j3.
 *  - Bags are given in CSR form: offsets[0..n_bags], offsets[0] = 0,
 *    non-decreasing, offsets[n_bags] = L; bag b pools positions
 *    offsets[b] <= k < offsets[b+1] by summation (Section 4.1).  offsets == NULL
 *    means n_bags == L and one index per bag.  alpha is an optional per-position
 *    weight (Eq. 5); NULL means 1.
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream) and the calls return without waiting for it.
 *  - Return value: TT_OK or a negative TT_ERR_* code; tt_last_error() gives a
 *    text for the last failure on the calling thread.  No C++ exception crosses
 *    the boundary.  On error nothing has been enqueued.
 *  - Every fp32 array (cores, outputs, gradients, cache rows, kept T0) and every
 *    workspace must start on a 16-byte boundary; TT_ERR_BAD_ARG otherwise.
 *  - Limits: d = 3, num_rows < 2^31, L < 2^31 (3 L < 2^31 in the backward pass of
 *    the shapes with a specialised kernel), n_bags * N < 2^31, fp32 data;
 *    TT_ERR_UNSUPPORTED beyond them.
 */
#ifndef TT_EMB_H
#define TT_EMB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    TT_OK = 0,
    TT_ERR_NULL = -1,        /* a required pointer is NULL                               */
    TT_ERR_BAD_SHAPE = -2,   /* d != 3, r[0] or r[3] != 1, a factor <= 0, prod(m) < rows  */
    TT_ERR_BAD_ARG = -3,     /* negative count, K > n_cand, capacity not a power of two.. */
    TT_ERR_WORKSPACE = -4,   /* workspace missing or smaller than the query's answer     */
    TT_ERR_HIP = -5,         /* a HIP call or a kernel launch failed                     */
    TT_ERR_UNSUPPORTED = -6  /* within the interface but beyond this build's limits      */
};

/* Shape of one TT-compressed table (Section 2, Eq. 2).  Host memory. */
typedef struct tt_shape_t {
    int32_t d;          /* number of cores, must be 3                               */
    int64_t num_rows;   /* rows that may be looked up, <= m[0]*m[1]*m[2]            */
    int32_t m[3];       /* row factorisation                                        */
    int32_t n[3];       /* column factorisation, N = n[0]*n[1]*n[2]                 */
    int32_t r[4];       /* TT ranks, r[0] = r[3] = 1                                */
} tt_shape_t;

/* The cache of uncompressed rows (Section 4.2).  The struct is host memory; the
 * three arrays are device memory that the caller allocates and tt_cache_build
 * fills.  Slot s holds row keys[s]; rows[s][0..N) is its embedding row.  `table`
 * is an open-addressing hash map row -> slot with `capacity` entries
 * (tt_cache_table_capacity(K)); its encoding is private to the library. */
typedef struct tt_cache_t {
    int64_t K;
    int64_t capacity;
    float *rows;          /* [K][N]     */
    int64_t *keys;        /* [K]        */
    uint64_t *table;      /* [capacity] */
} tt_cache_t;

/* Per-row use counts that feed the cache's refills (Section 4.2), held in a hash
 * table in device memory.  The struct is
 * host memory; `table` ([capacity] 64-bit words, private encoding) and `stats`
 * ([2]: distinct rows tracked, accesses dropped because the table was full) are
 * device memory that the caller allocates; capacity is a power of two >= 64 and
 * should be at least twice the number of distinct rows expected.  One row can be
 * counted up to 2^32 - 1 times between resets. */
typedef struct tt_freq_t {
    int64_t capacity;
    uint64_t *table;      /* [capacity] */
    int64_t *stats;       /* [2]        */
} tt_freq_t;

/* Shape of a table with any number of cores d in {2, 3, 4} (Section 4.1: the
 * algorithms are given for three cores and generalise to any TT dimension).  Host
 * memory.  Core k is fp32 [m[k]][r[k]][n[k]][r[k+1]], r[0] = r[d] = 1; the row digits
 * are mixed radix with digit 0 most significant.  Entries past d are ignored. */
typedef struct tt_shape_d_t {
    int32_t d;
    int64_t num_rows;
    int32_t m[4];
    int32_t n[4];
    int32_t r[5];
} tt_shape_d_t;

/* Text of the last error on this thread ("" if none).  Host pointer, valid until
 * the next failing call on the same thread. */
const char *tt_last_error(void);

/* Smallest table capacity tt_cache_build accepts for K rows (a power of two). */
int64_t tt_cache_table_capacity(int64_t K);

/* Bytes of device workspace that is always enough for tt_emb_fwd / tt_emb_bwd with L
 * positions in n_bags bags and a cache of cache_rows rows (0 = no cache).  tt_emb_fwd needs
 * none.  tt_emb_bwd needs none for a short index stream without a cache; with a cache, or from
 * 4096 positions on (from there on, depending on the shape, several workgroups share a slice and
 * leave partial sums in the workspace; from 32768 positions on, 16384 with a cache, the positions
 * are grouped with a device sort first), it reports TT_ERR_WORKSPACE if the workspace is missing
 * or too small.  Returns 0 on a bad shape. */
size_t tt_emb_workspace_bytes(const tt_shape_t *shape, int64_t L, int64_t n_bags, int64_t cache_rows);

/* Bytes of device workspace tt_cache_build needs for n_cand candidates. */
size_t tt_cache_build_workspace_bytes(const tt_shape_t *shape, int64_t n_cand, int64_t K);

/* Bytes of device workspace tt_emb_debug_dedup needs for L keys. */
size_t tt_emb_dedup_workspace_bytes(int64_t L);

/*
 * Forward pass (Section 4.1, Eq. 5-6, Alg. 1; cached rows per Section 4.2):
 *   output[b][:] = sum_{k in bag b} alpha[k] * row(indices[k]),
 *   row(i) = G1[i1] G2[i2] G3[i3] (Eq. 3), or cache->rows[slot] if i is cached.
 * cores:   host array of 3 device pointers.
 * indices: int64 [L].   offsets: int64 [n_bags+1] or NULL.   alpha: fp32 [L] or NULL.
 * cache:   NULL for no cache.
 * output:  fp32 [n_bags][N], overwritten; the row of an empty bag is zero.
 * L == 0 or n_bags == 0 is valid.
 */
int tt_emb_fwd(const tt_shape_t *shape, const float *const cores[3],
               const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
               const float *alpha, const tt_cache_t *cache,
               float *output, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward pass (Section 3.1, Eq. 4; Section 4.1, Alg. 2): gradients of
 * <output, grad_output> with respect to the cores and, with a cache, the cached
 * rows.  Positions whose row is cached contribute to grad_cache only, the others
 * to the cores only (Section 4.2).
 * grad_output: fp32 [n_bags][N].
 * grad_cores:  host array of 3 device pointers shaped like the cores.  The
 *              gradient is ADDED to them (Alg. 2's "+="); slices that no
 *              position touches are neither read nor written (where several
 *              workgroups share a slice, see tt_emb_workspace_bytes, a zero is
 *              added to them).
 * grad_cache:  fp32 [K][N], added to; required iff cache != NULL.
 * Duplicate indices are combined inside the library; no atomics are used, and the
 * result is bit-identical from run to run.
 */
int tt_emb_bwd(const tt_shape_t *shape, const float *const cores[3],
               const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
               const float *alpha, const tt_cache_t *cache,
               const float *grad_output,
               float *const grad_cores[3], float *grad_cache,
               void *workspace, size_t workspace_bytes, void *stream);

/*
 * Sampled Gaussian initialisation of the cores (Section 3.2, Alg. 3): every entry is
 * drawn from N(0,1), redrawn while it lies within two standard deviations of zero,
 * and scaled by (1 / (3 num_rows r1 r2 v^3))^(1/6), v = E[z^2 | |z| > 2] = 5.75, so
 * that an entry of the reconstructed table has variance 1 / (3 num_rows).  The draws
 * come from a counter-based generator keyed by (seed, core, element, attempt) and are
 * therefore the same on every run and launch shape (its definition is in the
 * library's tt_init.h).  cores: host array of 3 device pointers, overwritten.
 */
int tt_init_sampled_gaussian(const tt_shape_t *shape, float *const cores[3], uint64_t seed, void *stream);

/*
 * Mean pooling (Section 4.1: the rows of a bag are pooled by summation or by
 * averaging).  weights[k] = alpha[k] / (number of positions of the bag of k), alpha
 * == NULL meaning 1: passed as `alpha` to the forward and backward entry points they
 * give the bag average and its gradients.  offsets as above (n_bags + 1 entries,
 * offsets[n_bags] = L); weights: fp32 [L]; an empty bag has no positions to weigh.
 */
int tt_emb_mean_weights(const int64_t *offsets, int64_t n_bags, int64_t L, const float *alpha, float *weights, void *stream);

/*
 * The stored-intermediate variant (Section 4.2, first paragraph: the recomputation
 * in Alg. 2 can be eliminated by storing tensors from the forward pass, at the price
 * of a larger memory footprint).  tt_emb_fwd_keep_t0 is tt_emb_fwd that also writes,
 * for every position k whose row is not cached, the product of its first two core
 * slices, t0[k][(j1*n2 + j2)][b] (fp32, n1*n2*r[2] values per position; t0 has room
 * for L positions; entries of cached positions are not written).  tt_emb_bwd_t0 and
 * tt_emb_bwd_sgd_t0 are tt_emb_bwd and tt_emb_bwd_sgd given that array for the SAME
 * indices: the owners of the third core's slices read it instead of recomputing it
 * (they then read neither G1 nor G2).  Only for the shapes with a specialised kernel
 * (n = (2,2,4) or (4,4,4), equal ranks 8..64): TT_ERR_UNSUPPORTED otherwise.
 */
int tt_emb_fwd_keep_t0(const tt_shape_t *shape, const float *const cores[3],
                       const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                       const float *alpha, const tt_cache_t *cache,
                       float *output, float *t0, void *stream);
int tt_emb_bwd_t0(const tt_shape_t *shape, const float *const cores[3],
                  const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                  const float *alpha, const tt_cache_t *cache,
                  const float *grad_output, const float *t0,
                  float *const grad_cores[3], float *grad_cache,
                  void *workspace, size_t workspace_bytes, void *stream);
int tt_emb_bwd_sgd_t0(const tt_shape_t *shape, const float *const cores[3], float *const cores_out[3],
                      const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                      const float *alpha, const tt_cache_t *cache,
                      const float *grad_output, const float *t0, float lr,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * The stored-intermediate variant with the index work done ahead (Section 4.2, first paragraph;
 * Eq. 4; Alg. 2).  tt_emb_fwd_keep is tt_emb_fwd that also leaves in `kept`, for the backward pass of
 * the SAME batch (same shape, indices, L, offsets, n_bags, cache),
 *   - T0 = G1[i1] G2[i2] of every position whose row is not cached, exactly as tt_emb_fwd_keep_t0
 *     does (it sits at the start of the buffer), and
 *   - for every core slice the list of the positions that touch it, in position order, with the
 *     runs of equal rows marked (integer work on the indices; the encoding is private).
 * With these a slice owner of the backward pass loads its list instead of scanning and decoding the
 * whole index array, and the owners of the third core's slices read T0 instead of recomputing it.
 * tt_emb_bwd_kept and tt_emb_bwd_sgd_kept are tt_emb_bwd and tt_emb_bwd_sgd given that buffer;
 * results agree with theirs to rounding (sums are taken in another fixed order) and are
 * bit-identical from run to run.
 * kept:  device buffer of tt_emb_kept_bytes(shape, L) bytes, 16-byte aligned; written by the
 *        forward call (and by whoever files the lists, see below), read by the backward call,
 *        otherwise the caller's.  It begins with T0, fp32 [L][n1 n2][r[2]] (entries of cached
 *        positions are not written); the rest (the lists) is private.
 * Coverage: the lists exist for n = (2,2,4), equal ranks in {8,16,32}, L <= 8192 and
 * m1 + m2 + m3 <= 1536, without cached positions in the backward; any other call with a
 * specialised kernel keeps and uses T0 alone (exactly tt_emb_fwd_keep_t0 / tt_emb_bwd_t0 /
 * tt_emb_bwd_sgd_t0, workspace rules included); TT_ERR_UNSUPPORTED for shapes without one.
 * tt_emb_kept_bytes returns 0 for such shapes.  workspace: as for tt_emb_bwd / tt_emb_bwd_sgd
 * (none is needed where the lists exist).
 */
size_t tt_emb_kept_bytes(const tt_shape_t *shape, int64_t L);
/* 1 if lists are kept for such a call (see the coverage above), 0 if T0 alone or nothing is. */
int tt_emb_kept_has_lists(const tt_shape_t *shape, int64_t L);
int tt_emb_fwd_keep(const tt_shape_t *shape, const float *const cores[3],
                    const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                    const float *alpha, const tt_cache_t *cache,
                    float *output, void *kept, size_t kept_bytes, int lists_ready, void *stream);

/*
 * The lists depend on the indices (and the cache's row map) alone, so they can be filed before the
 * batch's forward pass: by tt_emb_kept_prepare (a small launch of its own), or by the backward call of
 * the batch BEFORE, whose launch has room for the few workgroups that do it (`next`, below; a loader
 * that is one batch ahead knows the indices).  lists_ready != 0 tells tt_emb_fwd_keep that `kept`
 * already holds the lists of exactly these indices (same L, same cache); it then only adds T0.
 * With lists_ready == 0 the call files them itself, in a second small launch behind the forward's.
 * indices / L / kept / kept_bytes of tt_next_batch_t: as for tt_emb_fwd_keep (host struct; the kept
 * buffer must differ from the current batch's).  Where no lists are kept for the next batch (see the
 * coverage above) nothing is done for it.
 */
typedef struct tt_next_batch_t {
    const int64_t *indices;
    int64_t L;
    void *kept;
    size_t kept_bytes;
} tt_next_batch_t;

int tt_emb_kept_prepare(const tt_shape_t *shape, const int64_t *indices, int64_t L, const tt_cache_t *cache,
                        void *kept, size_t kept_bytes, void *stream);
/* next == NULL: no next batch.  Otherwise its lists are in next->kept when the call's work is done. */
int tt_emb_bwd_kept(const tt_shape_t *shape, const float *const cores[3],
                    const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                    const float *alpha, const tt_cache_t *cache,
                    const float *grad_output, const void *kept, size_t kept_bytes,
                    float *const grad_cores[3], float *grad_cache, const tt_next_batch_t *next,
                    void *workspace, size_t workspace_bytes, void *stream);
int tt_emb_bwd_sgd_kept(const tt_shape_t *shape, const float *const cores[3], float *const cores_out[3],
                        const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                        const float *alpha, const tt_cache_t *cache,
                        const float *grad_output, const void *kept, size_t kept_bytes, float lr,
                        const tt_next_batch_t *next, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward pass and SGD step in one call (Section 3.1, Eq. 4; Alg. 2; Section 5):
 * cores_out = cores - lr * (gradient of <output, grad_output> for this batch), and,
 * with a cache, cache->rows -= lr * (gradient of the cached rows), in place
 * (Section 4.2).  Same result as tt_emb_bwd into zeroed gradients followed by
 * tt_emb_sgd_update, without the gradient buffers and the second pass.
 * cores_out: host array of 3 device pointers shaped like the cores; every element
 *            is written, also in slices that no position touches.  Must not alias
 *            cores (other workgroups still read the old slices); a training loop
 *            swaps the two sets after each step.
 * workspace: tt_emb_bwd_sgd_workspace_bytes(...) bytes (none needed without a cache
 *            below 4,096 positions, for the shapes with a specialised kernel).
 * L == 0 copies the cores.
 */
int tt_emb_bwd_sgd(const tt_shape_t *shape, const float *const cores[3], float *const cores_out[3],
                   const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                   const float *alpha, const tt_cache_t *cache,
                   const float *grad_output, float lr,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * tt_emb_bwd_sgd for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.
 * Same arguments and same result, bit for bit, as tt_emb_bwd_sgd; the scratch memory is an
 * array of tt_emb_static_scratch_bytes() (32 MiB) bytes inside the library's device image, of
 * which every GPU the library runs on holds its own copy until the process ends.  The call
 * allocates and frees nothing.  A call that needs more scratch memory than that (long index
 * lists, large caches: what tt_emb_bwd_sgd_workspace_bytes says, minus its allowance for
 * shapes without a specialised kernel) fails with TT_ERR_WORKSPACE and enqueues nothing.
 * The first call on a device also looks the array's address up (hipGetSymbolAddress): make
 * that call outside a capture.  All calls on one GPU share the array, which keeps what the
 * last call left in it (the kernels initialise what they read): calls that overlap on one GPU,
 * on different streams or from different threads, race and give wrong results.
 */
int tt_emb_bwd_sgd_static(const tt_shape_t *shape, const float *const cores[3], float *const cores_out[3],
                          const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                          const float *alpha, const tt_cache_t *cache,
                          const float *grad_output, float lr, void *stream);
size_t tt_emb_static_scratch_bytes(void);

/*
 * The fused step in two calls.  Part of the backward pass of Alg. 2 depends on the
 * indices and the cache's row map alone: which positions are cached (Section 4.2) and,
 * for long index lists, the grouping of the positions by the core slices they touch.
 * tt_emb_bwd_prepare runs that part into the workspace; tt_emb_bwd_sgd_prepared then
 * does the rest and gives the result of tt_emb_bwd_sgd (t0 == NULL) or
 * tt_emb_bwd_sgd_t0 (t0 != NULL): bit for bit, except where tt_emb_bwd_two_calls_group_earlier
 * says that the pair groups the positions at a length at which the one call does not yet
 * (the pre-pass can be hidden behind other work here, so it pays earlier); the two results
 * then differ in the order of their sums only.  A caller can enqueue the first call on
 * another stream next to the forward pass of the same batch (it reads neither the cores
 * nor the cache rows) and make the second wait for it.
 * Both calls take the same shape, indices, L, offsets, n_bags, cache and workspace;
 * kept_t0 != 0 says that the second call will pass a t0.  The workspace must not be
 * used by anything else between the two calls, and one prepare serves one step.
 * For a short list without a cache the first call has nothing to do and enqueues nothing.
 */
int tt_emb_bwd_prepare(const tt_shape_t *shape, const int64_t *indices, int64_t L,
                       const int64_t *offsets, int64_t n_bags, const tt_cache_t *cache, int kept_t0,
                       void *workspace, size_t workspace_bytes, void *stream);
/* 1 if tt_emb_bwd_prepare enqueues work for such a call (worth a stream of its own), else 0. */
int tt_emb_bwd_has_prepass(const tt_shape_t *shape, int64_t L, int64_t cache_rows, int kept_t0);
/* 1 if the pair tt_emb_bwd_prepare + tt_emb_bwd_sgd_prepared groups the positions of such a call
 * (Alg. 2's "+=" as sums over sorted lists) where the one call does not, else 0. */
int tt_emb_bwd_two_calls_group_earlier(const tt_shape_t *shape, int64_t L, int64_t cache_rows, int kept_t0);

/*
 * The forward pass of a call whose index-only pre-pass has run: tt_emb_fwd / tt_emb_fwd_keep_t0
 * (t0 != NULL) for a caller that has enqueued tt_emb_bwd_prepare with the same shape, indices,
 * offsets, cache and workspace (and kept_t0 = (t0 != NULL)) before it.  Where that pre-pass
 * groups the positions by the slices they touch (long index streams, tt_emb_bwd_has_prepass)
 * and the shape has such a kernel, the forward pass works from the lists: a workgroup takes
 * positions of one slice of the second core, multiplies their stacked first-core rows with
 * the slice on the matrix cores (Eq. 3, first product), and the rows of each bag are pooled
 * afterwards in position order.  Otherwise the call is tt_emb_fwd / tt_emb_fwd_keep_t0.
 * The workspace is read (lists) and written (one row per position, in a part of it that the
 * backward calls do not use); the backward call that follows takes the same workspace.
 * Same results as tt_emb_fwd up to the order of the fp32 sums over the rank indices.
 */
/* 1 if tt_emb_fwd_prepared works from the pre-pass's lists for such a call (then the forward pass has to
 * wait for tt_emb_bwd_prepare), 0 if it is tt_emb_fwd / tt_emb_fwd_keep_t0 and needs no pre-pass. */
int tt_emb_fwd_uses_lists(const tt_shape_t *shape, int64_t L, int64_t cache_rows, int kept_t0);
int tt_emb_fwd_prepared(const tt_shape_t *shape, const float *const cores[3],
                        const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                        const float *alpha, const tt_cache_t *cache,
                        float *output, float *t0, void *workspace, size_t workspace_bytes, void *stream);
int tt_emb_bwd_sgd_prepared(const tt_shape_t *shape, const float *const cores[3], float *const cores_out[3],
                            const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                            const float *alpha, const tt_cache_t *cache,
                            const float *grad_output, const float *t0, float lr,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Always-sufficient workspace size of tt_emb_bwd_sgd; 0 for an invalid shape. */
size_t tt_emb_bwd_sgd_workspace_bytes(const tt_shape_t *shape, int64_t L, int64_t n_bags, int64_t cache_rows);

/*
 * SGD step (Section 5; cached rows per Section 4.2): x <- x - lr * g for every
 * element of the three cores and, if cache != NULL, of cache->rows with
 * grad_cache.  zero_grad != 0 also clears the gradients afterwards.
 */
int tt_emb_sgd_update(const tt_shape_t *shape, float *const cores[3], float *const grad_cores[3],
                      float lr, const tt_cache_t *cache, float *grad_cache, int zero_grad,
                      void *stream);

/*
 * Cache population (Section 4.2): keep the K most frequently used of the
 * candidate rows, fill their lines from the TT cores, and build the row -> slot
 * map.  Order: count descending, ties by ascending row id; slot = rank in that
 * order.
 * cand_rows / cand_counts: int64 [n_cand], distinct rows with 0 <= count < 2^32.
 * out: host struct with K, capacity (>= tt_cache_table_capacity(K), power of two)
 *      and the three device arrays set by the caller; their contents are written.
 * K == 0 is valid and gives an empty cache.
 */
int tt_cache_build(const tt_shape_t *shape, const float *const cores[3],
                   const int64_t *cand_rows, const int64_t *cand_counts, int64_t n_cand,
                   const tt_cache_t *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * One refill of the cache under Section 4.2's semi-dynamic policy; the caller
 * decides how rarely to call it.  The weights of a row that leaves the cache are
 * dropped, not written back into the cores.  The K most used
 * candidates become the cached set, in tt_cache_build's order.  A row that was
 * cached before keeps its line as it is (with the weights it has learned); a row
 * that enters is rebuilt from the cores.
 * cache: a VALID cache (from tt_cache_build or an earlier refill); keys, rows and
 *        table are replaced.  K and capacity do not change.
 * Same candidate arrays and workspace rules as tt_cache_build
 * (tt_cache_refill_workspace_bytes).
 */
int tt_cache_refill(const tt_shape_t *shape, const float *const cores[3],
                    const int64_t *cand_rows, const int64_t *cand_counts, int64_t n_cand,
                    const tt_cache_t *cache, void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of device workspace tt_cache_refill needs. */
size_t tt_cache_refill_workspace_bytes(const tt_shape_t *shape, int64_t n_cand, int64_t K);

/* Access-frequency tracker (Section 4.2).  tt_freq_reset empties the table;
 * tt_freq_update counts every entry of indices[0..L) once (integer atomics: the
 * counts are exact whatever the order); tt_freq_export writes the tracked rows
 * and their counts, in no particular order, to rows / counts (int64, room for
 * `capacity` entries) and their number to *n_out (device) - the candidate arrays
 * of tt_cache_build / tt_cache_refill once the caller has read *n_out.
 * If the table fills up, further new rows are not tracked and stats[1] counts
 * the accesses that were dropped. */
int tt_freq_reset(const tt_freq_t *tracker, void *stream);
int tt_freq_update(const tt_freq_t *tracker, const int64_t *indices, int64_t L, void *stream);
int tt_freq_export(const tt_freq_t *tracker, int64_t *rows, int64_t *counts, int64_t *n_out, void *stream);

/* Cache probe (Section 4.2's split into cached and TT indices):
 * slot[k] = slot of indices[k], or -1 if the row is not cached.  slot: int32 [L]. */
int tt_cache_lookup(const tt_cache_t *cache, const int64_t *indices, int64_t L,
                    int32_t *slot, void *stream);

/* ---- exports used by the parity tests ------------------------------------ */

/*
 * Forward, backward and SGD step for d = 2, 3 or 4 cores (Section 4.1; Eq. 3-6 with the
 * chain of products extended or shortened).  Same conventions as tt_emb_fwd / tt_emb_bwd /
 * tt_emb_sgd_update (CSR bags, optional alpha, "+=" into grad_cores, deterministic),
 * without a cache and without a workspace.  cores / grad_cores: host arrays whose first d
 * entries are device pointers.  Plain kernels, meant for shapes off the tuned three-core
 * path: N, every core slice and every intermediate product of the chain must not exceed
 * 4096 values (TT_ERR_UNSUPPORTED otherwise).
 */
int tt_embd_fwd(const tt_shape_d_t *shape, const float *const cores[4],
                const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                const float *alpha, float *output, void *stream);
int tt_embd_bwd(const tt_shape_d_t *shape, const float *const cores[4],
                const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                const float *alpha, const float *grad_output, float *const grad_cores[4], void *stream);
int tt_embd_sgd_update(const tt_shape_d_t *shape, float *const cores[4], float *const grad_cores[4], float lr,
                       int zero_grad, void *stream);

/*
 * Uncompressed EmbeddingBag on the same GPU, the comparison of the microbenchmarks
 * (Sections 6.6-6.7: the TT kernels against an ordinary EmbeddingBag for pooling
 * factors 1, 10, 100 and for cache hit rates up to 99 %).  Not part of the TT path.
 * table: fp32 [num_rows][N], N a power of two in [4, 256].
 * tt_dense_bag_fwd:      output[b] = sum over the bag of alpha[k] * table[indices[k]].
 * tt_dense_bag_bwd_sgd:  table[indices[k]] -= lr * alpha[k] * grad_output[bag(k)] for
 *                        every position (sparse SGD with floating-point atomics: the
 *                        order in which duplicates are applied is not fixed).
 * tt_dense_bag_bwd_sgd_merged: the same update with duplicates merged first: positions sorted by
 *                        row, each row's gradients added in position order, every distinct row
 *                        written once.  No floating-point atomics, the result is the same in every
 *                        run; workspace of tt_dense_bag_bwd_workspace_bytes(L, N) bytes.  The
 *                        faster of the two stands for the uncompressed table in a comparison.
 */
int tt_dense_bag_fwd(const float *table, int64_t num_rows, int32_t N,
                     const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                     const float *alpha, float *output, void *stream);
int tt_dense_bag_bwd_sgd(float *table, int64_t num_rows, int32_t N,
                         const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                         const float *alpha, const float *grad_output, float lr, void *stream);
size_t tt_dense_bag_bwd_workspace_bytes(int64_t L, int32_t N);
int tt_dense_bag_bwd_sgd_merged(float *table, int64_t num_rows, int32_t N,
                                const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                                const float *alpha, const float *grad_output, float lr,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * The preconditions on the lookup arguments (Section 4.1's interface: row ids of the table, bags
 * in CSR form), checked on the device by a small kernel of its own; no other call checks them,
 * and what a call does with arguments that break them is undefined (it may read or write out of
 * bounds).  Meant for the boundary of a serving or training loop: validate a batch once, read
 * the flag, and only then hand the batch to the other calls.
 * indices, L, offsets, n_bags: as in tt_emb_fwd (offsets == NULL: n_bags == L, nothing to check
 *        on the bags).
 * flag:  int32 [1] on the device.  Written 0 if every precondition holds, else the OR of
 *        TT_BAD_INDEX         an index < 0 or >= num_rows,
 *        TT_BAD_OFFSETS_ORDER offsets[0] != 0 or offsets decreasing somewhere,
 *        TT_BAD_OFFSETS_RANGE an offset outside [0, L], or offsets[n_bags] != L.
 * The return value only covers what the host can see (NULL pointers, negative sizes).
 */
enum { TT_BAD_INDEX = 1, TT_BAD_OFFSETS_ORDER = 2, TT_BAD_OFFSETS_RANGE = 4 };
int tt_emb_validate(const tt_shape_t *shape, const int64_t *indices, int64_t L,
                    const int64_t *offsets, int64_t n_bags, int32_t *flag, void *stream);

/* For measurements: enqueues a kernel of `blocks` workgroups of 256 threads that does nothing
 * (if sink != NULL, device int32 [1], one thread stores 1 there).  Timed in a sequence of such
 * launches it gives the cost of a launch of that size, the floor under every kernel's time. */
int tt_emb_debug_launch_probe(int32_t blocks, int32_t *sink, void *stream);

/* Digits of every index (Section 3.1): i1, i2, i3 are int32 [L]. */
int tt_emb_debug_decode(const tt_shape_t *shape, const int64_t *indices, int64_t L,
                        int32_t *i1, int32_t *i2, int32_t *i3, void *stream);

/*
 * The same digits from the other decoders inside the library, which all must agree with
 * Section 3.1's digit map bit for bit.  mode 0: the integer decode (= tt_emb_debug_decode);
 * mode 1: the multiply-free floating-point decode with which the backward's slice owners find
 * the runs of equal rows;  mode 2: what the owners' selection of their positions decides:
 * i2 and i3 from the digit arithmetic of that test, i1 = the slice whose row range holds the
 * row (-1 if none of the neighbouring slices does, -2 if more than one does).
 */
int tt_emb_debug_decode_as(const tt_shape_t *shape, const int64_t *indices, int64_t L, int mode,
                           int32_t *i1, int32_t *i2, int32_t *i3, void *stream);

/*
 * What the lists that tt_emb_fwd_keep left in `kept` say, for the bit-exact tests of that
 * integer work (Section 3.1's digit map; the grouping that Alg. 2's "+=" implies).  For core
 * r = 0, 1, 2 and position k (arrays int32 [3][L], device):
 *   slice[r][k]: the slice of core r+1 whose list holds k (-1: none, a cached position),
 *   rep[r][k]:   the entry's run marker resolved to a position: the first position with the same
 *                row among the 256 positions [256 g, 256 (g+1)) that hold k,
 *   times[r][k]: in how many lists of core r+1 position k was found (must be 1, or 0 if cached).
 * TT_ERR_UNSUPPORTED where tt_emb_fwd_keep keeps no lists (see its coverage).
 */
int tt_emb_debug_kept_lists(const tt_shape_t *shape, const void *kept, size_t kept_bytes, int64_t L,
                            int32_t *slice, int32_t *rep, int32_t *times, void *stream);

/*
 * Canonical duplicate-free form of a key stream derived from `indices`:
 *   which = 0: the row id itself;  which = 1,2,3: digit i1, i2 or i3.
 * Positions with slot[k] >= 0 are skipped (slot may be NULL: nothing skipped).
 * uniq:  int64 [L]  ascending distinct keys        (first *n_uniq entries valid)
 * count: int32 [L]  occurrences of each            (first *n_uniq entries valid)
 * perm:  int32 [L]  positions grouped by key, ascending inside a group
 *                                                  (first *n_kept entries valid)
 * n_out: int64 [2] on the device: {n_uniq, n_kept}.
 */
int tt_emb_debug_dedup(const tt_shape_t *shape, const int64_t *indices, int64_t L,
                       const int32_t *slot, int which,
                       int64_t *uniq, int32_t *count, int32_t *perm, int64_t *n_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/* Kernel selection for the library calls that the CALLING THREAD makes from now on, meant for
 * tests: the value is per thread, every thread starts at 1, and no other thread's calls are
 * affected.  1: shapes with a specialised kernel use it, and the backward groups long index
 * streams first; with a kept T0 and no cache the grouped backward works on tiles of positions on
 * the matrix cores, else a workgroup per slice works through the slice's list.  0: every call
 * takes the shape-generic kernels.  2: as 1, but the backward always groups first and always
 * takes the list owners.  3: as 2, but the grouped backward with a kept T0 takes the tile kernels,
 * also with a cache.  Returns the thread's old value.  Workspace queries, tt_emb_bwd_prepare
 * and the backward call that follows must be made under the same value. */
int tt_emb_debug_set_fast_path(int mode);

#ifdef __cplusplus
}
#endif
#endif /* TT_EMB_H */
