"""Pins of the CPU oracle against things other than itself (CPU only).

Each oracle function is checked against what the paper and the mathematics
fix: the integers printed in Table 1, closed forms, a dense reconstruction of
the whole Tiny table with a library einsum, library embedding_bag + autograd in
fp64, finite differences (exact for a multilinear function), and brute force.
"""

import os

import numpy as np
import pytest
import torch

from oracle import tt_oracle as ora
from paper_2101_11714_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny():
    wl = W.WORKLOADS["tiny"]
    shape = ora.Shape.of(wl.tables[0])
    cores = W.make_cores(wl.tables[0], wl.init, wl.seed)
    batch = W.make_batch(wl)
    return wl, shape, cores, batch


def dense_table(shape, cores, dtype=np.float64):
    """Eq. 2 evaluated for every row at once by a library einsum (independent of ora.row)."""
    g1 = np.asarray(cores[0], dtype=dtype)[:, 0]          # [m1][n1][R1]
    g2 = np.asarray(cores[1], dtype=dtype)                # [m2][R1][n2][R2]
    g3 = np.asarray(cores[2], dtype=dtype)[..., 0]        # [m3][R2][n3]
    w = np.einsum("xja,yakb,zbl->xyzjkl", g1, g2, g3)
    return w.reshape(shape.m[0] * shape.m[1] * shape.m[2], shape.dim)


def dense_table_torch(cores_t):
    g1, g2, g3 = cores_t
    w = torch.einsum("xja,yakb,zbl->xyzjkl", g1[:, 0], g2, g3[..., 0])
    return w.reshape(g1.shape[0] * g2.shape[0] * g3.shape[0], -1)


# ---------------------------------------------------------------- shape arithmetic

def test_param_count_matches_table1():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table1_param_counts.txt")) if l[0] != "#"]
    assert len(rows) == 7
    for rec in rows:
        nrows, m1, m2, m3 = (int(x) for x in rec[:4])
        assert m1 * m2 * m3 >= nrows
        for col, R in enumerate((16, 32, 64)):
            shape = ora.Shape(nrows, (m1, m2, m3), (2, 2, 4), (1, R, R, 1))
            params = ora.param_count(shape)
            assert params == int(rec[4 + col])
            # the printed ratios are rows*16/params, truncated or rounded to an integer
            assert abs(nrows * 16 / params - int(rec[7 + col])) < 1.0
            assert params == sum(shape.core_size(k) for k in range(3))


def test_param_count_closed_form():
    # 10^7 x 64 as (200,200,250) x (4,4,4): 800 R^2 + 1800 R parameters
    for R in (1, 8, 16, 64):
        shape = ora.Shape(10_000_000, (200, 200, 250), (4, 4, 4), (1, R, R, 1))
        assert ora.param_count(shape) == 800 * R * R + 1800 * R


# ---------------------------------------------------------------- digits

def test_decode_decimal_digits():
    # with m = (10,10,10) the mixed-radix digits are the decimal digits
    shape = ora.Shape(1000, (10, 10, 10), (2, 2, 4), (1, 8, 8, 1))
    idx = np.arange(1000)
    i1, i2, i3 = ora.decode(shape, idx)
    for i in (0, 7, 42, 537, 999):
        s = "%03d" % i
        assert (i1[i], i2[i], i3[i]) == (int(s[0]), int(s[1]), int(s[2]))
    assert np.array_equal(i1 * 100 + i2 * 10 + i3, idx)


@pytest.mark.parametrize("name", ["kaggle_r32", "terabyte_r64"])
def test_decode_large_matches_unravel(name):
    t = W.WORKLOADS[name].tables[0]
    shape = ora.Shape.of(t)
    rng = np.random.default_rng(7)
    m1, m2, m3 = t.m
    edge = np.array([0, 1, m3 - 1, m3, m3 + 1, m2 * m3 - 1, m2 * m3, m2 * m3 + 1,
                     t.num_rows - 1, t.num_rows - m3, ((t.num_rows - 1) // (m2 * m3)) * m2 * m3])
    idx = np.concatenate([edge, rng.integers(0, t.num_rows, 1_000_000)])
    i1, i2, i3 = ora.decode(shape, idx)
    u1, u2, u3 = np.unravel_index(idx, t.m)       # library routine, row-major = i1 most significant
    assert np.array_equal(i1, u1) and np.array_equal(i2, u2) and np.array_equal(i3, u3)
    assert i1.max() < m1 and i2.max() < m2 and i3.max() < m3 and min(i1.min(), i2.min(), i3.min()) >= 0
    assert np.array_equal(i1.astype(np.int64) * m2 * m3 + i2.astype(np.int64) * m3 + i3, idx)


# ---------------------------------------------------------------- one row

def test_row_matches_dense_reconstruction_all_rows():
    _, shape, cores, _ = tiny()
    w = dense_table(shape, cores)
    for i in range(shape.num_rows):
        np.testing.assert_allclose(ora.row(shape, cores, i), w[i], rtol=1e-12, atol=1e-15)


def test_row_unequal_factors_and_ranks():
    # all six factors and both ranks different: catches swapped strides / transposed operands
    shape = ora.Shape(2 * 3 * 5, (2, 3, 5), (3, 2, 5), (1, 4, 7, 1))
    rng = np.random.default_rng(11)
    cores = [rng.standard_normal((shape.m[k], shape.r[k], shape.n[k], shape.r[k + 1])).astype(np.float32)
             for k in range(3)]
    w = dense_table(shape, cores)
    for i in range(shape.num_rows):
        np.testing.assert_allclose(ora.row(shape, cores, i), w[i], rtol=1e-12, atol=1e-14)


def test_row_rank1_is_outer_product():
    shape = ora.Shape(60, (3, 4, 5), (2, 3, 4), (1, 1, 1, 1))
    rng = np.random.default_rng(3)
    cores = [rng.standard_normal((shape.m[k], 1, shape.n[k], 1)).astype(np.float32) for k in range(3)]
    for i in (0, 17, 59):
        i1, i2, i3 = i // 20, (i // 5) % 4, i % 5
        a = cores[0][i1, 0, :, 0].astype(np.float64)
        b = cores[1][i2, 0, :, 0].astype(np.float64)
        c = cores[2][i3, 0, :, 0].astype(np.float64)
        expect = np.einsum("i,j,k->ijk", a, b, c).reshape(-1)
        np.testing.assert_allclose(ora.row(shape, cores, i), expect, rtol=1e-13)


def test_row_identity_middle_core_is_matmul():
    # G2[i2][a][j2][b] = delta_ab  =>  row(j1,j2,j3) = (G1[i1] @ G3[i3])[j1,j3] for every j2
    R = 6
    shape = ora.Shape(4 * 3 * 5, (4, 3, 5), (2, 3, 4), (1, R, R, 1))
    rng = np.random.default_rng(5)
    g1 = rng.standard_normal((4, 1, 2, R)).astype(np.float32)
    g3 = rng.standard_normal((5, R, 4, 1)).astype(np.float32)
    g2 = np.zeros((3, R, 3, R), dtype=np.float32)
    for a in range(R):
        g2[:, a, :, a] = 1.0
    for i in (0, 31, 59):
        i1, i3 = i // 15, i % 5
        prod = g1[i1, 0].astype(np.float64) @ g3[i3, :, :, 0].astype(np.float64)   # (n1 x n3)
        expect = np.repeat(prod[:, None, :], 3, axis=1).reshape(-1)
        np.testing.assert_allclose(ora.row(shape, [g1, g2, g3], i), expect, rtol=1e-13)


# ---------------------------------------------------------------- forward / pooling

def test_fwd_matches_library_embedding_bag():
    _, shape, cores, batch = tiny()
    w = torch.from_numpy(dense_table(shape, cores))
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(batch.indices), w,
                                            torch.from_numpy(batch.offsets[:-1]), mode="sum")
    out = ora.fwd(shape, cores, batch.indices, batch.offsets)
    np.testing.assert_allclose(out, ref.numpy(), rtol=2e-7, atol=1e-9)   # one fp32 rounding


def test_fwd_with_per_sample_weights():
    wl, shape, cores, _ = tiny()
    batch = W.make_batch(wl, with_alpha=True)
    w = torch.from_numpy(dense_table(shape, cores))
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(batch.indices), w,
                                            torch.from_numpy(batch.offsets[:-1]), mode="sum",
                                            per_sample_weights=torch.from_numpy(batch.alpha.astype(np.float64)))
    out = ora.fwd(shape, cores, batch.indices, batch.offsets, alpha=batch.alpha)
    np.testing.assert_allclose(out, ref.numpy(), rtol=2e-7, atol=1e-9)


def test_fwd_special_bags():
    _, shape, cores, _ = tiny()
    w = dense_table(shape, cores)
    # one index per bag: output is the row
    idx = np.array([5, 999, 123])
    out = ora.fwd(shape, cores, idx, np.arange(4))
    np.testing.assert_allclose(out, w[idx].astype(np.float32), rtol=2e-7)
    # the same index c times: c * row;  an empty bag in the middle and at the end: zeros
    idx = np.array([77] * 5 + [3])
    out = ora.fwd(shape, cores, idx, np.array([0, 5, 5, 6, 6]))
    np.testing.assert_allclose(out[0], (5 * w[77]).astype(np.float32), rtol=2e-7)
    assert np.all(out[1] == 0) and np.all(out[3] == 0)
    np.testing.assert_allclose(out[2], w[3].astype(np.float32), rtol=2e-7)


# ---------------------------------------------------------------- backward

def _autograd_reference(shape, cores, batch, alpha=None):
    ct = [torch.tensor(np.asarray(c, dtype=np.float64), requires_grad=True) for c in cores]
    w = dense_table_torch(ct)
    psw = None if alpha is None else torch.from_numpy(alpha.astype(np.float64))
    out = torch.nn.functional.embedding_bag(torch.from_numpy(batch.indices), w,
                                            torch.from_numpy(batch.offsets[:-1]), mode="sum",
                                            per_sample_weights=psw)
    loss = (out * torch.from_numpy(batch.grad_output.astype(np.float64))).sum()
    loss.backward()
    return [c.grad.numpy() for c in ct]


def test_bwd_matches_library_autograd():
    _, shape, cores, batch = tiny()
    ref = _autograd_reference(shape, cores, batch)
    dG, dC = ora.bwd(shape, cores, batch.indices, batch.offsets, batch.grad_output)
    assert dC is None
    for k in range(3):
        np.testing.assert_allclose(dG[k], ref[k], rtol=1e-11, atol=1e-13)


def test_bwd_with_alpha_matches_library_autograd():
    wl, shape, cores, _ = tiny()
    batch = W.make_batch(wl, with_alpha=True)
    ref = _autograd_reference(shape, cores, batch, alpha=batch.alpha)
    dG, _ = ora.bwd(shape, cores, batch.indices, batch.offsets, batch.grad_output, alpha=batch.alpha)
    for k in range(3):
        np.testing.assert_allclose(dG[k], ref[k], rtol=1e-11, atol=1e-13)


def test_bwd_unequal_factors_matches_autograd():
    shape = ora.Shape(2 * 3 * 5, (2, 3, 5), (3, 2, 5), (1, 4, 7, 1))
    rng = np.random.default_rng(13)
    cores = [rng.standard_normal((shape.m[k], shape.r[k], shape.n[k], shape.r[k + 1])).astype(np.float32)
             for k in range(3)]
    idx = rng.integers(0, 30, 40)
    off = np.array([0, 3, 3, 10, 25, 40])
    batch = W.Batch(idx, off, rng.standard_normal((5, shape.dim)).astype(np.float32))
    ref = _autograd_reference(shape, cores, batch)
    dG, _ = ora.bwd(shape, cores, idx, off, batch.grad_output)
    for k in range(3):
        np.testing.assert_allclose(dG[k], ref[k], rtol=1e-11, atol=1e-12)


def test_bwd_finite_differences_every_parameter():
    # L = <output, g> is multilinear in the cores, so a central difference in one core
    # element is exact up to rounding, whatever the step.
    wl, shape, cores, batch = tiny()
    dG, _ = ora.bwd(shape, cores, batch.indices, batch.offsets, batch.grad_output)
    w_of = lambda cs: dense_table(shape, cs)
    g64 = batch.grad_output.astype(np.float64)

    def loss(cs):
        w = w_of(cs)
        out = np.zeros_like(g64)
        bag = np.repeat(np.arange(batch.offsets.size - 1), np.diff(batch.offsets))
        np.add.at(out, bag, w[batch.indices])
        return float((out * g64).sum())

    h = 0.25   # multilinearity makes the step size irrelevant
    worst = 0.0
    c64 = [np.array(c, dtype=np.float64) for c in cores]      # perturb in fp64, not in fp32
    for k in range(3):
        flat = c64[k].reshape(-1)
        for e in range(flat.size):
            keep = flat[e]
            flat[e] = keep + h
            lp = loss(c64)
            flat[e] = keep - h
            lm = loss(c64)
            flat[e] = keep
            fd = (lp - lm) / (2 * h)
            worst = max(worst, abs(fd - dG[k].reshape(-1)[e]))
    scale = max(np.abs(d).max() for d in dG)
    assert worst <= 1e-10 * scale


def test_bwd_duplicates_add_and_empty_bags():
    _, shape, cores, _ = tiny()
    rng = np.random.default_rng(17)
    g = rng.standard_normal((1, shape.dim)).astype(np.float32)
    one, _ = ora.bwd(shape, cores, np.array([321]), np.array([0, 1]), g)
    five, _ = ora.bwd(shape, cores, np.array([321] * 5), np.array([0, 5]), g)
    for k in range(3):
        np.testing.assert_allclose(five[k], 5 * one[k], rtol=1e-13, atol=1e-16)
    # only the three slices picked by the digits (3,2,1) receive gradient
    assert np.count_nonzero(np.abs(one[0]).reshape(10, -1).sum(1)) == 1 and np.abs(one[0][3]).sum() > 0
    assert np.count_nonzero(np.abs(one[1]).reshape(10, -1).sum(1)) == 1 and np.abs(one[1][2]).sum() > 0
    assert np.count_nonzero(np.abs(one[2]).reshape(10, -1).sum(1)) == 1 and np.abs(one[2][1]).sum() > 0
    # empty bags contribute nothing
    g3 = np.concatenate([g, g, g])
    e, _ = ora.bwd(shape, cores, np.array([321]), np.array([0, 0, 1, 1]), g3)
    for k in range(3):
        np.testing.assert_allclose(e[k], one[k], rtol=1e-13, atol=1e-16)


# ---------------------------------------------------------------- SGD

def test_sgd_closed_form_and_effect_on_forward():
    wl, shape, cores, batch = tiny()
    dG, _ = ora.bwd(shape, cores, batch.indices, batch.offsets, batch.grad_output)
    g32 = [d.astype(np.float32) for d in dG]
    new = [ora.sgd(cores[k], g32[k], wl.lr) for k in range(3)]
    for k in range(3):
        expect = (cores[k].astype(np.float64) - wl.lr * g32[k].astype(np.float64)).astype(np.float32)
        assert np.array_equal(new[k], expect)
    out = ora.fwd(shape, new, batch.indices, batch.offsets)
    w = torch.from_numpy(dense_table(shape, new))
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(batch.indices), w,
                                            torch.from_numpy(batch.offsets[:-1]), mode="sum")
    np.testing.assert_allclose(out, ref.numpy(), rtol=2e-7, atol=1e-9)
    # a descent step on L = <output, g> lowers L
    before = float((ora.fwd(shape, cores, batch.indices, batch.offsets).astype(np.float64) * batch.grad_output).sum())
    after = float((out.astype(np.float64) * batch.grad_output).sum())
    assert after < before


# ---------------------------------------------------------------- cache

def test_cache_select_matches_brute_force_with_ties():
    rng = np.random.default_rng(19)
    rows = rng.permutation(5000)[:800].astype(np.int64)
    counts = rng.integers(1, 6, 800).astype(np.int64)          # many ties
    for K in (0, 1, 37, 800):
        keys = ora.cache_select(rows, counts, K)
        order = np.lexsort((rows, -counts))                    # count descending, then row ascending
        assert np.array_equal(keys, rows[order][:K])


def test_cache_lookup_and_cached_forward_equals_uncached():
    wl, shape, cores, batch = tiny()
    rows, counts = np.unique(batch.indices, return_counts=True)
    keys = ora.cache_select(rows, counts, 20)
    slot = ora.cache_lookup(shape, keys, batch.indices)
    pos = {int(r): s for s, r in enumerate(keys)}
    assert np.array_equal(slot, np.array([pos.get(int(i), -1) for i in batch.indices], dtype=np.int32))
    assert (slot >= 0).sum() > 0 and (slot < 0).sum() > 0
    crow = ora.cache_fill(shape, cores, keys)
    np.testing.assert_allclose(crow, dense_table(shape, cores)[keys].astype(np.float32), rtol=2e-7)
    plain = ora.fwd(shape, cores, batch.indices, batch.offsets)
    cached = ora.fwd(shape, cores, batch.indices, batch.offsets, cache_keys=keys, cache_rows=crow)
    np.testing.assert_allclose(cached, plain, rtol=1e-6, atol=1e-8)
    # the cache really is read: changing a cached row changes exactly the bags that hold it
    crow2 = crow.copy()
    crow2[0] += 1.0
    moved = ora.fwd(shape, cores, batch.indices, batch.offsets, cache_keys=keys, cache_rows=crow2)
    bag = np.repeat(np.arange(batch.offsets.size - 1), np.diff(batch.offsets))
    hit = np.zeros(batch.offsets.size - 1, dtype=bool)
    hit[bag[batch.indices == keys[0]]] = True
    assert np.array_equal(np.abs(moved - cached).max(1) > 0.5, hit)


def test_cached_backward_splits_gradients():
    wl, shape, cores, batch = tiny()
    rows, counts = np.unique(batch.indices, return_counts=True)
    keys = ora.cache_select(rows, counts, 20)
    dG, dC = ora.bwd(shape, cores, batch.indices, batch.offsets, batch.grad_output, cache_keys=keys)
    # cores: same as a run in which the cached lookups are removed from the bags
    slot = ora.cache_lookup(shape, keys, batch.indices)
    bag = np.repeat(np.arange(batch.offsets.size - 1), np.diff(batch.offsets))
    keep = slot < 0
    off2 = np.zeros_like(batch.offsets)
    np.cumsum(np.bincount(bag[keep], minlength=batch.offsets.size - 1), out=off2[1:])
    ref, _ = ora.bwd(shape, cores, batch.indices[keep], off2, batch.grad_output)
    for k in range(3):
        np.testing.assert_allclose(dG[k], ref[k], rtol=1e-13, atol=1e-16)
    # cache: sum of the upstream gradients of the bags each cached row occurs in
    expect = np.zeros((20, shape.dim))
    np.add.at(expect, slot[~keep], batch.grad_output[bag[~keep]].astype(np.float64))
    np.testing.assert_allclose(dC, expect, rtol=1e-13, atol=1e-16)


# ---------------------------------------------------------------- dedup

def test_dedup_matches_library_sort():
    rng = np.random.default_rng(23)
    keys = rng.integers(0, 50, 400).astype(np.int64)
    keys[rng.random(400) < 0.2] = -1                          # skipped (cached) positions
    uniq, count, perm = ora.dedup(keys)
    kept = np.flatnonzero(keys >= 0)
    u, c = np.unique(keys[kept], return_counts=True)
    assert np.array_equal(uniq, u) and np.array_equal(count, c)
    assert np.array_equal(perm, kept[np.argsort(keys[kept], kind="stable")])
    e = ora.dedup(np.array([], dtype=np.int64))
    assert e[0].size == 0 and e[1].size == 0 and e[2].size == 0


# ---- frequency tracking and refill (Section 4.2) ------------------------------------------

def test_freq_counts_match_library_unique():
    import collections
    rng = np.random.default_rng(41)
    counts = {}
    streams = [rng.zipf(1.3, 5000) % 977 for _ in range(4)]
    for s in streams:
        ora.freq_update(counts, s)
    rows, cnt = ora.freq_export(counts)
    u, c = np.unique(np.concatenate(streams), return_counts=True)
    assert np.array_equal(rows, u) and np.array_equal(cnt, c)
    brute = collections.Counter(int(x) for s in streams for x in s)
    assert {int(r): int(k) for r, k in zip(rows, cnt)} == dict(brute)


def test_refill_keeps_survivors_and_reinitialises_newcomers():
    wl = W.WORKLOADS["tiny"]
    t = wl.tables[0]
    shape = ora.Shape.of(t)
    cores = W.make_cores(t, wl.init, wl.seed)
    rng = np.random.default_rng(42)
    cand = np.arange(40, dtype=np.int64) * 7 % 1000
    cnt1 = rng.integers(1, 50, cand.size)
    K = 10
    # a first fill from nothing is the plain build
    k1, r1 = ora.cache_refill(shape, cores, np.zeros(0, np.int64), np.zeros((0, t.dim), np.float32), cand, cnt1, K)
    assert np.array_equal(k1, ora.cache_select(cand, cnt1, K))
    assert np.array_equal(r1, ora.cache_fill(shape, cores, k1))
    # the lines learn something; then the popularity shifts
    learned = (r1 + rng.standard_normal(r1.shape)).astype(np.float32)
    cnt2 = cnt1.copy()
    cnt2[rng.permutation(cand.size)[:15]] += 60
    k2, r2 = ora.cache_refill(shape, cores, k1, learned, cand, cnt2, K)
    assert np.array_equal(k2, ora.cache_select(cand, cnt2, K))
    stay = np.intersect1d(k1, k2)
    assert 0 < stay.size < K                                   # the case has survivors and newcomers
    for s, k in enumerate(k2):
        if k in stay:
            assert np.array_equal(r2[s], learned[list(k1).index(k)])          # learned weights kept, bit for bit
        else:
            assert np.array_equal(r2[s], ora.cache_fill(shape, cores, [k])[0])   # from the cores
    # unchanged popularity: nothing moves
    k3, r3 = ora.cache_refill(shape, cores, k2, r2, cand, cnt2, K)
    assert np.array_equal(k3, k2) and np.array_equal(r3, r2)
    # a row that was evicted and comes back has lost what it learned
    gone = np.setdiff1d(k1, k2)
    assert gone.size > 0
    cnt3 = cnt2.copy()
    cnt3[np.isin(cand, gone)] += 1000
    k4, r4 = ora.cache_refill(shape, cores, k2, r2, cand, cnt3, K)
    for s, k in enumerate(k4):
        if k in gone:
            assert np.array_equal(r4[s], ora.cache_fill(shape, cores, [k])[0])


def test_stored_intermediate_times_last_core_is_the_row():
    # unequal factors and ranks, so that a transposed or mis-reshaped T0 fails
    shape = ora.Shape(3 * 4 * 5, (3, 4, 5), (2, 3, 4), (1, 5, 6, 1))
    rng = np.random.default_rng(51)
    cores = [rng.standard_normal((3, 1, 2, 5)).astype(np.float32), rng.standard_normal((4, 5, 3, 6)).astype(np.float32),
             rng.standard_normal((5, 6, 4, 1)).astype(np.float32)]
    for r in (0, 17, 59):
        i1, i2, i3 = (int(x[0]) for x in ora.decode(shape, [r]))
        T0 = ora.t0(shape, cores, r)
        assert T0.shape == (6, 6)
        Cm = cores[2].astype(np.float64).reshape(5, 6, 4)[i3]
        assert np.allclose((T0 @ Cm).reshape(-1), ora.row(shape, cores, r), rtol=1e-13, atol=1e-13)
        # element by element from the definition: T0[(j1,j2), b] = sum_a G1[i1][j1][a] G2[i2][a][j2][b]
        ref = np.einsum("ja,akb->jkb", cores[0].astype(np.float64)[i1, 0], cores[1].astype(np.float64)[i2]).reshape(6, 6)
        assert np.allclose(T0, ref, rtol=1e-13, atol=1e-13)


def test_kept_lists_against_brute_force():
    shape = ora.Shape(1000, (10, 10, 10), (2, 2, 4), (1, 8, 8, 1))
    rng = np.random.default_rng(53)
    idx = rng.integers(0, 40, 700).astype(np.int64) * 25 + 3          # many repeats
    cached = rng.random(700) < 0.2
    sl, rep = ora.kept_lists(shape, idx, cached=cached, chunk=256)
    for k in range(700):
        if cached[k]:
            assert rep[k] == -1 and (sl[:, k] == -1).all()
            continue
        assert sl[0, k] * 100 + sl[1, k] * 10 + sl[2, k] == idx[k]      # decimal digits of the row
        lo = (k // 256) * 256
        same = [q for q in range(lo, k + 1) if idx[q] == idx[k] and not cached[q]]
        assert rep[k] == same[0]
    sl2, rep2 = ora.kept_lists(shape, idx)                               # default chunk for 700 positions: 256; nothing cached
    assert np.array_equal(sl2, np.stack(ora.decode(shape, idx)).astype(np.int32))
    _, first = np.unique(idx[:256], return_index=True)
    assert np.array_equal(np.flatnonzero(rep2[:256] == np.arange(256)), np.sort(first))   # the reps are the first occurrences
    assert np.array_equal(idx[rep2], idx) and np.all(rep2 <= np.arange(700)) and np.all(rep2 // 256 == np.arange(700) // 256)


def test_mean_pooling_matches_library_mean_mode():
    wl, shape, cores, batch = tiny()
    w = torch.from_numpy(dense_table(shape, cores))
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(batch.indices), w,
                                            torch.from_numpy(batch.offsets[:-1]), mode="mean")
    mw = ora.mean_weights(batch.offsets)
    lens = np.diff(batch.offsets)
    assert np.allclose(np.add.reduceat(mw.astype(np.float64), batch.offsets[:-1][lens > 0]), 1.0, atol=1e-6)
    out = ora.fwd(shape, cores, batch.indices, batch.offsets, alpha=mw)
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-6, atol=1e-8)   # the weights are rounded to fp32
    # gradients of the mean through library autograd
    ct = [torch.tensor(np.asarray(c, dtype=np.float64), requires_grad=True) for c in cores]
    o = torch.nn.functional.embedding_bag(torch.from_numpy(batch.indices), dense_table_torch(ct),
                                          torch.from_numpy(batch.offsets[:-1]), mode="mean")
    (o * torch.from_numpy(batch.grad_output.astype(np.float64))).sum().backward()
    g, _ = ora.bwd(shape, cores, batch.indices, batch.offsets, batch.grad_output, alpha=mw)
    for k in range(3):
        np.testing.assert_allclose(g[k], ct[k].grad.numpy(), rtol=1e-5, atol=1e-8)
    # with per-position weights on top, and an empty bag
    off = np.array([0, 3, 3, 4], dtype=np.int64)
    al = np.array([2.0, 4.0, 6.0, 8.0], dtype=np.float32)
    assert np.allclose(ora.mean_weights(off, al), [2 / 3, 4 / 3, 2.0, 8.0])


# ---- sampled Gaussian initialisation (Section 3.2, Alg. 3) ---------------------------------

def test_sampled_gaussian_draws_are_the_tail_of_a_standard_normal():
    import math
    n = 20000
    z, att = zip(*(ora.sampled_gaussian_draw(2024, 1, e) for e in range(n)))
    z, att = np.array(z), np.array(att)
    assert np.all(np.abs(z) > 2.0)                                  # nothing within two sigma of zero
    p_tail = math.erfc(2.0 / math.sqrt(2.0))                        # P(|z| > 2) = 0.0455
    assert abs(att.mean() - 1.0 / p_tail) < 0.05 / p_tail           # geometric number of attempts: the draws are N(0,1)
    assert abs((z > 0).mean() - 0.5) < 0.015                        # symmetric
    v = 1.0 + 2.0 * math.exp(-2.0) / math.sqrt(2.0 * math.pi) / (0.5 * p_tail)
    assert abs((z * z).mean() - v) < 0.03 * v                       # E[z^2 | |z| > 2] = 5.75 (closed form)
    # tail shape: P(|z| > 2.5 | |z| > 2) from the normal distribution
    assert abs((np.abs(z) > 2.5).mean() - math.erfc(2.5 / math.sqrt(2.0)) / p_tail) < 0.015
    # different cores, elements and seeds give different streams; the same arguments the same value
    assert ora.sampled_gaussian_draw(2024, 1, 5) == ora.sampled_gaussian_draw(2024, 1, 5)
    assert len({ora.sampled_gaussian_draw(s, c, e)[0] for s in (1, 2) for c in (0, 1, 2) for e in (0, 1)}) == 12


def test_sampled_gaussian_cores_give_the_target_variance():
    # Section 3.2: the product of the cores should approximate N(0, 1/(3 n)), n = number of rows
    shape = ora.Shape(20 * 20 * 25, (20, 20, 25), (2, 2, 4), (1, 8, 8, 1))
    cores = ora.init_sampled_gaussian(shape, 7)
    scale = ora.sampled_gaussian_scale(shape)
    assert np.all(np.abs(cores[1]) > 2.0 * scale * (1 - 1e-6))
    g = [c.reshape(shape.m[k], shape.r[k], shape.n[k], shape.r[k + 1]).astype(np.float64) for k, c in enumerate(cores)]
    rng = np.random.default_rng(3)
    rows = rng.integers(0, shape.num_rows, 4000)
    i1, i2, i3 = rows // 500, (rows // 25) % 20, rows % 25
    w = np.einsum("kja,kaxb,kby->kjxy", g[0][i1, 0], g[1][i2], g[2][i3, :, :, 0]).reshape(rows.size, -1)
    target = 1.0 / (3.0 * shape.num_rows)
    assert abs(w.var() / target - 1.0) < 0.1
    assert abs(w.mean()) < 0.05 * np.sqrt(target)


# ---- general number of cores ----------------------------------------------------------------

def _random_shape_d(d, rng):
    m = [int(x) for x in rng.integers(2, 5, d)]
    n = [int(x) for x in rng.integers(1, 4, d)]
    r = [1] + [int(x) for x in rng.integers(2, 5, d - 1)] + [1]
    cores = [rng.standard_normal((m[k], r[k], n[k], r[k + 1])).astype(np.float32) for k in range(d)]
    return m, n, r, cores


def _dense_d(m, n, r, cores):
    """The whole table from Eq. 2, one einsum over all cores (independent of row_d)."""
    d = len(m)
    g = [c.astype(np.float64) for c in cores]                       # written out per d to keep it readable
    if d == 2:
        w = np.einsum("pxiy,qyjz->pqij", g[0], g[1])
    elif d == 3:
        w = np.einsum("pxiy,qyjz,rzkw->pqrijk", g[0], g[1], g[2])
    else:
        w = np.einsum("pxiy,qyjz,rzkw,swlv->pqrsijkl", g[0], g[1], g[2], g[3])
    return w.reshape(int(np.prod(m)), int(np.prod(n)))


@pytest.mark.parametrize("d", [2, 3, 4])
def test_general_d_rows_and_gradients(d):
    rng = np.random.default_rng(80 + d)
    m, n, r, cores = _random_shape_d(d, rng)
    rows, N = int(np.prod(m)), int(np.prod(n))
    w = _dense_d(m, n, r, cores)
    for i in (0, rows // 2, rows - 1):
        np.testing.assert_allclose(ora.row_d(m, n, r, cores, i), w[i], rtol=1e-12, atol=1e-12)
    lens = np.array([2, 0, 3, 1])
    off = np.zeros(5, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    idx = rng.integers(0, rows, int(off[-1]))
    idx[1] = idx[0]                                                 # a repeated row
    alpha = (0.5 + rng.random(idx.size)).astype(np.float32)
    go = rng.standard_normal((4, N)).astype(np.float32)
    wt = torch.from_numpy(w)
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(idx), wt, torch.from_numpy(off[:-1]), mode="sum",
                                            per_sample_weights=torch.from_numpy(alpha.astype(np.float64)))
    np.testing.assert_allclose(ora.fwd_d(m, n, r, cores, idx, off, alpha), ref.numpy(), rtol=1e-6, atol=1e-7)
    # gradients through library autograd on the dense reconstruction
    ct = [torch.tensor(c.astype(np.float64), requires_grad=True) for c in cores]
    if d == 2:
        wd = torch.einsum("pxiy,qyjz->pqij", ct[0], ct[1])
    elif d == 3:
        wd = torch.einsum("pxiy,qyjz,rzkw->pqrijk", ct[0], ct[1], ct[2])
    else:
        wd = torch.einsum("pxiy,qyjz,rzkw,swlv->pqrsijkl", ct[0], ct[1], ct[2], ct[3])
    o = torch.nn.functional.embedding_bag(torch.from_numpy(idx), wd.reshape(rows, N), torch.from_numpy(off[:-1]), mode="sum",
                                          per_sample_weights=torch.from_numpy(alpha.astype(np.float64)))
    (o * torch.from_numpy(go.astype(np.float64))).sum().backward()
    g = ora.bwd_d(m, n, r, cores, idx, off, go, alpha)
    for k in range(d):
        np.testing.assert_allclose(g[k], ct[k].grad.numpy(), rtol=1e-5, atol=1e-6)


def test_general_d_with_three_cores_is_the_three_core_oracle():
    wl, shape, cores, batch = tiny()
    m, n, r = list(shape.m), list(shape.n), list(shape.r)
    np.testing.assert_allclose(ora.fwd_d(m, n, r, cores, batch.indices, batch.offsets),
                               ora.fwd(shape, cores, batch.indices, batch.offsets), rtol=1e-6, atol=1e-8)
    g3, _ = ora.bwd(shape, cores, batch.indices, batch.offsets, batch.grad_output)
    gd = ora.bwd_d(m, n, r, cores, batch.indices, batch.offsets, batch.grad_output)
    for k in range(3):
        np.testing.assert_allclose(gd[k].reshape(-1), np.asarray(g3[k]).reshape(-1), rtol=1e-5, atol=1e-7)


def test_threaded_forward_is_the_forward_bit_for_bit():
    """ora.fwd_threads only shares the bags out: ragged weighted bags with a cache, several thread counts."""
    rng = np.random.default_rng(77)
    shape = ora.Shape(4 * 5 * 6, (4, 5, 6), (2, 2, 4), (1, 3, 5, 1))
    cores = [rng.standard_normal(shape.core_size(k)).astype(np.float32) for k in range(3)]
    lens = rng.integers(0, 9, 57)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = rng.integers(0, shape.num_rows, off[-1]).astype(np.int64)
    alpha = rng.standard_normal(off[-1]).astype(np.float32)
    keys = np.array([3, 17, 99], dtype=np.int64)
    crow = rng.standard_normal((3, shape.dim)).astype(np.float32)
    ref = ora.fwd(shape, cores, idx, off, alpha=alpha, cache_keys=keys, cache_rows=crow)
    for threads in (1, 2, 3, 8):
        out, ran = ora.fwd_threads(shape, cores, idx, off, threads, alpha=alpha, cache_keys=keys, cache_rows=crow)
        assert 1 <= ran <= threads
        assert np.array_equal(out.view(np.uint32), ref.view(np.uint32))
