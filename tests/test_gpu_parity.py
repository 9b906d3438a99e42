"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle on the
same seeded inputs.  Integer work (digits, dedup, cache selection and probe) must be
bit-exact; floating point must meet max |gpu - ref| / max |ref| <= 1e-4 per tensor."""

import numpy as np
import pytest
import torch

from oracle import tt_oracle as ora
from paper_2101_11714_amd import binding as B
from paper_2101_11714_amd import workloads as W
from gpu_util import DeviceTable, assert_close, dev, sample_bags

pytestmark = pytest.mark.gpu

SINGLE = ["tiny", "kaggle_r32", "sweep_r8", "sweep_r16", "sweep_r32", "sweep_r64", "terabyte_r64"]


@pytest.fixture(params=[1, 0, 2], ids=["fast", "generic", "grouped"])
def path(request):
    old = B.set_fast_path(request.param)
    yield request.param
    B.set_fast_path(old)


# ------------------------------------------------------------------ integer work

@pytest.mark.parametrize("name", SINGLE + ["multihot_cache"])
def test_decode_bit_exact(name):
    wl = W.WORKLOADS[name]
    for table in (0, len(wl.tables) - 1):
        t = wl.tables[table]
        batch = W.make_batch(wl, table)
        m1, m2, m3 = t.m
        edge = np.array([0, 1, m3 - 1, m3, m2 * m3 - 1, m2 * m3, t.num_rows - 1, t.num_rows - m3], dtype=np.int64)
        edge = edge[(edge >= 0) & (edge < t.num_rows)]
        idx = np.concatenate([edge, batch.indices])
        got = B.tt_emb_debug_decode(B.shape_of(t), torch.from_numpy(idx).to(dev()))
        ref = ora.decode(ora.Shape.of(t), idx)
        for k in range(3):
            assert np.array_equal(got[k].cpu().numpy(), ref[k])


def test_decode_awkward_factors():
    # divisors 1, 2, powers of two, primes, and a large last factor
    for m in [(1, 1, 7), (3, 1, 5), (2, 2, 2), (7, 1, 1), (13, 17, 19), (64, 128, 256), (5, 100003, 3), (2, 3, 300000007)]:
        rows = min(m[0] * m[1] * m[2], 2 ** 31 - 1)
        shape = B.make_shape(rows, m, (2, 2, 4), (1, 8, 8, 1))
        rng = np.random.default_rng(1)
        idx = np.unique(np.concatenate([rng.integers(0, rows, 20000), [0, rows - 1]]))
        got = B.tt_emb_debug_decode(shape, torch.from_numpy(idx).to(dev()))
        ref = ora.decode(ora.Shape(rows, m, (2, 2, 4), (1, 8, 8, 1)), idx)
        for k in range(3):
            assert np.array_equal(got[k].cpu().numpy(), ref[k]), m


def _edge_rows(t):
    """Rows at which a digit changes: multiples of m3 and of m2 m3 and their neighbours, the ends of the table."""
    m1, m2, m3 = t.m
    rng = np.random.default_rng(11)
    k3 = rng.integers(0, max(1, t.num_rows // m3), 4096, dtype=np.int64) * m3
    k23 = np.arange(0, m1 + 1, dtype=np.int64) * (m2 * m3)
    e = np.concatenate([[0, 1, t.num_rows - 1, t.num_rows - 2], k3 - 1, k3, k3 + 1, k23 - 1, k23, k23 + 1])
    return np.unique(e[(e >= 0) & (e < t.num_rows)])


@pytest.mark.parametrize("mode", [1, 2], ids=["run_detection_decode", "owner_selection"])
@pytest.mark.parametrize("name", SINGLE + ["multihot_cache"])
def test_backward_decoders_bit_exact(name, mode):
    """The floating-point digit arithmetic that the backward's slice owners run (decode_f64 for the runs
    of equal rows, select_digit_f64 / the row range of i1 for the selection) against the oracle's digits:
    every table of every workload, 10^6 random rows, the rows where a digit changes, and the batch."""
    wl = W.WORKLOADS[name]
    for table, t in enumerate(wl.tables):
        rng = np.random.default_rng(100 + table)
        idx = np.concatenate([_edge_rows(t), rng.integers(0, t.num_rows, 1_000_000, dtype=np.int64),
                              W.make_batch(wl, table).indices])
        got = B.tt_emb_debug_decode_as(B.shape_of(t), torch.from_numpy(idx).to(dev()), mode)
        ref = ora.decode(ora.Shape.of(t), idx)
        for k in range(3):
            assert np.array_equal(got[k].cpu().numpy(), ref[k]), (name, table, k)


@pytest.mark.parametrize("mode", [1, 2], ids=["run_detection_decode", "owner_selection"])
def test_backward_decoders_awkward_factors(mode):
    # divisors 1, 2, powers of two, primes, a large last factor, and tables that reach the 2^31 row limit
    for m in [(1, 1, 7), (3, 1, 5), (2, 2, 2), (7, 1, 1), (13, 17, 19), (64, 128, 256), (5, 100003, 3), (2, 3, 300000007),
              (1290, 1291, 1289), (46340, 46340, 1), (1, 2, 2 ** 30), (2 ** 15, 2 ** 15, 2), (3, 715827882, 1)]:
        rows = min(m[0] * m[1] * m[2], 2 ** 31 - 1)
        t = W.TableShape(rows, m, (2, 2, 4), (1, 8, 8, 1))
        rng = np.random.default_rng(1)
        idx = np.unique(np.concatenate([rng.integers(0, rows, 200000), rng.integers(max(0, rows - 5000), rows, 5000),
                                        _edge_rows(t)]))
        got = B.tt_emb_debug_decode_as(B.shape_of(t), torch.from_numpy(idx).to(dev()), mode)
        ref = ora.decode(ora.Shape(rows, m, (2, 2, 4), (1, 8, 8, 1)), idx)
        for k in range(3):
            assert np.array_equal(got[k].cpu().numpy(), ref[k]), (m, k)


@pytest.mark.parametrize("name", ["tiny", "kaggle_r32", "terabyte_r64", "multihot_cache"])
@pytest.mark.parametrize("which", [0, 1, 2, 3])
def test_dedup_bit_exact(name, which):
    wl = W.WORKLOADS[name]
    t = wl.tables[0]
    batch = W.make_batch(wl)
    idx = batch.indices
    digits = ora.decode(ora.Shape.of(t), idx)
    keys = idx.copy() if which == 0 else digits[which - 1].astype(np.int64)
    # skip a pseudo-random 30 % of the positions, as cached lookups would be
    slot = np.where(np.random.default_rng(3).random(idx.size) < 0.3, 5, -1).astype(np.int32)
    for use_slot in (False, True):
        k = keys.copy()
        if use_slot:
            k[slot >= 0] = -1
        ru, rc, rp = ora.dedup(k)
        gu, gc, gp = B.tt_emb_debug_dedup(B.shape_of(t), torch.from_numpy(idx).to(dev()), which,
                                          torch.from_numpy(slot).to(dev()) if use_slot else None)
        assert np.array_equal(gu.cpu().numpy(), ru)
        assert np.array_equal(gc.cpu().numpy(), rc)
        assert np.array_equal(gp.cpu().numpy(), rp)


def test_dedup_all_equal_and_empty():
    t = W.WORKLOADS["tiny"].tables[0]
    idx = np.full(5000, 321, dtype=np.int64)
    gu, gc, gp = B.tt_emb_debug_dedup(B.shape_of(t), torch.from_numpy(idx).to(dev()), 0)
    assert gu.cpu().tolist() == [321] and gc.cpu().tolist() == [5000]
    assert np.array_equal(gp.cpu().numpy(), np.arange(5000))
    gu, gc, gp = B.tt_emb_debug_dedup(B.shape_of(t), torch.zeros(0, dtype=torch.int64, device=dev()), 0)
    assert gu.numel() == 0 and gc.numel() == 0 and gp.numel() == 0


@pytest.mark.parametrize("L", [2048 * 512, 2048 * 512 + 1, 1_300_003])
def test_dedup_long_lists_both_forms_of_the_sort(L):
    """Up to 512 tiles of 2048 keys the scatter kernel of the sort derives its own offsets; beyond, a scan kernel does."""
    t = W.WORKLOADS["terabyte_r64"].tables[0]
    rng = np.random.default_rng(L)
    idx = rng.integers(0, t.num_rows, L, dtype=np.int64)
    idx[rng.random(L) < 0.3] = 12345                                                      # one very long run
    idx[: L // 4] = idx[L // 2: L // 2 + L // 4]                                          # many pairs
    ru, rc, rp = ora.dedup(idx)
    gu, gc, gp = B.tt_emb_debug_dedup(B.shape_of(t), torch.from_numpy(idx).to(dev()), 0)
    assert np.array_equal(gu.cpu().numpy(), ru)
    assert np.array_equal(gc.cpu().numpy(), rc)
    assert np.array_equal(gp.cpu().numpy(), rp)


# ------------------------------------------------------------------ forward

@pytest.mark.parametrize("name", SINGLE)
def test_forward_matches_oracle(name, path):
    d = DeviceTable(W.WORKLOADS[name])
    out = d.fwd()
    ref = ora.fwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, alpha=d.batch.alpha)     # every bag
    assert_close(out, ref, name + " forward")
    if d.L == d.n_bags:                                   # one index per bag: offsets may be omitted
        assert np.array_equal(d.fwd(use_offsets=False), out)


def test_forward_ragged_weighted_and_empty_bags(path):
    wl = W.WORKLOADS["tiny"]
    t = wl.tables[0]
    rng = np.random.default_rng(5)
    lens = np.array([0, 3, 0, 0, 1, 70, 2, 0, 300, 1, 0], dtype=np.int64)
    off = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    idx = rng.integers(0, t.num_rows, int(off[-1]))
    idx[10:60] = 77                                        # a long run of one row
    batch = W.Batch(idx, off, rng.standard_normal((lens.size, t.dim)).astype(np.float32),
                    (0.5 + rng.random(idx.size)).astype(np.float32))
    d = DeviceTable(wl, batch=batch)
    out = d.fwd()
    ref = ora.fwd(d.oshape, d.cores, idx, off, alpha=batch.alpha)
    assert_close(out, ref, "ragged forward")
    assert np.all(out[lens == 0] == 0)


# ------------------------------------------------------------------ backward + SGD

@pytest.mark.parametrize("name", SINGLE)
def test_backward_and_sgd_match_oracle(name, path):
    wl = W.WORKLOADS[name]
    d = DeviceTable(wl)
    ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output)
    dg, _ = d.bwd()
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), ref[k], "%s dG%d" % (name, k + 1))
    # run-to-run determinism, bit for bit
    dg2, _ = d.bwd()
    for k in range(3):
        assert torch.equal(dg[k], dg2[k])
    # "+=": a second call on top of the first doubles the gradient
    d.bwd(grad_cores=dg2)
    for k in range(3):
        assert_close(dg2[k].cpu().numpy(), 2 * ref[k], "%s accumulate dG%d" % (name, k + 1))
    # SGD on the cores, then clear the gradients
    new_ref = [ora.sgd(d.cores[k], dg[k].cpu().numpy(), wl.lr) for k in range(3)]
    B.tt_emb_sgd_update(d.shape, d.g, dg, wl.lr, zero_grad=True)
    torch.cuda.synchronize()
    for k in range(3):
        assert_close(d.g[k].cpu().numpy(), new_ref[k], "%s sgd core %d" % (name, k + 1))
        assert float(dg[k].abs().max()) == 0.0


def test_backward_leaves_untouched_slices_alone(path):
    wl = W.WORKLOADS["tiny"]
    t = wl.tables[0]
    rng = np.random.default_rng(9)
    idx = np.array([123, 123, 456, 123], dtype=np.int64)      # digits (1,2,3) and (4,5,6)
    off = np.array([0, 2, 2, 4], dtype=np.int64)
    batch = W.Batch(idx, off, rng.standard_normal((3, t.dim)).astype(np.float32))
    d = DeviceTable(wl, batch=batch)
    marker = 7.25
    grads = [torch.full_like(x, marker) for x in d.g]
    d.bwd(grad_cores=grads)
    ref, _ = ora.bwd(d.oshape, d.cores, idx, off, batch.grad_output)
    touched = [{1, 4}, {2, 5}, {3, 6}]
    for k in range(3):
        got = grads[k].cpu().numpy()
        for s in range(10):
            if s in touched[k]:
                assert_close(got[s] - marker, ref[k][s], "touched slice")
            else:
                assert np.all(got[s] == marker)


def test_backward_ragged_weighted(path):
    wl = W.WORKLOADS["tiny"]
    t = wl.tables[0]
    rng = np.random.default_rng(15)
    lens = np.array([0, 3, 0, 1, 700, 2, 0, 1500, 1, 0], dtype=np.int64)   # > one selection round
    off = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    idx = rng.integers(0, t.num_rows, int(off[-1]))
    idx[100:400] = 77
    batch = W.Batch(idx, off, rng.standard_normal((lens.size, t.dim)).astype(np.float32),
                    (0.5 + rng.random(idx.size)).astype(np.float32))
    d = DeviceTable(wl, batch=batch)
    dg, _ = d.bwd()
    ref, _ = ora.bwd(d.oshape, d.cores, idx, off, batch.grad_output, alpha=batch.alpha)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), ref[k], "ragged dG%d" % (k + 1))


def test_adversarial_identity_rank_map(path):
    # all hot rows share i1 and i2: one slice owner gets almost every lookup
    import dataclasses
    wl = dataclasses.replace(W.WORKLOADS["kaggle_r32"], identity_rank_map=True, n_bags=1024)
    d = DeviceTable(wl)
    out = d.fwd()
    assert_close(out, ora.fwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets), "identity map forward")
    dg, _ = d.bwd()
    ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), ref[k], "identity map dG%d" % (k + 1))


def test_other_shapes_take_the_generic_kernels():
    # unequal factors and ranks (no specialised kernel exists for them)
    shape = W.TableShape(2 * 3 * 5 * 7, (6, 5, 7), (3, 2, 5), (1, 4, 7, 1))
    wl = W.Workload("odd", (shape,), 50, (0, 6), "uniform", 0.0, "normal0.1", 21)
    d = DeviceTable(wl, with_alpha=True)
    assert_close(d.fwd(), ora.fwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, alpha=d.batch.alpha), "odd fwd")
    dg, _ = d.bwd()
    ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, alpha=d.batch.alpha)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), ref[k], "odd dG%d" % (k + 1))


# ------------------------------------------------------------------ fused backward + SGD

@pytest.mark.parametrize("name", SINGLE)
def test_fused_backward_sgd_matches_oracle(name, path):
    wl = W.WORKLOADS[name]
    d = DeviceTable(wl)
    before = [x.clone() for x in d.g]
    new = d.bwd_sgd(wl.lr)
    ref_g, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), ora.sgd(d.cores[k], ref_g[k], wl.lr), "%s fused core %d" % (name, k + 1))
        assert torch.equal(d.g[k], before[k])                      # the input cores are not written
    # same bits as the two separate calls, and from run to run
    dg, _ = d.bwd()
    B.tt_emb_sgd_update(d.shape, d.g, dg, wl.lr)
    torch.cuda.synchronize()
    again = DeviceTable(wl).bwd_sgd(wl.lr)
    for k in range(3):
        assert torch.equal(new[k], d.g[k])
        assert torch.equal(new[k], again[k])


def test_fused_ragged_weighted_and_empty(path):
    wl = W.WORKLOADS["tiny"]
    t = wl.tables[0]
    rng = np.random.default_rng(16)
    lens = np.array([0, 3, 0, 1, 700, 2, 0, 1500, 1, 0], dtype=np.int64)
    off = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    idx = rng.integers(0, t.num_rows, int(off[-1]))
    idx[100:400] = 77
    batch = W.Batch(idx, off, rng.standard_normal((lens.size, t.dim)).astype(np.float32),
                    (0.5 + rng.random(idx.size)).astype(np.float32))
    d = DeviceTable(wl, batch=batch)
    new = d.bwd_sgd(0.05)
    ref, _ = ora.bwd(d.oshape, d.cores, idx, off, batch.grad_output, alpha=batch.alpha)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), ora.sgd(d.cores[k], ref[k], 0.05), "fused ragged core %d" % (k + 1))
    # no lookups at all: the step copies the cores
    empty = W.Batch(np.zeros(0, np.int64), np.zeros(4, np.int64), rng.standard_normal((3, t.dim)).astype(np.float32))
    d0 = DeviceTable(wl, batch=empty)
    new0 = d0.bwd_sgd(0.05)
    for k in range(3):
        assert torch.equal(new0[k], d0.g[k])


def test_fused_other_shapes():
    shape = W.TableShape(2 * 3 * 5 * 7, (6, 5, 7), (3, 2, 5), (1, 4, 7, 1))
    wl = W.Workload("odd", (shape,), 50, (0, 6), "uniform", 0.0, "normal0.1", 21)
    d = DeviceTable(wl, with_alpha=True)
    new = d.bwd_sgd(0.1)
    ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, alpha=d.batch.alpha)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), ora.sgd(d.cores[k], ref[k], 0.1), "fused odd core %d" % (k + 1))


def test_prepared_call_alone_where_the_library_reports_no_prepass():
    """A shape without a specialised kernel, no cache: tt_emb_bwd_has_prepass says 0, so a caller may skip
    tt_emb_bwd_prepare; tt_emb_bwd_sgd_prepared then clears its own gradient buffers (the workspace starts dirty)."""
    shape = W.TableShape(2 * 3 * 5 * 7, (6, 5, 7), (3, 2, 5), (1, 4, 7, 1))
    wl = W.Workload("odd", (shape,), 50, (0, 6), "uniform", 0.0, "normal0.1", 22)
    d = DeviceTable(wl, with_alpha=True)
    assert not B.bwd_has_prepass(d.shape, d.L, 0, False)
    out = [torch.full_like(x, float("nan")) for x in d.g]
    ws = torch.full((B.bwd_sgd_workspace_bytes(d.shape, d.L, d.n_bags, 0),), 0x7F, dtype=torch.uint8, device=dev())
    for _ in range(2):                                  # the second call finds the first call's gradients there
        B.tt_emb_bwd_sgd(d.shape, d.g, out, d.idx, d.off, d.n_bags, d.go, 0.1, alpha=d.alpha, workspace=ws, prepared=True)
    torch.cuda.synchronize()
    ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, alpha=d.batch.alpha)
    for k in range(3):
        assert_close(out[k].cpu().numpy(), ora.sgd(d.cores[k], ref[k], 0.1), "prepared-only odd core %d" % (k + 1))


def test_output_arrays_beyond_32_bit_offsets_are_refused():
    """n_bags * N >= 2^31: the call fails before anything is enqueued (no array of that size is needed to see it)."""
    wl = W.WORKLOADS["tiny"]
    d = DeviceTable(wl)
    import ctypes as C
    n_bags = (1 << 31) // d.t.dim
    out = torch.empty(16, dtype=torch.float32, device=dev())
    rc = B.lib().tt_emb_fwd(C.byref(d.shape), B._ptr_array(d.g), B._ptr(d.idx), d.idx.numel(), None, n_bags, None, None,
                            B._ptr(out), None, 0, None)
    assert rc == -6, B.lib().tt_last_error()            # TT_ERR_UNSUPPORTED
    assert b"n_bags * N" in B.lib().tt_last_error()


@pytest.mark.parametrize("name,table", [("tiny", 0), ("multihot_cache", 0), ("multihot_cache", 6)])
def test_fused_with_cache(name, table, path):
    wl = W.WORKLOADS[name]
    d = DeviceTable(wl, table=table)
    if name == "tiny":
        rows, counts = np.unique(d.batch.indices, return_counts=True)
        rows, counts, K = rows.astype(np.int64), counts.astype(np.int64), 20
        cache, _, _ = d.build_cache(K, rows, counts)
    else:
        K = W.cache_size(wl, table)
        cache, rows, counts = d.build_cache(K)
    keys = ora.cache_select(rows, counts, K)
    crow = (ora.cache_fill(d.oshape, d.cores, keys) * 1.5).astype(np.float32)
    cache.rows.copy_(torch.from_numpy(crow))
    new = d.bwd_sgd(wl.lr, cache=cache)
    rg, rc = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, cache_keys=keys)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), ora.sgd(d.cores[k], rg[k], wl.lr), "%s fused core %d" % (name, k + 1))
    assert_close(cache.rows.cpu().numpy()[:K], ora.sgd(crow, rc, wl.lr), "%s fused cache lines" % name)


@pytest.mark.parametrize("name,table,with_cache", [("tiny", 0, True), ("kaggle_r32", 0, False), ("kaggle_r32", 0, True),
                                                   ("terabyte_r64", 0, False), ("multihot_cache", 0, True),
                                                   ("multihot_cache", 6, False)])
@pytest.mark.parametrize("kept_t0", [False, True])
def test_fused_step_in_two_calls_is_the_same_bit_for_bit(name, table, with_cache, kept_t0, path):
    """tt_emb_bwd_prepare on another stream + tt_emb_bwd_sgd_prepared against the one call (itself checked against the
    oracle above): short lists with and without a cache, grouped lists with and without one."""
    if kept_t0 and path != 1:
        pytest.skip("a kept T0 always takes the specialised kernels: one run is enough")
    wl = W.WORKLOADS[name]
    d = DeviceTable(wl, table=table)
    cache = None
    if with_cache:
        if name == "multihot_cache":
            cache, _, _ = d.build_cache(W.cache_size(wl, table))
        else:
            rows, counts = np.unique(d.batch.indices, return_counts=True)
            cache, _, _ = d.build_cache(20 if name == "tiny" else 300, rows.astype(np.int64), counts.astype(np.int64))
    t0 = d.fwd_keep_t0(cache)[1] if kept_t0 else None
    lines = cache.rows.clone() if cache is not None else None
    one = d.bwd_sgd(wl.lr, cache=cache, t0=t0)
    if cache is not None:
        lines_one = cache.rows.clone()
        cache.rows.copy_(lines)
    two = d.bwd_sgd(wl.lr, cache=cache, t0=t0, two_calls=True)
    if B.bwd_two_calls_group_earlier(d.shape, d.L, 0 if cache is None else cache.K, kept_t0):
        # the pair groups the positions where the one call does not yet: the same sums in another order
        ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output)
        for k in range(3):
            assert_close(two[k].cpu().numpy(), ora.sgd(d.cores[k], ref[k], wl.lr), "%s core %d in two calls" % (name, k + 1))
        return
    for k in range(3):
        assert torch.equal(one[k], two[k]), "core %d" % (k + 1)
    if cache is not None:
        assert torch.equal(lines_one, cache.rows), "cache lines"


# ------------------------------------------------------------------ cache

def test_cache_on_tiny(path):
    wl = W.WORKLOADS["tiny"]
    d = DeviceTable(wl)
    rows, counts = np.unique(d.batch.indices, return_counts=True)
    p = np.random.default_rng(2).permutation(rows.size)
    rows, counts = rows[p].astype(np.int64), counts[p].astype(np.int64)
    K = 20
    cache, _, _ = d.build_cache(K, rows, counts)
    keys = ora.cache_select(rows, counts, K)
    assert np.array_equal(cache.keys.cpu().numpy(), keys)
    assert_close(cache.rows.cpu().numpy(), ora.cache_fill(d.oshape, d.cores, keys), "cache lines")
    slot = torch.empty(d.L, dtype=torch.int32, device=dev())
    B.tt_cache_lookup(cache, d.idx, slot)
    assert np.array_equal(slot.cpu().numpy(), ora.cache_lookup(d.oshape, keys, d.batch.indices))
    # right after the build the cached forward equals the uncached one
    assert_close(d.fwd(cache=cache), d.fwd(), "cached vs uncached forward")
    # lines that differ from the cores are really used
    crow = cache.rows.cpu().numpy().copy()
    crow += np.random.default_rng(4).standard_normal(crow.shape).astype(np.float32)
    cache.rows.copy_(torch.from_numpy(crow))
    ref = ora.fwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, cache_keys=keys, cache_rows=crow)
    assert_close(d.fwd(cache=cache), ref, "cached forward")
    dg, dc = d.bwd(cache=cache)
    rg, rc = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, cache_keys=keys)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), rg[k], "cached dG%d" % (k + 1))
    assert_close(dc.cpu().numpy()[:K], rc, "dCache")
    new_rows = ora.sgd(crow, dc.cpu().numpy()[:K], wl.lr)
    B.tt_emb_sgd_update(d.shape, d.g, dg, wl.lr, cache=cache, grad_cache=dc, zero_grad=True)
    torch.cuda.synchronize()
    assert_close(cache.rows.cpu().numpy(), new_rows, "sgd on cache lines")
    assert float(dc.abs().max()) == 0.0


# every table with the specialised kernels; the shape-generic and the always-grouped path on the smallest and the largest
@pytest.mark.parametrize("table,mode", [(tb, 1) for tb in range(7)] + [(0, 0), (6, 0), (0, 2), (6, 2)])
def test_multihot_with_cache(table, mode):
    old_mode = B.set_fast_path(mode)
    try:
        _multihot_with_cache(table)
    finally:
        B.set_fast_path(old_mode)


def _multihot_with_cache(table):
    wl = W.WORKLOADS["multihot_cache"]
    d = DeviceTable(wl, table=table)
    K = W.cache_size(wl, table)
    cache, rows, counts = d.build_cache(K)
    keys = ora.cache_select(rows, counts, K)
    assert np.array_equal(cache.keys.cpu().numpy(), keys)
    crow = ora.cache_fill(d.oshape, d.cores, keys)
    assert_close(cache.rows.cpu().numpy(), crow, "cache lines")
    slot = torch.empty(d.L, dtype=torch.int32, device=dev())
    B.tt_cache_lookup(cache, d.idx, slot)
    ref_slot = ora.cache_lookup(d.oshape, keys, d.batch.indices)
    assert np.array_equal(slot.cpu().numpy(), ref_slot)
    hit = float((ref_slot >= 0).mean())
    assert 0.3 < hit < 0.99, hit
    # perturb the lines so that cached and rebuilt rows differ, then compare a sample of bags
    crow = (crow * 1.5).astype(np.float32)
    cache.rows.copy_(torch.from_numpy(crow))
    out = d.fwd(cache=cache)
    ref = ora.fwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, cache_keys=keys, cache_rows=crow)   # every bag
    assert_close(out, ref, "multihot forward")
    dg, dc = d.bwd(cache=cache)
    rg, rc = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, cache_keys=keys)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), rg[k], "multihot dG%d" % (k + 1))
    assert_close(dc.cpu().numpy()[:K], rc, "multihot dCache")


def test_cache_selection_with_many_ties():
    t = W.WORKLOADS["kaggle_r32"].tables[0]
    rng = np.random.default_rng(33)
    rows = rng.choice(t.num_rows, 50_000, replace=False).astype(np.int64)
    counts = rng.integers(1, 4, rows.size).astype(np.int64)
    counts[:10] = 2 ** 31 + 5                                    # large counts sort first
    K = 1014
    d = DeviceTable(W.WORKLOADS["kaggle_r32"])
    cache, _, _ = d.build_cache(K, rows, counts)
    assert np.array_equal(cache.keys.cpu().numpy(), ora.cache_select(rows, counts, K))


# ------------------------------------------------------------------ frequency tracker and refill

@pytest.mark.parametrize("name", ["kaggle_r32", "multihot_cache"])
def test_freq_tracker_counts_exactly(name):
    wl = W.WORKLOADS[name]
    freq = B.Freq(1 << 19, dev())
    B.tt_freq_reset(freq)
    ref = {}
    for step in range(3):
        b = W.make_batch(wl, 0, step)
        B.tt_freq_update(freq, torch.from_numpy(b.indices).to(dev()))
        ora.freq_update(ref, b.indices)
    rows = torch.empty(freq.capacity, dtype=torch.int64, device=dev())
    counts = torch.empty_like(rows)
    n_out = torch.zeros(1, dtype=torch.int64, device=dev())
    B.tt_freq_export(freq, rows, counts, n_out)
    torch.cuda.synchronize()
    n = int(n_out.item())
    r, c = rows[:n].cpu().numpy(), counts[:n].cpu().numpy()
    order = np.argsort(r)
    ref_rows, ref_counts = ora.freq_export(ref)
    assert np.array_equal(r[order], ref_rows) and np.array_equal(c[order], ref_counts)
    stats = freq.stats.cpu().numpy()
    assert stats[0] == n and stats[1] == 0
    # a reset empties it
    B.tt_freq_reset(freq)
    B.tt_freq_export(freq, rows, counts, n_out)
    torch.cuda.synchronize()
    assert int(n_out.item()) == 0 and int(freq.stats.sum().item()) == 0


def test_freq_tracker_full_table_drops_and_says_so():
    freq = B.Freq(64, dev())
    B.tt_freq_reset(freq)
    rng = np.random.default_rng(5)
    idx = rng.integers(0, 300, 5000).astype(np.int64)
    B.tt_freq_update(freq, torch.from_numpy(idx).to(dev()))
    rows = torch.empty(64, dtype=torch.int64, device=dev())
    counts = torch.empty_like(rows)
    n_out = torch.zeros(1, dtype=torch.int64, device=dev())
    B.tt_freq_export(freq, rows, counts, n_out)
    torch.cuda.synchronize()
    n = int(n_out.item())
    stats = freq.stats.cpu().numpy()
    assert n == 64 and stats[0] == 64 and stats[1] > 0
    r, c = rows[:n].cpu().numpy(), counts[:n].cpu().numpy()
    assert np.unique(r).size == 64
    true = dict(zip(*np.unique(idx, return_counts=True)))
    assert all(1 <= c[i] <= true[r[i]] for i in range(n))         # a tracked row never counts too much
    assert int(c.sum()) + int(stats[1]) == idx.size                # every access is counted or reported dropped


@pytest.mark.parametrize("name", ["tiny", "multihot_cache"])
def test_cache_refill_matches_oracle(name, path):
    wl = W.WORKLOADS[name]
    d = DeviceTable(wl)
    rng = np.random.default_rng(8)
    if name == "tiny":
        cand = (np.arange(40, dtype=np.int64) * 7) % 1000
        cnt1 = rng.integers(1, 50, cand.size).astype(np.int64)
        cnt2 = cnt1.copy()
        cnt2[rng.permutation(cand.size)[:15]] += 60
        K = 10
    else:
        # counts of the warm-up stream, then of a later stream tracked on the device
        cand, cnt1 = W.warmup_counts(wl, 0)
        K = W.cache_size(wl, 0)
        freq = B.Freq(1 << 19, dev())
        B.tt_freq_reset(freq)
        for step in range(2):
            B.tt_freq_update(freq, torch.from_numpy(W.make_batch(wl, 0, step).indices).to(dev()))
        rows = torch.empty(freq.capacity, dtype=torch.int64, device=dev())
        counts = torch.empty_like(rows)
        n_out = torch.zeros(1, dtype=torch.int64, device=dev())
        B.tt_freq_export(freq, rows, counts, n_out)
        torch.cuda.synchronize()
        n = int(n_out.item())
        cand2, cnt2 = rows[:n].cpu().numpy(), counts[:n].cpu().numpy()
    cache, _, _ = d.build_cache(K, cand, cnt1)
    k1 = ora.cache_select(cand, cnt1, K)
    learned = (ora.cache_fill(d.oshape, d.cores, k1) * 1.25 + 0.5).astype(np.float32)
    cache.rows.copy_(torch.from_numpy(learned))
    if name == "tiny":
        cand2 = cand
    B.tt_cache_refill(d.shape, d.g, torch.from_numpy(cand2).to(dev()), torch.from_numpy(cnt2).to(dev()), cache)
    torch.cuda.synchronize()
    k2, r2 = ora.cache_refill(d.oshape, d.cores, k1, learned, cand2, cnt2, K)
    assert np.array_equal(cache.keys.cpu().numpy(), k2)
    got = cache.rows.cpu().numpy()[:K]
    stay = np.isin(k2, k1)
    assert 0 < stay.sum() < K                                       # survivors and newcomers both occur
    assert np.array_equal(got[stay], r2[stay])                      # learned lines are kept bit for bit
    assert_close(got[~stay], r2[~stay], "%s lines of the rows that enter" % name)
    slot = torch.empty(d.L, dtype=torch.int32, device=dev())
    B.tt_cache_lookup(cache, d.idx, slot)
    assert np.array_equal(slot.cpu().numpy(), ora.cache_lookup(d.oshape, k2, d.batch.indices))
    # the refilled cache serves the forward pass
    pick, idx, off, _ = sample_bags(d.batch, 64)
    out = d.fwd(cache=cache)
    assert_close(out[pick], ora.fwd(d.oshape, d.cores, idx, off, cache_keys=k2, cache_rows=got), "%s forward after refill" % name)


# ------------------------------------------------------------------ stored intermediate (T0)

@pytest.mark.parametrize("name", SINGLE)
def test_forward_keeps_t0(name):
    wl = W.WORKLOADS[name]
    d = DeviceTable(wl)
    out, t0 = d.fwd_keep_t0()
    assert np.array_equal(out, d.fwd())                             # the output is the plain forward's, bit for bit
    got = t0.cpu().numpy()
    pick = np.random.default_rng(3).choice(d.L, min(d.L, 48), replace=False)
    ref = np.stack([ora.t0(d.oshape, d.cores, int(d.batch.indices[k])).reshape(-1) for k in pick])
    assert_close(got[pick], ref, "%s T0" % name)


@pytest.mark.parametrize("name", SINGLE)
def test_backward_with_kept_t0(name, path):
    wl = W.WORKLOADS[name]
    d = DeviceTable(wl)
    _, t0 = d.fwd_keep_t0()
    ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output)
    dg, _ = d.bwd(t0=t0)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), ref[k], "%s dG%d with kept T0" % (name, k + 1))
    new = d.bwd_sgd(wl.lr, t0=t0)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), ora.sgd(d.cores[k], ref[k], wl.lr), "%s fused core %d with kept T0" % (name, k + 1))
    # where both calls run the slice owners, only the third core's owners use T0: the other two gradients are the
    # recomputing kernel's, bit for bit (a kept T0 always takes the specialised kernel, so the comparison needs it on
    # the other side too; where the call with T0 groups the positions and works on tiles, the sums have another order)
    same_kernels = B.bwd_has_prepass(d.shape, d.L, 0, kept_t0=True) == B.bwd_has_prepass(d.shape, d.L, 0, kept_t0=False)
    if path != 0 and same_kernels:
        plain, _ = d.bwd()
        assert torch.equal(dg[0], plain[0]) and torch.equal(dg[1], plain[1])


def test_kept_t0_ragged_weighted_with_cache(path):
    wl = W.WORKLOADS["tiny"]
    t = wl.tables[0]
    rng = np.random.default_rng(17)
    lens = np.array([0, 3, 0, 1, 700, 2, 0, 1500, 1, 0], dtype=np.int64)
    off = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    idx = rng.integers(0, t.num_rows, int(off[-1]))
    idx[100:400] = 77
    batch = W.Batch(idx, off, rng.standard_normal((lens.size, t.dim)).astype(np.float32),
                    (0.5 + rng.random(idx.size)).astype(np.float32))
    d = DeviceTable(wl, batch=batch)
    rows, counts = np.unique(idx, return_counts=True)
    K = 25
    cache, _, _ = d.build_cache(K, rows.astype(np.int64), counts.astype(np.int64))
    keys = ora.cache_select(rows, counts, K)
    out, t0 = d.fwd_keep_t0(cache=cache)
    if path != 0:                                                   # keeping T0 always takes the specialised kernel
        assert np.array_equal(out, d.fwd(cache=cache))
    assert_close(out, ora.fwd(d.oshape, d.cores, idx, off, alpha=batch.alpha, cache_keys=keys,
                              cache_rows=cache.rows.cpu().numpy()[:K]), "kept T0 + cache forward")
    got = t0.cpu().numpy()
    cached = ora.cache_lookup(d.oshape, keys, idx) >= 0
    assert np.isnan(got[cached]).all() and not np.isnan(got[~cached]).any()     # cached positions keep no T0
    dg, dc = d.bwd(cache=cache, t0=t0)
    rg, rc = ora.bwd(d.oshape, d.cores, idx, off, batch.grad_output, alpha=batch.alpha, cache_keys=keys)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), rg[k], "kept T0 + cache dG%d" % (k + 1))
    assert_close(dc.cpu().numpy()[:K], rc, "kept T0 + cache dCache")


@pytest.mark.parametrize("R", [32, 64])
def test_forward_long_bags_take_a_workgroup_each(R, path):
    """Bags of about 100 positions (the forward then gives every bag a whole workgroup), ragged, weighted, with a
    cache and with empty bags, on a (4,4,4) shape; the kept T0 must match as well."""
    import dataclasses
    t = W.TableShape(12 * 11 * 13, (12, 11, 13), (4, 4, 4), (1, R, R, 1))
    wl = dataclasses.replace(W.WORKLOADS["tiny"], tables=(t,), name="small444")
    rng = np.random.default_rng(60 + R)
    lens = rng.integers(60, 140, 40).astype(np.int64)
    lens[[3, 17]] = 0
    lens[5] = 1
    off = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    L = int(off[-1])
    idx = rng.integers(0, t.num_rows, L)
    idx[rng.random(L) < 0.3] = 17                                   # one hot row
    batch = W.Batch(idx, off, rng.standard_normal((lens.size, t.dim)).astype(np.float32),
                    (0.5 + rng.random(L)).astype(np.float32))
    d = DeviceTable(wl, batch=batch)
    rows, counts = np.unique(idx, return_counts=True)
    K = 25
    cache, _, _ = d.build_cache(K, rows.astype(np.int64), counts.astype(np.int64))
    keys = ora.cache_select(rows, counts, K)
    crows = cache.rows.cpu().numpy()[:K]
    ref = ora.fwd(d.oshape, d.cores, idx, off, alpha=batch.alpha, cache_keys=keys, cache_rows=crows)
    assert_close(d.fwd(cache=cache), ref, "long bags forward")
    out, t0 = d.fwd_keep_t0(cache=cache)
    assert_close(out, ref, "long bags forward keeping T0")
    got = t0.cpu().numpy()
    cached = ora.cache_lookup(d.oshape, keys, idx) >= 0
    assert np.isnan(got[cached]).all() and not np.isnan(got[~cached]).any()
    pick = np.random.default_rng(3).choice(np.flatnonzero(~cached), 48, replace=False)
    want = np.stack([ora.t0(d.oshape, d.cores, int(idx[k])).reshape(-1) for k in pick])
    assert_close(got[pick], want, "kept T0 of long bags")
    assert_close(d.fwd(), ora.fwd(d.oshape, d.cores, idx, off, alpha=batch.alpha), "long bags forward, no cache")


@pytest.mark.parametrize("with_cache", [False, True])
def test_forward_short_bags_large_second_core(with_cache):
    """Many short bags (0 to 3 positions, fewer than 2 on average) on a table whose second core is larger than one
    XCD's L2: the forward assigns the bags to the workgroups by the second digit of their first row.  A hot row
    fills its bucket and spills over; ragged, weighted, with empty bags, a tail segment, with and without a cache."""
    import dataclasses
    t = W.TableShape(16 * 50 * 16, (16, 50, 16), (4, 4, 4), (1, 64, 64, 1))
    wl = dataclasses.replace(W.WORKLOADS["tiny"], tables=(t,), name="shortbags")
    rng = np.random.default_rng(5)
    n_bags = 4096 + 19
    lens = rng.choice([0, 1, 1, 1, 1, 2, 3], n_bags).astype(np.int64)
    off = np.zeros(n_bags + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    L = int(off[-1])
    assert n_bags <= L < 2 * n_bags
    idx = rng.integers(0, t.num_rows, L)
    idx[rng.random(L) < 0.15] = 4321                                # a hot row
    batch = W.Batch(idx, off, rng.standard_normal((n_bags, t.dim)).astype(np.float32), (0.5 + rng.random(L)).astype(np.float32))
    d = DeviceTable(wl, batch=batch)
    cache, keys, crows = None, None, None
    if with_cache:
        rows, counts = np.unique(idx, return_counts=True)
        cache, _, _ = d.build_cache(30, rows.astype(np.int64), counts.astype(np.int64))
        keys = ora.cache_select(rows, counts, 30)
        crows = (cache.rows.cpu().numpy()[:30] * 1.25).astype(np.float32)
        cache.rows[:30].copy_(torch.from_numpy(crows))
    ref = ora.fwd(d.oshape, d.cores, idx, off, alpha=batch.alpha, cache_keys=keys, cache_rows=crows)
    assert_close(d.fwd(cache=cache), ref, "forward")
    out, t0 = d.fwd_keep_t0(cache=cache)
    assert_close(out, ref, "forward keeping T0")
    rg, rc = ora.bwd(d.oshape, d.cores, idx, off, batch.grad_output, alpha=batch.alpha, cache_keys=keys)
    new = d.bwd_sgd(0.01, cache=cache, t0=t0)                     # the kept T0 is the right one, position by position
    for k in range(3):
        assert_close((d.cores[k].astype(np.float64) - new[k].cpu().numpy()) / 0.01, rg[k], "gradient of core %d from the kept T0" % (k + 1))


@pytest.mark.parametrize("R,n_bags", [(32, 1500), (64, 1500), (32, 6000)])
@pytest.mark.parametrize("with_cache", [False, True])
def test_444_shapes_shared_slices_and_matrix_cores(R, n_bags, with_cache, path):
    """The (4,4,4) shapes from 4096 positions on: several workgroups share a slice (partial sums in the
    workspace), the G2 owners work on the matrix cores and, with the grouping pre-pass, also produce the G1
    gradients; with a cache its reduction rides along.  Ragged weighted bags, a hot row, a list length that
    is no multiple of anything; gradients are added to non-zero buffers."""
    import dataclasses
    t = W.TableShape(12 * 11 * 13, (12, 11, 13), (4, 4, 4), (1, R, R, 1))
    wl = dataclasses.replace(W.WORKLOADS["tiny"], tables=(t,), name="small444")
    rng = np.random.default_rng(40 + R)
    lens = rng.integers(0, 9, n_bags).astype(np.int64)           # 6000 bags: lists of > 512 entries per workgroup
    lens[7] = 431                                                   # one long bag
    off = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    L = int(off[-1])
    assert L >= 4096 + 17
    idx = rng.integers(0, t.num_rows, L)
    idx[rng.random(L) < 0.1] = 1234                                 # a hot row all over the stream
    idx[2000:2300] = 99                                             # and a run of equal rows
    batch = W.Batch(idx, off, rng.standard_normal((lens.size, t.dim)).astype(np.float32),
                    (0.5 + rng.random(L)).astype(np.float32))
    d = DeviceTable(wl, batch=batch)
    cache, keys, K = None, None, 0
    if with_cache:
        rows, counts = np.unique(idx, return_counts=True)
        K = 40
        cache, _, _ = d.build_cache(K, rows.astype(np.int64), counts.astype(np.int64))
        keys = ora.cache_select(rows, counts, K)
    crows = cache.rows.cpu().numpy()[:K].copy() if with_cache else None
    out, t0 = d.fwd_keep_t0(cache=cache)
    assert_close(out, ora.fwd(d.oshape, d.cores, idx, off, alpha=batch.alpha, cache_keys=keys, cache_rows=crows), "forward")
    rg, rc = ora.bwd(d.oshape, d.cores, idx, off, batch.grad_output, alpha=batch.alpha, cache_keys=keys)
    # separate backward, added to what the buffers hold
    for use_t0 in (False, True):
        start = [torch.full_like(x, 0.25) for x in d.g]
        gc0 = torch.full_like(cache.rows, -0.5) if with_cache else None
        dg, dc = d.bwd(cache=cache, grad_cores=start, grad_cache=gc0, t0=t0 if use_t0 else None)
        for k in range(3):
            assert_close(dg[k].cpu().numpy() - 0.25, rg[k], "dG%d (t0 %s)" % (k + 1, use_t0))
        if with_cache:
            assert_close(dc.cpu().numpy()[:K] + 0.5, rc, "dCache (t0 %s)" % use_t0)
    # fused step
    lr = 0.05
    new = d.bwd_sgd(lr, cache=cache, t0=t0)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), d.cores[k].astype(np.float64) - lr * rg[k], "fused core %d" % (k + 1))
    if with_cache:
        assert_close(cache.rows.cpu().numpy()[:K], crows.astype(np.float64) - lr * rc, "fused cache lines")


@pytest.mark.parametrize("n,R,n_bags", [((2, 2, 4), 8, 3000), ((4, 4, 4), 32, 500)])
@pytest.mark.parametrize("with_cache", [False, True])
def test_very_long_lists(n, R, n_bags, with_cache):
    """Bags of 120 positions on a small table, so that every row occurs many times and every owner walks its list in
    many pieces of 512 entries.  360,000 positions of the (2,2,4) shape: 3 L items are more than 512 tiles of the
    grouping sort (its scan-kernel form) and eight workgroups share a slice; 60,000 of the (4,4,4) shape (the
    oracle takes seconds per pass there)."""
    import dataclasses
    t = W.TableShape(12 * 11 * 13, (12, 11, 13), n, (1, R, R, 1))
    wl = dataclasses.replace(W.WORKLOADS["tiny"], tables=(t,), name="long")
    rng = np.random.default_rng(77 + R)
    lens = np.full(n_bags, 120, dtype=np.int64)
    lens[5] = 7
    lens[6] = 233
    off = np.zeros(n_bags + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    L = int(off[-1])
    assert n_bags < 3000 or 3 * L > 2048 * 512
    idx = rng.integers(0, t.num_rows, L)
    idx[rng.random(L) < 0.05] = 777
    batch = W.Batch(idx, off, rng.standard_normal((n_bags, t.dim)).astype(np.float32), (0.5 + rng.random(L)).astype(np.float32))
    d = DeviceTable(wl, batch=batch)
    cache, keys, K = None, None, 0
    if with_cache:
        rows, counts = np.unique(idx, return_counts=True)
        K = 50
        cache, _, _ = d.build_cache(K, rows.astype(np.int64), counts.astype(np.int64))
        keys = ora.cache_select(rows, counts, K)
    crows = cache.rows.cpu().numpy()[:K].copy() if with_cache else None
    out, t0 = d.fwd_keep_t0(cache=cache)
    assert_close(out, ora.fwd(d.oshape, d.cores, idx, off, alpha=batch.alpha, cache_keys=keys, cache_rows=crows), "forward")
    rg, rc = ora.bwd(d.oshape, d.cores, idx, off, batch.grad_output, alpha=batch.alpha, cache_keys=keys)
    lr = 1e-3
    new = d.bwd_sgd(lr, cache=cache, t0=t0, two_calls=True)
    for k in range(3):
        assert_close((d.cores[k].astype(np.float64) - new[k].cpu().numpy()) / lr, rg[k], "gradient of core %d" % (k + 1))
    if with_cache:
        assert_close((crows.astype(np.float64) - cache.rows.cpu().numpy()[:K]) / lr, rc, "gradient of the cache lines")
    dg, dc = d.bwd(cache=cache)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), rg[k], "dG%d" % (k + 1))
    if with_cache:
        assert_close(dc.cpu().numpy()[:K], rc, "dCache")


# ------------------------------------------------------------------ the uncompressed comparison kernels

@pytest.mark.parametrize("N,lens", [(16, (1, 1)), (16, (0, 7)), (64, (0, 30)), (256, (1, 3))])
def test_dense_embedding_bag_matches_its_definition(N, lens):
    rng = np.random.default_rng(61)
    rows, n_bags = 5000, 300
    table = rng.standard_normal((rows, N)).astype(np.float32)
    bl = rng.integers(lens[0], lens[1] + 1, n_bags)
    off = np.zeros(n_bags + 1, dtype=np.int64)
    np.cumsum(bl, out=off[1:])
    L = int(off[-1])
    idx = rng.integers(0, rows, L).astype(np.int64)
    idx[: L // 3] = 17                                             # a hot row
    alpha = (0.5 + rng.random(L)).astype(np.float32)
    go = rng.standard_normal((n_bags, N)).astype(np.float32)
    bag = np.repeat(np.arange(n_bags), bl)
    ref_out = np.zeros((n_bags, N))
    np.add.at(ref_out, bag, alpha[:, None].astype(np.float64) * table[idx])
    d = dev()
    tb = torch.from_numpy(table).to(d)
    out = torch.full((n_bags, N), float("nan"), dtype=torch.float32, device=d)
    B.tt_dense_bag_fwd(tb, torch.from_numpy(idx).to(d), torch.from_numpy(off).to(d), n_bags, out, alpha=torch.from_numpy(alpha).to(d))
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy(), ref_out, "dense forward")
    lr = 0.05
    ref_tab = table.astype(np.float64)
    np.add.at(ref_tab, idx, -lr * alpha[:, None].astype(np.float64) * go[bag])
    B.tt_dense_bag_bwd_sgd(tb, torch.from_numpy(idx).to(d), torch.from_numpy(off).to(d), n_bags, torch.from_numpy(go).to(d), lr,
                           alpha=torch.from_numpy(alpha).to(d))
    torch.cuda.synchronize()
    assert_close(tb.cpu().numpy(), ref_tab, "dense sparse SGD")
    # the same update with duplicates merged first: same definition, and the same bits in every run
    results = []
    for _ in range(2):
        tm = torch.from_numpy(table).to(d)
        B.tt_dense_bag_bwd_sgd_merged(tm, torch.from_numpy(idx).to(d), torch.from_numpy(off).to(d), n_bags,
                                      torch.from_numpy(go).to(d), lr, alpha=torch.from_numpy(alpha).to(d))
        torch.cuda.synchronize()
        results.append(tm)
    assert_close(results[0].cpu().numpy(), ref_tab, "dense merged SGD")
    assert torch.equal(results[0], results[1])


@pytest.mark.parametrize("N", [16, 64])
def test_dense_merged_update_runs_over_many_tiles(N):
    """Runs of equal rows of every kind for the tiled sum: one row that fills dozens of tiles, runs that begin or end
    on a tile border, a run over exactly one tile, single positions, one index per bag without an offsets array."""
    rng = np.random.default_rng(62)
    rows = 100000
    pieces = [np.full(64 * 70 + 5, 99999), np.full(64, 5), np.full(59, 7), np.full(128, 8), np.full(1, 9),
              rng.integers(10, 5000, 3000), np.full(64 * 65, 6000), rng.integers(7000, rows - 1, 777)]
    idx = np.concatenate(pieces).astype(np.int64)
    rng.shuffle(idx)
    L = idx.size
    table = rng.standard_normal((rows, N)).astype(np.float32)
    go = rng.standard_normal((L, N)).astype(np.float32)
    lr = 0.01
    ref = table.astype(np.float64)
    np.add.at(ref, idx, -lr * go.astype(np.float64))
    d = dev()
    tm = torch.from_numpy(table).to(d)
    B.tt_dense_bag_bwd_sgd_merged(tm, torch.from_numpy(idx).to(d), None, L, torch.from_numpy(go).to(d), lr)
    torch.cuda.synchronize()
    got = tm.cpu().numpy()
    touched = np.unique(idx)
    assert_close(got[touched], ref[touched], "dense merged SGD, long runs")
    untouched = np.setdiff1d(np.arange(rows), touched)
    assert np.array_equal(got[untouched], table[untouched])


# ------------------------------------------------------------------ mean pooling

def test_mean_pooling_weights_and_passes(path):
    wl = W.WORKLOADS["tiny"]
    t = wl.tables[0]
    rng = np.random.default_rng(71)
    lens = np.array([0, 3, 0, 1, 130, 2, 0, 65, 1, 0], dtype=np.int64)
    off = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    idx = rng.integers(0, t.num_rows, int(off[-1]))
    alpha = (0.5 + rng.random(idx.size)).astype(np.float32)
    batch = W.Batch(idx, off, rng.standard_normal((lens.size, t.dim)).astype(np.float32), None)
    d = DeviceTable(wl, batch=batch)
    for al in (None, alpha):
        w = torch.full((d.L,), float("nan"), dtype=torch.float32, device=dev())
        B.tt_emb_mean_weights(d.off, d.n_bags, d.L, w, alpha=None if al is None else torch.from_numpy(al).to(dev()))
        torch.cuda.synchronize()
        ref_w = ora.mean_weights(off, al)
        np.testing.assert_allclose(w.cpu().numpy(), ref_w, rtol=2e-7)      # one division, one rounding
        d.alpha = w
        assert_close(d.fwd(), ora.fwd(d.oshape, d.cores, idx, off, alpha=ref_w), "mean forward")
        dg, _ = d.bwd()
        rg, _ = ora.bwd(d.oshape, d.cores, idx, off, batch.grad_output, alpha=ref_w)
        for k in range(3):
            assert_close(dg[k].cpu().numpy(), rg[k], "mean dG%d" % (k + 1))


# ------------------------------------------------------------------ sampled Gaussian initialisation

@pytest.mark.parametrize("name", ["tiny", "kaggle_r32"])
def test_sampled_gaussian_init_matches_oracle(name):
    t = W.WORKLOADS[name].tables[0]
    shape, oshape = B.shape_of(t), ora.Shape.of(t)
    cores = [torch.full((oshape.core_size(k),), float("nan"), dtype=torch.float32, device=dev()) for k in range(3)]
    B.tt_init_sampled_gaussian(shape, cores, 12345)
    torch.cuda.synchronize()
    ref = ora.init_sampled_gaussian(oshape, 12345)
    scale = ora.sampled_gaussian_scale(oshape)
    for k in range(3):
        got = cores[k].cpu().numpy()
        # same draws (the generator is integer work), the transform within a few fp64 roundings: at most the
        # last bit of the fp32 result may differ
        np.testing.assert_allclose(got, ref[k], rtol=2e-7, atol=0)
        assert np.all(np.abs(got) > 2.0 * scale * (1 - 1e-6))
    again = [torch.empty_like(c) for c in cores]
    B.tt_init_sampled_gaussian(shape, again, 12345)
    other = [torch.empty_like(c) for c in cores]
    B.tt_init_sampled_gaussian(shape, other, 12346)
    torch.cuda.synchronize()
    assert all(torch.equal(a, c) for a, c in zip(again, cores))
    assert not torch.equal(other[1], cores[1])


# ------------------------------------------------------------------ any number of cores

@pytest.mark.parametrize("d,m,n,r", [
    (2, (40, 25), (4, 4), (1, 16, 1)),
    (3, (10, 10, 10), (2, 2, 4), (1, 8, 8, 1)),
    (4, (6, 5, 7, 4), (2, 3, 2, 2), (1, 4, 7, 5, 1)),
    (4, (8, 8, 8, 8), (2, 2, 2, 2), (1, 16, 16, 16, 1)),
])
def test_general_d_matches_oracle(d, m, n, r):
    rng = np.random.default_rng(90 + d + m[0])
    rows, N = int(np.prod(m)), int(np.prod(n))
    cores = [(0.3 * rng.standard_normal((m[k], r[k], n[k], r[k + 1]))).astype(np.float32) for k in range(d)]
    n_bags = 40
    lens = rng.integers(0, 9, n_bags)
    lens[3] = 300                                                  # more than one scan chunk
    off = np.zeros(n_bags + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    L = int(off[-1])
    idx = rng.integers(0, rows, L).astype(np.int64)
    idx[10:60] = idx[9]                                            # a hot row
    alpha = (0.5 + rng.random(L)).astype(np.float32)
    go = rng.standard_normal((n_bags, N)).astype(np.float32)
    dv = dev()
    shape = B.make_shape_d(rows, m, n, r)
    g = [torch.from_numpy(c).to(dv) for c in cores]
    ti, to, ta, tg = (torch.from_numpy(x).to(dv) for x in (idx, off, alpha, go))
    out = torch.full((n_bags, N), float("nan"), dtype=torch.float32, device=dv)
    B.tt_embd_fwd(shape, g, ti, to, n_bags, out, alpha=ta)
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy(), ora.fwd_d(m, n, r, cores, idx, off, alpha), "d=%d forward" % d)
    marker = 3.5
    grads = [torch.full_like(x, marker) for x in g]
    B.tt_embd_bwd(shape, g, ti, to, n_bags, tg, grads, alpha=ta)
    torch.cuda.synchronize()
    ref = ora.bwd_d(m, n, r, cores, idx, off, go, alpha)
    for k in range(d):
        assert_close(grads[k].cpu().numpy() - marker, ref[k], "d=%d dG%d" % (d, k + 1))      # "+=" on top of the marker
    again = [torch.full_like(x, marker) for x in g]
    B.tt_embd_bwd(shape, g, ti, to, n_bags, tg, again, alpha=ta)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(again, grads))    # deterministic
    only = [(x - marker) for x in grads]
    B.tt_embd_sgd_update(shape, g, only, 0.1, zero_grad=True)
    torch.cuda.synchronize()
    for k in range(d):
        assert_close(g[k].cpu().numpy(), ora.sgd(cores[k], ref[k], 0.1), "d=%d sgd core %d" % (d, k + 1))
        assert float(only[k].abs().max()) == 0.0


def test_general_d_three_cores_agree_with_the_tuned_path():
    wl = W.WORKLOADS["tiny"]
    d = DeviceTable(wl)
    t = wl.tables[0]
    shape = B.make_shape_d(t.num_rows, t.m, t.n, t.r)
    out = torch.empty((d.n_bags, t.dim), dtype=torch.float32, device=dev())
    B.tt_embd_fwd(shape, d.g, d.idx, d.off, d.n_bags, out)
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy(), d.fwd(), "general-d against tuned forward")


# ------------------------------------------------------------------ the benchmark's launch configuration

def test_graph_replays_of_the_benchmark_step_match_eager_calls():
    """bench.py replays a HIP graph of steps (forward keeping T0, then backward + SGD into the other
    set of cores).  Every replay must leave the same cores as the same steps launched one by one,
    and those match the oracle."""
    wl = W.WORKLOADS["kaggle_r32"]
    t = wl.tables[0]
    shape, oshape = B.shape_of(t), ora.Shape.of(t)
    cores_h = W.make_cores(t, wl.init, wl.seed)
    batches = [W.make_batch(wl, 0, j) for j in range(2)]
    d = dev()
    idx = [torch.from_numpy(b.indices).to(d) for b in batches]
    off = [torch.from_numpy(b.offsets).to(d) for b in batches]
    go = [torch.from_numpy(b.grad_output).to(d) for b in batches]
    lr = 0.01

    def fresh():
        a = [torch.from_numpy(c).to(d) for c in cores_h]
        return a, [torch.empty_like(x) for x in a]

    def two_steps(a, b, out, t0):
        for j in range(2):
            cur, nxt = (a, b) if j == 0 else (b, a)
            B.tt_emb_fwd_keep_t0(shape, cur, idx[j], off[j], wl.n_bags, out, t0[j])
            B.tt_emb_bwd_sgd(shape, cur, nxt, idx[j], off[j], wl.n_bags, go[j], lr, t0=t0[j])

    def buffers():
        return (torch.empty((wl.n_bags, t.dim), dtype=torch.float32, device=d),
                [torch.empty((wl.n_bags, B.t0_floats(shape)), dtype=torch.float32, device=d) for _ in range(2)])

    # eager: three times two steps, keeping the cores after every pair
    a, b = fresh()
    out, t0 = buffers()
    eager = []
    for _ in range(3):
        two_steps(a, b, out, t0)
        torch.cuda.synchronize()
        eager.append([x.clone() for x in a])
    # graph: capture the pair once, replay it three times with other work in between
    ga, gb = fresh()
    gout, gt0 = buffers()
    two_steps(ga, gb, gout, gt0)                                   # warm-up outside the capture
    for k in range(3):
        ga[k].copy_(torch.from_numpy(cores_h[k]))
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        two_steps(ga, gb, gout, gt0)
    for k in range(3):
        ga[k].copy_(torch.from_numpy(cores_h[k]))                  # the capture does not run anything
    for rep in range(3):
        g.replay()
        torch.cuda.synchronize()
        for k in range(3):
            assert torch.equal(ga[k], eager[rep][k]), (rep, k)
        _ = (gout * 2).sum().item()                                # unrelated eager work between replays
    # and the first pair against the oracle
    oc = [c.copy() for c in cores_h]
    for j in range(2):
        dg, _ = ora.bwd(oshape, oc, batches[j].indices, batches[j].offsets, batches[j].grad_output)
        oc = [ora.sgd(oc[k], dg[k], lr) for k in range(3)]
    for k in range(3):
        assert_close(eager[0][k].cpu().numpy(), oc[k], "two benchmark steps, core %d" % (k + 1))


def test_graph_replays_of_the_two_stream_step_match_eager_calls():
    """The steps as bench.py runs them where the backward has an index-only pre-pass (multi-hot table with its cache):
    tt_emb_bwd_prepare on a second stream, one step ahead, then tt_emb_bwd_sgd_prepared.  Replays of the
    captured pair of steps (forks and joins inside the graph) leave the same cores and cache lines, bit for bit,
    as the one-call steps launched one by one."""
    wl = W.WORKLOADS["multihot_cache"]
    t = wl.tables[0]
    shape = B.shape_of(t)
    cores_h = W.make_cores(t, wl.init, wl.seed)
    batches = [W.make_batch(wl, 0, j) for j in range(2)]
    d = dev()
    idx = [torch.from_numpy(b.indices).to(d) for b in batches]
    off = [torch.from_numpy(b.offsets).to(d) for b in batches]
    go = [torch.from_numpy(b.grad_output).to(d) for b in batches]
    L, lr, K = idx[0].numel(), 0.01, W.cache_size(wl, 0)
    rows_h, counts_h = W.warmup_counts(wl, 0)
    assert B.bwd_has_prepass(shape, L, K, True)

    def fresh():
        a = [torch.from_numpy(c).to(d) for c in cores_h]
        cache = B.Cache(K, t.dim, d)
        B.tt_cache_build(shape, a, torch.from_numpy(rows_h).to(d), torch.from_numpy(counts_h).to(d), cache)
        torch.cuda.synchronize()
        return a, [torch.empty_like(x) for x in a], cache

    out = torch.empty((wl.n_bags, t.dim), dtype=torch.float32, device=d)
    t0 = [torch.empty((L, B.t0_floats(shape)), dtype=torch.float32, device=d) for _ in range(2)]
    ws = [torch.empty(B.bwd_sgd_workspace_bytes(shape, L, wl.n_bags, K), dtype=torch.uint8, device=d) for _ in range(2)]
    side = torch.cuda.Stream()
    done = [torch.cuda.Event(), torch.cuda.Event()]

    def prepare_on_side(j, cache):
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            B.tt_emb_bwd_prepare(shape, idx[j], off[j], wl.n_bags, cache=cache, workspace=ws[j], kept_t0=True)
            done[j].record(side)

    def two_steps(a, b, cache, two_calls):
        # as in bench.py: the pre-pass of the first step next to its forward pass, the pre-pass of the second step
        # (workspace of its own) enqueued behind that forward pass, so that it runs next to the first backward pass
        for j in range(2):
            cur, nxt = (a, b) if j == 0 else (b, a)
            if two_calls and j == 0:
                prepare_on_side(0, cache)
            B.tt_emb_fwd_keep_t0(shape, cur, idx[j], off[j], wl.n_bags, out, t0[j], cache=cache)
            if two_calls:
                if j == 0:
                    prepare_on_side(1, cache)
                torch.cuda.current_stream().wait_event(done[j])
            B.tt_emb_bwd_sgd(shape, cur, nxt, idx[j], off[j], wl.n_bags, go[j], lr, cache=cache, workspace=ws[j], t0=t0[j],
                             prepared=two_calls)

    a, b, cache = fresh()
    eager = []
    for _ in range(3):
        two_steps(a, b, cache, False)
        torch.cuda.synchronize()
        eager.append(([x.clone() for x in a], cache.rows.clone()))
    ga, gb, gcache = fresh()
    start_rows = gcache.rows.clone()
    two_steps(ga, gb, gcache, True)                                # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        two_steps(ga, gb, gcache, True)
    for k in range(3):
        ga[k].copy_(torch.from_numpy(cores_h[k]))
    gcache.rows.copy_(start_rows)
    for rep in range(3):
        g.replay()
        torch.cuda.synchronize()
        for k in range(3):
            assert torch.equal(ga[k], eager[rep][0][k]), (rep, k)
        assert torch.equal(gcache.rows, eager[rep][1]), rep
        _ = (out * 2).sum().item()                                 # unrelated eager work between replays
