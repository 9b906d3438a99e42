"""The backward pass that works on tiles of positions on the matrix cores (the grouped backward with a kept T0 and no
cache; tt_emb_debug_set_fast_path(3) forces it for every length and with a cache): against the oracle, against the
list owners, and for bit-identical repeats."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import tt_oracle as ora
from paper_2101_11714_amd import binding as B
from paper_2101_11714_amd import workloads as W
from gpu_util import DeviceTable, assert_close, dev
from test_gpu_fwd_owner import SHAPES, _ragged

pytestmark = pytest.mark.gpu


@pytest.fixture
def always_grouped():
    old = B.set_fast_path(3)                      # groups whatever the number of positions, then the tile kernels
    yield
    B.set_fast_path(old)


@pytest.mark.parametrize("name,table", SHAPES)
def test_gradients_and_fused_step_match_oracle(name, table, always_grouped):
    wl = W.WORKLOADS[name]
    d = DeviceTable(wl, table=table, batch=_ragged(wl.tables[table], 41 + table))
    _, t0 = d.fwd_keep_t0()
    ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, alpha=d.batch.alpha)
    dg, _ = d.bwd(t0=t0)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), ref[k], "%s dG%d from tiles" % (name, k + 1))
    # gradients are added to what the arrays hold
    dg2, _ = d.bwd(t0=t0, grad_cores=[x.clone() for x in dg])
    for k in range(3):
        assert_close(dg2[k].cpu().numpy(), 2 * ref[k], "%s dG%d added twice" % (name, k + 1))
    new = d.bwd_sgd(0.05, t0=t0)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), ora.sgd(d.cores[k], ref[k], 0.05), "%s fused core %d from tiles" % (name, k + 1))
    again = d.bwd_sgd(0.05, t0=t0)
    for k in range(3):
        assert torch.equal(new[k], again[k]), "core %d differs between two runs" % (k + 1)
    # slices that no position touches are copied bit for bit
    m = d.t.m
    i1 = np.unique(d.batch.indices // (m[1] * m[2]))
    untouched = np.setdiff1d(np.arange(m[0]), i1)
    if untouched.size:
        g1 = d.g[0].reshape(m[0], -1)
        assert torch.equal(new[0].reshape(m[0], -1)[untouched], g1[untouched])
    # the list owners on the same lists: the same gradients up to the order of the sums
    old = B.set_fast_path(2)
    try:
        dg_lists, _ = d.bwd(t0=t0)
    finally:
        B.set_fast_path(old)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), dg_lists[k].cpu().numpy().astype(np.float64), "%s dG%d tiles against lists" % (name, k + 1))


@pytest.mark.parametrize("name,table", [("sweep_r64", 0), ("multihot_cache", 0)])
def test_with_cache(name, table, always_grouped):
    wl = W.WORKLOADS[name]
    d = DeviceTable(wl, table=table, batch=_ragged(wl.tables[table], 91))
    rows, counts = np.unique(d.batch.indices, return_counts=True)
    K = 40
    cache, _, _ = d.build_cache(K, rows.astype(np.int64), counts.astype(np.int64))
    keys = ora.cache_select(rows, counts, K)
    crow = cache.rows.cpu().numpy()[:K].copy()
    _, t0 = d.fwd_keep_t0(cache=cache)
    rg, rc = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, alpha=d.batch.alpha, cache_keys=keys)
    dg, dc = d.bwd(cache=cache, t0=t0)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), rg[k], "%s dG%d from tiles with cache" % (name, k + 1))
    assert_close(dc.cpu().numpy()[:K], rc, "%s dCache" % name)
    new = d.bwd_sgd(0.05, cache=cache, t0=t0)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), ora.sgd(d.cores[k], rg[k], 0.05), "%s fused core %d with cache" % (name, k + 1))
    assert_close(cache.rows.cpu().numpy()[:K], ora.sgd(crow, rc, 0.05), "%s cache lines" % name)


def test_every_position_cached_and_empty_input(always_grouped):
    wl = W.WORKLOADS["sweep_r64"]
    t = wl.tables[0]
    rng = np.random.default_rng(4)
    rows = rng.choice(t.num_rows, 30, replace=False).astype(np.int64)
    idx = rows[rng.integers(0, 30, 500)]
    off = np.arange(0, 501, 5, dtype=np.int64)
    batch = W.Batch(idx, off, rng.standard_normal((100, t.dim)).astype(np.float32), None)
    d = DeviceTable(wl, batch=batch)
    cache, _, _ = d.build_cache(30, rows, np.ones(30, dtype=np.int64))
    _, t0 = d.fwd_keep_t0(cache=cache)
    new = d.bwd_sgd(0.05, cache=cache, t0=t0)
    for k in range(3):
        assert torch.equal(new[k], d.g[k]), "core %d changed although every position is cached" % (k + 1)


@pytest.mark.parametrize("name", ["sweep_r32", "sweep_r64"])
def test_full_size_long_bags(name):
    """2048 bags of 100 positions: the whole fused step against the oracle."""
    old = B.set_fast_path(3)
    try:
        _full_size(name)
    finally:
        B.set_fast_path(old)


def _full_size(name):
    base = W.WORKLOADS[name]
    wl = dataclasses.replace(base, n_bags=2048, bag_len=(100, 100))
    d = DeviceTable(wl)
    _, t0 = d.fwd_keep_t0()
    ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output)
    new = d.bwd_sgd(wl.lr, t0=t0)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), ora.sgd(d.cores[k], ref[k], wl.lr), "%s P = 100 fused core %d" % (name, k + 1))


@pytest.mark.parametrize("name,n_bags,longest", [("terabyte_r64", 800, 24), ("sweep_r32", 1800, 24), ("sweep_r64", 1800, 24)])
def test_two_call_form_groups_earlier_and_matches_oracle(name, n_bags, longest):
    """The default kernel selection: with a kept T0 and no cache the pair tt_emb_bwd_prepare + tt_emb_bwd_sgd_prepared
    works on tiles from lengths on at which the one call still runs the slice owners (for the Terabyte-shaped table
    on tiles of 64 stacked rows).  Ragged, weighted bags with a hot row; both forms against the oracle, the pair twice."""
    wl = W.WORKLOADS[name]
    t = wl.tables[0]
    d = DeviceTable(wl, batch=_ragged(t, 7, n_bags=n_bags, longest=longest))
    assert B.bwd_two_calls_group_earlier(d.shape, d.L, 0, kept_t0=True), "the test's length no longer falls between the two limits"
    assert not B.bwd_two_calls_group_earlier(d.shape, d.L, 0, kept_t0=False)
    _, t0 = d.fwd_keep_t0()
    ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, alpha=d.batch.alpha)
    one = d.bwd_sgd(0.05, t0=t0)
    two = d.bwd_sgd(0.05, t0=t0, two_calls=True)
    again = d.bwd_sgd(0.05, t0=t0, two_calls=True)
    for k in range(3):
        want = ora.sgd(d.cores[k], ref[k], 0.05)
        assert_close(one[k].cpu().numpy(), want, "%s fused core %d in one call" % (name, k + 1))
        assert_close(two[k].cpu().numpy(), want, "%s fused core %d in two calls" % (name, k + 1))
        assert torch.equal(two[k], again[k]), "core %d differs between two runs of the pair" % (k + 1)


@pytest.mark.parametrize("name,table,n_bags,longest", [("multihot_cache", 0, 3600, 24), ("sweep_r64", 0, 7000, 24)])
def test_medium_streams_in_one_call(name, table, n_bags, longest):
    """Between 32,768 and 131,072 positions, default kernel selection, no cache, one call: the backward groups the
    positions and works on tiles, and the segmented sums take 16 or 32 items per wave (worked out on the device).
    Ragged, weighted bags with a hot row; gradients and the fused step against the oracle."""
    wl = W.WORKLOADS[name]
    t = wl.tables[table]
    d = DeviceTable(wl, table=table, batch=_ragged(t, 19 + table, n_bags=n_bags, longest=longest))
    assert 32768 <= d.L < 131072
    _, t0 = d.fwd_keep_t0()
    ref, _ = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, alpha=d.batch.alpha)
    dg, _ = d.bwd(t0=t0)
    for k in range(3):
        assert_close(dg[k].cpu().numpy(), ref[k], "%s dG%d, %d positions" % (name, k + 1, d.L))
    new = d.bwd_sgd(0.05, t0=t0)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), ora.sgd(d.cores[k], ref[k], 0.05), "%s fused core %d, %d positions" % (name, k + 1, d.L))
