"""tt_emb_fwd_prepared: the forward pass that works from the per-slice lists of the backward's pre-pass (workgroups own
slices of the second core, Eq. 3's first product on the matrix cores), against the oracle and against tt_emb_fwd."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import tt_oracle as ora
from paper_2101_11714_amd import binding as B
from paper_2101_11714_amd import workloads as W
from gpu_util import DeviceTable, assert_close, dev, sample_bags

pytestmark = pytest.mark.gpu

# (workload, table): the four shapes with such a kernel: (2,2,4) R = 32, 64 and (4,4,4) R = 32, 64
SHAPES = [("sweep_r32", 0), ("sweep_r64", 0), ("multihot_cache", 0), ("terabyte_r64", 0)]


def _prepared_forward(d, cache=None, keep=False, use_offsets=True):
    K = cache.K if cache is not None else 0
    assert B.bwd_has_prepass(d.shape, d.L, K, keep)
    ws = torch.empty(B.bwd_sgd_workspace_bytes(d.shape, d.L, d.n_bags, K), dtype=torch.uint8, device=dev())
    off = d.off if use_offsets else None
    B.tt_emb_bwd_prepare(d.shape, d.idx, off, d.n_bags, cache=cache, workspace=ws, kept_t0=keep)
    out = torch.full((d.n_bags, d.t.dim), float("nan"), dtype=torch.float32, device=dev())
    t0 = torch.full((d.L, B.t0_floats(d.shape)), float("nan"), dtype=torch.float32, device=dev()) if keep else None
    B.tt_emb_fwd_prepared(d.shape, d.g, d.idx, off, d.n_bags, out, ws, t0=t0, alpha=d.alpha, cache=cache)
    torch.cuda.synchronize()
    return out.cpu().numpy(), t0, ws


@pytest.fixture
def always_grouped():
    old = B.set_fast_path(2)                       # the pre-pass groups whatever the number of positions
    yield
    B.set_fast_path(old)


def _ragged(t, seed, n_bags=260, longest=40, hot=True):
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, longest + 1, n_bags)
    lens[::7] = 0
    lens[3] = 300                                  # one bag over several tiles
    off = np.zeros(n_bags + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    L = int(off[-1])
    idx = rng.integers(0, t.num_rows, L).astype(np.int64)
    if hot:
        idx[rng.choice(L, L // 5, replace=False)] = idx[0]          # a hot row: its slice fills several tiles
        second = (idx[1] // t.m[2]) * t.m[2]                          # and rows that share a slice of the second core only
        idx[rng.choice(L, L // 10, replace=False)] = second + rng.integers(0, t.m[2], L // 10)
    alpha = (0.5 + rng.random(L)).astype(np.float32)
    return W.Batch(idx, off, rng.standard_normal((n_bags, t.dim)).astype(np.float32), alpha)


@pytest.mark.parametrize("name,table", SHAPES)
@pytest.mark.parametrize("keep", [False, True])
def test_matches_oracle_on_ragged_weighted_bags(name, table, keep, always_grouped):
    wl = W.WORKLOADS[name]
    t = wl.tables[table]
    d = DeviceTable(wl, table=table, batch=_ragged(t, 31 + table))
    out, t0, _ = _prepared_forward(d, keep=keep)
    ref = ora.fwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, alpha=d.batch.alpha)
    assert_close(out, ref, "%s forward from lists" % name)
    assert_close(out, d.fwd(), "%s against tt_emb_fwd" % name)
    if keep:
        got = t0.cpu().numpy()
        assert not np.isnan(got).any()
        pick = np.random.default_rng(3).choice(d.L, 64, replace=False)
        want = np.stack([ora.t0(d.oshape, d.cores, int(d.batch.indices[k])).reshape(-1) for k in pick])
        assert_close(got[pick], want, "%s T0 from lists" % name)
        # the backward that follows reads this T0 and the same workspace
        _, t0_plain = d.fwd_keep_t0()
        assert_close(got, t0_plain.cpu().numpy(), "%s T0 against tt_emb_fwd_keep_t0" % name)


@pytest.mark.parametrize("name,table", [("sweep_r64", 0), ("terabyte_r64", 0), ("sweep_r32", 0)])   # (rank 32 with a cache: the wave-per-bag kernel)
def test_with_cache_and_backward_after_it(name, table, always_grouped):
    wl = W.WORKLOADS[name]
    t = wl.tables[table]
    d = DeviceTable(wl, table=table, batch=_ragged(t, 77))
    rows, counts = np.unique(d.batch.indices, return_counts=True)
    K = 40
    cache, _, _ = d.build_cache(K, rows.astype(np.int64), counts.astype(np.int64))
    keys = ora.cache_select(rows, counts, K)
    crow = (cache.rows.cpu().numpy()[:K] * 1.25).astype(np.float32)
    cache.rows[:K].copy_(torch.from_numpy(crow))
    out, t0, ws = _prepared_forward(d, cache=cache, keep=True)
    ref = ora.fwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, alpha=d.batch.alpha, cache_keys=keys, cache_rows=crow)
    assert_close(out, ref, "%s forward from lists with cache" % name)
    cached = ora.cache_lookup(d.oshape, keys, d.batch.indices) >= 0
    got = t0.cpu().numpy()
    assert cached.any() and np.isnan(got[cached]).all() and not np.isnan(got[~cached]).any()
    # the rest of the step on the same workspace: the lists are still there
    new = [torch.full_like(x, float("nan")) for x in d.g]
    B.tt_emb_bwd_sgd(d.shape, d.g, new, d.idx, d.off, d.n_bags, d.go, 0.05, alpha=d.alpha, cache=cache, workspace=ws, t0=t0,
                     prepared=True)
    torch.cuda.synchronize()
    rg, rc = ora.bwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, d.batch.grad_output, alpha=d.batch.alpha, cache_keys=keys)
    for k in range(3):
        assert_close(new[k].cpu().numpy(), ora.sgd(d.cores[k], rg[k], 0.05), "%s core %d after the prepared step" % (name, k + 1))
    assert_close(cache.rows.cpu().numpy()[:K], ora.sgd(crow, rc, 0.05), "%s cache lines" % name)


@pytest.mark.parametrize("name,P", [("sweep_r32", 100), ("sweep_r64", 100)])
def test_full_size_long_bags(name, P):
    """2048 bags of 100 positions (the pooling study's largest case), default kernel selection: sampled bags against the
    oracle, every bag against the wave-per-bag forward."""
    base = W.WORKLOADS[name]
    wl = dataclasses.replace(base, n_bags=2048, bag_len=(P, P))
    d = DeviceTable(wl)
    out, t0, _ = _prepared_forward(d, keep=True)
    pick, idx, off, alpha = sample_bags(d.batch, 24)
    assert_close(out[pick], ora.fwd(d.oshape, d.cores, idx, off, alpha=alpha), "%s P = %d sampled bags" % (name, P))
    assert_close(out, d.fwd(), "%s P = %d every bag" % (name, P))
    got = t0.cpu().numpy()
    ks = np.random.default_rng(5).choice(d.L, 32, replace=False)
    want = np.stack([ora.t0(d.oshape, d.cores, int(d.batch.indices[k])).reshape(-1) for k in ks])
    assert_close(got[ks], want, "%s P = %d T0" % (name, P))


def test_one_index_per_bag_without_offsets(always_grouped):
    wl = W.WORKLOADS["terabyte_r64"]
    d = DeviceTable(wl)
    out, _, _ = _prepared_forward(d, use_offsets=False)
    pick = np.random.default_rng(9).choice(d.n_bags, 200, replace=False)
    ref = ora.fwd(d.oshape, d.cores, d.batch.indices[pick], np.arange(pick.size + 1, dtype=np.int64))
    assert_close(out[pick], ref, "terabyte rows from lists")
    assert_close(out, d.fwd(use_offsets=False), "terabyte against tt_emb_fwd")


def test_short_streams_and_other_shapes_fall_back():
    """Where the pre-pass does not group (short streams) or the shape has no such kernel, the call is tt_emb_fwd."""
    wl = W.WORKLOADS["kaggle_r32"]
    d = DeviceTable(wl)
    ws = torch.empty(max(B.bwd_sgd_workspace_bytes(d.shape, d.L, d.n_bags, 0), 256), dtype=torch.uint8, device=dev())
    out = torch.full((d.n_bags, d.t.dim), float("nan"), dtype=torch.float32, device=dev())
    B.tt_emb_fwd_prepared(d.shape, d.g, d.idx, d.off, d.n_bags, out, ws)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), d.fwd())


@pytest.mark.parametrize("name,table,with_cache", [("sweep_r32", 0, False), ("terabyte_r64", 0, False), ("sweep_r64", 0, True)])
def test_ragged_weighted_bags_with_item_records(name, table, with_cache):
    """Where the backward that follows runs on tiles, the pre-pass also writes a record per sorted item (position, digits,
    bag) and the forward takes its tiles' positions and digits from those instead of reading and decoding the rows:
    ragged, weighted bags with a hot row, with and without a cache, the kept T0 as well."""
    old = B.set_fast_path(3)                       # groups whatever the number of positions; the backward on tiles, also with a cache
    try:
        wl = W.WORKLOADS[name]
        t = wl.tables[table]
        d = DeviceTable(wl, table=table, batch=_ragged(t, 53 + table))
        cache, keys, crow = None, None, None
        if with_cache:
            rows, counts = np.unique(d.batch.indices, return_counts=True)
            cache, _, _ = d.build_cache(40, rows.astype(np.int64), counts.astype(np.int64))
            keys = ora.cache_select(rows, counts, 40)
            crow = cache.rows.cpu().numpy()[:40].copy()
        out, t0, _ = _prepared_forward(d, cache=cache, keep=True)
        ref = ora.fwd(d.oshape, d.cores, d.batch.indices, d.batch.offsets, alpha=d.batch.alpha, cache_keys=keys, cache_rows=crow)
        assert_close(out, ref, "%s forward from lists and item records" % name)
        got = t0.cpu().numpy()
        cached = ora.cache_lookup(d.oshape, keys, d.batch.indices) >= 0 if with_cache else np.zeros(d.L, dtype=bool)
        pick = np.random.default_rng(3).choice(np.flatnonzero(~cached), 48, replace=False)
        want = np.stack([ora.t0(d.oshape, d.cores, int(d.batch.indices[k])).reshape(-1) for k in pick])
        assert_close(got[pick], want, "%s T0 from lists and item records" % name)
    finally:
        B.set_fast_path(old)
