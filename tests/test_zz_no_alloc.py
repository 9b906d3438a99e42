"""The entry point that allocates nothing (tt_emb_bwd_sgd_static: scratch memory in a static device
array of the library) against tt_emb_bwd_sgd with a caller's workspace, through the C ABI: same
bits, on calls in a row of which the later ones are smaller and leave stale data behind them in the
shared array."""

import numpy as np
import pytest
import torch

from paper_2101_11714_amd import binding as B
from paper_2101_11714_amd import workloads as W
from gpu_util import DeviceTable, dev

pytestmark = pytest.mark.gpu


def _both(d, lr, cache_pair=None):
    """New cores (and cache lines) from the workspace call and from the static call on the same inputs."""
    res = []
    for static in (False, True):
        cache = None
        if cache_pair is not None:
            cache = cache_pair[int(static)]
        out = [torch.full_like(x, float("nan")) for x in d.g]
        if static:
            B.tt_emb_bwd_sgd_static(d.shape, d.g, out, d.idx, d.off, d.n_bags, d.go, lr, alpha=d.alpha, cache=cache)
        else:
            ws = torch.empty(max(256, B.bwd_sgd_workspace_bytes(d.shape, d.L, d.n_bags, cache.K if cache else 0)),
                             dtype=torch.uint8, device=dev())
            B.tt_emb_bwd_sgd(d.shape, d.g, out, d.idx, d.off, d.n_bags, d.go, lr, alpha=d.alpha, cache=cache, workspace=ws)
        torch.cuda.synchronize()
        res.append([o.cpu().numpy() for o in out] + ([cache.rows.cpu().numpy()] if cache else []))
    return res


def _sub_batch(wl, n_bags, seed):
    """The first n_bags bags of a later batch of the workload."""
    b = W.make_batch(wl, 0, seed)
    L = int(b.offsets[n_bags])
    return W.Batch(b.indices[:L].copy(), b.offsets[:n_bags + 1].copy(), b.grad_output[:n_bags].copy(),
                   None if b.alpha is None else b.alpha[:L].copy())


def test_static_scratch_equals_workspace_call_large_then_small():
    # sweep_r64 at 4,096 positions: several workgroups share a slice and leave partial sums in the scratch memory
    wl = W.WORKLOADS["sweep_r64"]
    assert B.bwd_sgd_workspace_bytes(B.shape_of(wl.tables[0]), 4096, 4096, 0) <= B.static_scratch_bytes()
    for n_bags, seed in [(4096, 0), (1000, 1), (4096, 2), (3, 3)]:
        d = DeviceTable(wl, batch=_sub_batch(wl, n_bags, seed))
        a, b = _both(d, 0.05)
        for x, y in zip(a, b):
            assert np.array_equal(x, y), (n_bags, seed)
            assert np.isfinite(y).all()


def test_static_scratch_with_cache_and_long_stream_then_short():
    # multi-hot table 0: grouping pre-pass, cached-row gradients and per-row G1 gradients all live in the scratch memory
    wl = W.WORKLOADS["multihot_cache"]
    K = W.cache_size(wl, 0)
    rows, counts = W.warmup_counts(wl, 0)
    for n_bags, seed in [(1500, 0), (40, 1), (700, 2)]:
        d = DeviceTable(wl, batch=_sub_batch(wl, n_bags, seed))
        caches = []
        for _ in range(2):
            c = B.Cache(K, d.t.dim, dev())
            B.tt_cache_build(d.shape, d.g, torch.from_numpy(rows).to(dev()), torch.from_numpy(counts).to(dev()), c)
            caches.append(c)
        a, b = _both(d, 0.05, caches)
        for x, y in zip(a, b):
            assert np.array_equal(x, y), (n_bags, seed)


def test_static_scratch_rejects_what_does_not_fit():
    wl = W.WORKLOADS["multihot_cache"]
    d = DeviceTable(wl)                                      # 163,840 positions: far more than 32 MiB of scratch
    K = W.cache_size(wl, 0)
    assert B.bwd_sgd_workspace_bytes(d.shape, d.L, d.n_bags, K) > B.static_scratch_bytes()
    cache, _, _ = d.build_cache(K)
    out = [torch.zeros_like(x) for x in d.g]
    with pytest.raises(B.TTError) as e:
        B.tt_emb_bwd_sgd_static(d.shape, d.g, out, d.idx, d.off, d.n_bags, d.go, 0.05, cache=cache)
    assert e.value.code == -4 and "static" in str(e.value)
    torch.cuda.synchronize()
    assert all(float(o.abs().max()) == 0.0 for o in out)     # nothing was enqueued
