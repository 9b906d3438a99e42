"""Microbenchmarks of the TT-EmbeddingBag kernels against an uncompressed EmbeddingBag on the
same GPU (the studies of Sections 6.6 and 6.7 of the paper, on synthetic inputs):

  pooling : pooling factor P in {1, 10, 100} x TT rank, Kaggle-shaped table (10,131,227 rows,
            dimension 16), 2048 samples per step, Zipf(1.05) indices, no cache;
  hitrate : cache hit rate 0 .. 99 %, a 10 M-row table of dimension 64 at rank 32 with a cache
            of 0.01 % of its rows, 2048 samples per step, P in {10, 100}.

  tables  : the seven independent tables of the multi-hot workload (8192 samples x 20 indices each,
            caches of 0.01 %), one after the other on one stream against one stream per table.

A step is forward + backward + SGD.  TT: tt_emb_fwd_keep_t0 + tt_emb_bwd_sgd_t0 (tt_emb_fwd_keep +
tt_emb_bwd_sgd_kept where the library keeps position lists; tt_emb_bwd_prepare one step ahead on a second stream,
tt_emb_fwd_prepared and tt_emb_bwd_sgd_prepared where the backward has an index-only pre-pass); dense: tt_dense_bag_fwd + the faster
of tt_dense_bag_bwd_sgd (one float atomic per position and column) and tt_dense_bag_bwd_sgd_merged
(positions sorted by row, duplicates added up first, one write per distinct row), both reported.
Every step sequence is captured in a HIP graph, so the figures are GPU times.  Prints a markdown table.

    python -m paper_2101_11714_amd.microbench [pooling] [hitrate] [tables] [pooling:P:R]
"""

from __future__ import annotations

import dataclasses
import sys

import numpy as np
import torch

from . import binding as B
from . import workloads as W

N_BAGS = 2048
STEPS = 8            # steps per captured graph (distinct batches)


def _graph_us(fn) -> float:
    """GPU microseconds per call of fn(j), j = 0..STEPS-1, replayed from a HIP graph."""
    for j in range(STEPS):
        fn(j)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for j in range(STEPS):
            fn(j)
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 10
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (reps * STEPS)


class _Table:
    def __init__(self, shape: W.TableShape, init: str, seed: int, dev):
        self.shape, self.dev = shape, dev
        self.c = B.shape_of(shape)
        self.cores = [torch.from_numpy(x).to(dev) for x in W.make_cores(shape, init, seed)]
        self.cores2 = [torch.empty_like(x) for x in self.cores]
        self.dense = torch.empty((shape.num_rows, shape.dim), dtype=torch.float32, device=dev).normal_(0, 0.01)

    def time(self, batches, cache=None, lr=1e-6, dense=True):
        dev, n_bags = self.dev, batches[0].offsets.size - 1
        idx = [torch.from_numpy(b.indices).to(dev) for b in batches]
        off = [torch.from_numpy(b.offsets).to(dev) for b in batches]
        go = [torch.from_numpy(b.grad_output).to(dev) for b in batches]
        L = idx[0].numel()
        out = torch.empty((n_bags, self.shape.dim), dtype=torch.float32, device=dev)
        t0 = [torch.empty((L, B.t0_floats(self.c)), dtype=torch.float32, device=dev) for _ in batches]
        ws = torch.empty(B.bwd_sgd_workspace_bytes(self.c, L, n_bags, cache.K if cache else 0), dtype=torch.uint8, device=dev)

        # The index-only part of the backward (cache probe, grouping of long lists) on a second stream, one step ahead:
        # the pre-pass of step j + 1 is enqueued behind the forward pass of step j (two workspaces alternate), the first
        # one of a graph next to its own forward pass.
        two_calls = B.bwd_has_prepass(self.c, L, cache.K if cache else 0, True)
        fwd_lists = two_calls and B.fwd_uses_lists(self.c, L, cache.K if cache else 0, True)
        side = torch.cuda.Stream() if two_calls else None
        wsp = [ws, torch.empty_like(ws)] if two_calls else [ws, ws]
        done = [torch.cuda.Event(), torch.cuda.Event()] if two_calls else None

        def prepare_on_side(j):
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                B.tt_emb_bwd_prepare(self.c, idx[j], off[j], n_bags, cache=cache, workspace=wsp[j % 2], kept_t0=True)
                done[j % 2].record(side)

        def tt_step(j):
            cur, nxt = (self.cores, self.cores2) if j % 2 == 0 else (self.cores2, self.cores)
            if two_calls and j == 0:
                prepare_on_side(0)
            if fwd_lists:                                   # the forward pass works from the pre-pass's lists where it can
                torch.cuda.current_stream().wait_event(done[j % 2])
                B.tt_emb_fwd_prepared(self.c, cur, idx[j], off[j], n_bags, out, wsp[j % 2], t0=t0[j], cache=cache)
            else:
                B.tt_emb_fwd_keep_t0(self.c, cur, idx[j], off[j], n_bags, out, t0[j], cache=cache)
            if two_calls and j + 1 < STEPS:
                prepare_on_side(j + 1)                      # next to this step's backward pass
            if two_calls and not fwd_lists:
                torch.cuda.current_stream().wait_event(done[j % 2])
            B.tt_emb_bwd_sgd(self.c, cur, nxt, idx[j], off[j], n_bags, go[j], lr, cache=cache, workspace=wsp[j % 2], t0=t0[j],
                             prepared=two_calls)

        # short lists of the (2,2,4) shapes: per-slice position lists, filed for batch j + 1 by riders of batch j's backward
        lists = cache is None and B.kept_has_lists(self.c, L)
        if lists:
            kept = [torch.empty(B.kept_bytes(self.c, L), dtype=torch.uint8, device=dev) for _ in batches]
            B.tt_emb_kept_prepare(self.c, idx[0], kept[0])

            def tt_step(j):                                                  # noqa: F811
                cur, nxt = (self.cores, self.cores2) if j % 2 == 0 else (self.cores2, self.cores)
                jn = (j + 1) % STEPS
                B.tt_emb_fwd_keep(self.c, cur, idx[j], off[j], n_bags, out, kept[j], lists_ready=True)
                B.tt_emb_bwd_sgd_kept(self.c, cur, nxt, idx[j], off[j], n_bags, go[j], kept[j], lr, workspace=ws,
                                      next_batch=(idx[jn], kept[jn]))

        wsd = torch.empty(max(B.dense_bwd_workspace_bytes(L, self.shape.dim), 256), dtype=torch.uint8, device=dev)

        def dense_step_atomic(j):
            B.tt_dense_bag_fwd(self.dense, idx[j], off[j], n_bags, out)
            B.tt_dense_bag_bwd_sgd(self.dense, idx[j], off[j], n_bags, go[j], lr)

        def dense_step_merged(j):
            B.tt_dense_bag_fwd(self.dense, idx[j], off[j], n_bags, out)
            B.tt_dense_bag_bwd_sgd_merged(self.dense, idx[j], off[j], n_bags, go[j], lr, workspace=wsd)

        if not dense:                                       # (the TT side alone: for a kernel trace)
            return _graph_us(tt_step), float("nan"), float("nan")
        return _graph_us(tt_step), _graph_us(dense_step_atomic), _graph_us(dense_step_merged)


def pooling(dev, only=None):
    """only = (P, R): that configuration alone, TT side only (for a kernel trace of it)."""
    print("## Pooling factor x TT rank (Kaggle-shaped table, %d samples per step, no cache)\n" % N_BAGS)
    print("| P | lookups/step | R | TT step us | dense us, atomics | dense us, merged | TT / faster dense | TT us per sample | TT M lookups/s |")
    print("|---|---|---|---|---|---|---|---|---|")
    for R in (8, 16, 32, 64):
        if only and R != only[1]:
            continue
        base = W.WORKLOADS["sweep_r%d" % R]
        tab = _Table(base.tables[0], base.init, base.seed, dev)
        for P in (1, 10, 100):
            if only and P != only[0]:
                continue
            wl = dataclasses.replace(base, n_bags=N_BAGS, bag_len=(P, P))
            batches = [W.make_batch(wl, 0, j) for j in range(STEPS)]
            tt, da, dm = tab.time(batches, dense=not only)
            L = N_BAGS * P
            print("| %d | %d | %d | %.1f | %.1f | %.1f | %.1f | %.4f | %.1f |"
                  % (P, L, R, tt, da, dm, tt / min(da, dm), tt / N_BAGS, L / tt), flush=True)
        del tab
        torch.cuda.empty_cache()


def hitrate(dev):
    wl = W.WORKLOADS["multihot_cache"]
    shape = wl.tables[0]
    K = W.cache_size(wl, 0)
    print("\n## Cache hit rate (table of %d rows, dimension %d, R = %d, cache of %d rows, %d samples per step)\n"
          % (shape.num_rows, shape.dim, shape.r[1], K, N_BAGS))
    print("| P | hit rate | TT+cache step us | dense us, atomics | dense us, merged | TT / faster dense | TT M lookups/s |")
    print("|---|---|---|---|---|---|---|")
    tab = _Table(shape, wl.init, wl.seed, dev)
    rng = np.random.default_rng(77)
    cached = np.sort(rng.choice(shape.num_rows, K, replace=False)).astype(np.int64)
    cache = B.Cache(K, shape.dim, dev)
    B.tt_cache_build(tab.c, tab.cores, torch.from_numpy(cached).to(dev),
                     torch.ones(K, dtype=torch.int64, device=dev), cache)
    for P in (10, 100):
        for h in (0.0, 0.5, 0.75, 0.9, 0.95, 0.99):
            batches = [W.make_hit_rate_batch(shape, cached, N_BAGS, P, h, 100 + j) for j in range(STEPS)]
            tt, da, dm = tab.time(batches, cache=cache)
            L = N_BAGS * P
            print("| %d | %.0f %% | %.1f | %.1f | %.1f | %.1f | %.1f |" % (P, 100 * h, tt, da, dm, tt / min(da, dm), L / tt),
                  flush=True)


def tables(dev):
    """All tables of the multi-hot workload in one step: their kernels are independent, so a stream per
    table lets the GPU overlap one table's latency-bound kernels with another's."""
    wl = W.WORKLOADS["multihot_cache"]
    nt, nb = len(wl.tables), 2                                      # two distinct batches per table
    print("\n## The %d tables of the multi-hot workload in one step (%d samples x %d indices per table, caches of 0.01 %%)\n"
          % (nt, wl.n_bags, wl.bag_len[0]))
    state = []
    for tb in range(nt):
        shape = wl.tables[tb]
        c = B.shape_of(shape)
        cores = [torch.from_numpy(x).to(dev) for x in W.make_cores(shape, wl.init, wl.seed, tb)]
        cores2 = [torch.empty_like(x) for x in cores]
        K = W.cache_size(wl, tb)
        rows, counts = W.warmup_counts(wl, tb)
        cache = B.Cache(K, shape.dim, dev)
        B.tt_cache_build(c, cores, torch.from_numpy(rows).to(dev), torch.from_numpy(counts).to(dev), cache)
        bs = [W.make_batch(wl, tb, j) for j in range(nb)]
        L = bs[0].indices.size
        state.append(dict(
            c=c, cores=cores, cores2=cores2, cache=cache, L=L,
            idx=[torch.from_numpy(b.indices).to(dev) for b in bs], off=[torch.from_numpy(b.offsets).to(dev) for b in bs],
            go=[torch.from_numpy(b.grad_output).to(dev) for b in bs],
            out=torch.empty((wl.n_bags, shape.dim), dtype=torch.float32, device=dev),
            t0=[torch.empty((L, B.t0_floats(c)), dtype=torch.float32, device=dev) for _ in bs],
            ws=torch.empty(B.bwd_sgd_workspace_bytes(c, L, wl.n_bags, K), dtype=torch.uint8, device=dev)))
    total = sum(s["L"] for s in state)

    def step(s, j):
        cur, nxt = (s["cores"], s["cores2"]) if j % 2 == 0 else (s["cores2"], s["cores"])
        B.tt_emb_fwd_keep_t0(s["c"], cur, s["idx"][j], s["off"][j], wl.n_bags, s["out"], s["t0"][j], cache=s["cache"])
        B.tt_emb_bwd_sgd(s["c"], cur, nxt, s["idx"][j], s["off"][j], wl.n_bags, s["go"][j], 1e-6, cache=s["cache"],
                         workspace=s["ws"], t0=s["t0"][j])

    def run(streams):
        main_stream = torch.cuda.current_stream()
        for j in range(nb):
            for tb, s in enumerate(state):
                if streams is None:
                    step(s, j)
                else:
                    streams[tb].wait_stream(main_stream)
                    with torch.cuda.stream(streams[tb]):
                        step(s, j)
            if streams is not None:
                for st in streams:
                    main_stream.wait_stream(st)

    def graph_us(streams):
        run(streams)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            run(streams)
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * nb)

    seq = graph_us(None)
    par = graph_us([torch.cuda.Stream() for _ in range(nt)])
    print("| launch | step us (all %d tables) | M lookups/s |" % nt)
    print("|---|---|---|")
    print("| one stream, table after table | %.1f | %.1f |" % (seq, total / seq))
    print("| one stream per table | %.1f | %.1f |" % (par, total / par), flush=True)


def main():
    assert torch.cuda.is_available(), "the microbenchmarks need a GPU"
    dev = torch.device("cuda:0")
    which = sys.argv[1:] or ["pooling", "hitrate", "tables"]
    print("# TT-EmbeddingBag against an uncompressed EmbeddingBag on one MI355X (forward + backward + SGD per step)\n")
    if "pooling" in which:
        pooling(dev)
    for w in which:
        if w.startswith("pooling:"):                          # pooling:P:R, e.g. pooling:100:64
            pooling(dev, only=tuple(int(x) for x in w.split(":")[1:3]))
    if "hitrate" in which:
        hitrate(dev)
    if "tables" in which:
        tables(dev)


if __name__ == "__main__":
    main()
