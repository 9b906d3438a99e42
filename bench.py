"""Benchmark of the TT-EmbeddingBag hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input:
forward, backward and the SGD update of the cores, at the Kaggle-shaped R = 32
configuration (10,131,227 rows as 200x220x250, dimension 16 as 2x2x4, 2048 bags
of one index, Zipf(1.05) indices).  All inputs are resident in HBM before the
timed region.  By default the backward pass and the SGD update are one call
(two sets of cores used in turn), the forward pass keeps its intermediate T0 for
the backward pass, and where the library keeps per-slice position lists (short
index lists of the (2,2,4) shapes) the lists of batch i + 1 are filed by riders
of the backward launch of batch i (tt_emb_fwd_keep + tt_emb_bwd_sgd_kept);
--no-lists uses tt_emb_fwd_keep_t0 + tt_emb_bwd_sgd_t0, --recompute tt_emb_fwd +
tt_emb_bwd_sgd, --step separate tt_emb_fwd + tt_emb_bwd + tt_emb_sgd_update.
Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload kaggle_r32] [--step fused|separate] [--recompute] [--no-lists]
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
POOL = 16                      # distinct batches cycled through, so caches see a stream

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.md")


def measured_traffic(workload, table, variant, stage):
    """HBM bytes per launch (read + written) of one stage, from the tracked table of rocprofv3 counter runs
    (FETCH_SIZE / WRITE_SIZE, each scaled by what the counter reads for a copy of known size).  The table names the
    commit and the commands it was taken with; a figure is only valid for the workload and variant of its row.
    None if the table has no such row."""
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) >= 7 and cells[0] == workload and cells[1] == str(table) and cells[2] == variant and cells[3] == stage:
                    return float(cells[6]) * 1e6
    except OSError:
        pass
    return None


def pmc_means(dirs):
    """Mean counter value per kernel from rocprofv3 --pmc csv output (the figures the traffic table is made of)."""
    import collections, csv, glob
    for d in dirs:
        for path in sorted(glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)):
            acc = collections.defaultdict(lambda: [0.0, 0])
            with open(path) as f:
                for r in csv.DictReader(f):
                    k = (r["Kernel_Name"][:90], r["Counter_Name"])
                    acc[k][0] += float(r["Counter_Value"])
                    acc[k][1] += 1
            print(path)
            for k, (tot, n) in sorted(acc.items(), key=lambda kv: -kv[1][0]):
                print("  %-90s %-12s dispatches=%5d mean=%12.1f" % (k[0], k[1], n, tot / n))


def trace_context(dirs):
    """From rocprofv3 --kernel-trace csv output: duration of every kernel by the kernel that ran before it, and the idle
    time between the two (a kernel that follows another one finds different lines in the caches than one that follows
    itself, which is how the per-stage timings of this script and a trace of whole steps differ)."""
    import collections, csv, glob, statistics
    for d in dirs:
        for path in sorted(glob.glob(os.path.join(d, "**", "*kernel_trace.csv"), recursive=True)):
            with open(path) as f:
                rows = sorted(((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r["Kernel_Name"]) for r in csv.DictReader(f)))
            acc = collections.defaultdict(list)
            for (s0, e0, k0), (s1, e1, k1) in zip(rows, rows[1:]):
                name = lambda k: k.split("(")[0].split("<")[0].split("::")[-1].replace("void ", "")
                acc[(name(k0), name(k1))].append((e1 - s1, s1 - e0))
            print(path)
            for key, v in sorted(acc.items(), key=lambda kv: -len(kv[1])):
                if len(v) < 50:
                    continue
                dur, gap = sorted(x[0] for x in v), sorted(x[1] for x in v)
                q = lambda a, f: a[min(len(a) - 1, int(len(a) * f))]
                print("  %-22s after %-22s n=%6d  duration ns p10 %6d p50 %6d p90 %6d mean %8.1f | idle before ns p50 %6d mean %8.1f"
                      % (key[1], key[0], len(v), q(dur, .1), q(dur, .5), q(dur, .9), statistics.mean(dur), q(gap, .5),
                         statistics.mean(gap)))


FP32_PEAK_TFLOPS = 157.3       # MI355X fp32 vector, published


def algorithmic_flops(t, L_tt, keep_t0):
    """fp32 flops of the method for L_tt uncached lookups: F1 = 2 n1 R n2 R for T0, F2 = 2 n1 n2 R n3 for the row;
    the backward is 3 F1 + 2 F2 with recomputation (Alg. 2), 2 F1 + 2 F2 when T0 is kept."""
    F1 = 2 * t.n[0] * t.r[1] * t.n[1] * t.r[2]
    F2 = 2 * t.n[0] * t.n[1] * t.r[2] * t.n[2]
    bwd = (2 if keep_t0 else 3) * F1 + 2 * F2
    return {"fwd": L_tt * (F1 + F2), "bwd": L_tt * bwd, "bwd_sgd": L_tt * bwd, "sgd": 2 * sum(t.core_size(k) for k in range(3))}


def algorithmic_bytes(t, L, n_bags, touched_floats, n_cached=0):
    """Bytes the method must move per launch (no re-reads, no intermediates).

    forward : every lookup reads its three slices (S bytes) and its index, every bag
              writes its output row.
    backward: the same reads plus the upstream gradient row, and one write of every
              touched core slice.
    sgd     : read x, read g, write x for every core element.
    bwd_sgd : the fused call; no gradient buffers exist.
    """
    S = 4 * (t.n[0] * t.r[1] + t.r[1] * t.n[1] * t.r[2] + t.r[2] * t.n[2])
    N = t.dim
    # a cached position reads (forward) or updates (backward) its cache line instead of three slices
    reads = (L - n_cached) * (S + 8) + n_cached * (4 * N + 8)
    fwd = reads + n_bags * 4 * N
    bwd = reads + n_bags * 4 * N + 4 * touched_floats
    total = sum(t.core_size(k) for k in range(3))
    sgd = 12 * total
    # fused backward + SGD: the backward's reads, plus one read and one write of every core element
    bwd_sgd = reads + n_bags * 4 * N + 8 * total
    return {"fwd": fwd, "bwd": bwd, "sgd": sgd, "bwd_sgd": bwd_sgd}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="kaggle_r32")
    ap.add_argument("--table", type=int, default=0, help="which table of a multi-table workload")
    ap.add_argument("--weights", choices=["none", "alpha", "mean"], default="none",
                    help="alpha: per-position weights (Eq. 5); mean: average pooling (tt_emb_mean_weights)")
    ap.add_argument("--step", choices=["fused", "separate"], default="fused",
                    help="fused: forward, then backward and SGD in one call; separate: three calls")
    ap.add_argument("--recompute", action="store_true",
                    help="the backward pass recomputes the forward's intermediate T0 (tt_emb_fwd / tt_emb_bwd_sgd) "
                         "instead of reading the copy that the forward pass stored "
                         "(tt_emb_fwd_keep_t0 / tt_emb_bwd_sgd_t0, the default of the fused step)")
    ap.add_argument("--pmc-means", nargs="+", metavar="DIR",
                    help="no benchmark: print the mean counter value per kernel from rocprofv3 --pmc csv output under "
                         "the given folders")
    ap.add_argument("--trace-context", nargs="+", metavar="DIR",
                    help="no benchmark: from rocprofv3 --kernel-trace csv output under the given folders, print every "
                         "kernel's duration by the kernel that ran before it")
    ap.add_argument("--no-lists", action="store_true",
                    help="fused step with the stored T0 but without the per-slice position lists filed ahead "
                         "(tt_emb_fwd_keep_t0 / tt_emb_bwd_sgd_t0): every slice owner scans the index array itself")
    ap.add_argument("--offsets", choices=["csr", "none"], default="csr",
                    help="csr: bags given by an offsets array; none: the boundary's form for one index per bag "
                         "(offsets == NULL), for the workloads whose bags all hold one index")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--one-call", action="store_true",
                    help="fused step: the backward in one call on the step's stream, also where it has an index-only pre-pass "
                         "(by default that runs on a second stream next to the forward pass)")
    ap.add_argument("--launch", choices=["graph", "stream"], default="graph",
                    help="graph: the steps are captured once in a HIP graph of POOL steps and replayed; "
                         "stream: every kernel is launched from Python")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run ten 256 MiB device-to-device copies (a kernel of known traffic, used to "
                         "scale the rocprofv3 FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only; --gpus %d is not supported "
                 "(no collectives or sharding are part of it)" % args.gpus)

    import numpy as np
    import torch
    from paper_2101_11714_amd import binding as B
    from paper_2101_11714_amd import workloads as W

    if args.pmc_means:
        pmc_means(args.pmc_means)
        return
    if args.trace_context:
        trace_context(args.trace_context)
        return
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)      # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": "10 copies", "bytes_read_per_copy": src.numel() * 4,
                          "bytes_written_per_copy": src.numel() * 4}))
        return
    wl = W.WORKLOADS[args.workload]
    tab = args.table
    t = wl.tables[tab]
    shape = B.shape_of(t)
    cores_h = W.make_cores(t, wl.init, wl.seed, tab)
    cores = [torch.from_numpy(c).to(dev) for c in cores_h]
    grads = [torch.zeros_like(c) for c in cores]
    batches_h = [W.make_batch(wl, tab, step, with_alpha=args.weights == "alpha") for step in range(POOL)]
    idx = [torch.from_numpy(b.indices).to(dev) for b in batches_h]
    off = [torch.from_numpy(b.offsets).to(dev) for b in batches_h]
    if args.offsets == "none":                          # the boundary's form for "one index per bag": no offsets array
        assert wl.bag_len == (1, 1), "--offsets none needs a workload with one index per bag"
        off = [None] * POOL
    go = [torch.from_numpy(b.grad_output).to(dev) for b in batches_h]
    n_bags = wl.n_bags
    Ls = [int(b.indices.size) for b in batches_h]       # bags of random length: the batches differ a little
    L = int(round(sum(Ls) / POOL))
    out = torch.empty((n_bags, t.dim), dtype=torch.float32, device=dev)
    lr = 1e-3 * wl.lr            # small, so that thousands of steps keep the cores finite
    # per-position weights: none, the batch's alpha, or the weights of mean pooling
    alpha = [None] * POOL
    if args.weights == "alpha":
        alpha = [torch.from_numpy(b.alpha).to(dev) for b in batches_h]
    elif args.weights == "mean":
        alpha = [B.tt_emb_mean_weights(off[j], n_bags, Ls[j], torch.empty(Ls[j], dtype=torch.float32, device=dev)) for j in range(POOL)]
    # the cache of the workloads that have one, filled from the counts of the warm-up stream
    K = W.cache_size(wl, tab)
    cache, grad_cache, keys_h = None, None, None
    if K:
        rows_h, counts_h = W.warmup_counts(wl, tab)
        cache = B.Cache(K, t.dim, dev)
        B.tt_cache_build(shape, cores, torch.from_numpy(rows_h).to(dev), torch.from_numpy(counts_h).to(dev), cache)
        grad_cache = torch.zeros_like(cache.rows)
        keys_h = cache.keys.cpu().numpy()
    ws = torch.empty(max(B.bwd_sgd_workspace_bytes(shape, max(Ls), n_bags, K), 256), dtype=torch.uint8, device=dev)

    cores2 = [torch.empty_like(c) for c in cores]      # the fused step writes the other set of cores
    keep_t0 = args.step == "fused" and not args.recompute
    # one stored intermediate per batch of the pool (1 MB each at Kaggle R = 32)
    t0_pool = [torch.empty((max(Ls[j], 1), B.t0_floats(shape)), dtype=torch.float32, device=dev) for j in range(POOL)] if keep_t0 else None

    # per-slice position lists filed ahead of the backward pass, where the library keeps them
    use_lists = keep_t0 and not args.no_lists and K == 0 and all(B.kept_has_lists(shape, x) for x in Ls)
    kept_pool = [torch.empty(B.kept_bytes(shape, Ls[j]), dtype=torch.uint8, device=dev) for j in range(POOL)] if use_lists else None

    def fwd_call(cur, j):
        if use_lists:
            B.tt_emb_fwd_keep(shape, cur, idx[j], off[j], n_bags, out, kept_pool[j], alpha=alpha[j], lists_ready=True)
        elif keep_t0:
            B.tt_emb_fwd_keep_t0(shape, cur, idx[j], off[j], n_bags, out, t0_pool[j], alpha=alpha[j], cache=cache)
        else:
            B.tt_emb_fwd(shape, cur, idx[j], off[j], n_bags, out, alpha=alpha[j], cache=cache)

    def bwd_sgd_call(cur, nxt, j, jn):
        """Backward + SGD of batch j; with lists, riders of the launch file the lists of batch jn (the next one)."""
        if use_lists:
            B.tt_emb_bwd_sgd_kept(shape, cur, nxt, idx[j], off[j], n_bags, go[j], kept_pool[j], lr, alpha=alpha[j],
                                  workspace=ws, next_batch=(idx[jn], kept_pool[jn]))
        else:
            B.tt_emb_bwd_sgd(shape, cur, nxt, idx[j], off[j], n_bags, go[j], lr, alpha=alpha[j], cache=cache,
                             workspace=ws, t0=t0_pool[j] if keep_t0 else None)

    assert POOL % 2 == 0                                # so that every graph replay starts on the same set

    # The index-only pre-pass of the backward (cache probe, grouping sort of long lists) runs on a second stream where
    # there is one.  Within a sequence of steps (the captured graph) the pre-pass of step i + 1 is enqueued behind the
    # forward pass of step i, so that it runs next to the backward pass of step i (the indices of the next batch are
    # known, as with a data loader that is one batch ahead); it needs a workspace of its own, two alternate.  A step on its own (first = last
    # = True) runs its pre-pass next to its forward pass.  The graph keeps the forks and the joins.
    two_calls = args.step == "fused" and not args.one_call and B.bwd_has_prepass(shape, max(Ls), K, keep_t0)
    fwd_lists = two_calls and all(B.fwd_uses_lists(shape, x, K, keep_t0) for x in Ls)
    side = torch.cuda.Stream() if two_calls else None
    ws_pair = [ws, torch.empty_like(ws)] if two_calls else [ws, ws]
    prepared_ev = [torch.cuda.Event(), torch.cuda.Event()] if two_calls else None

    def prepare_on_side(i):
        """Pre-pass of step i on the second stream, after everything enqueued on the current stream so far."""
        j = i % POOL
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            B.tt_emb_bwd_prepare(shape, idx[j], off[j], n_bags, cache=cache, workspace=ws_pair[i % 2], kept_t0=keep_t0)
            prepared_ev[i % 2].record(side)

    def step(i, first=True, last=True):
        j = i % POOL
        if args.step == "fused":
            cur, nxt = (cores, cores2) if i % 2 == 0 else (cores2, cores)
            if two_calls:
                if first:
                    prepare_on_side(i)
            if fwd_lists:
                # the forward pass works from the pre-pass's lists where the library has such a kernel (long streams)
                torch.cuda.current_stream().wait_event(prepared_ev[i % 2])
                B.tt_emb_fwd_prepared(shape, cur, idx[j], off[j], n_bags, out, ws_pair[i % 2], t0=t0_pool[j] if keep_t0 else None,
                                      alpha=alpha[j], cache=cache)
            else:
                fwd_call(cur, j)
            if two_calls and not last:
                prepare_on_side(i + 1)                      # next to this step's backward (measured: better than next to
            if two_calls:                                   # its forward); its workspace was last read by step i - 1
                if not fwd_lists:
                    torch.cuda.current_stream().wait_event(prepared_ev[i % 2])
                B.tt_emb_bwd_sgd(shape, cur, nxt, idx[j], off[j], n_bags, go[j], lr, alpha=alpha[j], cache=cache,
                                 workspace=ws_pair[i % 2], t0=t0_pool[j] if keep_t0 else None, prepared=True)
            else:
                # (a graph starts with batch 0 again: its last step files the lists of batch 0)
                bwd_sgd_call(cur, nxt, j, 0 if last else (j + 1) % POOL)
        else:
            B.tt_emb_fwd(shape, cores, idx[j], off[j], n_bags, out, alpha=alpha[j], cache=cache)
            B.tt_emb_bwd(shape, cores, idx[j], off[j], n_bags, go[j], grads, alpha=alpha[j], cache=cache,
                         grad_cache=grad_cache, workspace=ws)
            B.tt_emb_sgd_update(shape, cores, grads, lr, cache=cache, grad_cache=grad_cache, zero_grad=True)

    REPS = 5                                            # repetitions of every timed region: the median is reported

    def sync_time(fn):
        """ms between two events on the current stream around fn(), bracketed by synchronize() on both sides."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    def captured(fn, count, sequence=False):
        """A HIP graph of the consecutive calls fn(0..count-1); replay() launches all of them.
        sequence: fn is told which call is the first and which the last of the graph (see step)."""
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(count):
                if sequence:
                    fn(i, first=i == 0, last=i == count - 1)
                else:
                    fn(i)
        return g

    def runner(fn, count, sequence=False):
        """A function that enqueues EXACTLY count consecutive calls of fn: call by call, or as replays of a graph of
        POOL calls plus one replay of a graph of the count % POOL calls that remain."""
        if args.launch == "stream":
            def run():
                for i in range(count):
                    fn(i)
            return run
        whole, rest = divmod(count, POOL)
        g_pool = captured(fn, POOL, sequence) if whole else None
        g_rest = captured(fn, rest, sequence) if rest else None
        for g in (g_pool, g_rest):
            if g is not None:
                g.replay()                                  # first replay: untimed

        def run():
            for _ in range(whole):
                g_pool.replay()
            if g_rest is not None:
                g_rest.replay()
        return run

    def timed_ms(fn, count, sequence=False):
        """ms per call: REPS repetitions of exactly count calls each; returns (median, min, max)."""
        run = runner(fn, count, sequence)
        per = sorted(sync_time(run) / count for _ in range(REPS))
        return per[REPS // 2], per[0], per[-1]

    steps = max(1, args.steps)
    if use_lists:
        B.tt_emb_kept_prepare(shape, idx[0], kept_pool[0])
    for i in range(args.warmup):
        step(i, last=False)
    if use_lists:
        B.tt_emb_kept_prepare(shape, idx[0], kept_pool[0])  # every timed graph starts with batch 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms_step, ms_step_min, ms_step_max = timed_ms(step, steps, sequence=True)
    wall = time.perf_counter() - t0
    value = L / (ms_step * 1e-3)

    # per-kernel durations: each stage alone, launched back to back on the stream the step runs on
    reps = max(POOL * 16, min(steps, 4096))
    ws_stage, ms_prepass = None, None
    if two_calls:
        # the step runs the fused backward in its two-call form: the stages are timed in that form too, the index-only
        # pre-pass on its own (in the step it runs beside other work) and the rest on one prepared workspace per batch
        ms_prepass = timed_ms(lambda i: B.tt_emb_bwd_prepare(shape, idx[i % POOL], off[i % POOL], n_bags, cache=cache, workspace=ws,
                                                             kept_t0=keep_t0), reps)[0]
        ws_stage = [torch.empty_like(ws) for _ in range(POOL)]
        for j in range(POOL):
            B.tt_emb_bwd_prepare(shape, idx[j], off[j], n_bags, cache=cache, workspace=ws_stage[j], kept_t0=keep_t0)
    if fwd_lists:
        # the forward pass of the step works from the lists of the pre-pass
        ms_fwd = timed_ms(lambda i: B.tt_emb_fwd_prepared(shape, cores, idx[i % POOL], off[i % POOL], n_bags, out, ws_stage[i % POOL],
                                                          t0=t0_pool[i % POOL] if keep_t0 else None, alpha=alpha[i % POOL],
                                                          cache=cache), reps)[0]
    else:
        ms_fwd = timed_ms(lambda i: fwd_call(cores, i % POOL), reps)[0]
    if args.step == "fused":
        # (the forward timing above has left the T0 of every batch of the pool in t0_pool)
        if two_calls:
            ms_bs = timed_ms(lambda i: B.tt_emb_bwd_sgd(shape, cores, cores2, idx[i % POOL], off[i % POOL], n_bags, go[i % POOL], lr,
                                                        alpha=alpha[i % POOL], cache=cache, workspace=ws_stage[i % POOL],
                                                        t0=t0_pool[i % POOL] if keep_t0 else None, prepared=True), reps)[0]
        else:
            ms_bs = timed_ms(lambda i: bwd_sgd_call(cores, cores2, i % POOL, (i + 1) % POOL), reps)[0]
        stage_ms = {"fwd": ms_fwd, "bwd_sgd": ms_bs}
        del ws_stage
    else:
        ms_bwd = timed_ms(lambda i: B.tt_emb_bwd(shape, cores, idx[i % POOL], off[i % POOL], n_bags, go[i % POOL], grads,
                                                 alpha=alpha[i % POOL], cache=cache, grad_cache=grad_cache, workspace=ws), reps)[0]
        for g in grads:
            g.zero_()
        ms_sgd = timed_ms(lambda i: B.tt_emb_sgd_update(shape, cores, grads, 0.0, cache=cache, grad_cache=grad_cache,
                                                        zero_grad=True), reps)[0]
        stage_ms = {"fwd": ms_fwd, "bwd": ms_bwd, "sgd": ms_sgd}

    # what a launch costs before it computes anything: kernels that do nothing, one workgroup and as many as the backward
    # pass starts, in the same kind of sequence (the floor under every stage's time above)
    n_wg = t.m[0] + t.m[1] + t.m[2]
    launch_floor = {"1_workgroup": round(timed_ms(lambda i: B.tt_emb_debug_launch_probe(1), reps)[0] * 1e3, 3),
                    "%d_workgroups" % n_wg: round(timed_ms(lambda i: B.tt_emb_debug_launch_probe(n_wg), reps)[0] * 1e3, 3)}

    # the same step with Alg. 2's recomputation instead of the stored intermediate, beside the headline
    ms_recompute, ms_stored_t0 = None, None
    if keep_t0:
        def step_recompute(i):
            j = i % POOL
            cur, nxt = (cores, cores2) if i % 2 == 0 else (cores2, cores)
            B.tt_emb_fwd(shape, cur, idx[j], off[j], n_bags, out, alpha=alpha[j], cache=cache)
            B.tt_emb_bwd_sgd(shape, cur, nxt, idx[j], off[j], n_bags, go[j], lr, alpha=alpha[j], cache=cache, workspace=ws)
        ms_recompute = timed_ms(step_recompute, min(steps, 20 * POOL))[0]
    if use_lists:
        # ... and with the stored T0 but every slice owner scanning the index array itself (no lists filed ahead)
        def step_stored_t0(i):
            j = i % POOL
            cur, nxt = (cores, cores2) if i % 2 == 0 else (cores2, cores)
            B.tt_emb_fwd_keep_t0(shape, cur, idx[j], off[j], n_bags, out, t0_pool[j], alpha=alpha[j], cache=cache)
            B.tt_emb_bwd_sgd(shape, cur, nxt, idx[j], off[j], n_bags, go[j], lr, alpha=alpha[j], cache=cache, workspace=ws,
                             t0=t0_pool[j])
        ms_stored_t0 = timed_ms(step_stored_t0, min(steps, 20 * POOL))[0]

    # touched slices of one batch (host arithmetic on the synthetic indices, for the byte model only)
    b0 = batches_h[0].indices
    m1, m2, m3 = t.m
    touched = (np.unique(b0 // (m2 * m3)).size * t.n[0] * t.r[1]
               + np.unique((b0 // m3) % m2).size * t.r[1] * t.n[1] * t.r[2]
               + np.unique(b0 % m3).size * t.r[2] * t.n[2])
    n_cached = int(np.isin(b0, keys_h).sum()) if keys_h is not None else 0
    ab = algorithmic_bytes(t, Ls[0], n_bags, touched, n_cached)
    af = algorithmic_flops(t, Ls[0] - n_cached, keep_t0)
    # the stored intermediate is written once and read once per uncached lookup: an intermediate, not part of the
    # method's algorithmic bytes, reported beside them
    kept_bytes = (Ls[0] - n_cached) * 4 * B.t0_floats(shape) if keep_t0 else 0
    list_bytes = 3 * Ls[0] * 16 if use_lists else 0      # one 16-byte list entry per position and core
    dominant = max(stage_ms, key=stage_ms.get)
    variant = "lists" if use_lists else ("two_calls" if two_calls else ("keep_t0" if keep_t0 else ("recompute" if args.step == "fused" else "separate")))
    # the time the roofline figures are taken over: the dominant stage, and where that is the backward in two calls, its
    # index-only first call as well (the step hides it beside other work, but it is work of the backward pass)
    roof_ms = stage_ms[dominant] + (ms_prepass if (ms_prepass is not None and dominant == "bwd_sgd") else 0.0)
    achieved = ab[dominant] / (roof_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(args.workload, tab, variant, dominant),
                "traffic_source": "profiles/hbm_traffic_table.md, row (%s, %d, %s, %s)" % (args.workload, tab, variant, dominant),
                "algorithmic_bytes": ab[dominant], "kept_intermediate_bytes": kept_bytes, "kept_list_bytes": list_bytes,
                "avg_us": round(roof_ms * 1e3, 3),
                "stages_us": {k: round(v * 1e3, 3) for k, v in stage_ms.items()},
                "prepass_us": None if ms_prepass is None else round(ms_prepass * 1e3, 3),
                "launch_floor_us": launch_floor,
                "stages_frac": {k: round(ab[k] / (stage_ms[k] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) for k in stage_ms},
                "fp32_tflops": round(af[dominant] / (roof_ms * 1e-3) / 1e12, 3),
                "fp32_frac": round(af[dominant] / (roof_ms * 1e-3) / 1e12 / FP32_PEAK_TFLOPS, 5),
                "cache_hit_rate": round(n_cached / Ls[0], 4) if keys_h is not None else None}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import tt_oracle as ora
        oshape = ora.Shape.of(t)
        budget, done, spent = 10.0, 0, 0.0
        oc = [c.copy() for c in cores_h]
        crow = ora.cache_fill(oshape, oc, keys_h) if keys_h is not None else None
        al_h = [None if a is None else a.cpu().numpy() for a in alpha]
        while done < 1 or (spent < budget and done < 64 * POOL):       # about 10 s of CPU work, cycling through the pool
            b = batches_h[done % POOL]
            s0 = time.perf_counter()
            ora.fwd(oshape, oc, b.indices, b.offsets, alpha=al_h[done % POOL], cache_keys=keys_h, cache_rows=crow)
            dg, dc = ora.bwd(oshape, oc, b.indices, b.offsets, b.grad_output, alpha=al_h[done % POOL], cache_keys=keys_h)
            oc = [ora.sgd(oc[k], dg[k].astype(np.float32), lr) for k in range(3)]
            if crow is not None:
                crow = ora.sgd(crow, dc.astype(np.float32), lr)
            spent += time.perf_counter() - s0
            done += 1
        cpu = {"value": round(done * L / spent, 1), "unit": "lookups/s", "cores": 1, "kind": "oracle",
               "sample": "%d whole steps (fwd+bwd+sgd) over the same pool of %d-lookup batches, %.1f s, single thread, fp64"
                         % (done, L, spent)}
        # secondary figure: the forward pass alone, on one thread and with the bags shared out among the host threads
        # this process may use (the backward keeps its one defined accumulation order, so it stays on one thread)
        want = int(os.environ.get("OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0))

        def fwd_rate(threads):
            n, t_spent, ran = 0, 0.0, 1
            while n < 1 or (t_spent < 3.0 and n < 256 * POOL):
                b = batches_h[n % POOL]
                s0 = time.perf_counter()
                if threads == 1:
                    ora.fwd(oshape, oc, b.indices, b.offsets, alpha=al_h[n % POOL], cache_keys=keys_h, cache_rows=crow)
                else:
                    ran = ora.fwd_threads(oshape, oc, b.indices, b.offsets, threads, alpha=al_h[n % POOL], cache_keys=keys_h,
                                          cache_rows=crow)[1]
                t_spent += time.perf_counter() - s0
                n += 1
            return round(n * L / t_spent, 1), ran, n

        f1, _, n1 = fwd_rate(1)
        fn, ran, nn = fwd_rate(want)
        cpu["forward_only"] = {"value": f1, "unit": "lookups/s", "cores": 1, "sample": "%d forward passes, single thread" % n1}
        cpu["forward_only_openmp"] = {"value": fn, "unit": "lookups/s", "cores": ran,
                                      "sample": "%d forward passes, bags shared out among %d threads, results bit-identical "
                                                "to the single thread's" % (nn, ran)}

    print(json.dumps({
        "metric": "TT-EmbeddingBag fwd+bwd lookups/sec; % of HBM/fp32 roofline at R=32",
        "value": round(value, 1), "unit": "lookups/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 6), "ms_per_step_min_max": [round(ms_step_min, 6), round(ms_step_max, 6)],
        "repetitions": REPS, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %d rows as %dx%dx%d, dim %d as %dx%dx%d, ranks (1,%d,%d,1), %d bags x %d index, "
                               "Zipf(%.2f)%s%s, fwd+bwd+SGD" % (wl.name, t.num_rows, *t.m, t.dim, *t.n, t.r[1], t.r[2],
                                                                n_bags, L // max(n_bags, 1), wl.zipf_alpha,
                                                                ", cache of %d rows" % K if K else "",
                                                                ", weights: %s" % args.weights if args.weights != "none" else ""),
                   "table": tab,
                   "lookups_per_step": L, "launch": args.launch, "step": args.step, "keep_t0": bool(keep_t0),
                   "prepass_on_second_stream": bool(two_calls), "prepass_one_step_ahead": bool(two_calls and args.launch == "graph"), "wall_s_timed_region": round(wall, 3),
                   "lists_filed_ahead": bool(use_lists), "forward_from_prepass_lists": bool(fwd_lists),
                   "ms_per_step_recompute": None if ms_recompute is None else round(ms_recompute, 6),
                   "ms_per_step_stored_t0_without_lists": None if ms_stored_t0 is None else round(ms_stored_t0, 6)},
        "roofline": roofline, "cpu_baseline": cpu}))


if __name__ == "__main__":
    main()
