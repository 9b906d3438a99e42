"""ctypes wrapper around the CPU oracle (oracle/tt_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product path never imports this module, and
this module imports nothing from the HIP package.
"""

from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tt_oracle.c")
_LIB = os.path.join(_HERE, "libtt_oracle.so")


_LIB_SAN = os.path.join(_HERE, "libtt_oracle_san.so")


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no intrinsics, no fast-math).  sanitize: a second library with the address
    and undefined-behaviour sanitizers, for a process that has their runtime preloaded (see TT_ORACLE_SANITIZE)."""
    lib = _LIB_SAN if sanitize else _LIB
    stale = (not os.path.exists(lib)) or os.path.getmtime(lib) < os.path.getmtime(_SRC)
    if force or stale:
        flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                 "-fno-omit-frame-pointer"] if sanitize else ["-O2"]
        tmp = "%s.%d.tmp" % (lib, os.getpid())
        subprocess.check_call(["gcc"] + flags + ["-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, lib)
    return lib


_lib = None


def _load():
    """The compiled oracle.  With TT_ORACLE_SANITIZE=1 in the environment: its sanitizer build (the process must have
    been started with the sanitizer runtime preloaded)."""
    global _lib
    if _lib is None:
        _lib = C.CDLL(build(sanitize=os.environ.get("TT_ORACLE_SANITIZE") == "1"))
        _lib.ora_param_count.restype = C.c_int64
        _lib.ora_dedup.restype = C.c_int64
    return _lib


def _i64x(values: Sequence[int]):
    return (C.c_int64 * len(values))(*[int(v) for v in values])


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


class Shape:
    """Row / column factorisations and ranks of one table (Section 2, Eq. 2)."""

    def __init__(self, num_rows: int, m, n, r):
        self.num_rows = int(num_rows)
        self.m = tuple(int(x) for x in m)
        self.n = tuple(int(x) for x in n)
        self.r = tuple(int(x) for x in r)
        assert len(self.m) == 3 and len(self.n) == 3 and len(self.r) == 4
        assert self.r[0] == 1 and self.r[3] == 1
        assert self.m[0] * self.m[1] * self.m[2] >= self.num_rows

    @classmethod
    def of(cls, s) -> "Shape":
        return cls(s.num_rows, s.m, s.n, s.r)

    @property
    def dim(self) -> int:
        return self.n[0] * self.n[1] * self.n[2]

    def core_size(self, k: int) -> int:
        return self.m[k] * self.r[k] * self.n[k] * self.r[k + 1]

    def c(self):
        return _i64x(self.m), _i64x(self.n), _i64x(self.r)


def param_count(shape: Shape) -> int:
    m, n, r = shape.c()
    return int(_load().ora_param_count(m, n, r))


def decode(shape: Shape, indices) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    idx = _i64(indices)
    out = [np.empty(idx.size, dtype=np.int32) for _ in range(3)]
    m, _, _ = shape.c()
    _load().ora_decode(m, _p(idx), C.c_int64(idx.size), _p(out[0]), _p(out[1]), _p(out[2]))
    return out[0], out[1], out[2]


def row(shape: Shape, cores: List[np.ndarray], row_id: int) -> np.ndarray:
    g = [_f32(c) for c in cores]
    out = np.empty(shape.dim, dtype=np.float64)
    m, n, r = shape.c()
    _load().ora_row(m, n, r, _p(g[0]), _p(g[1]), _p(g[2]), C.c_int64(int(row_id)), _p(out))
    return out


def cache_select(cand_rows, cand_counts, K: int) -> np.ndarray:
    rows, counts = _i64(cand_rows), _i64(cand_counts)
    assert rows.size == counts.size and 0 <= K <= rows.size
    keys = np.empty(K, dtype=np.int64)
    rc = _load().ora_cache_select(_p(rows), _p(counts), C.c_int64(rows.size), C.c_int64(K), _p(keys))
    assert rc == 0
    return keys


def cache_fill(shape: Shape, cores, keys) -> np.ndarray:
    g = [_f32(c) for c in cores]
    keys = _i64(keys)
    rows = np.empty((keys.size, shape.dim), dtype=np.float32)
    m, n, r = shape.c()
    _load().ora_cache_fill(m, n, r, _p(g[0]), _p(g[1]), _p(g[2]), _p(keys), C.c_int64(keys.size), _p(rows))
    return rows


def cache_lookup(shape: Shape, keys, indices) -> np.ndarray:
    keys, idx = _i64(keys), _i64(indices)
    slot = np.empty(idx.size, dtype=np.int32)
    rc = _load().ora_cache_lookup(C.c_int64(shape.num_rows), _p(keys), C.c_int64(keys.size),
                                  _p(idx), C.c_int64(idx.size), _p(slot))
    assert rc == 0
    return slot


def _check_csr(shape: Shape, indices: np.ndarray, offsets: np.ndarray):
    assert offsets.ndim == 1 and offsets.size >= 1
    assert offsets[0] == 0 and offsets[-1] == indices.size
    assert np.all(np.diff(offsets) >= 0)
    if indices.size:
        assert indices.min() >= 0 and indices.max() < shape.num_rows, "index out of range"


def fwd(shape: Shape, cores, indices, offsets, alpha=None, cache_keys=None, cache_rows=None) -> np.ndarray:
    g = [_f32(c) for c in cores]
    idx, off = _i64(indices), _i64(offsets)
    _check_csr(shape, idx, off)
    n_bags = off.size - 1
    a = None if alpha is None else _f32(alpha)
    K = 0 if cache_keys is None else int(np.asarray(cache_keys).size)
    ck = None if K == 0 else _i64(cache_keys)
    cr = None if K == 0 else _f32(cache_rows)
    out = np.empty((n_bags, shape.dim), dtype=np.float32)
    m, n, r = shape.c()
    rc = _load().ora_fwd(m, n, r, C.c_int64(shape.num_rows), _p(g[0]), _p(g[1]), _p(g[2]),
                         _p(idx), C.c_int64(idx.size), _p(off), C.c_int64(n_bags), _p(a),
                         _p(ck), _p(cr), C.c_int64(K), _p(out))
    assert rc == 0
    return out


def fwd_threads(shape: Shape, cores, indices, offsets, threads: int, alpha=None, cache_keys=None, cache_rows=None):
    """fwd with the bags shared out among host threads: (output, threads that ran).  Bit-identical to fwd."""
    g = [_f32(c) for c in cores]
    idx, off = _i64(indices), _i64(offsets)
    _check_csr(shape, idx, off)
    n_bags = off.size - 1
    a = None if alpha is None else _f32(alpha)
    K = 0 if cache_keys is None else int(np.asarray(cache_keys).size)
    ck = None if K == 0 else _i64(cache_keys)
    cr = None if K == 0 else _f32(cache_rows)
    out = np.empty((n_bags, shape.dim), dtype=np.float32)
    m, n, r = shape.c()
    ran = _load().ora_fwd_threads(m, n, r, C.c_int64(shape.num_rows), _p(g[0]), _p(g[1]), _p(g[2]),
                                  _p(idx), C.c_int64(idx.size), _p(off), C.c_int64(n_bags), _p(a),
                                  _p(ck), _p(cr), C.c_int64(K), _p(out), C.c_int(int(threads)))
    assert ran >= 1
    return out, int(ran)


def bwd(shape: Shape, cores, indices, offsets, grad_output, alpha=None, cache_keys=None):
    """Returns ([dG1, dG2, dG3] in fp64 with the cores' shapes, dCache fp64 [K][N] or None)."""
    g = [_f32(c) for c in cores]
    idx, off = _i64(indices), _i64(offsets)
    _check_csr(shape, idx, off)
    n_bags = off.size - 1
    go = _f32(grad_output)
    assert go.shape == (n_bags, shape.dim)
    a = None if alpha is None else _f32(alpha)
    K = 0 if cache_keys is None else int(np.asarray(cache_keys).size)
    ck = None if K == 0 else _i64(cache_keys)
    dG = [np.zeros(g[k].shape, dtype=np.float64) for k in range(3)]
    dC = None if K == 0 else np.zeros((K, shape.dim), dtype=np.float64)
    m, n, r = shape.c()
    rc = _load().ora_bwd(m, n, r, C.c_int64(shape.num_rows), _p(g[0]), _p(g[1]), _p(g[2]),
                         _p(idx), C.c_int64(idx.size), _p(off), C.c_int64(n_bags), _p(a),
                         _p(ck), C.c_int64(K), _p(go),
                         _p(dG[0]), _p(dG[1]), _p(dG[2]), _p(dC))
    assert rc == 0
    return dG, dC


def sgd(x: np.ndarray, g: np.ndarray, lr: float) -> np.ndarray:
    """Returns x - lr * g, evaluated in fp64 and rounded to fp32."""
    out = _f32(x).copy()
    gg = _f32(g)
    assert out.shape == gg.shape
    _load().ora_sgd(_p(out), _p(gg), C.c_int64(out.size), C.c_double(float(lr)))
    return out


def dedup(keys) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(ascending unique keys, counts, grouping permutation); keys < 0 are skipped."""
    k = _i64(keys)
    uniq = np.empty(k.size, dtype=np.int64)
    count = np.empty(k.size, dtype=np.int32)
    perm = np.empty(k.size, dtype=np.int32)
    kept = C.c_int64(0)
    u = int(_load().ora_dedup(_p(k), C.c_int64(k.size), _p(uniq), _p(count), _p(perm), C.byref(kept)))
    return uniq[:u].copy(), count[:u].copy(), perm[:kept.value].copy()


# ---- access-frequency tracking and the semi-dynamic cache (Section 4.2) -------------------
# Plain Python on purpose: a dictionary row -> number of accesses is the definition of what the
# open-addressing hash table of the paper holds.

def freq_update(counts: dict, indices) -> dict:
    """Add the accesses of one index stream to the running counts (in place, also returned)."""
    for i in _i64(indices).tolist():
        counts[i] = counts.get(i, 0) + 1
    return counts


def freq_export(counts: dict) -> Tuple[np.ndarray, np.ndarray]:
    """(rows, counts) of every tracked row, ascending by row."""
    rows = np.array(sorted(counts), dtype=np.int64)
    return rows, np.array([counts[int(r)] for r in rows], dtype=np.int64)


def cache_refill(shape: Shape, cores, old_keys, old_rows, cand_rows, cand_counts, K: int):
    """One refill of the semi-dynamic cache: the K most used candidates become the cached set
    (same order rule as cache_select).  A row that was cached before keeps its line, with the
    weights it has learned; a row that enters is initialised from the cores; what an evicted
    line has learned is dropped.  Returns (keys, rows)."""
    old_keys = _i64(old_keys)
    old_rows = np.asarray(old_rows, dtype=np.float32).reshape(old_keys.size, shape.dim)
    where = {int(k): s for s, k in enumerate(old_keys.tolist())}
    keys = cache_select(cand_rows, cand_counts, K)
    rows = np.empty((K, shape.dim), dtype=np.float32)
    for s, k in enumerate(keys.tolist()):
        rows[s] = old_rows[where[k]] if k in where else row(shape, cores, k)
    return keys, rows


# ---- stored intermediate of the forward pass (Section 4.2, first paragraph) ----------------

def t0(shape: Shape, cores, row_id: int) -> np.ndarray:
    """The product of the first two core slices of a row, T0 = A . Bm reshaped to (n1 n2) x R2
    (Section 3.1): the tensor that Alg. 2 recomputes in the backward pass unless the forward
    pass has kept it.  fp64; row = T0 . C."""
    i1, i2, _ = (int(x[0]) for x in decode(shape, [row_id]))
    n1, n2, _ = shape.n
    _, R1, R2, _ = shape.r
    A = np.asarray(cores[0], dtype=np.float64).reshape(shape.m[0], n1, R1)[i1]
    Bm = np.asarray(cores[1], dtype=np.float64).reshape(shape.m[1], R1, n2 * R2)[i2]
    return (A @ Bm).reshape(n1 * n2, R2)


def kept_lists(shape: Shape, indices, cached=None, chunk: Optional[int] = None):
    """What the per-slice lists of a forward pass that keeps them must say about every position k (the grouping
    that Alg. 2's "+=" into core slices implies, Section 3.1's digits): slice[r][k] = digit r of indices[k], and
    rep[k] = the first position k' <= k of the same chunk of `chunk` consecutive positions with indices[k'] ==
    indices[k] (cached positions, cached[k] true, are in no list: -1 and never a rep).  chunk defaults to
    256.  Returns (slice int32 [3][L], rep int32 [L])."""
    idx = np.asarray(indices, dtype=np.int64)
    L = idx.size
    if chunk is None:
        chunk = 256
    digits = decode(shape, idx)
    sl = np.stack([np.asarray(d, dtype=np.int32) for d in digits])
    rep = np.full(L, -1, dtype=np.int32)
    for lo in range(0, L, chunk):
        first = {}
        for k in range(lo, min(L, lo + chunk)):
            if cached is not None and cached[k]:
                continue
            r = int(idx[k])
            if r not in first:
                first[r] = k
            rep[k] = first[r]
    if cached is not None:
        sl[:, np.asarray(cached, dtype=bool)] = -1
    return sl, rep


# ---- mean pooling (Section 4.1: a bag is pooled by summation or by averaging) --------------

def mean_weights(offsets, alpha=None) -> np.ndarray:
    """Per-position weights that turn the weighted sum of Eq. 5 into the bag average:
    w[k] = alpha[k] / (number of positions of the bag of k)."""
    offsets = _i64(offsets)
    L = int(offsets[-1])
    w = np.ones(L, dtype=np.float64) if alpha is None else np.asarray(alpha, dtype=np.float64).copy()
    for b in range(offsets.size - 1):
        lo, hi = int(offsets[b]), int(offsets[b + 1])
        if hi > lo:
            w[lo:hi] /= float(hi - lo)
    return w.astype(np.float32)


# ---- sampled Gaussian initialisation (Section 3.2, Alg. 3) ---------------------------------

def sampled_gaussian_scale(shape: Shape) -> float:
    l = _load()
    l.ora_sampled_gaussian_scale.restype = C.c_double
    return float(l.ora_sampled_gaussian_scale(C.c_int64(shape.num_rows), C.c_int(shape.r[1]), C.c_int(shape.r[2])))


def sampled_gaussian_draw(seed: int, core: int, element: int) -> Tuple[float, int]:
    """One accepted N(0,1) draw with |z| > 2 and the number of attempts it took."""
    l = _load()
    l.ora_sampled_gaussian_draw.restype = C.c_double
    att = C.c_int(0)
    z = l.ora_sampled_gaussian_draw(C.c_uint64(seed), C.c_int(core), C.c_uint64(element), C.byref(att))
    return float(z), int(att.value)


def init_sampled_gaussian(shape: Shape, seed: int) -> List[np.ndarray]:
    """The three cores after Alg. 3 (flat fp32 arrays in storage order)."""
    scale = sampled_gaussian_scale(shape)
    cores = []
    for k in range(3):
        out = np.empty(shape.core_size(k), dtype=np.float32)
        _load().ora_init_sampled_gaussian(C.c_uint64(seed), C.c_int(k), C.c_int64(out.size), C.c_double(scale), _p(out))
        cores.append(out)
    return cores


# ---- general number of cores (Section 4.1: "can be generalized to any arbitrary TT dimension") --
# Plain numpy, fp64.  A shape is (num_rows, m[d], n[d], r[d+1]) with r[0] = r[d] = 1; core k is
# stored [m_k][r_k][n_k][r_{k+1}] like the three-core case.

def _digits_d(m, i: int):
    out = []
    for mk in reversed(m):
        out.append(i % mk)
        i //= mk
    return out[::-1]


def _slices_d(m, n, r, cores, i: int):
    d = len(m)
    dig = _digits_d(m, i)
    return [np.asarray(cores[k], dtype=np.float64).reshape(m[k], r[k], n[k], r[k + 1])[dig[k]] for k in range(d)]


def row_d(m, n, r, cores, i: int) -> np.ndarray:
    """Row i of the table: the chain of Eq. 3 over d cores, partial products reshaped row-major."""
    sl = _slices_d(m, n, r, cores, i)
    p = sl[0].reshape(n[0], r[1])                                  # (n1) x R1
    for k in range(1, len(m)):
        p = (p @ sl[k].reshape(r[k], n[k] * r[k + 1])).reshape(-1, r[k + 1])
    return p.reshape(-1)


def fwd_d(m, n, r, cores, indices, offsets, alpha=None) -> np.ndarray:
    idx, off = _i64(indices), _i64(offsets)
    N = int(np.prod(n))
    out = np.zeros((off.size - 1, N))
    for b in range(off.size - 1):
        for k in range(int(off[b]), int(off[b + 1])):
            out[b] += (1.0 if alpha is None else float(alpha[k])) * row_d(m, n, r, cores, int(idx[k]))
    return out.astype(np.float32)


def bwd_d(m, n, r, cores, indices, offsets, grad_output, alpha=None) -> List[np.ndarray]:
    """Gradients of <output, grad_output> with respect to every core (Eq. 4 for any d): for the slice
    of core k used by a lookup, dG_k[a][j_k][b] = sum over the other column digits of
    left[j_<k][a] * dY[j_<k, j_k, j_>k] * right[b][j_>k], left / right being the products of the
    slices before / after core k."""
    d = len(m)
    idx, off = _i64(indices), _i64(offsets)
    go = np.asarray(grad_output, dtype=np.float64)
    grads = [np.zeros((m[k], r[k], n[k], r[k + 1])) for k in range(d)]
    for b in range(off.size - 1):
        for pos in range(int(off[b]), int(off[b + 1])):
            i = int(idx[pos])
            dig = _digits_d(m, i)
            sl = _slices_d(m, n, r, cores, i)
            dY = (1.0 if alpha is None else float(alpha[pos])) * go[b]
            for k in range(d):
                left = np.ones((1, 1))                              # (prod n_<k) x r_k
                for q in range(k):
                    left = (left @ sl[q].reshape(r[q], n[q] * r[q + 1])).reshape(-1, r[q + 1])
                right = np.ones((1, 1))                             # r_{k+1} x (prod n_>k)
                for q in range(d - 1, k, -1):
                    right = (sl[q].reshape(r[q] * n[q], r[q + 1]) @ right).reshape(r[q], -1)
                nl, nr = left.shape[0], right.shape[1]
                dy3 = dY.reshape(nl, n[k], nr)
                grads[k][dig[k]] += np.einsum("la,ljr,br->ajb", left, dy3, right)
    return [g.astype(np.float32) for g in grads]
