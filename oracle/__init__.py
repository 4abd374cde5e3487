"""ctypes front-end of the CPU oracle (``moe_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's ``cpu_baseline``
leg may import this package; the GPU library and its binding never do.  Nothing in here
shares code with the GPU path.

All array arguments are NumPy arrays; floating-point inputs are float32 (bf16 values
widened exactly by the caller), every result is float64 / int32 / int64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``moe_oracle.c`` with gcc (-O2, OpenMP over tokens) into ``libmoe_oracle.so``."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    """The compiled oracle.  MOE_ORACLE_LIBRARY names another build of it to load instead: the
    mutation test compiles copies of moe_oracle.c with one planted mistake each and runs the pins
    against them."""
    global _lib
    if _lib is None:
        other = os.environ.get("MOE_ORACLE_LIBRARY")
        if other:
            _lib = ctypes.CDLL(other)
        else:
            build()
            _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a, ctype):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctype))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


c_f, c_d, c_i32, c_i64 = ctypes.c_float, ctypes.c_double, ctypes.c_int32, ctypes.c_int64


def threads() -> int:
    """Number of OpenMP threads the token-parallel loops use."""
    n = os.environ.get("OMP_NUM_THREADS")
    if n:
        return int(n)
    return len(os.sched_getaffinity(0))


def gate_logits(x, wg):
    x, wg = _f32(x), _f32(wg)
    T, d = x.shape
    E = wg.shape[0]
    assert wg.shape[1] == d
    out = np.empty((T, E), dtype=np.float64)
    _load().ref_gate_logits(_p(x, c_f), _p(wg, c_f), c_i64(T), d, E, _p(out, c_d))
    return out


def softmax(logits):
    logits = _f64(logits)
    T, E = logits.shape
    out = np.empty((T, E), dtype=np.float64)
    _load().ref_softmax(_p(logits, c_d), c_i64(T), E, _p(out, c_d))
    return out


def topk(logits, k, renormalize):
    logits = _f64(logits)
    T, E = logits.shape
    assert 1 <= k <= min(E, 8)
    idx = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float64)
    _load().ref_topk(_p(logits, c_d), c_i64(T), E, k, int(bool(renormalize)), _p(idx, c_i32), _p(w, c_d))
    return idx, w


def dispatch(topk_idx, expert_map, E, E_local):
    """Returns dict(src_of_sorted[kept], sorted_of_src[A], counts, offsets, n_invalid)."""
    topk_idx = _i32(topk_idx)
    T, k = topk_idx.shape
    A = T * k
    em = None if expert_map is None else _i32(expert_map)
    if em is not None:
        assert em.shape == (E,)
    src = np.full(A, -1, dtype=np.int32)
    inv = np.empty(A, dtype=np.int32)
    counts = np.empty(E_local, dtype=np.int32)
    offsets = np.empty(E_local + 1, dtype=np.int32)
    n_invalid = np.zeros(1, dtype=np.int64)
    fn = _load().ref_dispatch
    fn.restype = c_i64
    kept = fn(_p(topk_idx, c_i32), _p(em, c_i32), c_i64(T), k, E, E_local, _p(src, c_i32),
              _p(inv, c_i32), _p(counts, c_i32), _p(offsets, c_i32), _p(n_invalid, c_i64))
    return dict(src_of_sorted=src[:kept].copy(), sorted_of_src=inv, counts=counts, offsets=offsets,
                n_invalid=int(n_invalid[0]), kept=int(kept))


def gather_rows(x, src_of_sorted, k):
    x = _f32(x)
    src = _i32(src_of_sorted)
    d = x.shape[1]
    out = np.empty((src.shape[0], d), dtype=np.float32)
    _load().ref_gather_rows(_p(x, c_f), _p(src, c_i32), c_i64(src.shape[0]), k, d, _p(out, c_f))
    return out


def expert_ffn_rows(x_sorted, offsets, w1, b1, w2, b2, act, rows):
    """FFN output (float64 [len(rows), d]) of the listed sorted rows."""
    x_sorted, w1, w2 = _f32(x_sorted), _f32(w1), _f32(w2)
    offsets = _i32(offsets)
    rows = _i64(rows)
    E_local, f, d = w1.shape
    assert w2.shape == (E_local, d, f) and x_sorted.shape[1] == d and offsets.shape == (E_local + 1,)
    if rows.size:
        assert rows.min() >= 0 and rows.max() < x_sorted.shape[0]
    b1 = None if b1 is None else _f32(b1)
    b2 = None if b2 is None else _f32(b2)
    y = np.empty((rows.shape[0], d), dtype=np.float64)
    _load().ref_expert_ffn_rows(_p(x_sorted, c_f), _p(offsets, c_i32), _p(w1, c_f), _p(b1, c_f),
                                _p(w2, c_f), _p(b2, c_f), d, f, E_local, int(act), _p(rows, c_i64),
                                c_i64(rows.shape[0]), _p(y, c_d))
    return y


def expert_ffn(x_sorted, offsets, w1, b1, w2, b2, act):
    return expert_ffn_rows(x_sorted, offsets, w1, b1, w2, b2, act, np.arange(np.asarray(x_sorted).shape[0]))


def combine(y_sorted, sorted_of_src, topk_w):
    y_sorted = _f64(y_sorted)
    topk_w = _f64(topk_w)
    inv = _i32(sorted_of_src).reshape(-1)
    T, k = topk_w.shape
    d = y_sorted.shape[1]
    assert inv.shape[0] == T * k
    if inv.size:
        assert inv.max() < y_sorted.shape[0]
    out = np.empty((T, d), dtype=np.float64)
    _load().ref_combine(_p(y_sorted, c_d), _p(inv, c_i32), _p(topk_w, c_d), c_i64(T), d, k, _p(out, c_d))
    return out


def affinity_counts(trace, E):
    """Returns (counts int64 [L-1,E,E], loads int64 [L,E], n_invalid)."""
    trace = _i32(trace)
    L, N = trace.shape
    counts = np.zeros((max(L - 1, 0), E, E), dtype=np.int64)
    loads = np.zeros((L, E), dtype=np.int64)
    n_invalid = np.zeros(1, dtype=np.int64)
    _load().ref_affinity_counts(_p(trace, c_i32), L, c_i64(N), E, _p(counts, c_i64), _p(loads, c_i64),
                                _p(n_invalid, c_i64))
    return counts, loads, int(n_invalid[0])


def cond_prob(counts):
    counts = _i64(counts)
    Lm1, E, _ = counts.shape
    prob = np.zeros((Lm1, E, E), dtype=np.float64)
    _load().ref_cond_prob(_p(counts, c_i64), Lm1 + 1, E, _p(prob, c_d))
    return prob


def placement_locality(trace, placement):
    trace = _i32(trace)
    placement = _i32(placement)
    L, N = trace.shape
    E = placement.shape[1]
    assert placement.shape[0] == L
    out = np.zeros(max(L - 1, 0), dtype=np.int64)
    _load().ref_placement_locality(_p(trace, c_i32), _p(placement, c_i32), L, c_i64(N), E, _p(out, c_i64))
    return out


def placement_locality_from_counts(counts, placement):
    counts = _i64(counts)
    placement = _i32(placement)
    Lm1, E, _ = counts.shape
    assert placement.shape == (Lm1 + 1, E)
    out = np.zeros(Lm1, dtype=np.int64)
    _load().ref_placement_locality_from_counts(_p(counts, c_i64), _p(placement, c_i32), Lm1 + 1, E,
                                               _p(out, c_i64))
    return out


def multihop_pair_index(L, l, m):
    """Position of the layer pair (l, m), l < m, in the source-layer-first order."""
    assert 0 <= l < m < L
    return l * L - l * (l + 1) // 2 + (m - l - 1)


def affinity_counts_multihop(trace, E):
    """counts int64 [L(L-1)/2, E, E] for every ordered layer pair l < m (source layer first)."""
    trace = _i32(trace)
    L, N = trace.shape
    counts = np.zeros((L * (L - 1) // 2, E, E), dtype=np.int64)
    _load().ref_affinity_counts_multihop(_p(trace, c_i32), L, c_i64(N), E, _p(counts, c_i64))
    return counts


def routing_away(trace, placement, home):
    """away int64 [L]: tokens whose layer-l expert sits on another GPU than their request's home."""
    trace = _i32(trace)
    placement = _i32(placement)
    home = _i32(home)
    L, N = trace.shape
    E = placement.shape[1]
    assert placement.shape[0] == L and home.shape == (N,)
    out = np.zeros(L, dtype=np.int64)
    _load().ref_routing_away(_p(trace, c_i32), _p(placement, c_i32), _p(home, c_i32), L, c_i64(N), E, _p(out, c_i64))
    return out


def comm_volume(G, N, L, p, p_star):
    """Forward communication volumes of the paper's comparison table, in tokens:
    (vanilla top-1, vanilla top-2, coherent top-1, coherent top-2)."""
    vol = np.zeros(4, dtype=np.float64)
    _load().ref_comm_volume(int(G), c_i64(int(N)), int(L), c_d(p), c_d(p_star), _p(vol, c_d))
    return vol


def transfer_ratios(trace, placement, home):
    """(p, p_star) of a clean trace: the share of (token, layer) visits that leave home (vanilla) and
    the share at which a coherent context moves."""
    trace = _i32(trace)
    placement = _i32(placement)
    home = _i32(home)
    L, N = trace.shape
    E = placement.shape[1]
    assert placement.shape[0] == L and home.shape == (N,)
    assert trace.min() >= 0 and trace.max() < E
    r = np.zeros(2, dtype=np.float64)
    _load().ref_transfer_ratios(_p(trace, c_i32), _p(placement, c_i32), _p(home, c_i32), L, c_i64(N), E, _p(r, c_d))
    return float(r[0]), float(r[1])


# --------------------------------------------------------------------------- placement search
# Design, "Solving Affinity's duality by Integer Programming": minimise the number of crossing
# transitions sum_k sum_j R_{k,j} subject to load balance (every part holds E/P experts of every
# layer) and exclusivity (every expert on exactly one part).  In terms of the co-routing counts the
# objective is  total - sum_l sum_{i,p} counts[l][i][p] * [part_l(i) == part_{l+1}(p)],  so the
# optimum MAXIMISES the local transitions.  The functions below enumerate; they are for tiny cases.
def balanced_partitions(E, P):
    """All maps expert -> part in [0,P) with exactly E/P experts per part (labelled parts)."""
    import itertools

    assert E % P == 0
    cap = E // P
    out = []

    def rec(e, cur, left):
        if e == E:
            out.append(tuple(cur))
            return
        for p in range(P):
            if left[p] > 0:
                left[p] -= 1
                cur.append(p)
                rec(e + 1, cur, left)
                cur.pop()
                left[p] += 1

    rec(0, [], [cap] * P)
    del itertools
    return out


def placement_bruteforce(counts, P):
    """Exhaustive optimum of the integer program on tiny instances.

    counts int64 [L-1,E,E].  Tries EVERY combination of balanced partitions of the L layers
    (no decomposition, no pruning) and returns (best_local_total, placement int32 [L,E]) for the
    first combination, in lexicographic order, that attains the maximum of the local transitions.
    """
    import itertools

    counts = _i64(counts)
    Lm1, E, _ = counts.shape
    L = Lm1 + 1
    parts = balanced_partitions(E, P)
    assert len(parts) ** L <= 3_000_000, "brute force is for tiny instances only"
    best, best_pl = -1, None
    for combo in itertools.product(parts, repeat=L):
        pl = np.asarray(combo, dtype=np.int32)
        total = int(placement_locality_from_counts(counts, pl).sum())
        if total > best:
            best, best_pl = total, pl
    return best, best_pl
