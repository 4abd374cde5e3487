"""Pins for the CPU oracle: closed forms, invariants, brute force, library routines and the
paper's printed placement example.  None of these tests touches the GPU path.

Each pin is chosen so that a plausible slip in the oracle (a dropped term, a wrong sign or
index, a transposed operand) makes it fail.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch

import synth_inputs as syn

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- gate
def test_gate_logits_matches_library_matmul(oracle):
    g = syn.rng(11)
    x = g.standard_normal((37, 96), dtype=np.float32)
    wg = g.standard_normal((5, 96), dtype=np.float32)  # E != d, T != E: a transposed operand fails
    ref = (torch.from_numpy(x).double() @ torch.from_numpy(wg).double().T).numpy()
    got = oracle.gate_logits(x, wg)
    assert got.shape == (37, 5)
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)


def test_gate_logits_unit_vectors_pick_columns(oracle):
    d, E = 16, 6
    wg = syn.rng(12).standard_normal((E, d), dtype=np.float32)
    x = np.eye(d, dtype=np.float32)  # token c is the c-th unit vector -> logits[c][e] = Wg[e][c]
    got = oracle.gate_logits(x, wg)
    np.testing.assert_array_equal(got, wg.T.astype(np.float64))


def test_softmax_closed_forms(oracle):
    for E in (1, 8, 32, 64):
        p = oracle.softmax(np.full((3, E), 2.5))
        np.testing.assert_array_equal(p, np.full((3, E), 1.0 / E))
    l = np.array([[0.3, -1.2], [5.0, 5.5]])
    p = oracle.softmax(l)
    for t in range(2):
        assert p[t, 0] == pytest.approx(1.0 / (1.0 + math.exp(l[t, 1] - l[t, 0])), rel=1e-15)
    g = syn.rng(13)
    l = g.standard_normal((100, 17)) * 4
    p = oracle.softmax(l)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-14)
    # shift invariance and the defining ratio p_a/p_b = exp(l_a - l_b)
    np.testing.assert_allclose(oracle.softmax(l + 100.0), p, rtol=1e-12)
    np.testing.assert_allclose(p[:, 3] / p[:, 9], np.exp(l[:, 3] - l[:, 9]), rtol=1e-12)
    # large logits do not overflow
    assert np.isfinite(oracle.softmax(np.array([[1000.0, 999.0, -1000.0]]))).all()


# ----------------------------------------------------------------------------- top-k
def _brute_topk(l, k):
    order = sorted(range(len(l)), key=lambda e: (-l[e], e))
    return order[:k]


def test_topk_brute_force_and_ties(oracle):
    g = syn.rng(14)
    # integer-valued logits with many duplicates: ties must go to the lowest expert id
    l = g.integers(-2, 3, size=(200, 9)).astype(np.float64)
    for k in (1, 2, 3):
        idx, w = oracle.topk(l, k, False)
        for t in range(l.shape[0]):
            assert list(idx[t]) == _brute_topk(list(l[t]), k)
    idx, w = oracle.topk(np.zeros((4, 8)), 2, True)
    np.testing.assert_array_equal(idx, np.tile([0, 1], (4, 1)))
    np.testing.assert_array_equal(w, np.full((4, 2), 0.5))
    idx, w = oracle.topk(np.zeros((4, 8)), 1, False)
    np.testing.assert_array_equal(idx, np.zeros((4, 1), dtype=np.int32))
    np.testing.assert_array_equal(w, np.full((4, 1), 1.0 / 8))


def test_topk_weights_closed_forms(oracle):
    g = syn.rng(15)
    l = g.standard_normal((300, 16)) * 3
    p = oracle.softmax(l)
    idx, w = oracle.topk(l, 1, False)
    np.testing.assert_array_equal(idx[:, 0], np.argmax(l, axis=1))
    np.testing.assert_allclose(w[:, 0], p[np.arange(300), idx[:, 0]], rtol=1e-14)  # raw probability, not 1
    assert (w[:, 0] < 1.0).all()
    idx2, w2 = oracle.topk(l, 2, True)
    np.testing.assert_array_equal(idx2[:, 0], idx[:, 0])
    l0 = l[np.arange(300), idx2[:, 0]]
    l1 = l[np.arange(300), idx2[:, 1]]
    assert (l0 >= l1).all()
    np.testing.assert_allclose(w2[:, 0], 1.0 / (1.0 + np.exp(l1 - l0)), rtol=1e-13)  # sigmoid(l0 - l1)
    np.testing.assert_allclose(w2.sum(axis=1), 1.0, rtol=1e-14)
    idx3, w3 = oracle.topk(l, 2, False)
    np.testing.assert_array_equal(idx3, idx2)
    np.testing.assert_allclose(w3, np.take_along_axis(p, idx3.astype(np.int64), axis=1), rtol=1e-14)
    # E = 1
    idx, w = oracle.topk(l[:, :1], 1, False)
    assert (idx == 0).all() and (w == 1.0).all()


def test_topk_column_permutation_equivariance(oracle):
    g = syn.rng(16)
    l = g.standard_normal((128, 32))  # continuous: no ties
    perm = g.permutation(32)
    idx, w = oracle.topk(l, 2, True)
    idx_p, w_p = oracle.topk(l[:, perm], 2, True)
    np.testing.assert_array_equal(perm[idx_p], idx)
    np.testing.assert_allclose(w_p, w, rtol=1e-13)


# ----------------------------------------------------------------------------- dispatch
def _check_dispatch_invariants(res, topk_idx, expert_map, E, E_local):
    T, k = topk_idx.shape
    A = T * k
    flat = topk_idx.reshape(-1)
    src, inv, counts, offsets = res["src_of_sorted"], res["sorted_of_src"], res["counts"], res["offsets"]
    valid = (flat >= 0) & (flat < E)
    local = np.full(A, -1, dtype=np.int64)
    em = np.arange(E) if expert_map is None else expert_map
    local[valid] = em[flat[valid]]
    local[local >= E_local] = -1
    kept = local >= 0
    assert res["kept"] == kept.sum() == counts.sum() == offsets[-1]
    np.testing.assert_array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    assert sorted(src.tolist()) == np.nonzero(kept)[0].tolist()  # bijection onto kept assignments
    np.testing.assert_array_equal(inv[src], np.arange(src.shape[0]))
    assert (inv[~kept] == -1).all()
    e_sorted = local[src]
    assert (np.diff(e_sorted) >= 0).all()
    for e in range(E_local):
        seg = src[offsets[e]:offsets[e + 1]]
        assert (local[seg] == e).all()
        assert (np.diff(seg) > 0).all()  # stable: ascending t*k+j inside an expert


def test_dispatch_invariants_and_brute_force(oracle):
    g = syn.rng(17)
    for (T, k, E) in [(1, 1, 1), (64, 1, 8), (333, 2, 16), (1000, 1, 64)]:
        idx = g.integers(0, E, size=(T, k)).astype(np.int32)
        res = oracle.dispatch(idx, None, E, E)
        _check_dispatch_invariants(res, idx, None, E, E)
        flat = idx.reshape(-1)
        brute = sorted(range(T * k), key=lambda a: (flat[a], a))  # Python's sort is stable
        np.testing.assert_array_equal(res["src_of_sorted"], brute)
        np.testing.assert_array_equal(res["counts"], np.bincount(flat, minlength=E))
        assert res["n_invalid"] == 0


def test_dispatch_expert_map_and_invalid_ids(oracle):
    g = syn.rng(18)
    E, E_local, T = 16, 4, 500
    expert_map = np.full(E, -1, dtype=np.int32)
    resident = np.array([11, 2, 7, 13])  # deliberately not sorted: local id != rank of global id
    expert_map[resident] = np.arange(E_local)
    idx = g.integers(0, E, size=(T, 1)).astype(np.int32)
    idx[5, 0] = -3
    idx[77, 0] = E
    res = oracle.dispatch(idx, expert_map, E, E_local)
    _check_dispatch_invariants(res, idx, expert_map, E, E_local)
    assert res["n_invalid"] == 2
    for le, ge in enumerate(resident):
        assert res["counts"][le] == (idx[:, 0] == ge).sum()


def test_dispatch_single_expert_is_identity_and_empty(oracle):
    idx = np.full((40, 2), 3, dtype=np.int32)
    res = oracle.dispatch(idx, None, 8, 8)
    np.testing.assert_array_equal(res["src_of_sorted"], np.arange(80))
    np.testing.assert_array_equal(res["sorted_of_src"], np.arange(80))
    np.testing.assert_array_equal(res["counts"], [0, 0, 0, 80, 0, 0, 0, 0])
    res = oracle.dispatch(np.zeros((0, 1), dtype=np.int32), None, 8, 8)
    assert res["kept"] == 0 and (res["offsets"] == 0).all()


def test_gather_rows_is_a_copy(oracle):
    g = syn.rng(19)
    x = g.standard_normal((50, 24), dtype=np.float32)
    idx = g.integers(0, 4, size=(50, 2)).astype(np.int32)
    res = oracle.dispatch(idx, None, 4, 4)
    xs = oracle.gather_rows(x, res["src_of_sorted"], 2)
    np.testing.assert_array_equal(xs, x[res["src_of_sorted"] // 2])


# ----------------------------------------------------------------------------- expert FFN
def _torch_ffn(xs, offsets, w1, b1, w2, b2, act):
    xs_t = torch.from_numpy(xs).double()
    out = torch.zeros(xs.shape[0], w2.shape[1], dtype=torch.float64)
    for e in range(w1.shape[0]):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        h = xs_t[lo:hi] @ torch.from_numpy(w1[e]).double().T
        if b1 is not None:
            h = h + torch.from_numpy(b1[e]).double()
        h = torch.nn.functional.gelu(h, approximate="tanh" if act == 1 else "none")
        y = h @ torch.from_numpy(w2[e]).double().T
        if b2 is not None:
            y = y + torch.from_numpy(b2[e]).double()
        out[lo:hi] = y
    return out.numpy()


@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("bias", [False, True])
def test_ffn_matches_library_gemm_and_gelu(oracle, act, bias):
    g = syn.rng(20 + act)
    E, d, f = 3, 24, 56  # d != f: a transposed weight fails
    offsets = np.array([0, 7, 7, 19], dtype=np.int32)  # expert 1 is empty
    xs = g.standard_normal((19, d), dtype=np.float32)
    w1 = g.standard_normal((E, f, d), dtype=np.float32) * 0.3
    w2 = g.standard_normal((E, d, f), dtype=np.float32) * 0.3
    b1 = g.standard_normal((E, f), dtype=np.float32) if bias else None
    b2 = g.standard_normal((E, d), dtype=np.float32) if bias else None
    got = oracle.expert_ffn(xs, offsets, w1, b1, w2, b2, act)
    ref = _torch_ffn(xs, offsets, w1, b1, w2, b2, act)
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)
    # sampled rows agree with the full evaluation
    rows = np.array([18, 0, 7, 6])
    np.testing.assert_array_equal(oracle.expert_ffn_rows(xs, offsets, w1, b1, w2, b2, act, rows), got[rows])


@pytest.mark.parametrize("act", [0, 1])
def test_ffn_identity_expert_closed_form(oracle, act):
    # gelu(z) - gelu(-z) = z for both forms, so W1 = [I; -I; 0], W2 = [I, -I, 0] gives FFN(x) = x
    d, f = 12, 40
    w1 = np.zeros((2, f, d), dtype=np.float32)
    w2 = np.zeros((2, d, f), dtype=np.float32)
    for e in range(2):
        w1[e, :d] = np.eye(d)
        w1[e, d:2 * d] = -np.eye(d)
        w2[e, :, :d] = np.eye(d)
        w2[e, :, d:2 * d] = -np.eye(d)
    w2[1] *= 3.0  # expert 1 returns 3x: checks that rows use the weights of their own expert
    xs = syn.rng(22).standard_normal((10, d), dtype=np.float32)
    offsets = np.array([0, 4, 10], dtype=np.int32)
    y = oracle.expert_ffn(xs, offsets, w1, None, w2, None, act)
    np.testing.assert_allclose(y[:4], xs[:4].astype(np.float64), rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(y[4:], 3.0 * xs[4:].astype(np.float64), rtol=1e-14, atol=1e-15)
    # zero W2 -> zero output
    y0 = oracle.expert_ffn(xs, offsets, w1, None, np.zeros_like(w2), None, act)
    assert (y0 == 0).all()


def test_gelu_reference_values(oracle):
    # 1x1 "FFN" with W1 = W2 = 1 evaluates the activation itself
    z = np.array([[-3.0], [-1.0], [0.0], [0.5], [1.0], [2.0]], dtype=np.float32)
    one = np.ones((1, 1, 1), dtype=np.float32)
    off = np.array([0, 6], dtype=np.int32)
    y = oracle.expert_ffn(z, off, one, None, one, None, 0)[:, 0]
    phi = [0.5 * (1 + math.erf(float(v) / math.sqrt(2))) for v in z[:, 0]]
    np.testing.assert_allclose(y, z[:, 0].astype(np.float64) * np.array(phi), rtol=1e-15)
    assert y[4] == pytest.approx(0.8413447460685429, rel=1e-14)  # Phi(1), a textbook constant
    yt = oracle.expert_ffn(z, off, one, None, one, None, 1)[:, 0]
    assert yt[4] == pytest.approx(0.8411919906082768, rel=1e-12)  # tanh-form GELU(1)
    assert abs(yt - y).max() < 1e-3 and abs(yt - y).max() > 1e-6  # close but a different function


# ----------------------------------------------------------------------------- combine
def test_combine_identity_experts_returns_gate_weighted_input(oracle):
    g = syn.rng(23)
    T, d, E = 64, 8, 4
    x = g.standard_normal((T, d), dtype=np.float32)
    wg = g.standard_normal((E, d), dtype=np.float32)
    logits = oracle.gate_logits(x, wg)
    for k, renorm in ((1, False), (2, True), (2, False)):
        idx, w = oracle.topk(logits, k, renorm)
        res = oracle.dispatch(idx, None, E, E)
        xs = oracle.gather_rows(x, res["src_of_sorted"], k)  # identity experts: y_sorted = x_sorted
        out = oracle.combine(xs, res["sorted_of_src"], w)
        np.testing.assert_allclose(out, w.sum(axis=1, keepdims=True) * x, rtol=1e-13, atol=1e-15)
        if k == 2 and renorm:
            np.testing.assert_allclose(out, x, rtol=1e-13, atol=1e-15)
        if k == 1:
            p = oracle.softmax(logits)
            np.testing.assert_allclose(out, p.max(axis=1, keepdims=True) * x, rtol=1e-13)


def test_combine_linearity_skip_and_brute_force(oracle):
    g = syn.rng(24)
    T, d, k, S = 9, 5, 2, 14
    y = g.standard_normal((S, d))
    inv = g.permutation(T * k).astype(np.int32)
    inv[inv >= S] = -1  # four assignments are not local
    w = g.random((T, k))
    out = oracle.combine(y, inv, w)
    brute = np.zeros((T, d))
    for t in range(T):
        for j in range(k):
            if inv[t * k + j] >= 0:
                brute[t] += w[t, j] * y[inv[t * k + j]]
    np.testing.assert_allclose(out, brute, rtol=1e-15, atol=1e-16)
    np.testing.assert_allclose(oracle.combine(y, inv, 2.5 * w), 2.5 * out, rtol=1e-14)


# ----------------------------------------------------------------------------- affinity
def test_affinity_counts_brute_force_and_invariants(oracle):
    L, N, E = 5, 4000, 7
    trace, _ = syn.planted_trace(L, N, E, 0.6, seed=25)
    counts, loads, n_inv = oracle.affinity_counts(trace, E)
    assert n_inv == 0
    brute = np.zeros((L - 1, E, E), dtype=np.int64)
    for l in range(L - 1):
        np.add.at(brute[l], (trace[l], trace[l + 1]), 1)
    np.testing.assert_array_equal(counts, brute)
    for l in range(L):
        np.testing.assert_array_equal(loads[l], np.bincount(trace[l], minlength=E))
    np.testing.assert_array_equal(counts.sum(axis=2), loads[:-1])   # rows: experts of layer l
    np.testing.assert_array_equal(counts.sum(axis=1), loads[1:])    # columns: experts of layer l+1
    assert (counts.sum(axis=(1, 2)) == N).all()
    shuffled = trace[:, syn.rng(26).permutation(N)]
    np.testing.assert_array_equal(oracle.affinity_counts(shuffled, E)[0], counts)


def test_affinity_counts_orientation_and_special_cases(oracle):
    # every token goes expert 1 -> expert 2: the single non-zero bin is [row 1][col 2]
    trace = np.array([[1] * 10, [2] * 10], dtype=np.int32)
    counts, loads, _ = oracle.affinity_counts(trace, 4)
    assert counts[0, 1, 2] == 10 and counts.sum() == 10
    counts, _, _ = oracle.affinity_counts(np.array([[3], [0]], dtype=np.int32), 4)
    assert counts[0, 3, 0] == 1 and counts.sum() == 1
    # deterministic routing tr[l+1] = perm_l(tr[l]) puts all of a row's load on one column
    L, N, E = 4, 999, 6
    trace, perms = syn.planted_trace(L, N, E, 1.0, seed=27)
    counts, loads, _ = oracle.affinity_counts(trace, E)
    for l in range(L - 1):
        expect = np.zeros((E, E), dtype=np.int64)
        expect[np.arange(E), perms[l]] = loads[l]
        np.testing.assert_array_equal(counts[l], expect)
    # invalid ids are tallied and their transitions skipped
    trace = np.array([[0, 1, 9, 1], [1, -1, 0, 1]], dtype=np.int32)
    counts, loads, n_inv = oracle.affinity_counts(trace, 2)
    assert n_inv == 2 and counts.sum() == 2 and counts[0, 0, 1] == 1 and counts[0, 1, 1] == 1
    np.testing.assert_array_equal(loads, [[1, 2], [1, 2]])
    # L = 1: no pair
    counts, loads, _ = oracle.affinity_counts(np.array([[0, 1, 1]], dtype=np.int32), 2)
    assert counts.shape == (0, 2, 2) and list(loads[0]) == [1, 2]


def test_cond_prob_is_row_conditional(oracle):
    L, N, E = 3, 5000, 8
    trace, perms = syn.planted_trace(L, N, E, 0.7, seed=28)
    counts, loads, _ = oracle.affinity_counts(trace, E)
    P = oracle.cond_prob(counts)
    np.testing.assert_allclose(P.sum(axis=2), 1.0, rtol=1e-14)
    np.testing.assert_allclose(P, counts / loads[:-1, :, None], rtol=1e-15)
    # the planted successor is the hot column: P ~ rho + (1-rho)/E
    for l in range(L - 1):
        hot = P[l, np.arange(E), perms[l]]
        assert (abs(hot - (0.7 + 0.3 / E)) < 0.06).all()
    # empty row -> zeros
    counts2 = counts.copy()
    counts2[0, 3] = 0
    assert (oracle.cond_prob(counts2)[0, 3] == 0).all()


# ----------------------------------------------------------------------------- locality
def test_locality_paper_worked_example(oracle):
    with open(os.path.join(GOLDEN, "fig_compare_example.json")) as fh:
        ex = json.load(fh)
    L, E, G = ex["layers"], ex["experts"], ex["gpus"]
    default = syn.contiguous_placement(L, E, G)
    crossings = []
    for tok, vanilla, coherent in zip(ex["tokens"], ex["vanilla_transfers"], ex["coherent_transfers"]):
        trace = np.array(tok["experts"], dtype=np.int32).reshape(L, 1)
        local = oracle.placement_locality(trace, default)
        cross = (L - 1) - int(local.sum())  # the objective's sum of R_{k,j} for this token
        crossings.append(cross)
        first_hop = int(default[0, tok["experts"][0]] != tok["home_gpu"])
        assert first_hop + cross == coherent  # printed: 3 and 1
        remote_layers = sum(int(default[l, e] != tok["home_gpu"]) for l, e in enumerate(tok["experts"]))
        assert 2 * remote_layers == vanilla  # printed: 4 and 6 (context for the same placement)
    assert crossings == [2, 0]
    both = np.array([t["experts"] for t in ex["tokens"]], dtype=np.int32).T.copy()
    local = oracle.placement_locality(both, default)
    assert local.sum() / (2 * (L - 1)) == 0.5
    # panel (c): the experts of token 1 share GPU 0 on every layer -> no crossing, one transfer
    pc = np.full((L, E), -1, dtype=np.int32)
    for l in range(L):
        on0 = ex["panel_c_gpu0"][f"layer{l}"]
        pc[l, on0] = 0
        rest = [e for e in range(E) if e not in on0]
        pc[l, rest] = 1 + np.arange(len(rest)) // 2
    tok = ex["tokens"][0]
    trace = np.array(tok["experts"], dtype=np.int32).reshape(L, 1)
    local = oracle.placement_locality(trace, pc)
    assert int(local.sum()) == L - 1
    assert int(pc[0, tok["experts"][0]] != tok["home_gpu"]) + 0 == ex["panel_c_token1_transfers"]


def test_locality_routes_agree_and_brute_force_objective(oracle):
    L, N, E, G = 6, 3000, 8, 4
    trace, perms = syn.planted_trace(L, N, E, 0.7, seed=29)
    pl = syn.balanced_random_placement(L, E, G, seed=30)
    local = oracle.placement_locality(trace, pl)
    counts, _, _ = oracle.affinity_counts(trace, E)
    np.testing.assert_array_equal(local, oracle.placement_locality_from_counts(counts, pl))
    # objective of the integer program by brute force over R_{k,j}
    objective = 0
    for n in range(N):
        for l in range(L - 1):
            objective += int(pl[l, trace[l, n]] != pl[l + 1, trace[l + 1, n]])
    assert local.sum() == N * (L - 1) - objective
    # tiny exhaustive case: all placements of 2 experts on 2 devices over 2 layers
    tr = np.array([[0, 0, 1, 1, 0], [0, 1, 1, 0, 0]], dtype=np.int32)
    for a, b in itertools.product([(0, 1), (1, 0)], repeat=2):
        plc = np.array([a, b], dtype=np.int32)
        expect = sum(int(a[tr[0, n]] == b[tr[1, n]]) for n in range(5))
        assert oracle.placement_locality(tr, plc)[0] == expect


def test_locality_closed_forms(oracle):
    L, N, E = 5, 2000, 8
    trace, perms = syn.planted_trace(L, N, E, 0.7, seed=31)
    assert (oracle.placement_locality(trace, np.zeros((L, E), dtype=np.int32)) == N).all()
    same = np.tile(trace[:1], (L, 1))
    ident = np.tile(np.arange(E, dtype=np.int32), (L, 1))
    assert (oracle.placement_locality(same, ident) == N).all()
    # a placement that is constant per layer but differs between layers: nothing is local
    alt = (np.arange(L, dtype=np.int32) % 2)[:, None] * np.ones((1, E), dtype=np.int32)
    assert (oracle.placement_locality(trace, alt) == 0).all()


def test_locality_statistics_random_and_aligned(oracle):
    # affinity-free routing + balanced placement -> 1/G (any GPU with equal chance)
    L, N, E, G = 8, 20000, 16, 4
    trace, _ = syn.planted_trace(L, N, E, 0.0, seed=32)
    pl = syn.balanced_random_placement(L, E, G, seed=33)
    frac = oracle.placement_locality(trace, pl).sum() / (N * (L - 1))
    sigma = math.sqrt((1 / G) * (1 - 1 / G) / (N * (L - 1)))
    assert abs(frac - 1 / G) < 4 * sigma
    # planted affinity + placement aligned with the permutations -> at least rho
    rho = 0.7
    trace, perms = syn.planted_trace(L, N, E, rho, seed=34)
    pl = syn.aligned_placement(perms, E, G)
    frac = oracle.placement_locality(trace, pl).sum() / (N * (L - 1))
    expect = rho + (1 - rho) / G
    assert abs(frac - expect) < 4 * math.sqrt(expect * (1 - expect) / (N * (L - 1)))
    # and it beats the default contiguous placement clearly
    frac_default = oracle.placement_locality(trace, syn.contiguous_placement(L, E, G)).sum() / (N * (L - 1))
    assert frac > frac_default + 0.3


def test_routing_away_reproduces_the_printed_transfer_counts(oracle):
    """The walk-through's numbers from the counters alone: vanilla 2*sum(away) = 4 and 6,
    coherent away[0] + crossings = 3 and 1, and 1 for token 1 under the panel (c) placement."""
    with open(os.path.join(GOLDEN, "fig_compare_example.json")) as fh:
        ex = json.load(fh)
    L, E, G = ex["layers"], ex["experts"], ex["gpus"]
    default = syn.contiguous_placement(L, E, G)
    trace = np.array([t["experts"] for t in ex["tokens"]], dtype=np.int32).T.copy()   # [L, 2]
    home = np.array([t["home_gpu"] for t in ex["tokens"]], dtype=np.int32)
    for n in range(2):
        tr = trace[:, n:n + 1].copy()
        away = oracle.routing_away(tr, default, home[n:n + 1])
        local = oracle.placement_locality(tr, default)
        assert 2 * int(away.sum()) == ex["vanilla_transfers"][n]
        assert int(away[0]) + (L - 1) - int(local.sum()) == ex["coherent_transfers"][n]
    both = oracle.routing_away(trace, default, home)
    assert 2 * int(both.sum()) == sum(ex["vanilla_transfers"])
    pc = np.full((L, E), -1, dtype=np.int32)
    for l in range(L):
        on0 = ex["panel_c_gpu0"][f"layer{l}"]
        pc[l, on0] = 0
        rest = [e for e in range(E) if e not in on0]
        pc[l, rest] = 1 + np.arange(len(rest)) // 2
    tr = trace[:, 0:1].copy()
    away = oracle.routing_away(tr, pc, home[0:1])
    assert int(away[0]) + (L - 1) - int(oracle.placement_locality(tr, pc).sum()) == ex["panel_c_token1_transfers"]


def test_routing_away_closed_forms(oracle):
    L, N, E, G = 5, 4000, 8, 4
    trace, _ = syn.planted_trace(L, N, E, 0.5, seed=83)
    g = syn.rng(84)
    home = g.integers(0, G, size=N).astype(np.int32)
    pl = syn.balanced_random_placement(L, E, G, seed=85)
    away = oracle.routing_away(trace, pl, home)
    # the definition, vectorised independently
    dev = np.take_along_axis(pl, trace, axis=1)
    np.testing.assert_array_equal(away, (dev != home[None, :]).sum(axis=1))
    # every expert on GPU 0 and every token at home on GPU 0: nothing is ever away
    assert (oracle.routing_away(trace, np.zeros((L, E), np.int32), np.zeros(N, np.int32)) == 0).all()
    # home outside the placement's range: everything is away
    assert (oracle.routing_away(trace, pl, np.full(N, G, np.int32)) == N).all()
    # invalid ids are skipped
    bad = trace.copy()
    bad[2, :100] = E
    bad[3, :50] = -1
    a2 = oracle.routing_away(bad, pl, np.full(N, G, np.int32))
    assert a2[2] == N - 100 and a2[3] == N - 50 and a2[0] == N
    # uniform homes, balanced placement, uniform routing: about (G-1)/G of the tokens are away
    tr_u, _ = syn.planted_trace(L, 40000, E, 0.0, seed=86)
    home_u = syn.rng(87).integers(0, G, size=40000).astype(np.int32)
    frac = oracle.routing_away(tr_u, pl, home_u).sum() / (40000 * L)
    assert abs(frac - (G - 1) / G) < 0.01


def test_multihop_counts_pins(oracle):
    """Appendix statistic: adjacent pairs equal the one-hop counts; every pair equals an
    independently written scatter-add; on a deterministic chain the counts sit on the composed
    permutations; row / column sums are the layer loads."""
    L, N, E = 5, 3000, 8
    trace, perms = syn.planted_trace(L, N, E, 0.6, seed=91)
    trace[2, 10:200:7] = E        # a few invalid ids
    trace[0, 3:90:5] = -1
    multi = oracle.affinity_counts_multihop(trace, E)
    assert multi.shape == (L * (L - 1) // 2, E, E)
    one_hop, loads, _ = oracle.affinity_counts(trace, E)
    for l in range(L - 1):
        np.testing.assert_array_equal(multi[oracle.multihop_pair_index(L, l, l + 1)], one_hop[l])
    for l in range(L):
        for m in range(l + 1, L):
            a, b = trace[l], trace[m]
            ok = (a >= 0) & (a < E) & (b >= 0) & (b < E)
            ref = np.zeros((E, E), dtype=np.int64)
            np.add.at(ref, (a[ok], b[ok]), 1)
            np.testing.assert_array_equal(multi[oracle.multihop_pair_index(L, l, m)], ref)
    # deterministic chain: expert i of layer l leads to perm_{m-1}(...perm_l(i)) at layer m, always
    tr1, p1 = syn.planted_trace(L, N, E, 1.0, seed=92)
    m1 = oracle.affinity_counts_multihop(tr1, E)
    first = np.bincount(tr1[0], minlength=E)
    for m in range(1, L):
        comp = np.arange(E)
        for l in range(m):
            comp = p1[l][comp]
        c = m1[oracle.multihop_pair_index(L, 0, m)]
        assert (c[np.arange(E), comp] == first).all() and c.sum() == N
    # sums: with all ids valid, rows of (l, m) add up to the loads of layer l, columns to those of layer m
    _, loads1, _ = oracle.affinity_counts(tr1, E)
    for l in range(L):
        for m in range(l + 1, L):
            c = m1[oracle.multihop_pair_index(L, l, m)]
            np.testing.assert_array_equal(c.sum(axis=1), loads1[l])
            np.testing.assert_array_equal(c.sum(axis=0), loads1[m])
    assert [oracle.multihop_pair_index(4, l, m) for l in range(4) for m in range(l + 1, 4)] == list(range(6))


# --------------------------------------------------------------------------- communication volume model
def test_comm_volume_hand_computed_and_structure(oracle):
    """Table "Comparison with state-of-the-art GPT MoE optimization methods", evaluated by hand:
    G = 8 GPUs, N = 1000 tokens per GPU, L = 12 layers, p = 0.875, p* = 0.25."""
    v = oracle.comm_volume(8, 1000, 12, 0.875, 0.25)
    assert v.tolist() == [168000.0, 336000.0, 88000.0, 112000.0]  # 2*96000*.875, 4*..., 8000*(3+8), 8000*(6+8)
    # uniform routing over G GPUs leaves (G-1)/G of the tokens away from home: p = 7/8 above, and the
    # vanilla top-1 volume is then 2 (G-1) N L
    assert v[0] == 2 * 7 * 1000 * 12
    g = syn.rng(950)
    for _ in range(50):
        G, N, L = int(g.integers(1, 65)), int(g.integers(0, 100000)), int(g.integers(1, 49))
        p, ps = float(g.random()), float(g.random())
        a = oracle.comm_volume(G, N, L, p, ps)
        assert a[1] == 2 * a[0]                                   # top-2 doubles the vanilla volume
        gather = G * N * G
        assert math.isclose(a[3] - gather, 2 * (a[2] - gather), rel_tol=1e-12, abs_tol=1e-9)  # ... and only the Alltoall part of the coherent one
        assert math.isclose(a[2], oracle.comm_volume(G, N, L, p, 0.0)[2] + G * N * L * ps, rel_tol=1e-12, abs_tol=1e-9)
        assert oracle.comm_volume(G, N, L, p, 0.0)[2] == gather   # nothing moves: the AllGather term alone
        b = oracle.comm_volume(G, 3 * N, L, p, ps)
        np.testing.assert_allclose(b, 3 * a, rtol=1e-12)          # linear in the tokens per GPU
        # the coherent scheme wins exactly when L p* + G < 2 L p
        if not math.isclose(L * ps + G, 2 * L * p, rel_tol=1e-9):
            assert (a[2] < a[0]) == (L * ps + G < 2 * L * p)
    # an argument swap (p for p*, G for L) changes the result
    assert oracle.comm_volume(8, 1000, 12, 0.25, 0.875).tolist() != v.tolist()
    assert oracle.comm_volume(12, 1000, 8, 0.875, 0.25).tolist() != v.tolist()


def test_comm_volume_on_the_printed_walk_through(oracle):
    """Design, "Token Context Coherence in Expert Parallelism": the two tokens of the walk-through need
    4 + 6 transfers with vanilla expert parallelism and 3 + 1 with coherent contexts.  With G*N = 2
    resident tokens the table's Alltoall terms 2*G*N*L*p and G*N*L*p* must be those totals."""
    with open(os.path.join(GOLDEN, "fig_compare_example.json")) as fh:
        ex = json.load(fh)
    L, E, G = ex["layers"], ex["experts"], ex["gpus"]
    default = syn.contiguous_placement(L, E, G)
    trace = np.array([t["experts"] for t in ex["tokens"]], dtype=np.int32).T.copy()
    home = np.array([t["home_gpu"] for t in ex["tokens"]], dtype=np.int32)
    p, ps = oracle.transfer_ratios(trace, default, home)
    assert math.isclose(p, (4 + 6) / 2 / (2 * L)) and math.isclose(ps, (3 + 1) / (2 * L))
    vol = oracle.comm_volume(2, 1, L, p, ps)   # two GPUs' worth of one token each: G*N = 2 tokens
    assert math.isclose(vol[0], sum(ex["vanilla_transfers"]))
    assert math.isclose(vol[2] - 2 * 1 * 2, sum(ex["coherent_transfers"]))
    for n in range(2):  # token by token
        pn, psn = oracle.transfer_ratios(trace[:, n:n + 1].copy(), default, home[n:n + 1])
        assert math.isclose(2 * L * pn, ex["vanilla_transfers"][n]) and math.isclose(L * psn, ex["coherent_transfers"][n])


def test_transfer_ratios_against_the_counters(oracle):
    """The token walk agrees with the two counter formulas (2*sum away; away[0] + crossings), which
    are computed by separately written routines, and with closed forms."""
    L, N, E, G = 6, 5000, 16, 4
    g = syn.rng(951)
    trace = g.integers(0, E, size=(L, N)).astype(np.int32)
    pl = syn.balanced_random_placement(L, E, G, 952)
    home = g.integers(0, G, size=N).astype(np.int32)
    p, ps = oracle.transfer_ratios(trace, pl, home)
    away = oracle.routing_away(trace, pl, home)
    local = oracle.placement_locality(trace, pl)
    assert math.isclose(p, away.sum() / (N * L))
    assert math.isclose(ps, (away[0] + (N * (L - 1) - local.sum())) / (N * L))
    assert abs(p - (G - 1) / G) < 0.02 and abs(ps - (G - 1) / G) < 0.02   # uniform routing: any GPU equally likely
    one = np.zeros((L, E), dtype=np.int32)
    assert oracle.transfer_ratios(trace, one, np.zeros(N, np.int32)) == (0.0, 0.0)      # everything at home
    assert oracle.transfer_ratios(trace, one, np.ones(N, np.int32)) == (1.0, 1.0 / L)   # one move, then stays
