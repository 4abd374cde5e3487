"""Placement search (Design, "Solving Affinity's duality by Integer Programming", "Staged Experts
Affinity"): the host solver against the oracle's exhaustive search and against what the planted
traces fix; the GPU batch scoring against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2401_08383_amd as exf
import synth_inputs as syn
from paper_2401_08383_amd import binding as B


@pytest.fixture(scope="module", autouse=True)
def _built():
    oracle.build()


def _search(counts, G, nodes=1, restarts=4, seed=0):
    pl = B.placement_search(torch.from_numpy(np.ascontiguousarray(counts, dtype=np.int64)), G, nodes, restarts, seed)
    return pl.numpy()


@pytest.mark.parametrize("L,E,P,seed", [(3, 4, 2, 1), (4, 4, 2, 2), (3, 6, 3, 3), (2, 6, 2, 4), (3, 6, 2, 5)])
def test_solver_matches_exhaustive_optimum_on_tiny_instances(L, E, P, seed):
    g = syn.rng(900 + seed)
    counts = g.integers(0, 100, size=(L - 1, E, E)).astype(np.int64)
    best, _ = oracle.placement_bruteforce(counts, P)
    pl = _search(counts, P)
    assert B.check_placement(torch.from_numpy(pl), P)
    assert int(oracle.placement_locality_from_counts(counts, pl).sum()) == best


def test_solver_recovers_a_deterministic_chain_exactly():
    # rho = 1: an aligned placement keeps every transition local; the solver must find one of them
    for (L, N, E, G) in [(6, 4096, 8, 4), (12, 8192, 32, 8), (8, 5000, 64, 8)]:
        trace, _ = syn.planted_trace(L, N, E, 1.0, seed=31 + E)
        counts, _, _ = oracle.affinity_counts(trace, E)
        pl = _search(counts, G)
        assert B.check_placement(torch.from_numpy(pl), G)
        assert int(oracle.placement_locality(trace, pl).sum()) == N * (L - 1)


@pytest.mark.parametrize("marginal", ["uniform", "zipf"])
def test_solver_beats_the_planted_and_the_default_placements(marginal):
    L, N, E, G = 12, 20000, 32, 8
    trace, perms = syn.planted_trace(L, N, E, 0.7, seed=41, marginal=marginal)
    counts, _, _ = oracle.affinity_counts(trace, E)
    pl = _search(counts, G, restarts=3, seed=5)
    assert B.check_placement(torch.from_numpy(pl), G)
    found = int(oracle.placement_locality_from_counts(counts, pl).sum())
    aligned = int(oracle.placement_locality_from_counts(counts, syn.aligned_placement(perms, E, G)).sum())
    default = int(oracle.placement_locality_from_counts(counts, syn.contiguous_placement(L, E, G)).sum())
    rand = int(oracle.placement_locality_from_counts(counts, syn.balanced_random_placement(L, E, G, 9)).sum())
    assert found >= aligned > default      # the planted structure is a feasible point of the search
    assert found > rand
    assert found / (N * (L - 1)) > 0.7     # rho = 0.7 of the transitions follow the permutations


def test_two_stage_respects_nodes_and_both_levels_beat_the_default():
    L, N, E, G, nodes = 8, 20000, 32, 8, 2
    trace, perms = syn.planted_trace(L, N, E, 0.8, seed=51)
    counts, _, _ = oracle.affinity_counts(trace, E)
    pl = _search(counts, G, nodes=nodes, restarts=3, seed=2)
    assert B.check_placement(torch.from_numpy(pl), G)
    node_pl = (pl // (G // nodes)).astype(np.int32)
    assert B.check_placement(torch.from_numpy(np.ascontiguousarray(node_pl)), nodes)
    default = syn.contiguous_placement(L, E, G)
    gpu_found = int(oracle.placement_locality_from_counts(counts, pl).sum())
    node_found = int(oracle.placement_locality_from_counts(counts, node_pl).sum())
    assert gpu_found > int(oracle.placement_locality_from_counts(counts, default).sum())
    assert node_found > int(oracle.placement_locality_from_counts(counts, (default // (G // nodes)).astype(np.int32)).sum())
    assert node_found >= gpu_found  # a transition that stays on a GPU stays on its node


def test_solver_is_deterministic_and_validates():
    g = syn.rng(61)
    counts = g.integers(0, 1000, size=(5, 16, 16)).astype(np.int64)
    a = _search(counts, 4, restarts=3, seed=7)
    b = _search(counts, 4, restarts=3, seed=7)
    np.testing.assert_array_equal(a, b)
    lib = exf.lib()
    out = torch.empty((6, 16), dtype=torch.int32)
    c = torch.from_numpy(counts)
    assert lib.exf_placement_search(c.data_ptr(), 6, 16, 3, 1, 1, 0, out.data_ptr()) == B.EXF_ERR_BAD_SHAPE   # 3 does not divide 16
    assert lib.exf_placement_search(c.data_ptr(), 6, 16, 4, 3, 1, 0, out.data_ptr()) == B.EXF_ERR_BAD_SHAPE   # 3 does not divide 4
    assert lib.exf_placement_search(None, 6, 16, 4, 1, 1, 0, out.data_ptr()) == B.EXF_ERR_NULL_PTR
    neg = c.clone()
    neg[0, 0, 0] = -1
    assert lib.exf_placement_search(neg.data_ptr(), 6, 16, 4, 1, 1, 0, out.data_ptr()) == B.EXF_ERR_BAD_SHAPE
    one = _search(np.zeros((0, 8, 8), dtype=np.int64), 4)  # a single layer: any balanced map
    assert B.check_placement(torch.from_numpy(one), 4)


# ----------------------------------------------------------------------------- GPU batch scoring
@pytest.mark.gpu
@pytest.mark.parametrize("L,E,G,Bn", [(2, 8, 4, 1), (12, 8, 4, 130), (12, 32, 8, 257), (24, 64, 8, 1000), (5, 33, 3, 65), (1, 8, 2, 4)])
def test_gpu_scores_candidate_batches_exactly(L, E, G, Bn):
    print(f"[case] placement_locality_from_counts L={L} E={E} G={G} B={Bn}", flush=True)
    g = syn.rng(700 + L + E)
    counts = g.integers(0, 1 << 40, size=(max(L - 1, 0), E, E)).astype(np.int64)   # sums far beyond 32 bits
    pls = g.integers(0, G, size=(Bn, L, E)).astype(np.int32)
    if E % G == 0:
        pls[0] = syn.contiguous_placement(L, E, G)
    dev = "cuda:0"
    out = B.placement_locality_from_counts(torch.from_numpy(counts).to(dev), torch.from_numpy(pls).to(dev))
    got = out.cpu().numpy()
    assert got.shape == (Bn, max(L - 1, 0))
    for b in range(Bn) if Bn <= 300 else list(range(0, Bn, 7)) + [Bn - 1]:
        np.testing.assert_array_equal(got[b], oracle.placement_locality_from_counts(counts, pls[b]))


@pytest.mark.gpu
def test_gpu_search_pipeline_on_a_trace():
    """trace -> affinity_histogram (GPU) -> host solver -> scores of {found, default, random} from
    the counts (GPU batch) agree with placement_locality on the trace (GPU) and with the oracle."""
    print("[case] search pipeline", flush=True)
    L, N, E, G = 12, 50000, 32, 8
    trace, perms = syn.planted_trace(L, N, E, 0.7, seed=71)
    dev = "cuda:0"
    tr = torch.from_numpy(trace).to(dev)
    res = exf.affinity_histogram(tr, E)
    counts_ref, _, _ = oracle.affinity_counts(trace, E)
    np.testing.assert_array_equal(res["counts"].cpu().numpy(), counts_ref)
    found = B.placement_search(res["counts"].cpu(), G, 1, 3, 1)
    cands = np.stack([found.numpy(), syn.contiguous_placement(L, E, G), syn.balanced_random_placement(L, E, G, 3),
                      syn.aligned_placement(perms, E, G)]).astype(np.int32)
    scores = B.placement_locality_from_counts(res["counts"], torch.from_numpy(cands).to(dev)).cpu().numpy()
    for b in range(len(cands)):
        np.testing.assert_array_equal(scores[b], oracle.placement_locality(trace, cands[b]))
        on_trace = exf.placement_locality(tr, torch.from_numpy(cands[b]).to(dev), G).cpu().numpy()
        np.testing.assert_array_equal(scores[b], on_trace)
    assert scores[0].sum() >= scores[3].sum() > scores[1].sum()


# ----------------------------------------------------------------------------- transfer counters
@pytest.mark.gpu
@pytest.mark.parametrize("L,N,E,G", [(3, 2, 8, 4), (1, 777, 8, 2), (12, 8192, 8, 4), (5, 100001, 64, 8), (24, 1 << 18, 64, 8), (6, 70003, 16, 2)])
def test_routing_transfers_parity(L, N, E, G):
    print(f"[case] routing_transfers L={L} N={N} E={E} G={G}", flush=True)
    dev = "cuda:0"
    trace, _ = syn.planted_trace(L, N, E, 0.6, seed=800 + L + E)
    g = syn.rng(801 + N)
    if N > 1000:  # invalid ids in a few places
        trace[L // 2, 17:900:13] = E + 3
        trace[0, 5:600:11] = -2
    home = g.integers(0, G, size=N).astype(np.int32)
    pl = syn.balanced_random_placement(L, E, G, seed=802)
    local, away = exf.routing_transfers(torch.from_numpy(trace).to(dev), torch.from_numpy(pl).to(dev), torch.from_numpy(home).to(dev), G)
    np.testing.assert_array_equal(away.cpu().numpy(), oracle.routing_away(trace, pl, home))
    np.testing.assert_array_equal(local.cpu().numpy(), oracle.placement_locality(trace, pl))


@pytest.mark.gpu
def test_routing_transfers_paper_worked_example_on_gpu():
    import json
    import os
    print("[case] routing_transfers worked example", flush=True)
    with open(os.path.join(os.path.dirname(__file__), "golden", "fig_compare_example.json")) as fh:
        ex = json.load(fh)
    L, E, G = ex["layers"], ex["experts"], ex["gpus"]
    dev = "cuda:0"
    default = torch.from_numpy(syn.contiguous_placement(L, E, G)).to(dev)
    for tok, vanilla, coherent in zip(ex["tokens"], ex["vanilla_transfers"], ex["coherent_transfers"]):
        tr = torch.tensor(tok["experts"], dtype=torch.int32).reshape(L, 1).to(dev)
        home = torch.tensor([tok["home_gpu"]], dtype=torch.int32, device=dev)
        local, away = exf.routing_transfers(tr, default, home, G)
        assert 2 * int(away.sum()) == vanilla                                   # printed: 4 and 6
        assert int(away[0]) + (L - 1) - int(local.sum()) == coherent            # printed: 3 and 1


@pytest.mark.gpu
def test_send_buffer_is_a_dispatch_by_destination():
    """The per-destination send buffer of the single Alltoall: moe_dispatch with the layer's
    placement row as expert_map groups the rows by destination GPU, stable, counts = send counts."""
    print("[case] send buffer", flush=True)
    T, d, E, G = 3000, 128, 32, 8
    dev = "cuda:0"
    g = syn.rng(811)
    x = syn.quantize(g.standard_normal((T, d), dtype=np.float32), "bf16")
    idx = g.integers(0, E, size=(T, 1)).astype(np.int32)
    row = syn.balanced_random_placement(1, E, G, seed=812)[0]
    res = exf.moe_dispatch(torch.from_numpy(x).to(torch.bfloat16).to(dev), torch.from_numpy(idx).to(dev), E, G,
                           torch.from_numpy(row).to(dev))
    ref = oracle.dispatch(idx, row, E, G)
    np.testing.assert_array_equal(res.expert_counts.cpu().numpy(), np.bincount(row[idx[:, 0]], minlength=G))
    np.testing.assert_array_equal(res.src_of_sorted.cpu().numpy(), ref["src_of_sorted"])
    dest_sorted = row[idx[res.src_of_sorted.cpu().numpy(), 0]]
    assert (np.diff(dest_sorted) >= 0).all()                                     # grouped by destination
    np.testing.assert_array_equal(res.x_sorted.float().cpu().numpy(), x[ref["src_of_sorted"]])


# ----------------------------------------------------------------------------- multi-hop affinity
@pytest.mark.gpu
@pytest.mark.parametrize("L,N,E", [(2, 512, 8), (5, 8192, 8), (12, 16384, 32), (7, 100001, 64), (24, 70000, 64), (4, 70003, 16), (1, 100, 8)])
def test_affinity_multihop_parity(L, N, E):
    print(f"[case] affinity_multihop L={L} N={N} E={E}", flush=True)
    trace, _ = syn.planted_trace(L, N, E, 0.7, seed=850 + L + E)
    if N > 1000 and L > 2:
        trace[1, 7:700:9] = E
        trace[L - 1, 2:300:5] = -3
    res = exf.affinity_multihop(torch.from_numpy(trace).to("cuda:0"), E)
    ref = oracle.affinity_counts_multihop(trace, E)
    got = res["counts"].cpu().numpy()
    np.testing.assert_array_equal(got, ref)
    if L > 1:
        rows = ref.sum(axis=2, keepdims=True).astype(np.float64)
        prob = np.divide(ref, rows, out=np.zeros(ref.shape, dtype=np.float64), where=rows > 0).astype(np.float32)
        np.testing.assert_allclose(res["cond_prob"].cpu().numpy(), prob, rtol=1e-6, atol=0)
        # adjacent pairs are the one-hop statistic of the other entry point
        one = exf.affinity_histogram(torch.from_numpy(trace).to("cuda:0"), E)["counts"].cpu().numpy()
        for l in range(L - 1):
            np.testing.assert_array_equal(got[oracle.multihop_pair_index(L, l, l + 1)], one[l])
