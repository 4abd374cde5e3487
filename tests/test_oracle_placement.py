"""Pins of the oracle's exhaustive placement search (Design, "Solving Affinity's duality by Integer
Programming") against what the mathematics fixes: closed forms on structured traces, symmetry, and
dominance over every sampled feasible placement."""
import itertools

import numpy as np
import pytest

import oracle
import synth_inputs as syn


@pytest.fixture(scope="module", autouse=True)
def _built():
    oracle.build()


def test_balanced_partitions_count_is_the_multinomial():
    # E! / ((E/P)!)^P labelled balanced partitions
    assert len(oracle.balanced_partitions(4, 2)) == 6
    assert len(oracle.balanced_partitions(6, 3)) == 90
    assert len(oracle.balanced_partitions(6, 2)) == 20
    for part in oracle.balanced_partitions(6, 3):
        assert sorted(np.bincount(part, minlength=3)) == [2, 2, 2]


def test_bruteforce_reaches_full_locality_on_a_deterministic_chain():
    # rho = 1: every token follows the planted permutations, so the aligned placement keeps ALL
    # N(L-1) transitions local, and nothing can do better.
    L, N, E, P = 3, 600, 4, 2
    trace, perms = syn.planted_trace(L, N, E, 1.0, seed=11)
    counts, _, _ = oracle.affinity_counts(trace, E)
    best, pl = oracle.placement_bruteforce(counts, P)
    assert best == N * (L - 1)
    assert int(oracle.placement_locality(trace, pl).sum()) == N * (L - 1)
    aligned = syn.aligned_placement(perms, E, P)
    assert int(oracle.placement_locality_from_counts(counts, aligned).sum()) == best


def test_bruteforce_on_uniform_counts_gives_one_over_P():
    # all E*E transitions equally frequent: every balanced placement keeps exactly 1/P of them
    L, E, P = 3, 4, 2
    counts = np.full((L - 1, E, E), 5, dtype=np.int64)
    best, _ = oracle.placement_bruteforce(counts, P)
    assert best == (L - 1) * E * E * 5 // P


def test_bruteforce_dominates_every_feasible_placement_of_a_tiny_instance():
    # a plain maximum over an independently written enumeration (numpy scoring, not the oracle's)
    L, E, P = 3, 4, 2
    g = syn.rng(77)
    counts = g.integers(0, 50, size=(L - 1, E, E)).astype(np.int64)
    best, pl = oracle.placement_bruteforce(counts, P)
    parts = [p for p in itertools.product(range(P), repeat=E) if sorted(np.bincount(p, minlength=P)) == [E // P] * P]
    top = -1
    for combo in itertools.product(parts, repeat=L):
        s = 0
        for l in range(L - 1):
            same = np.equal.outer(np.asarray(combo[l]), np.asarray(combo[l + 1]))
            s += int((counts[l] * same).sum())
        top = max(top, s)
    assert best == top
    assert int(oracle.placement_locality_from_counts(counts, pl).sum()) == best


def test_bruteforce_is_invariant_to_relabelling_the_experts_of_a_layer():
    L, E, P = 3, 4, 2
    g = syn.rng(78)
    counts = g.integers(0, 30, size=(L - 1, E, E)).astype(np.int64)
    best, _ = oracle.placement_bruteforce(counts, P)
    perm = g.permutation(E)
    relabelled = counts.copy()
    relabelled[0] = counts[0][:, perm]      # experts of layer 1 renamed ...
    relabelled[1] = counts[1][perm, :]      # ... consistently in both pairs they take part in
    best2, _ = oracle.placement_bruteforce(relabelled, P)
    assert best2 == best
