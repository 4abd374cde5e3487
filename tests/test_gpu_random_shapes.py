"""Seeded random shapes inside the documented limits of every entry point, through the parity helpers
of the other GPU test modules (same oracles, same comparison rules).  The fixed cases there are chosen
by hand around tile edges; these fill in the combinations nobody thought of."""
import numpy as np
import pytest

import test_gpu_parity as P
import test_placement_search as Q

pytestmark = pytest.mark.gpu

_TAIL_COUNTS = [0, 1, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 511, 513, 700]


def _say(msg):
    print(f"[case] {msg}", flush=True)


def _one_case(oracle, g, seed):
    kind = int(g.integers(0, 12))
    if kind in (0, 1):  # index-only dispatch -> fused FFN + combine
        dtype = "bf16" if kind == 0 else "f32"
        if dtype == "bf16":
            d, f, T = int(g.integers(1, 13)) * 64, int(g.integers(1, 33)) * 64, int(g.integers(1, 6000))
        else:
            d, f, T = int(g.integers(1, 40)) * 4, int(g.integers(1, 60)) * 4, int(g.integers(1, 1500))
        E = int(g.integers(1, 17))
        k = int(g.integers(1, min(E, 2) + 1))
        E_local = int(g.integers(1, E + 1))
        act, bias, skew = int(g.integers(0, 2)), bool(g.integers(0, 2)), bool(g.integers(0, 2))
        _say(f"fused {dtype} T={T} d={d} f={f} E={E} E_local={E_local} k={k} act={act} bias={bias} skew={skew}")
        P._fused_case(oracle, T, d, f, E, E_local, k, act, bias, seed, skew=skew, dtype=dtype)
    elif kind in (2, 3):  # expert FFN on sorted rows, remainders of every kind
        dtype = "bf16" if kind == 2 else "f32"
        if dtype == "bf16":
            E, d, f = int(g.integers(1, 12)), int(g.integers(1, 20)) * 64, int(g.integers(1, 20)) * 64
            counts = [int(c) for c in g.choice(_TAIL_COUNTS, size=E)]
        else:
            E, d, f = int(g.integers(1, 9)), int(g.integers(1, 40)) * 4, int(g.integers(1, 60)) * 4
            counts = [int(c) for c in g.choice([0, 1, 3, 15, 16, 17, 63, 64, 65, 100, 200], size=E)]
        counts[int(g.integers(0, E))] += 1  # at least one row
        act, bias = int(g.integers(0, 2)), bool(g.integers(0, 2))
        _say(f"ffn {dtype} counts={counts} d={d} f={f} act={act} bias={bias}")
        P._ffn_case(oracle, dtype, counts, d, f, act, bias, seed)
    elif kind == 4:
        dtype = "bf16" if g.integers(0, 4) else "f32"
        E = int(g.integers(1, 65))
        k, renorm = int(g.integers(1, min(E, 2) + 1)), int(g.integers(0, 2))
        if dtype == "bf16":  # both bf16 kernels: the weights-in-LDS one starts at T = 16384
            d, T = int(g.integers(1, 160)) * 8, int(g.choice([1, 15, 17, 500, 4099, 16383, 16384, 16400, 20011, 40000]))
        else:
            d, T = int(g.integers(1, 25)) * 4, int(g.integers(1, 3000))
        P.test_gate_topk_parity(oracle, dtype, T, d, E, k, renorm)
    elif kind == 5:
        dtype = "bf16" if g.integers(0, 2) else "f32"
        T, k = int(g.choice([1, 2, 63, 64, 65, 1000, 4097, 33333, 100000])), int(g.integers(1, 3))
        E = int(g.integers(k, 65))
        d = int(g.integers(1, 33)) * (8 if dtype == "bf16" else 4)
        P.test_dispatch_parity(oracle, dtype, T, d, k, E)
    elif kind == 6:
        T, E = int(g.integers(1, 5000)), int(g.integers(1, 65))
        P.test_topk_from_logits_bit_exact(oracle, T, E, int(g.integers(1, min(E, 2) + 1)), int(g.integers(0, 2)))
    elif kind == 7:
        dtype = "bf16" if g.integers(0, 2) else "f32"
        T, k = int(g.integers(1, 5000)), int(g.integers(1, 3))
        P.test_combine_parity(oracle, dtype, T, int(g.integers(1, 200)) * (8 if dtype == "bf16" else 4), k)
    elif kind == 8:
        L, E = int(g.integers(1, 30)), int(g.integers(1, 65))
        Q.test_gpu_scores_candidate_batches_exactly(L, E, int(g.integers(1, E + 1)), int(g.choice([1, 2, 63, 64, 65, 300, 1000])))
    else:  # the three statistics over a trace
        L, E = int(g.integers(1, 26)), int(g.integers(1, 65))
        N = int(g.choice([1, 2, 63, 1000, 4097, 50001, 150003]))
        G = int(g.choice([x for x in range(1, E + 1) if E % x == 0]))
        if kind == 9:
            Q.test_routing_transfers_parity(L, N, E, G)
        elif kind == 10:
            Q.test_affinity_multihop_parity(L, N, E)
        else:
            P.test_affinity_and_locality_parity(oracle, L, N, E, G)


@pytest.mark.parametrize("seed", [11, 12, 13, 14, 15, 16])
def test_random_shapes_match_the_oracle(oracle, seed):
    g = np.random.default_rng(seed)
    for n in range(40):
        _one_case(oracle, g, seed * 1000 + n)
