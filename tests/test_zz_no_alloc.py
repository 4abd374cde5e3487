"""moe_dispatch_static, the entry point for callers that cannot allocate: same result as moe_dispatch
(bit for bit: every output is an integer array or a copy of rows), on two calls in a row, the second
with a smaller input, then on the index-only and the long (separate scan launch) paths."""
import numpy as np
import pytest
import torch

import paper_2401_08383_amd as exf
import synth_inputs as syn
from helpers import DEV, to_dev
from paper_2401_08383_amd.binding import DispatchResult

pytestmark = pytest.mark.gpu



def _case(seed, T, d, k, E, E_local, dtype, gather, with_map):
    print(f"[case] moe_dispatch_static seed={seed} T={T} d={d} k={k} E={E} E_local={E_local} {dtype} gather={gather} map={with_map}", flush=True)
    g = syn.rng(seed)
    x = to_dev(syn.quantize(g.standard_normal((T, d), dtype=np.float32), dtype), dtype)
    idx = g.integers(0, E, size=(T, k)).astype(np.int32)
    if T > 10:
        idx[3, 0] = E + 5  # an id outside [0,E): not kept
        idx[7, k - 1] = -2
    idx_d = torch.from_numpy(idx).to(DEV)
    emap = None
    if with_map:
        m = g.integers(-1, E_local, size=E).astype(np.int32)
        emap = torch.from_numpy(m).to(DEV)
    A = T * k
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32

    def fresh():
        return DispatchResult(torch.full((A, d), 3.0, dtype=tdt, device=DEV) if gather else None,
                              torch.full((A,), -7, dtype=torch.int32, device=DEV), torch.full((A,), -7, dtype=torch.int32, device=DEV),
                              torch.full((E_local,), -7, dtype=torch.int32, device=DEV),
                              torch.full((E_local + 1,), -7, dtype=torch.int32, device=DEV))

    ref = exf.moe_dispatch(x, idx_d, E, E_local=E_local, expert_map=emap, out=fresh(), gather=gather)
    out = fresh()
    before = torch.cuda.memory_allocated()
    exf.moe_dispatch_static(x, idx_d, E, out, E_local=E_local, expert_map=emap)
    assert torch.cuda.memory_allocated() == before  # the binding allocates nothing either
    torch.cuda.synchronize()
    for name in ("src_of_sorted", "sorted_of_src", "expert_counts", "expert_offsets"):
        assert torch.equal(getattr(out, name), getattr(ref, name)), name
    if gather:
        assert torch.equal(out.x_sorted.view(torch.int16 if dtype == "bf16" else torch.int32),
                           ref.x_sorted.view(torch.int16 if dtype == "bf16" else torch.int32)), "x_sorted"
    assert int(ref.expert_offsets[-1]) <= A


def test_static_dispatch_matches_moe_dispatch_on_consecutive_calls():
    # two calls in a row on one stream, the second smaller: stale chunk counts of the first must not leak
    _case(1, 20000, 128, 2, 32, 32, "bf16", True, False)
    _case(2, 3001, 128, 2, 32, 32, "bf16", True, False)
    _case(3, 777, 64, 1, 64, 8, "f32", True, True)        # expert map with -1 entries
    _case(4, 5000, 64, 1, 8, 8, "bf16", False, False)     # index maps only
    _case(5, 300000, 8, 2, 64, 64, "bf16", False, True)   # more than 256 chunks: the separate scan launch
    _case(6, 33, 8, 1, 4, 4, "f32", True, False)          # a single ragged chunk after the long one
    _case(7, 0, 64, 1, 8, 8, "bf16", True, False)         # no tokens: counts and offsets are still written


def test_static_dispatch_rejects_what_its_scratch_cannot_hold():
    lib = exf.lib()
    one = torch.zeros(64, dtype=torch.int32, device=DEV)
    p = one.data_ptr()
    rc = lib.moe_dispatch_static(p, p, None, (1 << 20) + 1, 64, 1, 8, 8, exf.binding.EXF_BF16, None, p, p, p, p, None)
    assert rc == exf.binding.EXF_ERR_BAD_SHAPE and "scratch" in exf.last_error()
    rc = lib.moe_dispatch_static(p, p, None, (1 << 19) + 1, 64, 2, 8, 8, exf.binding.EXF_BF16, None, p, p, p, p, None)
    assert rc == exf.binding.EXF_ERR_BAD_SHAPE
