"""Helpers shared by the GPU parity tests: host <-> device conversion and comparison rules."""
import numpy as np
import torch

import synth_inputs as syn

DEV = "cuda:0"

# Output tolerances (relative to max |reference|) fixed by the task: bf16 2e-2, fp32 1e-5.
OUT_RTOL = {"bf16": 2e-2, "f32": 1e-5}
# Gate logits / weights: identical stored inputs, fp32 accumulation in a different order than
# the fp64 reference: |delta| <= tol * max(1, |ref|).
GATE_TOL = {"bf16": 1e-4, "f32": 1e-5}


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 host array holding storage-exact values -> device tensor of the storage dtype."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)  # exact: the values are already bf16-representable
    return t.to(DEV)


def dev_i32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> host array; bf16 is widened exactly to fp32."""
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


def assert_close_max(got, ref, rtol, what="", mag=None):
    """max |got - ref| <= rtol * max |ref|, plus a per-element rule: |got - ref| <= rtol * (mag + rms),
    rms taken over the element's own row (an output row is a set of dot products with one hidden
    vector, so their rounding errors scale with that row; a row of zeros - a token without a kept
    assignment - must then be reproduced exactly).  `mag` is the magnitude the element's rounding errors are relative to: |ref| itself, unless the
    caller knows better - a top-2 output is the sum of two expert outputs that were each rounded to
    the storage dtype before the sum, so its error scales with the gate-weighted sum of their
    magnitudes even where the two nearly cancel."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return
    scale = np.abs(ref).max()
    err = np.abs(got - ref).max()
    assert np.isfinite(got).all(), what
    assert err <= rtol * max(scale, 1e-30), f"{what}: max err {err:.3e} > {rtol:.1e} * {scale:.3e}"
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    mag = np.abs(ref) if mag is None else np.asarray(mag, dtype=np.float64)
    bad = (np.abs(got - ref) > rtol * (mag + rms)).sum()
    assert bad == 0, f"{what}: {bad} elements outside rtol*(magnitude+rms)"


def assert_gate_close(got, ref, tol, what=""):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    if ref.size:
        lim = tol * np.maximum(1.0, np.abs(ref))
        assert (np.abs(got - ref) <= lim).all(), f"{what}: max excess {(np.abs(got - ref) - lim).max():.3e}"


def check_routing_against_fp64(idx_gpu, logits64, k, tol):
    """End-to-end routing check: tokens whose fp64 decision margins exceed `tol` must match the
    fp64 choice exactly; for the others the GPU's pick must be one of the near-tied experts.
    Returns the number of ambiguous tokens."""
    T, E = logits64.shape
    order = np.argsort(-logits64, axis=1, kind="stable")  # ties -> lowest id first
    srt = np.take_along_axis(logits64, order, axis=1)
    scale = np.maximum(1.0, np.abs(srt[:, 0]))
    ambiguous = np.zeros(T, dtype=bool)
    for j in range(k):
        if j + 1 < E:
            ambiguous |= (srt[:, j] - srt[:, j + 1]) < tol * scale
    clear = ~ambiguous
    assert (idx_gpu[clear] == order[clear, :k]).all(), "routing differs from fp64 on a clear-margin token"
    for t in np.nonzero(ambiguous)[0]:
        for j in range(k):
            chosen = logits64[t, idx_gpu[t, j]]
            assert abs(chosen - srt[t, j]) < 4 * tol * scale[t], (t, j)
        assert len(set(idx_gpu[t].tolist())) == k
    return int(ambiguous.sum())


def oracle_routing(oracle, x, wg, k, renorm, idx_gpu, w_gpu, tol):
    """(idx, weights, logits) of the fp64 oracle for inputs x, wg - after checking that the GPU took the
    same decisions.  Everything downstream of the gate is then compared with an oracle chain that was
    fed by the oracle's own routing, never by an array that came back from the GPU.  The seeded inputs
    of the test-suite hold no decision closer than the fp32 accumulation error, so the two routings
    are identical; should new inputs ever hold such a near-tie, the comparison below names it."""
    logits64 = oracle.gate_logits(x, wg)
    idx64, w64 = oracle.topk(logits64, k, renorm)
    n_amb = check_routing_against_fp64(idx_gpu, logits64, k, tol)
    assert n_amb <= max(3, idx_gpu.shape[0] * k // 250)  # near-ties are rare: the tolerance must not carry the comparison
    differ = np.nonzero((idx_gpu != idx64).any(axis=1))[0]
    assert differ.size == 0, f"routing differs from the fp64 oracle at near-tied tokens {differ[:8].tolist()}: pick inputs without them"
    assert_gate_close(w_gpu, w64, tol, "gate weights")
    return idx64, w64, logits64


def own_logits_selection(logits, k, renorm):
    """Property of a gate result, no oracle involved: the top-k (ties to the lowest id) and softmax
    weights that the returned logits themselves imply, in fp64."""
    lg = np.asarray(logits, dtype=np.float64)
    order = np.argsort(-lg, axis=1, kind="stable")[:, :k]
    p = np.exp(lg - lg.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, order, axis=1)
    if renorm and k > 1:
        w = w / w.sum(axis=1, keepdims=True)
    return order.astype(np.int32), w


def expected_dispatch_compare(res_gpu, ref, A):
    kept = ref["kept"]
    np.testing.assert_array_equal(res_gpu.expert_counts.cpu().numpy(), ref["counts"])
    np.testing.assert_array_equal(res_gpu.expert_offsets.cpu().numpy(), ref["offsets"])
    np.testing.assert_array_equal(res_gpu.src_of_sorted.cpu().numpy()[:kept], ref["src_of_sorted"])
    np.testing.assert_array_equal(res_gpu.sorted_of_src.cpu().numpy(), ref["sorted_of_src"])


STRATUM_ROWS = 64  # finer than any row tile a kernel may cut an expert's rows into (a power of two <= 64 rows divides it)


def sample_rows(offsets, per_stratum, seed, min_rows=0):
    """Stratified sample of sorted rows: every expert's rows are cut into consecutive blocks of
    STRATUM_ROWS rows (counted from the expert's first row, the last block ragged) and every block
    gives `per_stratum` random rows; the first and the last row of every expert are added.  Whatever
    row tiling the GPU path uses - full tiles, remainder tiles, a masked last tile - each of its row
    tiles then holds at least one row that the oracle evaluates.  `per_stratum` is raised until the
    sample has `min_rows` rows."""
    offsets = np.asarray(offsets, dtype=np.int64)
    total = int(offsets[-1] - offsets[0])
    while True:
        g = syn.rng(seed)
        rows = []
        for e in range(len(offsets) - 1):
            lo, hi = int(offsets[e]), int(offsets[e + 1])
            if hi <= lo:
                continue
            pick = {lo, hi - 1}
            for b in range(lo, hi, STRATUM_ROWS):
                top = min(b + STRATUM_ROWS, hi)
                pick.update(b + int(v) for v in g.permutation(top - b)[:per_stratum])
            rows.extend(sorted(pick))
        if len(rows) >= min(min_rows, total) or per_stratum >= STRATUM_ROWS:
            return np.array(rows, dtype=np.int64)
        per_stratum += 1


def strata_covered(offsets, rows):
    """Number of (expert, STRATUM_ROWS-row block) strata and how many of them hold a sampled row."""
    offsets = np.asarray(offsets, dtype=np.int64)
    owner = np.searchsorted(offsets, rows, side="right") - 1
    hit = {(int(e), int((r - offsets[e]) // STRATUM_ROWS)) for e, r in zip(owner, rows)}
    n = sum(int(-(-(offsets[e + 1] - offsets[e]) // STRATUM_ROWS)) for e in range(len(offsets) - 1))
    return n, len(hit)
