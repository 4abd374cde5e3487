"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element, at
sizes that span several tiles and a ragged tail, plus the edge cases of each step."""
import numpy as np
import pytest
import torch

import paper_2401_08383_amd as exf
import synth_inputs as syn
from helpers import (DEV, GATE_TOL, OUT_RTOL, assert_close_max, assert_gate_close, check_routing_against_fp64, dev_i32,
                     oracle_routing, own_logits_selection,
                     expected_dispatch_compare, to_dev, to_host)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


# ----------------------------------------------------------------------------- top-k from logits
@pytest.mark.parametrize("T,E,k,renorm", [(1, 1, 1, 0), (777, 8, 1, 0), (1000, 64, 2, 1), (513, 33, 2, 0), (4096, 32, 1, 0)])
def test_topk_from_logits_bit_exact(oracle, T, E, k, renorm):
    _say(f"topk_from_logits T={T} E={E} k={k} renorm={renorm}")
    g = syn.rng(100 + T)
    logits = g.standard_normal((T, E), dtype=np.float32)
    logits[::3] = np.round(logits[::3])  # many exact ties: the lowest id must win
    idx_ref, w_ref = oracle.topk(logits.astype(np.float64), k, renorm)
    idx, w = exf.moe_topk_from_logits(torch.from_numpy(logits).to(DEV), k, renorm)
    np.testing.assert_array_equal(idx.cpu().numpy(), idx_ref)
    assert_gate_close(w.cpu().numpy(), w_ref, 1e-6, "topk weights")


# ----------------------------------------------------------------------------- gate
GATE_CASES = [
    ("f32", 512, 64, 8, 1, 0), ("f32", 100, 100, 5, 2, 1),
    ("bf16", 512, 64, 8, 1, 0), ("bf16", 1000, 1024, 8, 1, 0), ("bf16", 300, 200, 17, 2, 1),
    ("bf16", 2500, 512, 32, 1, 0), ("bf16", 999, 1024, 64, 2, 1), ("bf16", 16, 4096, 64, 2, 1),
    ("bf16", 33000, 256, 48, 2, 0), ("bf16", 16500, 128, 64, 1, 0),
    ("bf16", 17000, 64, 8, 1, 0), ("bf16", 20001, 200, 20, 2, 1), ("bf16", 70000, 32, 33, 1, 0),
    ("bf16", 16400, 1088, 16, 1, 0),  # 136 16-byte pieces per row: partial XOR swizzle of the LDS-resident gate weight
]


@pytest.mark.parametrize("dtype,T,d,E,k,renorm", GATE_CASES)
def test_gate_topk_parity(oracle, dtype, T, d, E, k, renorm):
    _say(f"gate {dtype} T={T} d={d} E={E} k={k} renorm={renorm}")
    g = syn.rng(200 + T + E)
    x = syn.quantize(g.standard_normal((T, d), dtype=np.float32), dtype)
    wg = syn.quantize(g.standard_normal((E, d), dtype=np.float32) * np.float32(1.0 / np.sqrt(d)), dtype)
    idx, w, logits = exf.moe_gate_topk(to_dev(x, dtype), to_dev(wg, dtype), k, renorm, want_logits=True)
    idx, w, logits = idx.cpu().numpy(), w.cpu().numpy(), logits.cpu().numpy()
    logits64 = oracle.gate_logits(x, wg)
    assert_gate_close(logits, logits64, GATE_TOL[dtype], "logits")
    # the decision in the kernel's own precision: the routing must be the one its own fp32 logits imply
    idx_k, w_k = own_logits_selection(logits, k, renorm)
    np.testing.assert_array_equal(idx, idx_k)
    assert_gate_close(w, w_k, 1e-6, "weights vs own logits")
    # end to end against fp64 logits
    n_amb = check_routing_against_fp64(idx, logits64, k, GATE_TOL[dtype])
    assert n_amb <= max(3, T * k // 250)  # near-ties are rare: the tolerance above must not carry the comparison
    _, w64 = oracle.topk(logits64, k, renorm)
    clear = (idx == oracle.topk(logits64, k, renorm)[0]).all(axis=1)
    assert_gate_close(w[clear], w64[clear], GATE_TOL[dtype], "weights")
    # without the optional logits output the routing is the same
    idx2, w2, none = exf.moe_gate_topk(to_dev(x, dtype), to_dev(wg, dtype), k, renorm, want_logits=False)
    assert none is None
    np.testing.assert_array_equal(idx2.cpu().numpy(), idx)
    np.testing.assert_array_equal(w2.cpu().numpy(), w)


def test_gate_all_equal_logits_pick_lowest_ids():
    x = torch.zeros((64, 128), dtype=torch.bfloat16, device=DEV)
    wg = torch.ones((32, 128), dtype=torch.bfloat16, device=DEV)
    idx, w, _ = exf.moe_gate_topk(x, wg, 2, True)
    assert (idx.cpu().numpy() == np.array([0, 1])).all()
    assert (w.cpu().numpy() == 0.5).all()
    idx, w, _ = exf.moe_gate_topk(x, wg, 1, False)
    assert (idx.cpu().numpy() == 0).all() and (w.cpu().numpy() == np.float32(1 / 32)).all()


# ----------------------------------------------------------------------------- dispatch
def _run_dispatch(oracle, x, idx, E, E_local, expert_map, dtype):
    T, k = idx.shape
    ref = oracle.dispatch(idx, expert_map, E, E_local)
    res = exf.moe_dispatch(to_dev(x, dtype), dev_i32(idx), E, E_local, None if expert_map is None else dev_i32(expert_map))
    expected_dispatch_compare(res, ref, T * k)
    kept = ref["kept"]
    xs = to_host(res.x_sorted)[:kept]
    np.testing.assert_array_equal(xs, x[ref["src_of_sorted"] // k])  # a pure copy: bit-exact
    # index-only mode (no sorted rows; short batches take a single launch): the same maps
    only = exf.moe_dispatch(to_dev(x, dtype), dev_i32(idx), E, E_local, None if expert_map is None else dev_i32(expert_map),
                            gather=False)
    expected_dispatch_compare(only, ref, T * k)
    return res, ref


@pytest.mark.parametrize("dtype,T,d,k,E", [("f32", 512, 64, 1, 8), ("bf16", 1, 64, 1, 8), ("bf16", 1023, 128, 1, 8),
                                           ("bf16", 5000, 256, 2, 64), ("bf16", 3333, 64, 1, 32), ("f32", 2049, 32, 2, 5),
                                           ("bf16", 300001, 8, 1, 16)])
def test_dispatch_parity(oracle, dtype, T, d, k, E):
    _say(f"dispatch {dtype} T={T} d={d} k={k} E={E}")
    g = syn.rng(300 + T)
    x = syn.quantize(g.standard_normal((T, d), dtype=np.float32), dtype)
    idx = g.integers(0, E, size=(T, k)).astype(np.int32)
    _run_dispatch(oracle, x, idx, E, E, None, dtype)


def test_dispatch_expert_map_invalid_and_degenerate(oracle):
    g = syn.rng(310)
    T, d, E, E_local = 4000, 64, 64, 8
    x = syn.quantize(g.standard_normal((T, d), dtype=np.float32), "bf16")
    expert_map = np.full(E, -1, dtype=np.int32)
    resident = g.permutation(E)[:E_local]
    expert_map[resident] = np.arange(E_local)
    idx = g.integers(0, E, size=(T, 1)).astype(np.int32)  # 7/8 of the tokens are not local
    idx[3] = -1
    idx[1999] = E
    idx[2000] = 1 << 30
    res, ref = _run_dispatch(oracle, x, idx, E, E_local, expert_map, "bf16")
    assert ref["n_invalid"] == 3 and ref["kept"] < T // 4
    # everything to one expert: identity permutation
    idx = np.full((1500, 2), 5, dtype=np.int32)
    x = syn.quantize(g.standard_normal((1500, 64), dtype=np.float32), "bf16")
    res, ref = _run_dispatch(oracle, x, idx, 8, 8, None, "bf16")
    np.testing.assert_array_equal(res.src_of_sorted.cpu().numpy(), np.arange(3000))
    # nothing local at all
    res, ref = _run_dispatch(oracle, x, idx, 8, 8, np.full(8, -1, dtype=np.int32), "bf16")
    assert ref["kept"] == 0 and (res.sorted_of_src.cpu().numpy() == -1).all()
    # skewed (Zipf) loads
    tr, _ = syn.planted_trace(1, 6000, 32, 0.0, seed=311, marginal="zipf")
    x = syn.quantize(g.standard_normal((6000, 64), dtype=np.float32), "bf16")
    _run_dispatch(oracle, x, tr[0].reshape(-1, 1).copy(), 32, 32, None, "bf16")


@pytest.mark.parametrize("A,E,E_local", [(4096, 8, 8), (4097, 64, 64), (8192, 8, 8), (8193, 3, 3), (16384, 64, 8), (16385, 64, 8),
                                         (65, 64, 64), (9000, 1, 1)])
def test_dispatch_index_only_short_lists(oracle, A, E, E_local):
    """Index-only dispatch around the sizes where the single-launch kernel changes its round count
    and hands over to the chunked kernels: the same unique stable permutation on both sides."""
    _say(f"dispatch index-only A={A} E={E} E_local={E_local}")
    g = syn.rng(320 + A)
    idx = g.integers(0, E, size=(A, 1)).astype(np.int32)
    idx[g.integers(0, A, size=5)] = -3  # a few entries outside [0,E)
    expert_map = None
    if E_local < E:
        expert_map = np.full(E, -1, dtype=np.int32)
        expert_map[g.permutation(E)[:E_local]] = np.arange(E_local, dtype=np.int32)
    ref = oracle.dispatch(idx, expert_map, E, E_local)
    x = torch.zeros((A, 8), dtype=torch.bfloat16, device=DEV)
    for _ in range(2):  # twice: nothing is carried from one call to the next
        res = exf.moe_dispatch(x, dev_i32(idx), E, E_local, None if expert_map is None else dev_i32(expert_map), gather=False)
        expected_dispatch_compare(res, ref, A)


def test_dispatch_empty_batch():
    x = torch.empty((0, 64), dtype=torch.bfloat16, device=DEV)
    idx = torch.empty((0, 1), dtype=torch.int32, device=DEV)
    res = exf.moe_dispatch(x, idx, 8)
    assert (res.expert_counts.cpu().numpy() == 0).all() and (res.expert_offsets.cpu().numpy() == 0).all()


# ----------------------------------------------------------------------------- expert FFN
def _ffn_case(oracle, dtype, counts, d, f, act, bias, seed, rows=None):
    g = syn.rng(seed)
    E = len(counts)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    A = int(offsets[-1])
    cap = A + 5  # buffers larger than the kept rows: the tail must stay untouched
    xs = syn.quantize(g.standard_normal((cap, d), dtype=np.float32), dtype)
    w1 = syn.quantize(g.standard_normal((E, f, d), dtype=np.float32) * np.float32(0.05), dtype)
    w2 = syn.quantize(g.standard_normal((E, d, f), dtype=np.float32) * np.float32(0.05), dtype)
    b1 = syn.quantize(g.standard_normal((E, f), dtype=np.float32) * np.float32(0.1), dtype) if bias else None
    b2 = syn.quantize(g.standard_normal((E, d), dtype=np.float32) * np.float32(0.1), dtype) if bias else None
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    y = torch.full((cap, d), 7.0, dtype=tdt, device=DEV)
    exf.moe_expert_ffn(to_dev(xs, dtype), dev_i32(offsets), to_dev(w1, dtype), to_dev(w2, dtype),
                       None if b1 is None else to_dev(b1, dtype), None if b2 is None else to_dev(b2, dtype), act, out=y)
    y = to_host(y)
    assert (y[A:] == 7.0).all(), "rows beyond expert_offsets[E_local] were written"
    rows = np.arange(A) if rows is None else rows
    ref = oracle.expert_ffn_rows(xs, offsets, w1, b1, w2, b2, act, rows)
    assert_close_max(y[rows], ref, OUT_RTOL[dtype], f"ffn {dtype}")


@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("bias", [False, True])
def test_ffn_f32_parity(oracle, act, bias):
    _say(f"ffn f32 act={act} bias={bias}")
    _ffn_case(oracle, "f32", [70, 0, 129, 1, 64, 3], 64, 256, act, bias, seed=400 + act)
    _ffn_case(oracle, "f32", [5], 36, 20, act, bias, seed=402)  # tiles with ragged N and K tails


@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("bias", [False, True])
def test_ffn_bf16_parity(oracle, act, bias):
    _say(f"ffn bf16 act={act} bias={bias}")
    _ffn_case(oracle, "bf16", [130, 0, 257, 1, 128, 31], 128, 320, act, bias, seed=410 + act)
    _ffn_case(oracle, "bf16", [300], 64, 64, act, bias, seed=412)


def test_ffn_bf16_long_reduction(oracle):
    """Many K tiles per output tile (the LDS ring wraps several times), full, masked and tail row tiles."""
    _say("ffn bf16 long K")
    _ffn_case(oracle, "bf16", [600, 200, 70, 0, 256], 1024, 512, 0, False, seed=430)


@pytest.mark.parametrize("bias", [False, True])
def test_ffn_bf16_remainder_tiles_in_k_slices(oracle, bias):
    """Few remainder tiles and a long second reduction: they run as K slices added by a second kernel."""
    _say(f"ffn bf16 K-sliced remainder tiles bias={bias}")
    _ffn_case(oracle, "bf16", [70, 300, 5], 128, 1024, 0, bias, seed=440)          # 4 tail tiles x 4 slices
    _ffn_case(oracle, "bf16", [257, 0, 129, 64, 1], 256, 2048, 1, bias, seed=441)  # 8 slices, two column tiles


def test_ffn_bf16_wide_second_contraction(oracle):
    """Enough rows and output columns that the second contraction takes its 256x256 tile (with K-sliced
    remainder tiles); sampled rows of every expert against the oracle."""
    _say("ffn bf16 wide second contraction")
    counts = [9000, 70, 7430]
    off = np.concatenate([[0], np.cumsum(counts)])
    g = syn.rng(450)
    rows = np.unique(np.concatenate([off[:-1], off[1:] - 1, g.integers(0, off[-1], size=40)]))
    _ffn_case(oracle, "bf16", counts, 2048, 512, 0, True, seed=451, rows=rows)
    # output width that is no multiple of the tile width (4 tiles of 256 columns and one of 64)
    counts = [20000, 6600]
    off = np.concatenate([[0], np.cumsum(counts)])
    rows = np.unique(np.concatenate([off[:-1], off[1:] - 1, g.integers(0, off[-1], size=30)]))
    _ffn_case(oracle, "bf16", counts, 1088, 128, 1, False, seed=452, rows=rows)


@pytest.mark.parametrize("bias", [False, True])
def test_ffn_bf16_tall_tiles(oracle, bias):
    """Launches with two or more rounds of 256-row tiles fold small remainders into taller last tiles
    of the expert (320 rows): remainders of 1, 64, 65 and 128 rows (one and two tall tiles), 129 rows (a
    masked full tile instead), a remainder larger than the expert's full tiles can take (tail tiles),
    experts without a full tile.  Every element against the oracle; first contraction (wide hidden
    layer), then second contraction (wide output)."""
    counts = [6 * 256 + 1, 3 * 256 + 65, 2 * 256 + 128, 5 * 256 + 129, 256 + 44, 256 + 100, 200, 100, 0, 2 * 256 + 64]
    _say(f"ffn bf16 tall tiles bias={bias}: first contraction")
    _ffn_case(oracle, "bf16", counts, 64, 8192, 0, bias, seed=460)
    _say(f"ffn bf16 tall tiles bias={bias}: second contraction")
    _ffn_case(oracle, "bf16", counts, 8192, 64, 1, bias, seed=461)


def test_ffn_bf16_many_experts_skewed(oracle):
    _say("ffn bf16 skewed 32 experts")
    tr, _ = syn.planted_trace(1, 3000, 32, 0.0, seed=420, marginal="zipf")
    counts = np.bincount(tr[0], minlength=32)
    _ffn_case(oracle, "bf16", counts.tolist(), 256, 512, 0, False, seed=421)


def test_ffn_identity_expert_returns_input(oracle):
    # gelu(z) - gelu(-z) = z: W1 = [I; -I], W2 = [I, -I] makes every expert the identity
    d, f = 64, 128
    w1 = np.zeros((2, f, d), dtype=np.float32)
    w2 = np.zeros((2, d, f), dtype=np.float32)
    for e in range(2):
        w1[e, :d], w1[e, d:] = np.eye(d), -np.eye(d)
        w2[e, :, :d], w2[e, :, d:] = np.eye(d), -np.eye(d)
    xs = syn.quantize(syn.rng(430).standard_normal((200, d), dtype=np.float32), "bf16")
    off = dev_i32(np.array([0, 77, 200]))
    y = to_host(exf.moe_expert_ffn(to_dev(xs, "bf16"), off, to_dev(w1, "bf16"), to_dev(w2, "bf16")))
    assert_close_max(y, xs, 2e-2, "identity expert")


# ----------------------------------------------------------------------------- combine
@pytest.mark.parametrize("dtype,T,d,k", [("f32", 512, 64, 1), ("bf16", 1000, 128, 1), ("bf16", 777, 256, 2), ("f32", 50, 36, 2)])
def test_combine_parity(oracle, dtype, T, d, k):
    _say(f"combine {dtype} T={T} d={d} k={k}")
    g = syn.rng(500 + T)
    A = T * k
    y = syn.quantize(g.standard_normal((A, d), dtype=np.float32), dtype)
    inv = g.permutation(A).astype(np.int32)
    inv[g.random(A) < 0.1] = -1  # some assignments are not local
    w = g.random((T, k), dtype=np.float32)
    out = exf.moe_combine(to_dev(y, dtype), dev_i32(inv), torch.from_numpy(w).to(DEV))
    ref = oracle.combine(y, inv, w)
    got = to_host(out)
    # one rounding to the storage type on top of an fp32 accumulation of k terms: the error is
    # bounded relative to sum_j |w_j y_j| (the terms may cancel)
    mag = oracle.combine(np.abs(y), inv, np.abs(w))
    eps = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -22
    assert (np.abs(got - ref) <= eps * mag + 1e-30).all()


# ----------------------------------------------------------------------------- whole layer, small
@pytest.mark.parametrize("cfg_id,dtype,T,d,f,E,k,renorm", [(1, "f32", 512, 64, 256, 8, 1, False), (0, "bf16", 700, 128, 256, 8, 2, True)])
def test_layer_small_end_to_end(oracle, cfg_id, dtype, T, d, f, E, k, renorm):
    _say(f"layer end-to-end {dtype} T={T} d={d} f={f} E={E} k={k}")
    if cfg_id == 1:
        cfg = syn.CONFIGS[1]
        x, wg = syn.tokens(cfg), syn.gate_weight(cfg)
        w1, w2 = syn.expert_weights(cfg)
    else:
        g = syn.rng(600)
        x = syn.quantize(g.standard_normal((T, d), dtype=np.float32), dtype)
        wg = syn.quantize(g.standard_normal((E, d), dtype=np.float32) * np.float32(0.1), dtype)
        w1 = syn.quantize(g.standard_normal((E, f, d), dtype=np.float32) * np.float32(0.05), dtype)
        w2 = syn.quantize(g.standard_normal((E, d, f), dtype=np.float32) * np.float32(0.05), dtype)
    xd = to_dev(x, dtype)
    idx, w, logits = exf.moe_gate_topk(xd, to_dev(wg, dtype), k, renorm, want_logits=True)
    disp = exf.moe_dispatch(xd, idx, E)
    y = exf.moe_expert_ffn(disp.x_sorted, disp.expert_offsets, to_dev(w1, dtype), to_dev(w2, dtype))
    out = exf.moe_combine(y, disp.sorted_of_src, w)
    # oracle chain on the oracle's own routing (checked to be the GPU's)
    idx_h, w_ref, _ = oracle_routing(oracle, x, wg, k, renorm, idx.cpu().numpy(), w.cpu().numpy(), GATE_TOL[dtype])
    ref_d = oracle.dispatch(idx_h, None, E, E)
    expected_dispatch_compare(disp, ref_d, T * k)
    xs_ref = oracle.gather_rows(x, ref_d["src_of_sorted"], k)
    y_ref = oracle.expert_ffn(xs_ref, ref_d["offsets"], w1, None, w2, None, 0)
    assert_close_max(to_host(y)[: ref_d["kept"]], y_ref, OUT_RTOL[dtype], "y_sorted")
    out_ref = oracle.combine(y_ref, ref_d["sorted_of_src"], w_ref)
    mag = oracle.combine(np.abs(y_ref), ref_d["sorted_of_src"], w_ref)  # what the summands' roundings are relative to
    assert_close_max(to_host(out), out_ref, OUT_RTOL[dtype], "layer output", mag=mag)
    # the same layer without sorted copies: index-only dispatch and the fused FFN + combine
    only = exf.moe_dispatch(xd, idx, E, gather=False)
    fused = exf.moe_expert_ffn_fused(xd, only.src_of_sorted, only.sorted_of_src, w, only.expert_offsets, to_dev(w1, dtype),
                                     to_dev(w2, dtype))
    assert_close_max(to_host(fused), out_ref, OUT_RTOL[dtype], "fused layer output", mag=mag)


# ----------------------------------------------------------------------------- fused FFN + combine
def _fused_case(oracle, T, d, f, E, E_local, k, act, bias, seed, skew=False, dtype="bf16"):
    """moe_dispatch (index-only) -> moe_expert_ffn_fused against oracle gather -> FFN -> combine."""
    g = syn.rng(seed)
    x = syn.quantize(g.standard_normal((T, d), dtype=np.float32), dtype)
    w1 = syn.quantize(g.standard_normal((E_local, f, d), dtype=np.float32) * np.float32(0.05), dtype)
    w2 = syn.quantize(g.standard_normal((E_local, d, f), dtype=np.float32) * np.float32(0.05), dtype)
    b1 = syn.quantize(g.standard_normal((E_local, f), dtype=np.float32) * np.float32(0.1), dtype) if bias else None
    b2 = syn.quantize(g.standard_normal((E_local, d), dtype=np.float32) * np.float32(0.1), dtype) if bias else None
    if skew:  # a few heavy experts, several empty ones
        p = 1.0 / np.arange(1, E + 1) ** 1.5
        idx = np.stack([g.choice(E, size=k, replace=False, p=p / p.sum()) for _ in range(T)]).astype(np.int32)
    else:
        idx = np.stack([g.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32)
    gate = g.random((T, k), dtype=np.float32) + np.float32(0.05)
    expert_map = None
    if E_local < E:  # the first E_local of a shuffled list of experts live here; the others' tokens are dropped
        expert_map = np.full(E, -1, dtype=np.int32)
        expert_map[g.permutation(E)[:E_local]] = np.arange(E_local, dtype=np.int32)
    xd = to_dev(x, dtype)
    disp = exf.moe_dispatch(xd, torch.from_numpy(idx).to(DEV), E, E_local=E_local,
                            expert_map=None if expert_map is None else torch.from_numpy(expert_map).to(DEV), gather=False)
    out = torch.full((T, d), 7.0, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device=DEV)
    exf.moe_expert_ffn_fused(xd, disp.src_of_sorted, disp.sorted_of_src, torch.from_numpy(gate).to(DEV), disp.expert_offsets,
                             to_dev(w1, dtype), to_dev(w2, dtype), None if b1 is None else to_dev(b1, dtype),
                             None if b2 is None else to_dev(b2, dtype), act, out=out)
    ref_d = oracle.dispatch(idx, expert_map, E, E_local)
    expected_dispatch_compare(disp, ref_d, T * k)
    xs_ref = oracle.gather_rows(x, ref_d["src_of_sorted"], k)
    y_ref = oracle.expert_ffn(xs_ref, ref_d["offsets"], w1, b1, w2, b2, act)
    out_ref = oracle.combine(y_ref, ref_d["sorted_of_src"], gate)
    got = to_host(out)
    unrouted = (ref_d["sorted_of_src"].reshape(T, k) < 0).all(axis=1)
    assert (got[unrouted] == 0).all(), "rows of tokens without a kept assignment must be zero"
    mag = oracle.combine(np.abs(y_ref), ref_d["sorted_of_src"], gate)  # what the summands' roundings are relative to
    assert_close_max(got, out_ref, OUT_RTOL[dtype], "fused layer output", mag=mag)
    return int(unrouted.sum())


@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("bias", [False, True])
def test_ffn_fused_top1_parity(oracle, act, bias):
    _say(f"ffn fused top-1 act={act} bias={bias}")
    assert _fused_case(oracle, 700, 128, 320, 6, 6, 1, act, bias, seed=700 + act) == 0
    assert _fused_case(oracle, 1500, 64, 128, 16, 5, 1, act, bias, seed=702) > 0  # most tokens belong to other GPUs


def test_ffn_fused_top1_skewed_and_tiny(oracle):
    _say("ffn fused top-1 skewed / tiny")
    _fused_case(oracle, 900, 128, 1024, 6, 6, 1, 0, True, seed=713)  # remainder tiles in K slices, scattered by the adding kernel
    _fused_case(oracle, 3000, 256, 512, 32, 32, 1, 0, False, seed=710, skew=True)
    _fused_case(oracle, 1, 64, 64, 4, 4, 1, 0, False, seed=711)
    _fused_case(oracle, 67, 64, 64, 8, 1, 1, 0, True, seed=712)  # one resident expert, seven of eight tokens unrouted


@pytest.mark.parametrize("k,E_local,bias", [(1, 6, True), (1, 2, False), (2, 6, False)])
def test_ffn_fused_f32_parity(oracle, k, E_local, bias):
    _say(f"ffn fused f32 k={k} E_local={E_local} bias={bias}")
    _fused_case(oracle, 333, 36, 20, 6, E_local, k, 0, bias, seed=740 + k, dtype="f32")
    _fused_case(oracle, 700, 64, 256, 6, E_local, k, 1, bias, seed=742 + k, dtype="f32")


@pytest.mark.parametrize("E_local", [8, 3])
def test_ffn_fused_top2_parity(oracle, E_local):
    _say(f"ffn fused top-2 E_local={E_local}")
    _fused_case(oracle, 900, 128, 256, 8, E_local, 2, 0, True, seed=720 + E_local)


def test_ffn_fused_no_kept_assignment_clears_output(oracle):
    """Every token routed to an expert that lives elsewhere: the output is all zeros."""
    T, d, f = 300, 64, 128
    g = syn.rng(730)
    x = syn.quantize(g.standard_normal((T, d), dtype=np.float32), "bf16")
    w1 = to_dev(np.zeros((2, f, d), dtype=np.float32), "bf16")
    w2 = to_dev(np.zeros((2, d, f), dtype=np.float32), "bf16")
    idx = np.full((T, 1), 3, dtype=np.int32)
    expert_map = np.array([0, 1, -1, -1], dtype=np.int32)
    disp = exf.moe_dispatch(to_dev(x, "bf16"), torch.from_numpy(idx).to(DEV), 4, E_local=2,
                            expert_map=torch.from_numpy(expert_map).to(DEV), gather=False)
    out = torch.full((T, d), 7.0, dtype=torch.bfloat16, device=DEV)
    exf.moe_expert_ffn_fused(to_dev(x, "bf16"), disp.src_of_sorted, disp.sorted_of_src, torch.ones((T, 1), device=DEV),
                             disp.expert_offsets, w1, w2, out=out)
    assert (to_host(out) == 0).all()


# ----------------------------------------------------------------------------- affinity / locality
def _affinity_case(oracle, trace, E, placement=None, G=1):
    L, N = trace.shape
    res = exf.affinity_histogram(dev_i32(trace).reshape(L, N), E)
    counts, loads, n_inv = oracle.affinity_counts(trace, E)
    np.testing.assert_array_equal(res["counts"].cpu().numpy(), counts)
    np.testing.assert_array_equal(res["loads"].cpu().numpy(), loads)
    assert int(res["n_invalid"].cpu()) == n_inv
    prob = oracle.cond_prob(counts).astype(np.float32)
    got = res["cond_prob"].cpu().numpy()
    assert (np.abs(got - prob) <= np.spacing(prob)).all()  # <= 1 ulp
    if placement is not None and L > 1:
        loc = exf.placement_locality(dev_i32(trace).reshape(L, N), dev_i32(placement), G)
        np.testing.assert_array_equal(loc.cpu().numpy(), oracle.placement_locality(trace, placement))
        # both results from one pass over the trace; called twice into the same (first garbage-filled)
        # outputs: the locality numerators are accumulated, so they must start from zero every time
        both = None
        for _ in range(2):
            if both is not None:
                both["local_per_pair"].fill_(123456789)
            both = exf.affinity_statistics(dev_i32(trace).reshape(L, N), dev_i32(placement), G, out=both)
            np.testing.assert_array_equal(both["counts"].cpu().numpy(), counts)
            np.testing.assert_array_equal(both["loads"].cpu().numpy(), loads)
            assert int(both["n_invalid"].cpu()) == n_inv
            assert (np.abs(both["cond_prob"].cpu().numpy() - prob) <= np.spacing(prob)).all()
            np.testing.assert_array_equal(both["local_per_pair"].cpu().numpy(), oracle.placement_locality(trace, placement))


@pytest.mark.parametrize("L,N,E,G", [(2, 512, 8, 4), (12, 8192, 8, 4), (12, 16384, 32, 8), (5, 100001, 64, 8), (3, 70003, 16, 2),
                                     (2, 1, 1, 1), (7, 40000, 33, 3), (24, 131072, 64, 8)])
def test_affinity_and_locality_parity(oracle, L, N, E, G):
    _say(f"affinity L={L} N={N} E={E} G={G}")
    trace, perms = syn.planted_trace(L, N, E, 0.7, seed=700 + L + E, marginal="zipf" if E == 32 else "uniform")
    if E % G == 0:
        pl = syn.balanced_random_placement(L, E, G, seed=701)
    else:
        pl = syn.rng(702).integers(0, G, size=(L, E)).astype(np.int32)
    _affinity_case(oracle, trace, E, pl, G)


def test_affinity_invalid_ids_and_degenerate(oracle):
    _say("affinity invalid ids / degenerate shapes")
    L, N, E = 6, 30000, 16
    trace, _ = syn.planted_trace(L, N, E, 0.5, seed=710)
    g = syn.rng(711)
    bad = g.random((L, N)) < 0.01
    trace[bad] = g.choice(np.array([-1, E, 1 << 20, -(1 << 31)]), size=int(bad.sum())).astype(np.int32)
    pl = syn.balanced_random_placement(L, E, 4, seed=712)
    _affinity_case(oracle, trace, E, pl, 4)
    # a single layer: loads only
    t1, _ = syn.planted_trace(1, 5000, 8, 0.0, seed=713)
    t1[0, 17] = 99
    _affinity_case(oracle, t1, 8)
    # no tokens
    res = exf.affinity_histogram(torch.empty((4, 0), dtype=torch.int32, device=DEV), 8)
    assert (res["counts"].cpu().numpy() == 0).all() and (res["loads"].cpu().numpy() == 0).all()
    assert (res["cond_prob"].cpu().numpy() == 0).all() and int(res["n_invalid"].cpu()) == 0
    loc = exf.placement_locality(torch.empty((4, 0), dtype=torch.int32, device=DEV), dev_i32(np.zeros((4, 8))), 1)
    assert (loc.cpu().numpy() == 0).all()
    both = exf.affinity_statistics(torch.empty((4, 0), dtype=torch.int32, device=DEV), dev_i32(np.zeros((4, 8))), 1)
    assert (both["local_per_pair"].cpu().numpy() == 0).all() and (both["counts"].cpu().numpy() == 0).all()
    # deterministic routing: one hot column per row, and an aligned placement keeps every token local
    tr, perms = syn.planted_trace(5, 9999, 8, 1.0, seed=714)
    pl = syn.aligned_placement(perms, 8, 4)
    loc = exf.placement_locality(dev_i32(tr).reshape(5, 9999), dev_i32(pl), 4)
    assert (loc.cpu().numpy() == 9999).all()
    _affinity_case(oracle, tr, 8, pl, 4)


@pytest.mark.parametrize("L,N,E,G", [(6, 8000, 16, 4), (24, 5461, 64, 8), (3, 1000, 64, 8), (1, 131072, 8, 2), (2, 65536, 5, 5),
                                     (2, 65537, 5, 5)])
def test_affinity_short_traces_with_invalid_ids(oracle, L, N, E, G):
    """Short traces (one or two token chunks, several groups of layer pairs at 64 experts, a single
    layer) with ids outside [0,E) in every layer."""
    _say(f"affinity short trace L={L} N={N} E={E} G={G}")
    trace, _ = syn.planted_trace(L, N, E, 0.6, seed=730 + L + E)
    g = syn.rng(731 + N)
    bad = g.random((L, N)) < 0.02
    trace[bad] = g.choice(np.array([-1, E, 1 << 20, -(1 << 31)]), size=int(bad.sum())).astype(np.int32)
    pl = g.integers(0, G, size=(L, E)).astype(np.int32)
    _affinity_case(oracle, trace, E, pl, G)


def test_locality_paper_worked_example_on_gpu():
    # the 3-layer MoE-8 walk-through: default placement gpu = e // 2 keeps 2 of 4 transitions local
    trace = np.array([[0, 5], [4, 5], [2, 4]], dtype=np.int32)
    pl = syn.contiguous_placement(3, 8, 4)
    loc = exf.placement_locality(dev_i32(trace), dev_i32(pl), 4).cpu().numpy()
    assert loc.sum() == 2 and loc.tolist() == [1, 1]
    assert exf.affinity_statistics(dev_i32(trace), dev_i32(pl), 4)["local_per_pair"].cpu().numpy().tolist() == [1, 1]
    assert exf.check_placement(torch.from_numpy(pl), 4)


def test_repeat_calls_are_deterministic():
    trace, _ = syn.planted_trace(6, 50000, 64, 0.7, seed=720)
    t = dev_i32(trace).reshape(6, 50000)
    a = exf.affinity_histogram(t, 64)
    b = exf.affinity_histogram(t, 64)
    assert torch.equal(a["counts"], b["counts"]) and torch.equal(a["cond_prob"], b["cond_prob"])
    idx = dev_i32(trace[0].reshape(-1, 1).copy())
    x = torch.randn((50000, 64), device=DEV).to(torch.bfloat16)
    r1 = exf.moe_dispatch(x, idx, 64)
    r2 = exf.moe_dispatch(x, idx, 64)
    assert torch.equal(r1.src_of_sorted, r2.src_of_sorted) and torch.equal(r1.x_sorted, r2.x_sorted)
    # expert FFN with remainder tiles in K slices (the slices are added in a fixed order), through both
    # entry points, with the workspace overwritten between the calls
    g = syn.rng(721)
    T, d, f, E = 2100, 128, 1024, 6
    xs = to_dev(g.standard_normal((T, d), dtype=np.float32), "bf16")
    w1 = to_dev(g.standard_normal((E, f, d), dtype=np.float32) * np.float32(0.05), "bf16")
    w2 = to_dev(g.standard_normal((E, d, f), dtype=np.float32) * np.float32(0.05), "bf16")
    idx = dev_i32(g.integers(0, E, size=(T, 1)))
    gate = torch.rand((T, 1), device=DEV)
    disp = exf.moe_dispatch(xs, idx, E)
    nbytes = max(exf.lib().moe_expert_ffn_workspace_bytes(T, d, f, E, exf.EXF_BF16),
                 exf.lib().moe_expert_ffn_fused_workspace_bytes(T, 1, d, f, E, exf.EXF_BF16))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    outs = []
    for fill in (0, 255):
        ws.fill_(fill)
        y = exf.moe_expert_ffn(disp.x_sorted, disp.expert_offsets, w1, w2, workspace=ws)
        ws.fill_(255 - fill)
        o = exf.moe_expert_ffn_fused(xs, disp.src_of_sorted, disp.sorted_of_src, gate, disp.expert_offsets, w1, w2, workspace=ws)
        outs.append((y.clone(), o.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


def test_trace_reductions_repeat_on_one_workspace(oracle):
    """placement_locality and routing_transfers keep per-chunk counts in the workspace: many calls in
    a row on one workspace, of changing size, with the workspace filled with zeros, ones, and whatever
    the previous call left, must all give the oracle's counts; then 50 calls queued back to back."""
    _say("trace reductions: repeated calls on one workspace")
    L, E, G = 7, 32, 4
    g = syn.rng(730)
    cases = []
    for N in (300000, 4096, 1, 70001, 300000):
        trace = g.integers(0, E, size=(L, N)).astype(np.int32)
        pl = syn.balanced_random_placement(L, E, G, 731 + N % 7)
        home = g.integers(0, G, size=N).astype(np.int32)
        cases.append((dev_i32(trace).reshape(L, N), dev_i32(pl).reshape(L, E), dev_i32(home), oracle.placement_locality(trace, pl),
                      oracle.routing_away(trace, pl, home)))
    nbytes = max(exf.lib().routing_transfers_workspace_bytes(L, 300000), exf.lib().placement_locality_workspace_bytes(L, 300000))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    for rep in range(12):
        if rep < 3:
            ws.fill_((0, 255, 1)[rep])
        for t, p, h, loc_ref, away_ref in cases:
            loc = exf.placement_locality(t, p, G, workspace=ws)
            np.testing.assert_array_equal(loc.cpu().numpy(), loc_ref)
            loc2, away = exf.routing_transfers(t, p, h, G, workspace=ws)
            np.testing.assert_array_equal(loc2.cpu().numpy(), loc_ref)
            np.testing.assert_array_equal(away.cpu().numpy(), away_ref)
    # back to back without host synchronisation in between: 50 calls queued on the stream, every result kept
    t, p, h, loc_ref, away_ref = cases[0]
    outs = [exf.placement_locality(t, p, G, workspace=ws) for _ in range(50)]
    torch.cuda.synchronize()
    for o in outs:
        np.testing.assert_array_equal(o.cpu().numpy(), loc_ref)
