"""The five workload configurations at their full sizes, run through the same pre-allocated
pipeline the benchmark times, and checked against the CPU oracle: integer outputs in full,
floating-point outputs on a stratified sample of rows the oracle evaluates one by one (every block
of 64 rows of every expert holds sampled rows, at least 1024 rows at the two large prefill
configurations; every row of the first decode layer)."""
import numpy as np
import pytest
import torch

import paper_2401_08383_amd as exf
import synth_inputs as syn
from helpers import (DEV, GATE_TOL, OUT_RTOL, STRATUM_ROWS, assert_close_max, dev_i32, oracle_routing, sample_rows, strata_covered, to_dev, to_host)
from paper_2401_08383_amd.pipeline import AffinityRun, MoELayerRun

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _ffn_rows_ref(oracle, xs_ref, offsets, w1, w2, rows, d):
    """Oracle FFN of the sorted rows `rows`.  w1/w2: host fp32 arrays, or device tensors from which only
    the experts that own a row are copied back (one at a time)."""
    if isinstance(w1, np.ndarray):
        return oracle.expert_ffn_rows(xs_ref, offsets, w1, None, w2, None, 0, rows)
    y_ref = np.zeros((len(rows), d))
    owner = np.searchsorted(offsets, rows, side="right") - 1
    for e in np.unique(owner):
        sel = np.nonzero(owner == e)[0]
        w1e = w1[e].float().cpu().numpy()[None]
        w2e = w2[e].float().cpu().numpy()[None]
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        y_ref[sel] = oracle.expert_ffn_rows(xs_ref[lo:hi], np.array([0, hi - lo], dtype=np.int32), w1e, None, w2e, None, 0, rows[sel] - lo)
    return y_ref


def _check_chain(oracle, cfg, layer, x, w1, w2, ref, w_ref, rows, seed, dense=True):
    """Expert FFN and layer output of one executed MoELayerRun against the oracle chain gather -> FFN ->
    combine, which is fed by the seeded inputs and the oracle's own routing, dispatch and gate weights:
    sampled sorted rows, then every sorted row of the tokens that own them, then those tokens' outputs."""
    dtype, k, T = cfg.dtype, cfg.k, cfg.T
    kept = ref["kept"]
    xs_ref = x[ref["src_of_sorted"] // k]
    np.testing.assert_array_equal(to_host(layer.x_sorted)[:kept], xs_ref)  # a pure copy: bit-exact
    inv = ref["sorted_of_src"].reshape(T, k)
    toks = np.unique(ref["src_of_sorted"][rows] // k)
    pos = inv[toks]
    rows_all = np.unique(np.concatenate([rows, pos[pos >= 0]]))
    y_ref = _ffn_rows_ref(oracle, xs_ref, ref["offsets"], w1, w2, rows_all, cfg.d)
    y = to_host(layer.y_sorted)
    n_strata, n_hit = strata_covered(ref["offsets"], rows_all)
    _say(f"    expert FFN: {len(rows_all)} of {kept} sorted rows evaluated by the oracle, "
         f"{n_hit} of {n_strata} blocks of {STRATUM_ROWS} rows, {len(np.unique(np.searchsorted(ref['offsets'], rows_all, side='right') - 1))} experts")
    assert n_hit == n_strata or not dense, "the sample must reach every block of every expert"
    assert_close_max(y[rows_all], y_ref, OUT_RTOL[dtype], "expert FFN rows")
    # the sampled tokens as a layer of their own: their sorted rows renumbered into y_ref
    inv_small = np.where(pos >= 0, np.searchsorted(rows_all, np.maximum(pos, 0)), -1).astype(np.int32)
    w_small = np.ascontiguousarray(w_ref[toks], dtype=np.float64)
    out_ref = oracle.combine(y_ref, inv_small, w_small)
    mag = oracle.combine(np.abs(y_ref), inv_small, np.abs(w_small))
    assert_close_max(to_host(layer.out)[toks], out_ref, OUT_RTOL[dtype], "layer output of sampled tokens", mag=mag)
    # the combine alone at the full size, on seeded expert outputs: one rounding to storage after an
    # fp32 sum of k terms, relative to the summands
    g = syn.rng(seed + 1000)
    y_syn = syn.quantize(g.standard_normal((T * k, cfg.d), dtype=np.float32), dtype)
    w32 = np.ascontiguousarray(w_ref, dtype=np.float32)
    got = to_host(exf.moe_combine(to_dev(y_syn, dtype), dev_i32(ref["sorted_of_src"]), torch.from_numpy(w32).to(DEV)))
    full_ref = oracle.combine(y_syn, ref["sorted_of_src"], w32)
    full_mag = oracle.combine(np.abs(y_syn), ref["sorted_of_src"], np.abs(w32))
    eps = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -22
    assert (np.abs(got - full_ref) <= eps * full_mag + 1e-30).all(), "combine"


def _check_layer(oracle, cfg, layer, x, wg, w1, w2, forced_idx=None, combine_w=None, expert_map=None, per_stratum=1, min_rows=0, seed=0):
    """Compares one executed MoELayerRun with the oracle.  Routing: the oracle's own (checked to be what
    the GPU decided), or `forced_idx` with the combine weights `combine_w` the caller gave the run.
    w1/w2: host fp32 arrays or device tensors."""
    k, E, E_local = cfg.k, cfg.E, cfg.E_local
    if forced_idx is None:
        idx, w_ref, _ = oracle_routing(oracle, x, wg, k, cfg.renormalize, layer.topk_idx.cpu().numpy(), layer.topk_w.cpu().numpy(),
                                       GATE_TOL[cfg.dtype])
    else:
        idx, w_ref = forced_idx, combine_w
    ref = oracle.dispatch(idx, expert_map, E, E_local)
    kept = ref["kept"]
    np.testing.assert_array_equal(layer.expert_counts.cpu().numpy(), ref["counts"])
    np.testing.assert_array_equal(layer.expert_offsets.cpu().numpy(), ref["offsets"])
    np.testing.assert_array_equal(layer.src_of_sorted.cpu().numpy()[:kept], ref["src_of_sorted"])
    np.testing.assert_array_equal(layer.sorted_of_src.cpu().numpy(), ref["sorted_of_src"])
    _check_chain(oracle, cfg, layer, x, w1, w2, ref, w_ref, sample_rows(ref["offsets"], per_stratum, seed, min_rows), seed)
    ref["w_ref"] = w_ref
    return ref


def _check_fused(oracle, cfg, plain, x, w1, w2, ref, per_stratum, seed, min_rows=0):
    """The same layer through moe_expert_ffn_fused (index-only dispatch): sampled tokens against the
    oracle's gather -> FFN -> combine, every token against the three-call path (which differs by one
    extra rounding of the expert output when k = 1 and not at all when k > 1)."""
    k = cfg.k
    fused = MoELayerRun(plain.x, plain.w_gate, plain.w1, plain.w2, k, cfg.renormalize, expert_map=plain.expert_map,
                        topk_idx=plain.forced_idx, fused=True)
    fused.out.fill_(7.0)
    fused.topk_idx.copy_(plain.topk_idx)  # the gate is not what differs: take its result as the plain run has it
    fused.topk_w.copy_(plain.topk_w)
    fused.dispatch()
    fused.ffn()
    fused.combine()
    np.testing.assert_array_equal(fused.sorted_of_src.cpu().numpy(), ref["sorted_of_src"])
    np.testing.assert_array_equal(fused.expert_offsets.cpu().numpy(), ref["offsets"])
    out = to_host(fused.out)
    out_plain = to_host(plain.out)
    if k == 1:
        assert (np.abs(out - out_plain) <= 2.0 ** -7 * np.abs(out_plain) + 1e-30).all(), "fused against the three-call path"
    else:
        np.testing.assert_array_equal(out, out_plain)
    unrouted = (ref["sorted_of_src"].reshape(cfg.T, k) < 0).all(axis=1)
    assert (out[unrouted] == 0).all()
    if k != 1 or not isinstance(w1, np.ndarray):
        return
    rows = sample_rows(ref["offsets"], per_stratum, seed, min_rows)
    toks = ref["src_of_sorted"][rows]
    w = ref["w_ref"]
    xs = x[ref["src_of_sorted"]]
    y_ref = oracle.expert_ffn_rows(xs, ref["offsets"], w1, None, w2, None, 0, rows)
    out_ref = w[toks, 0][:, None].astype(np.float64) * y_ref
    n_strata, n_hit = strata_covered(ref["offsets"], rows)
    _say(f"    fused layer: {len(rows)} tokens evaluated by the oracle, {n_hit} of {n_strata} blocks of {STRATUM_ROWS} rows")
    assert n_hit == n_strata
    assert_close_max(out[toks], out_ref, OUT_RTOL[cfg.dtype], "fused layer output rows")


def _check_affinity(oracle, cfg, trace, placement):
    frac = None
    for one_pass in (True, False):  # affinity_statistics, then affinity_histogram + placement_locality
        frac = _check_affinity_run(oracle, cfg, trace, placement, one_pass)
    return frac


def _check_affinity_run(oracle, cfg, trace, placement, one_pass):
    aff = AffinityRun(torch.from_numpy(trace).to(DEV), torch.from_numpy(placement).to(DEV), cfg.trace_E, cfg.G, one_pass=one_pass)
    aff.step()
    counts, loads, n_inv = oracle.affinity_counts(trace, cfg.trace_E)
    np.testing.assert_array_equal(aff.counts.cpu().numpy(), counts)
    np.testing.assert_array_equal(aff.loads.cpu().numpy(), loads)
    assert int(aff.n_invalid.cpu()) == n_inv == 0
    prob = oracle.cond_prob(counts).astype(np.float32)
    assert (np.abs(aff.cond_prob.cpu().numpy() - prob) <= np.spacing(prob)).all()
    loc = aff.local_per_pair.cpu().numpy()
    np.testing.assert_array_equal(loc, oracle.placement_locality(trace, placement))
    np.testing.assert_array_equal(loc, oracle.placement_locality_from_counts(counts, placement))
    return loc.sum() / (trace.shape[1] * (trace.shape[0] - 1))


def test_config2_gpt_moe_350m(oracle):
    cfg = syn.CONFIGS[2]
    _say("config 2: T=8192 d=1024 f=4096 E=8 top-1 bf16")
    x, wg = syn.tokens(cfg), syn.gate_weight(cfg)
    w1, w2 = syn.expert_weights(cfg)
    layer = MoELayerRun(to_dev(x, "bf16"), to_dev(wg, "bf16"), to_dev(w1, "bf16"), to_dev(w2, "bf16"), cfg.k, cfg.renormalize)
    layer.step()
    ref = _check_layer(oracle, cfg, layer, x, wg, w1, w2, per_stratum=2, seed=21)
    assert ref["counts"].min() > 800  # the synthetic gate is roughly balanced, as trained models are
    _check_fused(oracle, cfg, layer, x, w1, w2, ref, per_stratum=2, seed=22)
    trace, perms = syn.config_trace(cfg)
    frac = _check_affinity(oracle, cfg, trace, syn.balanced_random_placement(cfg.trace_L, cfg.trace_E, cfg.G, syn.seed_for(2, 5)))
    assert abs(frac - 1 / cfg.G) < 0.15  # few (88) hot transitions: a wide band around 1/G
    aligned = _check_affinity(oracle, cfg, trace, syn.aligned_placement(perms, cfg.trace_E, cfg.G))
    assert aligned > 0.7  # a placement that follows the planted affinity keeps most tokens local


def test_config3_xl_skewed(oracle):
    cfg = syn.CONFIGS[3]
    _say("config 3: T=16384 d=2048 f=8192 E=32 top-1 bf16, Zipf loads from the trace")
    x, wg = syn.tokens(cfg), syn.gate_weight(cfg)
    _say("  drawing expert weights (2 x 2.1 GB on the host)")
    w1, w2 = syn.expert_weights(cfg)
    trace, _ = syn.config_trace(cfg)
    forced = trace[0].reshape(-1, 1).copy()
    xd = to_dev(x, "bf16")
    # the gate is checked on x as it stands; the oracle's probabilities of the forced experts weight the combine
    idx_g, w_g, _ = exf.moe_gate_topk(xd, to_dev(wg, "bf16"), 1, False)
    _, _, logits64 = oracle_routing(oracle, x, wg, 1, False, idx_g.cpu().numpy(), w_g.cpu().numpy(), GATE_TOL["bf16"])
    forced_w = np.take_along_axis(oracle.softmax(logits64), forced.astype(np.int64), axis=1).astype(np.float32)
    layer = MoELayerRun(xd, to_dev(wg, "bf16"), to_dev(w1, "bf16"), to_dev(w2, "bf16"), 1, False,
                        topk_idx=torch.from_numpy(forced).to(DEV))
    layer.topk_w.copy_(torch.from_numpy(forced_w))
    layer.dispatch()
    layer.ffn()
    layer.combine()
    _say("  oracle on sampled rows")
    ref = _check_layer(oracle, cfg, layer, x, wg, w1, w2, forced_idx=forced, combine_w=forced_w, per_stratum=3, min_rows=1024, seed=31)
    assert ref["counts"].max() > 10 * max(1, ref["counts"].min())  # skewed loads
    _check_fused(oracle, cfg, layer, x, w1, w2, ref, per_stratum=1, seed=32)
    _check_affinity(oracle, cfg, trace, syn.balanced_random_placement(cfg.trace_L, cfg.trace_E, cfg.G, syn.seed_for(3, 5)))


def test_config4_one_gpu_share(oracle):
    cfg = syn.CONFIGS[4]
    _say("config 4: T=32768 d=1024 f=4096, 8 local of 64 experts, bf16; 24 x 1M trace")
    x, wg = syn.tokens(cfg), syn.gate_weight(cfg)
    w1, w2 = syn.expert_weights(cfg)
    idx, expert_map = syn.local_routing(cfg, syn.seed_for(4, 4, 1))
    xd, wgd = to_dev(x, "bf16"), to_dev(wg, "bf16")
    layer = MoELayerRun(xd, wgd, to_dev(w1, "bf16"), to_dev(w2, "bf16"), 1, False, expert_map=torch.from_numpy(expert_map).to(DEV),
                        topk_idx=torch.from_numpy(idx).to(DEV))
    layer.gate()  # the shared gate over all 64 experts on the tokens this GPU holds
    _, w_gate, _ = oracle_routing(oracle, x, wg, 1, False, layer.topk_idx.cpu().numpy(), layer.topk_w.cpu().numpy(), GATE_TOL["bf16"])
    layer.dispatch()  # post-exchange share: every token is routed to one of the 8 resident experts
    layer.ffn()
    layer.combine()
    ref = _check_layer(oracle, cfg, layer, x, wg, w1, w2, forced_idx=idx, combine_w=w_gate, expert_map=expert_map, per_stratum=2,
                       min_rows=1024, seed=41)
    assert ref["kept"] == cfg.T
    _check_fused(oracle, cfg, layer, x, w1, w2, ref, per_stratum=1, seed=43)
    # the same layer fed with the gate's own routing: 7 of 8 tokens belong to other GPUs and are dropped here
    layer2 = MoELayerRun(xd, wgd, layer.w1, layer.w2, 1, False, expert_map=layer.expert_map)
    layer2.step()
    ref2 = _check_layer(oracle, cfg, layer2, x, wg, w1, w2, expert_map=expert_map, per_stratum=2, seed=42)
    assert 0 < ref2["kept"] < cfg.T // 4
    dropped = ref2["sorted_of_src"] < 0
    assert (to_host(layer2.out)[dropped] == 0).all()
    _check_fused(oracle, cfg, layer2, x, w1, w2, ref2, per_stratum=1, seed=44)
    _say("  affinity on the 24 x 1M trace")
    trace, _ = syn.config_trace(cfg)
    frac = _check_affinity(oracle, cfg, trace, syn.balanced_random_placement(cfg.trace_L, cfg.trace_E, cfg.G, syn.seed_for(4, 5)))
    assert abs(frac - 1 / cfg.G) < 0.03  # without placement optimisation any GPU is equally likely


def test_config5_decode_top2(oracle):
    cfg = syn.CONFIGS[5]
    _say("config 5: T=256 d=4096 f=16384 E=64 top-2 renormalised, 8 layers with distinct weights (137 GB)")
    free, _ = torch.cuda.mem_get_info()
    layers = cfg.layers if free > 150e9 else 2  # the weights of all 8 layers need 137 GB of HBM
    _say(f"  {layers} of {cfg.layers} layers resident ({free / 1e9:.0f} GB of HBM free)" +
         ("" if layers == cfg.layers else ": REDUCED CASE, the configuration is only partly covered"))
    runs = []
    for l in range(layers):
        x, wg = syn.tokens(cfg, l), syn.gate_weight(cfg, l)
        w1, w2 = syn.device_expert_weights(cfg, l, DEV)
        runs.append((x, wg, w1, w2, MoELayerRun(to_dev(x, "bf16"), to_dev(wg, "bf16"), w1, w2, cfg.k, cfg.renormalize)))
    for r in runs:  # consecutive layers back to back on one stream, no host synchronisation
        r[4].step()
    torch.cuda.synchronize()
    for l, (x, wg, w1, w2, layer) in enumerate(runs):
        w = layer.topk_w.cpu().numpy()
        np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=1e-6)  # renormalised top-2 gates
        idx, w_ref, _ = oracle_routing(oracle, x, wg, cfg.k, cfg.renormalize, layer.topk_idx.cpu().numpy(), w, GATE_TOL["bf16"])
        ref = oracle.dispatch(idx, None, cfg.E, cfg.E_local)
        assert ref["kept"] == cfg.T * cfg.k
        np.testing.assert_array_equal(layer.expert_offsets.cpu().numpy(), ref["offsets"])
        np.testing.assert_array_equal(layer.src_of_sorted.cpu().numpy(), ref["src_of_sorted"])
        np.testing.assert_array_equal(layer.sorted_of_src.cpu().numpy(), ref["sorted_of_src"])
        if l == 0:
            # the first layer in full: all 512 sorted rows, i.e. every expert that received a token
            # (the experts' weights come back from the device one expert at a time, 2 x 256 MB each)
            rows = np.arange(ref["kept"], dtype=np.int64)
            _say(f"  layer 0: oracle on all {len(rows)} sorted rows, {int((ref['counts'] > 0).sum())} of {cfg.E} experts have rows")
            _check_chain(oracle, cfg, layer, x, w1, w2, ref, w_ref, rows, 50)
            ref["w_ref"] = w_ref
            _check_fused(oracle, cfg, layer, x, w1, w2, ref, per_stratum=0, seed=0)
        else:
            # later layers: two random tokens, whose four sorted rows lie in at most four experts
            toks = syn.rng(50 + l).choice(cfg.T, size=2, replace=False)
            rows = np.sort(ref["sorted_of_src"].reshape(cfg.T, cfg.k)[toks].ravel()).astype(np.int64)
            _say(f"  layer {l}: oracle on the sorted rows of tokens {toks.tolist()}")
            _check_chain(oracle, cfg, layer, x, w1, w2, ref, w_ref, rows, 50 + l, dense=False)
