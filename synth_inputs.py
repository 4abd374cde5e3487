"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds NO arithmetic of the method: it only draws random tensors, routing traces
and placements with the shapes and distributions of GPT-MoE workloads (Table "List of MoE
models": D = 1024 / 2048, E = 8 .. 64 experts, top-1 gating) and stores them in the dtype
the path consumes.  They stand in for the trained checkpoints and Pile-derived routing
traces of the paper, which are not available.

Generator: NumPy ``Generator(Philox(key=seed))``; seed = 1000*config + tensor index
(x=0, Wg=1, W1=2, W2=3, trace=4, placement=5, trace model=6) + 100*layer.
Values are drawn in fp32 and rounded once (round-to-nearest-even) to the storage dtype; the
rounded array is what both the GPU path and the CPU checker receive.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


# --------------------------------------------------------------------------- dtypes
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(a: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 array holding values exactly representable in ``dtype`` ('f32' or 'bf16')."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    return a


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=seed))


# --------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class MoEConfig:
    index: int
    name: str
    T: int          # tokens per layer
    d: int          # d_model
    f: int          # d_ff
    E: int          # experts seen by the gate
    E_local: int    # experts resident on this GPU
    k: int          # top-k
    renormalize: bool
    dtype: str      # 'f32' | 'bf16'
    layers: int     # consecutive MoE layers run by the workload
    gate_std: float  # std of the gate weights
    trace_L: int    # routing trace: MoE layers (0 = no affinity part)
    trace_N: int
    trace_E: int
    G: int          # devices of the placement scored by placement_locality


CONFIGS = {
    1: MoEConfig(1, "tiny-fp32", 512, 64, 256, 8, 8, 1, False, "f32", 1, 0.02, 2, 512, 8, 4),
    2: MoEConfig(2, "gpt-moe-350m", 8192, 1024, 4096, 8, 8, 1, False, "bf16", 1, 0.02, 12, 8192, 8, 4),
    3: MoEConfig(3, "gpt-moe-xl-skewed", 16384, 2048, 8192, 32, 32, 1, False, "bf16", 1, 0.02, 12, 16384, 32, 8),
    4: MoEConfig(4, "e64-share-8-local", 32768, 1024, 4096, 64, 8, 1, False, "bf16", 1, 0.02, 24, 1 << 20, 64, 8),
    5: MoEConfig(5, "decode-top2", 256, 4096, 16384, 64, 64, 2, True, "bf16", 8, 1.0 / 64.0, 0, 0, 0, 0),
}


def seed_for(config: int, tensor: int, layer: int = 0) -> int:
    return 1000 * config + tensor + 100 * layer


def tokens(cfg: MoEConfig, layer: int = 0, T: int | None = None) -> np.ndarray:
    """x ~ N(0,1), [T,d]."""
    T = cfg.T if T is None else T
    return quantize(rng(seed_for(cfg.index, 0, layer)).standard_normal((T, cfg.d), dtype=np.float32), cfg.dtype)


def gate_weight(cfg: MoEConfig, layer: int = 0) -> np.ndarray:
    """Wg ~ N(0, gate_std), [E,d].  (Config 5: std = 1/sqrt(d) so that logits ~ N(0,1).)"""
    w = rng(seed_for(cfg.index, 1, layer)).standard_normal((cfg.E, cfg.d), dtype=np.float32) * np.float32(cfg.gate_std)
    return quantize(w, cfg.dtype)


def expert_weights(cfg: MoEConfig, layer: int = 0, E_local: int | None = None):
    """W1 [E_local,f,d], W2 [E_local,d,f] ~ N(0,0.02)."""
    E_local = cfg.E_local if E_local is None else E_local
    g1 = rng(seed_for(cfg.index, 2, layer))
    g2 = rng(seed_for(cfg.index, 3, layer))
    w1 = np.empty((E_local, cfg.f, cfg.d), dtype=np.float32)
    w2 = np.empty((E_local, cfg.d, cfg.f), dtype=np.float32)
    for e in range(E_local):  # expert by expert keeps the fp32 staging copy small
        w1[e] = quantize(g1.standard_normal((cfg.f, cfg.d), dtype=np.float32) * np.float32(0.02), cfg.dtype)
        w2[e] = quantize(g2.standard_normal((cfg.d, cfg.f), dtype=np.float32) * np.float32(0.02), cfg.dtype)
    return w1, w2


def device_expert_weights(cfg: MoEConfig, layer: int, device: str):
    """W1 [E_local,f,d], W2 [E_local,d,f] ~ N(0,0.02) drawn ON THE DEVICE in the storage dtype (torch's
    seeded device generator).  For configurations whose weights are too large to draw on the host
    in reasonable time (the decode-shaped one: 17 GB per layer); checks copy back the experts they need."""
    import torch

    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    out = []
    for tensor, shape in ((2, (cfg.E_local, cfg.f, cfg.d)), (3, (cfg.E_local, cfg.d, cfg.f))):
        g = torch.Generator(device=device)
        g.manual_seed(seed_for(cfg.index, tensor, layer))
        w = torch.empty(shape, dtype=dt, device=device)
        w.normal_(0.0, 0.02, generator=g)
        out.append(w)
    return out[0], out[1]


# --------------------------------------------------------------------------- routing traces
def zipf_loads(E: int, s: float) -> np.ndarray:
    p = 1.0 / np.arange(1, E + 1, dtype=np.float64) ** s
    return p / p.sum()


def planted_trace(L: int, N: int, E: int, rho: float, seed: int, marginal: str = "uniform",
                  zipf_s: float = 1.1, dirichlet_alpha: float = 0.5):
    """Routing trace int32 [L,N] with planted inter-layer affinity.

    Layer 0 is drawn from the marginal (uniform, or Zipf(s) over a random expert order).
    For each later layer: with probability rho the token goes to perm_l(previous expert),
    otherwise to an expert drawn from q_l (uniform, or Dirichlet(alpha)-distributed for the
    'zipf' recipe).  Returns (trace, perms [L-1,E]).
    """
    g = rng(seed)
    trace = np.empty((L, N), dtype=np.int32)
    if marginal == "zipf":
        order = g.permutation(E)
        first = order[g.choice(E, size=N, p=zipf_loads(E, zipf_s))]
    else:
        first = g.integers(0, E, size=N)
    trace[0] = first.astype(np.int32)
    perms = np.empty((max(L - 1, 0), E), dtype=np.int32)
    for l in range(1, L):
        perm = g.permutation(E).astype(np.int32)
        perms[l - 1] = perm
        follow = g.random(N) < rho
        if marginal == "zipf":
            q = g.dirichlet(np.full(E, dirichlet_alpha))
            other = g.choice(E, size=N, p=q)
        else:
            other = g.integers(0, E, size=N)
        trace[l] = np.where(follow, perm[trace[l - 1]], other).astype(np.int32)
    return trace, perms


def config_trace(cfg: MoEConfig):
    """The routing trace of a config (None if it has no affinity part)."""
    if cfg.trace_L == 0:
        return None, None
    marginal = "zipf" if cfg.index == 3 else "uniform"
    return planted_trace(cfg.trace_L, cfg.trace_N, cfg.trace_E, 0.7, seed_for(cfg.index, 4), marginal)


def balanced_random_placement(L: int, E: int, G: int, seed: int) -> np.ndarray:
    """int32 [L,E]: per layer a random permutation of the experts cut into G equal chunks
    (every device holds E/G experts of every layer, every expert sits on one device)."""
    assert E % G == 0
    g = rng(seed)
    pl = np.empty((L, E), dtype=np.int32)
    for l in range(L):
        order = g.permutation(E)
        pl[l, order] = np.arange(E, dtype=np.int32) // (E // G)
    return pl


def contiguous_placement(L: int, E: int, G: int) -> np.ndarray:
    """Framework-default placement: expert e of every layer on device e // (E/G)."""
    return np.tile((np.arange(E, dtype=np.int32) // (E // G))[None, :], (L, 1))


def aligned_placement(perms: np.ndarray, E: int, G: int) -> np.ndarray:
    """Placement that follows the planted permutations: layer 0 contiguous, then
    device(l+1, perm_l[e]) = device(l, e)."""
    L = perms.shape[0] + 1
    pl = np.empty((L, E), dtype=np.int32)
    pl[0] = np.arange(E, dtype=np.int32) // (E // G)
    for l in range(L - 1):
        pl[l + 1, perms[l]] = pl[l]
    return pl


def local_routing(cfg: MoEConfig, seed: int):
    """Config 4: this GPU's post-exchange share.  Picks E_local of the E global experts
    as resident (a random placement row), draws global ids uniformly among them, and
    returns (topk_idx [T,1] global ids, expert_map [E] global -> local or -1)."""
    g = rng(seed)
    resident = np.sort(g.permutation(cfg.E)[: cfg.E_local]).astype(np.int32)
    expert_map = np.full(cfg.E, -1, dtype=np.int32)
    expert_map[resident] = np.arange(cfg.E_local, dtype=np.int32)
    idx = resident[g.integers(0, cfg.E_local, size=(cfg.T, cfg.k))].astype(np.int32)
    return idx, expert_map
