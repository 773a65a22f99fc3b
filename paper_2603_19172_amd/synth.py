"""Seeded synthetic inputs for the DyMoE MoE-layer workloads.

This module only draws random tensors and rounds them to bf16; it holds none
of the method's arithmetic and is the one module both the GPU tests and the
CPU oracle's tests read their inputs from.  Tensors are numpy arrays; bf16
tensors travel as uint16 bit patterns so that every consumer sees the same
bytes.

The paper measures on ShareGPT prompts through trained Mixtral-8x7B and
Qwen3-30B-A3B (its Sec. 6.1).  Neither is available here, so the workloads
take those models' layer shapes and the qualitative structure the paper
reports (a few percent of heavy-hitter tokens, skewed expert load; Sec. 3.1)
and fill them with seeded Gaussians.
"""
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 20260319

# tensor ids (mixed into the Philox key)
_TID_X, _TID_WG, _TID_HEAVY, _TID_BIAS = 1, 2, 3, 4
_TID_EXPERT = 1000  # + 3*e + {0: W1, 1: W3, 2: W2}


@dataclass(frozen=True)
class MoEConfig:
    """One MoE layer workload (shapes follow the benchmark's configs)."""
    name: str
    config_id: int
    T: int            # tokens in the step
    H: int            # hidden size
    F: int            # expert SwiGLU width
    E: int            # experts
    k: int            # experts per token
    phase: str        # "prefill" or "decode"
    tier_count: Tuple[int, ...]   # experts per tier, best first
    tier_bits: Tuple[int, ...] = (16, 4, 2)
    k_hh: int = 0     # heavy-hitter tokens (prefill)
    heavy_scale: float = 1.0      # heavy-hitter rows are multiplied by this
    zipf_bias: float = 0.0        # router bias  -zipf_bias * ln(rank_e)
    group: int = 64
    weight_std: float = 0.02


CONFIGS = {
    # tiny layer, every element checked
    "tiny": MoEConfig("tiny", 1, T=16, H=256, F=512, E=8, k=2, phase="prefill",
                      tier_count=(2, 3, 3), k_hh=1),
    # Mixtral-8x7B-shaped layer, decode, one token
    "mixtral_decode": MoEConfig("mixtral_decode", 2, T=1, H=4096, F=14336, E=8, k=2,
                                phase="decode", tier_count=(1, 3, 4)),
    # Mixtral-8x7B-shaped layer, prefill of 512 tokens, 26 heavy hitters scaled x8
    "mixtral_prefill": MoEConfig("mixtral_prefill", 3, T=512, H=4096, F=14336, E=8, k=2,
                                 phase="prefill", tier_count=(1, 3, 4), k_hh=26,
                                 heavy_scale=8.0),
    # fine-grained layer: 128 experts top-8, Zipf(1.2)-skewed router bias
    "fine_grained": MoEConfig("fine_grained", 4, T=2048, H=2048, F=768, E=128, k=8,
                              phase="prefill", tier_count=(13, 39, 76), k_hh=103,
                              zipf_bias=1.2),
}


def scaled(cfg: MoEConfig, **kw) -> MoEConfig:
    """A copy of cfg with some fields replaced (reduced sizes for CPU tests)."""
    d = dict(cfg.__dict__)
    d.update(kw)
    return MoEConfig(**d)


def _rng(config_id: int, tensor_id: int) -> np.random.Generator:
    # Philox is counter based: the stream depends only on the key.
    return np.random.Generator(np.random.Philox(key=[BASE_SEED, (config_id << 32) | tensor_id]))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u >> np.uint32(16)
    r &= np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    # the rounded value is the high half of each little-endian word
    return np.ascontiguousarray(r.view(np.uint16).reshape(u.shape + (2,))[..., 1])


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(config_id: int, tensor_id: int, shape, std: float) -> np.ndarray:
    g = _rng(config_id, tensor_id)
    a = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return f32_to_bf16_bits(a)


def activations(cfg: MoEConfig) -> Tuple[np.ndarray, np.ndarray]:
    """x [T,H] bf16 bits ~ N(0,1); k_hh seeded rows multiplied by heavy_scale
    (a power of two, so the product is exact).  Returns (x, heavy_rows)."""
    x = normal_bf16(cfg.config_id, _TID_X, (cfg.T, cfg.H), 1.0)
    heavy = np.zeros(0, np.int64)
    if cfg.heavy_scale != 1.0 and cfg.k_hh > 0:
        g = _rng(cfg.config_id, _TID_HEAVY)
        heavy = np.sort(g.permutation(cfg.T)[:cfg.k_hh])
        xf = bf16_bits_to_f32(x)
        xf[heavy] *= np.float32(cfg.heavy_scale)
        x = f32_to_bf16_bits(xf)
    return x, heavy


def router(cfg: MoEConfig) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Wg [E,H] bf16 bits ~ N(0, weight_std); bias [E] float32 or None."""
    wg = normal_bf16(cfg.config_id, _TID_WG, (cfg.E, cfg.H), cfg.weight_std)
    bias = None
    if cfg.zipf_bias != 0.0:
        g = _rng(cfg.config_id, _TID_BIAS)
        rank = g.permutation(cfg.E) + 1
        bias = (-cfg.zipf_bias * np.log(rank.astype(np.float64))).astype(np.float32)
    return wg, bias


def expert_matrix(cfg: MoEConfig, e: int, i: int) -> np.ndarray:
    """Matrix i (0: W1 [F,H], 1: W3 [F,H], 2: W2 [H,F]) of expert e, bf16 bits ~ N(0, weight_std)."""
    shape = (cfg.F, cfg.H) if i < 2 else (cfg.H, cfg.F)
    return normal_bf16(cfg.config_id, _TID_EXPERT + 3 * e + i, shape, cfg.weight_std)


def expert_weights(cfg: MoEConfig, e: int) -> List[np.ndarray]:
    """[W1 [F,H], W3 [F,H], W2 [H,F]] bf16 bits ~ N(0, weight_std)."""
    return [expert_matrix(cfg, e, i) for i in range(3)]


def expert_weights_many(cfg: MoEConfig, experts, workers: int = 8):
    """{e: [W1, W3, W2]} for several experts, drawn on a thread pool (every
    matrix has its own key, so the bytes do not depend on the schedule)."""
    from concurrent.futures import ThreadPoolExecutor
    jobs = [(e, i) for e in experts for i in range(3)]
    with ThreadPoolExecutor(max_workers=max(1, workers)) as pool:
        mats = list(pool.map(lambda j: expert_matrix(cfg, j[0], j[1]), jobs))
    out = {}
    for (e, i), m in zip(jobs, mats):
        out.setdefault(e, [None, None, None])[i] = m
    return out


_TID_ATTN = 5000  # + {0: queries, 1: keys, 2: per-head direction}


def attention_inputs(cfg: MoEConfig, n_heads: int, n_kv_heads: int, head_dim: int, boost: float = 1.0):
    """Queries [T, n_heads, d] and keys [T, n_kv_heads, d] ~ N(0,1) as bf16 bits, for the
    attention-derived token score.  Every query carries a per-head direction u (|u| = sqrt(d)/2), and
    the keys of the config's heavy-hitter tokens (the same seeded rows `activations` scales) carry
    boost * u of their head as well, so that those tokens receive more attention, as heavy hitters do
    in trained models.  Returns (q bits, k bits, heavy token indices)."""
    T = cfg.T
    rq = _rng(cfg.config_id, _TID_ATTN + 0)
    rk = _rng(cfg.config_id, _TID_ATTN + 1)
    ru = _rng(cfg.config_id, _TID_ATTN + 2)
    q = rq.standard_normal((T, n_heads, head_dim), dtype=np.float32)
    k = rk.standard_normal((T, n_kv_heads, head_dim), dtype=np.float32)
    u = ru.standard_normal((n_kv_heads, head_dim), dtype=np.float32)
    u *= (0.5 * np.sqrt(head_dim)) / np.linalg.norm(u, axis=1, keepdims=True)
    group = n_heads // n_kv_heads
    q += np.repeat(u, group, axis=0)[None, :, :]
    _, heavy = activations(cfg)
    if heavy.size:
        k[heavy] += boost * u[None, :, :]
    return f32_to_bf16_bits(q), f32_to_bf16_bits(k), heavy


_TID_CALIB = 3000


def calibration_inputs(config_id: int, n: int, K: int, rank: int = 4, strength: float = 1.5) -> np.ndarray:
    """Calibration activations [n, K] as bf16 bits for the error-compensated quantizer: unit Gaussians plus
    `rank` shared directions of weight `strength` (trained models' activations are strongly correlated
    across channels, which is what error compensation exploits), and per-channel magnitudes spread
    log-uniformly over a factor 4 (a few loud channels)."""
    rz = _rng(config_id, _TID_CALIB + 0)
    ra = _rng(config_id, _TID_CALIB + 1)
    rb = _rng(config_id, _TID_CALIB + 2)
    rs = _rng(config_id, _TID_CALIB + 3)
    x = rz.standard_normal((n, K), dtype=np.float32)
    if rank > 0:
        x += strength * (ra.standard_normal((n, rank), dtype=np.float32) @ rb.standard_normal((rank, K), dtype=np.float32))
    x *= np.exp2(rs.uniform(-1.0, 1.0, size=(1, K))).astype(np.float32)
    return f32_to_bf16_bits(x)
