"""Seeded synthetic workloads for the Virtual-Expert MoE layer.

This module only draws random tensors and formats them (fp32 or bf16 bit
patterns).  It contains none of the layer's arithmetic: no router product, no
softmax, no sorting, no FFN.  The CPU oracle's tests and the HIP path's tests
and benchmark both take their inputs from here, which is the only thing the
two sides have in common.

The paper evaluates on pretrained Switch Transformer / GPTSAN checkpoints with
the samsum and Wikipedia-japanese datasets (Evaluation, "Tasks, datasets and
models"); none of those exist here, so hidden states are drawn from Gaussian
clusters with Zipf-distributed cluster frequencies, which reproduces the
skewed, locally stable expert popularity that the paper's "activation
locality" discussion (Background, "Activation Locality in MoE Models")
describes.  Shapes are the Switch-base / Switch-large MoE layer shapes.

Every tensor has its own child stream of one `numpy.random.SeedSequence`, keyed
by (config seed, layer, tensor kind, expert), so any subset of a bank can be
produced without generating the rest and the values never depend on the order
of the calls.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

F32 = 0
BF16 = 1

# tensor kinds, used as SeedSequence spawn keys
_ROUTER, _W1, _W2, _CENTRES, _ASSIGN, _NOISE, _STREAM = range(7)


@dataclass(frozen=True)
class MoEConfig:
    """One workload: layer shape, resident-set size and hidden-state recipe."""
    name: str
    E: int                 # experts in the full bank
    K: int                 # resident slots (Virtual Experts)
    d_model: int
    d_ff: int
    T: int                 # tokens per layer forward
    layers: int = 1
    dtype: int = BF16      # activations and expert weights; router is always fp32
    clusters: int = 0      # 0 = plain N(0,1) hidden states
    zipf: float = 0.0      # 0 = uniform cluster frequencies
    sigma: float = 0.5     # within-cluster standard deviation
    seed: int = 0
    steps: int = 1         # decode steps (one forward of T tokens per step)
    period: int = 0        # resident-set update period in steps; 0 = never

    def scaled(self, **kw) -> "MoEConfig":
        return replace(self, **kw)


CONFIGS = {
    "c1": MoEConfig("c1-tiny-fp32", E=8, K=2, d_model=64, d_ff=256, T=256,
                    dtype=F32, seed=0),
    "c2": MoEConfig("c2-switch-base-8", E=8, K=4, d_model=768, d_ff=3072,
                    T=4096, clusters=16, seed=1),
    "c3": MoEConfig("c3-switch-base-64-prefill", E=64, K=16, d_model=768,
                    d_ff=3072, T=4096, layers=6, clusters=32, zipf=1.1, seed=2),
    "c4": MoEConfig("c4-switch-base-64-decode", E=64, K=16, d_model=768,
                    d_ff=3072, T=32, clusters=32, zipf=1.1, seed=3, steps=256,
                    period=16),
    "c5": MoEConfig("c5-switch-large-128", E=128, K=32, d_model=1024,
                    d_ff=4096, T=16384, layers=12, clusters=64, zipf=1.1,
                    seed=4),
}


# --------------------------------------------------------------------------
# bf16 formatting (storage format only: 1 sign, 8 exponent, 7 mantissa bits)
# --------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 with round-to-nearest-even; returns uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def format_tensor(a: np.ndarray, dtype: int) -> np.ndarray:
    """fp32 array for F32, uint16 bit patterns for BF16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a if dtype == F32 else f32_to_bf16_bits(a)


def as_f32(a: np.ndarray, dtype: int) -> np.ndarray:
    return np.ascontiguousarray(a, np.float32) if dtype == F32 else bf16_bits_to_f32(a)


# --------------------------------------------------------------------------
# random streams
# --------------------------------------------------------------------------

def _rng(cfg: MoEConfig, layer: int, kind: int, index: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence(entropy=cfg.seed, spawn_key=(layer, kind, index))
    return np.random.default_rng(ss)


def router_weights(cfg: MoEConfig, layer: int = 0) -> np.ndarray:
    """W_r [E, d_model] fp32 ~ N(0, 0.02^2)."""
    g = _rng(cfg, layer, _ROUTER)
    return (0.02 * g.standard_normal((cfg.E, cfg.d_model), dtype=np.float32)).astype(np.float32)


def expert_weights(cfg: MoEConfig, expert: int, layer: int = 0):
    """(W1_e [d_model, d_ff], W2_e [d_ff, d_model]) of one expert of the bank,
    ~ N(0, 0.02^2), in the config's storage dtype."""
    g1 = _rng(cfg, layer, _W1, expert)
    g2 = _rng(cfg, layer, _W2, expert)
    w1 = 0.02 * g1.standard_normal((cfg.d_model, cfg.d_ff), dtype=np.float32)
    w2 = 0.02 * g2.standard_normal((cfg.d_ff, cfg.d_model), dtype=np.float32)
    return format_tensor(w1, cfg.dtype), format_tensor(w2, cfg.dtype)


def expert_bank(cfg: MoEConfig, layer: int = 0, experts=None):
    """Stacked (W1 [n, d, f], W2 [n, f, d]) for `experts` (default: all E)."""
    experts = range(cfg.E) if experts is None else experts
    pairs = [expert_weights(cfg, e, layer) for e in experts]
    return np.stack([p[0] for p in pairs]), np.stack([p[1] for p in pairs])


def cluster_probs(cfg: MoEConfig) -> np.ndarray:
    c = np.arange(cfg.clusters, dtype=np.float64)
    p = (c + 1.0) ** (-cfg.zipf) if cfg.zipf > 0 else np.ones_like(c)
    return p / p.sum()


def cluster_centres(cfg: MoEConfig) -> np.ndarray:
    g = _rng(cfg, 0, _CENTRES)
    return g.standard_normal((cfg.clusters, cfg.d_model), dtype=np.float32)


def hidden_states(cfg: MoEConfig, layer: int = 0, T: int | None = None) -> np.ndarray:
    """x [T, d_model] in the config's storage dtype.

    Layers of a stacked config get independent draws from the same mixture
    (same centres, fresh assignments and noise), so each layer of a parity test
    can be checked on its own."""
    T = cfg.T if T is None else T
    gn = _rng(cfg, layer, _NOISE)
    if cfg.clusters == 0:
        x = gn.standard_normal((T, cfg.d_model), dtype=np.float32)
    else:
        ga = _rng(cfg, layer, _ASSIGN)
        assign = ga.choice(cfg.clusters, size=T, p=cluster_probs(cfg))
        mu = cluster_centres(cfg)
        x = mu[assign] + np.float32(cfg.sigma) * gn.standard_normal((T, cfg.d_model), dtype=np.float32)
    return format_tensor(x, cfg.dtype)


def decode_stream(cfg: MoEConfig, steps: int | None = None) -> np.ndarray:
    """x [steps, T, d_model]: T concurrent streams, one token per stream per step.

    Each stream holds a current cluster drawn from the Zipf mixture and
    re-draws it with probability 1/32 per step, which gives the step-to-step
    activation locality the resident-set update relies on."""
    steps = cfg.steps if steps is None else steps
    g = _rng(cfg, 0, _STREAM)
    p = cluster_probs(cfg)
    mu = cluster_centres(cfg)
    cur = g.choice(cfg.clusters, size=cfg.T, p=p)
    out = np.empty((steps, cfg.T, cfg.d_model), dtype=np.float32)
    for s in range(steps):
        redraw = g.random(cfg.T) < (1.0 / 32.0)
        fresh = g.choice(cfg.clusters, size=cfg.T, p=p)
        cur = np.where(redraw, fresh, cur)
        out[s] = mu[cur] + np.float32(cfg.sigma) * g.standard_normal((cfg.T, cfg.d_model), dtype=np.float32)
    return format_tensor(out, cfg.dtype)


def initial_resident(cfg: MoEConfig):
    """Slots 0..K-1 hold experts 0..K-1.  Returns (slot_to_expert, expert_to_slot)."""
    s2e = np.arange(cfg.K, dtype=np.int32)
    e2s = np.full(cfg.E, -1, dtype=np.int32)
    e2s[:cfg.K] = s2e
    return s2e, e2s
