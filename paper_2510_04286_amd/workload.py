"""Seeded synthetic inputs for the SliceMoE layer forward pass.

This module only *draws inputs* (hidden states, router and expert weights, random
top-k index tables, and the random draws a training-time router consumes).  It contains none of the layer's arithmetic (no router, no
softmax, no expert FFN, no dispatch), so the CPU oracle and the HIP path can both be
fed from it without sharing any code of the method.

Shapes follow the paper's layer (Section 3, Section 3.1, Appendix A): a token vector of
width ``d`` split into ``S`` contiguous slices of width ``d_s = d / S``, one shared router
``Linear(d_s -> H_r = 256) -> ReLU -> Linear(256 -> E)``, ``E`` experts that are
two-layer MLPs ``d_s -> H_e -> d_s``, top-``k`` routing per slice.

Generator: a counter-based PRNG.  Element ``i`` of tensor ``tid`` under ``seed`` is
``splitmix64(key(seed, tid) + (i + 1) * GOLDEN)`` mapped to a 53-bit uniform; normals
come from Box-Muller on two independent streams.  The value of an element depends
only on ``(seed, tid, i)``: it is independent of generation order, chunking and library
versions.  Storage rounding to bf16 is round-to-nearest-even, done once here, so every
consumer sees identical values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

H_R = 256  # router hidden width (Section 3.1, Appendix A)

# tensor ids (streams) of the generator
TID_H, TID_WR1, TID_BR1, TID_WR2, TID_BR2, TID_W1, TID_B1, TID_W2, TID_B2, TID_IDX, TID_NOISE, TID_DROP, TID_DOUT = range(13)


@dataclass(frozen=True)
class SliceMoEShape:
    """One workload: sizes, storage dtype and capacity factor (<= 0 means dropless)."""

    name: str
    T: int
    d: int
    S: int
    E: int
    k: int
    He: int
    dtype: str = "bf16"  # "f32" | "bf16": storage type of h, h' and all weights
    capacity_factor: float = 0.0
    Hr: int = H_R
    layernorm: bool = False  # per-token (x - mean) / sqrt(var + 1e-5) before rounding
    zipf_s: float = 0.0  # > 0: second router bias calibrated to Zipf(s) popularity

    @property
    def ds(self) -> int:
        return self.d // self.S

    @property
    def Ns(self) -> int:
        return self.T * self.S

    @property
    def Na(self) -> int:
        return self.T * self.S * self.k

    def capacity(self) -> int:
        """Per-expert row capacity C = ceil(float32(capacity_factor) * Na / E); -1 when dropless."""
        if self.capacity_factor <= 0:
            return -1
        return int(math.ceil(float(np.float32(self.capacity_factor)) * self.Na / self.E))

    def scaled(self, T: int, name: str | None = None) -> "SliceMoEShape":
        """Same layer, fewer (or more) tokens."""
        return replace(self, T=T, name=name or f"{self.name}@T{T}")


def paper_shape(S: int = 8, k: int = 2, T: int = 16384) -> SliceMoEShape:
    """The paper's own layer (Appendix A): d = 768, 16 experts, expert hidden width 4 * d/S; S = 8 and k = 2 are its
    defaults, S in {2, 4, 8, 16, 32} its slice-count ablation (Table 2), k in {1, 2, 3} its top-k ablation
    (Table 4).  Not one of the five benchmark workloads."""
    name = "paper" if (S, k) == (8, 2) else f"paper_S{S}_k{k}"
    return SliceMoEShape(name, T=T, d=768, S=S, E=16, k=k, He=4 * (768 // S))


CONFIGS = {
    "tiny": SliceMoEShape("tiny", T=512, d=256, S=4, E=8, k=2, He=256, dtype="f32"),
    "lm": SliceMoEShape("lm", T=4096, d=512, S=8, E=16, k=2, He=256, layernorm=True),
    "headline": SliceMoEShape("headline", T=16384, d=1024, S=16, E=32, k=2, He=256),
    "skewed": SliceMoEShape("skewed", T=16384, d=1024, S=16, E=32, k=2, He=256,
                            capacity_factor=1.25, zipf_s=1.2),
    "large": SliceMoEShape("large", T=65536, d=4096, S=32, E=64, k=2, He=512),
    "paper": paper_shape(),
    "paper_S2_k2": paper_shape(S=2),
    "paper_S4_k2": paper_shape(S=4),
    "paper_S16_k2": paper_shape(S=16),
    "paper_S32_k2": paper_shape(S=32),
}
CONFIG_ORDER = ["tiny", "lm", "headline", "skewed", "large"]


# --------------------------------------------------------------------------- PRNG
def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(seed: int, tid: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        z = np.array([(seed * 0x1000003 + tid * 0x10001 + stream * 0x101 + 0x5EED) & 0xFFFFFFFFFFFFFFFF],
                     dtype=np.uint64)
        return _mix(_mix(z) + _GOLDEN)[0]


def random_u64(seed: int, tid: int, start: int, count: int, stream: int = 0) -> np.ndarray:
    """64 random bits for elements ``start .. start+count-1`` of a tensor."""
    with np.errstate(over="ignore"):
        i = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        return _mix(_key(seed, tid, stream) + i * _GOLDEN)


def uniform01(seed: int, tid: int, start: int, count: int, stream: int = 0) -> np.ndarray:
    """fp64 uniforms in [0, 1) with 53 random bits."""
    return (random_u64(seed, tid, start, count, stream) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def normal(seed: int, tid: int, start: int, count: int) -> np.ndarray:
    """fp64 standard normals (Box-Muller, one normal per element from two uniform streams)."""
    u1 = 1.0 - uniform01(seed, tid, start, count, 0)  # (0, 1]
    u2 = uniform01(seed, tid, start, count, 1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


# --------------------------------------------------------------------------- bf16 storage
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    b = x.view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((b + r) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return out.view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of fp32 values that are already bf16-representable."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(b & np.uint32(0xFFFF)), "value is not bf16-representable"
    return (b >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 array holding values representable in the storage dtype."""
    x = np.asarray(x, dtype=np.float64).astype(np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


# --------------------------------------------------------------------------- tensors
def _kaiming_uniform(seed: int, tid: int, shape: tuple, fan_in: int, dtype: str) -> np.ndarray:
    """U(-1/sqrt(fan_in), +1/sqrt(fan_in)): the usual Linear-layer default for weight and bias."""
    n = int(np.prod(shape))
    bound = 1.0 / math.sqrt(fan_in)
    u = uniform01(seed, tid, 0, n)
    return to_storage(((2.0 * u - 1.0) * bound).reshape(shape), dtype)


def make_weights(cfg: SliceMoEShape, seed: int = 0) -> dict:
    """Router and expert parameters in the logical layout ``y = x @ W + b``.

    Wr1 [ds, Hr], br1 [Hr], Wr2 [Hr, E], br2 [E]; W1 [E, ds, He], b1 [E, He],
    W2 [E, He, ds], b2 [E, ds].  All fp32 arrays holding storage-representable values.
    """
    ds, Hr, E, He, dt = cfg.ds, cfg.Hr, cfg.E, cfg.He, cfg.dtype
    return {
        "Wr1": _kaiming_uniform(seed, TID_WR1, (ds, Hr), ds, dt),
        "br1": _kaiming_uniform(seed, TID_BR1, (Hr,), ds, dt),
        "Wr2": _kaiming_uniform(seed, TID_WR2, (Hr, E), Hr, dt),
        "br2": _kaiming_uniform(seed, TID_BR2, (E,), Hr, dt),
        "W1": _kaiming_uniform(seed, TID_W1, (E, ds, He), ds, dt),
        "b1": _kaiming_uniform(seed, TID_B1, (E, He), ds, dt),
        "W2": _kaiming_uniform(seed, TID_W2, (E, He, ds), He, dt),
        "b2": _kaiming_uniform(seed, TID_B2, (E, ds), He, dt),
    }


def make_h(cfg: SliceMoEShape, seed: int = 1, t0: int = 0, t1: int | None = None) -> np.ndarray:
    """Hidden states h[t0:t1, d] ~ N(0,1) (optionally LayerNorm-scaled), storage-rounded."""
    t1 = cfg.T if t1 is None else t1
    d = cfg.d
    out = np.empty((t1 - t0, d), dtype=np.float32)
    step = max(1, (1 << 22) // d)  # ~4M elements per chunk keeps temporaries small
    for a in range(t0, t1, step):
        b = min(t1, a + step)
        x = normal(seed, TID_H, a * d, (b - a) * d).reshape(b - a, d)
        if cfg.layernorm:
            mu = x.mean(axis=1, keepdims=True)
            var = x.var(axis=1, keepdims=True)
            x = (x - mu) / np.sqrt(var + 1e-5)
        out[a - t0:b - t0] = to_storage(x, cfg.dtype)
    return out


def make_topk_idx(Ns: int, k: int, E: int, seed: int = 2, zipf_s: float = 0.0) -> np.ndarray:
    """Random routing table idx[Ns, k] (int32) with k distinct experts per slice.

    Used to exercise the dispatch stage on its own at sizes where running a router on
    the host would be slow.  ``zipf_s > 0`` skews expert popularity ~ rank^-s.
    """
    w = np.arange(1, E + 1, dtype=np.float64) ** (-zipf_s) if zipf_s > 0 else np.ones(E)
    # Gumbel-style keys: the k largest of log(w) - log(-log(u)) are k distinct experts
    out = np.empty((Ns, k), dtype=np.int32)
    step = max(1, (1 << 22) // E)
    for a in range(0, Ns, step):
        b = min(Ns, a + step)
        u = uniform01(seed, TID_IDX, a * E, (b - a) * E).reshape(b - a, E)
        key = np.log(w)[None, :] - np.log(-np.log(np.clip(u, 1e-300, 1 - 1e-16)))
        out[a:b] = np.argsort(-key, axis=1, kind="stable")[:, :k].astype(np.int32)
    return out


def make_router_draws(cfg: SliceMoEShape, seed: int = 2) -> tuple:
    """The random numbers a training-time router consumes, as inputs: standard normals noise[Ns, E] for the logit noise
    (Section 5) and uniforms drop_u[Ns, k] in [0, 1) for the cross-slice dropout (Section 3.3), both fp32."""
    noise = normal(seed, TID_NOISE, 0, cfg.Ns * cfg.E).astype(np.float32).reshape(cfg.Ns, cfg.E)
    drop_u = uniform01(seed, TID_DROP, 0, cfg.Na).astype(np.float32).reshape(cfg.Ns, cfg.k)
    drop_u = np.minimum(drop_u, np.float32(1.0 - 2.0 ** -24))   # rounding to fp32 must not reach 1
    return noise, drop_u


def make_dout(cfg: SliceMoEShape, seed: int = 3) -> np.ndarray:
    """Upstream gradient dL/dh'[T, d] ~ N(0,1) for the backward pass, storage-rounded."""
    g = normal(seed, TID_DOUT, 0, cfg.T * cfg.d).reshape(cfg.T, cfg.d)
    return to_storage(g, cfg.dtype)
