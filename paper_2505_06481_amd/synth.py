"""Seeded synthetic workloads for the multi-model MoE layer.

This module only produces *inputs*: hidden states, variant ids, per-variant
router weights and biases, the consolidation table ``M[v][e]`` and the shared
expert pool.  It contains none of the layer's arithmetic, and is the one piece
of code that both the CPU oracle's tests and the GPU path's tests draw from.

The workloads take the layer shapes of the two model families the paper
evaluates (Mixtral-8x7B: 8 experts per layer, top-2, 176.16 M parameters per
expert, section 3.2; Switch-Base-8: 8 experts per MoE layer, up to four
fine-tuned variants, section 4) and stand in for the trained checkpoints and
text datasets the paper used, which are not available offline.

bf16 tensors are carried as ``uint16`` numpy arrays holding the raw bit pattern.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_GEN_SRC = os.path.join(_HERE, "synth_gen.c")
_GEN_LIB = os.path.join(_HERE, "libmmoe_synth.so")

# stream ids of the counter-based generator
_ST_X, _ST_VID, _ST_WR, _ST_COIN = 1, 2, 3, 4
_ST_W1, _ST_W3, _ST_W2 = 1000, 2000, 3000  # + slot


def build_generator(force: bool = False) -> str:
    """Compile the host generator with gcc (a second or two)."""
    if force or not os.path.exists(_GEN_LIB) or os.path.getmtime(_GEN_LIB) < os.path.getmtime(_GEN_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _GEN_LIB, _GEN_SRC, "-lm"]
        )
    return _GEN_LIB


_lib = None


def _gen():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_generator())
        u64, sz, dbl, vp = ctypes.c_uint64, ctypes.c_size_t, ctypes.c_double, ctypes.c_void_p
        lib.synth_uniform_f64.argtypes = [u64, u64, sz, vp]
        lib.synth_normal_f32.argtypes = [u64, u64, sz, dbl, vp]
        lib.synth_normal_bf16.argtypes = [u64, u64, sz, dbl, vp]
        for f in (lib.synth_uniform_f64, lib.synth_normal_f32, lib.synth_normal_bf16):
            f.restype = None
        _lib = lib
    return _lib


def uniform(seed: int, stream: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.float64)
    _gen().synth_uniform_f64(seed, stream, n, out.ctypes.data)
    return out


def normal(seed: int, stream: int, shape, sigma: float, dtype: str) -> np.ndarray:
    """N(0, sigma^2) samples as fp32, or as bf16 bit patterns (uint16), rounded once (RNE)."""
    n = int(np.prod(shape))
    if dtype == "f32":
        out = np.empty(n, dtype=np.float32)
        _gen().synth_normal_f32(seed, stream, n, sigma, out.ctypes.data)
    elif dtype == "bf16":
        out = np.empty(n, dtype=np.uint16)
        _gen().synth_normal_bf16(seed, stream, n, sigma, out.ctypes.data)
    else:
        raise ValueError(dtype)
    return out.reshape(shape)


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32 (format conversion only)."""
    return (a.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return ((u + (0x7FFF + ((u >> 16) & 1))) >> 16).astype(np.uint16)


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    T: int
    d_model: int
    d_ff: int
    V: int
    E: int
    top_k: int
    dtype: str  # "f32" | "bf16"
    act: str  # "relu" | "swiglu" | "gelu"
    vid_mode: str = "uniform"  # "uniform" | "interleave" | "zipf"
    vid_zipf_s: float = 1.2
    # br[v][e] = -alpha * ln(e + 1); 0 -> no bias tensor.  alpha = 1 is a Zipf(1) prior over the
    # experts; the router's own logits (sigma ~ 1.3 at d = 4096) dilute it, so the skewed
    # workload uses alpha = 2.5 to spread per-slot counts from tens to thousands
    bias_alpha: float = 0.0
    share_prob: float = 0.5
    w_sigma: float = 0.02
    seed: int = 0
    gate: str = "selected"  # "selected": softmax over the picks; "all": probabilities over all experts

    @property
    def P(self) -> int:
        return self.T * self.top_k

    def replace(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


# The five benchmark workloads.  Shapes: Switch-Base-8 (d=768, f=3072, ReLU, top-1)
# and Mixtral-8x7B (d=4096, f=14336, SwiGLU, top-2; 3*4096*14336 = 176.16 M
# parameters per expert, section 3.2).
CONFIGS: Dict[str, Config] = {
    c.name: c
    for c in [
        Config("switch8_fp32_v2_t128", 128, 768, 3072, 2, 8, 1, "f32", "relu"),
        Config("switch8_bf16_v4_t4096", 4096, 768, 3072, 4, 8, 1, "bf16", "relu"),
        Config("mixtral_decode_bf16_v2_t64", 64, 4096, 14336, 2, 8, 2, "bf16", "swiglu"),
        Config("mixtral_prefill_bf16_v2_t8192", 8192, 4096, 14336, 2, 8, 2, "bf16", "swiglu",
               vid_mode="interleave"),
        Config("mixtral_skew_bf16_v4_t16384", 16384, 4096, 14336, 4, 8, 2, "bf16", "swiglu",
               vid_mode="zipf", bias_alpha=2.5),
        # beyond the five: the Switch family's own gate (top-1 probability over all experts, not
        # renormalised) in the three-variant scenario of the paper's scalability experiment (section 4.3)
        Config("switch8_bf16_v3_t4096_gate_all", 4096, 768, 3072, 3, 8, 1, "bf16", "relu", gate="all"),
    ]
}


def make_mapping(cfg: Config) -> np.ndarray:
    """Consolidation table M[V, E] -> pool slot.

    Variant 0 owns slots 0..E-1.  Every expert of a later variant either shares
    variant 0's slot at the same position (probability ``share_prob``: a
    consolidated location, served by one resident copy whoever asks) or gets a
    private slot of its own (a non-consolidated location, served by the
    requesting variant's own expert).
    """
    M = np.empty((cfg.V, cfg.E), dtype=np.int32)
    M[0] = np.arange(cfg.E, dtype=np.int32)
    nxt = cfg.E
    coins = uniform(cfg.seed, _ST_COIN, cfg.V * cfg.E).reshape(cfg.V, cfg.E)
    for v in range(1, cfg.V):
        for e in range(cfg.E):
            if coins[v, e] < cfg.share_prob:
                M[v, e] = e
            else:
                M[v, e] = nxt
                nxt += 1
    return M


def make_vid(cfg: Config) -> np.ndarray:
    if cfg.vid_mode == "interleave":
        return (np.arange(cfg.T) % cfg.V).astype(np.int32)
    u = uniform(cfg.seed, _ST_VID, cfg.T)
    if cfg.vid_mode == "uniform":
        return np.minimum((u * cfg.V).astype(np.int32), cfg.V - 1)
    if cfg.vid_mode == "zipf":
        p = (np.arange(cfg.V) + 1.0) ** (-cfg.vid_zipf_s)
        cdf = np.cumsum(p / p.sum())
        return np.minimum(np.searchsorted(cdf, u, side="right"), cfg.V - 1).astype(np.int32)
    raise ValueError(cfg.vid_mode)


def make_inputs(cfg: Config, weights: bool = True) -> Dict[str, Optional[np.ndarray]]:
    """All buffers of one workload, in the boundary's plain layouts.

    X[T,d], vid[T], Wr[V,E,d], br[V,E] or None, M[V,E], and (if ``weights``) the
    pool W1[S,d,f], W3[S,d,f] (SwiGLU only, else None), W2[S,f,d] -- "in x out".
    """
    dt = cfg.dtype
    M = make_mapping(cfg)
    S = int(M.max()) + 1
    out: Dict[str, Optional[np.ndarray]] = {
        "X": normal(cfg.seed, _ST_X, (cfg.T, cfg.d_model), 1.0, dt),
        "vid": make_vid(cfg),
        "Wr": normal(cfg.seed, _ST_WR, (cfg.V, cfg.E, cfg.d_model), cfg.w_sigma, dt),
        "br": None,
        "M": M,
        "S": S,
    }
    if cfg.bias_alpha != 0.0:
        row = (-cfg.bias_alpha * np.log(np.arange(cfg.E) + 1.0)).astype(np.float32)
        out["br"] = np.tile(row, (cfg.V, 1))
    if weights:
        d, f = cfg.d_model, cfg.d_ff
        np_dt = np.float32 if dt == "f32" else np.uint16
        W1 = np.empty((S, d, f), dtype=np_dt)
        W2 = np.empty((S, f, d), dtype=np_dt)
        W3 = np.empty((S, d, f), dtype=np_dt) if cfg.act == "swiglu" else None
        for s in range(S):
            W1[s] = normal(cfg.seed, _ST_W1 + s, (d, f), cfg.w_sigma, dt)
            W2[s] = normal(cfg.seed, _ST_W2 + s, (f, d), cfg.w_sigma, dt)
            if W3 is not None:
                W3[s] = normal(cfg.seed, _ST_W3 + s, (d, f), cfg.w_sigma, dt)
        out.update(W1=W1, W3=W3, W2=W2)
    return out


def tiny_config(name="tiny", T=13, d_model=32, d_ff=48, V=2, E=4, top_k=2, dtype="f32",
                act="swiglu", **kw) -> Config:
    """A small configuration for brute-force checks."""
    return Config(name, T, d_model, d_ff, V, E, top_k, dtype, act, **kw)


# ---- variants of one model for the expert-map builder (Algorithm 1) ------------------------------
_ST_BASE, _ST_DELTA, _ST_GAIN = 5000, 6000, 7000


@dataclasses.dataclass(frozen=True)
class TableConfig:
    """Shapes of the models handed to the initial expert loader: V variants of one MoE model with
    L layers of E experts; an expert block is `mats` matrices of d_model x d_ff elements."""
    name: str
    V: int
    L: int
    E: int
    d_model: int
    d_ff: int
    act: str            # "relu" | "gelu": 2 matrices; "swiglu": 3
    dtype: str
    capacity: int       # expert locations that are consolidated
    w_sigma: float = 0.02
    ft_sigma: float = 3e-4   # fine-tuning drift per element: distances of a few units at Mixtral size
    seed: int = 0

    @property
    def mats(self) -> int:
        return 3 if self.act == "swiglu" else 2

    @property
    def n_params(self) -> int:
        return self.mats * self.d_model * self.d_ff

    def replace(self, **kw) -> "TableConfig":
        return dataclasses.replace(self, **kw)


TABLE_CONFIGS: Dict[str, TableConfig] = {
    c.name: c
    for c in [
        # the paper's scalability scenario at full size: Switch-Base-8, 12 MoE layers, 4 variants
        TableConfig("switch8_table_v4_l12", 4, 12, 8, 768, 3072, "relu", "bf16", capacity=48),
        # Mixtral-8x7B-shaped experts (176.16 M parameters each), two variants, four layers
        TableConfig("mixtral_table_v2_l4", 2, 4, 8, 4096, 14336, "swiglu", "bf16", capacity=16),
    ]
}


def make_variants(cfg: TableConfig):
    """variants[v][m]: matrix m of model v, shape [L, E, d_model*d_ff] (flattened), storage dtype.

    Stand-in for fine-tuned checkpoints: a base model N(0, w_sigma^2) plus, for every variant, a
    drift N(0, (ft_sigma * gain[l, e])^2) per element.  The gain grows with depth by about a third
    (the paper's distance map shows same-position distances of 3.6 to 4.9, larger in deeper layers)
    with a per-location jitter, so that the locations' distances are distinct at the percent level.
    """
    n = cfg.d_model * cfg.d_ff
    jit = uniform(cfg.seed, _ST_GAIN, cfg.L * cfg.E).reshape(cfg.L, cfg.E)
    depth = np.arange(cfg.L)[:, None] / max(cfg.L - 1, 1)
    gain = 1.0 + 0.36 * depth + 0.1 * jit
    np_dt = np.float32 if cfg.dtype == "f32" else np.uint16
    out = [[np.empty((cfg.L, cfg.E, n), np_dt) for _ in range(cfg.mats)] for _ in range(cfg.V)]
    for l in range(cfg.L):
        for e in range(cfg.E):
            for m in range(cfg.mats):
                loc = (l * cfg.E + e) * cfg.mats + m
                base = normal(cfg.seed, _ST_BASE + loc, (n,), cfg.w_sigma, "f32")
                for v in range(cfg.V):
                    drift = normal(cfg.seed, _ST_DELTA + loc * 64 + v, (n,), cfg.ft_sigma * float(gain[l, e]), "f32")
                    w = base + drift
                    out[v][m][l, e] = w if cfg.dtype == "f32" else f32_to_bf16_bits(w)
    return out
