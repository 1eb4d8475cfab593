"""CPU oracle of the multi-model MoE layer -- TEST INFRASTRUCTURE ONLY.

A thin ctypes wrapper over ``mmoe_oracle.c`` (plain C loops, fp64 sums) plus the
index plumbing needed to run the stages one after another.  Nothing here is
part of the product: only ``tests/``, the smoke check and the benchmark's
reported CPU baseline may import this package, and it imports nothing from the
GPU library.

Stages follow the per-layer body of the paper's Algorithm 2 (gate -> expert-map
lookup -> resident expert -> combination with the gate's coefficients), see the
header of ``mmoe_oracle.c`` for every reading taken where the paper gives no
formula.

Parity pins (tests marked "not gpu"): a second, independent per-token
implementation in exact/fp64 Python arithmetic (``oracle.bruteforce``), a dense
"run every expert and mask" standard MoE layer for the identity table, library
matmul special cases, closed forms of the coefficients, integer invariants of
the grouping, equivariance under token shuffles, tie cases, and the parameter
count the paper prints for a Mixtral expert.  Absolute output values at the
benchmark shapes are not printed anywhere in the paper: for those, parity is
unpinned by the paper and rests on the pins above.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mmoe_oracle.c")
_LIB = os.path.join(_HERE, "libmmoe_oracle.so")

DTYPE = {"f32": 0, "bf16": 1}
ACT = {"relu": 0, "swiglu": 1, "gelu": 2}
GATE = {"selected": 0, "all": 1}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math, no contraction: the code's
    arithmetic is exactly what is written."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ftree-vectorize", "-mavx2", "-mfma", "-ffp-contract=off", "-fno-fast-math",
             "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i, vp = ctypes.c_int, ctypes.c_void_p
        L.mmoe_oracle_threads.restype = ctypes.c_int
        L.mmoe_oracle_route.argtypes = [i, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, vp]
        L.mmoe_oracle_remap_group.argtypes = [i, i, i, i, vp, vp, vp, vp, vp, vp, vp, vp]
        L.mmoe_oracle_gather.argtypes = [i, i, i, i, vp, vp, vp]
        L.mmoe_oracle_ffn_rows.argtypes = [i, vp, vp, i, i, i, i, vp, vp, vp, vp, vp]
        L.mmoe_oracle_combine.argtypes = [i, i, i, vp, vp, vp, vp]
        for fn in (L.mmoe_oracle_route, L.mmoe_oracle_remap_group, L.mmoe_oracle_gather,
                   L.mmoe_oracle_ffn_rows, L.mmoe_oracle_combine):
            fn.restype = None
        _lib = L
    return _lib


def threads() -> int:
    return int(lib().mmoe_oracle_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def _stored(a: np.ndarray, dtype: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    if a.dtype != want:
        raise TypeError(f"expected {want} storage for dtype {dtype}, got {a.dtype}")
    return np.ascontiguousarray(a)


def route(X, vid, Wr, br, top_k: int, dtype: str, gate: str = "selected"):
    """Step R.  Returns (topk_idx [T,k] int32, topk_w [T,k] float64, logits [T,E] float32).
    ``gate``: "selected" = softmax over the k selected logits; "all" = softmax over all E
    logits, the selected experts keeping their probabilities without renormalisation."""
    X, Wr = _stored(X, dtype), _stored(Wr, dtype)
    T, d = X.shape
    V, E, _ = Wr.shape
    vid = _c(vid, np.int32)
    br = None if br is None else _c(br, np.float32)
    idx = np.empty((T, top_k), np.int32)
    w = np.empty((T, top_k), np.float64)
    logits = np.empty((T, E), np.float32)
    lib().mmoe_oracle_route(T, d, V, E, top_k, DTYPE[dtype], GATE[gate], _p(X), _p(vid), _p(Wr), _p(br),
                            _p(idx), _p(w), _p(logits))
    return idx, w, logits


def remap_group(vid, topk_idx, M, S: int):
    """Steps M and G.  Returns slot[P], counts[S], offsets[S+1], perm[P], inv_perm[P]."""
    vid, topk_idx, M = _c(vid, np.int32), _c(topk_idx, np.int32), _c(M, np.int32)
    T, k = topk_idx.shape
    E = M.shape[1]
    P = T * k
    slot = np.empty(P, np.int32)
    counts = np.empty(S, np.int32)
    offsets = np.empty(S + 1, np.int32)
    perm = np.empty(P, np.int32)
    inv = np.empty(P, np.int32)
    lib().mmoe_oracle_remap_group(T, k, E, S, _p(vid), _p(topk_idx), _p(M), _p(slot), _p(counts),
                                  _p(offsets), _p(perm), _p(inv))
    return slot, counts, offsets, perm, inv


def gather(X, perm, top_k: int, dtype: str):
    X = _stored(X, dtype)
    perm = _c(perm, np.int32)
    Xg = np.empty((perm.shape[0], X.shape[1]), X.dtype)
    lib().mmoe_oracle_gather(perm.shape[0], X.shape[1], top_k, DTYPE[dtype], _p(X), _p(perm), _p(Xg))
    return Xg


def ffn_rows(Xsrc, xrow, rslot, W1, W3, W2, dtype: str, act: str):
    """Step F on a list of rows: out[i,:] = expert rslot[i] applied to Xsrc[xrow[i],:] (float64)."""
    Xsrc, W1, W2 = _stored(Xsrc, dtype), _stored(W1, dtype), _stored(W2, dtype)
    W3 = None if W3 is None else _stored(W3, dtype)
    if (act == "swiglu") != (W3 is not None):
        raise ValueError("W3 is given exactly when the expert is gated")
    S, d, f = W1.shape
    assert W2.shape == (S, f, d) and Xsrc.shape[1] == d
    xrow, rslot = _c(xrow, np.int32), _c(rslot, np.int32)
    n = xrow.shape[0]
    assert n == 0 or (0 <= rslot.min() and rslot.max() < S and xrow.max() < Xsrc.shape[0])
    out = np.empty((n, d), np.float64)
    lib().mmoe_oracle_ffn_rows(n, _p(xrow), _p(rslot), d, f, DTYPE[dtype], ACT[act], _p(Xsrc), _p(W1),
                               _p(W3), _p(W2), _p(out))
    return out


def expert_ffn(Xg, offsets, W1, W3, W2, dtype: str, act: str):
    """Step F in its grouped form: rows [offsets[s], offsets[s+1]) go through slot s."""
    P = Xg.shape[0]
    S = len(offsets) - 1
    rslot = np.repeat(np.arange(S, dtype=np.int32), np.diff(offsets))
    assert rslot.shape[0] == P
    return ffn_rows(Xg, np.arange(P, dtype=np.int32), rslot, W1, W3, W2, dtype, act)


def combine(Yg, inv_perm, topk_w):
    """Step C (float64)."""
    Yg = _c(Yg, np.float64)
    topk_w = _c(topk_w, np.float64)
    T, k = topk_w.shape
    inv_perm = _c(inv_perm, np.int32)
    Y = np.empty((T, Yg.shape[1]), np.float64)
    lib().mmoe_oracle_combine(T, Yg.shape[1], k, _p(Yg), _p(inv_perm), _p(topk_w), _p(Y))
    return Y


def layer_forward(inp: Dict, top_k: int, dtype: str, act: str, gate: str = "selected") -> Dict[str, np.ndarray]:
    """The staged layer R -> M -> G -> F -> C over every token; returns all intermediates."""
    S = int(inp["S"])
    idx, w, logits = route(inp["X"], inp["vid"], inp["Wr"], inp["br"], top_k, dtype, gate)
    slot, counts, offsets, perm, inv = remap_group(inp["vid"], idx, inp["M"], S)
    Xg = gather(inp["X"], perm, top_k, dtype)
    Yg = expert_ffn(Xg, offsets, inp["W1"], inp["W3"], inp["W2"], dtype, act)
    Y = combine(Yg, inv, w)
    return dict(topk_idx=idx, topk_w=w, logits=logits, slot=slot, counts=counts, offsets=offsets,
                perm=perm, inv_perm=inv, Xg=Xg, Yg=Yg, Y=Y)


def layer_tokens(inp: Dict, top_k: int, dtype: str, act: str, tokens: Sequence[int],
                 routed=None, gate: str = "selected") -> np.ndarray:
    """Y[t,:] (float64) for the listed tokens only: the same stage functions, with the
    expert stage restricted to the rows those tokens own.  Routing and grouping run on
    every token (they are cheap); ``routed`` may pass their results in."""
    S = int(inp["S"])
    tokens = np.asarray(tokens, dtype=np.int64)
    if routed is None:
        idx, w, _ = route(inp["X"], inp["vid"], inp["Wr"], inp["br"], top_k, dtype, gate)
        slot, *_ = remap_group(inp["vid"], idx, inp["M"], S)
    else:
        idx, w, slot = routed
    pairs = (tokens[:, None] * top_k + np.arange(top_k)[None, :]).reshape(-1)
    Yrows = ffn_rows(inp["X"], (pairs // top_k).astype(np.int32), slot[pairs], inp["W1"], inp["W3"],
                     inp["W2"], dtype, act)
    # rows are already in (token, pick) order: the compact inverse permutation is the identity
    inv = np.arange(pairs.shape[0], dtype=np.int32)
    return combine(Yrows, inv, w[tokens])
