"""CPU oracle of the initial expert loader's table (Algorithm 1) -- TEST INFRASTRUCTURE ONLY.

The steps, in the paper's order (section 3.1): (1) the degree of similarity of every expert
location (layer, expert) is the L2 distance between the flattened experts that the models hold
there, summed over all model-to-model combinations; (2) locations are ranked by it, the lowest
distance first; (3) starting from the highest rank, locations are given to the models in turn
(round robin) until the expert capacity C is used up: the resident expert of such a location is
the owner's, and every model uses it; (4) every other location stays with each model's own expert.

Readings where the paper is loose:
  - pairs: the text says "all model-to-model combinations", the listing iterates over ordered
    pairs; the second is exactly twice the first and ranks identically.  Unordered pairs here.
  - ties in the ranking: lower (layer, expert) index first (a stable sort); the paper is silent.
  - first owner: the text gives, for two models, odd ranks to the first model and even ranks to
    the second; the listing's "count mod |M|" after incrementing count, read with 0-based lists,
    starts with the second.  The text is followed: rank r (1-based) goes to model (r-1) mod V.

The per-layer table of the forward pass follows from the owners: a consolidated location is one
shared slot for every variant, filled with the owner's expert; any other location is one private
slot per variant.  Slot numbers inside a layer: variant 0's locations take slots 0..E-1 (shared
or private alike); the private slots of variants 1.. follow in (variant, expert) order.
"""
from __future__ import annotations

import ctypes
from typing import List, Sequence

import numpy as np

from . import DTYPE, lib


def location_distance(experts: Sequence[np.ndarray], dtype: str) -> float:
    """Degree of similarity of one location: ``experts[v]`` is model v's flattened expert there
    (fp32, or bf16 bit patterns as uint16)."""
    L = lib()
    L.mmoe_oracle_location_distance.restype = ctypes.c_double
    L.mmoe_oracle_location_distance.argtypes = [ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
    arrs = [np.ascontiguousarray(a).reshape(-1) for a in experts]
    n = arrs[0].size
    assert all(a.size == n and a.dtype == arrs[0].dtype for a in arrs)
    ptrs = (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])
    return float(L.mmoe_oracle_location_distance(len(arrs), n, DTYPE[dtype], ptrs))


def distances(variants: Sequence[Sequence[np.ndarray]], dtype: str) -> np.ndarray:
    """``variants[v][m]``: matrix m of every location of model v, shape [L, E, ...].  The expert block
    of a location is the concatenation of its matrices.  Returns float64 [L, E]."""
    L_, E = variants[0][0].shape[:2]
    out = np.empty((L_, E), np.float64)
    for l in range(L_):
        for e in range(E):
            flat = [np.concatenate([np.ascontiguousarray(m[l, e]).reshape(-1) for m in mats]) for mats in variants]
            out[l, e] = location_distance(flat, dtype)
    return out


def build_table(distance: np.ndarray, V: int, capacity: int):
    """Steps (2)-(4).  Returns dict with
         order     [L*E] location ids (l*E + e), most similar first;
         rank      [L, E] 1-based rank of every location;
         owner     [L, E] owning model of a consolidated location, -1 otherwise;
         M         [L, V, E] pool slot, per layer;
         S         [L] slots of each layer's pool;
         slot_src  list per layer of [S_l, 2] (variant, expert) whose weights fill each slot."""
    L_, E = distance.shape
    flat = distance.reshape(-1)
    order = np.argsort(flat, kind="stable")                 # ascending distance, ties to the lower index
    rank = np.empty(L_ * E, np.int32)
    rank[order] = np.arange(1, L_ * E + 1, dtype=np.int32)
    owner = np.full(L_ * E, -1, np.int32)
    count = 0
    for loc in order:                                       # highest rank first, while capacity remains
        if count >= capacity:
            break
        count += 1
        owner[loc] = (count - 1) % V                        # rank 1 -> first model, rank 2 -> second, ...
    owner = owner.reshape(L_, E)
    M = np.empty((L_, V, E), np.int32)
    S = np.empty(L_, np.int32)
    slot_src: List[np.ndarray] = []
    for l in range(L_):
        src = [(int(owner[l, e]) if owner[l, e] >= 0 else 0, e) for e in range(E)]
        M[l, 0] = np.arange(E)
        nxt = E
        for v in range(1, V):
            for e in range(E):
                if owner[l, e] >= 0:
                    M[l, v, e] = e
                else:
                    M[l, v, e] = nxt
                    src.append((v, e))
                    nxt += 1
        S[l] = nxt
        slot_src.append(np.asarray(src, np.int32))
    return dict(order=order.astype(np.int32), rank=rank.reshape(L_, E), owner=owner, M=M, S=S, slot_src=slot_src)
