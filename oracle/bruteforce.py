"""Per-token brute force of the multi-model MoE layer -- TEST INFRASTRUCTURE ONLY.

A second implementation of the oracle, written token by token with no grouping
stage at all, used on tiny inputs to pin ``mmoe_oracle.c``.  It shares nothing
with the C file: the fp32 fused multiply-adds of the router are reproduced with
exact rational arithmetic and an explicit round-to-nearest-even, the experts
are evaluated with Python/numpy float64 scalars and vectors.

For each token t (per-layer body of the paper's Algorithm 2): v = vid[t]; the
variant's gate scores the E experts; the k best are taken (ties to the lower
index); their coefficients are the softmax over the selected logits (gate
"selected") or their own entries of the softmax over all E logits (gate "all");
each pick e goes through the table to slot M[v][e]; y = sum_j w_j * FFN_slot_j(x_t).
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np


def round_to_f32(fr: Fraction) -> float:
    """Nearest fp32 to an exact rational, ties to even (normal and subnormal range)."""
    if fr == 0:
        return 0.0
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, -126)
    q = Fraction(2) ** (e - 23)
    n = a / q
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    val = fl * q
    out = sign * float(val)  # exact: at most 24 significant bits
    assert abs(out) < 3.5e38
    return out


def fmaf_exact(a: float, b: float, c: float) -> float:
    return round_to_f32(Fraction(a) * Fraction(b) + Fraction(c))


def addf_exact(a: float, b: float) -> float:
    return round_to_f32(Fraction(a) + Fraction(b))


def router_logit(x, w, bias=None) -> float:
    """fp32 dot product in the contract's order: element i -> lane (i//4) % 64, per-lane
    ascending fused multiply-adds from +0, then the xor butterfly 32,16,8,4,2,1."""
    p = [0.0] * 64
    for i in range(len(x)):
        lane = (i // 4) % 64
        p[lane] = fmaf_exact(float(x[i]), float(w[i]), p[lane])
    off = 32
    while off >= 1:
        p = [addf_exact(p[l], p[l ^ off]) for l in range(64)]
        off //= 2
    assert all(v == p[0] for v in p)
    s = p[0]
    if bias is not None:
        s = addf_exact(s, float(bias))
    return s


def _bf16_round(x: float) -> float:
    """float64 -> nearest bf16 value (8 significant bits), ties to even."""
    if x == 0.0:
        return x
    fr = Fraction(x)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    e = max(e, -126)
    q = Fraction(2) ** (e - 7)
    n = a / q
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return sign * float(fl * q)


def expert(x, W1, W3, W2, act: str, bf16_h: bool):
    """One expert on one token, float64.  W1, W3: [d, f]; W2: [f, d] (in x out)."""
    g = x @ W1
    if act == "swiglu":
        u = x @ W3
        h = np.array([gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)])
    elif act == "gelu":
        h = np.array([0.5 * gi * math.erfc(-gi / math.sqrt(2.0)) for gi in g])   # a * Phi(a), Phi by erfc
    else:
        h = np.array([gi if gi > 0.0 else 0.0 for gi in g])
    if bf16_h:
        h = np.array([_bf16_round(float(v)) for v in h])
    return h @ W2


def layer(X, vid, Wr, br, M, W1, W3, W2, top_k: int, act: str, bf16_h: bool, gate: str = "selected"):
    """X [T,d], Wr [V,E,d], W* as float arrays holding the stored values exactly.
    Returns (topk_idx [T,k], topk_w [T,k] float64, Y [T,d] float64)."""
    X = np.asarray(X, dtype=np.float64)
    T, d = X.shape
    E = Wr.shape[1]
    idx = np.zeros((T, top_k), dtype=np.int32)
    wts = np.zeros((T, top_k), dtype=np.float64)
    Y = np.zeros((T, d), dtype=np.float64)
    for t in range(T):
        v = int(vid[t])
        logit = [router_logit(X[t], Wr[v, e], None if br is None else br[v, e]) for e in range(E)]
        order = sorted(range(E), key=lambda e: (-logit[e], e))[:top_k]
        m = logit[order[0]]
        z = [math.exp(logit[e] - m) for e in order]
        tot = sum(z) if gate == "selected" else math.fsum(math.exp(l - m) for l in logit)
        for j, e in enumerate(order):
            idx[t, j] = e
            wts[t, j] = z[j] / tot
            s = int(M[v][e])
            W3s = None if W3 is None else np.asarray(W3[s], dtype=np.float64)
            Y[t] += wts[t, j] * expert(X[t], np.asarray(W1[s], dtype=np.float64), W3s,
                                       np.asarray(W2[s], dtype=np.float64), act, bf16_h)
    return idx, wts, Y
