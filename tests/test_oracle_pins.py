"""Pins of the CPU oracle against things other than itself (no GPU needed).

Every test here is chosen so that a plausible mistake in ``oracle/mmoe_oracle.c``
(dropped term, wrong sign or index, transposed operand, wrong tie rule, wrong
summation order) fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import bruteforce
from paper_2505_06481_amd import synth


def as_f64(a, dtype):
    if a is None:
        return None
    return (synth.bf16_bits_to_f32(a) if dtype == "bf16" else a).astype(np.float64)


def run_brute(inp, cfg, gate="selected"):
    dt = cfg.dtype
    f32 = lambda a: None if a is None else (synth.bf16_bits_to_f32(a) if dt == "bf16" else a)
    return bruteforce.layer(f32(inp["X"]), inp["vid"], f32(inp["Wr"]), inp["br"], inp["M"],
                            as_f64(inp["W1"], dt), as_f64(inp["W3"], dt), as_f64(inp["W2"], dt),
                            cfg.top_k, cfg.act, bf16_h=(dt == "bf16"), gate=gate)


TINY = [
    dict(dtype="f32", act="swiglu", top_k=2, V=2, E=4),
    dict(dtype="f32", act="relu", top_k=1, V=3, E=4),
    dict(dtype="bf16", act="swiglu", top_k=2, V=3, E=4, bias_alpha=0.7),
    dict(dtype="bf16", act="relu", top_k=1, V=2, E=3),
    dict(dtype="f32", act="swiglu", top_k=3, V=2, E=4, d_model=264, d_ff=24, T=5),  # d > 256: lanes wrap
]


@pytest.mark.parametrize("kw", TINY)
def test_staged_oracle_equals_per_token_bruteforce(oracle, kw):
    cfg = synth.tiny_config(seed=3, **kw)
    inp = synth.make_inputs(cfg)
    got = oracle.layer_forward(inp, cfg.top_k, cfg.dtype, cfg.act)
    idx, w, Y = run_brute(inp, cfg)
    assert np.array_equal(got["topk_idx"], idx)
    np.testing.assert_allclose(got["topk_w"], w, rtol=1e-14, atol=0)
    np.testing.assert_allclose(got["Y"], Y, rtol=1e-11, atol=1e-13)
    # the sampled-token entry point is the same computation
    toks = [0, cfg.T - 1, cfg.T // 2]
    Ys = oracle.layer_tokens(inp, cfg.top_k, cfg.dtype, cfg.act, toks)
    np.testing.assert_allclose(Ys, Y[toks], rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("kw", [
    dict(dtype="f32", act="gelu", top_k=1, V=3, E=4),
    dict(dtype="bf16", act="gelu", top_k=2, V=2, E=5, bias_alpha=0.4),
    dict(dtype="f32", act="relu", top_k=4, V=3, E=6),
    dict(dtype="bf16", act="swiglu", top_k=4, V=2, E=4),      # k = E
])
def test_gate_over_all_experts_and_gelu_equal_the_bruteforce(oracle, kw):
    """The Switch-style gate (probability over all experts, not renormalised) and the GELU
    expert against the independent per-token implementation."""
    cfg = synth.tiny_config(seed=5, **kw)
    inp = synth.make_inputs(cfg)
    for gate in ("all", "selected"):
        got = oracle.layer_forward(inp, cfg.top_k, cfg.dtype, cfg.act, gate=gate)
        idx, w, Y = run_brute(inp, cfg, gate)
        assert np.array_equal(got["topk_idx"], idx)
        np.testing.assert_allclose(got["topk_w"], w, rtol=1e-14, atol=0)
        np.testing.assert_allclose(got["Y"], Y, rtol=1e-11, atol=1e-13)


def test_gate_over_all_experts_closed_forms(oracle):
    """Gate mode "all": every selected expert keeps its entry of the softmax over ALL logits.
    Pins: a library softmax; the coefficients do NOT sum to 1 unless every expert is selected;
    renormalising them gives the other gate mode; two experts, top-1: 1 / (1 + e^(l_other - l_top))."""
    cfg = synth.tiny_config(seed=6, T=40, E=6, V=3, top_k=2, d_model=64, bias_alpha=0.3)
    inp = synth.make_inputs(cfg, weights=False)
    idx, w, logits = oracle.route(inp["X"], inp["vid"], inp["Wr"], inp["br"], 2, "f32", gate="all")
    probs = torch.softmax(torch.from_numpy(logits).double(), dim=1).numpy()
    np.testing.assert_allclose(w, np.take_along_axis(probs, idx, 1), rtol=1e-13)
    assert np.all(w.sum(1) < 1.0 - 1e-3)                       # four experts were left out
    idx_s, w_s, _ = oracle.route(inp["X"], inp["vid"], inp["Wr"], inp["br"], 2, "f32", gate="selected")
    assert np.array_equal(idx, idx_s)                          # the mode changes coefficients, never picks
    np.testing.assert_allclose(w / w.sum(1, keepdims=True), w_s, rtol=1e-14)
    # every expert selected: both modes coincide and sum to 1
    _, w_all, _ = oracle.route(inp["X"], inp["vid"], inp["Wr"], inp["br"], 6, "f32", gate="all")
    _, w_sel, _ = oracle.route(inp["X"], inp["vid"], inp["Wr"], inp["br"], 6, "f32", gate="selected")
    np.testing.assert_allclose(w_all, w_sel, rtol=1e-14)
    np.testing.assert_allclose(w_all.sum(1), 1.0, rtol=1e-14)
    # two experts, top-1 (the Switch case): the logistic function of the logit gap
    cfg2 = synth.tiny_config(seed=7, T=30, E=2, V=1, top_k=1, d_model=32)
    inp2 = synth.make_inputs(cfg2, weights=False)
    idx2, w2, lg2 = oracle.route(inp2["X"], inp2["vid"], inp2["Wr"], None, 1, "f32", gate="all")
    top = np.take_along_axis(lg2, idx2, 1)[:, 0].astype(np.float64)
    other = np.take_along_axis(lg2, 1 - idx2, 1)[:, 0].astype(np.float64)
    np.testing.assert_allclose(w2[:, 0], 1.0 / (1.0 + np.exp(other - top)), rtol=1e-14)
    assert np.all(w2 > 0.5) and np.all(w2 < 1.0)               # the top-1 weight is a probability, not 1


def test_switch_style_layer_is_the_dense_definition(oracle):
    """Identity table, one variant, top-1 with the probability as the coefficient and a GELU
    expert: Y[t] = p[t, e*] * gelu(x W1[e*]) W2[e*], written here with library routines."""
    cfg = synth.tiny_config(seed=8, T=12, d_model=16, d_ff=20, V=1, E=4, top_k=1, dtype="f32", act="gelu")
    inp = synth.make_inputs(cfg)
    got = oracle.layer_forward(inp, 1, "f32", "gelu", gate="all")
    X = torch.from_numpy(inp["X"]).double()
    logits = torch.from_numpy(got["logits"]).double()
    p = torch.softmax(logits, 1)
    Y = torch.zeros(cfg.T, cfg.d_model, dtype=torch.float64)
    for e in range(cfg.E):
        W1, W2 = torch.from_numpy(inp["W1"][e]).double(), torch.from_numpy(inp["W2"][e]).double()
        ye = torch.nn.functional.gelu(X @ W1) @ W2              # the library's exact (erf) GELU
        Y += (logits.argmax(1) == e).double()[:, None] * p[:, e:e + 1] * ye
    np.testing.assert_allclose(got["Y"], Y.numpy(), rtol=1e-12, atol=1e-14)
    # special values of the activation through d = f = 1: gelu(0) = 0, gelu(a) -> a, gelu(-a) -> 0,
    # and gelu(a) - gelu(-a) = a exactly in exact arithmetic
    one = np.ones((1, 1, 1), np.float32)
    for a in (0.0, 0.5, 3.0, 12.0):
        xs = np.array([[a], [-a]], np.float32)
        tiny = dict(X=xs, vid=np.zeros(2, np.int32), Wr=one, br=None, M=np.zeros((1, 1), np.int32), S=1,
                    W1=one, W3=None, W2=one)
        y = oracle.layer_forward(tiny, 1, "f32", "gelu")["Y"][:, 0]
        np.testing.assert_allclose(y[0] - y[1], a, rtol=1e-15, atol=1e-300)
        np.testing.assert_allclose(y[0], a * 0.5 * math.erfc(-a / math.sqrt(2.0)), rtol=1e-14)
    assert y[0] == 12.0 and abs(y[1]) < 1e-30


def test_router_logits_bitexact_vs_exact_rational(oracle):
    cfg = synth.tiny_config(seed=11, d_model=520, T=4, E=3, V=2, top_k=1, act="relu", d_ff=8)
    inp = synth.make_inputs(cfg)
    _, _, logits = oracle.route(inp["X"], inp["vid"], inp["Wr"], None, 1, "f32")
    for t in range(cfg.T):
        for e in range(cfg.E):
            ref = bruteforce.router_logit(inp["X"][t], inp["Wr"][inp["vid"][t], e])
            assert np.float32(ref) == logits[t, e]


def test_router_summation_order_hand_example(oracle):
    # d = 8: elements 0..3 belong to lane 0, 4..7 to lane 1.  fp32 absorbs +1 at 2^24.
    big = np.float32(2.0 ** 24)
    w = np.ones((1, 1, 8), np.float32)
    vid = np.zeros(1, np.int32)
    x1 = np.array([[big, 1, 1, 1, -big, 0, 0, 0]], np.float32)   # lane0: 2^24 (ones absorbed); lane1: -2^24
    x2 = np.array([[big, 0, 0, 0, -big, 1, 1, 1]], np.float32)   # lane1: -2^24+3 exactly
    _, _, l1 = oracle.route(x1, vid, w, None, 1, "f32")
    _, _, l2 = oracle.route(x2, vid, w, None, 1, "f32")
    assert l1[0, 0] == 0.0
    assert l2[0, 0] == 3.0
    # bias is added last, in fp32
    _, _, l3 = oracle.route(x2, vid, w, np.array([[0.5]], np.float32), 1, "f32")
    assert l3[0, 0] == 3.5


def test_identity_table_single_variant_is_a_standard_moe_layer(oracle):
    cfg = synth.tiny_config(seed=5, V=1, E=4, top_k=2, T=17, dtype="f32", act="swiglu")
    inp = synth.make_inputs(cfg)
    assert np.array_equal(inp["M"], np.arange(4)[None, :])
    got = oracle.layer_forward(inp, 2, "f32", "swiglu")
    # dense formulation, written separately: run every expert on every token, mask by gate
    X = inp["X"].astype(np.float64)
    logits = X @ inp["Wr"][0].astype(np.float64).T          # [T, E]
    order = np.argsort(-logits, axis=1, kind="stable")[:, :2]
    gate = np.zeros_like(logits)
    for t in range(cfg.T):
        sel = logits[t, order[t]]
        z = np.exp(sel - sel.max())
        gate[t, order[t]] = z / z.sum()
    Y = np.zeros_like(X)
    for e in range(cfg.E):
        g = X @ inp["W1"][e].astype(np.float64)
        u = X @ inp["W3"][e].astype(np.float64)
        h = g / (1.0 + np.exp(-g)) * u
        Y += gate[:, e:e + 1] * (h @ inp["W2"][e].astype(np.float64))
    assert np.array_equal(got["topk_idx"], order)
    np.testing.assert_allclose(got["Y"], Y, rtol=1e-6, atol=1e-8)  # gate from fp32 vs fp64 logits


def test_shared_slot_gives_identical_outputs_for_identical_tokens(oracle):
    # Two variants with the same router and the same table row: a token's output cannot
    # depend on which of the two asks (hit path: the resident expert serves both).
    cfg = synth.tiny_config(seed=9, V=2, E=4, top_k=2, T=8, dtype="bf16", act="swiglu")
    inp = synth.make_inputs(cfg)
    inp["Wr"][1] = inp["Wr"][0]
    inp["M"][1] = inp["M"][0]
    inp["X"][4:] = inp["X"][:4]
    inp["vid"] = np.array([0, 0, 0, 0, 1, 1, 1, 1], np.int32)
    got = oracle.layer_forward(inp, 2, "bf16", "swiglu")
    assert np.array_equal(got["Y"][:4], got["Y"][4:])
    # and with private slots holding different weights the outputs differ (miss path)
    inp["M"][1] = inp["M"][0][::-1].copy()
    got2 = oracle.layer_forward(inp, 2, "bf16", "swiglu")
    assert np.array_equal(got2["Y"][:4], got["Y"][:4])
    assert not np.allclose(got2["Y"][4:], got["Y"][4:])


def test_all_experts_to_one_slot_top1(oracle):
    cfg = synth.tiny_config(seed=2, V=2, E=4, top_k=1, T=6, dtype="f32", act="relu")
    inp = synth.make_inputs(cfg)
    inp["M"][:] = 1
    inp["X"][3:] = inp["X"][:3]
    inp["vid"] = np.array([0, 0, 0, 1, 1, 1], np.int32)
    got = oracle.layer_forward(inp, 1, "f32", "relu")
    assert np.array_equal(got["Y"][:3], got["Y"][3:])          # routers differ, slot does not
    assert got["counts"][1] == 6 and got["counts"].sum() == 6
    X = inp["X"].astype(np.float64)
    ref = np.maximum(X @ inp["W1"][1].astype(np.float64), 0) @ inp["W2"][1].astype(np.float64)
    np.testing.assert_allclose(got["Y"], ref, rtol=1e-12, atol=1e-14)


def test_gate_coefficients_closed_forms(oracle):
    cfg = synth.tiny_config(seed=4, T=64, E=8, V=2, top_k=2, d_model=64)
    inp = synth.make_inputs(cfg, weights=False)
    idx, w, logits = oracle.route(inp["X"], inp["vid"], inp["Wr"], None, 2, "f32")
    assert np.all(np.abs(w.sum(1) - 1.0) <= 2 * np.finfo(np.float64).eps)
    l0 = np.take_along_axis(logits, idx[:, :1], 1)[:, 0].astype(np.float64)
    l1 = np.take_along_axis(logits, idx[:, 1:2], 1)[:, 0].astype(np.float64)
    assert np.all(l0 >= l1)                                     # picks in descending logit
    np.testing.assert_allclose(w[:, 0], 1.0 / (1.0 + np.exp(l1 - l0)), rtol=1e-14)
    # every unselected logit is <= the last selected one
    for t in range(cfg.T):
        rest = np.delete(logits[t], idx[t])
        assert rest.max() <= logits[t, idx[t, 1]]
    idx1, w1, _ = oracle.route(inp["X"], inp["vid"], inp["Wr"], None, 1, "f32")
    assert np.all(w1 == 1.0)
    assert np.array_equal(idx1[:, 0], idx[:, 0])
    # logits agree with a plain fp64 dot product to fp32 accumulation accuracy
    ref = np.einsum("td,ted->te", inp["X"].astype(np.float64), inp["Wr"][inp["vid"]].astype(np.float64))
    np.testing.assert_allclose(logits, ref, rtol=0, atol=1e-5)


def test_grouping_invariants(oracle):
    rng = np.random.default_rng(0)
    T, k, V, E, S = 257, 2, 3, 5, 9
    vid = rng.integers(0, V, T).astype(np.int32)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    M = rng.integers(0, S, (V, E)).astype(np.int32)             # non-injective rows on purpose
    M[M == 4] = 3                                               # slot 4 stays empty
    slot, counts, offsets, perm, inv = oracle.remap_group(vid, idx, M, S)
    P = T * k
    assert np.array_equal(slot, M[np.repeat(vid, k), idx.reshape(-1)])
    assert np.array_equal(counts, np.bincount(slot, minlength=S))
    assert counts[4] == 0
    assert offsets[0] == 0 and offsets[S] == P and np.array_equal(np.diff(offsets), counts)
    assert np.array_equal(np.sort(perm), np.arange(P))
    assert np.array_equal(inv[perm], np.arange(P))
    assert np.all(np.diff(slot[perm]) >= 0)
    for s in range(S):
        seg = perm[offsets[s]:offsets[s + 1]]
        assert np.all(np.diff(seg) > 0)
    assert np.array_equal(perm, np.argsort(slot, kind="stable"))  # library stable sort
    X = rng.standard_normal((T, 8)).astype(np.float32)
    assert np.array_equal(oracle.gather(X, perm, k, "f32"), X[perm // k])


def test_two_picks_of_one_token_into_the_same_slot_are_both_summed(oracle):
    cfg = synth.tiny_config(seed=6, V=1, E=3, top_k=2, T=4, dtype="f32", act="relu")
    inp = synth.make_inputs(cfg)
    inp["M"][:] = 0
    got = oracle.layer_forward(inp, 2, "f32", "relu")
    assert got["counts"][0] == 8
    X = inp["X"].astype(np.float64)
    ref = np.maximum(X @ inp["W1"][0].astype(np.float64), 0) @ inp["W2"][0].astype(np.float64)
    np.testing.assert_allclose(got["Y"], ref, rtol=1e-12, atol=1e-14)   # w0 + w1 = 1


def test_textbook_special_cases(oracle):
    rng = np.random.default_rng(1)
    T, d, f = 9, 16, 24
    X = rng.standard_normal((T, d)).astype(np.float32)
    vid = np.zeros(T, np.int32)
    Wr = rng.standard_normal((1, 1, d)).astype(np.float32)
    W1 = rng.standard_normal((1, d, f)).astype(np.float32)
    W2 = rng.standard_normal((1, f, d)).astype(np.float32)
    inp = dict(X=X, vid=vid, Wr=Wr, br=None, M=np.zeros((1, 1), np.int32), S=1, W1=W1, W3=None, W2=W2)
    # S = V = E = k = 1: a plain two-matmul FFN, against a library matmul
    got = oracle.layer_forward(inp, 1, "f32", "relu")
    tX, tW1, tW2 = (torch.from_numpy(a).double() for a in (X, W1[0], W2[0]))
    ref = (torch.relu(tX @ tW1) @ tW2).numpy()
    np.testing.assert_allclose(got["Y"], ref, rtol=1e-12, atol=1e-13)
    # gated expert, against the library's silu
    W3 = rng.standard_normal((1, d, f)).astype(np.float32)
    got = oracle.layer_forward(dict(inp, W3=W3), 1, "f32", "swiglu")
    ref = ((torch.nn.functional.silu(tX @ tW1) * (tX @ torch.from_numpy(W3[0]).double())) @ tW2).numpy()
    np.testing.assert_allclose(got["Y"], ref, rtol=1e-12, atol=1e-13)
    # identity weights: Y = relu(X)
    eye = np.eye(d, dtype=np.float32)[None]
    got = oracle.layer_forward(dict(inp, W1=eye, W2=eye), 1, "f32", "relu")
    assert np.array_equal(got["Y"], np.maximum(X, 0).astype(np.float64))
    # zero output projection: Y = 0
    got = oracle.layer_forward(dict(inp, W2=np.zeros_like(W2)), 1, "f32", "relu")
    assert np.all(got["Y"] == 0)
    # a non-square, non-symmetric case catches a transposed operand: W1 = [I | 0] picks the
    # first columns, W2 sends hidden unit n to output column n+1
    W1p = np.zeros((1, d, f), np.float32); W1p[0, :, :d] = np.eye(d)
    W2p = np.zeros((1, f, d), np.float32)
    for n in range(d - 1):
        W2p[0, n, n + 1] = 1.0
    got = oracle.layer_forward(dict(inp, W1=W1p, W2=W2p), 1, "f32", "relu")
    ref = np.zeros((T, d)); ref[:, 1:] = np.maximum(X, 0)[:, :-1]
    assert np.array_equal(got["Y"], ref)


def test_one_hot_rows_read_the_router_column(oracle):
    d, E, V = 12, 5, 2
    rng = np.random.default_rng(2)
    Wr = rng.standard_normal((V, E, d)).astype(np.float32)
    X = np.eye(d, dtype=np.float32)
    vid = (np.arange(d) % V).astype(np.int32)
    idx, w, logits = oracle.route(X, vid, Wr, None, 2, "f32")
    for t in range(d):
        assert np.array_equal(logits[t], Wr[vid[t], :, t])
        assert np.array_equal(idx[t], np.argsort(-Wr[vid[t], :, t], kind="stable")[:2])


def test_bf16_hidden_rounding_point(oracle):
    # d = f = 1, relu: y = bf16(x*w1) * w2.  x*w1 = 1 + 2^-8 is a bf16 tie -> rounds to even (1.0);
    # 1 + 3*2^-8 is a tie that rounds up to 1 + 2^-6... check both, and that f32 does not round.
    bf = lambda v: synth.f32_to_bf16_bits(np.array(v, np.float32))
    def run(x, w1, w2, dtype):
        conv = (lambda v: bf(v)) if dtype == "bf16" else (lambda v: np.array(v, np.float32))
        inp = dict(X=conv([[x]]), vid=np.zeros(1, np.int32), Wr=conv([[[1.0]]]), br=None,
                   M=np.zeros((1, 1), np.int32), S=1, W1=conv([[[w1]]]), W3=None, W2=conv([[[w2]]]))
        return oracle.layer_forward(inp, 1, dtype, "relu")["Y"][0, 0]
    a = 1.0 + 2.0 ** -4          # exactly bf16
    # a*a = 1 + 2^-3 + 2^-8 -> nearest bf16 values 1.125 and 1.1328125: tie -> even mantissa (1.125)
    assert run(a, a, 2.0, "bf16") == 2.0 * 1.125
    assert run(a, a, 2.0, "f32") == 2.0 * (a * a)
    b = 1.0 + 2.0 ** -4 + 2.0 ** -7   # bf16-exact (7 fraction bits)
    prod = b * a                       # 1.1337890625 + ... not a tie
    h = float(synth.bf16_bits_to_f32(bf([prod]))[0])
    assert run(b, a, 1.0, "bf16") == h


def test_token_shuffle_equivariance(oracle):
    cfg = synth.tiny_config(seed=8, T=31, V=3, E=4, top_k=2, dtype="bf16", act="swiglu")
    inp = synth.make_inputs(cfg)
    base = oracle.layer_forward(inp, 2, "bf16", "swiglu")
    sh = np.random.default_rng(3).permutation(cfg.T)
    inp2 = dict(inp, X=inp["X"][sh].copy(), vid=inp["vid"][sh].copy())
    got = oracle.layer_forward(inp2, 2, "bf16", "swiglu")
    assert np.array_equal(got["Y"], base["Y"][sh])
    assert np.array_equal(got["topk_idx"], base["topk_idx"][sh])
    assert np.array_equal(got["counts"], base["counts"])


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_contract_summation_order_selects_what_exact_logits_select(oracle, name):
    """The fp32 summation order of the router logit is part of the written contract because it
    decides integer outputs.  Diagnostic for the five benchmark workloads: the experts selected
    from the contract-order fp32 logits are the ones selected from float64 logits (a library
    matrix product of the exactly widened inputs), on every token; the smallest gap at the
    top-k boundary is printed and must dwarf what fp32 summation can move a logit by."""
    cfg = synth.CONFIGS[name]
    inp = synth.make_inputs(cfg, weights=False)
    idx, _, logits = oracle.route(inp["X"], inp["vid"], inp["Wr"], inp["br"], cfg.top_k, cfg.dtype)
    X, Wr = as_f64(inp["X"], cfg.dtype), as_f64(inp["Wr"], cfg.dtype)
    exact = np.empty((cfg.T, cfg.E))
    for v in range(cfg.V):
        rows = np.nonzero(inp["vid"] == v)[0]
        exact[rows] = X[rows] @ Wr[v].T
        if inp["br"] is not None:
            exact[rows] += inp["br"][v].astype(np.float64)
    order = np.argsort(-exact, axis=1, kind="stable")          # descending logit, ties to the lower index
    assert np.array_equal(order[:, :cfg.top_k], idx), "contract-order picks differ from exact-logit picks"
    srt = np.take_along_axis(exact, order, axis=1)
    margin = (srt[:, cfg.top_k - 1] - srt[:, cfg.top_k]).min() if cfg.E > cfg.top_k else np.inf
    within = np.abs(np.diff(srt[:, :cfg.top_k], axis=1)).min() if cfg.top_k > 1 else np.inf
    noise = np.abs(logits.astype(np.float64) - exact).max()
    print(f"{name}: min top-k boundary margin {margin:.3e}, min gap between picks {within:.3e}, "
          f"max |fp32 contract logit - exact| {noise:.3e}")
    assert min(margin, within) > 4 * noise


def test_ties_go_to_the_lower_expert_index(oracle):
    d, E = 16, 6
    rng = np.random.default_rng(4)
    Wr = rng.standard_normal((1, E, d)).astype(np.float32)
    Wr[0, 4] = Wr[0, 1]                      # exact duplicate rows -> exact ties
    Wr[0, 5] = Wr[0, 2]
    X = rng.standard_normal((50, d)).astype(np.float32)
    X[7] = 0.0                               # all logits equal (+0)
    X[8] = -0.0
    vid = np.zeros(50, np.int32)
    idx, w, logits = oracle.route(X, vid, Wr, None, 3, "f32")
    assert np.array_equal(idx[7], [0, 1, 2]) and np.array_equal(idx[8], [0, 1, 2])
    np.testing.assert_allclose(w[7], 1 / 3, rtol=1e-15)
    for t in range(50):
        assert np.array_equal(idx[t], np.argsort(-logits[t].astype(np.float64), kind="stable")[:3])
        pos = {int(e): j for j, e in enumerate(idx[t])}
        if 4 in pos:
            assert 1 in pos and pos[1] < pos[4]
        if 5 in pos:
            assert 2 in pos and pos[2] < pos[5]
    # -0.0 and +0.0 compare equal
    Wz = np.zeros((1, 2, d), np.float32); Wz[0, 0, 0] = -1.0
    Xz = np.zeros((1, d), np.float32)        # logit0 = -0.0 * ... = fma(0,-1,+0) = +0 ; both zero
    idx, _, lg = oracle.route(Xz, np.zeros(1, np.int32), Wz, None, 1, "f32")
    assert idx[0, 0] == 0


def test_parameter_count_matches_the_paper():
    vals = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_shapes.txt")
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    c = synth.CONFIGS["mixtral_prefill_bf16_v2_t8192"]
    per_expert = 3 * c.d_model * c.d_ff
    assert per_expert == 176_160_768
    assert round(per_expert / 1e6, 2) == vals["mixtral_expert_params_million"]
    assert c.E == vals["mixtral_experts_per_layer"] and c.top_k == vals["mixtral_top_k"]
    # 2 bytes per parameter and 27.8 ms per expert copy give a plausible PCIe Gen4 rate
    gbps = per_expert * vals["bytes_per_param"] / (vals["pcie_ms_per_expert"] * 1e-3) / 1e9
    assert 10 < gbps < 32
    sw = synth.CONFIGS["switch8_bf16_v4_t4096"]
    assert sw.E == vals["switch_experts_per_layer"] and sw.V <= vals["switch_variants_max"]


def test_generator_is_deterministic_and_shaped_like_the_recipe():
    cfg = synth.CONFIGS["switch8_fp32_v2_t128"]
    a = synth.make_inputs(cfg, weights=False)
    b = synth.make_inputs(cfg, weights=False)
    assert all(np.array_equal(a[k], b[k]) for k in ("X", "vid", "Wr", "M"))
    assert np.array_equal(a["M"][0], np.arange(8)) and a["S"] == a["M"].max() + 1
    shared = a["M"][1] < 8
    assert np.array_equal(a["M"][1][shared], np.arange(8)[shared])
    assert np.array_equal(np.sort(a["M"][1][~shared]), np.arange(8, a["S"]))
    x = synth.normal(1, 77, (200000,), 1.0, "f32")
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1) < 0.01
    w = synth.bf16_bits_to_f32(synth.normal(1, 78, (200000,), 0.02, "bf16"))
    assert abs(w.std() - 0.02) < 3e-4
    sk = synth.CONFIGS["mixtral_skew_bf16_v4_t16384"]
    vid = synth.make_vid(sk)
    frac = np.bincount(vid, minlength=4) / sk.T
    p = (np.arange(4) + 1.0) ** -1.2; p /= p.sum()
    assert np.all(np.abs(frac - p) < 0.02)
