"""Pins of the expert-map builder's oracle (Algorithm 1, section 3.1) against things other than
itself: a library norm, closed forms, the paper's own round-robin example, a brute-force greedy
loop, and structural invariants of the emitted table.  No GPU needed."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import table as tab
from paper_2505_06481_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_distance_is_the_library_norm_summed_over_model_pairs(oracle):
    rng = np.random.default_rng(0)
    for V, n in ((2, 1000), (3, 4097), (4, 70000)):
        xs = [rng.standard_normal(n).astype(np.float32) for _ in range(V)]
        ref = sum(np.linalg.norm(xs[i].astype(np.float64) - xs[j].astype(np.float64))
                  for i, j in itertools.combinations(range(V), 2))
        np.testing.assert_allclose(tab.location_distance(xs, "f32"), ref, rtol=1e-13)
    # bf16 storage is widened exactly
    bits = synth.f32_to_bf16_bits(rng.standard_normal((2, 513)).astype(np.float32))
    wide = synth.bf16_bits_to_f32(bits).astype(np.float64)
    np.testing.assert_allclose(tab.location_distance([bits[0], bits[1]], "bf16"), np.linalg.norm(wide[0] - wide[1]),
                               rtol=1e-14)


def test_distance_closed_forms(oracle):
    e = np.eye(3, dtype=np.float32)
    # three unit vectors: every pair is sqrt 2 apart, three combinations
    np.testing.assert_allclose(tab.location_distance([e[0], e[1], e[2]], "f32"), 3 * math.sqrt(2.0), rtol=1e-15)
    # identical experts are at distance 0; a single model has no pair
    assert tab.location_distance([e[0], e[0].copy()], "f32") == 0.0
    assert tab.location_distance([e[0]], "f32") == 0.0
    # a 3-4-5 triangle, and the sum is not the norm of a sum: (0,0), (3,4), (3,0) -> 5 + 3 + 4
    pts = [np.array([0, 0], np.float32), np.array([3, 4], np.float32), np.array([3, 0], np.float32)]
    assert tab.location_distance(pts, "f32") == 12.0
    # scaling both experts scales the distance (catches a missing square root)
    a, b = np.arange(8, dtype=np.float32), np.ones(8, np.float32)
    d1 = tab.location_distance([a, b], "f32")
    np.testing.assert_allclose(tab.location_distance([4 * a, 4 * b], "f32"), 4 * d1, rtol=1e-15)
    # the expert block is the concatenation of its matrices: distances() over two matrices
    v0 = [np.zeros((1, 1, 4), np.float32), np.zeros((1, 1, 2), np.float32)]
    v1 = [np.full((1, 1, 4), 1, np.float32), np.full((1, 1, 2), 2, np.float32)]
    np.testing.assert_allclose(tab.distances([v0, v1], "f32")[0, 0], math.sqrt(4 * 1 + 2 * 4), rtol=1e-15)


def test_round_robin_is_the_papers_example():
    want = {}
    for line in open(os.path.join(GOLDEN, "round_robin_two_models.txt")):
        line = line.split("#")[0].strip()
        if line:
            r, o = line.split("=")
            want[int(r)] = int(o)
    dist = np.array([[0.5, 0.1, 0.3], [0.2, 0.6, 0.4]])       # ranks: (0,1)=1 (1,0)=2 (0,2)=3 (1,2)=4 (0,0)=5 (1,1)=6
    t = tab.build_table(dist, V=2, capacity=6)
    assert t["rank"].tolist() == [[5, 1, 3], [2, 6, 4]]
    for l in range(2):
        for e in range(3):
            assert t["owner"][l, e] == want[int(t["rank"][l, e])]


def brute_table(dist, V, C):
    """The loader's loop written out: repeatedly take the most similar location not yet taken."""
    L, E = dist.shape
    left = {(l, e) for l in range(L) for e in range(E)}
    owner = -np.ones((L, E), int)
    count = 0
    while left and count < C:
        best = min(left, key=lambda le: (dist[le], le))
        left.remove(best)
        count += 1
        owner[best] = (count - 1) % V
    return owner


@pytest.mark.parametrize("V,L,E,C", [(2, 3, 4, 5), (3, 2, 5, 10), (4, 4, 8, 16), (2, 1, 8, 0), (3, 2, 2, 99)])
def test_table_structure_and_bruteforce(V, L, E, C):
    rng = np.random.default_rng(V * 100 + C)
    dist = rng.random((L, E))
    dist[0, 0] = dist[L - 1, E - 1]                           # an exact tie: the lower location ranks first
    t = tab.build_table(dist, V, C)
    assert np.array_equal(t["owner"], brute_table(dist, V, C))
    n_cons = int((t["owner"] >= 0).sum())
    assert n_cons == min(C, L * E)
    # "equally representative": owners differ by at most one location
    per_model = [int((t["owner"] == v).sum()) for v in range(V)]
    assert max(per_model) - min(per_model) <= 1
    # consolidated locations are exactly the n_cons most similar ones
    assert set(np.flatnonzero(t["owner"].reshape(-1) >= 0)) == set(t["order"][:n_cons].tolist())
    assert t["rank"][0, 0] < t["rank"][L - 1, E - 1]
    for l in range(L):
        M, S, src = t["M"][l], int(t["S"][l]), t["slot_src"][l]
        cons = t["owner"][l] >= 0
        assert S == E + (V - 1) * int((~cons).sum()) and src.shape == (S, 2)
        assert M.min() >= 0 and M.max() == S - 1
        for e in range(E):
            if cons[e]:
                assert len(set(M[:, e])) == 1                       # one resident expert, used by every variant
                assert tuple(src[M[0, e]]) == (t["owner"][l, e], e)  # and it is the owner's
            else:
                assert len(set(M[:, e])) == V                       # every variant keeps its own
                for v in range(V):
                    assert tuple(src[M[v, e]]) == (v, e)
        assert len({(v, e) for v in range(V) for e in range(E) if not cons[e]} | {e for e in range(E) if cons[e]}) \
            == len(set(M.reshape(-1)))


def test_generated_variants_rank_distinctly(oracle):
    """The synthetic fine-tuned variants: distances grow with depth (as in the paper's distance map)
    and neighbouring ranks are separated far beyond any summation error."""
    cfg = synth.TableConfig("tiny_table", 3, 4, 4, 64, 96, "swiglu", "bf16", capacity=7, seed=3)
    variants = synth.make_variants(cfg)
    d = tab.distances(variants, cfg.dtype)
    assert d.shape == (4, 4) and (d > 0).all()
    assert d[3].mean() > d[0].mean() * 1.2
    gaps = np.diff(np.sort(d.reshape(-1)))
    print("relative gaps between neighbouring ranks: min %.2e median %.2e" % (gaps.min() / d.mean(),
                                                                              np.median(gaps) / d.mean()))
    assert gaps.min() / d.mean() > 1e-6
