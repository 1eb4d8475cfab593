"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs.  Integer outputs (selected experts, slots, histogram, offsets,
permutation, gathered rows) must match bit for bit; floating-point outputs within

    bf16 storage:  |got - ref| <= 1e-2 + 2e-2 |ref|
    fp32 storage:  |got - ref| <= 1e-4 |ref| + 1e-4 rms(ref)

Small cases compare every element; the full benchmark shapes compare every integer output,
every row of the smallest and the largest slot, and 512 seeded tokens.
"""
import numpy as np
import pytest
import torch

from paper_2505_06481_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mm():
    from paper_2505_06481_amd import mmoe
    mmoe.lib()
    assert torch.cuda.is_available()
    return mmoe


@pytest.fixture(scope="module")
def gc():
    import gpu_common
    return gpu_common


def staged_vs_oracle(mm, gc, oracle, cfg, inp=None, tile_rows=0):
    """Run the four stages one by one through the C ABI and compare each with the oracle."""
    print(f"case {cfg.name} T={cfg.T} d={cfg.d_model} f={cfg.d_ff} V={cfg.V} E={cfg.E} k={cfg.top_k} "
          f"{cfg.dtype} {cfg.act} seed={cfg.seed}", flush=True)
    case = gc.DeviceCase(cfg, inp, tile_rows=tile_rows)
    inp, sh, dt = case.inp, case.shape, cfg.dtype
    ref = oracle.layer_forward(inp, cfg.top_k, dt, cfg.act, gate=cfg.gate)

    idx, w = mm.route(sh, case.X, case.vid, case.Wr, case.br)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), ref["topk_idx"]), "selected experts differ"
    np.testing.assert_allclose(w.cpu().numpy(), ref["topk_w"], rtol=2e-6, atol=1e-7)

    slot, counts, offsets, perm, inv, Xg = mm.remap_permute(sh, case.X, case.vid, idx, case.M, case.ws)
    torch.cuda.synchronize()
    for name, t in (("slot", slot), ("counts", counts), ("offsets", offsets), ("perm", perm), ("inv_perm", inv)):
        assert np.array_equal(t.cpu().numpy(), ref[name]), name
    assert np.array_equal(gc.bits(Xg), ref["Xg"]), "gathered rows differ"

    Yg = mm.expert_ffn(sh, Xg, offsets, case.W1p, case.W3p, case.W2p, case.ws)
    torch.cuda.synchronize()
    gc.assert_close(gc.to_np64(Yg), ref["Yg"], dt, "Yg")

    Y = mm.combine(sh, Yg, inv, w)
    torch.cuda.synchronize()
    gc.assert_close(gc.to_np64(Y), ref["Y"], dt, "Y (staged)")

    Y2 = case.forward()
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y), "fused entry point differs from the staged path"
    Y3 = case.forward()
    torch.cuda.synchronize()
    assert torch.equal(Y3, Y2), "two runs differ: the path is not deterministic"
    return case, ref


SMALL = [
    # weight-streaming kernels (few rows per slot), ragged row counts, several 16-row blocks
    synth.Config("s_bf16_swiglu", 45, 512, 768, 3, 4, 2, "bf16", "swiglu", seed=1),
    synth.Config("s_bf16_relu", 70, 256, 512, 2, 8, 1, "bf16", "relu", seed=2),
    synth.Config("s_f32_relu", 33, 256, 512, 2, 4, 1, "f32", "relu", seed=3),
    synth.Config("s_f32_swiglu", 50, 512, 256, 2, 4, 2, "f32", "swiglu", seed=4, bias_alpha=0.5),
    synth.Config("s_f32_many_rows", 300, 256, 256, 1, 2, 1, "f32", "relu", seed=5),     # > 32 rows: passes
    # few rows per slot on average, but a biased router fills one slot beyond a 32-row pass
    synth.Config("s_bf16_skewed_passes", 100, 512, 256, 1, 8, 1, "bf16", "swiglu", seed=26, bias_alpha=3.0),
    # matrix-core tiled kernels (many rows per slot), ragged tails, several tiles per slot
    synth.Config("t_bf16_swiglu", 700, 512, 768, 2, 4, 2, "bf16", "swiglu", seed=6),
    synth.Config("t_bf16_relu", 900, 256, 512, 3, 4, 1, "bf16", "relu", seed=7),
    synth.Config("t_bf16_skew", 1500, 256, 256, 4, 8, 2, "bf16", "swiglu", seed=8, vid_mode="zipf",
                 bias_alpha=1.0),
    synth.Config("t_bf16_topk_all", 400, 256, 256, 1, 3, 3, "bf16", "swiglu", seed=9),   # top_k = E
    # batches large enough for the wavefront-per-token router, odd expert counts, fp32 and bf16
    synth.Config("r_f32_odd_e", 2100, 512, 256, 2, 5, 2, "f32", "swiglu", seed=17, bias_alpha=0.7),
    synth.Config("r_bf16_odd_e", 2060, 1536, 256, 3, 7, 2, "bf16", "relu", seed=18, bias_alpha=0.3),
    # one pick per token (the down product writes the layer's output rows itself) where the grouping
    # kernels have run: streaming kernels in fp32 and, with many slots, in bf16; matrix-core kernels at
    # both tile heights are t_bf16_relu
    synth.Config("k1_f32_grouped", 1500, 256, 512, 2, 6, 1, "f32", "gelu", seed=27),
    synth.Config("k1_bf16_grouped_stream", 1300, 512, 256, 8, 16, 1, "bf16", "relu", seed=28, share_prob=0.1),
    synth.Config("k1_bf16_long_k", 1100, 2048, 256, 2, 4, 1, "bf16", "relu", seed=29),     # tall-tile shape rule
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_small_cases_every_stage(mm, gc, oracle, cfg):
    staged_vs_oracle(mm, gc, oracle, cfg)


@pytest.mark.parametrize("rows", [256, 128])
@pytest.mark.parametrize("cfg", [c for c in SMALL if c.name.startswith("t_")], ids=lambda c: c.name)
def test_both_tile_heights(mm, gc, oracle, cfg, rows):
    """The matrix-core kernels at a forced tile height (by shape these small batches would only
    ever get the 128-row tiles): every stage against the oracle, ragged last tiles of 1..8 sub-tiles."""
    staged_vs_oracle(mm, gc, oracle, cfg, tile_rows=rows)


GATES_AND_ACTS = [
    # Switch-style gate (probability over all experts, not renormalised), top-1, ReLU and GELU experts,
    # three variants; streaming kernels and matrix-core kernels, fp32 and bf16
    synth.Config("g_switch_f32_gelu", 60, 256, 512, 3, 8, 1, "f32", "gelu", seed=41, gate="all"),
    synth.Config("g_switch_bf16_relu_tiled", 1200, 256, 512, 3, 8, 1, "bf16", "relu", seed=42, gate="all"),
    synth.Config("g_switch_bf16_gelu_tiled", 1000, 512, 768, 3, 8, 1, "bf16", "gelu", seed=43, gate="all"),
    synth.Config("g_switch_bf16_gelu_stream", 90, 512, 256, 3, 8, 1, "bf16", "gelu", seed=44, gate="all"),
    # k = 2 and 4 with either gate, up to 64 experts per variant, gated and plain experts
    synth.Config("g_all_k2_e64", 500, 256, 256, 2, 64, 2, "bf16", "swiglu", seed=45, gate="all"),
    synth.Config("g_all_k4_e64", 300, 256, 256, 3, 64, 4, "bf16", "gelu", seed=46, gate="all", bias_alpha=0.5),
    synth.Config("g_sel_k4_e16", 2100, 256, 256, 3, 16, 4, "bf16", "gelu", seed=47),
    synth.Config("g_all_k4_f32", 2060, 512, 256, 3, 16, 4, "f32", "swiglu", seed=48, gate="all"),
    synth.Config("g_all_k_equals_e", 70, 256, 256, 2, 4, 4, "f32", "relu", seed=49, gate="all"),   # sums to 1 again
]


@pytest.mark.parametrize("cfg", GATES_AND_ACTS, ids=lambda c: c.name)
def test_gate_modes_and_activations(mm, gc, oracle, cfg):
    """Section 3.2's coefficients "for each expert" read the Switch way (section 4.3's family), and the
    GELU expert: every stage against the oracle, both router kernels, both expert-stage kernels."""
    case, ref = staged_vs_oracle(mm, gc, oracle, cfg)
    if cfg.gate == "all" and cfg.top_k < cfg.E:
        assert (ref["topk_w"].sum(1) < 1.0).all()        # not renormalised


def test_edge_cases(mm, gc, oracle):
    # a single token
    staged_vs_oracle(mm, gc, oracle, synth.Config("one_token", 1, 256, 256, 2, 4, 2, "bf16", "swiglu", seed=10))
    # every pick lands in one slot, all other slots are empty; two picks of a token share a slot
    cfg = synth.Config("one_slot", 130, 256, 256, 2, 4, 2, "bf16", "swiglu", seed=11)
    inp = synth.make_inputs(cfg)
    inp["M"][:] = 2
    case, ref = staged_vs_oracle(mm, gc, oracle, cfg, inp)
    assert ref["counts"][2] == 260 and ref["counts"].sum() == 260
    # exact ties in the router: duplicated router rows and an all-zero token
    cfg = synth.Config("ties", 64, 256, 256, 1, 6, 3, "f32", "relu", seed=12)
    inp = synth.make_inputs(cfg)
    inp["Wr"][0, 4] = inp["Wr"][0, 1]
    inp["Wr"][0, 5] = inp["Wr"][0, 2]
    inp["X"][7] = 0.0
    case, ref = staged_vs_oracle(mm, gc, oracle, cfg, inp)
    assert list(ref["topk_idx"][7]) == [0, 1, 2]
    # E above one wavefront's width, k = 8
    staged_vs_oracle(mm, gc, oracle, synth.Config("wide_e", 40, 256, 256, 1, 130, 8, "bf16", "relu", seed=13))
    staged_vs_oracle(mm, gc, oracle, synth.Config("wide_e_many", 2050, 256, 256, 1, 130, 8, "bf16", "relu", seed=19))


def test_validate_inputs(mm, gc):
    cfg = synth.Config("val", 16, 256, 256, 2, 4, 1, "f32", "relu", seed=14)
    case = gc.DeviceCase(cfg)
    assert mm.validate_inputs(case.shape, case.vid, case.M, case.ws)
    bad = case.vid.clone()
    bad[3] = 2
    assert not mm.validate_inputs(case.shape, bad, case.M, case.ws)
    badM = case.M.clone()
    badM[1, 1] = case.S
    assert not mm.validate_inputs(case.shape, case.vid, badM, case.ws)


def packed_layout_bf16(W):
    """Plain [S, K, N] ("in x out") bf16 bit patterns -> the documented fragment layout, by the
    index formula of include/mmoe.h (written with numpy index arithmetic, no kernel code)."""
    S, K, N = W.shape
    n = np.arange(N)[None, :]
    k = np.arange(K)[:, None]
    m, h, kk = k // 64, (k % 64) // 32, (k % 32) // 8
    ks = 4 * m + kk
    off = ((((n // 32) * (K // 16) + ks) * 64 + 32 * h + n % 32) * 8 + k % 8)        # [K, N], within a slot
    out = np.empty((S, K * N), W.dtype)
    for s in range(S):
        out[s, off.reshape(-1)] = W[s].reshape(-1)
    return out


def test_pack_round_trip(mm, gc):
    cfg = synth.Config("pack", 4, 256, 512, 1, 3, 1, "bf16", "swiglu", seed=15)
    inp = synth.make_inputs(cfg)
    case = gc.DeviceCase(cfg, inp)
    for packed, plain in ((case.W1p, inp["W1"]), (case.W3p, inp["W3"]), (case.W2p, inp["W2"])):
        got = gc.bits(packed).reshape(plain.shape[0], -1)
        assert np.array_equal(got, packed_layout_bf16(plain))
    cfg = synth.Config("pack32", 4, 256, 512, 1, 2, 1, "f32", "relu", seed=16)
    inp = synth.make_inputs(cfg)
    case = gc.DeviceCase(cfg, inp)
    assert np.array_equal(gc.bits(case.W1p), inp["W1"].transpose(0, 2, 1))      # fp32: the transpose
    assert np.array_equal(gc.bits(case.W2p), inp["W2"].transpose(0, 2, 1))


FULL_SMALL = ["switch8_fp32_v2_t128", "switch8_bf16_v4_t4096", "mixtral_decode_bf16_v2_t64"]


@pytest.mark.parametrize("name", FULL_SMALL)
def test_benchmark_shapes_full_parity(mm, gc, oracle, name):
    staged_vs_oracle(mm, gc, oracle, synth.CONFIGS[name])


@pytest.mark.parametrize("name,seed", [("mixtral_prefill_bf16_v2_t8192", 0), ("mixtral_skew_bf16_v4_t16384", 0),
                                       ("mixtral_prefill_bf16_v2_t8192", 1)])
def test_benchmark_shapes_sampled_parity(mm, gc, oracle, name, seed):
    """Full-size layers in the benchmark's launch configuration: integer outputs on every
    token; expert outputs on every row of the smallest and of the largest slot; layer outputs
    on 512 seeded tokens that the oracle evaluates one by one."""
    cfg = synth.CONFIGS[name].replace(seed=seed)
    print(f"case {name} seed {seed}: generating", flush=True)
    case = gc.DeviceCase(cfg)
    inp, sh = case.inp, case.shape
    print("routing oracle", flush=True)
    idx_ref, w_ref, _ = oracle.route(inp["X"], inp["vid"], inp["Wr"], inp["br"], cfg.top_k, cfg.dtype)
    slot_ref, counts_ref, offsets_ref, perm_ref, inv_ref = oracle.remap_group(inp["vid"], idx_ref, inp["M"], case.S)

    idx, w = mm.route(sh, case.X, case.vid, case.Wr, case.br)
    slot, counts, offsets, perm, inv, Xg = mm.remap_permute(sh, case.X, case.vid, idx, case.M, case.ws)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), idx_ref)
    np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=2e-6, atol=1e-7)
    for got, ref in ((slot, slot_ref), (counts, counts_ref), (offsets, offsets_ref), (perm, perm_ref), (inv, inv_ref)):
        assert np.array_equal(got.cpu().numpy(), ref)
    assert np.array_equal(gc.bits(Xg), inp["X"][perm_ref // cfg.top_k])
    print("slot counts min/median/max:", counts_ref.min(), int(np.median(counts_ref)), counts_ref.max(), flush=True)

    # staged expert stage and combination, then the fused entry point: bit-equal to each other
    Yg = mm.expert_ffn(sh, Xg, offsets, case.W1p, case.W3p, case.W2p, case.ws)
    Ys = mm.combine(sh, Yg, inv, w)
    Y = case.forward()
    torch.cuda.synchronize()
    assert torch.isfinite(Y.float()).all()
    assert torch.equal(Y, Ys), "fused entry point differs from the staged path"

    # every row of the smallest and of the largest slot, one expert evaluation each
    smallest, largest = int(np.argmin(np.where(counts_ref > 0, counts_ref, 1 << 30))), int(np.argmax(counts_ref))
    for s in (smallest, largest):
        r0, r1 = int(offsets_ref[s]), int(offsets_ref[s + 1])
        print(f"expert oracle on all {r1 - r0} rows of slot {s}", flush=True)
        rows = np.arange(r0, r1)
        Yg_ref = oracle.ffn_rows(inp["X"], (perm_ref[rows] // cfg.top_k).astype(np.int32),
                                 np.full(r1 - r0, s, np.int32), inp["W1"], inp["W3"], inp["W2"], cfg.dtype, cfg.act)
        gc.assert_close(gc.to_np64(Yg[r0:r1]), Yg_ref, cfg.dtype, f"Yg (all rows of slot {s})")
    # a seeded sample of tokens through the whole layer
    toks = np.sort(np.random.default_rng(7).choice(cfg.T, 512, replace=False))
    print(f"layer oracle on {len(toks)} sampled tokens", flush=True)
    Y_ref = oracle.layer_tokens(inp, cfg.top_k, cfg.dtype, cfg.act, toks, routed=(idx_ref, w_ref, slot_ref))
    gc.assert_close(gc.to_np64(Y[torch.from_numpy(toks).cuda()]), Y_ref, cfg.dtype, "Y (sampled)")


def test_decode_sizes_one_to_sixty_four_tokens(mm, gc, oracle):
    """Single-request decode is the paper's own workload (section 4).  The Mixtral-shaped layer at
    1, 2, 4, ... 64 tokens on one pool: the fused entry point (four launches, the expert kernels
    group the pairs themselves) against the oracle on every token, bit-equal to the staged calls
    and to itself on a second run."""
    cfg64 = synth.CONFIGS["mixtral_decode_bf16_v2_t64"]
    case = gc.DeviceCase(cfg64)
    for T in (1, 2, 4, 8, 16, 32, 64):
        print(f"decode T={T}", flush=True)
        cfg = cfg64.replace(T=T)
        sh = mm.make_shape(T, cfg.d_model, cfg.d_ff, cfg.V, cfg.E, case.S, cfg.top_k, cfg.dtype, cfg.act)
        inp = dict(case.inp, X=case.inp["X"][:T], vid=case.inp["vid"][:T])
        X, vid = case.X[:T].contiguous(), case.vid[:T].contiguous()
        ref = oracle.layer_forward(inp, cfg.top_k, cfg.dtype, cfg.act)
        Y = mm.layer_forward(sh, X, vid, case.Wr, case.br, case.M, case.W1p, case.W3p, case.W2p, case.ws)
        torch.cuda.synchronize()
        gc.assert_close(gc.to_np64(Y), ref["Y"], cfg.dtype, f"Y at T={T}")
        idx, w = mm.route(sh, X, vid, case.Wr, case.br)
        slot, counts, offsets, perm, inv, Xg = mm.remap_permute(sh, X, vid, idx, case.M, case.ws)
        assert np.array_equal(idx.cpu().numpy(), ref["topk_idx"]) and np.array_equal(perm.cpu().numpy(), ref["perm"])
        Ys = mm.combine(sh, mm.expert_ffn(sh, Xg, offsets, case.W1p, case.W3p, case.W2p, case.ws), inv, w)
        Y2 = mm.layer_forward(sh, X, vid, case.Wr, case.br, case.M, case.W1p, case.W3p, case.W2p, case.ws)
        torch.cuda.synchronize()
        assert torch.equal(Y, Ys), f"T={T}: fused entry point differs from the staged path"
        assert torch.equal(Y, Y2), f"T={T}: two runs differ"


def test_limits_many_slots_and_widest_router(mm, gc, oracle):
    """Close to the documented limits: a pool of several hundred slots (most of them empty or
    nearly empty for a small batch), and E = 256 experts with k = 8."""
    cfg = synth.Config("many_slots", 300, 256, 256, 64, 16, 2, "bf16", "swiglu", seed=20, share_prob=0.1)
    case, ref = staged_vs_oracle(mm, gc, oracle, cfg)
    assert 800 < case.S <= 1024 and (ref["counts"] == 0).any()
    cfg = synth.Config("many_slots_f32", 90, 256, 256, 40, 16, 1, "f32", "relu", seed=21, share_prob=0.2)
    staged_vs_oracle(mm, gc, oracle, cfg)
    staged_vs_oracle(mm, gc, oracle, synth.Config("widest_e", 70, 512, 256, 1, 256, 8, "bf16", "relu", seed=22))
    # many slots and enough rows for the matrix-core kernels (hundreds of short tile lists)
    cfg = synth.Config("many_slots_tiled", 6000, 256, 256, 8, 16, 2, "bf16", "swiglu", seed=23, share_prob=0.3)
    case, ref = staged_vs_oracle(mm, gc, oracle, cfg)
    assert case.S > 80
    # several hundred slots and more pairs than one grouping workgroup takes: the scatter workgroups sum
    # four slots per thread of the per-workgroup histograms themselves
    cfg = synth.Config("many_slots_two_chunks", 1200, 256, 256, 64, 16, 2, "bf16", "swiglu", seed=30, share_prob=0.1)
    case, ref = staged_vs_oracle(mm, gc, oracle, cfg)
    assert 800 < case.S <= 1024
    # the same pool with enough rows per slot for the matrix-core kernels: nine hundred short tile lists,
    # a target height chosen over all of them
    cfg = synth.Config("many_slots_tiled_wide", 20000, 256, 256, 64, 16, 2, "bf16", "relu", seed=31, share_prob=0.1)
    case, ref = staged_vs_oracle(mm, gc, oracle, cfg)
    assert 800 < case.S <= 1024 and mm.expert_plan(case.shape)[0] is False


@pytest.mark.parametrize("name", ["switch8_fp32_v2_t128", "switch8_bf16_v4_t4096", "mixtral_decode_bf16_v2_t64"])
def test_benchmark_shapes_second_seed(mm, gc, oracle, name):
    """Robustness row: the same shapes with another seed (another table, other counts)."""
    staged_vs_oracle(mm, gc, oracle, synth.CONFIGS[name].replace(seed=1))


def test_layer_forward_in_a_captured_graph(mm, gc, oracle):
    """The fused entry point allocates nothing and never synchronises, so a caller can record
    it into a HIP graph.  Every replay, with new tokens written into the same buffers in
    between and eager work around it, must reproduce the eager result bit for bit."""
    for cfg in (synth.Config("graph_stream", 48, 512, 768, 2, 4, 2, "bf16", "swiglu", seed=24),
                synth.Config("graph_tiled", 800, 256, 512, 2, 4, 2, "bf16", "swiglu", seed=25),
                # one pick per token: three launches (stream) or five (tiled), the down product writes Y
                synth.Config("graph_stream_top1", 40, 256, 512, 3, 8, 1, "f32", "gelu", seed=32, gate="all"),
                synth.Config("graph_tiled_top1", 2500, 256, 512, 3, 8, 1, "bf16", "relu", seed=33, gate="all")):
        case = gc.DeviceCase(cfg)
        sh = case.shape
        Y = torch.empty((cfg.T, cfg.d_model), dtype=case.X.dtype, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):    # warm-up on the capture stream, as graph capture requires
            mm.layer_forward(sh, case.X, case.vid, case.Wr, case.br, case.M, case.W1p, case.W3p, case.W2p,
                             case.ws, Y=Y)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            mm.layer_forward(sh, case.X, case.vid, case.Wr, case.br, case.M, case.W1p, case.W3p, case.W2p,
                             case.ws, Y=Y)
        for rep in range(3):
            inp = synth.make_inputs(cfg.replace(seed=100 + rep), weights=False)
            case.X.copy_(gc.to_dev(inp["X"], cfg.dtype))
            case.vid.copy_(torch.from_numpy(inp["vid"]).cuda())
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = Y.clone()
            eager = case.forward()
            torch.cuda.synchronize()
            assert torch.equal(got, eager), f"{cfg.name}: replay {rep} differs from the eager result"
        # and against the oracle once, for the last batch (same pool and table, new tokens)
        last = dict(case.inp, X=inp["X"], vid=inp["vid"])
        ref = oracle.layer_forward(last, cfg.top_k, cfg.dtype, cfg.act, gate=cfg.gate)
        gc.assert_close(gc.to_np64(got), ref["Y"], cfg.dtype, "Y (graph replay)")


def _random_configs(n, seed):
    """Seeded sweep over shapes: both dtypes and activations, every k up to E, token counts on
    both sides of every dispatch threshold (router variants, streaming vs tiled expert
    kernels, one or several grouping workgroups), with and without a router bias."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        dtype = "f32" if i % 4 == 3 else "bf16"
        act = "relu" if i % 3 == 2 else "swiglu"
        d = int(rng.choice([256, 512, 768, 1024]))
        f = int(rng.choice([256, 512, 1280]))
        V = int(rng.integers(1, 5))
        E = int(rng.integers(1, 10))
        k = int(rng.integers(1, min(E, 4) + 1))
        T = int(rng.choice([1, 7, 64, 200, 511, 512, 700, 1100, 2047, 2048, 2300]))
        if dtype == "f32":
            T = min(T, 300) if i % 2 else T  # fp32 never uses the tiled kernels; half the cases stay small
        out.append(synth.Config(f"rnd{i}_{dtype}_{act}_T{T}_d{d}_f{f}_V{V}_E{E}_k{k}", T, d, f, V, E, k, dtype, act,
                                seed=1000 + i, bias_alpha=float(rng.choice([0.0, 0.5])),
                                vid_mode=str(rng.choice(["uniform", "zipf", "interleave"])),
                                share_prob=float(rng.choice([0.0, 0.5, 1.0]))))
    return out


@pytest.mark.parametrize("cfg", _random_configs(24, seed=2024), ids=lambda c: c.name)
def test_random_shapes(mm, gc, oracle, cfg):
    staged_vs_oracle(mm, gc, oracle, cfg)


def test_ceiling_probe_reports_plausible_rates(mm):
    gbs, tflops = mm.probe_ceilings(gib=1)
    assert 2000.0 < gbs < 8000.0, gbs          # below the 8 TB/s data-sheet peak, above a third of it
    assert 500.0 < tflops < 2500.0, tflops     # below the 2.5 PFLOP/s data-sheet peak
