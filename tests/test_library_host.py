"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, sizes the workspace, and turns bad arguments into error codes."""
import ctypes
import os
import re

import pytest

from paper_2505_06481_amd import build as mbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mm():
    if mbuild.is_stale():
        mbuild.build()
    from paper_2505_06481_amd import mmoe
    mmoe.lib()
    return mmoe


def test_every_declared_symbol_is_exported(mm):
    header = open(os.path.join(ROOT, "include", "mmoe.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(mmoe_[a-z_0-9]+)\s*\(", header))
    assert declared == set(mm.EXPORTS)
    L = ctypes.CDLL(os.path.join(ROOT, "paper_2505_06481_amd", "libmmoe.so"))
    for name in declared:
        assert hasattr(L, name), name


def test_workspace_size_accounts_for_every_intermediate(mm):
    sh = mm.make_shape(8192, 4096, 14336, 2, 8, 12, 2, "bf16", "swiglu")
    P = 8192 * 2
    need = P * 14336 * 2 + P * 4096 * 4     # H + Yg (the fused layer keeps no gathered copy of the tokens)
    got = mm.workspace_bytes(sh)
    assert need <= got <= need + (1 << 20)
    assert mm.workspace_bytes(mm.make_shape(8, 100, 256, 1, 1, 1, 1, "f32", "relu")) == 0


def test_bad_arguments_become_error_codes(mm):
    L = mm.lib()
    ok = mm.make_shape(4, 256, 256, 1, 2, 2, 1, "f32", "relu")
    p = ctypes.c_void_p(4096)          # never dereferenced: checks fail before any launch
    none = None

    def route(shape, X=p, vid=p, Wr=p):
        return L.mmoe_route(ctypes.byref(shape), X, vid, Wr, none, p, p, none)

    assert route(ok, X=none) == -1                                                       # NULL
    assert route(mm.make_shape(0, 256, 256, 1, 2, 2, 1, "f32", "relu")) == -2            # dimension
    assert route(mm.make_shape(4, 256, 256, 1, 2, 2, 3, "f32", "relu")) == -3            # top_k > E
    assert route(mm.make_shape(4, 256, 256, 1, 16, 2, 9, "f32", "relu")) == -3           # top_k > 8
    assert route(mm.make_shape(4, 256, 256, 1, 2, 2, 1, 7, "relu")) == -4                # dtype
    assert route(mm.make_shape(4, 256, 256, 1, 2, 2, 1, "f32", 5)) == -4                 # activation
    assert route(mm.make_shape(4, 256, 256, 1, 2, 2, 1, "f32", "gelu", gate=2)) == -4     # gate mode
    assert route(mm.make_shape(4, 256, 256, 1, 2, 2, 1, "f32", "gelu", gate="all"), X=none) == -1
    assert route(mm.make_shape(4, 200, 256, 1, 2, 2, 1, "f32", "relu")) == -8            # multiple of 256
    assert route(mm.make_shape(4, 256, 256, 1, 300, 2, 1, "f32", "relu")) == -9          # E limit
    assert route(mm.make_shape(4, 256, 256, 1, 2, 5000, 1, "f32", "relu")) == -9         # S limit
    assert route(ok, X=ctypes.c_void_p(4100)) == -7                                      # alignment
    # the 2^31 limit of the matrix-core expert path is a property of the shape: refused by every entry
    # point before anything is launched, and the workspace size of such a shape is 0
    huge = mm.make_shape(100000, 4096, 14336, 2, 8, 12, 2, "bf16", "swiglu")
    assert route(huge) == -9 and mm.workspace_bytes(huge) == 0
    # expert stage: W3 must match the activation; workspace must be large enough
    gated = mm.make_shape(4, 256, 256, 1, 2, 2, 1, "bf16", "swiglu")
    assert L.mmoe_expert_ffn(ctypes.byref(gated), p, p, p, none, p, p, p, 1 << 30, none) == -5
    assert L.mmoe_expert_ffn(ctypes.byref(ok), p, p, p, p, p, p, p, 1 << 30, none) == -5
    gelu = mm.make_shape(4, 256, 256, 1, 2, 2, 1, "bf16", "gelu")
    assert L.mmoe_expert_ffn(ctypes.byref(gelu), p, p, p, p, p, p, p, 1 << 30, none) == -5   # GELU takes no W3
    assert L.mmoe_expert_ffn(ctypes.byref(ok), p, p, p, none, p, p, p, 16, none) == -6
    assert L.mmoe_expert_ffn(ctypes.byref(ok), p, p, p, none, p, p, none, 1 << 30, none) == -6
    assert L.mmoe_layer_forward(ctypes.byref(ok), p, p, p, none, p, p, none, p, p, ctypes.c_void_p(4352), 8,
                                none) == -6
    assert L.mmoe_layer_forward(ctypes.byref(ok), p, p, p, none, p, p, none, p, p, ctypes.c_void_p(4100),
                                1 << 30, none) == -7
    assert L.mmoe_pack_weights(ctypes.byref(gated), p, none, p, p, p, p, none) == -5
    assert L.mmoe_combine(ctypes.byref(ok), none, p, p, p, none) == -1
    assert L.mmoe_remap_permute(ctypes.byref(ok), p, p, p, p, p, p, p, p, p, p, none, 0, none) == -6
    # the entry point without a workspace refuses, before any GPU call, what its fixed array cannot hold
    big = mm.make_shape(8192, 4096, 14336, 2, 8, 12, 2, "bf16", "swiglu")
    assert mm.workspace_bytes(big) > mm.STATIC_WORKSPACE_BYTES
    assert L.mmoe_layer_forward_static(ctypes.byref(big), p, p, p, none, p, p, p, p, p, none) == -11
    assert L.mmoe_layer_forward_static(ctypes.byref(mm.make_shape(0, 256, 256, 1, 2, 2, 1, "f32", "relu")),
                                       p, p, p, none, p, p, none, p, p, none) == -2
    for code in range(0, -12, -1):
        assert mm.strerror(code) != "unknown status"
    assert mm.strerror(-99) == "unknown status"


def test_paged_layer_argument_checks(mm):
    L = mm.lib()
    p = ctypes.c_void_p(4096)
    q = ctypes.c_void_p(8192)
    sh = mm.make_shape(4, 256, 256, 1, 2, 2, 1, "f32", "relu")
    res = (ctypes.c_uint8 * 2)(1, 0)
    hp = (ctypes.c_void_p * 2)(None, 4096)
    none_hp = (ctypes.c_void_p * 2)(None, None)
    big = ctypes.c_size_t(1 << 30)

    def call(resident=res, h1=hp, h2=hp, h3=None, W3=None, stream=p, copy=q, ws=p, ws_bytes=big):
        return L.mmoe_layer_forward_paged(ctypes.byref(sh), p, p, p, None, p, p, W3, p, resident, h1, h3, h2, p, ws,
                                          ws_bytes, stream, copy, None)

    assert call(resident=None) == -1
    assert call(h1=none_hp) == -1                      # a non-resident slot without a host copy
    assert call(copy=p) == -1                          # the copies need a stream of their own
    assert call(copy=None) == -1
    assert call(W3=p) == -5                            # RELU takes no W3
    assert call(ws_bytes=ctypes.c_size_t(8)) == -6


def test_expert_map_builder_argument_checks(mm):
    L = mm.lib()
    p = ctypes.c_void_p(4096)
    ok = mm.make_loader_shape(2, 3, 4, [256 * 512] * 2, "bf16", 5)
    ptrs = (ctypes.c_void_p * 4)(4096, 4096, 4096, 4096)
    need = L.mmoe_loader_workspace_bytes(ctypes.byref(ok))
    assert need >= 3 * 4 * 2 * 8                               # a partial sum per location and chunk
    assert L.mmoe_expert_distance(ctypes.byref(ok), ptrs, p, p, 16, None) == -6          # workspace too small
    assert L.mmoe_expert_distance(ctypes.byref(ok), None, p, p, need, None) == -1
    bad = (ctypes.c_void_p * 4)(4096, 4100, 4096, 4096)
    assert L.mmoe_expert_distance(ctypes.byref(ok), bad, p, p, need, None) == -7          # misaligned matrix
    for shape, code in ((mm.make_loader_shape(9, 3, 4, [256], "bf16", 1), -9),           # more than 8 variants
                        (mm.make_loader_shape(2, 100, 100, [256], "bf16", 1), -9),       # more than 4096 locations
                        (mm.make_loader_shape(2, 3, 4, [100], "bf16", 1), -8),           # not a multiple of 256
                        (mm.make_loader_shape(2, 3, 4, [256], "bf16", -1), -2),          # negative capacity
                        (mm.make_loader_shape(2, 0, 4, [256], "bf16", 1), -2),
                        (mm.make_loader_shape(2, 3, 4, [256], 7, 1), -4)):
        assert L.mmoe_loader_workspace_bytes(ctypes.byref(shape)) == 0
        assert L.mmoe_build_expert_map(ctypes.byref(shape), p, p, p, p, p, p, None) == code
    assert L.mmoe_build_expert_map(ctypes.byref(ok), p, p, None, p, p, p, None) == -1
    pool = (ctypes.c_void_p * 2)(4096, 4096)
    assert L.mmoe_assemble_pool(ctypes.byref(ok), ptrs, p, 3, 4, pool, None) == -2      # layer out of range
    assert L.mmoe_assemble_pool(ctypes.byref(ok), ptrs, p, 0, 9, pool, None) == -2      # more slots than V*E
    assert L.mmoe_assemble_pool(ctypes.byref(ok), ptrs, None, 0, 4, pool, None) == -1
    assert L.mmoe_assemble_pool(ctypes.byref(ok), ptrs, p, 0, 4, (ctypes.c_void_p * 2)(4096, 4100), None) == -7


def test_binding_refuses_host_tensors(mm):
    import torch
    sh = mm.make_shape(4, 256, 256, 1, 2, 2, 1, "f32", "relu")
    with pytest.raises(ValueError):
        mm.route(sh, torch.zeros(4, 256), torch.zeros(4, dtype=torch.int32), torch.zeros(1, 2, 256))


def test_tile_rows_field_accepts_only_its_three_values(mm):
    for good in (128, 256, 0):
        assert mm.workspace_bytes(mm.make_shape(512, 256, 256, 1, 2, 2, 1, "bf16", "relu", tile_rows=good)) > 0
    p = ctypes.c_void_p(4096)
    for bad in (64, 512, -1, 100):
        sh = mm.make_shape(512, 256, 256, 1, 2, 2, 1, "bf16", "relu", tile_rows=bad)
        assert mm.workspace_bytes(sh) == 0
        assert mm.lib().mmoe_route(ctypes.byref(sh), p, p, p, None, p, p, None) == -2


def test_probe_rejects_bad_arguments_before_touching_the_gpu(mm):
    L = mm.lib()
    out = (ctypes.c_float * 2)()
    p = ctypes.c_void_p(4096)
    assert L.mmoe_probe_ceilings(None, ctypes.c_size_t(1 << 30), out, None) == -1
    assert L.mmoe_probe_ceilings(p, ctypes.c_size_t(1 << 30), None, None) == -1
    assert L.mmoe_probe_ceilings(p, ctypes.c_size_t(1 << 20), out, None) == -6     # buffer too small
    assert L.mmoe_probe_ceilings(ctypes.c_void_p(4097), ctypes.c_size_t(1 << 30), out, None) == -7


def test_expert_plan_follows_the_documented_dispatch(mm):
    from paper_2505_06481_amd import synth

    def plan(name_or_cfg, S, tile_rows=0):
        c = synth.CONFIGS[name_or_cfg] if isinstance(name_or_cfg, str) else name_or_cfg
        return mm.expert_plan(mm.make_shape(c.T, c.d_model, c.d_ff, c.V, c.E, S, c.top_k, c.dtype, c.act,
                                            tile_rows=tile_rows))

    assert plan("switch8_fp32_v2_t128", 12) == (True, 32)            # fp32 always streams
    assert plan("mixtral_decode_bf16_v2_t64", 13) == (True, 32)      # 10 rows per slot
    assert plan("switch8_bf16_v4_t4096", 20) == (False, 128)         # short reduction: 128-row tiles
    assert plan("mixtral_prefill_bf16_v2_t8192", 13) == (False, 256)
    assert plan("mixtral_skew_bf16_v4_t16384", 20) == (False, 256)
    mix = synth.CONFIGS["mixtral_decode_bf16_v2_t64"]
    assert plan(mix.replace(T=104), 13) == (True, 32)                # 16 rows per slot: still streaming
    assert plan(mix.replace(T=105), 13) == (False, 128)              # beyond: matrix-core kernels, small tiles
    assert plan(mix.replace(T=415), 13) == (False, 128)              # under 64 rows per slot
    assert plan(mix.replace(T=416), 13) == (False, 256)
    # the tuning field overrides the tile height only, and only for the call it is passed to
    assert plan("mixtral_prefill_bf16_v2_t8192", 13, tile_rows=128) == (False, 128)
    assert plan("mixtral_decode_bf16_v2_t64", 13, tile_rows=128) == (True, 32)
    assert plan("mixtral_prefill_bf16_v2_t8192", 13) == (False, 256)
