"""The entry point that allocates nothing (mmoe_layer_forward_static) against mmoe_layer_forward:
same kernels, so the outputs must be bit-identical; two calls in a row share the library's one
scratch array, the second with a smaller batch (so it runs over whatever the first left there)."""
import numpy as np
import pytest
import torch

from paper_2505_06481_amd import synth

pytestmark = pytest.mark.gpu


def test_static_workspace_entry_point_matches_the_workspace_one(oracle):
    import gpu_common as gc
    from paper_2505_06481_amd import mmoe

    mmoe.lib()
    assert torch.cuda.is_available()
    cases = [
        # matrix-core expert kernels, several tiles per slot
        synth.Config("static_first", 900, 512, 768, 3, 4, 2, "bf16", "swiglu", seed=31),
        # weight-streaming expert kernels, fewer pairs, fewer slots, another dtype of the intermediates
        synth.Config("static_second_smaller", 40, 256, 512, 2, 4, 1, "f32", "relu", seed=32),
        # and a third, between the two in size, so that it also runs over a smaller call's leftovers
        synth.Config("static_third", 300, 256, 256, 2, 8, 2, "bf16", "relu", seed=33),
    ]
    for cfg in cases:
        print(f"case {cfg.name} T={cfg.T} d={cfg.d_model} f={cfg.d_ff} {cfg.dtype} {cfg.act}", flush=True)
        case = gc.DeviceCase(cfg)
        assert mmoe.workspace_bytes(case.shape) <= mmoe.STATIC_WORKSPACE_BYTES
        Y = torch.empty((cfg.T, cfg.d_model), dtype=case.X.dtype, device="cuda")
        Y.fill_(float("nan"))
        mmoe.layer_forward_static(case.shape, case.X, case.vid, case.Wr, case.br, case.M, case.W1p, case.W3p,
                                  case.W2p, Y=Y)
        torch.cuda.synchronize()
        want = case.forward()                      # the existing entry point, caller's workspace
        torch.cuda.synchronize()
        assert torch.equal(Y, want), f"{cfg.name}: differs from mmoe_layer_forward"
        ref = oracle.layer_forward(case.inp, cfg.top_k, cfg.dtype, cfg.act)
        gc.assert_close(gc.to_np64(Y), ref["Y"], cfg.dtype, cfg.name)
    # too large for the fixed array: refused with its own status, nothing launched
    import ctypes
    big = mmoe.make_shape(8192, 4096, 14336, 2, 8, 12, 2, "bf16", "swiglu")
    p = torch.zeros(64, device="cuda").data_ptr()
    rc = mmoe.lib().mmoe_layer_forward_static(ctypes.byref(big), p, p, p, None, p, p, p, p, p, None)
    assert rc == -11 and "MMOE_STATIC_WORKSPACE_BYTES" in mmoe.strerror(rc)
