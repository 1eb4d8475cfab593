"""The layer with part of the pool in host memory (Algorithm 2's miss branch) through the C ABI:
the output must be bit-identical to the fully resident layer and match the oracle; the set of
fetched slots must be exactly the non-resident slots that the oracle's histogram says are touched."""
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


def paged_case(mm, gc, oracle, cfg, resident_of):
    print(f"case {cfg.name} T={cfg.T} d={cfg.d_model} f={cfg.d_ff} V={cfg.V} E={cfg.E} k={cfg.top_k} {cfg.dtype} "
          f"{cfg.act}", flush=True)
    case = gc.DeviceCase(cfg)
    S, sh = case.S, case.shape
    ref = oracle.layer_forward(case.inp, cfg.top_k, cfg.dtype, cfg.act, gate=cfg.gate)
    want_full = case.forward()
    torch.cuda.synchronize()
    gated = case.W3p is not None
    pools = [p for p in (case.W1p, case.W3p, case.W2p)]
    keep = [None if p is None else p.clone() for p in pools]
    resident = resident_of(S, ref["counts"])
    # pinned host copies of the non-resident slots (packed layout, one slot each); their place in the
    # device pool is overwritten with a pattern that would wreck the output if it were ever used
    host = []
    for p in pools:
        if p is None:
            host.append(None)
            continue
        flat = p.view(S, -1)
        lst = []
        for s in range(S):
            if resident[s]:
                lst.append(None)
            else:
                lst.append(flat[s].cpu().pin_memory())
                flat[s].fill_(float("nan"))
        host.append(lst)
    torch.cuda.synchronize()
    copy_stream = torch.cuda.Stream()
    Y, fetched = mm.layer_forward_paged(sh, case.X, case.vid, case.Wr, case.br, case.M, case.W1p, case.W3p, case.W2p,
                                        resident, host, case.ws, copy_stream)
    torch.cuda.synchronize()
    want_fetched = [int((not resident[s]) and ref["counts"][s] > 0) for s in range(S)]
    assert fetched == want_fetched, (fetched, want_fetched)
    assert torch.equal(Y, want_full), "paged layer differs from the fully resident one"
    gc.assert_close(gc.to_np64(Y), ref["Y"], cfg.dtype, "Y (paged)")
    # the fetched slots are now valid in the device pool; untouched non-resident ones still are not
    for p, k in zip(pools, keep):
        if p is None:
            continue
        for s in range(S):
            same = torch.equal(p.view(S, -1)[s].view(torch.int16 if p.dtype == torch.bfloat16 else torch.int32),
                               k.view(S, -1)[s].view(torch.int16 if p.dtype == torch.bfloat16 else torch.int32))
            assert same == bool(resident[s] or fetched[s]), (s, same)
    # next call with the arrivals marked resident: nothing left to fetch among the touched slots
    resident2 = [bool(r or f) for r, f in zip(resident, fetched)]
    Y2, fetched2 = mm.layer_forward_paged(sh, case.X, case.vid, case.Wr, case.br, case.M, case.W1p, case.W3p, case.W2p,
                                          resident2, host, case.ws, copy_stream)
    torch.cuda.synchronize()
    assert sum(fetched2) == 0 and torch.equal(Y2, want_full)
    return sum(fetched)


def every_other(S, counts):
    return [s % 2 == 0 for s in range(S)]


def none_resident(S, counts):
    return [False] * S


def all_resident(S, counts):
    return [True] * S


CASES = [
    (synth.Config("p_stream_bf16", 40, 512, 768, 2, 4, 2, "bf16", "swiglu", seed=61), every_other),
    (synth.Config("p_stream_f32", 50, 256, 512, 3, 4, 1, "f32", "relu", seed=62), none_resident),
    (synth.Config("p_tiled_bf16", 900, 512, 768, 2, 4, 2, "bf16", "swiglu", seed=63), every_other),
    (synth.Config("p_tiled_gelu_all", 1100, 256, 512, 3, 8, 1, "bf16", "gelu", seed=64, gate="all"), none_resident),
    (synth.Config("p_all_resident", 64, 256, 256, 2, 4, 2, "bf16", "swiglu", seed=65), all_resident),
    # a pool with slots that no token touches: those are never fetched
    (synth.Config("p_untouched", 6, 256, 256, 4, 8, 1, "bf16", "relu", seed=66), none_resident),
]


@pytest.mark.parametrize("cfg,resident_of", CASES, ids=lambda c: getattr(c, "name", None))
def test_paged_layer(mm, oracle, cfg, resident_of):
    import gpu_common as gc
    n = paged_case(mm, gc, oracle, cfg, resident_of)
    if resident_of is all_resident:
        assert n == 0
    else:
        assert n > 0
