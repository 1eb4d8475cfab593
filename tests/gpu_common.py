"""Helpers shared by the GPU parity tests: upload of synthetic inputs, tolerances."""
import numpy as np
import torch

from paper_2505_06481_amd import mmoe, synth


def to_dev(a, dtype):
    """numpy array in storage form (fp32, or bf16 bit patterns as uint16) -> device tensor."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_np64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def bits(t):
    """device tensor -> numpy storage form (bf16 as uint16 bit patterns)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class DeviceCase:
    """One workload resident on the GPU, pool packed once (not part of any timed region)."""

    def __init__(self, cfg, inp=None, tile_rows=0):
        self.cfg = cfg
        self.inp = inp if inp is not None else synth.make_inputs(cfg)
        i = self.inp
        self.S = int(i["S"])
        self.shape = mmoe.make_shape(cfg.T, cfg.d_model, cfg.d_ff, cfg.V, cfg.E, self.S, cfg.top_k, cfg.dtype, cfg.act,
                                     tile_rows=tile_rows, gate=cfg.gate)
        dt = cfg.dtype
        self.X, self.Wr = to_dev(i["X"], dt), to_dev(i["Wr"], dt)
        self.vid = torch.from_numpy(i["vid"]).cuda()
        self.M = torch.from_numpy(i["M"]).cuda()
        self.br = None if i["br"] is None else torch.from_numpy(i["br"]).cuda()
        W1, W3, W2 = to_dev(i["W1"], dt), to_dev(i["W3"], dt), to_dev(i["W2"], dt)
        self.W1p, self.W3p, self.W2p = mmoe.pack_weights(self.shape, W1, W3, W2)
        torch.cuda.synchronize()
        del W1, W3, W2
        self.ws = mmoe.alloc_workspace(self.shape)

    def forward(self):
        return mmoe.layer_forward(self.shape, self.X, self.vid, self.Wr, self.br, self.M, self.W1p, self.W3p,
                                  self.W2p, self.ws)


def assert_close_bf16(got, ref, what=""):
    """|got - ref| <= 1e-2 + 2e-2 |ref| elementwise (bf16 storage, fp32 accumulation)."""
    err = np.abs(got - ref)
    bound = 1e-2 + 2e-2 * np.abs(ref)
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst {err.max():.4g} " \
                          f"at ref {ref.flat[np.argmax(err - bound)]:.4g}"


def assert_close_f32(got, ref, what=""):
    """|got - ref| <= 1e-4 |ref| + 1e-4 rms(ref) elementwise (pure relative error is
    ill-posed at zero crossings)."""
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    err = np.abs(got - ref)
    bound = 1e-4 * np.abs(ref) + 1e-4 * rms
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst {err.max():.4g} (rms {rms:.4g})"


def assert_close(got, ref, dtype, what=""):
    (assert_close_bf16 if dtype == "bf16" else assert_close_f32)(got, ref, what)
