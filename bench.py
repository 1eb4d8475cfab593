#!/usr/bin/env python3
"""Benchmark of the multi-model MoE layer forward on one MI355X.

One step = one pass of the whole layer (route -> map/group -> expert FFN -> combine,
``mmoe_layer_forward``) over one batch of seeded synthetic input that is already resident
in HBM.  The default workload is the Mixtral-8x7B-shaped prefill layer (8192 tokens,
2 variants); the Mixtral-shaped decode layer (64 tokens) is run right after it on the same
pool and reported in the same JSON line under "decode".

Prints ONE JSON line: tokens/s of the layer, the roofline fraction of its dominant kernel
(timed live with HIP events recorded between the kernels of every timed step), and the CPU
oracle timed on a bounded sample of the same workload as a reported baseline.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM traffic of the dominant kernels, from two rocprofv3 --pmc passes over this script
# (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch; summaries under profiles/), each scaled by
# what the same counter reads for a plain 1 GiB device copy (--copy-calibration): FETCH_SIZE
# reads 0.5 KiB per KiB copied (factor 2.0), WRITE_SIZE 1.0 (factor 1.0).  The figures belong
# to one version of the kernel's sources (the kernel file and the tile-list builder that decides
# which tiles it runs); with any other version `traffic` is null.
TRAFFIC = {
    "ffn_tiled.hip": {"sources": ("ffn_tiled.hip", "tile_table.h"), "sha256": "010729f1edd0a95d7f56e6be3a7c729c20803eaf7298375dcf71424eaabbcee0",
                      "workload": "mixtral_prefill_bf16_v2_t8192",
                      "fetch_bytes": 10971821914, "write_bytes": 469762380},
    "ffn_skinny.hip": {"sources": ("ffn_skinny.hip",), "sha256": "6251fdfca2475672fcf8c0de351e5d1c7ea8df1bf17f56ce71ef8f3fdd6a3716",
                       "workload": "mixtral_decode_bf16_v2_t64",
                       "fetch_bytes": 3068027183, "write_bytes": 3670794},
}


TRAFFIC_SOURCE = ("recorded from two rocprofv3 --pmc passes (profiles/*counters.txt), not measured in this run; "
                  "null when the kernel source has changed since")


def measured_traffic(source, workload):
    """Counter-derived HBM bytes (read + written) per launch of the up-product kernel, or None
    if the kernel source has changed since the counters were taken."""
    import hashlib

    rec = TRAFFIC[source]
    h = hashlib.sha256()
    for name in rec["sources"]:
        with open(os.path.join(ROOT, "paper_2505_06481_amd", "csrc", name), "rb") as fh:
            h.update(fh.read())
    if h.hexdigest() != rec["sha256"] or workload != rec["workload"]:
        return None
    return rec["fetch_bytes"] + rec["write_bytes"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="mixtral_prefill_bf16_v2_t8192")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-shaped companion run")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing and the parity block")
    ap.add_argument("--no-second-seed", action="store_true", help="skip the robustness row (same workload, seed + 1)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the streaming-read / matrix-loop probes")
    ap.add_argument("--zero-pool", action="store_true",
                    help="diagnostic: same batch, routing and launch configuration, but an all-zero expert pool "
                         "(nothing toggles in the multipliers): separates the chip's power limit from the "
                         "kernels' cycle efficiency; the result is not a benchmark figure")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="0 = 96 tokens per oracle thread")
    ap.add_argument("--decode-sweep", action="store_true",
                    help="after the main workload (Mixtral-shaped pools only): the layer at 1, 2, 4, ... 64 tokens on "
                         "the same pool, with the weight bytes of the slots each batch touches and the fraction of "
                         "HBM peak over the whole layer")
    ap.add_argument("--miss-sweep", action="store_true",
                    help="after the main workload: one decode token on the same pool with 0, 1 and 2 of its two "
                         "experts held in pinned host memory instead of HBM (the paper's per-layer latency by hit "
                         "rate: the miss path of Algorithm 2)")
    ap.add_argument("--loader", default=None, metavar="TABLE_WORKLOAD",
                    help="instead of the layer: time the expert-map builder (Algorithm 1) on one of "
                         "synth.TABLE_CONFIGS; one step = distances of every expert location + ranking + tables")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy three times (reference point for HBM byte counters)")
    return ap.parse_args()


def to_dev(a):
    """numpy array in storage form (fp32, or bf16 bit patterns as uint16) -> device tensor."""
    import numpy as np
    import torch

    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


class HipEvents:
    """hipEvent_t handles created straight from the HIP runtime (timing enabled)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.ev = (ctypes.c_void_p * n)()
        for i in range(n):
            h = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(h))
            assert rc == 0, f"hipEventCreate failed ({rc})"
            self.ev[i] = h

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.ev[a], self.ev[b])
        assert rc == 0, f"hipEventElapsedTime failed ({rc})"
        return float(ms.value)

    def destroy(self):
        for h in self.ev:
            self.hip.hipEventDestroy(h)


def run_workload(cfg, inp, pool, steps, warmup):
    """Upload (pool already packed on the device), warm up, then two passes of `steps` layer
    forwards each.  Timed pass: the host clock around all steps, and inside every step two HIP
    events around the dominant kernel (the experts' up product) on the launch stream: the
    roofline's launch duration comes from the timed region itself.  Breakdown pass: the same
    launches with an event after every stage (an event record costs about 3 us of stream time,
    as much as one of the small kernels, so the five extra ones stay out of the timed pass)."""
    import numpy as np
    import torch

    from paper_2505_06481_amd import mmoe

    S = int(inp["S"])
    shape = mmoe.make_shape(cfg.T, cfg.d_model, cfg.d_ff, cfg.V, cfg.E, S, cfg.top_k, cfg.dtype, cfg.act, gate=cfg.gate)
    X, Wr = to_dev(inp["X"]), to_dev(inp["Wr"])
    vid, M = torch.from_numpy(inp["vid"]).cuda(), torch.from_numpy(inp["M"]).cuda()
    br = None if inp["br"] is None else torch.from_numpy(inp["br"]).cuda()
    ws = mmoe.alloc_workspace(shape)
    Y = torch.empty((cfg.T, cfg.d_model), dtype=X.dtype, device="cuda")
    W1p, W3p, W2p = pool
    NE = mmoe.NUM_EVENTS
    events = HipEvents(NE * steps)
    vp = ctypes.c_void_p

    def step(i=None, only=None):
        ev = None
        if i is not None:
            ev = (vp * NE)(*[events.ev[i * NE + s] if only is None or s in only else None for s in range(NE)])
        mmoe.layer_forward(shape, X, vid, Wr, br, M, W1p, W3p, W2p, ws, Y=Y, events=ev)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    around_up = (mmoe.EV_PERMUTE, mmoe.EV_FFN_UP)
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, only=around_up)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    up_ms = np.array([events.elapsed_ms(i * NE + around_up[0], i * NE + around_up[1]) for i in range(steps)])

    # the same steps with no event at all: what a caller that does not time stages sees (the two
    # events of the timed pass are a tenth of a step of the small workloads)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    wall_plain = time.perf_counter() - t0

    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    stage_ms = np.zeros((steps, NE - 1))
    for i in range(steps):
        for s in range(NE - 1):
            stage_ms[i, s] = events.elapsed_ms(i * NE + s, i * NE + s + 1)
    events.destroy()
    names = ["route", "permute", "ffn_up", "ffn_down", "combine"]
    stages = {n: float(stage_ms[:, j].mean()) for j, n in enumerate(names)}
    per_step = stage_ms.sum(axis=1)   # first kernel's start to last kernel's end, per step (HIP events)

    # per-slot row counts of this batch (for the byte/flop accounting of the roofline)
    idx = mmoe.route(shape, X, vid, Wr, br)[0]
    sl = mmoe.remap_permute(shape, X, vid, idx, M, ws)
    counts = sl[1].cpu().numpy()
    torch.cuda.synchronize()
    return dict(ms_per_step=wall / steps * 1e3, ms_per_step_no_events=wall_plain / steps * 1e3, up_ms=float(up_ms.mean()), stages_ms=stages, counts=counts, S=S, Y=Y,
                topk_idx=idx.cpu().numpy(), perm=sl[3].cpu().numpy(),
                events_ms={"median": float(np.median(per_step)), "min": float(per_step.min())})


def miss_sweep(cfg, inp, pool, shape, steps):
    """One token, its top-k experts in k slots: the whole layer (gate, map lookup, host
    synchronisation, copies of the missing experts from pinned host memory, experts, combination)
    with 0 .. k of those slots not resident.  Host clock around `steps` calls, each ending in a
    stream synchronisation."""
    import torch

    from paper_2505_06481_amd import mmoe, synth

    tcfg = cfg.replace(name=cfg.name + "_T1", T=1, vid_mode="uniform", bias_alpha=0.0)
    tinp = synth.make_inputs(tcfg, weights=False)
    S = int(inp["S"])
    sh = mmoe.make_shape(1, cfg.d_model, cfg.d_ff, cfg.V, cfg.E, S, cfg.top_k, cfg.dtype, cfg.act, gate=cfg.gate)
    X, Wr = to_dev(tinp["X"]), to_dev(tinp["Wr"])
    vid, M = torch.from_numpy(tinp["vid"]).cuda(), torch.from_numpy(inp["M"]).cuda()
    ws = mmoe.alloc_workspace(sh)
    idx = mmoe.route(sh, X, vid, Wr, None)[0]
    slots = [int(inp["M"][int(tinp["vid"][0]), int(e)]) for e in idx[0].cpu().numpy()]
    W1p, W3p, W2p = pool
    host = []
    for p in (W1p, W3p, W2p):
        host.append(None if p is None else
                    [p.view(S, -1)[s].cpu().pin_memory() if s in slots else None for s in range(S)])
    copy_stream = torch.cuda.Stream()
    mats = 3 if W3p is not None else 2
    expert_bytes = mats * cfg.d_model * cfg.d_ff * (2 if cfg.dtype == "bf16" else 4)
    rows, base_ms = [], None
    for missing in range(len(set(slots)) + 1):
        gone = set(slots[len(slots) - missing:]) if missing else set()
        resident = [s not in gone for s in range(S)]
        for _ in range(3):
            mmoe.layer_forward_paged(sh, X, vid, Wr, None, M, W1p, W3p, W2p, resident, host, ws, copy_stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            _, fetched = mmoe.layer_forward_paged(sh, X, vid, Wr, None, M, W1p, W3p, W2p, resident, host, ws, copy_stream)
            torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        assert sum(fetched) == len(gone)
        base_ms = ms if missing == 0 else base_ms
        row = {"experts_missing": missing, "of": len(slots), "ms_per_layer": ms}
        if missing:
            row["ms_per_missing_expert"] = (ms - base_ms) / missing
            row["host_to_device_GBps"] = missing * expert_bytes / ((ms - base_ms) * 1e-3) / 1e9
        rows.append(row)
    return {"tokens": 1, "expert_bytes": expert_bytes, "rows": rows,
            "note": "paper, one A100 over PCIe Gen4 (section 5.1, per-layer latency by hit rate): "
                    "1.2 / 29.2 / 56.8 ms with 2 / 1 / 0 experts resident, 27.8 ms per missing expert"}


def stage_rates(cfg, stages):
    """Algorithmic HBM bytes of the three small stages over their measured durations (GB/s):
    the router reads every token row once; grouping reads three and writes three integers per
    (token, pick) pair (the fused layer makes no gathered copy of the rows); the combination
    reads k fp32 expert-output rows per token and writes one row in the storage type."""
    es = 2 if cfg.dtype == "bf16" else 4
    P = cfg.T * cfg.top_k
    nbytes = {"route": cfg.T * cfg.d_model * es, "permute": P * 6 * 4,
              "combine": P * cfg.d_model * 4 + cfg.T * cfg.d_model * es}
    return {k: v / (stages[k] * 1e-3) / 1e9 for k, v in nbytes.items()}


def roofline(cfg, res, skinny):
    """Roofline of the dominant kernel, the experts' up product (W1 and, when gated, W3)."""
    d, f, k = cfg.d_model, cfg.d_ff, cfg.top_k
    nw = 2 if cfg.act == "swiglu" else 1
    es = 2 if cfg.dtype == "bf16" else 4
    P = cfg.T * k
    dur_s = res["up_ms"] * 1e-3     # HIP events around the kernel, in every step of the timed pass
    if skinny:
        # weight streaming: every slot with at least one row reads its nw [f, d] matrices once
        active = int((res["counts"] > 0).sum())
        alg_bytes = active * nw * d * f * es + P * d * es + P * f * es
        ach = alg_bytes / dur_s / 1e9
        return dict(bound="hbm", achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s", frac=ach / PEAK_HBM_GBS,
                    traffic=measured_traffic("ffn_skinny.hip", cfg.name), traffic_source=TRAFFIC_SOURCE,
                    kernel=("skinny_frag_kernel" if cfg.dtype == "bf16" else "skinny_kernel") + " (up product)",
                    bytes_per_launch=alg_bytes,
                    avg_launch_ms=dur_s * 1e3)
    flops = 2.0 * P * d * f * nw
    ach = flops / dur_s / 1e12
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_MFMA_TFLOPS
    return dict(bound="mfma", achieved=ach, peak=peak, unit="TFLOP/s", frac=ach / peak,
                traffic=measured_traffic("ffn_tiled.hip", cfg.name), traffic_source=TRAFFIC_SOURCE,
                kernel="tiled_kernel (up product)",
                flops_per_launch=flops, avg_launch_ms=dur_s * 1e3)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, inp, n_tokens, res):
    """The oracle as it stands, timed on this host: routing and grouping over every token,
    the expert stage and the combination over a seeded sample of tokens, extrapolated
    linearly to the whole batch.  The oracle's results are then compared with what the GPU
    produced in the timed runs: second return value, the parity block."""
    import numpy as np

    import oracle

    threads = oracle.threads()
    n = n_tokens if n_tokens > 0 else 96 * threads
    n = min(n, cfg.T)
    t0 = time.perf_counter()
    idx, w, _ = oracle.route(inp["X"], inp["vid"], inp["Wr"], inp["br"], cfg.top_k, cfg.dtype, cfg.gate)
    slot, _, _, perm, _ = oracle.remap_group(inp["vid"], idx, inp["M"], int(inp["S"]))
    t_route = time.perf_counter() - t0
    toks = np.sort(np.random.default_rng(0).choice(cfg.T, n, replace=False))
    t0 = time.perf_counter()
    Y_ref = oracle.layer_tokens(inp, cfg.top_k, cfg.dtype, cfg.act, toks, routed=(idx, w, slot))
    t_ffn = time.perf_counter() - t0
    est = t_route + t_ffn * cfg.T / n
    base = dict(value=cfg.T / est, unit="tokens/s", cores=threads, cpu=cpu_model(), kind="oracle",
                sample=f"routing+grouping on all {cfg.T} tokens ({t_route:.2f} s); expert FFN+combine on {n} "
                       f"seeded tokens ({t_ffn:.2f} s), extrapolated linearly to {cfg.T}")
    # parity of the timed GPU path with the oracle: integer outputs on every token, the layer's
    # output on the sampled tokens, to the tolerance the tests use
    import torch

    got = res["Y"][torch.from_numpy(toks).cuda()].float().cpu().numpy().astype(np.float64)
    err = np.abs(got - Y_ref)
    if cfg.dtype == "bf16":
        bound, tol = 1e-2 + 2e-2 * np.abs(Y_ref), "|d| <= 1e-2 + 2e-2 |ref|"
    else:
        rms = float(np.sqrt(np.mean(Y_ref * Y_ref)))
        bound, tol = 1e-4 * np.abs(Y_ref) + 1e-4 * rms, "|d| <= 1e-4 |ref| + 1e-4 rms(ref)"
    parity = dict(selected_experts_bit_equal=bool(np.array_equal(res["topk_idx"], idx)),
                  permutation_bit_equal=bool(np.array_equal(res["perm"], perm)),
                  tokens=int(n), max_abs=float(err.max()), max_abs_ref=float(np.abs(Y_ref).max()),
                  outside_tol=int((err > bound).sum()), tolerance=tol)
    return base, parity


def bench_loader(a):
    """The initial expert loader's table (Algorithm 1): every variant's experts resident in HBM, one step
    = distances of all locations, ranking, owners and per-layer tables.  HBM-bound: every stored element
    is read once."""
    import numpy as np
    import torch

    from paper_2505_06481_amd import mmoe, synth

    mmoe.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = synth.TABLE_CONFIGS[a.loader]
    t0 = time.perf_counter()
    variants = synth.make_variants(cfg)
    t_gen = time.perf_counter() - t0
    sh = mmoe.make_loader_shape(cfg.V, cfg.L, cfg.E, [cfg.d_model * cfg.d_ff] * cfg.mats, cfg.dtype, cfg.capacity)
    dev = [[to_dev(m) for m in mats] for mats in variants]
    torch.cuda.synchronize()
    es = 2 if cfg.dtype == "bf16" else 4
    nbytes = cfg.V * cfg.L * cfg.E * cfg.n_params * es
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * a.steps)]
    for _ in range(a.warmup):
        dist = mmoe.expert_distance(sh, dev)
        out = mmoe.build_expert_map(sh, dist)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        ev[2 * i].record()
        dist = mmoe.expert_distance(sh, dev)
        ev[2 * i + 1].record()
        out = mmoe.build_expert_map(sh, dist)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / a.steps * 1e3
    dist_ms = float(np.mean([ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(a.steps)]))
    ach = nbytes / (dist_ms * 1e-3) / 1e9
    res = {
        "metric": "expert-map builder (Algorithm 1): bytes of expert weights ranked per second",
        "value": nbytes / (ms * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "V": cfg.V, "L": cfg.L, "E": cfg.E, "d_model": cfg.d_model, "d_ff": cfg.d_ff,
                   "matrices_per_expert": cfg.mats, "capacity": cfg.capacity, "seed": cfg.seed,
                   "expert_bytes_total": nbytes, "host_generation_s": t_gen},
        "roofline": {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                     "traffic": None, "kernel": "expert_distance_kernel (+ its fixed-order finish)",
                     "bytes_per_launch": nbytes, "avg_launch_ms": dist_ms},
    }
    if not a.no_cpu_baseline:
        from oracle import table as tab

        # the oracle on a bounded sample of locations (all of them when that takes seconds), then the table
        n_loc = cfg.L * cfg.E
        per_loc = cfg.V * cfg.n_params * es
        sample = n_loc if n_loc * per_loc <= (8 << 30) else max(1, (8 << 30) // per_loc)
        locs = np.sort(np.random.default_rng(0).choice(n_loc, sample, replace=False))
        t0 = time.perf_counter()
        d_ref = np.array([tab.location_distance(
            [np.concatenate([m[l, e] for m in mats]) for mats in variants], cfg.dtype)
            for l, e in ((int(x) // cfg.E, int(x) % cfg.E) for x in locs)])
        t_cpu = time.perf_counter() - t0
        d_got = dist.cpu().numpy().reshape(-1)
        res["cpu_baseline"] = {"value": sample * per_loc / t_cpu / 1e9, "unit": "GB/s", "cores": oracle_threads(),
                               "cpu": cpu_model(), "kind": "oracle",
                               "sample": f"distances of {sample} of {n_loc} locations ({t_cpu:.2f} s)"}
        par = {"locations": int(sample), "max_rel_distance_err": float(np.max(np.abs(d_got[locs] - d_ref) / d_ref))}
        if sample == n_loc:
            ref = tab.build_table(d_ref.reshape(cfg.L, cfg.E), cfg.V, cfg.capacity)
            rank, owner, M, S, src = (t.cpu().numpy() for t in out)
            par.update(rank_bit_equal=bool(np.array_equal(rank, ref["rank"])),
                       owner_bit_equal=bool(np.array_equal(owner, ref["owner"])),
                       tables_bit_equal=bool(np.array_equal(M, ref["M"]) and np.array_equal(S, ref["S"])))
        res["parity"] = par
    print(json.dumps(res))


def oracle_threads():
    import oracle

    return oracle.threads()


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this layer runs on one GPU; --gpus must be 1 (no sharding, no collectives)", file=sys.stderr)
        sys.exit(2)
    if a.loader:
        return bench_loader(a)
    import torch

    from paper_2505_06481_amd import mmoe, synth

    mmoe.lib()  # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[a.workload]
    inp = synth.make_inputs(cfg)
    S = int(inp["S"])
    shape = mmoe.make_shape(cfg.T, cfg.d_model, cfg.d_ff, cfg.V, cfg.E, S, cfg.top_k, cfg.dtype, cfg.act, gate=cfg.gate)
    W1, W3, W2 = (to_dev(inp[k]) for k in ("W1", "W3", "W2"))
    pool = mmoe.pack_weights(shape, W1, W3, W2)   # one-time repacking at pool load, untimed
    if a.zero_pool:
        for w in pool:
            if w is not None:
                w.zero_()
    torch.cuda.synchronize()
    del W1, W3, W2
    torch.cuda.empty_cache()

    skinny, tile_rows = mmoe.expert_plan(shape)   # which expert-stage kernels the library uses for this shape
    res = run_workload(cfg, inp, pool, a.steps, a.warmup)
    ms = res["ms_per_step"]
    nw = 3 if cfg.act == "swiglu" else 2
    layer_flops = 2.0 * cfg.T * cfg.top_k * cfg.d_model * cfg.d_ff * nw
    out = {
        "metric": "MoE-layer tokens/s (multi-model consolidated pool, layer forward)",
        "value": cfg.T / (ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic" if not a.zero_pool else "synthetic tokens and routers, ALL-ZERO expert pool (diagnostic)",
        "config": {"workload": cfg.name, "T": cfg.T, "d_model": cfg.d_model, "d_ff": cfg.d_ff, "V": cfg.V,
                   "E": cfg.E, "top_k": cfg.top_k, "S": S, "act": cfg.act, "seed": cfg.seed,
                   "slot_rows_min_med_max": [int(res["counts"].min()), int(sorted(res["counts"])[S // 2]),
                                             int(res["counts"].max())],
                   "slot_rows": [int(c) for c in res["counts"]],
                   "expert_kernels": "weight-streaming" if skinny else f"matrix-core, {tile_rows}-row tiles"},
        "layer_tflops": layer_flops / (ms * 1e-3) / 1e12,
        "stages_ms": res["stages_ms"],
        "stages_GBps": stage_rates(cfg, res["stages_ms"]),
        "step_ms_by_events": res["events_ms"],
        "ms_per_step_no_events": res["ms_per_step_no_events"],
        "roofline": roofline(cfg, res, skinny),
    }

    if not a.no_decode and cfg.name == "mixtral_prefill_bf16_v2_t8192":
        dcfg = synth.CONFIGS["mixtral_decode_bf16_v2_t64"]
        dinp = synth.make_inputs(dcfg, weights=False)   # same seed, same pool: only the batch differs
        assert int(dinp["S"]) == S and (dinp["M"] == inp["M"]).all()
        dres = run_workload(dcfg, dinp, pool, max(a.steps, 50), a.warmup)
        dms = dres["ms_per_step"]
        active = int((dres["counts"] > 0).sum())
        out["decode"] = {
            "config": {"workload": dcfg.name, "T": dcfg.T, "S": S, "active_slots": active},
            "value": dcfg.T / (dms * 1e-3), "unit": "tokens/s", "ms_per_step": dms,
            "layer_gbs": active * 3 * dcfg.d_model * dcfg.d_ff * 2 / (dms * 1e-3) / 1e9,
            "stages_ms": dres["stages_ms"], "stages_GBps": stage_rates(dcfg, dres["stages_ms"]),
            "step_ms_by_events": dres["events_ms"], "ms_per_step_no_events": dres["ms_per_step_no_events"],
            "roofline": roofline(dcfg, dres, True),
        }

    if a.decode_sweep:
        # single-request decode is the paper's own workload (section 4: one request at a time, one
        # token per step); the layer's cost is then the weights of the few slots the batch touches
        base = synth.CONFIGS["mixtral_decode_bf16_v2_t64"] if cfg.d_model == 4096 else cfg
        sweep = []
        for T in (1, 2, 4, 8, 16, 32, 64):
            scfg = base.replace(name=f"{base.name}_T{T}", T=T, seed=cfg.seed, V=cfg.V, vid_mode="uniform",
                                bias_alpha=0.0)
            sinp = synth.make_inputs(scfg, weights=False)
            assert (sinp["M"] == inp["M"]).all()
            sres = run_workload(scfg, sinp, pool, max(a.steps, 200), a.warmup)
            active = int((sres["counts"] > 0).sum())
            nbytes = active * (3 if scfg.act == "swiglu" else 2) * scfg.d_model * scfg.d_ff * 2
            ms = sres["ms_per_step"]
            sweep.append({"T": T, "active_slots": active, "ms_per_step": ms, "weight_bytes": nbytes,
                          "layer_GBps": nbytes / (ms * 1e-3) / 1e9,
                          "hbm_frac": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                          "stages_ms": sres["stages_ms"]})
        out["decode_sweep"] = sweep

    if a.miss_sweep:
        out["miss_path"] = miss_sweep(cfg, inp, pool, shape, max(a.steps, 20))

    if not a.no_ceilings:
        # what this GPU delivers with nothing else in the way: a pure streaming read and a pure
        # matrix-instruction loop (the chip clocks down under matrix load, so the second figure is
        # well below the data-sheet peak that `roofline.peak` quotes)
        gbs, tflops = mmoe.probe_ceilings()
        out["achievable"] = {"stream_read_GBps": gbs, "mfma_bf16_loop_TFLOPps": tflops,
                             "roofline_frac_of_achievable": out["roofline"]["achieved"] / tflops}
        if "decode" in out:
            out["decode"]["roofline_frac_of_achievable"] = out["decode"]["roofline"]["achieved"] / gbs

    if a.copy_calibration:
        # a plain elementwise copy of known size: reads 1 GiB, writes 1 GiB per launch
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if not a.no_cpu_baseline:
        out["cpu_baseline"], out["parity"] = cpu_baseline(cfg, inp, a.cpu_sample_tokens, res)

    if not a.no_second_seed and not a.zero_pool:
        # robustness row: the same workload from another seed (another table, pool and batch)
        del pool
        torch.cuda.empty_cache()
        cfg2 = cfg.replace(seed=cfg.seed + 1)
        inp2 = synth.make_inputs(cfg2)
        S2 = int(inp2["S"])
        shape2 = mmoe.make_shape(cfg2.T, cfg2.d_model, cfg2.d_ff, cfg2.V, cfg2.E, S2, cfg2.top_k, cfg2.dtype, cfg2.act, gate=cfg2.gate)
        W1, W3, W2 = (to_dev(inp2[k]) for k in ("W1", "W3", "W2"))
        pool2 = mmoe.pack_weights(shape2, W1, W3, W2)
        torch.cuda.synchronize()
        del W1, W3, W2
        torch.cuda.empty_cache()
        res2 = run_workload(cfg2, inp2, pool2, a.steps, a.warmup)
        out["second_seed"] = {"seed": cfg2.seed, "S": S2, "ms_per_step": res2["ms_per_step"],
                              "value": cfg2.T / (res2["ms_per_step"] * 1e-3), "unit": "tokens/s",
                              "stages_ms": res2["stages_ms"],
                              "slot_rows_min_med_max": [int(res2["counts"].min()), int(sorted(res2["counts"])[S2 // 2]),
                                                        int(res2["counts"].max())]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
