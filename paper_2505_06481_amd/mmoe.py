"""Python binding of libmmoe's C ABI (see include/mmoe.h).

Argument marshalling only: tensors are checked for device, dtype and contiguity, their
raw device pointers and the current HIP stream are handed to the library, and every
step of the layer runs in the library's kernels.  PyTorch supplies device memory and
streams, nothing else.  There is no fallback: if the HIP library is missing the import
of a function fails with an explanation.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmmoe.so")

F32, BF16 = 0, 1
RELU, SWIGLU, GELU = 0, 1, 2
GATE_SELECTED, GATE_ALL = 0, 1
_DTYPES = {"f32": F32, "bf16": BF16}
_ACTS = {"relu": RELU, "swiglu": SWIGLU, "gelu": GELU}
_GATES = {"selected": GATE_SELECTED, "all": GATE_ALL}
_TORCH_DT = {F32: torch.float32, BF16: torch.bfloat16}

EXPORTS = [
    "mmoe_workspace_bytes", "mmoe_strerror", "mmoe_pack_weights", "mmoe_route", "mmoe_remap_permute",
    "mmoe_expert_ffn", "mmoe_combine", "mmoe_layer_forward", "mmoe_layer_forward_events",
    "mmoe_layer_forward_static", "mmoe_layer_forward_paged", "mmoe_loader_workspace_bytes", "mmoe_expert_distance", "mmoe_build_expert_map",
    "mmoe_assemble_pool", "mmoe_validate_inputs", "mmoe_probe_ceilings", "mmoe_expert_plan",
]


class MmoeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("T", "d_model", "d_ff", "V", "E", "S", "top_k", "dtype", "act", "gate", "tile_rows")]


def make_shape(T, d_model, d_ff, V, E, S, top_k, dtype, act, tile_rows=0, gate="selected") -> Shape:
    """``gate``: "selected" (softmax over the selected logits) or "all" (probabilities over all
    experts, not renormalised).  ``tile_rows``: tuning field of the matrix-core expert kernels,
    0 = chosen by shape."""
    dt = _DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
    ac = _ACTS[act] if isinstance(act, str) else int(act)
    ga = _GATES[gate] if isinstance(gate, str) else int(gate)
    return Shape(T, d_model, d_ff, V, E, S, top_k, dt, ac, ga, tile_rows)


class LoaderShape(ctypes.Structure):
    _fields_ = [("V", ctypes.c_int32), ("L", ctypes.c_int32), ("E", ctypes.c_int32), ("n_mats", ctypes.c_int32),
                ("mat_elems", ctypes.c_int64 * 3), ("dtype", ctypes.c_int32), ("capacity", ctypes.c_int32)]


def make_loader_shape(V, L, E, mat_elems, dtype, capacity) -> LoaderShape:
    dt = _DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
    me = list(mat_elems) + [0] * (3 - len(mat_elems))
    return LoaderShape(V, L, E, len(mat_elems), (ctypes.c_int64 * 3)(*me), dt, capacity)


_lib = None


def lib():
    """Load libmmoe.so (built in-tree by ``__graft_entry__.build()`` / ``build.py``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2505_06481_amd.build` "
                "(hipcc, gfx950).  There is no CPU fallback.")
        L = ctypes.CDLL(_LIB_PATH)
        vp, sz, i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        sp = ctypes.POINTER(Shape)
        L.mmoe_workspace_bytes.restype = sz
        L.mmoe_workspace_bytes.argtypes = [sp]
        L.mmoe_strerror.restype = ctypes.c_char_p
        L.mmoe_strerror.argtypes = [i]
        L.mmoe_pack_weights.argtypes = [sp] + [vp] * 7
        L.mmoe_route.argtypes = [sp] + [vp] * 7
        L.mmoe_remap_permute.argtypes = [sp] + [vp] * 11 + [sz, vp]
        L.mmoe_expert_ffn.argtypes = [sp] + [vp] * 7 + [sz, vp]
        L.mmoe_combine.argtypes = [sp] + [vp] * 5
        L.mmoe_layer_forward.argtypes = [sp] + [vp] * 10 + [sz, vp]
        L.mmoe_layer_forward_events.argtypes = [sp] + [vp] * 10 + [sz, vp, vp]
        L.mmoe_layer_forward_static.argtypes = [sp] + [vp] * 10
        L.mmoe_layer_forward_paged.argtypes = [sp] + [vp] * 14 + [sz, vp, vp, vp]
        L.mmoe_validate_inputs.argtypes = [sp, vp, vp, vp, sz, vp]
        lp = ctypes.POINTER(LoaderShape)
        L.mmoe_loader_workspace_bytes.restype = sz
        L.mmoe_loader_workspace_bytes.argtypes = [lp]
        L.mmoe_expert_distance.argtypes = [lp, ctypes.POINTER(vp), vp, vp, sz, vp]
        L.mmoe_build_expert_map.argtypes = [lp] + [vp] * 7
        L.mmoe_assemble_pool.argtypes = [lp, ctypes.POINTER(vp), vp, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.POINTER(vp), vp]
        L.mmoe_expert_plan.argtypes = [sp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.mmoe_probe_ceilings.argtypes = [vp, sz, ctypes.POINTER(ctypes.c_float), vp]
        for n in EXPORTS[2:]:
            if n != "mmoe_loader_workspace_bytes":
                getattr(L, n).restype = i
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().mmoe_strerror(int(status)).decode()


def workspace_bytes(shape: Shape) -> int:
    return int(lib().mmoe_workspace_bytes(ctypes.byref(shape)))


def _ptr(t: Optional[torch.Tensor], dtype=None, numel=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name}: needs {numel} elements, has {t.numel()}")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str):
    if rc != 0:
        raise MmoeError(rc, where)


def alloc_workspace(shape: Shape, device="cuda") -> torch.Tensor:
    n = workspace_bytes(shape)
    if n == 0:
        raise MmoeError(int(lib().mmoe_route(ctypes.byref(shape), *([None] * 7))), "mmoe_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def pack_weights(shape: Shape, W1, W3, W2):
    """Plain [S,d,f]/[S,f,d] pool -> packed [S,f,d]/[S,d,f] pool (new tensors)."""
    dt = _TORCH_DT[shape.dtype]
    S, d, f = shape.S, shape.d_model, shape.d_ff
    W1p = torch.empty((S, f, d), dtype=dt, device=W1.device)
    W2p = torch.empty((S, d, f), dtype=dt, device=W1.device)
    W3p = torch.empty((S, f, d), dtype=dt, device=W1.device) if W3 is not None else None
    rc = lib().mmoe_pack_weights(ctypes.byref(shape), _ptr(W1, dt, S * d * f, "W1"), _ptr(W3, dt, S * d * f, "W3"),
                                 _ptr(W2, dt, S * d * f, "W2"), _ptr(W1p), _ptr(W3p), _ptr(W2p), _stream())
    _check(rc, "mmoe_pack_weights")
    return W1p, W3p, W2p


def route(shape: Shape, X, vid, Wr, br=None):
    dt = _TORCH_DT[shape.dtype]
    T, k = shape.T, shape.top_k
    idx = torch.empty((T, k), dtype=torch.int32, device=X.device)
    w = torch.empty((T, k), dtype=torch.float32, device=X.device)
    rc = lib().mmoe_route(ctypes.byref(shape), _ptr(X, dt, T * shape.d_model, "X"), _ptr(vid, torch.int32, T, "vid"),
                          _ptr(Wr, dt, shape.V * shape.E * shape.d_model, "Wr"),
                          _ptr(br, torch.float32, shape.V * shape.E, "br"), _ptr(idx), _ptr(w), _stream())
    _check(rc, "mmoe_route")
    return idx, w


def remap_permute(shape: Shape, X, vid, topk_idx, M, ws):
    dt = _TORCH_DT[shape.dtype]
    P, S = shape.T * shape.top_k, shape.S
    dev = X.device
    i32 = dict(dtype=torch.int32, device=dev)
    slot, perm, inv = (torch.empty(P, **i32) for _ in range(3))
    counts, offsets = torch.empty(S, **i32), torch.empty(S + 1, **i32)
    Xg = torch.empty((P, shape.d_model), dtype=dt, device=dev)
    rc = lib().mmoe_remap_permute(ctypes.byref(shape), _ptr(X, dt, shape.T * shape.d_model, "X"),
                                  _ptr(vid, torch.int32, shape.T, "vid"), _ptr(topk_idx, torch.int32, P, "topk_idx"),
                                  _ptr(M, torch.int32, shape.V * shape.E, "M"), _ptr(slot), _ptr(counts),
                                  _ptr(offsets), _ptr(perm), _ptr(inv), _ptr(Xg), _ptr(ws, torch.uint8, None, "ws"),
                                  ws.numel(), _stream())
    _check(rc, "mmoe_remap_permute")
    return slot, counts, offsets, perm, inv, Xg


def expert_ffn(shape: Shape, Xg, offsets, W1p, W3p, W2p, ws):
    dt = _TORCH_DT[shape.dtype]
    P, d, f, S = shape.T * shape.top_k, shape.d_model, shape.d_ff, shape.S
    Yg = torch.empty((P, d), dtype=torch.float32, device=Xg.device)
    rc = lib().mmoe_expert_ffn(ctypes.byref(shape), _ptr(Xg, dt, P * d, "Xg"),
                               _ptr(offsets, torch.int32, S + 1, "offsets"), _ptr(W1p, dt, S * d * f, "W1p"),
                               _ptr(W3p, dt, S * d * f, "W3p"), _ptr(W2p, dt, S * d * f, "W2p"), _ptr(Yg),
                               _ptr(ws, torch.uint8, None, "ws"), ws.numel(), _stream())
    _check(rc, "mmoe_expert_ffn")
    return Yg


def combine(shape: Shape, Yg, inv_perm, topk_w):
    dt = _TORCH_DT[shape.dtype]
    P = shape.T * shape.top_k
    Y = torch.empty((shape.T, shape.d_model), dtype=dt, device=Yg.device)
    rc = lib().mmoe_combine(ctypes.byref(shape), _ptr(Yg, torch.float32, P * shape.d_model, "Yg"),
                            _ptr(inv_perm, torch.int32, P, "inv_perm"), _ptr(topk_w, torch.float32, P, "topk_w"),
                            _ptr(Y), _stream())
    _check(rc, "mmoe_combine")
    return Y


NUM_EVENTS = 6
EV_START, EV_ROUTE, EV_PERMUTE, EV_FFN_UP, EV_FFN_DOWN, EV_COMBINE = range(NUM_EVENTS)


def layer_forward(shape: Shape, X, vid, Wr, br, M, W1p, W3p, W2p, ws, Y=None, events=None):
    """``events``: optional ctypes array of NUM_EVENTS hipEvent_t handles (c_void_p); null entries are skipped."""
    dt = _TORCH_DT[shape.dtype]
    S, d, f = shape.S, shape.d_model, shape.d_ff
    if Y is None:
        Y = torch.empty((shape.T, d), dtype=dt, device=X.device)
    rc = lib().mmoe_layer_forward_events(ctypes.byref(shape), _ptr(X, dt, shape.T * d, "X"),
                                  _ptr(vid, torch.int32, shape.T, "vid"), _ptr(Wr, dt, shape.V * shape.E * d, "Wr"),
                                  _ptr(br, torch.float32, shape.V * shape.E, "br"),
                                  _ptr(M, torch.int32, shape.V * shape.E, "M"), _ptr(W1p, dt, S * d * f, "W1p"),
                                  _ptr(W3p, dt, S * d * f, "W3p"), _ptr(W2p, dt, S * d * f, "W2p"),
                                  _ptr(Y, dt, shape.T * d, "Y"), _ptr(ws, torch.uint8, None, "ws"), ws.numel(),
                                  _stream(), events)
    _check(rc, "mmoe_layer_forward")
    return Y


STATIC_WORKSPACE_BYTES = 64 << 20


def layer_forward_static(shape: Shape, X, vid, Wr, br, M, W1p, W3p, W2p, Y=None):
    """The layer without a workspace argument (intermediates in the library's fixed device array)."""
    dt = _TORCH_DT[shape.dtype]
    S, d, f = shape.S, shape.d_model, shape.d_ff
    if Y is None:
        Y = torch.empty((shape.T, d), dtype=dt, device=X.device)
    rc = lib().mmoe_layer_forward_static(ctypes.byref(shape), _ptr(X, dt, shape.T * d, "X"),
                                         _ptr(vid, torch.int32, shape.T, "vid"),
                                         _ptr(Wr, dt, shape.V * shape.E * d, "Wr"),
                                         _ptr(br, torch.float32, shape.V * shape.E, "br"),
                                         _ptr(M, torch.int32, shape.V * shape.E, "M"),
                                         _ptr(W1p, dt, S * d * f, "W1p"), _ptr(W3p, dt, S * d * f, "W3p"),
                                         _ptr(W2p, dt, S * d * f, "W2p"), _ptr(Y, dt, shape.T * d, "Y"), _stream())
    _check(rc, "mmoe_layer_forward_static")
    return Y


def validate_inputs(shape: Shape, vid, M, ws) -> bool:
    rc = lib().mmoe_validate_inputs(ctypes.byref(shape), _ptr(vid, torch.int32, shape.T, "vid"),
                                    _ptr(M, torch.int32, shape.V * shape.E, "M"), _ptr(ws, torch.uint8, 256, "ws"),
                                    ws.numel(), _stream())
    if rc < 0:
        raise MmoeError(rc, "mmoe_validate_inputs")
    return rc == 0


def probe_ceilings(gib: int = 4):
    """(GB/s of a pure streaming read, TFLOP/s of a pure bf16 matrix-instruction loop) on this GPU."""
    buf = torch.zeros(gib << 30, dtype=torch.uint8, device="cuda")
    out = (ctypes.c_float * 2)()
    _check(lib().mmoe_probe_ceilings(_ptr(buf, torch.uint8, None, "buf"), buf.numel(), out, _stream()),
           "mmoe_probe_ceilings")
    return float(out[0]), float(out[1])


def expert_plan(shape: Shape):
    """(streaming, tile_rows): the expert-stage kernels the library will use for this shape."""
    streaming, rows = ctypes.c_int(), ctypes.c_int()
    _check(lib().mmoe_expert_plan(ctypes.byref(shape), ctypes.byref(streaming), ctypes.byref(rows)),
           "mmoe_expert_plan")
    return bool(streaming.value), int(rows.value)


def expert_distance(shape: LoaderShape, mats):
    """``mats[v][m]``: device tensor [L, E, mat_elems[m]] of variant v.  Returns distance [L, E] float64."""
    dt = _TORCH_DT[shape.dtype]
    n = shape.V * shape.n_mats
    ptrs = (ctypes.c_void_p * n)()
    for v in range(shape.V):
        for m in range(shape.n_mats):
            ptrs[v * shape.n_mats + m] = _ptr(mats[v][m], dt, shape.L * shape.E * shape.mat_elems[m], f"mats[{v}][{m}]")
    dev = mats[0][0].device
    need = int(lib().mmoe_loader_workspace_bytes(ctypes.byref(shape)))
    if need == 0:
        raise MmoeError(int(lib().mmoe_expert_distance(ctypes.byref(shape), ptrs, None, None, 0, None)),
                        "mmoe_loader_workspace_bytes")
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    dist = torch.empty((shape.L, shape.E), dtype=torch.float64, device=dev)
    _check(lib().mmoe_expert_distance(ctypes.byref(shape), ptrs, _ptr(dist), _ptr(ws), ws.numel(), _stream()),
           "mmoe_expert_distance")
    return dist


def build_expert_map(shape: LoaderShape, distance):
    """Returns (rank [L,E], owner [L,E], M [L,V,E], S [L], slot_src [L, V*E, 2]), int32 device tensors."""
    dev = distance.device
    i32 = dict(dtype=torch.int32, device=dev)
    V, L, E = shape.V, shape.L, shape.E
    rank, owner = torch.empty((L, E), **i32), torch.empty((L, E), **i32)
    M, S, src = torch.empty((L, V, E), **i32), torch.empty(L, **i32), torch.empty((L, V * E, 2), **i32)
    _check(lib().mmoe_build_expert_map(ctypes.byref(shape), _ptr(distance, torch.float64, L * E, "distance"),
                                       _ptr(rank), _ptr(owner), _ptr(M), _ptr(S), _ptr(src), _stream()),
           "mmoe_build_expert_map")
    return rank, owner, M, S, src


def assemble_pool(shape: LoaderShape, mats, slot_src, layer: int, n_slots: int):
    """The plain pool of one layer, copied from the variants as ``slot_src`` says: list of n_mats device
    tensors [n_slots, mat_elems[m]]."""
    dt = _TORCH_DT[shape.dtype]
    n = shape.V * shape.n_mats
    ptrs = (ctypes.c_void_p * n)()
    for v in range(shape.V):
        for m in range(shape.n_mats):
            ptrs[v * shape.n_mats + m] = _ptr(mats[v][m], dt, shape.L * shape.E * shape.mat_elems[m], f"mats[{v}][{m}]")
    pool = [torch.empty((n_slots, shape.mat_elems[m]), dtype=dt, device=mats[0][0].device) for m in range(shape.n_mats)]
    pp = (ctypes.c_void_p * shape.n_mats)(*[p.data_ptr() for p in pool])
    _check(lib().mmoe_assemble_pool(ctypes.byref(shape), ptrs,
                                    _ptr(slot_src, torch.int32, shape.L * shape.V * shape.E * 2, "slot_src"),
                                    int(layer), int(n_slots), pp, _stream()), "mmoe_assemble_pool")
    return pool


def layer_forward_paged(shape: Shape, X, vid, Wr, br, M, W1p, W3p, W2p, resident, host_pool, ws, copy_stream,
                        Y=None):
    """The layer with part of the pool in pinned host memory (the paper's miss path).
    ``resident``: sequence of S flags; ``host_pool``: (hW1p, hW3p, hW2p), each a list of S pinned CPU
    tensors (one packed slot each) or None for resident slots; ``copy_stream``: a torch.cuda.Stream.
    Returns (Y, fetched flags as a list)."""
    dt = _TORCH_DT[shape.dtype]
    S, d, f = shape.S, shape.d_model, shape.d_ff
    if Y is None:
        Y = torch.empty((shape.T, d), dtype=dt, device=X.device)
    res = (ctypes.c_uint8 * S)(*[1 if r else 0 for r in resident])
    fetched = (ctypes.c_uint8 * S)()

    def host_ptrs(lst):
        if lst is None:
            return None
        arr = (ctypes.c_void_p * S)()
        for s in range(S):
            t = lst[s]
            if t is not None:
                if t.is_cuda or not t.is_pinned() or not t.is_contiguous() or t.dtype != dt or t.numel() != d * f:
                    raise ValueError(f"host slot {s}: needs a pinned, contiguous CPU tensor of {d * f} {dt} elements")
                arr[s] = t.data_ptr()
        return arr

    h1, h3, h2 = (host_ptrs(l) for l in host_pool)
    rc = lib().mmoe_layer_forward_paged(ctypes.byref(shape), _ptr(X, dt, shape.T * d, "X"),
                                        _ptr(vid, torch.int32, shape.T, "vid"), _ptr(Wr, dt, shape.V * shape.E * d, "Wr"),
                                        _ptr(br, torch.float32, shape.V * shape.E, "br"),
                                        _ptr(M, torch.int32, shape.V * shape.E, "M"), _ptr(W1p, dt, S * d * f, "W1p"),
                                        _ptr(W3p, dt, S * d * f, "W3p"), _ptr(W2p, dt, S * d * f, "W2p"), res, h1, h3, h2,
                                        _ptr(Y, dt, shape.T * d, "Y"), _ptr(ws, torch.uint8, None, "ws"), ws.numel(),
                                        _stream(), copy_stream.cuda_stream, fetched)
    if rc < 0:
        raise MmoeError(rc, "mmoe_layer_forward_paged")
    return Y, [int(x) for x in fetched]
