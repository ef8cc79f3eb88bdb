"""ctypes binding of libslicemoe.so: the same entry points as include/slicemoe.h.

Argument marshalling only.  PyTorch supplies device memory (tensors) and streams; every step
of the layer runs in the HIP kernels of the library.  There is no fallback: if the library is
not built, or no GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libslicemoe.so")

SLICEMOE_OK = 0
SLICEMOE_ERR_INVALID_ARG = 1
SLICEMOE_ERR_UNSUPPORTED = 2
SLICEMOE_ERR_WORKSPACE = 3
SLICEMOE_ERR_HIP = 4
SLICEMOE_F32 = 0
SLICEMOE_BF16 = 1
SLICEMOE_FLAG_FORCE_GENERIC = 1
SLICEMOE_FLAG_REQUIRE_MFMA = 2
SLICEMOE_FLAG_SINGLE_STREAM = 4

EXPORTS = [
    "slicemoe_status_string", "slicemoe_uses_mfma", "slicemoe_capacity", "slicemoe_workspace_bytes",
    "slicemoe_dispatch_workspace_bytes", "slicemoe_get_workspace_layout", "slicemoe_packed_bytes",
    "slicemoe_pack_weights", "slicemoe_route", "slicemoe_dispatch", "slicemoe_expert_ffn",
    "slicemoe_combine", "slicemoe_load_stats", "slicemoe_forward",
    "slicemoe_route_train", "slicemoe_forward_train", "slicemoe_backward_workspace_bytes", "slicemoe_backward",
    "slicemoe_backward_uses_mfma", "slicemoe_dispatch_noalloc",
]


class SliceMoEError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status}")


class slicemoe_config(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d", ctypes.c_int32), ("S", ctypes.c_int32), ("k", ctypes.c_int32),
                ("E", ctypes.c_int32), ("Hr", ctypes.c_int32), ("He", ctypes.c_int32),
                ("capacity_factor", ctypes.c_float), ("dtype", ctypes.c_int32), ("flags", ctypes.c_uint32)]


class slicemoe_weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("Wr1", "br1", "Wr2", "br2", "W1", "b1", "W2", "b2", "packed")]


class slicemoe_route_train_params(ctypes.Structure):
    _fields_ = [("temperature", ctypes.c_float), ("noise_std", ctypes.c_float), ("dropout_rate", ctypes.c_float),
                ("capacity_alpha", ctypes.c_float)]


class slicemoe_weight_grads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("Wr1", "br1", "Wr2", "br2", "W1", "b1", "W2", "b2")]


class slicemoe_workspace_layout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in ("topk_idx", "topk_p", "counts_raw", "counts", "offsets", "perm",
                                               "inv", "y", "stats", "scratch", "packed", "total")]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libslicemoe.so (built in-tree by paper_2510_04286_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2510_04286_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        cfgp, wp, vp, st = ctypes.POINTER(slicemoe_config), ctypes.POINTER(slicemoe_weights), ctypes.c_void_p, ctypes.c_size_t
        L.slicemoe_status_string.restype = ctypes.c_char_p
        L.slicemoe_status_string.argtypes = [ctypes.c_int]
        L.slicemoe_uses_mfma.restype = ctypes.c_int
        L.slicemoe_uses_mfma.argtypes = [cfgp]
        L.slicemoe_capacity.restype = ctypes.c_int64
        L.slicemoe_capacity.argtypes = [cfgp]
        for f in (L.slicemoe_workspace_bytes, L.slicemoe_dispatch_workspace_bytes, L.slicemoe_packed_bytes):
            f.restype = st
            f.argtypes = [cfgp]
        L.slicemoe_get_workspace_layout.restype = ctypes.c_int
        L.slicemoe_get_workspace_layout.argtypes = [cfgp, ctypes.POINTER(slicemoe_workspace_layout)]
        L.slicemoe_pack_weights.restype = ctypes.c_int
        L.slicemoe_pack_weights.argtypes = [cfgp, wp, vp, st, vp]
        L.slicemoe_route.restype = ctypes.c_int
        L.slicemoe_route.argtypes = [cfgp, vp, wp, vp, vp, vp, st, vp]
        L.slicemoe_dispatch.restype = ctypes.c_int
        L.slicemoe_dispatch.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, st, vp]
        L.slicemoe_expert_ffn.restype = ctypes.c_int
        L.slicemoe_expert_ffn.argtypes = [cfgp, vp, vp, vp, vp, wp, vp, vp, st, vp]
        L.slicemoe_combine.restype = ctypes.c_int
        L.slicemoe_combine.argtypes = [cfgp, vp, vp, vp, vp]
        L.slicemoe_load_stats.restype = ctypes.c_int
        L.slicemoe_load_stats.argtypes = [cfgp, vp, vp, vp, vp]
        L.slicemoe_forward.restype = ctypes.c_int
        L.slicemoe_forward.argtypes = [cfgp, vp, wp, vp, vp, st, vp]
        tpp = ctypes.POINTER(slicemoe_route_train_params)
        L.slicemoe_route_train.restype = ctypes.c_int
        L.slicemoe_route_train.argtypes = [cfgp, vp, wp, tpp, vp, vp, vp, vp, vp, st, vp]
        L.slicemoe_forward_train.restype = ctypes.c_int
        L.slicemoe_forward_train.argtypes = [cfgp, vp, wp, tpp, vp, vp, vp, vp, st, vp]
        L.slicemoe_dispatch_noalloc.restype = ctypes.c_int
        L.slicemoe_dispatch_noalloc.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp]
        L.slicemoe_backward_uses_mfma.restype = ctypes.c_int
        L.slicemoe_backward_uses_mfma.argtypes = [cfgp]
        L.slicemoe_backward_workspace_bytes.restype = ctypes.c_size_t
        L.slicemoe_backward_workspace_bytes.argtypes = [cfgp]
        L.slicemoe_backward.restype = ctypes.c_int
        L.slicemoe_backward.argtypes = [cfgp, vp, wp, tpp, vp, vp, vp, st, vp, vp, ctypes.POINTER(slicemoe_weight_grads),
                                        vp, st, vp]
        _lib = L
    return _lib


def make_config(T, d, S, k, E, He, dtype="bf16", capacity_factor=0.0, Hr=256, flags=0) -> slicemoe_config:
    return slicemoe_config(T, d, S, k, E, Hr, He, float(capacity_factor),
                           SLICEMOE_BF16 if dtype in ("bf16", SLICEMOE_BF16) else SLICEMOE_F32, flags)


def config_of(shape, flags=0) -> slicemoe_config:
    """slicemoe_config of a workload.SliceMoEShape."""
    return make_config(shape.T, shape.d, shape.S, shape.k, shape.E, shape.He, shape.dtype,
                       shape.capacity_factor, shape.Hr, flags)


def _ptr(t, dtype=None, numel=None, name="tensor"):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA/HIP tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name} has {t.numel()} elements, needs {numel}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _tdtype(cfg):
    return torch.bfloat16 if cfg.dtype == SLICEMOE_BF16 else torch.float32


def y_dtype(cfg):
    """Element type of the stacked expert outputs y: fp16 with bf16 storage, fp32 with fp32 storage."""
    return torch.float16 if cfg.dtype == SLICEMOE_BF16 else torch.float32


def _weights(cfg, w) -> slicemoe_weights:
    """dict of device tensors (logical layout, optional 'packed' uint8 buffer) -> C struct."""
    dt = _tdtype(cfg)
    ds = cfg.d // cfg.S
    sizes = {"Wr1": ds * cfg.Hr, "br1": cfg.Hr, "Wr2": cfg.Hr * cfg.E, "br2": cfg.E,
             "W1": cfg.E * ds * cfg.He, "b1": cfg.E * cfg.He, "W2": cfg.E * cfg.He * ds, "b2": cfg.E * ds}
    out = slicemoe_weights()
    for n, sz in sizes.items():
        t = w.get(n)
        setattr(out, n, None if t is None else _ptr(t, dt, sz, n).value)
    pk = w.get("packed")
    out.packed = None if pk is None else _ptr(pk, torch.uint8, lib().slicemoe_packed_bytes(ctypes.byref(cfg)), "packed").value
    return out


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _ptr(workspace, torch.uint8, None, "workspace"), workspace.numel()


def _check(status, what):
    if status != SLICEMOE_OK:
        raise SliceMoEError(status, f"{what}: {lib().slicemoe_status_string(status).decode()}")


# ------------------------------------------------------------------ queries
def slicemoe_status_string(status: int) -> str:
    return lib().slicemoe_status_string(status).decode()


def slicemoe_uses_mfma(cfg) -> int:
    return lib().slicemoe_uses_mfma(ctypes.byref(cfg))


def slicemoe_capacity(cfg) -> int:
    return lib().slicemoe_capacity(ctypes.byref(cfg))


def slicemoe_workspace_bytes(cfg) -> int:
    return lib().slicemoe_workspace_bytes(ctypes.byref(cfg))


def slicemoe_dispatch_workspace_bytes(cfg) -> int:
    return lib().slicemoe_dispatch_workspace_bytes(ctypes.byref(cfg))


def slicemoe_packed_bytes(cfg) -> int:
    return lib().slicemoe_packed_bytes(ctypes.byref(cfg))


def slicemoe_get_workspace_layout(cfg) -> slicemoe_workspace_layout:
    out = slicemoe_workspace_layout()
    _check(lib().slicemoe_get_workspace_layout(ctypes.byref(cfg), ctypes.byref(out)), "slicemoe_get_workspace_layout")
    return out


# ------------------------------------------------------------------ stages
def slicemoe_pack_weights(cfg, w, packed_out, stream=None):
    ws = _weights(cfg, {k: v for k, v in w.items() if k != "packed"})
    _check(lib().slicemoe_pack_weights(ctypes.byref(cfg), ctypes.byref(ws), _ptr(packed_out, torch.uint8, None, "packed_out"),
                                       packed_out.numel(), _stream(stream)), "slicemoe_pack_weights")


def slicemoe_route(cfg, h, w, topk_idx, topk_p, workspace=None, stream=None):
    Ns = cfg.T * cfg.S
    wsp, wsb = _ws(workspace)
    ws = _weights(cfg, w)
    _check(lib().slicemoe_route(ctypes.byref(cfg), _ptr(h, _tdtype(cfg), cfg.T * cfg.d, "h"), ctypes.byref(ws),
                                _ptr(topk_idx, torch.int32, Ns * cfg.k, "topk_idx"),
                                _ptr(topk_p, torch.float32, Ns * cfg.k, "topk_p"), wsp, wsb, _stream(stream)),
           "slicemoe_route")


def slicemoe_dispatch(cfg, topk_idx, counts_raw, counts, offsets, perm, inv, workspace, stream=None):
    Na = cfg.T * cfg.S * cfg.k
    wsp, wsb = _ws(workspace)
    _check(lib().slicemoe_dispatch(ctypes.byref(cfg), _ptr(topk_idx, torch.int32, Na, "topk_idx"),
                                   _ptr(counts_raw, torch.int32, cfg.E, "counts_raw"),
                                   _ptr(counts, torch.int32, cfg.E, "counts"),
                                   _ptr(offsets, torch.int32, cfg.E + 1, "offsets"),
                                   _ptr(perm, torch.int32, Na, "perm"), _ptr(inv, torch.int32, Na, "inv"),
                                   wsp, wsb, _stream(stream)), "slicemoe_dispatch")


def slicemoe_dispatch_noalloc(cfg, topk_idx, counts_raw, counts, offsets, perm, inv, stream=None):
    Na = cfg.T * cfg.S * cfg.k
    _check(lib().slicemoe_dispatch_noalloc(ctypes.byref(cfg), _ptr(topk_idx, torch.int32, Na, "topk_idx"),
                                           _ptr(counts_raw, torch.int32, cfg.E, "counts_raw"),
                                           _ptr(counts, torch.int32, cfg.E, "counts"),
                                           _ptr(offsets, torch.int32, cfg.E + 1, "offsets"),
                                           _ptr(perm, torch.int32, Na, "perm"), _ptr(inv, torch.int32, Na, "inv"),
                                           _stream(stream)), "slicemoe_dispatch_noalloc")


def slicemoe_expert_ffn(cfg, h, topk_p, offsets, perm, w, y, workspace=None, stream=None):
    Na = cfg.T * cfg.S * cfg.k
    wsp, wsb = _ws(workspace)
    ws = _weights(cfg, w)
    _check(lib().slicemoe_expert_ffn(ctypes.byref(cfg), _ptr(h, _tdtype(cfg), cfg.T * cfg.d, "h"),
                                     _ptr(topk_p, torch.float32, Na, "topk_p"),
                                     _ptr(offsets, torch.int32, cfg.E + 1, "offsets"),
                                     _ptr(perm, torch.int32, Na, "perm"), ctypes.byref(ws),
                                     _ptr(y, y_dtype(cfg), Na * (cfg.d // cfg.S), "y"), wsp, wsb, _stream(stream)),
           "slicemoe_expert_ffn")


def slicemoe_combine(cfg, y, inv, h_out, stream=None):
    Na = cfg.T * cfg.S * cfg.k
    _check(lib().slicemoe_combine(ctypes.byref(cfg), _ptr(y, y_dtype(cfg), Na * (cfg.d // cfg.S), "y"),
                                  _ptr(inv, torch.int32, Na, "inv"),
                                  _ptr(h_out, _tdtype(cfg), cfg.T * cfg.d, "h_out"), _stream(stream)),
           "slicemoe_combine")


def slicemoe_load_stats(cfg, counts_raw, counts, stats, stream=None):
    _check(lib().slicemoe_load_stats(ctypes.byref(cfg), _ptr(counts_raw, torch.int32, cfg.E, "counts_raw"),
                                     _ptr(counts, torch.int32, cfg.E, "counts"),
                                     _ptr(stats, torch.float32, 4, "stats"), _stream(stream)), "slicemoe_load_stats")


def slicemoe_forward(cfg, h, w, h_out, workspace, stream=None):
    wsp, wsb = _ws(workspace)
    ws = _weights(cfg, w)
    _check(lib().slicemoe_forward(ctypes.byref(cfg), _ptr(h, _tdtype(cfg), cfg.T * cfg.d, "h"), ctypes.byref(ws),
                                  _ptr(h_out, _tdtype(cfg), cfg.T * cfg.d, "h_out"), wsp, wsb, _stream(stream)),
           "slicemoe_forward")


def _train_args(cfg, temperature, noise_std, dropout_rate, noise, drop_u, capacity_alpha=0.0):
    tp = slicemoe_route_train_params(temperature, noise_std, dropout_rate, capacity_alpha)
    Ns = cfg.T * cfg.S
    npt = None if noise is None else _ptr(noise, torch.float32, Ns * cfg.E, "noise")
    upt = None if drop_u is None else _ptr(drop_u, torch.float32, Ns * cfg.k, "drop_u")
    return tp, npt, upt


def slicemoe_route_train(cfg, h, w, topk_idx, topk_p, temperature=1.0, noise_std=0.0, dropout_rate=0.0, noise=None,
                         drop_u=None, workspace=None, stream=None, capacity_alpha=0.0):
    """capacity_alpha travels in the parameter struct; only slicemoe_backward reads it."""
    Ns = cfg.T * cfg.S
    wsp, wsb = _ws(workspace)
    ws = _weights(cfg, w)
    tp, npt, upt = _train_args(cfg, temperature, noise_std, dropout_rate, noise, drop_u, capacity_alpha)
    _check(lib().slicemoe_route_train(ctypes.byref(cfg), _ptr(h, _tdtype(cfg), cfg.T * cfg.d, "h"), ctypes.byref(ws),
                                      ctypes.byref(tp), npt, upt, _ptr(topk_idx, torch.int32, Ns * cfg.k, "topk_idx"),
                                      _ptr(topk_p, torch.float32, Ns * cfg.k, "topk_p"), wsp, wsb, _stream(stream)),
           "slicemoe_route_train")


def slicemoe_forward_train(cfg, h, w, h_out, workspace, temperature=1.0, noise_std=0.0, dropout_rate=0.0, noise=None,
                           drop_u=None, stream=None, capacity_alpha=0.0):
    """capacity_alpha travels in the parameter struct; only slicemoe_backward reads it."""
    wsp, wsb = _ws(workspace)
    ws = _weights(cfg, w)
    tp, npt, upt = _train_args(cfg, temperature, noise_std, dropout_rate, noise, drop_u, capacity_alpha)
    _check(lib().slicemoe_forward_train(ctypes.byref(cfg), _ptr(h, _tdtype(cfg), cfg.T * cfg.d, "h"), ctypes.byref(ws),
                                        ctypes.byref(tp), npt, upt, _ptr(h_out, _tdtype(cfg), cfg.T * cfg.d, "h_out"),
                                        wsp, wsb, _stream(stream)), "slicemoe_forward_train")


def slicemoe_backward_uses_mfma(cfg) -> int:
    return int(lib().slicemoe_backward_uses_mfma(ctypes.byref(cfg)))


def slicemoe_backward_workspace_bytes(cfg) -> int:
    return int(lib().slicemoe_backward_workspace_bytes(ctypes.byref(cfg)))


def alloc_weight_grads(cfg, device="cuda:0") -> dict:
    """fp32 device tensors in the logical layout of each weight tensor (contents undefined until slicemoe_backward)."""
    ds = cfg.d // cfg.S
    shapes = {"Wr1": (ds, cfg.Hr), "br1": (cfg.Hr,), "Wr2": (cfg.Hr, cfg.E), "br2": (cfg.E,),
              "W1": (cfg.E, ds, cfg.He), "b1": (cfg.E, cfg.He), "W2": (cfg.E, cfg.He, ds), "b2": (cfg.E, ds)}
    return {n: torch.empty(sh, dtype=torch.float32, device=device) for n, sh in shapes.items()}


def slicemoe_backward(cfg, h, w, forward_workspace, d_out, d_h, grads: dict, workspace, train: dict | None = None,
                      stream=None):
    """train: None after slicemoe_forward, else the keyword arguments given to slicemoe_forward_train, and optionally
    capacity_alpha (weight of the capacity loss's gradient; the forward calls do not read it)."""
    fwp, fwb = _ws(forward_workspace)
    wsp, wsb = _ws(workspace)
    ws = _weights(cfg, w)
    tpp, npt, upt = None, None, None
    if train is not None:
        tp, npt, upt = _train_args(cfg, train.get("temperature", 1.0), train.get("noise_std", 0.0),
                                   train.get("dropout_rate", 0.0), train.get("noise"), train.get("drop_u"),
                                   train.get("capacity_alpha", 0.0))
        tpp = ctypes.byref(tp)
    g = slicemoe_weight_grads()
    ds = cfg.d // cfg.S
    sizes = {"Wr1": ds * cfg.Hr, "br1": cfg.Hr, "Wr2": cfg.Hr * cfg.E, "br2": cfg.E, "W1": cfg.E * ds * cfg.He,
             "b1": cfg.E * cfg.He, "W2": cfg.E * cfg.He * ds, "b2": cfg.E * ds}
    for n, numel in sizes.items():
        setattr(g, n, _ptr(grads[n], torch.float32, numel, "grads." + n).value)
    _check(lib().slicemoe_backward(ctypes.byref(cfg), _ptr(h, _tdtype(cfg), cfg.T * cfg.d, "h"), ctypes.byref(ws), tpp,
                                   npt, upt, fwp, fwb, _ptr(d_out, _tdtype(cfg), cfg.T * cfg.d, "d_out"),
                                   _ptr(d_h, _tdtype(cfg), cfg.T * cfg.d, "d_h"), ctypes.byref(g), wsp, wsb,
                                   _stream(stream)), "slicemoe_backward")


# ------------------------------------------------------------------ plumbing helpers (device memory only)
def to_device(arr, dtype: str, device="cuda:0") -> torch.Tensor:
    """Host fp32 array holding storage-representable values -> device tensor of the storage dtype."""
    t = torch.from_numpy(arr).to(device)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def weights_to_device(weights: dict, dtype: str, device="cuda:0") -> dict:
    return {n: to_device(a, dtype, device).contiguous() for n, a in weights.items()}


def alloc_workspace(cfg, device="cuda:0") -> torch.Tensor:
    n = slicemoe_workspace_bytes(cfg)
    if n == 0:
        raise SliceMoEError(SLICEMOE_ERR_UNSUPPORTED, "slicemoe_workspace_bytes returned 0 (invalid or unsupported config)")
    return torch.empty(n, dtype=torch.uint8, device=device)


def pack(cfg, w: dict, device="cuda:0") -> dict:
    """Return a copy of the weight dict with the 'packed' buffer added (no-op on generic configs)."""
    n = slicemoe_packed_bytes(cfg)
    out = dict(w)
    if n > 0:
        buf = torch.empty(n, dtype=torch.uint8, device=device)
        slicemoe_pack_weights(cfg, w, buf)
        out["packed"] = buf
    return out


def workspace_views(cfg, workspace: torch.Tensor) -> dict:
    """Typed views of the intermediates slicemoe_forward left in its workspace."""
    L = slicemoe_get_workspace_layout(cfg)
    Na = cfg.T * cfg.S * cfg.k
    ds = cfg.d // cfg.S

    def view(off, n, dt):
        return workspace[off:off + n * torch.empty(0, dtype=dt).element_size()].view(dt)

    return {
        "topk_idx": view(L.topk_idx, Na, torch.int32).view(-1, cfg.k),
        "topk_p": view(L.topk_p, Na, torch.float32).view(-1, cfg.k),
        "counts_raw": view(L.counts_raw, cfg.E, torch.int32),
        "counts": view(L.counts, cfg.E, torch.int32),
        "offsets": view(L.offsets, cfg.E + 1, torch.int32),
        "perm": view(L.perm, Na, torch.int32),
        "inv": view(L.inv, Na, torch.int32),
        "y": view(L.y, Na * ds, y_dtype(cfg)).view(-1, ds),
        "stats": view(L.stats, 4, torch.float32),
    }
