"""fp64 CPU oracle of the SliceMoE layer forward pass -- TEST INFRASTRUCTURE ONLY.

Thin ctypes binding over ``slicemoe_oracle.c`` (plain C, fp64, per-slice definition of
paper Section 3 / Section 3.1 / Eq. 1).  Only ``tests/``, the smoke check and the
benchmark's CPU-baseline leg may import this package.  It shares no code with the HIP
path and never imports it.

All array arguments are numpy arrays on the host; floating-point inputs are widened to
fp64 here, so callers pass the storage-rounded fp32 values the GPU path also receives.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slicemoe_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

ACT_GELU = 0
ACT_IDENTITY = 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP) if the library is missing or stale."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_gelu.restype = ctypes.c_double
        _lib.oracle_gelu.argtypes = [ctypes.c_double]
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed (rc={rc})")


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def gelu(z: float) -> float:
    return float(lib().oracle_gelu(float(z)))


def route(x, Wr1, br1, Wr2, br2, k: int, want_logits: bool = False):
    """x[Ns, ds] -> dict(idx[Ns,k] int32, pk[Ns,k] f64, margin[Ns] f64[, logits[Ns,E]])."""
    x = _f64(x)
    Ns, ds = x.shape
    Wr1, br1, Wr2, br2 = _f64(Wr1), _f64(br1), _f64(Wr2), _f64(br2)
    Hr, E = Wr2.shape
    assert Wr1.shape == (ds, Hr) and br1.shape == (Hr,) and br2.shape == (E,)
    idx = np.empty((Ns, k), dtype=np.int32)
    pk = np.empty((Ns, k), dtype=np.float64)
    margin = np.empty((Ns,), dtype=np.float64)
    logits = np.empty((Ns, E), dtype=np.float64) if want_logits else None
    rc = lib().oracle_route(_p(x), ctypes.c_int64(Ns), ds, Hr, E, k, _p(Wr1), _p(br1), _p(Wr2), _p(br2),
                            _p(idx), _p(pk), _p(logits), _p(margin))
    _check(rc, "oracle_route")
    out = {"idx": idx, "pk": pk, "margin": margin}
    if want_logits:
        out["logits"] = logits
    return out


def route_train(x, Wr1, br1, Wr2, br2, k: int, tau: float = 1.0, sigma: float = 0.0, noise=None,
                rate: float = 0.0, drop_u=None, want_logits: bool = False):
    """Training-time router (temperature: Appendix B; logit noise: Section 5; cross-slice dropout: Section 3.3).
    noise[Ns, E] standard-normal draws and drop_u[Ns, k] uniform draws are inputs.  Output as route()."""
    x = _f64(x)
    Ns, ds = x.shape
    Wr1, br1, Wr2, br2 = _f64(Wr1), _f64(br1), _f64(Wr2), _f64(br2)
    Hr, E = Wr2.shape
    assert Wr1.shape == (ds, Hr) and br1.shape == (Hr,) and br2.shape == (E,)
    noise = None if noise is None else _f64(noise)
    drop_u = None if drop_u is None else _f64(drop_u)
    assert noise is None or noise.shape == (Ns, E)
    assert drop_u is None or drop_u.shape == (Ns, k)
    idx = np.empty((Ns, k), dtype=np.int32)
    pk = np.empty((Ns, k), dtype=np.float64)
    margin = np.empty((Ns,), dtype=np.float64)
    logits = np.empty((Ns, E), dtype=np.float64) if want_logits else None
    rc = lib().oracle_route_train(_p(x), ctypes.c_int64(Ns), ds, Hr, E, k, _p(Wr1), _p(br1), _p(Wr2), _p(br2),
                                  ctypes.c_double(tau), ctypes.c_double(sigma), _p(noise), ctypes.c_double(rate),
                                  _p(drop_u), _p(idx), _p(pk), _p(logits), _p(margin))
    _check(rc, "oracle_route_train")
    out = {"idx": idx, "pk": pk, "margin": margin}
    if want_logits:
        out["logits"] = logits
    return out


def dispatch(idx, E: int, capacity: int = -1):
    """idx[Ns,k] -> dict(counts_raw[E], counts[E], offsets[E+1], perm[Ns*k], inv[Ns*k])."""
    idx = _i32(idx)
    Ns, k = idx.shape
    counts_raw = np.empty(E, dtype=np.int32)
    counts = np.empty(E, dtype=np.int32)
    offsets = np.empty(E + 1, dtype=np.int32)
    perm = np.empty(Ns * k, dtype=np.int32)
    inv = np.empty(Ns * k, dtype=np.int32)
    rc = lib().oracle_dispatch(_p(idx), ctypes.c_int64(Ns), k, E, ctypes.c_int64(capacity),
                               _p(counts_raw), _p(counts), _p(offsets), _p(perm), _p(inv))
    _check(rc, "oracle_dispatch")
    return {"counts_raw": counts_raw, "counts": counts, "offsets": offsets, "perm": perm, "inv": inv}


def expert_rows(x, idx, pk, perm, n_rows: int, W1, b1, W2, b2, act: int = ACT_GELU):
    """y[n_rows, ds]: row r = phi_e(pk[a] * x[a // k]) with a = perm[r], e = idx[a]."""
    x = _f64(x)
    Ns, ds = x.shape
    idx, perm, pk = _i32(idx), _i32(perm), _f64(pk)
    k = idx.shape[1]
    W1, b1, W2, b2 = _f64(W1), _f64(b1), _f64(W2), _f64(b2)
    E, ds_, He = W1.shape
    assert ds_ == ds and W2.shape == (E, He, ds) and b1.shape == (E, He) and b2.shape == (E, ds)
    y = np.empty((n_rows, ds), dtype=np.float64)
    rc = lib().oracle_expert_rows(_p(x), ds, He, k, _p(idx), _p(pk), _p(perm), ctypes.c_int64(n_rows),
                                  _p(W1), _p(b1), _p(W2), _p(b2), act, _p(y))
    _check(rc, "oracle_expert_rows")
    return y


def combine(y, inv, Ns: int, k: int):
    """out[Ns, ds] = sum of the kept rows of each slice."""
    y = _f64(y)
    ds = y.shape[1]
    inv = _i32(inv)
    out = np.empty((Ns, ds), dtype=np.float64)
    rc = lib().oracle_combine(_p(y), _p(inv), ctypes.c_int64(Ns), k, ds, _p(out))
    _check(rc, "oracle_combine")
    return out


def slices(x, idx, pk, inv, W1, b1, W2, b2, act: int = ACT_GELU):
    """Per-slice definition: out[n] = sum_j kept phi_{idx[n,j]}(pk[n,j] * x[n]).  inv may be None."""
    x = _f64(x)
    Ns, ds = x.shape
    idx, pk = _i32(idx), _f64(pk)
    k = idx.shape[1]
    inv = None if inv is None else _i32(inv)
    W1, b1, W2, b2 = _f64(W1), _f64(b1), _f64(W2), _f64(b2)
    E, ds_, He = W1.shape
    assert ds_ == ds and W2.shape == (E, He, ds)
    out = np.empty((Ns, ds), dtype=np.float64)
    rc = lib().oracle_slices(_p(x), ctypes.c_int64(Ns), ds, He, k, _p(idx), _p(pk), _p(inv),
                             _p(W1), _p(b1), _p(W2), _p(b2), act, _p(out))
    _check(rc, "oracle_slices")
    return out


def forward(h, S: int, k: int, weights: dict, capacity: int = -1, act: int = ACT_GELU):
    """Whole layer.  h[T, d] -> dict(h_out[T,d], idx, pk, margin, counts_raw, counts, offsets, perm, inv)."""
    h = _f64(h)
    T, d = h.shape
    w = {n: _f64(weights[n]) for n in ("Wr1", "br1", "Wr2", "br2", "W1", "b1", "W2", "b2")}
    Hr, E = w["Wr2"].shape
    _, ds, He = w["W1"].shape
    assert ds * S == d
    Ns = T * S
    out = {
        "h_out": np.empty((T, d), dtype=np.float64),
        "idx": np.empty((Ns, k), dtype=np.int32),
        "pk": np.empty((Ns, k), dtype=np.float64),
        "margin": np.empty((Ns,), dtype=np.float64),
        "counts_raw": np.empty(E, dtype=np.int32),
        "counts": np.empty(E, dtype=np.int32),
        "offsets": np.empty(E + 1, dtype=np.int32),
        "perm": np.empty(Ns * k, dtype=np.int32),
        "inv": np.empty(Ns * k, dtype=np.int32),
    }
    rc = lib().oracle_forward(_p(h), ctypes.c_int64(T), d, S, Hr, E, k, He, ctypes.c_int64(capacity),
                              _p(w["Wr1"]), _p(w["br1"]), _p(w["Wr2"]), _p(w["br2"]),
                              _p(w["W1"]), _p(w["b1"]), _p(w["W2"]), _p(w["b2"]), act,
                              _p(out["h_out"]), _p(out["idx"]), _p(out["pk"]), _p(out["margin"]),
                              _p(out["counts_raw"]), _p(out["counts"]), _p(out["offsets"]),
                              _p(out["perm"]), _p(out["inv"]))
    _check(rc, "oracle_forward")
    return out


def forward_train(h, S: int, k: int, weights: dict, tau: float = 1.0, sigma: float = 0.0, noise=None,
                  rate: float = 0.0, drop_u=None, capacity: int = -1):
    """Whole layer with the training-time router: route_train, then dispatch, experts and combine as in forward()."""
    h = _f64(h)
    T, d = h.shape
    x = h.reshape(T * S, d // S)
    r = route_train(x, weights["Wr1"], weights["br1"], weights["Wr2"], weights["br2"], k, tau, sigma, noise, rate,
                    drop_u, want_logits=True)
    E = np.asarray(weights["Wr2"]).shape[1]
    dsp = dispatch(r["idx"], E, capacity)
    out = slices(x, r["idx"], r["pk"], dsp["inv"], weights["W1"], weights["b1"], weights["W2"], weights["b2"])
    res = {"h_out": out.reshape(T, d), "idx": r["idx"], "pk": r["pk"], "margin": r["margin"], "logits": r["logits"]}
    res.update(dsp)
    return res


def capacity_surrogate(idx, pk, E: int, alpha: float):
    """The differentiable reading of the capacity loss (Section 3.2, Eq. 2): counts replaced by the sums of the final
    probabilities routed to each expert, c_e = sum over assignments a with idx[a] == e of pk[a].
    Returns dict(sums[E], value = alpha * CV^2(c) with the population variance, grad[E] = d value / d c_e)."""
    idx = _i32(idx).reshape(-1)
    pk = _f64(pk).reshape(-1)
    assert idx.shape == pk.shape
    c = np.zeros(E, dtype=np.float64)
    for e in range(E):
        c[e] = pk[idx == e].sum()
    total, squares = c.sum(), np.square(c).sum()
    value = alpha * (E * squares / total ** 2 - 1.0)           # var / mean^2 = E sum c^2 / (sum c)^2 - 1
    grad = alpha * (2.0 * E / total ** 2) * (c - squares / total)
    return {"sums": c, "value": float(value), "grad": grad}


def backward(h, S: int, k: int, weights: dict, d_out, idx, inv, tau: float = 1.0, sigma: float = 0.0, noise=None,
             rate: float = 0.0, drop_u=None, capg=None):
    """Gradients of a loss with dL/dh' = d_out[T, d], given the forward pass's idx[Ns,k] and inv[Ns*k].
    capg[E] (optional): d L_cap / d c_e of capacity_surrogate(), added to dL/dp of every assignment of expert e.
    Returns dict(d_h[T,d], Wr1, br1, Wr2, br2, W1, b1, W2, b2) in the logical layouts, fp64."""
    h = _f64(h)
    T, d = h.shape
    ds = d // S
    Ns = T * S
    w = {n: _f64(weights[n]) for n in ("Wr1", "br1", "Wr2", "br2", "W1", "b1", "W2", "b2")}
    Hr, E = w["Wr2"].shape
    He = w["W1"].shape[2]
    G = _f64(d_out)
    assert G.shape == (T, d)
    idx, inv = _i32(idx), _i32(inv)
    assert idx.shape == (Ns, k) and inv.shape == (Ns * k,)
    noise = None if noise is None else _f64(noise)
    drop_u = None if drop_u is None else _f64(drop_u)
    capg = None if capg is None else _f64(capg)
    assert capg is None or capg.shape == (E,)
    out = {"d_h": np.empty((T, d), dtype=np.float64)}
    for n in ("Wr1", "br1", "Wr2", "br2", "W1", "b1", "W2", "b2"):
        out[n] = np.empty_like(w[n])
    rc = lib().oracle_backward(_p(h), ctypes.c_int64(Ns), ds, Hr, E, k, He,
                               _p(w["Wr1"]), _p(w["br1"]), _p(w["Wr2"]), _p(w["br2"]),
                               _p(w["W1"]), _p(w["b1"]), _p(w["W2"]), _p(w["b2"]),
                               ctypes.c_double(tau), ctypes.c_double(sigma), _p(noise), ctypes.c_double(rate),
                               _p(drop_u), _p(idx), _p(inv), _p(G), _p(capg), _p(out["d_h"]),
                               _p(out["Wr1"]), _p(out["br1"]), _p(out["Wr2"]), _p(out["br2"]),
                               _p(out["W1"]), _p(out["b1"]), _p(out["W2"]), _p(out["b2"]))
    _check(rc, "oracle_backward")
    return out


def load_stats(counts):
    """dict(cv_pop, cv_sample, ele) of per-expert counts (Eq. 2 statistic; ELE of Section 4)."""
    counts = _i32(counts)
    a, b, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    rc = lib().oracle_load_stats(_p(counts), int(counts.shape[0]), ctypes.byref(a), ctypes.byref(b),
                                 ctypes.byref(c))
    _check(rc, "oracle_load_stats")
    return {"cv_pop": a.value, "cv_sample": b.value, "ele": c.value}
