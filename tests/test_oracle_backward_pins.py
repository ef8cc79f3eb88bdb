"""Pins of the oracle's backward pass against the definition of a derivative: central finite differences of the
oracle's own FORWARD functions (already pinned elsewhere), parameter by parameter, in fp64 on shapes small enough to
perturb every entry.  The loss is a fixed random linear functional of h', so dL/dh' is that functional.  CPU only.
"""
import numpy as np
import pytest

import oracle
from paper_2510_04286_amd import workload as wl

NAMES = ("Wr1", "br1", "Wr2", "br2", "W1", "b1", "W2", "b2")


def small_problem(seed, T=5, d=8, S=2, E=4, k=2, He=6, Hr=7):
    rng = np.random.default_rng(seed)
    ds = d // S
    w = {"Wr1": rng.normal(0, 0.6, (ds, Hr)), "br1": rng.normal(0, 0.3, (Hr,)),
         "Wr2": rng.normal(0, 0.6, (Hr, E)), "br2": rng.normal(0, 0.3, (E,)),
         "W1": rng.normal(0, 0.6, (E, ds, He)), "b1": rng.normal(0, 0.3, (E, He)),
         "W2": rng.normal(0, 0.6, (E, He, ds)), "b2": rng.normal(0, 0.3, (E, ds))}
    h = rng.normal(0, 1, (T, d))
    R = rng.normal(0, 1, (T, d))
    noise = rng.normal(0, 1, (T * S, E))
    drop_u = rng.uniform(0, 1, (T * S, k)).astype(np.float32).astype(np.float64)
    return h, w, R, noise, drop_u, S, k


def loss(h, w, R, S, k, variant, capacity):
    f = oracle.forward_train(h, S, k, w, capacity=capacity, **variant)
    return float(np.sum(f["h_out"] * R)), f


def finite_difference(h, w, R, S, k, variant, capacity, name, eps=1e-6):
    """dL/d(tensor `name`) entry by entry; `name` == "h" perturbs the input."""
    base = h if name == "h" else w[name]
    out = np.zeros_like(base)
    it = np.nditer(base, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        vals = []
        for sgn in (+1, -1):
            pert = base.copy()
            pert[i] += sgn * eps
            hh = pert if name == "h" else h
            ww = w if name == "h" else {**w, name: pert}
            vals.append(loss(hh, ww, R, S, k, variant, capacity)[0])
        out[i] = (vals[0] - vals[1]) / (2 * eps)
    return out


VARIANTS = {
    "inference": dict(),
    "temperature": dict(tau=0.6),
    "noise": dict(sigma=0.4),
    "dropout": dict(rate=0.35),
    "all": dict(tau=1.7, sigma=0.3, rate=0.35),
}


@pytest.mark.parametrize("vname", list(VARIANTS))
@pytest.mark.parametrize("capacity", [-1, 3])
def test_backward_equals_finite_differences(vname, capacity):
    h, w, R, noise, drop_u, S, k = small_problem(seed=11)
    variant = dict(VARIANTS[vname])
    if "sigma" in variant:
        variant["noise"] = noise
    if "rate" in variant:
        variant["drop_u"] = drop_u
    _, f = loss(h, w, R, S, k, variant, capacity)
    # the decisions must be stable under the perturbations: no near-tie in the selection
    assert f["margin"].min() > 1e-3
    if capacity >= 0:
        assert np.any(f["inv"] < 0)           # the capacity did drop something
    if "rate" in variant:
        assert np.any(f["pk"] == 0)            # and so did the dropout
    g = oracle.backward(h, S, k, w, R, f["idx"], f["inv"], **variant)
    for name in NAMES + ("h",):
        fd = finite_difference(h, w, R, S, k, variant, capacity, name)
        got = g["d_h"] if name == "h" else g[name]
        scale = max(1.0, np.abs(fd).max())
        np.testing.assert_allclose(got, fd, rtol=0, atol=2e-7 * scale, err_msg=f"{vname} cap={capacity} {name}")
        assert np.abs(fd).max() > 1e-3, name       # the check is not vacuous


def test_backward_three_experts_per_slice_and_single_slice():
    for kw in (dict(T=4, d=6, S=1, E=5, k=3, He=4, Hr=5), dict(T=3, d=12, S=3, E=3, k=3, He=5, Hr=4)):
        h, w, R, noise, drop_u, S, k = small_problem(seed=5, **kw)
        variant = dict(tau=0.9, sigma=0.2, noise=noise, rate=0.3, drop_u=drop_u)
        _, f = loss(h, w, R, S, k, variant, -1)
        if k < w["Wr2"].shape[1]:
            assert f["margin"].min() > 1e-3
        g = oracle.backward(h, S, k, w, R, f["idx"], f["inv"], **variant)
        for name in NAMES + ("h",):
            fd = finite_difference(h, w, R, S, k, variant, -1, name)
            got = g["d_h"] if name == "h" else g[name]
            np.testing.assert_allclose(got, fd, rtol=0, atol=2e-7 * max(1.0, np.abs(fd).max()), err_msg=name)


def test_backward_closed_forms():
    h, w, R, noise, drop_u, S, k = small_problem(seed=3)
    f = oracle.forward_train(h, S, k, w)
    g = oracle.backward(h, S, k, w, R, f["idx"], f["inv"])
    ds = h.shape[1] // S
    Rn = R.reshape(-1, ds)
    # the output bias of expert e collects dL/dh' of every slice assigned to it
    E = w["Wr2"].shape[1]
    expect = np.zeros((E, ds))
    for n in range(Rn.shape[0]):
        for j in range(k):
            expect[f["idx"][n, j]] += Rn[n]
    np.testing.assert_allclose(g["b2"], expect, rtol=1e-13, atol=1e-15)
    # W2 = 0: nothing upstream of the second layer receives gradient
    w0 = {**w, "W2": np.zeros_like(w["W2"])}
    f0 = oracle.forward_train(h, S, k, w0)
    g0 = oracle.backward(h, S, k, w0, R, f0["idx"], f0["inv"])
    for name in ("Wr1", "br1", "Wr2", "br2", "W1", "b1"):
        assert np.all(g0[name] == 0), name
    assert np.all(g0["d_h"] == 0)
    assert np.any(g0["W2"] != 0)
    # k = E = 1: p = 1 whatever the router says, so the router gets no gradient and the layer is a dense FFN
    h1, w1, R1, _, _, S1, _ = small_problem(seed=4, E=1, k=1)
    f1 = oracle.forward_train(h1, S1, 1, w1)
    g1 = oracle.backward(h1, S1, 1, w1, R1, f1["idx"], f1["inv"])
    for name in ("Wr1", "br1", "Wr2", "br2"):
        np.testing.assert_allclose(g1[name], 0, atol=1e-15)


def test_backward_is_linear_in_the_upstream_gradient():
    h, w, R, noise, drop_u, S, k = small_problem(seed=8)
    f = oracle.forward_train(h, S, k, w, tau=1.3, rate=0.3, drop_u=drop_u)
    kw = dict(tau=1.3, rate=0.3, drop_u=drop_u)
    R2 = np.random.default_rng(9).normal(0, 1, R.shape)
    a = oracle.backward(h, S, k, w, R, f["idx"], f["inv"], **kw)
    b = oracle.backward(h, S, k, w, R2, f["idx"], f["inv"], **kw)
    c = oracle.backward(h, S, k, w, 2.0 * R - 0.5 * R2, f["idx"], f["inv"], **kw)
    for name in NAMES + ("d_h",):
        np.testing.assert_allclose(c[name], 2.0 * a[name] - 0.5 * b[name], rtol=1e-11, atol=1e-13)


# ---- the differentiable reading of the capacity loss (Section 3.2, Eq. 2): gate sums in place of counts

def test_capacity_surrogate_closed_forms():
    rng = np.random.default_rng(21)
    E, alpha = 6, 0.1
    idx = rng.integers(0, E, size=(40, 2)).astype(np.int32)
    # probabilities of one: the sums are the counts, and the value is Eq. 2 on the counts
    ones = oracle.capacity_surrogate(idx, np.ones(idx.shape), E, alpha)
    counts = np.bincount(idx.ravel(), minlength=E)
    np.testing.assert_array_equal(ones["sums"], counts)
    np.testing.assert_allclose(ones["value"], alpha * np.var(counts) / np.mean(counts) ** 2, rtol=1e-13)
    np.testing.assert_allclose(ones["value"], alpha * oracle.load_stats(counts.astype(np.int32))["cv_pop"] ** 2, rtol=1e-12)
    # equal sums: no imbalance, no gradient
    eq = oracle.capacity_surrogate(np.arange(E, dtype=np.int32), np.full(E, 0.37), E, alpha)
    assert abs(eq["value"]) < 1e-15 and np.all(np.abs(eq["grad"]) < 1e-15)
    # the gradient is the derivative of the value with respect to the sums, and CV is scale-free (Euler: c . grad = 0)
    pk = rng.uniform(0.05, 0.95, idx.shape)
    s = oracle.capacity_surrogate(idx, pk, E, alpha)
    np.testing.assert_allclose(np.dot(s["sums"], s["grad"]), 0.0, atol=1e-15)
    for a in range(0, idx.size, 7):
        vals = []
        for sgn in (+1, -1):
            q = pk.copy().ravel()
            q[a] += sgn * 1e-6
            vals.append(oracle.capacity_surrogate(idx, q.reshape(pk.shape), E, alpha)["value"])
        np.testing.assert_allclose((vals[0] - vals[1]) / 2e-6, s["grad"][idx.ravel()[a]], rtol=0, atol=1e-10)
    # an expert above the mean is pushed down, one below is pushed up
    assert np.all(np.sign(s["grad"]) == np.sign(s["sums"] - np.square(s["sums"]).sum() / s["sums"].sum()))


@pytest.mark.parametrize("vname", ["inference", "all"])
@pytest.mark.parametrize("capacity", [-1, 3])
def test_backward_with_capacity_surrogate_equals_finite_differences(vname, capacity):
    """Total loss = linear functional of h' + alpha CV^2 of the gate sums.  The second term sees the router only, but
    through every assignment: also those the capacity limit dropped (they never reach an expert)."""
    alpha = 0.8
    h, w, R, noise, drop_u, S, k = small_problem(seed=11)
    E = w["Wr2"].shape[1]
    variant = dict(VARIANTS[vname])
    if "sigma" in variant:
        variant["noise"] = noise
    if "rate" in variant:
        variant["drop_u"] = drop_u

    def total(hh, ww):
        f = oracle.forward_train(hh, S, k, ww, capacity=capacity, **variant)
        return float(np.sum(f["h_out"] * R)) + oracle.capacity_surrogate(f["idx"], f["pk"], E, alpha)["value"], f

    _, f = total(h, w)
    assert f["margin"].min() > 1e-3
    if capacity >= 0:
        assert np.any(f["inv"] < 0)
    cap = oracle.capacity_surrogate(f["idx"], f["pk"], E, alpha)
    g = oracle.backward(h, S, k, w, R, f["idx"], f["inv"], capg=cap["grad"], **variant)
    g0 = oracle.backward(h, S, k, w, R, f["idx"], f["inv"], **variant)
    for name in NAMES + ("h",):
        base = h if name == "h" else w[name]
        fd = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            vals = []
            for sgn in (+1, -1):
                pert = base.copy()
                pert[i] += sgn * 1e-6
                vals.append(total(pert if name == "h" else h, w if name == "h" else {**w, name: pert})[0])
            fd[i] = (vals[0] - vals[1]) / 2e-6
        got = g["d_h"] if name == "h" else g[name]
        np.testing.assert_allclose(got, fd, rtol=0, atol=2e-7 * max(1.0, np.abs(fd).max()), err_msg=f"{vname} {name}")
    # the term reaches the router and the input, and nothing else
    for name in ("W1", "b1", "W2", "b2"):
        np.testing.assert_allclose(g[name], g0[name], rtol=1e-12, atol=1e-15)
    for name in ("Wr1", "br1", "Wr2", "br2", "d_h"):
        assert np.abs(g[name] - g0[name]).max() > 1e-4, name
