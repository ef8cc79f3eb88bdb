"""Property tests of the oracle over drawn shapes (CPU only): the invariants of the benchmark contract and of the
paper's definitions that hold for any input -- count sums, the bijection of kept rows, stable order inside an expert,
capacity semantics, probability mass, and the linearity of the backward in the upstream gradient."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 300), st.integers(1, 4), st.integers(1, 9), st.integers(-1, 40), st.integers(0, 2 ** 31 - 1))
def test_dispatch_invariants(Ns, k, E, cap, seed):
    k = min(k, E)
    rng = np.random.default_rng(seed)
    # k distinct experts per slice, skewed popularity
    w = rng.exponential(1.0, E)
    idx = np.stack([rng.choice(E, size=k, replace=False, p=w / w.sum()) for _ in range(Ns)]).astype(np.int32)
    d = oracle.dispatch(idx, E, cap)
    flat = idx.reshape(-1)
    np.testing.assert_array_equal(d["counts_raw"], np.bincount(flat, minlength=E))
    assert d["counts_raw"].sum() == Ns * k                                     # every assignment counted once
    want = d["counts_raw"] if cap < 0 else np.minimum(d["counts_raw"], cap)
    np.testing.assert_array_equal(d["counts"], want)
    np.testing.assert_array_equal(d["offsets"], np.concatenate([[0], np.cumsum(want)]))
    kept = int(d["offsets"][-1])
    perm, inv = d["perm"][:kept], d["inv"]
    assert np.all(perm >= 0) and len(set(perm.tolist())) == kept                # kept rows are distinct assignments
    np.testing.assert_array_equal(inv[perm], np.arange(kept))                   # and inv undoes perm
    assert np.count_nonzero(inv >= 0) == kept and np.all(inv[inv < 0] == -1)
    e_of_row = flat[perm]
    assert np.all(np.diff(e_of_row) >= 0)                                       # rows grouped by expert
    same = np.diff(e_of_row) == 0
    assert np.all(np.diff(perm)[same] > 0)                                      # ascending slice order inside an expert
    for e in range(E):                                                          # the dropped are exactly the latest ones
        a_e = np.nonzero(flat == e)[0]
        np.testing.assert_array_equal(inv[a_e] >= 0, np.arange(a_e.size) < want[e])


@settings(max_examples=40, deadline=None)
@given(st.integers(1, 40), st.integers(1, 6), st.integers(1, 7), st.integers(1, 9), st.floats(0.3, 3.0),
       st.floats(0.0, 1.0), st.floats(0.0, 0.9), st.integers(0, 2 ** 31 - 1))
def test_route_train_invariants(Ns, ds, Hr, E, tau, sigma, rate, seed):
    rng = np.random.default_rng(seed)
    k = int(rng.integers(1, E + 1))
    w = (rng.normal(0, 0.5, (ds, Hr)), rng.normal(0, 0.5, Hr), rng.normal(0, 0.5, (Hr, E)), rng.normal(0, 0.5, E))
    x = rng.normal(0, 1, (Ns, ds))
    noise = rng.normal(0, 1, (Ns, E))
    u = rng.uniform(0, 1, (Ns, k)).astype(np.float32)
    r = oracle.route_train(x, *w, k, tau=tau, sigma=sigma, noise=noise, rate=rate, drop_u=u, want_logits=True)
    assert all(len(set(row)) == k for row in r["idx"].tolist())
    g32 = r["logits"].astype(np.float32)
    sel = np.take_along_axis(g32, r["idx"].astype(np.int64), axis=1)
    assert np.all(np.diff(sel, axis=1) <= 0)                                    # slots in descending logit order
    chosen = np.zeros((Ns, E), dtype=bool)
    np.put_along_axis(chosen, r["idx"].astype(np.int64), True, axis=1)
    rest = np.where(chosen, -np.inf, g32)
    assert np.all(sel[:, -1] >= rest.max(axis=1))                               # nothing unselected beats the k-th
    assert np.all(r["pk"] >= 0)
    if rate > 0:
        np.testing.assert_allclose(r["pk"].sum(axis=1), 1.0, rtol=1e-12)        # renormalised to one
        dropped = np.float32(u) < np.float32(rate)
        alld = dropped.all(axis=1)
        assert np.all((r["pk"] == 0)[~alld] == dropped[~alld])                  # exactly the drawn ones are zero
        assert np.all(r["pk"][alld, 0] == 1.0)                                  # all drawn: the first survives
    else:
        assert np.all(r["pk"].sum(axis=1) <= 1.0 + 1e-12)                       # a part of the full softmax mass
        if k == E:
            np.testing.assert_allclose(r["pk"].sum(axis=1), 1.0, rtol=1e-12)
