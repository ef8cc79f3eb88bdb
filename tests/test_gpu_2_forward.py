"""End-to-end GPU parity of slicemoe_forward against the fp64 CPU oracle on the five benchmark
workloads (seeded synthetic stand-ins for the paper's language-modelling / translation shapes).

Bars: dispatch integers bit-exact given equal routing; routing equal except near-ties (logit
gap < 1e-6 in fp32), which are counted, reported and masked out of the output comparison;
max |h' - h'_oracle| <= 1e-4 RMS(h') for fp32 storage and <= 2e-2 RMS(h') for bf16 storage.
"""
import numpy as np
import pytest

import oracle
from paper_2510_04286_amd import workload as wl
from tests.common import TOL_BF16, TOL_F32, large_inputs, make_inputs, progress, rms, routing_agreement

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need an MI355X"
    from paper_2510_04286_amd import binding
    binding.lib()
    return binding


def gpu_forward(B, shape, h, w, flags=0, prepack=True, f64=True):
    import torch
    cfg = B.config_of(shape, flags=flags)
    wd = B.weights_to_device(w, shape.dtype)
    if prepack:
        wd = B.pack(cfg, wd)
    ws = B.alloc_workspace(cfg)
    tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
    out = torch.full((shape.T, shape.d), 3.0, dtype=tdt, device="cuda:0")
    B.slicemoe_forward(cfg, B.to_device(h, shape.dtype), wd, out, ws)
    torch.cuda.synchronize()
    views = {n: v.cpu().numpy() for n, v in B.workspace_views(cfg, ws).items() if n != "y"}
    got = out.float().cpu().numpy()
    return (got.astype(np.float64) if f64 else got), views


def check_against_full_oracle(B, shape, h, w, flags=0, prepack=True):
    x = h.reshape(-1, shape.ds)
    ref = oracle.forward(h, shape.S, shape.k, w, capacity=shape.capacity())
    logits = oracle.route(x, w["Wr1"], w["br1"], w["Wr2"], w["br2"], shape.k, want_logits=True)["logits"]
    got, ws = gpu_forward(B, shape, h, w, flags, prepack)
    mism, n_tie = routing_agreement(ws["topk_idx"], ref["idx"], logits)
    tol = TOL_F32 if shape.dtype == "f32" else TOL_BF16
    scale = rms(ref["h_out"])
    diff = np.abs(got - ref["h_out"]).reshape(-1, shape.ds)
    if n_tie == 0:
        # identical routing: the integer side must be bit-exact
        for name in ("counts_raw", "counts", "offsets", "inv"):
            np.testing.assert_array_equal(ws[name], ref[name], err_msg=name)
        kept = int(ref["offsets"][-1])
        np.testing.assert_array_equal(ws["perm"][:kept], ref["perm"][:kept])
        bad = np.zeros(shape.Ns, bool)
    else:
        # a near-tie flips one assignment; under a capacity limit that can shift which later
        # slices of the two experts involved are dropped, so mask every slice whose keep mask differs
        bad = mism | np.any((ws["inv"].reshape(-1, shape.k) >= 0) != (ref["inv"].reshape(-1, shape.k) >= 0), axis=1)
        assert ws["counts_raw"].sum() == shape.Na
    err = diff[~bad].max() / scale
    st = oracle.load_stats(ref["counts_raw"])
    drop = 1 - ref["counts"].sum() / shape.Na
    print(f"\n[forward {shape.name}] slices={shape.Ns} near-tie mismatches={n_tie} masked={int(bad.sum())} "
          f"max|err|/rms={err:.3e} (bar {tol:g}) CV={st['cv_pop']:.3f} ELE={st['ele']:.3f} drop={drop:.3f}")
    assert err <= tol, f"max|err|/rms {err:.3e} over the bar {tol:g}"
    assert bad.sum() <= max(8, 1e-4 * shape.Ns), f"{int(bad.sum())} slices masked ({n_tie} near-tie mismatches)"
    if n_tie == 0:
        assert ws["stats"][0] == pytest.approx(st["cv_pop"] ** 2, rel=1e-4)
        assert ws["stats"][1] == pytest.approx(st["ele"], rel=1e-4)
        assert ws["stats"][2] == pytest.approx(drop, rel=1e-4, abs=1e-7)
    return err


def test_forward_tiny_fp32(B):
    shape, h, w = make_inputs(wl.CONFIGS["tiny"])
    check_against_full_oracle(B, shape, h, w)


def test_forward_lm_bf16(B):
    shape, h, w = make_inputs(wl.CONFIGS["lm"])
    check_against_full_oracle(B, shape, h, w)


@pytest.mark.parametrize("seed", [0, 11])   # the workload's own inputs, and a second draw of weights and hidden states
def test_forward_headline_bf16(B, seed):
    shape, h, w = make_inputs(wl.CONFIGS["headline"], seed=seed)
    check_against_full_oracle(B, shape, h, w)


@pytest.mark.parametrize("seed", [0, 11])
def test_forward_skewed_bf16_with_capacity_drop(B, seed):
    shape, h, w = make_inputs(wl.CONFIGS["skewed"], seed=seed)
    assert shape.capacity() == 20480
    check_against_full_oracle(B, shape, h, w)


def check_sampled_slices_and_dispatch_properties(B, shape, n_sample):
    """Full-size run of a dropless workload; the oracle evaluates a seeded sample of slices one by one (a slice's
    output depends on nothing but its own routing), and the dispatch tables are checked through properties that hold
    at any size."""
    assert shape.capacity() < 0
    if shape.name == "large":
        _, h, w = large_inputs()
    else:
        w = wl.make_weights(shape)
        h = wl.make_h(shape)
    got, ws = gpu_forward(B, shape, h, w)
    x = h.reshape(-1, shape.ds)
    sample = np.unique((wl.uniform01(77, 0, 0, n_sample) * shape.Ns).astype(np.int64))
    r = oracle.route(x[sample], w["Wr1"], w["br1"], w["Wr2"], w["br2"], shape.k, want_logits=True)
    ref = oracle.slices(x[sample], r["idx"], r["pk"], None, w["W1"], w["b1"], w["W2"], w["b2"])
    mism, n_tie = routing_agreement(ws["topk_idx"][sample], r["idx"], r["logits"])
    # RMS over the sampled outputs stands for RMS(h')
    err = np.abs(got.reshape(-1, shape.ds)[sample] - ref)[~mism].max() / rms(ref)
    print(f"\n[forward {shape.name}] sampled slices={sample.size} near-tie mismatches={n_tie} max|err|/rms={err:.3e}")
    assert err <= TOL_BF16
    assert n_tie <= 4
    # dispatch properties at full size
    idx, inv, perm, off = ws["topk_idx"], ws["inv"], ws["perm"], ws["offsets"]
    assert idx.min() >= 0 and idx.max() < shape.E
    srt = np.sort(idx, axis=1)
    assert np.all(srt[:, 1:] != srt[:, :-1])                           # k distinct experts per slice
    counts = np.bincount(idx.reshape(-1), minlength=shape.E)
    np.testing.assert_array_equal(ws["counts_raw"], counts)
    np.testing.assert_array_equal(ws["counts"], counts)
    np.testing.assert_array_equal(off, np.concatenate([[0], np.cumsum(counts)]))
    assert off[-1] == shape.Na
    np.testing.assert_array_equal(inv[perm], np.arange(shape.Na))       # bijection
    e_of_row = idx.reshape(-1)[perm]
    assert np.all(np.diff(e_of_row) >= 0)                              # grouped by expert
    assert np.all(np.diff(perm)[np.diff(e_of_row) == 0] > 0)           # stable inside an expert


def test_forward_large_bf16_sampled(B):
    check_sampled_slices_and_dispatch_properties(B, wl.CONFIGS["large"], 8192)


def test_forward_large_bf16_every_slice(B):
    """The Large workload compared in full: every one of its 2 097 152 slices goes through the oracle, in chunks of
    tokens (dropless, so a slice's routing and output depend on that slice alone: Section 3.1, Eq. 1), and the
    dispatch tables, which need the whole routing table at once, come from one oracle.dispatch call over all of it."""
    shape, h, w = large_inputs()
    assert shape.capacity() < 0
    got, ws = gpu_forward(B, shape, h, w, f64=False)
    S, k, ds, E = shape.S, shape.k, shape.ds, shape.E
    chunk = 4096
    idx_ref = np.empty((shape.Ns, k), dtype=np.int32)
    mism_all = np.zeros(shape.Ns, dtype=bool)
    n_tie, worst, sumsq = 0, 0.0, 0.0
    for t0 in range(0, shape.T, chunk):
        t1 = min(shape.T, t0 + chunk)
        n0, n1 = t0 * S, t1 * S
        x = h[t0:t1].reshape(-1, ds)
        r = oracle.route(x, w["Wr1"], w["br1"], w["Wr2"], w["br2"], k, want_logits=True)
        ref = oracle.slices(x, r["idx"], r["pk"], None, w["W1"], w["b1"], w["W2"], w["b2"])
        mism, nt = routing_agreement(ws["topk_idx"][n0:n1], r["idx"], r["logits"])
        diff = np.abs(got[t0:t1].reshape(-1, ds) - ref)
        diff[mism] = 0.0
        worst = max(worst, float(diff.max()))
        sumsq += float(np.square(ref).sum())
        idx_ref[n0:n1] = r["idx"]
        mism_all[n0:n1] = mism
        n_tie += nt
        progress(f"forward large: tokens {t1}/{shape.T} checked")
    err = worst / np.sqrt(sumsq / (shape.T * shape.d))
    print(f"\n[forward large, every slice] slices={shape.Ns} near-tie mismatches={n_tie} max|err|/rms={err:.3e} (bar {TOL_BF16:g})")
    assert err <= TOL_BF16, err
    assert n_tie <= 8, n_tie
    # the integer side, bit for bit: against the oracle's dispatch of its own routing when the routing is identical;
    # a near-tie resolved the other way moves one assignment between two experts, so then against the oracle's dispatch
    # of the routing the GPU took (every other slice of which equals the oracle's)
    np.testing.assert_array_equal(ws["topk_idx"][~mism_all], idx_ref[~mism_all])
    ref_d = oracle.dispatch(idx_ref if n_tie == 0 else ws["topk_idx"], E, -1)
    for name in ("counts_raw", "counts", "offsets", "perm", "inv"):
        np.testing.assert_array_equal(ws[name], ref_d[name], err_msg=name)
    assert int(ref_d["offsets"][-1]) == shape.Na


@pytest.mark.parametrize("S,k,n_sample", [(2, 2, 1024), (4, 2, 2048), (8, 2, 4096), (16, 2, 4096), (32, 2, 8192), (8, 1, 4096),
                                          (8, 3, 4096)])
def test_forward_paper_shapes_at_measured_size_sampled(B, S, k, n_sample):
    """The paper's own layer at the token count the measurements use (16 384), every slice count and top-k of its
    ablations, in the launch configuration that is timed."""
    check_sampled_slices_and_dispatch_properties(B, wl.paper_shape(S, k), n_sample)


def test_forward_without_prepacked_weights_and_generic_kernels_agree(B):
    """Packing on the fly gives the same bits as pre-packed weights; the generic kernels on the
    same bf16 inputs agree with the matrix-core path to the bf16 bar."""
    shape, h, w = make_inputs(wl.CONFIGS["lm"], 512)
    a, wsa = gpu_forward(B, shape, h, w, prepack=True)
    b, wsb = gpu_forward(B, shape, h, w, prepack=False)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(wsa["topk_idx"], wsb["topk_idx"])
    check_against_full_oracle(B, shape, h, w, flags=B.SLICEMOE_FLAG_FORCE_GENERIC)


def test_forward_ragged_token_counts(B):
    """Token counts that leave partial wavefront tiles, partial row tiles and partial dispatch chunks."""
    for T in (1, 3, 37, 129):
        shape, h, w = make_inputs(wl.CONFIGS["headline"], T)
        check_against_full_oracle(B, shape, h, w)
    shape, h, w = make_inputs(wl.CONFIGS["tiny"], 7)
    check_against_full_oracle(B, shape, h, w)


def test_forward_paper_native_shape(B):
    """d = 768, S = 8 (slice width 96), E = 16, k = 2 -- the shape of the paper's Appendix A, on the matrix-core
    kernels (six K-steps, three output tiles) and on the generic ones."""
    shape = wl.CONFIGS["paper"].scaled(256)
    w = wl.make_weights(shape)
    h = wl.make_h(shape)
    assert B.slicemoe_uses_mfma(B.config_of(shape)) == 1
    check_against_full_oracle(B, shape, h, w)
    check_against_full_oracle(B, shape, h, w, flags=B.SLICEMOE_FLAG_FORCE_GENERIC)
    # slice widths the matrix-core kernels do not take (here 40) stay on the generic kernels
    shape40 = wl.SliceMoEShape("d640_S16", T=96, d=640, S=16, E=16, k=2, He=160)
    assert B.slicemoe_uses_mfma(B.config_of(shape40)) == 0
    check_against_full_oracle(B, shape40, wl.make_h(shape40), wl.make_weights(shape40))


@pytest.mark.parametrize("S,k,T,mfma", [(2, 2, 700, 1), (4, 2, 320, 1), (16, 2, 96, 1), (32, 2, 67, 1), (8, 1, 200, 1), (8, 3, 200, 1),
                                        (4, 3, 130, 1), (16, 3, 257, 1), (32, 1, 129, 1), (2, 3, 33, 1)])
def test_forward_paper_slice_count_and_topk_sweeps(B, S, k, T, mfma):
    """The paper's ablation shapes: d = 768 cut into S in {2, 4, 8, 16, 32} slices (Table 2) and k in {1, 2, 3}
    experts per slice (Table 4), 16 experts of hidden width 4 d/S.  All of these slice widths, 24 to 384, run on the
    matrix-core kernels (24 and 48 zero-padded to whole K-steps and output tiles)."""
    shape = wl.paper_shape(S, k, T)
    assert B.slicemoe_uses_mfma(B.config_of(shape)) == mfma
    check_against_full_oracle(B, shape, wl.make_h(shape), wl.make_weights(shape))


@pytest.mark.parametrize("d,S,E,He,T", [(384, 8, 8, 256, 300), (96, 4, 40, 160, 500), (768, 8, 16, 160, 200), (256, 4, 8, 96, 333)])
def test_forward_streamed_expert_kernel_on_other_hidden_widths(B, d, S, E, He, T):
    """Hidden widths without a resident instantiation (any multiple of 32, odd tile counts included) take the
    streamed expert kernel at every slice width, padded ones too; E = 40 uses two expert tiles in the router."""
    shape = wl.SliceMoEShape(f"d{d}_S{S}_He{He}", T=T, d=d, S=S, E=E, k=2, He=He)
    assert B.slicemoe_uses_mfma(B.config_of(shape)) == 1
    check_against_full_oracle(B, shape, wl.make_h(shape), wl.make_weights(shape))


def test_forward_other_k(B):
    for k in (1, 3):
        shape = wl.SliceMoEShape(f"k{k}", T=300, d=512, S=8, E=16, k=k, He=256)
        check_against_full_oracle(B, shape, wl.make_h(shape), wl.make_weights(shape))


def test_forward_is_deterministic(B):
    shape, h, w = make_inputs(wl.CONFIGS["skewed"], 2048)
    a, wa = gpu_forward(B, shape, h, w)
    b, wb = gpu_forward(B, shape, h, w)
    np.testing.assert_array_equal(a, b)
    for name in ("topk_idx", "perm", "inv", "counts"):
        np.testing.assert_array_equal(wa[name], wb[name])


def test_forward_and_backward_captured_in_a_hip_graph_replay_identically(B):
    """The entry points only launch kernels on the caller's stream (no allocation, no memset, no host wait), so after one
    eager call (which sets the kernels' LDS attributes) a caller may capture them in a HIP graph.  Every replay is checked
    against the eager result for the inputs then in the captured buffers, with the program's own eager work and
    synchronisations between the replays."""
    import torch
    shape, h, w = make_inputs(wl.CONFIGS["headline"], 1024)
    cfg = B.config_of(shape)
    wd = B.pack(cfg, B.weights_to_device(w, shape.dtype))
    hs = [B.to_device(wl.make_h(shape, seed=s), shape.dtype) for s in (1, 5, 9, 13)]
    douts = [B.to_device(wl.make_dout(shape, seed=3 + i), shape.dtype) for i in range(4)]

    def eager(hd, dd):
        ws = B.alloc_workspace(cfg)
        out = torch.empty_like(hd)
        d_h = torch.empty_like(hd)
        grads = B.alloc_weight_grads(cfg)
        bws = torch.empty(B.slicemoe_backward_workspace_bytes(cfg), dtype=torch.uint8, device="cuda:0")
        B.slicemoe_forward(cfg, hd, wd, out, ws)
        B.slicemoe_backward(cfg, hd, wd, ws, dd, d_h, grads, bws)
        torch.cuda.synchronize()
        return out.float().cpu().numpy(), d_h.float().cpu().numpy(), {n: t.cpu().numpy() for n, t in grads.items()}

    refs = [eager(hd, dd) for hd, dd in zip(hs, douts)]   # (also the warm-up calls)

    h_in, d_in = torch.empty_like(hs[0]), torch.empty_like(douts[0])
    out, d_h = torch.empty_like(h_in), torch.empty_like(h_in)
    ws = B.alloc_workspace(cfg)
    grads = B.alloc_weight_grads(cfg)
    bws = torch.empty(B.slicemoe_backward_workspace_bytes(cfg), dtype=torch.uint8, device="cuda:0")
    h_in.copy_(hs[0])
    d_in.copy_(douts[0])
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.slicemoe_forward(cfg, h_in, wd, out, ws)
        B.slicemoe_backward(cfg, h_in, wd, ws, d_in, d_h, grads, bws)
    for i in (1, 2, 3, 0, 2):
        h_in.copy_(hs[i])
        d_in.copy_(douts[i])
        out.fill_(3.0)
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out.float().cpu().numpy(), refs[i][0], err_msg=f"h' of replay with input {i}")
        np.testing.assert_array_equal(d_h.float().cpu().numpy(), refs[i][1], err_msg=f"dL/dh of replay with input {i}")
        for n, t in grads.items():
            np.testing.assert_array_equal(t.cpu().numpy(), refs[i][2][n], err_msg=f"{n} of replay with input {i}")
        _ = eager(hs[(i + 1) % 4], douts[i])   # eager work between the replays
