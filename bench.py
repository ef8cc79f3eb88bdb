#!/usr/bin/env python3
"""Benchmark of the SliceMoE layer forward pass on one MI355X.

A step is one slicemoe_forward over the headline workload (16384 tokens, d=1024, S=16,
E=32, k=2, bf16 storage, fp32 accumulation; seeded synthetic inputs already resident in HBM,
weights pre-packed once outside the timed region as at model load).  Prints ONE JSON line:
whole-layer tokens/s, the per-stage breakdown, the roofline of the dominant kernel (the
grouped expert FFN, matrix-core bound) and the CPU oracle timed on this machine's host cores.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload headline|lm|skewed|large|paper [--slices S] [--topk k]]
                  [--train-router TAU,SIGMA,RATE[,ALPHA]] [--no-overlap]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "SliceMoE layer fwd tokens/sec (bf16) + % of MFMA / HBM roofline per stage"
PEAK_MFMA_BF16_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0           # MI355X HBM3E
# HBM bytes per launch of the expert FFN kernel from rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, each scaled by what
# the same counter reads for a copy kernel of known size): read from the committed summary of that run, so the figure
# printed here is the profile's own; a workload without a summary reports null.
FFN_TRAFFIC_PROFILE = {
    "headline": "profiles/headline_forward_backward_hbm_traffic.md",
    "large": "profiles/large_forward_backward_hbm_traffic.md",
}


def ffn_traffic_bytes(workload):
    """(bytes per launch, summary it comes from) or (None, None)."""
    import re
    rel = FFN_TRAFFIC_PROFILE.get(workload)
    if rel is None:
        return None, None
    try:
        with open(os.path.join(ROOT, rel)) as f:
            m = re.search(r"^Expert FFN[^:\n]*: (\d+) bytes per launch", f.read(), re.M)
    except OSError:
        return None, None
    return (int(m.group(1)), rel) if m else (None, None)


NEAR_TIE = 1e-6   # routing differences below this logit gap (fp32) are near-ties: counted, not errors


def n_kept_rows(B, cfg, ws):
    return int(B.workspace_views(cfg, ws)["offsets"][-1].item())


def parity_record(oracle, B, cfg, shape, bufs, step, ref, hc, w, Tc, train):
    """One more forward on the first buffer set, outside every timed region, compared with the oracle output that the
    CPU-baseline leg just produced (the first Tc tokens): output error over RMS(h'), routing differences split into
    near-ties (slot by slot, the expert the GPU picked has an oracle fp32 logit within NEAR_TIE of the oracle's pick)
    and others, and whether the dispatch tables equal the oracle's bit for bit (only meaningful when the oracle ran
    the whole batch and the routing is identical)."""
    import numpy as np
    import torch
    step(0)
    torch.cuda.synchronize()
    hh, oo, ws = bufs
    v = {n: t.cpu().numpy() for n, t in B.workspace_views(cfg, ws).items() if n != "y"}
    Nsc = Tc * shape.S
    g_idx = v["topk_idx"][:Nsc]
    rows = np.nonzero(np.any(g_idx != ref["idx"], axis=1))[0]
    near = 0
    if rows.size:
        if "logits" in ref:
            lg = ref["logits"][rows]
        else:
            x = hc.reshape(-1, shape.ds)[rows]
            lg = oracle.route(x, w["Wr1"], w["br1"], w["Wr2"], w["br2"], shape.k, want_logits=True)["logits"]
        g32 = lg.astype(np.float32).astype(np.float64)
        got = np.take_along_axis(g32, g_idx[rows].astype(np.int64), axis=1)
        want = np.take_along_axis(g32, ref["idx"][rows].astype(np.int64), axis=1)
        near = int(np.count_nonzero(np.all(want - got < NEAR_TIE, axis=1)))
    out = oo[:Tc].float().cpu().numpy().astype(np.float64)
    mask = np.ones(Nsc, dtype=bool)
    mask[rows] = False
    whole = Tc == shape.T
    if whole and rows.size:   # under a capacity limit a flipped assignment can change which later slices are dropped
        mask &= ~np.any((v["inv"].reshape(-1, shape.k) >= 0) != (ref["inv"].reshape(-1, shape.k) >= 0), axis=1)
    scale = float(np.sqrt(np.mean(ref["h_out"] ** 2)))
    err = float(np.abs(out - ref["h_out"]).reshape(Nsc, shape.ds)[mask].max() / scale)
    exact = None
    if whole and rows.size == 0:
        kept = int(ref["offsets"][-1])
        exact = bool(all(np.array_equal(v[n], ref[n]) for n in ("counts_raw", "counts", "offsets", "inv"))
                     and np.array_equal(v["perm"][:kept], ref["perm"][:kept]))
    return {"tokens_compared": Tc, "max_abs_err_over_rms": round(err, 6), "bar": 2e-2 if shape.dtype == "bf16" else 1e-4,
            "near_tie_mismatches": near, "non_tie_mismatches": int(rows.size) - near, "masked_slices": int(Nsc - mask.sum()),
            "dispatch_bit_exact": exact}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="headline", choices=["lm", "headline", "skewed", "large", "paper"])
    ap.add_argument("--slices", type=int, default=8, help="S of the paper workload (its Table 2 sweep)")
    ap.add_argument("--topk", type=int, default=2, help="k of the paper workload (its Table 4 sweep)")
    ap.add_argument("--train-router", default=None, metavar="TAU,SIGMA,RATE[,ALPHA]",
                    help="run the layer with the training-time router: softmax temperature, logit-noise std, "
                         "cross-slice dropout rate (e.g. 1.0,0.1,0.2); the draws are seeded inputs resident in HBM. "
                         "ALPHA: weight of the capacity loss's gradient in --backward (default 0: none)")
    ap.add_argument("--backward", action="store_true",
                    help="also time slicemoe_backward after the forward (reported under \"backward\"; the metric stays the forward)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true",
                    help="skip the extra measurement with independent batches on several streams and keep the backward "
                         "on one stream (for kernel traces: kernels that run concurrently stretch each other's durations)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch

    from paper_2510_04286_amd import binding as B
    from paper_2510_04286_amd import workload as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    B.lib()
    shape = wl.CONFIGS[args.workload]
    if args.workload == "paper":
        shape = wl.paper_shape(args.slices, args.topk)
    w = wl.make_weights(shape)
    if shape.zipf_s > 0:
        vals = [float(l.split("#")[0]) for l in open(os.path.join(ROOT, "tests", "golden", "zipf_bias_skewed.txt"))
                if l.split("#")[0].strip()]
        w["br2"] = np.array(vals, dtype=np.float32)
    h = wl.make_h(shape)
    # profiling runs keep the backward's kernels on one stream too: concurrent kernels stretch each other's durations
    cfg = B.config_of(shape, flags=B.SLICEMOE_FLAG_SINGLE_STREAM if args.no_overlap else 0)
    # every benchmark workload runs on the matrix-core kernels; of the paper's slice-count sweep, S = 4 and 8 do
    assert args.workload == "paper" or B.slicemoe_uses_mfma(cfg) == 1
    dev = "cuda:0"
    wd = B.pack(cfg, B.weights_to_device(w, shape.dtype, dev), dev)
    torch.cuda.synchronize()

    # Rotate over enough independent input / workspace / output sets that consecutive steps do not
    # find their data in the 256 MB last-level cache: total footprint > 512 MiB.
    ws_bytes = B.slicemoe_workspace_bytes(cfg)
    per_set = ws_bytes + 2 * shape.T * shape.d * 2
    nsets = max(2, min(8, -(-(640 << 20) // per_set)))
    h_dev = B.to_device(h, shape.dtype, dev)
    sets = []
    for _ in range(nsets):
        sets.append((h_dev.clone(), torch.empty((shape.T, shape.d), dtype=torch.bfloat16, device=dev),
                     torch.empty(ws_bytes, dtype=torch.uint8, device=dev)))
    del h_dev

    train = None
    if args.train_router:
        tau, sigma, rate, alpha = ([float(v) for v in args.train_router.split(",")] + [0.0])[:4]
        noise_h, drop_h = wl.make_router_draws(shape)
        train = dict(temperature=tau, noise_std=sigma, dropout_rate=rate, capacity_alpha=alpha,
                     noise=torch.from_numpy(noise_h).to(dev), drop_u=torch.from_numpy(drop_h).to(dev))

    def step(i, stream=None, among=nsets):
        hh, oo, ws = sets[i % among]
        if train:
            B.slicemoe_forward_train(cfg, hh, wd, oo, ws, stream=stream, **train)
        else:
            B.slicemoe_forward(cfg, hh, wd, oo, ws, stream=stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = shape.T / (ms_per_step * 1e-3)

    # ---- independent batches in flight together: the same steps issued round-robin on two or three streams of the
    # default priority (every buffer set belongs to one stream, so no two steps in flight share memory).  One step's
    # memory-bound kernels then run under another's matrix-bound ones and the launch gaps are filled.  Reported
    # beside `value`, which stays the one-stream figure: inside a model consecutive layers depend on each other, and
    # only a caller with several micro-batches in flight gets this rate.
    overlapped = None
    if not args.no_overlap:
        nstreams = 3 if nsets >= 3 else 2
        among = nsets - nsets % nstreams
        streams = [torch.cuda.Stream(device=dev) for _ in range(nstreams)]
        for st in streams:
            st.wait_stream(torch.cuda.current_stream())
        ksteps = max(nstreams, min(args.steps, 300))
        for i in range(2 * nstreams):
            step(i, streams[i % nstreams], among)
        torch.cuda.synchronize()
        o0 = time.perf_counter()
        for i in range(ksteps):
            step(i, streams[i % nstreams], among)
        torch.cuda.synchronize()
        o1 = time.perf_counter()
        overlapped = {"streams": nstreams, "steps": ksteps, "ms_per_step": round((o1 - o0) * 1e3 / ksteps, 5),
                      "value": round(shape.T / ((o1 - o0) / ksteps), 1), "unit": "tokens/s",
                      "note": "independent batches issued round-robin on the streams; value above is the one-stream figure"}

    # ---- per-stage durations: the same launches through the stage entry points, with events on
    # the launch stream (torch's current stream) between them
    names = ["route", "dispatch", "expert_ffn", "combine", "load_stats"]
    acc = {n: 0.0 for n in names}
    nprof = max(10, min(args.steps, 50))
    views = [B.workspace_views(cfg, s[2]) for s in sets]
    L = B.slicemoe_get_workspace_layout(cfg)
    all_events = []
    for i in range(nprof):
        hh, oo, ws = sets[i % nsets]
        v = views[i % nsets]
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
        ev[0].record()
        if train:
            B.slicemoe_route_train(cfg, hh, wd, v["topk_idx"], v["topk_p"], **train)
        else:
            B.slicemoe_route(cfg, hh, wd, v["topk_idx"], v["topk_p"])
        ev[1].record()
        B.slicemoe_dispatch(cfg, v["topk_idx"], v["counts_raw"], v["counts"], v["offsets"], v["perm"], v["inv"],
                            ws[L.scratch:L.packed])
        ev[2].record()
        B.slicemoe_expert_ffn(cfg, hh, v["topk_p"], v["offsets"], v["perm"], wd, v["y"])
        ev[3].record()
        B.slicemoe_combine(cfg, v["y"], v["inv"], oo)
        ev[4].record()
        B.slicemoe_load_stats(cfg, v["counts_raw"], v["counts"], v["stats"])
        ev[5].record()
        all_events.append(ev)
    torch.cuda.synchronize()
    for ev in all_events:
        for j, n in enumerate(names):
            acc[n] += ev[j].elapsed_time(ev[j + 1])
    stage_ms = {n: acc[n] / nprof for n in names}

    v0 = views[0]
    n_kept = int(v0["offsets"][-1].item())
    stats = v0["stats"].cpu().numpy().tolist()
    Ns, Na, ds, He, E, Hr = shape.Ns, shape.Na, shape.ds, shape.He, shape.E, shape.Hr
    # algorithmic work per launch (real rows only, single-pass flops, no padding)
    flops = {
        "route": Ns * (2 * ds * Hr + 2 * Hr * E),
        "expert_ffn": n_kept * 4 * ds * He,
    }
    bytes_ = {
        "route": Ns * ds * 2 + Na * 8,
        "dispatch": Na * 4 + n_kept * 4 + Na * 4,
        "expert_ffn": n_kept * (ds * 2 + 8 + ds * 2),  # x row + perm/p + fp16 y row
        "combine": n_kept * ds * 2 + Na * 4 + Ns * ds * 2,
    }
    stages = {}
    for n in names:
        t = stage_ms[n] * 1e-3
        s = {"us": round(stage_ms[n] * 1e3, 2), "slices_per_s": round(Ns / t, 1) if t > 0 else None}
        if n in flops:
            s["tflops"] = round(flops[n] / t / 1e12, 2)
            s["mfma_frac"] = round(flops[n] / t / 1e12 / PEAK_MFMA_BF16_TFLOPS, 4)
        if n in bytes_:
            s["gbs"] = round(bytes_[n] / t / 1e9, 1)
            s["hbm_frac"] = round(bytes_[n] / t / 1e9 / PEAK_HBM_GBS, 4)
        stages[n] = s

    t_ffn = stage_ms["expert_ffn"] * 1e-3
    achieved = flops["expert_ffn"] / t_ffn / 1e12
    resident = (shape.ds, shape.He) in ((64, 64), (64, 128), (64, 256), (96, 384), (48, 192), (24, 96))  # as the library plans
    pipelined = shape.ds == 64 and shape.He in (64, 128, 256)
    kernel = ("ffn_generic_kernel" if not B.slicemoe_uses_mfma(cfg) else "ffn_pipelined_kernel" if pipelined
              else "ffn_resident_kernel" if resident else "ffn_streamed_kernel")
    roofline = {"kernel": kernel, "bound": "mfma", "achieved": round(achieved, 2),
                "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_MFMA_BF16_TFLOPS, 4),
                "traffic": ffn_traffic_bytes(args.workload)[0],
                "traffic_source": ffn_traffic_bytes(args.workload)[1], "launch_us": round(t_ffn * 1e6, 2),
                "flops_per_launch": flops["expert_ffn"], "hbm_bytes_algorithmic": bytes_["expert_ffn"]}

    backward = None
    if args.backward:
        # one forward leaves the routing in sets[0]'s workspace; the backward is timed on it with events on the launch stream
        hh, oo, ws = sets[0]
        step(0)
        grads = B.alloc_weight_grads(cfg)
        bws = torch.empty(B.slicemoe_backward_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
        d_out = B.to_device(wl.make_dout(shape), shape.dtype, dev)
        d_h = torch.empty_like(hh)
        nb = max(3, min(args.steps, 10))
        evs = []
        for i in range(2 + nb):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            B.slicemoe_backward(cfg, hh, wd, ws, d_out, d_h, grads, bws, train=train)
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        bms = sum(a.elapsed_time(b) for a, b in evs[2:]) / nb
        # five contractions of 2 ds He flop per kept row (recomputed x W1, dy W2^T, dz W1^T, and the two weight
        # gradients) plus the router's three passes forward-size each way
        bflops = 10 * ds * He * n_kept_rows(B, cfg, ws) + 6 * Ns * (ds * Hr + Hr * E)
        backward = {"ms": round(bms, 4), "calls": nb, "flops": bflops, "tflops": round(bflops / (bms * 1e-3) / 1e12, 2),
                    "expert_kernels": "matrix-core" if B.slicemoe_backward_uses_mfma(cfg) == 1 else "vector-ALU fp32",
                    "router_kernels": "matrix-core" if B.slicemoe_backward_uses_mfma(cfg) == 1 and shape.Hr == 256 and shape.E <= 64 else "vector-ALU fp32"}

    cpu = parity = None
    if not args.no_cpu_baseline:
        import oracle
        if shape.Na * shape.ds * shape.He <= 524288 * 64 * 256:
            Tc, sample = shape.T, f"all {shape.T} tokens of the {shape.name} workload, one oracle_forward"
            hc = h
        else:
            Tc = 4096
            sample = f"first {Tc} of {shape.T} tokens of the {shape.name} workload, one oracle_forward"
            hc = h[:Tc]
        cap = -1 if shape.capacity_factor <= 0 else int(np.ceil(float(np.float32(shape.capacity_factor)) * Tc * shape.S * shape.k / shape.E))
        c0 = time.perf_counter()
        if train:
            ref = oracle.forward_train(hc, shape.S, shape.k, w, tau=tau, sigma=sigma, noise=noise_h[:Tc * shape.S], rate=rate,
                                       drop_u=drop_h[:Tc * shape.S], capacity=cap)
        else:
            ref = oracle.forward(hc, shape.S, shape.k, w, capacity=cap)
        c1 = time.perf_counter()
        parity = parity_record(oracle, B, cfg, shape, sets[0], step, ref, hc, w, Tc, train)
        cpu = {"value": round(Tc / (c1 - c0), 1), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": sample, "seconds": round(c1 - c0, 2)}

    line = {
        "metric": METRIC, "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{shape.name}: T={shape.T} d={shape.d} S={shape.S} E={shape.E} k={shape.k} "
                               f"Hr={shape.Hr} He={shape.He} capacity_factor={shape.capacity_factor}",
                   "router": f"training-time: temperature {tau}, noise std {sigma}, dropout {rate}" if train else "inference",
                   "rotating_sets": nsets, "prepacked_weights": True, "kept_rows": n_kept},
        "slices_per_s": round(Ns / (ms_per_step * 1e-3), 1),
        "stages": stages,
        "stage_sum_us": round(sum(stage_ms.values()) * 1e3, 2),
        "stages_note": "each stage through its own entry point; inside slicemoe_forward the router leaves the per-chunk "
                       "histogram behind, so its dispatch is the scatter kernel alone (see profiles/)",
        "load": {"cv2": round(stats[0], 5), "ele": round(stats[1], 5), "drop_fraction": round(stats[2], 5)},
        "overlapped_batches": overlapped,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity": parity,
        **({"backward": backward} if backward else {}),
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
