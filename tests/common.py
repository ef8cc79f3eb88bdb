"""Helpers shared by the tests: golden inputs, tolerance rules, GPU plumbing."""
import functools
import os

import numpy as np

from paper_2510_04286_amd import workload as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

# Output tolerances of the layer: max |h'_gpu - h'_oracle| <= TOL * RMS(h'_oracle).
TOL_F32 = 1e-4
TOL_BF16 = 2e-2
# A routing difference counts as a near-tie when the logits involved differ by less than this
# (fp32 logits; the selection is taken in fp32 on both sides).
NEAR_TIE = 1e-6


def zipf_bias():
    """Second router bias of the skewed-load workload (written by golden/make_zipf_bias.py)."""
    vals = [float(line.split("#")[0]) for line in open(os.path.join(GOLDEN, "zipf_bias_skewed.txt"))
            if line.split("#")[0].strip()]
    b = np.array(vals, dtype=np.float32)
    wl.bf16_bits(b)  # must be representable
    return b


def make_inputs(cfg, T=None, seed=0):
    """(cfg', h, weights) of a workload, optionally with fewer tokens; seed: weights from `seed`, hidden states from
    `seed + 1` (0 gives the workload's own inputs, the ones bench.py runs)."""
    if T is not None and T != cfg.T:
        cfg = cfg.scaled(T)
    w = wl.make_weights(cfg, seed=seed)
    if cfg.zipf_s > 0:
        assert cfg.E == 32 and cfg.zipf_s == 1.2
        w["br2"] = zipf_bias()
    return cfg, wl.make_h(cfg, seed=seed + 1), w


@functools.lru_cache(maxsize=1)
def large_inputs():
    """(shape, h, weights) of the Large workload; generating its 268M hidden-state values takes a while, so the
    full-size tests share one copy."""
    shape = wl.CONFIGS["large"]
    return shape, wl.make_h(shape), wl.make_weights(shape)


@functools.lru_cache(maxsize=1)
def large_dout():
    return wl.make_dout(wl.CONFIGS["large"])


def progress(msg):
    """A line for a long test to leave behind while it runs (output is captured until the test ends): appended to the
    file that the environment variable SLICEMOE_PROGRESS_LOG names, if it is set."""
    path = os.environ.get("SLICEMOE_PROGRESS_LOG")
    if path:
        with open(path, "a") as f:
            f.write(msg + "\n")


def rms(a):
    return float(np.sqrt(np.mean(np.square(np.asarray(a, dtype=np.float64)))))


def routing_agreement(gpu_idx, oracle_idx, oracle_logits):
    """Compare routing tables.  Returns (mismatch mask [Ns], number of near-tie mismatches).

    A slice whose indices differ is accepted only as a near-tie: in every slot j the expert the
    GPU picked has an oracle fp32 logit within NEAR_TIE of the j-th largest one, and the picks
    are distinct.  Anything else raises.
    """
    gpu_idx = np.asarray(gpu_idx)
    mism = np.any(gpu_idx != oracle_idx, axis=1)
    rows = np.nonzero(mism)[0]
    if rows.size:
        g32 = oracle_logits[rows].astype(np.float32).astype(np.float64)
        got = np.take_along_axis(g32, gpu_idx[rows].astype(np.int64), axis=1)
        want = np.take_along_axis(g32, oracle_idx[rows].astype(np.int64), axis=1)
        bad = np.any(want - got >= NEAR_TIE, axis=1)
        distinct = np.array([len(set(r)) == len(r) for r in gpu_idx[rows]])
        assert not np.any(bad) and np.all(distinct), (
            f"{int(np.count_nonzero(bad | ~distinct))} routing mismatches are not near-ties; first slice "
            f"{rows[np.nonzero(bad | ~distinct)[0][0]]}")
    return mism, int(rows.size)
