#!/usr/bin/env python3
"""Writes tests/golden/config{3,4}_samples.npz: oracle outputs of the full-size configurations at sampled rows.

Calls only oracle/ (plus the seeded input generators).  The full chains take minutes on the CPU, so the GPU
tests compare against these stored samples instead of re-running the oracle: every layer's output at a
fixed random set of owned nodes, the H_ij blocks at a fixed random set of edges, and the max-abs of every
full tensor (the scale of the relative error).  The work is spread over processes by destination-node
chunks; each chunk goes through the oracle's own functions unchanged.

    python tests/golden/make_golden.py 3 4
"""
import os
import sys
import time
from concurrent.futures import ProcessPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import egnn_oracle as O                      # noqa: E402
from paper_2507_03840_amd import synth                   # noqa: E402
from tests import gpu_util as U                          # noqa: E402

N_NODE_SAMPLES = 48
N_EDGE_SAMPLES = 256
CHUNK = 96
_state = {}


def _messages_chunk(args):
    j0, j1 = args
    w, g, h, W, agg = _state["w"], _state["g"], _state["h"], _state["W"], _state["agg"]
    src, dst, shift, row_ptr = g
    k0, k1 = int(row_ptr[j0]), int(row_ptr[j1])
    sub = (src[k0:k1], dst[k0:k1], shift[k0:k1], row_ptr[j0:j1 + 1] - k0)
    fn = lambda d, a, b, paths: O.radial_weights(d, W["W_r1"], W["W_r2"], paths, w.channels, w.n_rbf, w.r_cut)
    return j0, O.edge_messages_sum(sub, w.pos, w.box, h, fn, w.lmax, w.lmax, agg)


def _readout_chunk(args):
    k0, k1 = args
    w, g, x, Wr = _state["w"], _state["g"], _state["x"], _state["Wr"]
    return k0, O.readout_hij(g, w.pos, w.box, x, Wr, w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, w.orb_l,
                             k_range=(k0, k1))


def layer_parallel(pool_size, w, g, x, W, agg):
    """Same composition as oracle.layer_forward, the message sum split over destination chunks."""
    h = O.mix_channels(x, W["W_pre"], w.lmax)
    _state.update(w=w, g=g, h=h, W=W, agg=agg)
    jobs = [(j0, min(w.n_owned, j0 + CHUNK)) for j0 in range(0, w.n_owned, CHUNK)]
    a = np.zeros((w.n_owned, (w.lmax + 1) ** 2, w.channels))
    with ProcessPoolExecutor(pool_size) as ex:       # fork: children inherit _state
        for j0, part in ex.map(_messages_chunk, jobs):
            a[j0:j0 + part.shape[0]] = part
    return O.mix_channels(a, W["W_post"], w.lmax) + O.mix_channels(x[:w.n_owned], W["W_self"], w.lmax)


def make(index, pool_size):
    t0 = time.time()
    w = synth.workload(index)
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = U.mean_degree(g, w.n_owned)
    rng = np.random.default_rng([w.seed, 4242])
    nodes = np.sort(rng.choice(w.n_owned, N_NODE_SAMPLES, replace=False))
    out = dict(nodes=nodes, n_edges=len(g[0]), agg=agg)
    x = O.species_embed(wt["x0"], w.species, wt["table"])
    for t in range(w.n_layers):
        y = layer_parallel(pool_size, w, g, x, wt["layers"][t], agg)
        out[f"x{t + 1}_rows"] = y[nodes]
        out[f"x{t + 1}_maxabs"] = np.abs(y).max()
        print(f"config {index}: layer {t} done, max|x| {np.abs(y).max():.4f}, {time.time() - t0:.0f} s", flush=True)
        x = np.concatenate([y, wt["halo"][(t + 1) % w.n_layers].astype(np.float64)], axis=0) \
            if w.n_total > w.n_owned else y
    if w.readout:
        edges = np.sort(rng.choice(len(g[0]), N_EDGE_SAMPLES, replace=False))
        _state.update(w=w, g=g, x=x, Wr=wt["readout"])
        H = np.zeros((N_EDGE_SAMPLES, w.n_orb, w.n_orb))
        with ProcessPoolExecutor(pool_size) as ex:
            for i, (k0, part) in enumerate(ex.map(_readout_chunk, [(int(k), int(k) + 1) for k in edges])):
                H[i] = part[0]
        # scale of the whole tensor: estimated on a larger random sample of edges
        more = np.sort(rng.choice(len(g[0]), 2048, replace=False))
        with ProcessPoolExecutor(pool_size) as ex:
            mx = max(np.abs(p).max() for _, p in ex.map(_readout_chunk, [(int(k), int(k) + 1) for k in more]))
        out.update(edges=edges, H_rows=H, H_maxabs=max(mx, np.abs(H).max()))
        print(f"config {index}: readout done, {time.time() - t0:.0f} s", flush=True)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"config{index}_samples.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, f"{os.path.getsize(path) / 1e3:.0f} kB", flush=True)


if __name__ == "__main__":
    which = [int(a) for a in sys.argv[1:]] or [3, 4]
    for idx in which:
        make(idx, int(os.environ.get("GOLDEN_PROCS", "6")))
