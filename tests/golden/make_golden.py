#!/usr/bin/env python3
"""Writes tests/golden/config{3,4}_samples.npz: oracle outputs of the full-size configurations at sampled rows.

Calls only oracle/ (plus the seeded input generators).  The full chains take minutes on the CPU, so the GPU
tests compare against these stored samples instead of re-running the oracle: every layer's output at a
fixed set of owned nodes (random ones plus the first and last node, the nodes of least and greatest degree and
the owned atoms next to the halo), the H_ij blocks at a fixed set of edges (random ones, the first and the last
64), and the max-abs of every full tensor, of each of its degrees and of each shell block of H (the scales of
the relative errors).  The work is spread over processes by destination-node chunks; each chunk goes through the
oracle's own functions unchanged, and tests/test_golden_writer.py checks on config 1 that the chains composed here
equal the oracle's own composite calls.

    python tests/golden/make_golden.py 3 4 5
    python tests/golden/make_golden.py so2:3 so2:4      (SO(2) message sums at sampled nodes)
    python tests/golden/make_golden.py so2bwd:3         (adjoint of the SO(2) message sum: weight gradients, rows of dx)
    python tests/golden/make_golden.py blocksbwd:3      (adjoints of the node block and of the edge block)
    python tests/golden/make_golden.py w16:3 w16:4      (first layer and readout with half-precision path weights)
    python tests/golden/make_golden.py blocks:3 blocks:4  (node block and edge block with full message content)
"""
import os
import sys
import time
from concurrent.futures import ProcessPoolExecutor

if __name__ == "__main__":
    # one BLAS thread per worker process: the pool already uses every core, and oversubscribed BLAS threads make the
    # many small products of the per-node loops an order of magnitude slower
    for _v in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS"):
        os.environ.setdefault(_v, "1")

import numpy as np                                       # noqa: E402

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import egnn_oracle as O                      # noqa: E402
from paper_2507_03840_amd import synth                   # noqa: E402
from tests import gpu_util as U                          # noqa: E402

N_NODE_SAMPLES = 48
N_EDGE_SAMPLES = 256
CHUNK = 96
_state = {}


def aimed_nodes(w, g, rng, n_rows):
    """Rows to store: a random set plus the rows where an indexing mistake would show first -- the first and the
    last owned node, the owned nodes of least and greatest degree, and (with a halo) the owned atoms closest to
    each face of the owned region along every open axis, i.e. the ones whose sources are mostly halo atoms.
    n_rows = w.n_owned for layer outputs, w.n_total for gradients w.r.t. the input features (then the first and
    last halo rows are added too)."""
    row_ptr = g[3]
    deg = np.diff(row_ptr)
    picks = [rng.choice(n_rows, N_NODE_SAMPLES, replace=False), [0, w.n_owned - 1, int(np.argmin(deg)), int(np.argmax(deg))]]
    if w.n_total > w.n_owned:
        owned = np.asarray(w.pos[:w.n_owned], np.float64)
        for a in range(3):
            if not w.pbc[a]:
                order = np.argsort(owned[:, a], kind="stable")
                picks += [order[:4], order[-4:]]
        if n_rows == w.n_total:
            picks.append([w.n_owned, w.n_total - 1])
    return np.unique(np.concatenate([np.asarray(p, np.int64) for p in picks]))


def aimed_edges(g, rng):
    """Edges to store: a random set, the first edge, and the last 64 edges (the ragged tail of every edge tiling)."""
    n_e = len(g[0])
    return np.unique(np.concatenate([rng.choice(n_e, N_EDGE_SAMPLES, replace=False), [0],
                                     np.arange(max(0, n_e - 64), n_e)]).astype(np.int64))


def maxabs_per_degree(x, lmax):
    """Largest magnitude of every degree l of a node tensor [n][(lmax+1)^2][E]: the scale a degree's error is judged by."""
    return np.array([np.abs(x[:, O.sl(l), :]).max() for l in range(lmax + 1)])


def maxabs_per_shell_block(H, orb_l):
    """Largest magnitude of every (alpha, beta) shell block of H [n][n_orb][n_orb]."""
    off = np.concatenate([[0], np.cumsum([2 * l + 1 for l in orb_l])])
    return np.array([[np.abs(H[:, off[a]:off[a + 1], off[b]:off[b + 1]]).max() for b in range(len(orb_l))]
                     for a in range(len(orb_l))])


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


def _so2_chunk(nodes):
    from oracle import so2_oracle as S
    w, g, x, Wso2, agg = _state["w"], _state["g"], _state["x"], _state["Wso2"], _state["agg"]
    W_e, W0, Wr, Wi = Wso2
    return S.so2_message_sum(g, w.pos, w.box, x, W_e, W0, Wr, Wi, w.lmax, w.channels, w.n_rbf, w.r_cut, agg, nodes=nodes)


def make_so2(index, pool_size):
    """SO(2) message sums of the full-size configuration at sampled destination nodes -> config{index}_so2_samples.npz.
    Inputs: the model's layer-0 features (species embedded) and synth.so2_weights with seed [w.seed, 777]."""
    t0 = time.time()
    w = synth.workload(index)
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = U.mean_degree(g, w.n_owned)
    rng = np.random.default_rng([w.seed, 4243])
    nodes = np.sort(rng.choice(w.n_owned, N_NODE_SAMPLES, replace=False))
    x = O.species_embed(wt["x0"], w.species, wt["table"])
    Wso2 = synth.so2_weights(np.random.default_rng([w.seed, 777]), w.lmax, w.channels, w.n_rbf)
    _state.update(w=w, g=g, x=x, Wso2=Wso2, agg=agg)
    parts = [nodes[i::pool_size] for i in range(pool_size)]
    rows = np.zeros((N_NODE_SAMPLES, (w.lmax + 1) ** 2, w.channels))
    with ProcessPoolExecutor(pool_size) as ex:
        for i, part in enumerate(ex.map(_so2_chunk, parts)):
            rows[i::pool_size] = part
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"config{index}_so2_samples.npz")
    np.savez_compressed(path, nodes=nodes, rows=rows, agg=agg, n_edges=len(g[0]))
    print(f"config {index} so2: wrote {path}, max|a| over samples {np.abs(rows).max():.4f}, {time.time() - t0:.0f} s", flush=True)


def _so2_backward_chunk(k_range):
    """Edges k_range of the adjoint of the SO(2) message sum (it is a sum over the edges)."""
    from oracle import so2_oracle as S
    w, g, x, Wso2, agg, da = _state["w"], _state["g"], _state["x"], _state["Wso2"], _state["agg"], _state["da"]
    W_e, W0, Wr, Wi = Wso2
    k0, k1 = k_range
    sub = (g[0][k0:k1], g[1][k0:k1], g[2][k0:k1], g[3])
    return S.so2_message_sum_backward(sub, w.pos, w.box, x, W_e, W0, Wr, Wi, w.lmax, w.channels, w.n_rbf, w.r_cut, agg, da)


def make_so2_backward(index, pool_size):
    """Adjoint of the SO(2) message sum of the full-size configuration -> config{index}_so2_backward.npz: all weight
    gradients and the rows of dx at aimed nodes.  Inputs as make_so2; da ~ N(0, 1) from seed [w.seed, 778]."""
    t0 = time.time()
    w = synth.workload(index)
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = U.mean_degree(g, w.n_owned)
    x = O.species_embed(wt["x0"], w.species, wt["table"])
    Wso2 = synth.so2_weights(np.random.default_rng([w.seed, 777]), w.lmax, w.channels, w.n_rbf)
    da = U.so2_da(w)
    _state.update(w=w, g=g, x=x, Wso2=Wso2, agg=agg, da=da)
    n_e = len(g[0])
    # (few large ranges: every job returns a full dx, 0.26 GB at config 4)
    step = max(8192, -(-n_e // (2 * pool_size)))
    jobs = [(k0, min(n_e, k0 + step)) for k0 in range(0, n_e, step)]
    total = None
    with ProcessPoolExecutor(pool_size) as ex:
        for part in ex.map(_so2_backward_chunk, jobs):
            flat = [part[0], part[1], part[2]] + list(part[3]) + list(part[4])
            if total is None:
                total = flat
            else:
                for acc, v in zip(total, flat):
                    acc += v
    dx, dW_e, dW0 = total[0], total[1], total[2]
    dWr, dWi = total[3:3 + w.lmax], total[3 + w.lmax:]
    from oracle import so2_oracle as S
    rng = np.random.default_rng([w.seed, 4244])
    nodes = aimed_nodes(w, g, rng, w.n_total)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"config{index}_so2_backward.npz")
    # (weight gradients in fp32 beyond config 3: 1e6 entries, and 6e-8 of rounding is far below the bar they are held to)
    wdt = np.float64 if index <= 3 else np.float32
    out = dict(nodes=nodes, dx_rows=dx[nodes], dx_maxabs=np.abs(dx).max(), dx_maxabs_l=maxabs_per_degree(dx, w.lmax),
               dW_e=dW_e, dW0=dW0.astype(wdt), agg=agg, n_edges=n_e)
    for m in range(w.lmax):
        out[f"dWr{m + 1}"] = dWr[m].astype(wdt)
        out[f"dWi{m + 1}"] = dWi[m].astype(wdt)
    np.savez_compressed(path, **out)
    print(f"config {index} so2 backward: wrote {path}, {os.path.getsize(path) / 1e3:.0f} kB, max|dx| {np.abs(dx).max():.4f}, "
          f"{time.time() - t0:.0f} s", flush=True)


def _blocks_nodes(nodes):
    from oracle import so2_oracle as S
    w, g, x, T, Wn, w_att = (_state[k] for k in ("w", "g", "x", "T", "Wn", "w_att"))
    return S.so2_node_block(g, w.pos, w.box, x, T, Wn[1], Wn[2], Wn[3], w_att, w.lmax, w.channels, w.r_cut, nodes=nodes)


def _blocks_edges(edges):
    from oracle import so2_oracle as S
    w, g, x, T, We = (_state[k] for k in ("w", "g", "x", "T", "We"))
    return np.concatenate([S.so2_edge_block(g, w.pos, w.box, x, T, We[1], We[2], We[3], w.lmax, w.channels, w.r_cut,
                                            k_range=(int(k), int(k) + 1)) for k in edges])


def make_blocks(index, pool_size):
    """Node block at sampled owned nodes and edge block at sampled edges of the full-size configuration, inputs from
    tests/gpu_util.block_inputs -> config{index}_so2_blocks_samples.npz."""
    t0 = time.time()
    w = synth.workload(index)
    g, x, T, Wn, We, w_att = U.block_inputs(w)
    rng = np.random.default_rng([w.seed, 4245])
    nodes = np.sort(rng.choice(w.n_owned, N_NODE_SAMPLES, replace=False))
    edges = np.sort(rng.choice(len(g[0]), N_EDGE_SAMPLES, replace=False))
    _state.update(w=w, g=g, x=x, T=T, Wn=Wn, We=We, w_att=w_att)
    with ProcessPoolExecutor(pool_size) as ex:
        a_parts = list(ex.map(_blocks_nodes, [nodes[i::pool_size] for i in range(pool_size)]))
        t_parts = list(ex.map(_blocks_edges, [edges[i::pool_size] for i in range(pool_size)]))
    a_rows = np.zeros((N_NODE_SAMPLES,) + a_parts[0].shape[1:])
    T_rows = np.zeros((N_EDGE_SAMPLES,) + t_parts[0].shape[1:])
    for i in range(pool_size):
        a_rows[i::pool_size] = a_parts[i]
        T_rows[i::pool_size] = t_parts[i]
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"config{index}_so2_blocks_samples.npz")
    np.savez_compressed(path, nodes=nodes, edges=edges, a_rows=a_rows, T_rows=T_rows, n_edges=len(g[0]))
    print(f"config {index} blocks: wrote {path}, max|a| {np.abs(a_rows).max():.4f}, {time.time() - t0:.0f} s", flush=True)


def _blocks_backward_nodes(j_range):
    """Destination nodes j_range of the node block's adjoint (a sum over destination nodes)."""
    from oracle import so2_oracle as S
    w, g, x, T, Wn, w_att, da, edges = (_state[k] for k in ("w", "g", "x", "T", "Wn", "w_att", "da", "edges"))
    j0, j1 = j_range
    src, dst, shift, row_ptr = g
    k0, k1 = int(row_ptr[j0]), int(row_ptr[j1])
    sub = (src[k0:k1], dst[k0:k1], shift[k0:k1], row_ptr[j0:j1 + 1] - k0)
    kink = []
    dx, dT, dW0, dWr, dWi, dw_att = S.so2_node_block_backward(sub, w.pos, w.box, x, T[k0:k1], Wn[1], Wn[2], Wn[3], w_att,
                                                              w.lmax, w.channels, w.r_cut, da[j0:j1], near_kink=kink,
                                                              kink_eps=KINK_EPS)
    pick = edges[(edges >= k0) & (edges < k1)]
    return dx, (pick, dT[pick - k0]), [dW0] + list(dWr) + list(dWi) + [dw_att, np.asarray(kink, np.int64) + k0]


# score inputs closer to zero than this are where an fp32 evaluation may take the other branch of LeakyReLU'
KINK_EPS = 4e-6
EDGE_PIECE = 8192     # edges per oracle call inside a job of the edge block's adjoint


def _blocks_backward_edges(k_range):
    """Edges k_range of the edge block's adjoint (a sum over the edges)."""
    from oracle import so2_oracle as S
    w, g, x, T, We, dT_out, edges = (_state[k] for k in ("w", "g", "x", "T", "We", "dT_out", "edges"))
    k0, k1 = k_range
    pick = edges[(edges >= k0) & (edges < k1)]
    dx, flat, rows = None, None, []
    for a in range(k0, k1, EDGE_PIECE):      # (small pieces: the oracle call holds several fp64 copies of its range)
        b = min(k1, a + EDGE_PIECE)
        sub = (g[0][a:b], g[1][a:b], g[2][a:b], g[3])
        pdx, dT_in, dW0, dWr, dWi = S.so2_edge_block_backward(sub, w.pos, w.box, x, T[a:b], We[1], We[2], We[3], w.lmax,
                                                              w.channels, w.r_cut, dT_out[a:b])
        part = [dW0] + list(dWr) + list(dWi)
        if dx is None:
            dx, flat = pdx, part
        else:
            dx += pdx
            for acc, v in zip(flat, part):
                acc += v
        here = pick[(pick >= a) & (pick < b)]
        rows.append(dT_in[here - a])
    return dx, (pick, np.concatenate(rows)), flat


def make_blocks_backward(index, pool_size):
    """Adjoints of the node block and of the edge block of the full-size configuration ->
    config{index}_so2_blocks_backward.npz: all weight gradients (and dw_att), dx at aimed nodes, the gradient of the
    edge embeddings at aimed edges.  Inputs from tests/gpu_util.block_inputs; da and dT_out from tests/gpu_util
    (so2_da, blocks_dT_out)."""
    t0 = time.time()
    w = synth.workload(index)
    g, x, T, Wn, We, w_att = U.block_inputs(w)
    n_e = len(g[0])
    rng = np.random.default_rng([w.seed, 4246])
    nodes = aimed_nodes(w, g, rng, w.n_total)
    edges = aimed_edges(g, rng)
    _state.update(w=w, g=g, x=x, T=T, Wn=Wn, We=We, w_att=w_att, da=U.so2_da(w), dT_out=U.blocks_dT_out(w, n_e), edges=edges)
    out = dict(nodes=nodes, edges=edges, n_edges=n_e)
    # (few large ranges: every job returns a full dx, 0.26 GB at config 4; a node job also holds the gradient of the
    # edge embeddings of its range)
    step_n = max(32, -(-w.n_owned // (4 * pool_size)))
    step_e = max(8192, -(-n_e // (2 * pool_size)))
    jobs_n = [(j0, min(w.n_owned, j0 + step_n)) for j0 in range(0, w.n_owned, step_n)]
    jobs_e = [(k0, min(n_e, k0 + step_e)) for k0 in range(0, n_e, step_e)]
    for tag, fn, jobs, names in (("node", _blocks_backward_nodes, jobs_n, ["dW0", "dWr", "dWi", "dw_att"]),
                                 ("edge", _blocks_backward_edges, jobs_e, ["dW0", "dWr", "dWi"])):
        dx, flat, kinks = None, None, []
        dT_rows = np.zeros((len(edges),) + T.shape[1:])
        with ProcessPoolExecutor(pool_size) as ex:
            for part_dx, (pick, rows), part_w in ex.map(fn, jobs):
                if tag == "node":
                    kinks.append(part_w.pop())
                if dx is None:
                    dx, flat = part_dx, part_w
                else:
                    dx += part_dx
                    for acc, v in zip(flat, part_w):
                        acc += v
                dT_rows[np.searchsorted(edges, pick)] = rows
        wdt = np.float64 if index <= 3 else np.float32   # (as in make_so2_backward; the stored rows likewise)
        out[f"{tag}_dx_rows"] = dx[nodes].astype(wdt)
        out[f"{tag}_dx_maxabs_l"] = maxabs_per_degree(dx, w.lmax)
        out[f"{tag}_dT_rows"] = dT_rows.astype(wdt)
        out[f"{tag}_dW0"] = flat[0].astype(wdt)
        for m in range(w.lmax):
            out[f"{tag}_dWr{m + 1}"] = flat[1 + m].astype(wdt)
            out[f"{tag}_dWi{m + 1}"] = flat[1 + w.lmax + m].astype(wdt)
        if tag == "node":
            out["node_dw_att"] = flat[-1]
            # edges with a score input within KINK_EPS of zero, and the nodes whose rows of dx they reach
            kink_edges = np.unique(np.concatenate(kinks)) if kinks else np.zeros(0, np.int64)
            out["node_kink_edges"] = kink_edges
            out["node_kink_nodes"] = np.unique(np.concatenate([g[0][kink_edges], g[1][kink_edges]])).astype(np.int64)
        print(f"config {index} blocks backward: {tag} block done, {time.time() - t0:.0f} s", flush=True)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"config{index}_so2_blocks_backward.npz")
    np.savez_compressed(path, **out)
    print(f"config {index} blocks backward: wrote {path}, {os.path.getsize(path) / 1e3:.0f} kB, {time.time() - t0:.0f} s", flush=True)


def _w16_node(j):
    """Layer output row of owned node j from the layer-0 input, with (half) and without (full) rounding of w."""
    w, g, x, h, W, agg = (_state[k] for k in ("w", "g", "x", "h", "W", "agg"))
    src, dst, shift, row_ptr = g
    k0, k1 = int(row_ptr[j]), int(row_ptr[j + 1])
    sub = (src[k0:k1], dst[k0:k1], shift[k0:k1], row_ptr[j:j + 2] - k0)
    out = []
    for w_dtype in (np.float16, None):
        fn = lambda d, a, b, paths: O.radial_weights(d, W["W_r1"], W["W_r2"], paths, w.channels, w.n_rbf, w.r_cut,
                                                     w_dtype)
        a = O.edge_messages_sum(sub, w.pos, w.box, h, fn, w.lmax, w.lmax, agg)
        out.append((O.mix_channels(a, W["W_post"], w.lmax) + O.mix_channels(x[j:j + 1], W["W_self"], w.lmax))[0])
    return out


def _w16_edge(k):
    w, g, x, Wr = _state["w"], _state["g"], _state["x"], _state["Wr"]
    return [O.readout_hij(g, w.pos, w.box, x, Wr, w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, w.orb_l,
                          k_range=(k, k + 1), w_dtype=dt)[0] for dt in (np.float16, None)]


def make_w16(index, pool_size):
    """First layer (sampled owned nodes) and readout (sampled edges) of the full-size configuration, both applied to
    the layer-0 features, with the per-edge path weights rounded to half precision -> config{index}_w16_samples.npz
    (the unrounded results of the same rows are stored next to them)."""
    t0 = time.time()
    w = synth.workload(index)
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = U.mean_degree(g, w.n_owned)
    rng = np.random.default_rng([w.seed, 4244])
    nodes = np.sort(rng.choice(w.n_owned, N_NODE_SAMPLES, replace=False))
    edges = np.sort(rng.choice(len(g[0]), N_EDGE_SAMPLES, replace=False))
    x = O.species_embed(wt["x0"], w.species, wt["table"])
    W = wt["layers"][0]
    _state.update(w=w, g=g, x=x, h=O.mix_channels(x, W["W_pre"], w.lmax), W=W, agg=agg, Wr=wt["readout"])
    with ProcessPoolExecutor(pool_size) as ex:
        rows = list(ex.map(_w16_node, [int(j) for j in nodes]))
        blocks = list(ex.map(_w16_edge, [int(k) for k in edges]))
    out = dict(nodes=nodes, edges=edges, agg=agg, n_edges=len(g[0]),
               x1_rows=np.array([r[0] for r in rows]), x1_rows_full=np.array([r[1] for r in rows]),
               H_rows=np.array([b[0] for b in blocks]), H_rows_full=np.array([b[1] for b in blocks]))
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"config{index}_w16_samples.npz")
    np.savez_compressed(path, **out)
    d1 = np.abs(out["x1_rows"] - out["x1_rows_full"]).max() / np.abs(out["x1_rows_full"]).max()
    d2 = np.abs(out["H_rows"] - out["H_rows_full"]).max() / np.abs(out["H_rows_full"]).max()
    print(f"config {index} w16: wrote {path}; effect of the rounding: layer {d1:.2e}, H {d2:.2e}; "
          f"{time.time() - t0:.0f} s", flush=True)


def make(index, pool_size):
    t0 = time.time()
    w = synth.workload(index)
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = U.mean_degree(g, w.n_owned)
    rng = np.random.default_rng([w.seed, 4242])
    nodes = aimed_nodes(w, g, rng, w.n_owned)
    out = dict(nodes=nodes, n_edges=len(g[0]), agg=agg)
    x = O.species_embed(wt["x0"], w.species, wt["table"])
    for t in range(w.n_layers):
        y = layer_parallel(pool_size, w, g, x, wt["layers"][t], agg)
        out[f"x{t + 1}_rows"] = y[nodes]
        out[f"x{t + 1}_maxabs"] = np.abs(y).max()
        out[f"x{t + 1}_maxabs_l"] = maxabs_per_degree(y, w.lmax)
        print(f"config {index}: layer {t} done, max|x| {np.abs(y).max():.4f}, {time.time() - t0:.0f} s", flush=True)
        x = np.concatenate([y, wt["halo"][(t + 1) % w.n_layers].astype(np.float64)], axis=0) \
            if w.n_total > w.n_owned else y
    if w.readout:
        edges = aimed_edges(g, rng)
        _state.update(w=w, g=g, x=x, Wr=wt["readout"])
        H = np.zeros((len(edges), w.n_orb, w.n_orb))
        with ProcessPoolExecutor(pool_size) as ex:
            for i, (k0, part) in enumerate(ex.map(_readout_chunk, [(int(k), int(k) + 1) for k in edges])):
                H[i] = part[0]
        # scale of the whole tensor and of every shell block: estimated on a larger random sample of edges
        more = np.sort(rng.choice(len(g[0]), 2048, replace=False))
        with ProcessPoolExecutor(pool_size) as ex:
            Hm = np.concatenate([p for _, p in ex.map(_readout_chunk, [(int(k), int(k) + 1) for k in more])] + [H])
        out.update(edges=edges, H_rows=H, H_maxabs=np.abs(Hm).max(), H_maxabs_blocks=maxabs_per_shell_block(Hm, w.orb_l))
        print(f"config {index}: readout done, {time.time() - t0:.0f} s", flush=True)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"config{index}_samples.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, f"{os.path.getsize(path) / 1e3:.0f} kB", flush=True)




# ------------------------------------------------------------------------------------------------------------
# training step (config 5): loss and every gradient.  The reverse pass of the oracle is spread over processes
# by edge chunks; each chunk goes through the oracle's own adjoint functions, partial sums are added in order.
# ------------------------------------------------------------------------------------------------------------
EDGE_CHUNK = 8192


def _layer_bwd_chunk(args):
    k0, k1 = args
    w, g, h, W, da, agg = (_state[k] for k in ("w", "g", "h", "W", "da", "agg"))
    src, dst, shift, row_ptr = g
    paths = O.tp_paths(w.lmax, w.lmax, w.lmax)
    r = O.edge_vectors(w.pos, w.box, src[k0:k1], dst[k0:k1], shift[k0:k1])
    d = np.sqrt(np.einsum("ka,ka->k", r, r))
    Y = O.sph_harm_real(w.lmax, r / d[:, None])
    wk = O.radial_weights(d, W["W_r1"], W["W_r2"], paths, w.channels, w.n_rbf, w.r_cut)
    dh_k, dw_k = O.tensor_product_backward(h[src[k0:k1]], Y, wk, paths, da[dst[k0:k1]] / np.sqrt(agg))
    dh = np.zeros_like(h)
    np.add.at(dh, src[k0:k1], dh_k)
    g1, g2 = O.radial_weights_backward(d, W["W_r1"], W["W_r2"], paths, w.channels, w.n_rbf, w.r_cut, dw_k)
    return dh, g1, g2


def layer_backward_parallel(pool_size, w, g, x, W, agg, dx_out):
    """Same composition as oracle.layer_backward, the edge loop split over processes."""
    h = O.mix_channels(x, W["W_pre"], w.lmax)
    _state.update(w=w, g=g, h=h, W=W, agg=agg)
    a = np.zeros((w.n_owned, (w.lmax + 1) ** 2, w.channels))
    jobs = [(j0, min(w.n_owned, j0 + CHUNK)) for j0 in range(0, w.n_owned, CHUNK)]
    with ProcessPoolExecutor(pool_size) as ex:
        for j0, part in ex.map(_messages_chunk, jobs):
            a[j0:j0 + part.shape[0]] = part
    da, dW_post = O.mix_channels_backward(a, W["W_post"], dx_out, w.lmax)
    dx_self, dW_self = O.mix_channels_backward(x[:w.n_owned], W["W_self"], dx_out, w.lmax)
    _state.update(da=da)
    dh = np.zeros_like(h)
    dW_r1 = np.zeros(np.shape(W["W_r1"]))
    dW_r2 = np.zeros(np.shape(W["W_r2"]))
    n_e = len(g[0])
    with ProcessPoolExecutor(pool_size) as ex:
        for p_dh, g1, g2 in ex.map(_layer_bwd_chunk, [(k, min(n_e, k + EDGE_CHUNK)) for k in range(0, n_e, EDGE_CHUNK)]):
            dh += p_dh
            dW_r1 += g1
            dW_r2 += g2
    dx, dW_pre = O.mix_channels_backward(x, W["W_pre"], dh, w.lmax)
    dx[:w.n_owned] += dx_self
    return dx, dict(W_pre=dW_pre, W_post=dW_post, W_self=dW_self, W_r1=dW_r1, W_r2=dW_r2)


def _readout_fwd_bwd_chunk(args):
    """H of a chunk of edges, its contribution to the loss, and the chunk's share of every readout gradient."""
    k0, k1 = args
    w, g, x, Wr, T, n_values = (_state[k] for k in ("w", "g", "x", "Wr", "T", "n_values"))
    src, dst, shift, row_ptr = g
    H = O.readout_hij(g, w.pos, w.box, x, Wr, w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, w.orb_l, k_range=(k0, k1))
    diff = H - T[k0:k1]
    dH = 2.0 * diff / n_values
    sub = (src[k0:k1], dst[k0:k1], shift[k0:k1], None)
    dx, gr = O.readout_backward(sub, w.pos, w.box, x, Wr, w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, w.orb_l, dH)
    return float(np.sum(diff * diff)), dx, gr, np.abs(H).max()


def training_parallel(pool_size, w, wt, g, agg, T):
    """Same chain as tests/gpu_util.oracle_training_step (forward, MSE, reverse pass), the loops over destination
    nodes and over edges spread over processes.  Returns dict(loss, grads, H_maxabs)."""
    n_e = len(g[0])
    xs = [O.species_embed(wt["x0"], w.species, wt["table"])]
    for t in range(w.n_layers):
        y = layer_parallel(pool_size, w, g, xs[-1], wt["layers"][t], agg)
        xs.append(np.concatenate([y, wt["halo"][(t + 1) % w.n_layers].astype(np.float64)], axis=0)
                  if w.n_total > w.n_owned else y)
        print(f"training chain: forward layer {t} done", flush=True)
    _state.update(w=w, g=g, x=xs[-1], Wr=wt["readout"], T=T, n_values=float(T.size))
    sq, dx, g_ro, hmax = 0.0, np.zeros_like(xs[-1]), None, 0.0
    with ProcessPoolExecutor(pool_size) as ex:
        for s_part, dx_part, gr, hm in ex.map(_readout_fwd_bwd_chunk,
                                              [(k, min(n_e, k + EDGE_CHUNK)) for k in range(0, n_e, EDGE_CHUNK)]):
            sq += s_part
            dx += dx_part
            hmax = max(hmax, hm)
            g_ro = gr if g_ro is None else {k: g_ro[k] + gr[k] for k in gr}
    grads = {f"readout.{k}": v for k, v in g_ro.items()}
    print(f"training chain: readout forward+backward done, loss {sq / T.size:.6f}", flush=True)
    for t in reversed(range(w.n_layers)):
        dx, g_l = layer_backward_parallel(pool_size, w, g, xs[t], wt["layers"][t], agg, dx[:w.n_owned])
        grads.update({f"layer{t}.{k}": v for k, v in g_l.items()})
        print(f"training chain: backward layer {t} done", flush=True)
    grads["x0"] = dx
    return dict(loss=sq / T.size, grads=grads, H_maxabs=hmax)


def make_training(index, pool_size):
    t0 = time.time()
    w = synth.workload(index)
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = U.mean_degree(g, w.n_owned)
    n_e = len(g[0])
    T = synth.normal(np.random.default_rng([w.seed, 99]), (n_e, w.n_orb, w.n_orb))
    res = training_parallel(pool_size, w, wt, g, agg, T)
    out = dict(loss=res["loss"], n_edges=n_e, agg=agg, H_maxabs=res["H_maxabs"])
    dx = res["grads"].pop("x0")
    out.update(res["grads"])
    rng = np.random.default_rng([w.seed, 4242])
    nodes = aimed_nodes(w, g, rng, w.n_total)
    out.update(nodes=nodes, x0_rows=dx[nodes], x0_maxabs=np.abs(dx).max(), x0_maxabs_l=maxabs_per_degree(dx, w.lmax))
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"config{index}_training.npz")
    np.savez_compressed(path, **out)
    print("wrote", path, f"{os.path.getsize(path) / 1e3:.0f} kB, {time.time() - t0:.0f} s", flush=True)


if __name__ == "__main__":
    which = [int(a) for a in sys.argv[1:] if ":" not in a] or ([] if len(sys.argv) > 1 else [3, 4, 5])
    procs = int(os.environ.get("GOLDEN_PROCS", "6"))
    for a in sys.argv[1:]:
        if a.startswith("so2:"):   # e.g. so2:3 so2:4
            make_so2(int(a[4:]), procs)
        if a.startswith("so2bwd:"):
            make_so2_backward(int(a[7:]), procs)
        if a.startswith("blocksbwd:"):
            make_blocks_backward(int(a[10:]), procs)
        if a.startswith("w16:"):
            make_w16(int(a[4:]), procs)
        if a.startswith("blocks:"):
            make_blocks(int(a[7:]), procs)
    for idx in which:
        if idx == 5:               # training step
            make_training(idx, procs)
        else:
            make(idx, procs)
