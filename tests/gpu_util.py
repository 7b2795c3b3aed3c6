"""Shared helpers of the GPU parity tests: build both sides from one seeded workload."""
import numpy as np
from oracle import egnn_oracle as O
from paper_2507_03840_amd import synth

TOL = 1e-4   # max|gpu - oracle| / max|oracle| per output tensor (fp32 path vs fp64 oracle)


def rel_err(gpu, ref):
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    scale = np.abs(ref).max()
    return float(np.abs(gpu - ref).max() / (scale if scale > 0 else 1.0))


def model_weights(w, seed_offset=0):
    """Random weights for every layer and the readout of workload w (dict of numpy arrays)."""
    rng = np.random.default_rng([w.seed, 1000 + seed_offset])
    P = len(O.tp_paths(w.lmax, w.lmax, w.lmax))
    P_ro = len(O.tp_paths(w.lmax, w.lmax, O.L_READOUT))
    _, n_out = O.readout_slots(w.orb_l)
    layers = [synth.layer_weights(rng, w.lmax, w.channels, w.n_rbf, w.n_hidden, P) for _ in range(w.n_layers)]
    ro = synth.readout_weights(rng, w.lmax, w.channels, w.n_rbf, w.n_hidden, P_ro, sum(n_out))
    x0 = synth.node_features(rng, w.n_total, w.lmax, w.channels)
    table = synth.species_table(rng, w.n_species, w.channels)
    halo = [synth.node_features(rng, w.n_total - w.n_owned, w.lmax, w.channels) for _ in range(w.n_layers)]
    return dict(layers=layers, readout=ro, x0=x0, table=table, halo=halo)


def oracle_graph(w):
    return O.neighbour_list(w.pos, w.n_owned, w.box, w.pbc, w.r_cut)


def mean_degree(g, n_owned):
    return float(len(g[0])) / max(1, n_owned)


def block_inputs(w, seed=0):
    """Seeded inputs of both sides: node features, edge embeddings with every plane filled, SO(2) weights of the node
    and of the edge block, attention vector."""
    g = oracle_graph(w)
    rng = np.random.default_rng([w.seed if getattr(w, "seed", 0) else 0, 17, seed])
    x = synth.node_features(rng, w.n_total, w.lmax, w.channels)
    # (drawn in fp32 directly: at config 4 this tensor has 3.8e9 entries)
    T = rng.standard_normal(size=(len(g[0]), (w.lmax + 1) ** 2, w.channels), dtype=np.float32)
    Wn = synth.so2_weights(rng, w.lmax, w.channels, w.n_rbf)
    We = synth.so2_weights(rng, w.lmax, w.channels, w.n_rbf)
    w_att = synth.normal(rng, (w.channels,), 2.0 / np.sqrt(w.channels))
    return g, x, T, Wn, We, w_att


def so2_da(w):
    """Seeded gradient with respect to the SO(2) message sums of a workload (input of both sides of the adjoint test)."""
    rng = np.random.default_rng([w.seed if getattr(w, "seed", 0) else 0, 778])
    return rng.standard_normal(size=(w.n_owned, (w.lmax + 1) ** 2, w.channels), dtype=np.float32)


def blocks_dT_out(w, n_edges):
    """Seeded gradient with respect to the output of the edge block (input of both sides of the adjoint test)."""
    rng = np.random.default_rng([w.seed if getattr(w, "seed", 0) else 0, 779])
    return rng.standard_normal(size=(n_edges, (w.lmax + 1) ** 2, w.channels), dtype=np.float32)


def oracle_so2_layer_step(w, g, x, T, Wn, We, w_att, W_g, target_h, target_T, grads=True):
    """One training step of a layer built from the SO(2) blocks, on the oracle: h = gate(node_block(x, T)),
    T' = edge_block(x, T), loss = MSE(h, target_h) + MSE(T', target_T); with grads, the chain of the oracle's adjoints
    back to x, T and every weight.  (A composition of oracle functions for the tests; the order of the steps is the one
    of Sec. 3 "Message passing": node block, non-linearity, edge block.)"""
    from oracle import so2_oracle as S
    L, E = w.lmax, w.channels
    a = S.so2_node_block(g, w.pos, w.box, x, T, Wn[1], Wn[2], Wn[3], w_att, L, E, w.r_cut)
    h = S.gate(a, W_g, L)
    T2 = S.so2_edge_block(g, w.pos, w.box, x, T, We[1], We[2], We[3], L, E, w.r_cut)
    loss = O.loss_mse(h, target_h) + O.loss_mse(T2, target_T)
    if not grads:
        return loss
    da, dW_g = S.gate_backward(a, W_g, L, O.loss_mse_backward(h, target_h))
    dx1, dT1, n0, nr, ni, dw_att = S.so2_node_block_backward(g, w.pos, w.box, x, T, Wn[1], Wn[2], Wn[3], w_att, L, E,
                                                            w.r_cut, da)
    dx2, dT2, e0, er, ei = S.so2_edge_block_backward(g, w.pos, w.box, x, T, We[1], We[2], We[3], L, E, w.r_cut,
                                                     O.loss_mse_backward(T2, target_T))
    return loss, dict(x=dx1 + dx2, T=dT1 + dT2, Wn=(n0, nr, ni), We=(e0, er, ei), w_att=dw_att, W_g=dW_g)


def oracle_forward(w, wt, g, agg_norm, with_readout=True, w_dtype=None):
    """Whole model on the oracle: species embedding, n_layers layers, readout.  Returns (xs, H).
    w_dtype: storage precision of the per-edge path weights (None: not rounded)."""
    x = O.species_embed(wt["x0"], w.species, wt["table"])
    xs = []
    for t in range(w.n_layers):
        y = O.layer_forward(g, w.pos, w.box, x, wt["layers"][t], w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut,
                            agg_norm, w_dtype=w_dtype)
        xs.append(y)
        if t + 1 < w.n_layers:
            x = np.concatenate([y, wt["halo"][t + 1].astype(np.float64)], axis=0)
    H = None
    if with_readout:
        xr = np.concatenate([xs[-1], wt["halo"][0].astype(np.float64)], axis=0) if w.n_total > w.n_owned else xs[-1]
        H = O.readout_hij(g, w.pos, w.box, xr, wt["readout"], w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, w.orb_l,
                          w_dtype=w_dtype)
    return xs, H


def gpu_forward(w, wt, agg_norm, with_readout=True, fused=False, w_fp16=False, shared_rows=False):
    """Same model through the C ABI.  Returns (model, graph, xs (device tensors), H).
    shared_rows: one row of radial weights per unordered pair of owned atoms (egnn_edge_pairs)."""
    import torch
    from paper_2507_03840_amd import binding as B
    m = B.Egnn(w.lmax, w.channels, w.n_rbf, w.r_cut, agg_norm, n_layers=w.n_layers, orb_l=w.orb_l)
    if fused:
        m.egnn_set_option(B.OPT_FUSED, int(fused))   # True / 1: first fused design, 2: second
    if w_fp16:
        m.egnn_set_option(B.OPT_W_FP16, 1)
    pos = B.to_device(w.pos)
    graph = m.egnn_nlist(pos, w.n_owned, w.box, w.pbc)
    if shared_rows:
        m.egnn_edge_pairs(graph)
    ws = m.workspace(graph)
    x = B.to_device(wt["x0"])
    m.egnn_species_embed(B.to_device(w.species), B.to_device(wt["table"]), x)
    xs = []
    for t in range(w.n_layers):
        y = m.egnn_layer_forward(graph, pos, w.box, x, B.to_device(wt["layers"][t]), ws)
        xs.append(y)
        if t + 1 < w.n_layers:
            x = torch.cat([y, B.to_device(wt["halo"][t + 1])], dim=0).contiguous()
    H = None
    if with_readout:
        xr = torch.cat([xs[-1], B.to_device(wt["halo"][0])], dim=0).contiguous() if w.n_total > w.n_owned else xs[-1]
        H = m.egnn_readout_hij(graph, pos, w.box, xr, B.to_device(wt["readout"]), ws)
    torch.cuda.synchronize()
    return m, graph, xs, H


def oracle_training_step(w, wt, g, agg, T):
    """Forward, MSE loss and reverse pass on the oracle.  Gradients keyed 'x0', 'layer{t}.{name}', 'readout.{name}'."""
    x = O.species_embed(wt["x0"], w.species, wt["table"])
    xs = [x]
    for t in range(w.n_layers):
        y = O.layer_forward(g, w.pos, w.box, xs[-1], wt["layers"][t], w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, agg)
        nxt = np.concatenate([y, wt["halo"][(t + 1) % w.n_layers].astype(np.float64)], axis=0) \
            if w.n_total > w.n_owned else y
        xs.append(nxt)
    H = O.readout_hij(g, w.pos, w.box, xs[-1], wt["readout"], w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, w.orb_l)
    loss = O.loss_mse(H, T)
    dx, g_ro = O.readout_backward(g, w.pos, w.box, xs[-1], wt["readout"], w.lmax, w.lmax, w.channels, w.n_rbf,
                                  w.r_cut, w.orb_l, O.loss_mse_backward(H, T))
    grads = {f"readout.{k}": v for k, v in g_ro.items()}
    for t in reversed(range(w.n_layers)):
        dx, g_l = O.layer_backward(g, w.pos, w.box, xs[t], wt["layers"][t], w.lmax, w.lmax, w.channels, w.n_rbf,
                                   w.r_cut, agg, dx[:w.n_owned])
        grads.update({f"layer{t}.{k}": v for k, v in g_l.items()})
    grads["x0"] = dx
    return dict(loss=loss, grads=grads)


def gpu_training_step(w, wt, agg, T, repeats=1, timing=None, keep=False, shared_rows=False, length_bins=None):
    """The same step through the C ABI.  Layer inputs are kept; everything else is recomputed in the reverse pass, or
    (keep=True) the radial weights and summed messages of the forward pass are kept and handed back."""
    import torch
    from paper_2507_03840_amd import binding as B
    m = B.Egnn(w.lmax, w.channels, w.n_rbf, w.r_cut, agg, n_layers=w.n_layers, orb_l=w.orb_l)
    pos = B.to_device(w.pos)
    graph = m.egnn_nlist(pos, w.n_owned, w.box, w.pbc)
    if shared_rows:
        m.egnn_edge_pairs(graph)
    if shared_rows if length_bins is None else length_bins:
        m.egnn_length_bins(graph, pos, w.box)      # the per-graph index of the radial MLP's reverse pass
    ws = torch.empty(max(m.egnn_backward_workspace_bytes(graph.n_edges, graph.n_owned, graph.n_total),
                         m.egnn_workspace_bytes(graph.n_edges, graph.n_owned, graph.n_total)),
                     dtype=torch.uint8, device="cuda")
    col_ptr, perm = m.egnn_graph_transpose(graph, ws)
    layers = [B.to_device(l) for l in wt["layers"]]
    ro = B.to_device(wt["readout"])
    Td = B.to_device(T)
    x = B.to_device(wt["x0"])
    m.egnn_species_embed(B.to_device(w.species), B.to_device(wt["table"]), x)
    out = None
    for _ in range(repeats):
        if timing is not None:
            torch.cuda.synchronize()
            t0 = __import__("time").perf_counter()
        xs = [x]
        kept = []
        for t in range(w.n_layers):
            if keep:
                y, sv = m.egnn_layer_forward_save(graph, pos, w.box, xs[-1], layers[t], ws)
                kept.append(sv)
            else:
                y = m.egnn_layer_forward(graph, pos, w.box, xs[-1], layers[t], ws)
            nxt = torch.cat([y, B.to_device(wt["halo"][(t + 1) % w.n_layers])], dim=0).contiguous() \
                if w.n_total > w.n_owned else y
            xs.append(nxt)
        if keep:
            H, w_ro = m.egnn_readout_hij_save(graph, pos, w.box, xs[-1], ro, ws)
        else:
            H = m.egnn_readout_hij(graph, pos, w.box, xs[-1], ro, ws)
        loss, dH = m.egnn_loss_mse(H, Td, ws)
        if keep:
            dx, g_ro = m.egnn_readout_backward_saved(graph, col_ptr, perm, pos, w.box, xs[-1], ro, w_ro, dH, ws)
        else:
            dx, g_ro = m.egnn_readout_backward(graph, col_ptr, perm, pos, w.box, xs[-1], ro, dH, ws)
        grads = {f"readout.{k}": v for k, v in g_ro.items()}
        for t in reversed(range(w.n_layers)):
            if keep:
                dx, g_l = m.egnn_layer_backward_saved(graph, col_ptr, perm, pos, w.box, xs[t], layers[t], kept[t],
                                                      dx[:w.n_owned].contiguous(), ws)
            else:
                dx, g_l = m.egnn_layer_backward(graph, col_ptr, perm, pos, w.box, xs[t], layers[t],
                                                dx[:w.n_owned].contiguous(), ws)
            grads.update({f"layer{t}.{k}": v for k, v in g_l.items()})
        grads["x0"] = dx
        torch.cuda.synchronize()
        if timing is not None:
            timing.append(__import__("time").perf_counter() - t0)
        out = dict(loss=float(loss.cpu()[0]), grads={k: v.cpu().numpy() for k, v in grads.items()},
                   n_edges=graph.n_edges)
    return out
