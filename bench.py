#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

A step = neighbour list (S1) + species embedding + n_layers message-passing layers (S2-S5 each) + H_ij
readout (S6, where the configuration has one) of one synthetic structure, all through the C ABI, inputs resident
in HBM.  The headline value is edge-layer evaluations per second: n_edges * n_layers / step time.  The roofline
object prices the longest-running kernel of the step; per-stage times come from HIP events recorded by the library
on the stream the kernels run on, inside the timed region.

Without --config the line's headline is config 4 (one GPU's share of a large structure: 12,000 owned + 8,000 halo
atoms, 64 channels, the largest single-GPU configuration), and the same measurement of config 3 (3,000 atoms, 32
channels, with readout), the config-5 training step and the extra timings are nested in it as `config3`.  With
--config N only that configuration is run (what the rocprofv3 summaries under profiles/ use).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N] [--no-cpu-baseline] [--forward-only]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
FP32_MFMA_PEAK_TFLOPS = 157.3  # dense fp32 matrix peak


def stage_model(w, n_edges, n_paths, n_paths_ro):
    """Algorithmic bytes per launch of the three heavy kernels (all HBM-bound by design): the per-edge figures of
    the stage table (gathered rows counted once per edge, whether or not a cache serves them)."""
    E, D = w.channels, (w.lmax + 1) ** 2
    # S4: per edge the weight row (P*E floats), the gathered source row (D*E floats), indices and unit vector
    # (24 bytes); per owned node one output row.
    s4_bytes = n_edges * (4 * (n_paths * E + D * E) + 24) + w.n_owned * 4 * D * E
    # S3: per edge one (r_hat, d) record read and the weight row written; the contraction itself
    # (2*(n_rbf*64 + 64*P*E) flop per edge) runs on the half-precision matrix cores and is far from their roofline.
    s3_bytes = n_edges * (4 * n_paths * E + 16)
    s3_flops = n_edges * 2.0 * (w.n_rbf * 64 + 64 * n_paths * E)
    # S6: weight row, two gathered rows, indices/unit vector, one n_orb x n_orb block written
    s6_bytes = n_edges * (4 * (n_paths_ro * E + 2 * D * E) + 24 + 4 * w.n_orb ** 2)
    return s4_bytes, s3_bytes, s3_flops, s6_bytes


def read_traffic(kernel, workload):
    """HBM bytes per launch measured with rocprofv3 --pmc, if a summary for this kernel/workload is committed."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


def compulsory_bytes(w, n_edges, n_paths, n_paths_ro):
    """Bytes the S4 / S6 kernels must move through HBM at least: every gathered node row once (the rows of one
    tensor are re-read from cache by the ~200 edges that use them), the weight rows, indices, unit vectors, outputs."""
    E, D = w.channels, (w.lmax + 1) ** 2
    s4 = n_edges * (4 * n_paths * E + 24) + (w.n_total + w.n_owned) * 4 * D * E
    s6 = n_edges * (4 * n_paths_ro * E + 24 + 4 * w.n_orb ** 2) + 2 * w.n_total * 4 * D * E
    return s4, s6


def _cpu_chunk(args):
    """One worker of the oracle leg: oracle.layer_forward, unchanged, on a structure relabelled so that the
    destination nodes of this chunk are the owned prefix."""
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import egnn_oracle as O
    (j0, j1, w, x, W, agg) = args
    order = np.concatenate([np.arange(j0, j1), np.arange(0, j0), np.arange(j1, w.n_total)])
    pos, xx = w.pos[order], x[order]
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        g = O.neighbour_list(pos, j1 - j0, w.box, w.pbc, w.r_cut)
        t1 = time.perf_counter()
        y = O.layer_forward(g, pos, w.box, xx, W, w.lmax, w.lmax, w.channels, w.n_rbf, w.r_cut, agg)
        t2 = time.perf_counter()
    return len(g[0]), t1 - t0, t2 - t1, float(np.abs(y).max())


def cpu_baseline(w, wt, n_nodes, cores):
    """The oracle's layer_forward, as it stands, on the first n_nodes destination nodes of the workload, spread over
    `cores` processes by destination chunks (one numpy thread each).  Runs before anything touches the GPU."""
    import numpy as np
    from concurrent.futures import ProcessPoolExecutor
    from oracle import egnn_oracle as O
    n_nodes = max(cores, min(n_nodes, w.n_owned))
    x = O.species_embed(wt["x0"], w.species, wt["table"]).astype(np.float32)
    cuts = np.linspace(0, n_nodes, cores + 1).astype(int)
    agg = 200.0          # the normalisation constant does not change the work
    jobs = [(int(cuts[i]), int(cuts[i + 1]), w, x, wt["layers"][0], agg) for i in range(cores) if cuts[i + 1] > cuts[i]]
    t0 = time.perf_counter()
    with ProcessPoolExecutor(len(jobs)) as ex:
        res = list(ex.map(_cpu_chunk, jobs))
    wall = time.perf_counter() - t0
    k = sum(r[0] for r in res)
    t_layer = max(r[2] for r in res)
    return dict(value=k / t_layer, unit="edge-layer evaluations/s", cores=len(jobs), kind="oracle",
                sample=f"one layer forward (oracle.layer_forward, numpy fp64) into the first {n_nodes} destination "
                       f"nodes ({k} edges) of {w.name}, split into {len(jobs)} chunks of destination nodes, one process "
                       f"with one numpy thread per chunk; {t_layer:.1f} s for the slowest chunk (the time used), "
                       f"{wall:.1f} s wall including the chunks' brute-force neighbour search and process start")


def model_weights(w, synth, n_paths, n_paths_readout, n_vrows):
    """Random weights of every layer and of the readout of workload w, drawn in the order the parity tests draw them."""
    import numpy as np
    rng = np.random.default_rng([w.seed, 1000])
    layers = [synth.layer_weights(rng, w.lmax, w.channels, w.n_rbf, w.n_hidden, n_paths) for _ in range(w.n_layers)]
    ro = synth.readout_weights(rng, w.lmax, w.channels, w.n_rbf, w.n_hidden, n_paths_readout, n_vrows)
    x0 = synth.node_features(rng, w.n_total, w.lmax, w.channels)
    table = synth.species_table(rng, w.n_species, w.channels)
    halo = [synth.node_features(rng, w.n_total - w.n_owned, w.lmax, w.channels) for _ in range(w.n_layers)]
    return dict(layers=layers, readout=ro, x0=x0, table=table, halo=halo)


def _so2_flat(ws):
    """(W_e, W0, Wr, Wi) -> [W0, Wr_1, Wi_1, ...] in the order of the C ABI."""
    W_e, W0, Wr, Wi = ws
    return [W0] + [a for pair in zip(Wr, Wi) for a in pair]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=0, choices=[0, 1, 2, 3, 4],
                    help="0 (default): config 4 as the headline with config 3 nested; N: only configuration N")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-nodes", type=int, default=0,
                    help="destination nodes of the oracle sample (0: sized for about 20 s on the cores used)")
    ap.add_argument("--cpu-cores", type=int, default=0, help="processes of the oracle leg (0: min(16, host cores))")
    ap.add_argument("--train-steps", type=int, default=3,
                    help="training steps (forward + loss + reverse pass, config 5) timed after the main region; 0 = skip")
    ap.add_argument("--fused", type=int, default=0, choices=[0, 1, 2],
                    help="1 / 2: radial weights and messages in one kernel (weights never written to memory), first / second design")
    ap.add_argument("--per-edge-rows", action="store_true",
                    help="one row of radial weights per edge (no egnn_edge_pairs): the route before rows were shared "
                         "between an edge and its reverse")
    ap.add_argument("--forward-only", action="store_true",
                    help="only the timed forward steps (no variants, no training step, no extra timings): for profiling runs")
    ap.add_argument("--spatial-order", action="store_true",
                    help="relabel the atoms with egnn_spatial_order first (cubes of r_cut / 2 along a Morton curve)")
    ap.add_argument("--no-partition", action="store_true",
                    help="skip the extra timing of the Low-NN partitioner and of the halo pack / unpack")
    ap.add_argument("--no-hamiltonian", action="store_true",
                    help="skip the extra timing of the Hamiltonian assembly (on-site blocks, padding, L1+L2 loss, CSC matrix)")
    ap.add_argument("--no-so2", action="store_true",
                    help="skip the extra timing of the SO(2) form of the message transform (egnn_so2_message_sum)")
    ap.add_argument("--sweep", action="store_true",
                    help="also time one layer forward on growing prefixes of the destination nodes (saturation curve)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.forward_only:
        args.train_steps, args.no_partition, args.no_hamiltonian, args.no_so2 = 0, True, True, True

    headline = args.config if args.config else 4
    # ---- the oracle on the host cores: first, before this process touches the GPU (its workers are forked) ----
    cpu = None
    if not args.no_cpu_baseline:
        from paper_2507_03840_amd import synth
        from tests import gpu_util as U                      # (the oracle and its helpers: this leg only)
        wc = synth.workload(headline, check_cutoff=False)
        cores = args.cpu_cores or min(16, os.cpu_count() or 1)
        # about 1.2e4 (32 channels) / 0.6e4 (64 channels) edge-layer evaluations per second and core at l_max 4
        per_core = {16: 3.0e4, 32: 1.2e4, 64: 0.6e4}.get(wc.channels, 0.6e4) * (1.0 if wc.lmax >= 4 else 4.0)
        nodes = args.cpu_nodes or int(cores * 15.0 * per_core / 200.0)
        cpu = cpu_baseline(wc, U.model_weights(wc), nodes, cores)
        del wc

    out = run_config(args, headline, extras=bool(args.config) or headline != 4)
    if not args.config:
        # the 3,000-atom configuration with readout, the config-5 training step and the extra timings, nested
        sub = run_config(args, 3, extras=True)
        out["config3"] = {k: sub[k] for k in sub if k not in ("metric", "n_gpus", "higher_is_better", "scaling",
                                                              "vs_baseline", "data")}
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


def run_config(args, index, extras):
    """One configuration: the timed forward steps and their roofline objects; with extras the variants (half-precision
    storage of w, fused S3+S4), the training step and the timings of the other rows."""
    import numpy as np
    import torch
    from paper_2507_03840_amd import binding as B
    from paper_2507_03840_amd import synth

    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    B.load_library()
    w = synth.workload(index, check_cutoff=False)
    if args.spatial_order:
        # the same structure with its atoms relabelled along a Morton curve (egnn_spatial_order): what a caller whose
        # atoms come unordered would do before building the graph; not the default (the parity tests use the
        # generators' numbering)
        perm = B.egnn_spatial_order(w.pos, w.n_owned, w.r_cut / 2)
        w.pos, w.species = np.ascontiguousarray(w.pos[perm]), np.ascontiguousarray(w.species[perm])
    # weights sized from the library's own path and readout-slot counts (nothing of the oracle runs in this leg)
    sizes = B.Egnn(w.lmax, w.channels, w.n_rbf, w.r_cut, 1.0, orb_l=w.orb_l)
    wt = model_weights(w, synth, sizes.n_paths, sizes.n_paths_readout, sum(sizes.egnn_readout_widths()))
    del sizes
    pos = B.to_device(w.pos)
    species = B.to_device(w.species)
    table = B.to_device(wt["table"])
    x0 = B.to_device(wt["x0"])
    layers = [B.to_device(l) for l in wt["layers"]]
    halo = [B.to_device(h) for h in wt["halo"]]
    ro = B.to_device(wt["readout"])

    # the mean degree (aggregation norm) comes from a first neighbour-list build
    probe = B.Egnn(w.lmax, w.channels, w.n_rbf, w.r_cut, 1.0, orb_l=w.orb_l)
    g0 = probe.egnn_nlist(pos, w.n_owned, w.box, w.pbc)
    if not args.per_edge_rows:
        probe.egnn_edge_pairs(g0)
    n_edges, n_rows = g0.n_edges, g0.n_weight_rows
    agg = n_edges / max(1, w.n_owned)
    m = B.Egnn(w.lmax, w.channels, w.n_rbf, w.r_cut, agg, n_layers=w.n_layers, orb_l=w.orb_l)
    m.egnn_set_option(B.OPT_FUSED, args.fused)
    ws = m.workspace(g0)
    x_out = [torch.empty((w.n_owned, m.dim, w.channels), dtype=torch.float32, device="cuda") for _ in range(2)]
    H = torch.empty((n_edges, m.n_orb, m.n_orb), dtype=torch.float32, device="cuda") if w.readout else None
    x_full = torch.empty((w.n_total, m.dim, w.channels), dtype=torch.float32, device="cuda")
    del g0, probe

    def build_graph():
        # S1 and, unless switched off, the row index that lets an edge and its reverse share their radial weights
        graph = m.egnn_nlist(pos, w.n_owned, w.box, w.pbc)
        return graph if args.per_edge_rows else m.egnn_edge_pairs(graph)

    def step():
        graph = build_graph()
        x_full.copy_(x0)
        m.egnn_species_embed(species, table, x_full)
        x = x_full
        for t in range(w.n_layers):
            y = m.egnn_layer_forward(graph, pos, w.box, x, layers[t], ws, out=x_out[t % 2])
            if w.n_total > w.n_owned:
                nxt = halo[(t + 1) % w.n_layers]
                x_full[:w.n_owned].copy_(y)
                x_full[w.n_owned:].copy_(nxt)
                x = x_full
            else:
                x = y
        if w.readout:
            m.egnn_readout_hij(graph, pos, w.box, x, ro, ws, out=H)
        return graph

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    m.egnn_timing_enable(args.steps * (w.n_layers + 1))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms, n_calls = m.egnn_timing_read()
    m.egnn_timing_enable(0)

    # ---- the same step with the radial weights stored in half precision between S3 and S4 / S6 (a reduced-precision
    #      option; reported next to `value`, never as `value`) ----
    w_fp16 = None
    if not args.forward_only:
        m.egnn_set_option(B.OPT_W_FP16, 1)
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        n16 = max(3, args.steps // 2)
        m.egnn_timing_enable(n16 * (w.n_layers + 1))
        t1 = time.perf_counter()
        for _ in range(n16):
            step()
        torch.cuda.synchronize()
        dt16 = (time.perf_counter() - t1) / n16
        ms16, calls16 = m.egnn_timing_read()
        m.egnn_timing_enable(0)
        m.egnn_set_option(B.OPT_W_FP16, 0)
        w_fp16 = dict(ms_per_step=1e3 * dt16, steps=n16, edge_layer_evaluations_per_s=n_edges * w.n_layers / dt16,
                      layer_ms={n: ms16[i] / max(1, calls16[0]) for i, n in enumerate(B.LAYER_STAGES)},
                      readout_ms={n: ms16[5 + i] / max(1, calls16[1]) for i, n in enumerate(B.READOUT_STAGES)} if w.readout else None,
                      note="EGNN_OPT_W_FP16: only the per-edge path weights w are rounded to half precision (once); node "
                           "features, gathered rows and H stay fp32, products and sums fp32; not the fp32 figure")

    # ---- the same fp32 step with S3 and S4 as one kernel whose radial weights never leave the registers
    #      (EGNN_OPT_FUSED = 2); reported next to the main figure unless --fused already selected a fused route ----
    fused_lane = None
    if args.fused == 0 and not args.forward_only:
        m.egnn_set_option(B.OPT_FUSED, 2)
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        nfl = max(3, args.steps // 2)
        m.egnn_timing_enable(nfl * (w.n_layers + 1))
        t1 = time.perf_counter()
        for _ in range(nfl):
            step()
        torch.cuda.synchronize()
        dtfl = (time.perf_counter() - t1) / nfl
        msfl, callsfl = m.egnn_timing_read()
        m.egnn_timing_enable(0)
        m.egnn_set_option(B.OPT_FUSED, 0)
        layer_fl = msfl[3] / max(1, callsfl[0])
        # matrix-core work of the radial contraction in this kernel: three half-precision piece products per fp32
        # product (48 rows of W_r2 per 42 paths are multiplied: the padded tile rows count as work done)
        mfma_flop = 3.0 * 2.0 * 64 * 16 * ((m.n_paths + 15) // 16) * w.channels * n_edges
        fused_lane = dict(ms_per_step=1e3 * dtfl, steps=nfl, edge_layer_evaluations_per_s=n_edges * w.n_layers / dtfl,
                          s3_s4_kernel_ms=layer_fl, edges_per_s=n_edges / (layer_fl * 1e-3),
                          f16_mfma_TFLOPs=mfma_flop / (layer_fl * 1e-3) / 1e12, f16_mfma_peak_TFLOPs=2500.0,
                          note="EGNN_OPT_FUSED = 2: radial weights produced on the matrix cores in the registers of the "
                               "lane that consumes them, no weight tensor in memory; bound by matrix-core plus vector "
                               "work of the same SIMD, not by HBM")

    # ---- S7: training step on the same graph and model (config 5 when the workload is config 3) ----
    training = None
    if extras and w.readout and args.train_steps > 0:
        bws = torch.empty(max(m.egnn_backward_workspace_bytes(n_edges, w.n_owned, w.n_total), ws.numel()),
                          dtype=torch.uint8, device="cuda")
        graph = build_graph()
        col_ptr, perm = m.egnn_graph_transpose(graph, bws)
        m.egnn_length_bins(graph, pos, w.box)      # (with the transpose: the per-graph indices of the reverse pass)
        target = B.to_device(synth.normal(np.random.default_rng([w.seed, 99]), (n_edges, w.n_orb, w.n_orb)))

        def train_step(keep=False):
            x_full.copy_(x0)
            m.egnn_species_embed(species, table, x_full)
            xs, kept = [x_full], []
            for t in range(w.n_layers):
                if keep:
                    y, sv = m.egnn_layer_forward_save(graph, pos, w.box, xs[-1], layers[t], bws)
                    kept.append(sv)
                    xs.append(y)
                else:
                    xs.append(m.egnn_layer_forward(graph, pos, w.box, xs[-1], layers[t], bws))
            if keep:
                Hh, w_ro = m.egnn_readout_hij_save(graph, pos, w.box, xs[-1], ro, bws, out=H)
            else:
                Hh = m.egnn_readout_hij(graph, pos, w.box, xs[-1], ro, bws, out=H)
            loss, dH = m.egnn_loss_mse(Hh, target, bws)
            if keep:
                dx, g_ro = m.egnn_readout_backward_saved(graph, col_ptr, perm, pos, w.box, xs[-1], ro, w_ro, dH, bws)
            else:
                dx, g_ro = m.egnn_readout_backward(graph, col_ptr, perm, pos, w.box, xs[-1], ro, dH, bws)
            for t in reversed(range(w.n_layers)):
                if keep:
                    dx, g_l = m.egnn_layer_backward_saved(graph, col_ptr, perm, pos, w.box, xs[t], layers[t], kept[t],
                                                          dx[:w.n_owned], bws)
                else:
                    dx, g_l = m.egnn_layer_backward(graph, col_ptr, perm, pos, w.box, xs[t], layers[t],
                                                    dx[:w.n_owned], bws)
            return loss

        if w.n_total == w.n_owned:
            train_step()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.train_steps):
                loss = train_step()
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t1) / args.train_steps
            train_step(keep=True)
            torch.cuda.synchronize()
            m.egnn_timing_enable(2 * args.train_steps * (w.n_layers + 1))
            t1 = time.perf_counter()
            for _ in range(args.train_steps):
                loss_k = train_step(keep=True)
            torch.cuda.synchronize()
            dt_k = (time.perf_counter() - t1) / args.train_steps
            ms_k, calls_k = m.egnn_timing_read()
            m.egnn_timing_enable(0)
            # stages of the reverse pass (HIP events of the library on the launch stream) with the bytes each one
            # has to move at least: tp_backward reads w and writes dw; the readout adjoint reads w and dH and writes
            # dw and dz; the radial MLP's reverse pass reads dw once (grid route; the exact route reads it twice)
            wbytes = 4 * n_edges * m.n_paths * w.channels
            wbytes_ro = 4 * n_edges * m.n_paths_readout * w.channels
            row = 4 * m.dim * w.channels
            adj = {n: ms_k[10 + i] / max(1, calls_k[2]) for i, n in enumerate(B.LAYER_ADJOINT_STAGES)}
            adj_ro = {n: ms_k[15 + i] / max(1, calls_k[3]) for i, n in enumerate(B.READOUT_ADJOINT_STAGES)}
            stage_bytes = dict(tp_backward=2 * wbytes, radial_backward=wbytes,
                               readout_backward=2 * wbytes_ro + n_edges * (row + 4 * w.n_orb * w.n_orb))
            reverse = dict(layer_ms=adj, readout_ms=adj_ro,
                           tp_backward_GBs=stage_bytes["tp_backward"] / adj["tp_backward"] / 1e6,
                           radial_backward_GBs=stage_bytes["radial_backward"] / adj["radial_backward"] / 1e6,
                           readout_backward_GBs=stage_bytes["readout_backward"] / adj_ro["readout_backward"] / 1e6,
                           note="per call, forward quantities kept; GB/s = the bytes the stage has to move at least "
                                "(w, dw, dz, dH) over its time, against 8,000 GB/s")
            training = dict(ms_per_step=1e3 * dt, steps=args.train_steps, loss=float(loss.cpu()[0]),
                            edge_layer_evaluations_per_s=n_edges * w.n_layers / dt,
                            step="layers fwd + readout + MSE + readout bwd + layers bwd (forward recomputed inside bwd)",
                            keeping_forward_quantities=dict(
                                ms_per_step=1e3 * dt_k, loss=float(loss_k.cpu()[0]), reverse_pass_stages=reverse,
                                kept_GB=4 * n_rows * w.channels * (w.n_layers * m.n_paths + m.n_paths_readout) / 1e9,
                                note="radial weights of every layer and of the readout and the summed messages kept "
                                     "by the caller (egnn_*_save / egnn_*_backward_saved); gradients bit-identical"))
        del bws

    # ---- what this GPU's memory system delivers to the simplest kernels: 1 GiB elementwise copy and 1 GiB fill ----
    def timed(fn, reps):
        fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(reps):
            fn()
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / reps

    a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    copy_ms = timed(lambda: torch.mul(a, 1.0, out=b), 3)      # the same launch the --pmc calibration reads
    fill_ms = timed(lambda: b.zero_(), 3)
    calibration = dict(copy_GBs=2 * a.numel() * 4 / copy_ms / 1e6, fill_GBs=a.numel() * 4 / fill_ms / 1e6,
                       note="torch elementwise copy (1 GiB read + 1 GiB write) and fill (1 GiB write)")
    del a, b

    # ---- S4 on half-precision weights, with the gathered features in fp32 and in half precision (stage calls, one
    #      weight row per edge; the paper's runs keep embeddings in half precision and aggregate in fp32, Sec. 4.1) ----
    s4_half = None
    if extras and 8 <= w.channels <= 128:
        graph = m.egnn_nlist(pos, w.n_owned, w.box, w.pbc)
        rhat_d = m.egnn_edge_geometry(graph, pos, w.box)[0]
        w16 = m.egnn_radial_weights_f16(0, rhat_d, layers[0]["W_r1"], layers[0]["W_r2"])
        h16 = m.egnn_pack_rows(x0, torch.arange(w.n_total, dtype=torch.int32, device="cuda"), half=True)
        t16 = timed(lambda: m.egnn_tp_segsum_f16(graph, rhat_d, x0, w16, out=x_out[0]), 10)
        t16h = timed(lambda: m.egnn_tp_segsum_f16h(graph, rhat_d, h16, w16, out=x_out[0]), 10)
        s4_half = dict(w_half_features_fp32_ms=t16, w_half_features_half_ms=t16h, rows="one weight row per edge",
                       note="egnn_tp_segsum_f16 / egnn_tp_segsum_f16h: storage precision only, products and sums in fp32")
        del w16, h16, rhat_d

    # ---- the message transform in its SO(2) form (dense per-m linear layers, 3E -> E), same graph and features ----
    so2 = None
    if extras and not args.no_so2 and w.channels >= 8:
        graph = m.egnn_nlist(pos, w.n_owned, w.box, w.pbc)
        W_e, W0, Wr, Wi = synth.so2_weights(np.random.default_rng([w.seed, 777]), w.lmax, w.channels, w.n_rbf)
        flat = B.to_device(np.concatenate([W0.ravel()] + [a.ravel() for pair in zip(Wr, Wi) for a in pair]))
        assert flat.numel() == m.egnn_so2_weight_count()
        We = B.to_device(W_e)
        ws2 = torch.empty(m.egnn_so2_workspace_bytes(n_edges), dtype=torch.uint8, device="cuda")
        so2_ms = timed(lambda: m.egnn_so2_message_sum(graph, pos, w.box, x0, We, flat, ws2, out=x_out[0]), 5)
        E_, L_ = w.channels, w.lmax
        macs = sum((1 if q == 0 else 4) * ((L_ + 1 - q) * E_) * ((L_ + 1 - q) * 2 * E_) for q in range(L_ + 1)) + (L_ + 1) * E_ * E_
        so2 = dict(ms=so2_ms, edges_per_s=n_edges / so2_ms * 1e3, flop_per_edge=2 * macs,
                   TFLOPs_fp32_equivalent=2 * macs * n_edges / so2_ms / 1e9,
                   f16_mfma_TFLOPs=3 * 2 * macs * n_edges / so2_ms / 1e9, f16_mfma_peak_TFLOPs=2500.0,
                   workspace_GB=ws2.numel() / 1e9,
                   note="gather+rotate, five GEMMs on half-precision pieces of the fp32 operands (three products per fp32 product), rotate back + segmented sum")
        del ws2
        # its reverse pass (gradients of the node embeddings, W_e and the per-order weights)
        ws2b = torch.empty(max(m.egnn_so2_backward_workspace_bytes(n_edges, w.n_owned),
                               m.egnn_backward_workspace_bytes(n_edges, w.n_owned, w.n_total)),
                           dtype=torch.uint8, device="cuda")
        cp2, pm2 = m.egnn_graph_transpose(graph, ws2b)
        da2 = torch.ones((w.n_owned, (L_ + 1) ** 2, E_), dtype=torch.float32, device="cuda")
        so2_bwd_ms = timed(lambda: m.egnn_so2_message_sum_backward(graph, cp2, pm2, pos, w.box, x0, We, flat, da2, ws2b), 3)
        so2["backward_ms"] = so2_bwd_ms
        so2["backward_workspace_GB"] = ws2b.numel() / 1e9
        del ws2b, cp2, pm2, da2
        # the same transform with the full message content: persistent edge embeddings, attention-weighted node block,
        # gate, edge block (one layer in the shape the paper describes)
        ws3 = torch.empty(m.egnn_so2_blocks_workspace_bytes(n_edges), dtype=torch.uint8, device="cuda")
        rng_b = np.random.default_rng([w.seed, 778])
        Wn = B.to_device(np.concatenate([a.ravel() for a in _so2_flat(synth.so2_weights(rng_b, w.lmax, w.channels, w.n_rbf))]))
        Wed = B.to_device(np.concatenate([a.ravel() for a in _so2_flat(synth.so2_weights(rng_b, w.lmax, w.channels, w.n_rbf))]))
        w_att = B.to_device(synth.normal(rng_b, (w.channels,), 2.0 / np.sqrt(w.channels)))
        W_g = B.to_device(synth.normal(rng_b, (max(1, w.lmax), w.channels, w.channels), w.channels ** -0.5))
        T_edge = m.egnn_edge_embed_init(graph, pos, w.box, We, ws3)
        xb = x0.clone()
        t_node = timed(lambda: m.egnn_so2_node_block(graph, pos, w.box, xb, T_edge, Wn, w_att, ws3, out=x_out[0]), 3)
        t_gate = timed(lambda: m.egnn_gate(x_out[0], W_g, out=x_out[1]), 3)
        t_edge = timed(lambda: m.egnn_so2_edge_block(graph, pos, w.box, xb, T_edge, Wed, ws3, out=T_edge), 3)
        # their reverse passes
        ws3b = torch.empty(max(m.egnn_so2_blocks_backward_workspace_bytes(n_edges, w.n_owned),
                               m.egnn_backward_workspace_bytes(n_edges, w.n_owned, w.n_total)),
                           dtype=torch.uint8, device="cuda")
        cp3, pm3 = m.egnn_graph_transpose(graph, ws3b)
        da3 = torch.ones((w.n_owned, (L_ + 1) ** 2, E_), dtype=torch.float32, device="cuda")
        dT3 = torch.ones_like(T_edge)
        t_node_b = timed(lambda: m.egnn_so2_node_block_backward(graph, cp3, pm3, pos, w.box, xb, T_edge, Wn, w_att, da3, ws3b), 3)
        t_edge_b = timed(lambda: m.egnn_so2_edge_block_backward(graph, cp3, pm3, pos, w.box, xb, T_edge, Wed, dT3, ws3b, dT_in=dT3), 3)
        t_gate_b = timed(lambda: m.egnn_gate_backward(x_out[0], W_g, x_out[1]), 3)
        del ws3b, cp3, pm3, da3, dT3
        macs_full = sum((1 if q == 0 else 4) * ((L_ + 1 - q) * E_) * ((L_ + 1 - q) * 3 * E_) for q in range(L_ + 1))
        so2["full_content"] = dict(node_block_ms=t_node, gate_ms=t_gate, edge_block_ms=t_edge,
                                   node_block_backward_ms=t_node_b, gate_backward_ms=t_gate_b,
                                   edge_block_backward_ms=t_edge_b,
                                   layer_ms=t_node + t_gate + t_edge,
                                   messages_per_s=2 * n_edges / (t_node + t_edge) * 1e3,
                                   floats_per_message=3 * (L_ + 1) ** 2 * E_, flop_per_message=2 * macs_full,
                                   f16_mfma_TFLOPs=3 * 2 * macs_full * n_edges * 2 / (t_node + t_edge) / 1e9,
                                   workspace_GB=ws3.numel() / 1e9, edge_embeddings_GB=T_edge.numel() * 4 / 1e9,
                                   note="node block = gather (3 x 25 x E floats per message) + GEMMs + attention + "
                                        "weighted segmented sum; edge block = the same transform with its own weights, "
                                        "then T_edge += f_c y")
        del ws3, T_edge, xb

    # ---- assembly of the predicted Hamiltonian from the blocks of this step: on-site blocks, padding for two species
    #      with 10 and 4 of the 13 orbitals, L1+L2 loss, column-compressed matrix ----
    ham = None
    if extras and w.readout and not args.no_hamiltonian:
        graph = m.egnn_nlist(pos, w.n_owned, w.box, w.pbc)
        off = np.concatenate([[0], np.cumsum([2 * l + 1 for l in w.orb_l])])
        def bits_of(shells):
            return sum(1 << o for s in shells for o in range(off[s], off[s + 1]))
        orb_bits = B.to_device(np.array([bits_of([0, 1, 2, 4]), bits_of([0, 2])], np.uint32).view(np.int32))
        n_out = m.egnn_readout_widths()
        V_node = B.to_device((synth.normal(np.random.default_rng([w.seed, 555]), (sum(n_out), w.channels)) /
                              np.sqrt(w.channels)).astype(np.float32))
        hws, plan = m.hamiltonian_workspace(graph)
        target = B.to_device(synth.normal(np.random.default_rng([w.seed, 99]), (n_edges, w.n_orb, w.n_orb)))
        H_node = m.egnn_onsite_hii(x_full, V_node, hws)
        orb_off, col_ptr, nnz = m.egnn_hamiltonian_structure(graph, species, orb_bits, plan)
        vals = torch.empty(nnz, dtype=torch.float32, device="cuda")
        rows = torch.empty(nnz, dtype=torch.int32, device="cuda")
        t_on = timed(lambda: m.egnn_onsite_hii(x_full, V_node, hws, out=H_node), 5)
        t_pad = timed(lambda: m.egnn_apply_padding(H, graph.src, graph.dst, species, orb_bits), 5)
        t_loss = timed(lambda: m.egnn_loss_l1l2(H, target, graph.src, graph.dst, species, orb_bits, hws), 5)
        t_struct = timed(lambda: m.egnn_hamiltonian_structure(graph, species, orb_bits, plan), 5)
        t_fill = timed(lambda: m.egnn_hamiltonian_fill(graph, species, orb_bits, orb_off, plan, H, H_node, nnz,
                                                       values=vals, row_idx=rows), 5)
        t_vals = timed(lambda: m.egnn_hamiltonian_fill(graph, species, orb_bits, orb_off, plan, H, H_node, nnz,
                                                       want_rows=False, values=vals), 5)
        nq = w.n_orb * w.n_orb
        cnt = torch.tensor([10, 4], device="cuda")[species.long()]
        n_present = int((cnt[graph.src.long()] * cnt[graph.dst.long()]).sum())
        blocks_bytes = (n_edges + w.n_owned) * nq * 4
        ham = dict(matrix=[int(orb_off[-1]), int(col_ptr.numel() - 1)], stored_entries=int(nnz),
                   onsite_ms=t_on, padding_ms=t_pad, loss_l1l2_ms=t_loss, structure_ms=t_struct,
                   fill_ms=t_fill, fill_values_only_ms=t_vals,
                   padding_GBs=(n_edges * nq - n_present) * 4 / t_pad / 1e6,
                   loss_GBs=n_edges * nq * 4 * 3 / t_loss / 1e6,
                   fill_GBs=(blocks_bytes + 8 * nnz) / t_fill / 1e6,
                   fill_values_only_GBs=(blocks_bytes + 4 * nnz) / t_vals / 1e6,
                   edge_entries_not_padding=n_present,
                   note="species 0 / 1 own 10 / 4 of the 13 orbitals; GB/s = algorithmic bytes over time (padding: "
                        "the zeros written; loss: H, T read, dH written; fill: blocks read once, outputs written once)")
        del vals, rows, target, H_node, hws, plan

    # ---- Low-NN partitioner on the structure tiled 2 x 2 x 2 (the shape of the paper's partitioning example: 24,000
    #      atoms into 64 parts), and pack / unpack of the halo rows of one part ----
    lownn = None
    if extras and not args.no_partition and all(w.pbc):
        shifts = np.array([[i, j, k] for i in range(2) for j in range(2) for k in range(2)], np.float32)
        big_pos = np.concatenate([w.pos + sft * w.box for sft in shifts]).astype(np.float32)
        big_box = (2 * w.box).astype(np.float32)
        mb = B.Egnn(w.lmax, w.channels, w.n_rbf, w.r_cut, 1.0)
        gb = mb.egnn_nlist(B.to_device(big_pos), len(big_pos), big_box, w.pbc)
        deg = torch.diff(gb.row_ptr).cpu().numpy().astype(np.int32)
        t0p = time.perf_counter()
        part, cut_log = B.egnn_partition_low_nn(big_pos, deg, big_box, w.pbc, w.r_cut, 6)
        t_part = time.perf_counter() - t0p
        pt = torch.from_numpy(part.astype(np.int64)).cuda()
        ps, pd = pt[gb.src.long()], pt[gb.dst.long()]
        cross = ps != pd
        pairs = torch.unique(ps[cross] * 64 + pd[cross])
        n_nb = torch.bincount(pairs % 64, minlength=64).cpu().numpy()
        dsum = np.bincount(part, weights=deg, minlength=64)
        # halo of part 0: distinct sources of its incoming edges that it does not own
        halo_idx = torch.unique(gb.src[(pd == 0) & cross]).to(torch.int32)
        xb = torch.randn((len(big_pos), m.dim, w.channels), device="cuda")
        xf = torch.empty((int((pt == 0).sum()) + halo_idx.numel(), m.dim, w.channels), device="cuda")
        t_pack = timed(lambda: m.egnn_pack_rows(xb, halo_idx, half=True), 5)
        buf = m.egnn_pack_rows(xb, halo_idx, half=True)
        t_unpack = timed(lambda: m.egnn_unpack_rows(buf, xf, int((pt == 0).sum())), 5)
        lownn = dict(atoms=int(len(big_pos)), edges=int(gb.n_edges), parts=64, host_ms=1e3 * t_part,
                     cut_dimensions_by_level={int(l): sorted({int(e[1]) for e in cut_log if e[0] == l}) for l in range(6, 0, -1)},
                     degree_sum_max_over_mean=float(dsum.max() / dsum.mean()),
                     neighbour_parts_min_mean_max=[int(n_nb.min()), float(n_nb.mean()), int(n_nb.max())],
                     part0_owned=int((pt == 0).sum()), part0_halo_rows=int(halo_idx.numel()),
                     pack_f16_ms=t_pack, unpack_f16_ms=t_unpack,
                     pack_GBs=halo_idx.numel() * m.dim * w.channels * 6 / t_pack / 1e6,
                     note="host code, one core; the paper quotes 1.41 s for 64 parts of its 24,000-atom structure (another "
                          "machine and implementation: context only)")
        del xb, xf, buf, gb

    # ---- saturation curve: one layer forward into the first n destination nodes ----
    sweep = None
    if args.sweep:
        graph = m.egnn_nlist(pos, w.n_owned, w.box, w.pbc)
        row = graph.row_ptr.cpu().numpy()
        x_full.copy_(x0)
        sweep = []
        n = max(1, w.n_owned // 256)
        while True:
            n = min(n, w.n_owned)
            k = int(row[n])
            sub = B.Graph(graph.src[:k], graph.dst[:k], graph.row_ptr[:n + 1], graph.shift[:3 * k], n, w.n_total)
            if not args.per_edge_rows:
                sub = m.egnn_edge_pairs(sub)       # (sources beyond the prefix count as halo atoms: no reverse edge)
            t_ms = timed(lambda: m.egnn_layer_forward(sub, pos, w.box, x_full, layers[0], ws, out=x_out[0][:n]), 10)
            sweep.append(dict(n_dst=n, n_edges=k, ms=t_ms, edges_per_s=k / t_ms * 1e3))
            if n == w.n_owned:
                break
            n *= 2

    ms_per_step = 1e3 * elapsed / args.steps
    value = n_edges * w.n_layers / (elapsed / args.steps)
    layer_ms = {n: ms[i] / max(1, n_calls[0]) for i, n in enumerate(B.LAYER_STAGES)}
    ro_ms = {n: ms[5 + i] / max(1, n_calls[1]) for i, n in enumerate(B.READOUT_STAGES)}

    s4_bytes, s3_bytes, s3_flops, s6_bytes = stage_model(w, n_edges, m.n_paths, m.n_paths_readout)
    # S3 processes one unit per row of the weight tensor: rows, not edges, when an edge and its reverse share a row
    s3_bytes, s3_flops = s3_bytes * n_rows / max(1, n_edges), s3_flops * n_rows / max(1, n_edges)
    s4_min, s6_min = compulsory_bytes(w, n_edges, m.n_paths, m.n_paths_readout)

    def hbm_roof(kernel, nbytes, avg_ms, calls_per_step, table_bytes=None, **extra):
        """achieved / frac: `nbytes` per launch over the launch time.  For S3 nbytes is the stage table's algorithmic
        figure (every byte of it goes to HBM).  For S4 / S6 it is the compulsory HBM traffic (each gathered node row
        once): the stage table counts a gathered row once per edge, which the caches serve, so its rate can exceed the
        HBM peak; it is reported beside, as a rate and a ratio, never as `frac`."""
        t = avg_ms * 1e-3
        traffic = read_traffic(kernel, w.name)
        d = dict(kernel=kernel, bound="hbm", achieved=nbytes / t / 1e9, peak=HBM_PEAK_GBS, unit="GB/s",
                 frac=nbytes / t / 1e9 / HBM_PEAK_GBS, traffic=traffic,
                 frac_traffic=(traffic / t / 1e9 / HBM_PEAK_GBS) if traffic else None, avg_ms=avg_ms,
                 bytes_per_launch=nbytes, launches_per_step=calls_per_step, ms_per_step=avg_ms * calls_per_step,
                 edges_per_s=n_edges / t)
        if table_bytes is not None:
            d["bytes_counted"] = "compulsory HBM traffic: weight rows, every node row once, indices, unit vectors, outputs"
            d["stage_table"] = dict(bytes_per_launch=table_bytes, GBs=table_bytes / t / 1e9,
                                    ratio_to_hbm_peak=table_bytes / t / 1e9 / HBM_PEAK_GBS,
                                    note="per-edge figure with one gathered row per edge; the caches serve most of "
                                         "those rows, so this is a work rate, not an HBM bandwidth fraction")
        else:
            d["bytes_counted"] = ("stage table's algorithmic bytes per unit (one weight row written, 16 bytes read) x the "
                              "rows one launch writes: one per edge, or one per unordered pair of owned atoms plus "
                              "one per halo edge when rows are shared (config.n_weight_rows)")
        d.update(extra)
        return d

    n_ro = 1 if w.readout else 0
    s3_ms = (layer_ms["radial_weights"] * n_calls[0] + ro_ms["radial_weights"] * n_calls[1]) / max(1, sum(n_calls))
    roofs = [hbm_roof("tp_segsum_kernel", s4_min, layer_ms["tp_segsum"], w.n_layers, table_bytes=s4_bytes),
             hbm_roof("radial_weights_kernel", s3_bytes, s3_ms, w.n_layers + n_ro,
                      mfma_TFLOPs=s3_flops / (s3_ms * 1e-3) / 1e12, mfma_peak_TFLOPs_f16=2500.0,
                      note="fp32-equivalent rate; the contraction runs on the f16 matrix cores with both operands "
                           "cut into two half-precision pieces (3 products per fp32 product, 3 x this rate in f16 work)")]
    if w.readout:
        roofs.append(hbm_roof("readout_kernel", s6_min, ro_ms["readout"], 1, table_bytes=s6_bytes))
    roofs.sort(key=lambda r: -r["ms_per_step"])
    dominant, other = roofs[0], roofs[1:]

    out = {
        "metric": "edges/sec per eGNN message-passing layer (fwd) + % of peak HBM GB/s on 1 GPU",
        "value": value, "unit": "edge-layer evaluations/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {index}: {w.name}", "n_atoms_owned": w.n_owned, "n_atoms_total": w.n_total,
                   "n_edges": n_edges, "n_weight_rows": n_rows, "lmax": w.lmax, "channels": w.channels, "n_rbf": w.n_rbf,
                   "n_layers": w.n_layers, "readout": bool(w.readout), "r_cut": w.r_cut,
                   "step": "nlist + species embed + %d layers fwd" % w.n_layers + (" + H_ij readout" if w.readout else
                           " (messages only into owned nodes; halo rows are read-only inputs; no readout in this configuration)")},
        "roofline": dominant, "roofline_others": other,
        "atom_order": "egnn_spatial_order (cubes of r_cut / 2 along a Morton curve)" if args.spatial_order else "as generated",
        "stage_ms": {"layer": layer_ms, "readout": ro_ms if w.readout else None,
                     "layer_total": sum(layer_ms.values()),
                     "layer_edges_per_s": n_edges / (sum(layer_ms.values()) * 1e-3)},
    }
    out["training_step"] = training
    out["w_fp16_storage"] = w_fp16
    if s4_half is not None:
        out["s4_half_precision_storage"] = s4_half
    out["s3_s4_fused_in_registers"] = fused_lane
    out["hbm_calibration"] = calibration
    if so2 is not None:
        out["so2_message_sum"] = so2
    if ham is not None:
        out["hamiltonian_assembly"] = ham
    if lownn is not None:
        out["low_nn_partition"] = lownn
    if sweep is not None:
        out["saturation_sweep"] = sweep
    del ws, x_out, H, x_full, m
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
