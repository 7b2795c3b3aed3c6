"""The message-passing layers under HIP graph capture: egnn_layer_forward enqueues kernels only (no copies, no memsets,
no host synchronisation), so a caller can record a stack of layers once and replay it.  Every replay is checked
against the eager result, with eager work and synchronisations between the replays and with new inputs written into
the recorded buffers."""
import numpy as np
import pytest

from paper_2507_03840_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2507_03840_amd import binding
    return binding


@pytest.mark.parametrize("fused", [0, "shared", 1, 2])
def test_layers_replay_from_a_graph(B, fused):
    """fused: 0 = S3 then S4, "shared" = the same on a graph with shared rows of radial weights, 1 / 2 = fused designs."""
    import torch
    w = synth.small_cluster(150, 110, 3, 32, 6, 4.0, 41, False, 0.05)
    w.n_layers = 2
    wt = U.model_weights(w)
    g = U.oracle_graph(w)
    agg = max(1.0, U.mean_degree(g, w.n_owned))
    m = B.Egnn(w.lmax, w.channels, w.n_rbf, w.r_cut, agg, n_layers=w.n_layers, orb_l=w.orb_l)
    shared = fused == "shared"
    fused = 0 if shared else fused
    m.egnn_set_option(B.OPT_FUSED, fused)
    pos = B.to_device(w.pos)
    graph = m.egnn_nlist(pos, w.n_owned, w.box, w.pbc)
    if shared:
        m.egnn_edge_pairs(graph)          # (before the capture: it reads the row count back)
    ws = m.workspace(graph)
    Wd = [B.to_device(wt["layers"][t]) for t in range(2)]
    halo1 = B.to_device(wt["halo"][1])
    x0 = B.to_device(wt["x0"])
    # recorded buffers
    x_in = x0.clone()
    x_mid = torch.empty((w.n_total, m.dim, w.channels), dtype=torch.float32, device="cuda")
    x_mid[w.n_owned:] = halo1
    y1 = x_mid[:w.n_owned]
    y2 = torch.empty((w.n_owned, m.dim, w.channels), dtype=torch.float32, device="cuda")

    def two_layers(xa, xm, out):
        m.egnn_layer_forward(graph, pos, w.box, xa, Wd[0], ws, out=xm[:w.n_owned])
        m.egnn_layer_forward(graph, pos, w.box, xm, Wd[1], ws, out=out)

    def eager(xa):
        xm = torch.empty_like(x_mid)
        xm[w.n_owned:] = halo1
        out = torch.empty_like(y2)
        two_layers(xa, xm, out)
        torch.cuda.synchronize()
        return xm[:w.n_owned].clone(), out

    ref1, ref2 = eager(x0)
    # (parity of the layers themselves is covered by test_gpu_parity.py; here replays are compared with eager runs)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up on the capture stream, as torch asks for
        two_layers(x_in, x_mid, y2)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    cg = torch.cuda.CUDAGraph()
    with torch.cuda.graph(cg, stream=side):
        two_layers(x_in, x_mid, y2)
    torch.cuda.synchronize()

    rng = np.random.default_rng(7)
    for rep in range(4):
        print("replay", rep, "fused", fused, flush=True)
        if rep >= 2:                       # new input in the recorded buffer
            x_new = B.to_device(rng.standard_normal(wt["x0"].shape).astype(np.float32))
            x_in.copy_(x_new)
            ref1, ref2 = eager(x_new)
        y2.zero_()
        x_mid[:w.n_owned].zero_()
        torch.cuda.synchronize()
        cg.replay()
        torch.cuda.synchronize()
        assert torch.equal(y1, ref1)
        assert torch.equal(y2, ref2)
