"""Thin ctypes binding of libegnn_hip.so: argument marshalling only, same names as include/egnn.h.

torch supplies device memory and the stream; every step of the path runs in the library's kernels.
There is no fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os
import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libegnn_hip.so")
MAX_SHELLS = 8
OPT_FUSED = 1
OPT_W_FP16 = 2
LENGTH_BINS = 2048
OPT_RADIAL_BWD = 3   # 0: route chosen on the device, 1: exact (matrix cores, two passes over dw), 2: grid of distances (one pass)

SYMBOLS = [
    "egnn_create", "egnn_destroy", "egnn_last_error", "egnn_path_count", "egnn_readout_widths",
    "egnn_workspace_bytes", "egnn_nlist_workspace_bytes", "egnn_nlist_count", "egnn_nlist_fill", "egnn_species_embed",
    "egnn_edge_geometry", "egnn_radial_weights", "egnn_tp_segsum", "egnn_node_mix",
    "egnn_layer_forward", "egnn_readout_hij", "egnn_timing_enable", "egnn_timing_read",
    "egnn_backward_workspace_bytes", "egnn_graph_transpose", "egnn_loss_mse", "egnn_layer_backward",
    "egnn_readout_backward", "egnn_set_option", "egnn_radial_weights_f16", "egnn_tp_segsum_f16", "egnn_tp_segsum_f16h", "egnn_so2_weight_count", "egnn_so2_workspace_bytes",
    "egnn_so2_message_sum", "egnn_so2_backward_workspace_bytes", "egnn_so2_message_sum_backward",
    "egnn_so2_blocks_backward_workspace_bytes", "egnn_so2_node_block_backward", "egnn_so2_edge_block_backward",
    "egnn_gate_backward_workspace_bytes", "egnn_gate_backward",
    "egnn_so2_blocks_workspace_bytes", "egnn_edge_embed_init", "egnn_so2_node_block",
    "egnn_so2_edge_block", "egnn_gate", "egnn_hamiltonian_workspace_bytes", "egnn_onsite_hii", "egnn_apply_padding", "egnn_loss_l1l2",
    "egnn_hamiltonian_structure", "egnn_hamiltonian_fill", "egnn_onsite_backward_workspace_bytes", "egnn_onsite_backward",
    "egnn_partition_low_nn", "egnn_spatial_order", "egnn_pack_rows", "egnn_unpack_rows",
    "egnn_layer_forward_save", "egnn_readout_hij_save", "egnn_layer_backward_saved", "egnn_readout_backward_saved",
    "egnn_radial_weights_static", "egnn_edge_pairs_workspace_bytes", "egnn_edge_pairs",
    "egnn_length_bins_workspace_bytes", "egnn_length_bins",
]


class ModelDesc(C.Structure):
    _fields_ = [("size", C.c_uint32), ("lmax", C.c_int32), ("lmax_sh", C.c_int32), ("channels", C.c_int32),
                ("n_rbf", C.c_int32), ("n_radial_hidden", C.c_int32), ("n_layers", C.c_int32),
                ("r_cut", C.c_float), ("agg_norm", C.c_float), ("n_orb_shells", C.c_int32),
                ("orb_l", C.c_int32 * MAX_SHELLS)]


class GraphDesc(C.Structure):
    _fields_ = [("src", C.c_void_p), ("dst", C.c_void_p), ("row_ptr", C.c_void_p), ("shift", C.c_void_p),
                ("n_edges", C.c_int64), ("n_owned", C.c_int32), ("n_total", C.c_int32),
                ("w_row", C.c_void_p), ("n_w_rows", C.c_int64), ("len_ptr", C.c_void_p), ("len_perm", C.c_void_p)]


class EgnnError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"egnn error {code}: {text}")
        self.code = code


_lib = None


def load_library():
    """Loads the built library; raises if it has not been built (python -m paper_2507_03840_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built; run `python -m paper_2507_03840_amd.build`")
        lib = C.CDLL(LIB_PATH)
        lib.egnn_last_error.restype = C.c_char_p
        lib.egnn_last_error.argtypes = [C.c_void_p]
        lib.egnn_destroy.restype = None
        lib.egnn_destroy.argtypes = [C.c_void_p]
        _lib = lib
    return _lib


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor required"
    return C.c_void_p(t.data_ptr())


def _f3(a):
    return (C.c_float * 3)(*[float(v) for v in a])


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Graph:
    """Device-resident edge list sorted by (dst, src) with its CSR index."""

    def __init__(self, src, dst, row_ptr, shift, n_owned, n_total):
        self.src, self.dst, self.row_ptr, self.shift = src, dst, row_ptr, shift
        self.n_edges, self.n_owned, self.n_total = int(src.numel()), int(n_owned), int(n_total)
        self.w_row, self.n_w_rows = None, 0      # set by Egnn.egnn_edge_pairs: shared rows of radial weights
        self.len_ptr, self.len_perm = None, None # set by Egnn.egnn_length_bins: edges grouped by length (reverse pass)

    def desc(self):
        return GraphDesc(_ptr(self.src).value, _ptr(self.dst).value, _ptr(self.row_ptr).value,
                         _ptr(self.shift).value if self.shift is not None else None,
                         self.n_edges, self.n_owned, self.n_total,
                         _ptr(self.w_row).value if self.w_row is not None else None, int(self.n_w_rows),
                         _ptr(self.len_ptr).value if self.len_ptr is not None else None,
                         _ptr(self.len_perm).value if self.len_perm is not None else None)

    def per_edge(self):
        """The same edge list without shared rows of radial weights."""
        g = Graph(self.src, self.dst, self.row_ptr, self.shift, self.n_owned, self.n_total)
        g.len_ptr, g.len_perm = self.len_ptr, self.len_perm
        return g

    @property
    def n_weight_rows(self):
        """Rows of the weight tensor the composite calls write for this graph."""
        return self.n_w_rows if self.w_row is not None else self.n_edges


LAYER_STAGES = ["geometry", "radial_weights", "mix_pre", "tp_segsum", "mix_post"]
READOUT_STAGES = ["geometry", "radial_weights", "mix_src", "mix_dst", "readout"]
LAYER_ADJOINT_STAGES = ["forward_quantities", "mix_post_adjoint", "tp_backward", "mix_pre_adjoint", "radial_backward"]
READOUT_ADJOINT_STAGES = ["forward_quantities", "readout_backward", "row_sums_and_mix_adjoints", "radial_backward"]


def egnn_spatial_order(pos, n_owned, cell):
    """Host call (numpy in, numpy out; no GPU needed): perm [n_total] with perm[new index] = old index."""
    lib = load_library()
    pos = np.ascontiguousarray(pos, np.float32)
    perm = np.zeros(pos.shape[0], np.int32)
    lib.egnn_spatial_order.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p]
    rc = lib.egnn_spatial_order(pos.ctypes.data, int(n_owned), pos.shape[0], float(cell), perm.ctypes.data)
    if rc:
        raise EgnnError(rc, "egnn_spatial_order: bad argument")
    return perm


def egnn_partition_low_nn(pos, degree, box, pbc, r_cut, levels):
    """Host call (numpy in, numpy out; no GPU needed): returns (part [n], cut_log [n_cuts][4])."""
    lib = load_library()
    pos = np.ascontiguousarray(pos, np.float32)
    degree = np.ascontiguousarray(degree, np.int32)
    n = pos.shape[0]
    part = np.full(n, -1, np.int32)
    log = np.zeros((max(1, (1 << levels) - 1), 4), np.int32)
    n_cuts = C.c_int32()
    pbc3 = (C.c_uint8 * 3)(*[int(v) for v in pbc])
    lib.egnn_partition_low_nn.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_double,
                                          C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    rc = lib.egnn_partition_low_nn(pos.ctypes.data, degree.ctypes.data, n, _f3(box), pbc3, float(r_cut), int(levels),
                                   part.ctypes.data, log.ctypes.data, C.byref(n_cuts))
    if rc:
        raise EgnnError(rc, "egnn_partition_low_nn: bad argument")
    return part, log[:min(n_cuts.value, log.shape[0])]


class Egnn:
    """One model context (egnn_ctx) plus the calls of the C ABI."""

    def __init__(self, lmax, channels, n_rbf, r_cut, agg_norm, n_layers=1, orb_l=(0, 0, 1, 1, 2), lmax_sh=None,
                 n_radial_hidden=64):
        self.lib = load_library()
        d = ModelDesc()
        d.size = C.sizeof(ModelDesc)
        d.lmax, d.lmax_sh = lmax, lmax if lmax_sh is None else lmax_sh
        d.channels, d.n_rbf, d.n_radial_hidden, d.n_layers = channels, n_rbf, n_radial_hidden, n_layers
        d.r_cut, d.agg_norm = r_cut, agg_norm
        d.n_orb_shells = len(orb_l)
        for i, l in enumerate(orb_l):
            d.orb_l[i] = l
        self.desc = d
        self.ctx = C.c_void_p()
        rc = self.lib.egnn_create(C.byref(d), C.byref(self.ctx))
        if rc:
            raise EgnnError(rc, self.lib.egnn_last_error(None).decode())
        self.lmax, self.channels, self.n_rbf = lmax, channels, n_rbf
        self.dim = (lmax + 1) ** 2
        self.n_orb = sum(2 * l + 1 for l in orb_l)
        self.n_paths, self.paths = self.egnn_path_count(0)
        self.n_paths_readout, self.paths_readout = self.egnn_path_count(1)
        self.n_out = self.egnn_readout_widths()

    def __del__(self):
        ctx = getattr(self, "ctx", None)
        if ctx is not None and ctx.value:
            self.lib.egnn_destroy(ctx)
            self.ctx = None

    def _check(self, rc):
        if rc:
            raise EgnnError(rc, self.lib.egnn_last_error(self.ctx).decode())

    def egnn_set_option(self, option, value):
        self._check(self.lib.egnn_set_option(self.ctx, int(option), int(value)))

    # ---- queries
    def egnn_path_count(self, which):
        n = C.c_int32()
        self._check(self.lib.egnn_path_count(self.ctx, which, C.byref(n), None))
        buf = (C.c_int32 * (3 * n.value))()
        self._check(self.lib.egnn_path_count(self.ctx, which, C.byref(n), buf))
        return n.value, [tuple(buf[3 * p:3 * p + 3]) for p in range(n.value)]

    def egnn_readout_widths(self):
        buf = (C.c_int32 * 5)()
        self._check(self.lib.egnn_readout_widths(self.ctx, buf))
        return list(buf)

    def egnn_workspace_bytes(self, n_edges, n_owned, n_total, with_weights=True):
        out = C.c_size_t()
        self._check(self.lib.egnn_workspace_bytes(self.ctx, C.c_int64(n_edges), n_owned, n_total,
                                                  1 if with_weights else 0, C.byref(out)))
        return out.value

    def workspace(self, graph, with_weights=True):
        nbytes = self.egnn_workspace_bytes(graph.n_edges, graph.n_owned, graph.n_total, with_weights)
        return torch.empty(nbytes, dtype=torch.uint8, device="cuda")

    # ---- S1
    def egnn_nlist_workspace_bytes(self, n_total):
        out = C.c_size_t()
        self._check(self.lib.egnn_nlist_workspace_bytes(self.ctx, int(n_total), C.byref(out)))
        return out.value

    def egnn_nlist(self, pos, n_owned, box, pbc, with_shift=True, cell_list=True):
        """count + allocate + fill; returns a Graph.  cell_list=False: every destination sweeps all atoms."""
        n_total = pos.shape[0]
        pbc_c = (C.c_uint8 * 3)(*[int(v) for v in pbc])
        row_ptr = torch.empty(n_owned + 1, dtype=torch.int32, device="cuda")
        n_edges = C.c_int64()
        ws = torch.empty(self.egnn_nlist_workspace_bytes(n_total), dtype=torch.uint8, device="cuda") if cell_list else None
        ws_n = C.c_size_t(ws.numel() if ws is not None else 0)
        self._check(self.lib.egnn_nlist_count(self.ctx, _ptr(pos), n_owned, n_total, _f3(box), pbc_c, _ptr(row_ptr),
                                              C.byref(n_edges), _ptr(ws), ws_n, _stream()))
        n = n_edges.value
        src = torch.empty(n, dtype=torch.int32, device="cuda")
        dst = torch.empty(n, dtype=torch.int32, device="cuda")
        shift = torch.empty((n, 3), dtype=torch.int8, device="cuda") if with_shift else None
        self._check(self.lib.egnn_nlist_fill(self.ctx, _ptr(pos), n_owned, n_total, _f3(box), pbc_c, _ptr(row_ptr),
                                             C.c_int64(n), _ptr(src), _ptr(dst), _ptr(shift), _ptr(ws), ws_n, _stream()))
        return Graph(src, dst, row_ptr, shift, n_owned, n_total)

    def egnn_edge_pairs(self, graph):
        """Sets graph.w_row / graph.n_w_rows (one row of radial weights per unordered pair of owned atoms)."""
        out = C.c_size_t()
        self._check(self.lib.egnn_edge_pairs_workspace_bytes(self.ctx, graph.n_owned, C.byref(out)))
        ws = torch.empty(max(256, out.value), dtype=torch.uint8, device="cuda")
        w_row = torch.empty(graph.n_edges, dtype=torch.int32, device="cuda")
        n_rows = C.c_int64()
        g = graph.per_edge().desc()
        self._check(self.lib.egnn_edge_pairs(self.ctx, C.byref(g), _ptr(w_row), C.byref(n_rows), _ptr(ws),
                                             C.c_size_t(ws.numel()), _stream()))
        graph.w_row, graph.n_w_rows = w_row, n_rows.value
        return graph

    def egnn_length_bins(self, graph, pos, box):
        """Sets graph.len_ptr / graph.len_perm (edges grouped by length interval, for the reverse pass)."""
        out = C.c_size_t()
        self._check(self.lib.egnn_length_bins_workspace_bytes(self.ctx, C.c_int64(graph.n_edges), C.byref(out)))
        ws = torch.empty(max(256, out.value), dtype=torch.uint8, device="cuda")
        len_ptr = torch.empty(LENGTH_BINS + 1, dtype=torch.int32, device="cuda")
        len_perm = torch.empty(graph.n_edges, dtype=torch.int32, device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_length_bins(self.ctx, C.byref(g), _ptr(pos), _f3(box), _ptr(len_ptr), _ptr(len_perm),
                                              _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        graph.len_ptr, graph.len_perm = len_ptr, len_perm
        return graph

    # ---- node init
    def egnn_species_embed(self, species, table, x):
        self._check(self.lib.egnn_species_embed(self.ctx, _ptr(species), _ptr(table), table.shape[0], _ptr(x),
                                                x.shape[0], _stream()))

    # ---- S2
    def egnn_edge_geometry(self, graph, pos, box, want_Y=False, want_rbf=False, want_fc=False):
        n = graph.n_edges
        rhat_d = torch.empty((n, 4), dtype=torch.float32, device="cuda")
        Y = torch.empty((n, self.dim), dtype=torch.float32, device="cuda") if want_Y else None
        rbf = torch.empty((n, self.n_rbf), dtype=torch.float32, device="cuda") if want_rbf else None
        fc = torch.empty(n, dtype=torch.float32, device="cuda") if want_fc else None
        g = graph.desc()
        self._check(self.lib.egnn_edge_geometry(self.ctx, C.byref(g), _ptr(pos), _f3(box), _ptr(rhat_d), _ptr(Y),
                                                _ptr(rbf), _ptr(fc), _stream()))
        return rhat_d, Y, rbf, fc

    # ---- S3
    def egnn_radial_weights(self, which, rhat_d, W_r1, W_r2, out=None):
        n = rhat_d.shape[0]
        P = self.n_paths if which == 0 else self.n_paths_readout
        w = out if out is not None else torch.empty((n, P, self.channels), dtype=torch.float32, device="cuda")
        ws = torch.empty(384 * P * self.channels, dtype=torch.uint8, device="cuda")
        self._check(self.lib.egnn_radial_weights(self.ctx, which, _ptr(rhat_d), C.c_int64(n), _ptr(W_r1), _ptr(W_r2),
                                                 _ptr(w), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return w

    def egnn_radial_weights_static(self, which, rhat_d, W_r1, W_r2, out):
        """The same weights through the entry point that allocates nothing: `out` must be preallocated."""
        n = rhat_d.shape[0]
        self._check(self.lib.egnn_radial_weights_static(self.ctx, which, _ptr(rhat_d), C.c_int64(n), _ptr(W_r1),
                                                        _ptr(W_r2), _ptr(out), _stream()))
        return out

    def egnn_radial_weights_f16(self, which, rhat_d, W_r1, W_r2):
        """Half-precision weights, packed: int32 tensor [n_edges][32 * ceil(P * channels / 64)]."""
        n = rhat_d.shape[0]
        P = self.n_paths if which == 0 else self.n_paths_readout
        w16 = torch.empty((n, 32 * ((P * self.channels + 63) // 64)), dtype=torch.int32, device="cuda")
        ws = torch.empty(384 * P * self.channels, dtype=torch.uint8, device="cuda")
        self._check(self.lib.egnn_radial_weights_f16(self.ctx, which, _ptr(rhat_d), C.c_int64(n), _ptr(W_r1),
                                                     _ptr(W_r2), _ptr(w16), _ptr(ws), C.c_size_t(ws.numel()),
                                                     _stream()))
        return w16

    def egnn_tp_segsum_f16(self, graph, rhat_d, h, w16, out=None):
        a = out if out is not None else torch.empty((graph.n_owned, self.dim, self.channels), dtype=torch.float32,
                                                    device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_tp_segsum_f16(self.ctx, C.byref(g), _ptr(rhat_d), _ptr(h), _ptr(w16), _ptr(a),
                                                _stream()))
        return a

    def egnn_tp_segsum_f16h(self, graph, rhat_d, h16, w16, out=None):
        """h16: torch.float16 tensor [n_total][dim][channels]."""
        a = out if out is not None else torch.empty((graph.n_owned, self.dim, self.channels), dtype=torch.float32,
                                                    device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_tp_segsum_f16h(self.ctx, C.byref(g), _ptr(rhat_d), _ptr(h16), _ptr(w16), _ptr(a),
                                                 _stream()))
        return a

    # ---- S4
    def egnn_tp_segsum(self, graph, rhat_d, h, w, out=None):
        a = out if out is not None else torch.empty((graph.n_owned, self.dim, self.channels), dtype=torch.float32,
                                                    device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_tp_segsum(self.ctx, C.byref(g), _ptr(rhat_d), _ptr(h), _ptr(w), _ptr(a), _stream()))
        return a

    # ---- S5
    def egnn_node_mix(self, x1, W1, x2=None, W2=None, out=None):
        y = out if out is not None else torch.empty_like(x1)
        self._check(self.lib.egnn_node_mix(self.ctx, _ptr(x1), _ptr(W1), _ptr(x2), _ptr(W2), _ptr(y), x1.shape[0],
                                           _stream()))
        return y

    # ---- SO(2) form of the message transform
    def egnn_so2_weight_count(self):
        out = C.c_int64()
        self._check(self.lib.egnn_so2_weight_count(self.ctx, C.byref(out)))
        return out.value

    def egnn_so2_workspace_bytes(self, n_edges):
        out = C.c_size_t()
        self._check(self.lib.egnn_so2_workspace_bytes(self.ctx, C.c_int64(n_edges), C.byref(out)))
        return out.value

    def egnn_so2_message_sum(self, graph, pos, box, x, W_e, W_so2, ws, out=None):
        a = out if out is not None else torch.empty((graph.n_owned, self.dim, self.channels), dtype=torch.float32,
                                                    device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_so2_message_sum(self.ctx, C.byref(g), _ptr(pos), _f3(box), _ptr(x), _ptr(W_e),
                                                  _ptr(W_so2), _ptr(a), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return a

    def egnn_so2_backward_workspace_bytes(self, n_edges, n_owned):
        out = C.c_size_t()
        self._check(self.lib.egnn_so2_backward_workspace_bytes(self.ctx, C.c_int64(n_edges), C.c_int32(n_owned),
                                                               C.byref(out)))
        return out.value

    def egnn_so2_message_sum_backward(self, graph, col_ptr, perm, pos, box, x, W_e, W_so2, da, ws):
        """(dx [n_total][dim][channels], dW_e, dW_so2) from da [n_owned][dim][channels]."""
        dx = torch.empty((graph.n_total, self.dim, self.channels), dtype=torch.float32, device="cuda")
        dW_e, dW_so2 = torch.empty_like(W_e), torch.empty_like(W_so2)
        g = graph.desc()
        self._check(self.lib.egnn_so2_message_sum_backward(
            self.ctx, C.byref(g), _ptr(col_ptr), _ptr(perm), _ptr(pos), _f3(box), _ptr(x), _ptr(W_e), _ptr(W_so2),
            _ptr(da), _ptr(dx), _ptr(dW_e), _ptr(dW_so2), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return dx, dW_e, dW_so2

    def egnn_so2_blocks_backward_workspace_bytes(self, n_edges, n_owned):
        out = C.c_size_t()
        self._check(self.lib.egnn_so2_blocks_backward_workspace_bytes(self.ctx, C.c_int64(n_edges), C.c_int32(n_owned),
                                                                      C.byref(out)))
        return out.value

    def egnn_so2_node_block_backward(self, graph, col_ptr, perm, pos, box, x, T_edge, W_so2, w_att, da, ws):
        """(dx, dT_edge, dW_so2, dw_att) from da [n_owned][dim][channels]."""
        dx = torch.empty((graph.n_total, self.dim, self.channels), dtype=torch.float32, device="cuda")
        dT, dW, dw_att = torch.empty_like(T_edge), torch.empty_like(W_so2), torch.empty_like(w_att)
        g = graph.desc()
        self._check(self.lib.egnn_so2_node_block_backward(
            self.ctx, C.byref(g), _ptr(col_ptr), _ptr(perm), _ptr(pos), _f3(box), _ptr(x), _ptr(T_edge), _ptr(W_so2),
            _ptr(w_att), _ptr(da), _ptr(dx), _ptr(dT), _ptr(dW), _ptr(dw_att), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return dx, dT, dW, dw_att

    def egnn_so2_edge_block_backward(self, graph, col_ptr, perm, pos, box, x, T_edge_in, W_so2, dT_out, ws, dT_in=None):
        """(dx, dT_in, dW_so2) from dT_out [n_edges][dim][channels]; dT_in may be dT_out itself."""
        dx = torch.empty((graph.n_total, self.dim, self.channels), dtype=torch.float32, device="cuda")
        dT = dT_in if dT_in is not None else torch.empty_like(dT_out)
        dW = torch.empty_like(W_so2)
        g = graph.desc()
        self._check(self.lib.egnn_so2_edge_block_backward(
            self.ctx, C.byref(g), _ptr(col_ptr), _ptr(perm), _ptr(pos), _f3(box), _ptr(x), _ptr(T_edge_in), _ptr(W_so2),
            _ptr(dT_out), _ptr(dx), _ptr(dT), _ptr(dW), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return dx, dT, dW

    def egnn_gate_backward(self, x, W_g, dy):
        """(dx, dW_g) of the gate."""
        out = C.c_size_t()
        self._check(self.lib.egnn_gate_backward_workspace_bytes(self.ctx, C.c_int32(x.shape[0]), C.byref(out)))
        ws = torch.empty(out.value, dtype=torch.uint8, device="cuda")
        dx, dW = torch.empty_like(x), torch.empty_like(W_g)
        self._check(self.lib.egnn_gate_backward(self.ctx, _ptr(x), _ptr(W_g), _ptr(dy), _ptr(dx), _ptr(dW),
                                                C.c_int32(x.shape[0]), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return dx, dW

    def egnn_so2_blocks_workspace_bytes(self, n_edges):
        out = C.c_size_t()
        self._check(self.lib.egnn_so2_blocks_workspace_bytes(self.ctx, C.c_int64(n_edges), C.byref(out)))
        return out.value

    def egnn_edge_embed_init(self, graph, pos, box, W_e, ws, out=None):
        T = out if out is not None else torch.empty((graph.n_edges, self.dim, self.channels), dtype=torch.float32,
                                                    device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_edge_embed_init(self.ctx, C.byref(g), _ptr(pos), _f3(box), _ptr(W_e), _ptr(T), _ptr(ws),
                                                  C.c_size_t(ws.numel()), _stream()))
        return T

    def egnn_so2_node_block(self, graph, pos, box, x, T_edge, W_so2, w_att, ws, out=None):
        a = out if out is not None else torch.empty((graph.n_owned, self.dim, self.channels), dtype=torch.float32,
                                                    device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_so2_node_block(self.ctx, C.byref(g), _ptr(pos), _f3(box), _ptr(x), _ptr(T_edge),
                                                 _ptr(W_so2), _ptr(w_att), _ptr(a), _ptr(ws), C.c_size_t(ws.numel()),
                                                 _stream()))
        return a

    def egnn_so2_edge_block(self, graph, pos, box, x, T_edge, W_so2, ws, out=None):
        T = out if out is not None else torch.empty_like(T_edge)
        g = graph.desc()
        self._check(self.lib.egnn_so2_edge_block(self.ctx, C.byref(g), _ptr(pos), _f3(box), _ptr(x), _ptr(T_edge),
                                                 _ptr(W_so2), _ptr(T), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return T

    def egnn_gate(self, x, W_g, out=None):
        y = out if out is not None else torch.empty_like(x)
        self._check(self.lib.egnn_gate(self.ctx, _ptr(x), _ptr(W_g), _ptr(y), x.shape[0], _stream()))
        return y

    # ---- layer / readout
    def egnn_layer_forward(self, graph, pos, box, x_in, W, ws, w_edge=None, out=None):
        x_out = out if out is not None else torch.empty((graph.n_owned, self.dim, self.channels),
                                                        dtype=torch.float32, device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_layer_forward(
            self.ctx, C.byref(g), _ptr(pos), _f3(box), _ptr(x_in), _ptr(W["W_pre"]), _ptr(W["W_post"]),
            _ptr(W["W_self"]), _ptr(W.get("W_r1")), _ptr(W.get("W_r2")), _ptr(w_edge), _ptr(x_out), _ptr(ws),
            C.c_size_t(ws.numel()), _stream()))
        return x_out

    def egnn_readout_hij(self, graph, pos, box, x, W, ws, out=None):
        H = out if out is not None else torch.empty((graph.n_edges, self.n_orb, self.n_orb), dtype=torch.float32,
                                                    device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_readout_hij(
            self.ctx, C.byref(g), _ptr(pos), _f3(box), _ptr(x), _ptr(W["W_s"]), _ptr(W["W_t"]), _ptr(W["W_r1"]),
            _ptr(W["W_r2"]), _ptr(W["V"]), _ptr(H), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return H


    # ---- halo rows
    def egnn_pack_rows(self, x, idx, half=False):
        out = torch.empty((idx.numel(),) + tuple(x.shape[1:]), dtype=torch.float16 if half else torch.float32,
                          device="cuda")
        self._check(self.lib.egnn_pack_rows(self.ctx, _ptr(x), x.shape[0], _ptr(idx), idx.numel(), int(half), _ptr(out),
                                            _stream()))
        return out

    def egnn_unpack_rows(self, buf, x_full, first_row):
        self._check(self.lib.egnn_unpack_rows(self.ctx, _ptr(buf), buf.shape[0], int(buf.dtype == torch.float16),
                                              _ptr(x_full), int(first_row), _stream()))
        return x_full

    # ---- assembly of the predicted Hamiltonian
    def egnn_hamiltonian_workspace_bytes(self, n_edges, n_owned, n_total):
        ws, plan = C.c_size_t(), C.c_size_t()
        self._check(self.lib.egnn_hamiltonian_workspace_bytes(self.ctx, C.c_int64(n_edges), n_owned, n_total,
                                                              C.byref(ws), C.byref(plan)))
        return ws.value, plan.value

    def hamiltonian_workspace(self, graph):
        ws, plan = self.egnn_hamiltonian_workspace_bytes(graph.n_edges, graph.n_owned, graph.n_total)
        return (torch.empty(ws, dtype=torch.uint8, device="cuda"), torch.empty(plan, dtype=torch.uint8, device="cuda"))

    def egnn_onsite_hii(self, x, V_node, ws, out=None):
        n = x.shape[0]
        H = out if out is not None else torch.empty((n, self.n_orb, self.n_orb), dtype=torch.float32, device="cuda")
        self._check(self.lib.egnn_onsite_hii(self.ctx, _ptr(x), _ptr(V_node), _ptr(H), n, _ptr(ws),
                                             C.c_size_t(ws.numel()), _stream()))
        return H

    def egnn_onsite_backward(self, x, V_node, dH):
        n = x.shape[0]
        nb = C.c_size_t()
        self._check(self.lib.egnn_onsite_backward_workspace_bytes(self.ctx, n, C.byref(nb)))
        ws = torch.empty(nb.value, dtype=torch.uint8, device="cuda")
        dx, dV = torch.empty_like(x), torch.empty_like(V_node)
        self._check(self.lib.egnn_onsite_backward(self.ctx, _ptr(x), _ptr(V_node), _ptr(dH), _ptr(dx), _ptr(dV), n,
                                                  _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return dx, dV

    def egnn_apply_padding(self, H, row_atom, col_atom, species, orb_bits):
        self._check(self.lib.egnn_apply_padding(self.ctx, _ptr(H), C.c_int64(H.shape[0]), _ptr(row_atom), _ptr(col_atom),
                                                _ptr(species), _ptr(orb_bits), int(orb_bits.numel()), _stream()))
        return H

    def egnn_loss_l1l2(self, H, T, row_atom, col_atom, species, orb_bits, ws, want_grad=True):
        """Returns (loss [3]: total, L1 term, L2 term; device), dH or None."""
        loss = torch.empty(3, dtype=torch.float32, device="cuda")
        dH = torch.empty_like(H) if want_grad else None
        self._check(self.lib.egnn_loss_l1l2(self.ctx, _ptr(H), _ptr(T), C.c_int64(H.shape[0]), _ptr(row_atom),
                                            _ptr(col_atom), _ptr(species), _ptr(orb_bits), int(orb_bits.numel()),
                                            _ptr(loss), _ptr(dH), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return loss, dH

    def egnn_hamiltonian_structure(self, graph, species, orb_bits, plan):
        """Returns (orb_off [n_total+1] int32, col_ptr [n_cols+1] int64, nnz)."""
        orb_off = torch.empty(graph.n_total + 1, dtype=torch.int32, device="cuda")
        col_ptr = torch.empty(graph.n_owned * self.n_orb + 1, dtype=torch.int64, device="cuda")
        n_cols, nnz = C.c_int64(), C.c_int64()
        g = graph.desc()
        self._check(self.lib.egnn_hamiltonian_structure(self.ctx, C.byref(g), _ptr(species), _ptr(orb_bits),
                                                        int(orb_bits.numel()), _ptr(orb_off), _ptr(col_ptr), _ptr(plan),
                                                        C.c_size_t(plan.numel()), C.byref(n_cols), C.byref(nnz),
                                                        _stream()))
        return orb_off, col_ptr[:n_cols.value + 1], nnz.value

    def egnn_hamiltonian_fill(self, graph, species, orb_bits, orb_off, plan, H_edge, H_node, nnz, want_rows=True,
                              values=None, row_idx=None):
        if values is None:
            values = torch.empty(nnz, dtype=torch.float32, device="cuda")
        if row_idx is None and want_rows:
            row_idx = torch.empty(nnz, dtype=torch.int32, device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_hamiltonian_fill(self.ctx, C.byref(g), _ptr(species), _ptr(orb_bits),
                                                   int(orb_bits.numel()), _ptr(orb_off), _ptr(plan),
                                                   C.c_size_t(plan.numel()), _ptr(H_edge), _ptr(H_node), _ptr(row_idx),
                                                   _ptr(values), _stream()))
        return row_idx, values

    # ---- forward calls that leave w (and a) with the caller, reverse calls that take them back
    def egnn_layer_forward_save(self, graph, pos, box, x_in, W, ws, out=None):
        """Returns (x_out, saved) with saved = (w [rows][P][E], a [n_owned][dim][E]); rows = n_edges, or the
        graph's n_w_rows when it carries shared rows."""
        x_out = out if out is not None else torch.empty((graph.n_owned, self.dim, self.channels),
                                                        dtype=torch.float32, device="cuda")
        w = torch.empty((graph.n_weight_rows, self.n_paths, self.channels), dtype=torch.float32, device="cuda")
        a = torch.empty((graph.n_owned, self.dim, self.channels), dtype=torch.float32, device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_layer_forward_save(
            self.ctx, C.byref(g), _ptr(pos), _f3(box), _ptr(x_in), _ptr(W["W_pre"]), _ptr(W["W_post"]),
            _ptr(W["W_self"]), _ptr(W["W_r1"]), _ptr(W["W_r2"]), _ptr(x_out), _ptr(w), _ptr(a), _ptr(ws),
            C.c_size_t(ws.numel()), _stream()))
        return x_out, (w, a)

    def egnn_readout_hij_save(self, graph, pos, box, x, W, ws, out=None):
        H = out if out is not None else torch.empty((graph.n_edges, self.n_orb, self.n_orb), dtype=torch.float32,
                                                    device="cuda")
        w = torch.empty((graph.n_weight_rows, self.n_paths_readout, self.channels), dtype=torch.float32, device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_readout_hij_save(
            self.ctx, C.byref(g), _ptr(pos), _f3(box), _ptr(x), _ptr(W["W_s"]), _ptr(W["W_t"]), _ptr(W["W_r1"]),
            _ptr(W["W_r2"]), _ptr(W["V"]), _ptr(H), _ptr(w), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return H, w

    def egnn_layer_backward_saved(self, graph, col_ptr, perm, pos, box, x_in, W, saved, dx_out, ws):
        w, a = saved
        dx_in = torch.empty((graph.n_total, self.dim, self.channels), dtype=torch.float32, device="cuda")
        grads = {k: torch.empty_like(W[k]) for k in ("W_pre", "W_post", "W_self", "W_r1", "W_r2")}
        g = graph.desc()
        self._check(self.lib.egnn_layer_backward_saved(
            self.ctx, C.byref(g), _ptr(col_ptr), _ptr(perm), _ptr(pos), _f3(box), _ptr(x_in), _ptr(W["W_pre"]),
            _ptr(W["W_post"]), _ptr(W["W_self"]), _ptr(W["W_r1"]), _ptr(W["W_r2"]), _ptr(w), _ptr(a), _ptr(dx_out),
            _ptr(dx_in), _ptr(grads["W_pre"]), _ptr(grads["W_post"]), _ptr(grads["W_self"]), _ptr(grads["W_r1"]),
            _ptr(grads["W_r2"]), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return dx_in, grads

    def egnn_readout_backward_saved(self, graph, col_ptr, perm, pos, box, x, W, w_saved, dH, ws):
        dx = torch.empty((graph.n_total, self.dim, self.channels), dtype=torch.float32, device="cuda")
        grads = {k: torch.empty_like(W[k]) for k in ("W_s", "W_t", "W_r1", "W_r2", "V")}
        g = graph.desc()
        self._check(self.lib.egnn_readout_backward_saved(
            self.ctx, C.byref(g), _ptr(col_ptr), _ptr(perm), _ptr(pos), _f3(box), _ptr(x), _ptr(W["W_s"]),
            _ptr(W["W_t"]), _ptr(W["W_r1"]), _ptr(W["W_r2"]), _ptr(W["V"]), _ptr(w_saved), _ptr(dH), _ptr(dx),
            _ptr(grads["W_s"]), _ptr(grads["W_t"]), _ptr(grads["W_r1"]), _ptr(grads["W_r2"]), _ptr(grads["V"]), _ptr(ws),
            C.c_size_t(ws.numel()), _stream()))
        return dx, grads

    # ---- S7: loss and reverse pass
    def egnn_backward_workspace_bytes(self, n_edges, n_owned, n_total):
        out = C.c_size_t()
        self._check(self.lib.egnn_backward_workspace_bytes(self.ctx, C.c_int64(n_edges), n_owned, n_total,
                                                           C.byref(out)))
        return out.value

    def backward_workspace(self, graph):
        nbytes = self.egnn_backward_workspace_bytes(graph.n_edges, graph.n_owned, graph.n_total)
        return torch.empty(nbytes, dtype=torch.uint8, device="cuda")

    def egnn_graph_transpose(self, graph, ws):
        col_ptr = torch.empty(graph.n_total + 1, dtype=torch.int32, device="cuda")
        perm = torch.empty(graph.n_edges, dtype=torch.int32, device="cuda")
        g = graph.desc()
        self._check(self.lib.egnn_graph_transpose(self.ctx, C.byref(g), _ptr(col_ptr), _ptr(perm), _ptr(ws),
                                                  C.c_size_t(ws.numel()), _stream()))
        return col_ptr, perm

    def egnn_loss_mse(self, H, T, ws, want_grad=True):
        loss = torch.empty(1, dtype=torch.float32, device="cuda")
        dH = torch.empty_like(H) if want_grad else None
        self._check(self.lib.egnn_loss_mse(self.ctx, _ptr(H), _ptr(T), C.c_int64(H.numel()), _ptr(loss), _ptr(dH),
                                           _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return loss, dH

    def egnn_layer_backward(self, graph, col_ptr, perm, pos, box, x_in, W, dx_out, ws):
        dx_in = torch.empty((graph.n_total, self.dim, self.channels), dtype=torch.float32, device="cuda")
        grads = {k: torch.empty_like(W[k]) for k in ("W_pre", "W_post", "W_self", "W_r1", "W_r2")}
        g = graph.desc()
        self._check(self.lib.egnn_layer_backward(
            self.ctx, C.byref(g), _ptr(col_ptr), _ptr(perm), _ptr(pos), _f3(box), _ptr(x_in), _ptr(W["W_pre"]),
            _ptr(W["W_post"]), _ptr(W["W_self"]), _ptr(W["W_r1"]), _ptr(W["W_r2"]), _ptr(dx_out), _ptr(dx_in),
            _ptr(grads["W_pre"]), _ptr(grads["W_post"]), _ptr(grads["W_self"]), _ptr(grads["W_r1"]),
            _ptr(grads["W_r2"]), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
        return dx_in, grads

    def egnn_readout_backward(self, graph, col_ptr, perm, pos, box, x, W, dH, ws):
        dx = torch.empty((graph.n_total, self.dim, self.channels), dtype=torch.float32, device="cuda")
        grads = {k: torch.empty_like(W[k]) for k in ("W_s", "W_t", "W_r1", "W_r2", "V")}
        g = graph.desc()
        self._check(self.lib.egnn_readout_backward(
            self.ctx, C.byref(g), _ptr(col_ptr), _ptr(perm), _ptr(pos), _f3(box), _ptr(x), _ptr(W["W_s"]),
            _ptr(W["W_t"]), _ptr(W["W_r1"]), _ptr(W["W_r2"]), _ptr(W["V"]), _ptr(dH), _ptr(dx), _ptr(grads["W_s"]),
            _ptr(grads["W_t"]), _ptr(grads["W_r1"]), _ptr(grads["W_r2"]), _ptr(grads["V"]), _ptr(ws),
            C.c_size_t(ws.numel()), _stream()))
        return dx, grads

    # ---- stage timing
    def egnn_timing_enable(self, max_calls):
        self._check(self.lib.egnn_timing_enable(self.ctx, int(max_calls)))

    def egnn_timing_read(self):
        ms = (C.c_float * 20)()
        n = (C.c_int32 * 4)()
        self._check(self.lib.egnn_timing_read(self.ctx, ms, n))
        return list(ms), list(n)


def to_device(d):
    """numpy array / dict of arrays -> contiguous device tensors."""
    if isinstance(d, dict):
        return {k: to_device(v) for k, v in d.items()}
    return torch.from_numpy(np.ascontiguousarray(d)).cuda()
