/*
 * egnn.h -- C ABI of the MI355X (gfx950) hot path of the equivariant message-passing network of
 * arXiv 2507.03840 ("Distributed Equivariant Graph Neural Networks for Large-Scale Electronic
 * Structure Prediction"): radius graph -> per-edge equivariant messages -> sums over incoming
 * edges -> per-degree channel mixes -> orbital blocks H_ij.
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer unless its comment says "host".  The caller owns every
 *     buffer, including the workspace; the library allocates no device memory, keeps no pointer
 *     after a call returns, and enqueues all work on the stream passed in (a hipStream_t, passed
 *     as void*; NULL = the default stream).  egnn_nlist_count (edge count read-back) and
 *     egnn_hamiltonian_structure (size read-back) synchronise the stream; nothing else does.  The readout and
 *     on-site calls upload small index tables from memory owned by the context; egnn_destroy therefore waits for
 *     the device if such a call has been made.
 *   - Node tensors: float [n_nodes][(lmax+1)^2][channels], channel fastest; the (l, m) axis is
 *     flattened as l*l + l + m, m = -l..l  (Sec. 3 "Initialization": T^node of shape
 *     (l_max+1)^2 x E per atom).
 *   - Real spherical harmonics: z polar axis; m > 0 ~ cos(m phi), m < 0 ~ sin(|m| phi); no
 *     Condon-Shortley sign in the real form; component normalisation (sum_m Y_lm^2 = 2l+1).
 *   - Coupling paths P(l_in, l_sh, l_out): all (l1, l2, l3) with l1 <= l_in, l2 <= l_sh,
 *     |l1-l2| <= l3 <= min(l1+l2, l_out), l1+l2+l3 even, in lexicographic order; the path index p
 *     is the position in that list.  Real coupling tensors are the real (even l1+l2+l3) or imaginary
 *     (odd) part of the Condon-Shortley Clebsch-Gordan coefficients of Eq. 1 in the real basis.
 *   - Edge k = (src i -> dst j); its vector is r_k = pos[i] + shift_k * box - pos[j].  Edges are
 *     sorted by (dst, src); row_ptr[j] .. row_ptr[j+1] are the edges into owned node j
 *     ("incoming edge" ownership, Sec. 3 "Distribution").  Owned nodes are rows 0 .. n_owned-1,
 *     halo nodes (read-only sources) follow.
 *   - Return value: 0 on success, a negative EGNN_E* code otherwise; egnn_last_error() gives text.
 *     Nothing throws or aborts across this boundary.  Identical inputs give bit-identical
 *     outputs (no floating-point atomics anywhere).  A context keeps the last error text and a few
 *     lazily built tables: use it from one thread at a time.
 */
#ifndef EGNN_H
#define EGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EGNN_OK 0
#define EGNN_EINVAL (-1) /* bad descriptor, null pointer, unsupported shape            */
#define EGNN_EBOX (-2)   /* periodic box edge < 2*r_cut: minimum image not unique      */
#define EGNN_EWS (-3)    /* workspace too small                                        */
#define EGNN_EHIP (-4)   /* a HIP call failed; text in egnn_last_error                 */

#define EGNN_MAX_SHELLS 8

typedef struct egnn_ctx egnn_ctx; /* opaque: host-side constant tables and the last error text */

/* Model description, filled by the caller.  .size = sizeof(egnn_model_desc).
 * Supported: lmax == lmax_sh in 0..4; channels in {8,16,32,64,128}; n_rbf in 2..32;
 * n_radial_hidden == 64; orbital shells with l <= 2 (Sec. 6: 13 orbitals = 2s + 2p + 1d). */
typedef struct {
  uint32_t size;
  int32_t lmax, lmax_sh, channels, n_rbf, n_radial_hidden, n_layers;
  float r_cut;
  float agg_norm; /* nbar > 0: messages are summed and divided by sqrt(nbar) */
  int32_t n_orb_shells;
  int32_t orb_l[EGNN_MAX_SHELLS];
} egnn_model_desc;

typedef struct {
  const int32_t* src;     /* [n_edges] */
  const int32_t* dst;     /* [n_edges] */
  const int32_t* row_ptr; /* [n_owned+1] */
  const int8_t* shift;    /* [n_edges][3], periodic image of the source; may be NULL (all zero) */
  int64_t n_edges;
  int32_t n_owned, n_total;
  /* Optional, from egnn_edge_pairs (NULL / 0: every edge has its own row of radial weights): */
  const int32_t* w_row;   /* [n_edges] row of radial weights edge k reads: w_row[k] if >= 0 (the edge owns the row),
                             ~w_row[k] (bitwise complement) if negative (the row belongs to the reverse edge) */
  int64_t n_w_rows;       /* number of rows */
  /* Optional, from egnn_length_bins (NULL: the reverse pass builds them in every call that needs them): */
  const int32_t* len_ptr;  /* [EGNN_LENGTH_BINS + 1] */
  const int32_t* len_perm; /* [n_edges] edge ids grouped by length interval, ascending inside an interval */
} egnn_graph;

int egnn_create(const egnn_model_desc* desc, egnn_ctx** out);
void egnn_destroy(egnn_ctx* ctx);
const char* egnn_last_error(const egnn_ctx* ctx); /* ctx-owned string; ctx may be NULL (create errors) */

/* Number of coupling paths: which = 0 -> layers, P(lmax, lmax_sh, lmax); 1 -> readout, P(lmax, lmax_sh, 4).
 * If paths (host, [n][3]) is not NULL the (l1,l2,l3) triples are written to it. */
int egnn_path_count(const egnn_ctx* ctx, int which, int32_t* n_paths, int32_t* paths);

/* Rows of the packed collapse matrix V of the readout per coupled degree L = 0..4 (host, [5]). */
int egnn_readout_widths(const egnn_ctx* ctx, int32_t n_out[5]);

/* Bytes of workspace egnn_layer_forward / egnn_readout_hij need when they build the radial
 * weights themselves (with_weights != 0) or get them from the caller (0). */
int egnn_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, int32_t n_total,
                         int with_weights, size_t* bytes);

/* ---- S1  radius graph (Sec. 3 "Initialization": edges i -> j within r_cut; Sec. 4.4: periodic) ----
 * Ordered pairs (i, j), i != j, j < n_owned, i < n_total, |pos_i + shift*box - pos_j| < r_cut with
 * the minimum image on periodic axes; fp64 predicate on the fp32 data; strict '<'.
 * Two phases because n_edges depends on the data: count fills row_ptr and returns n_edges (host),
 * the caller allocates src/dst/shift (n_edges entries; may be NULL when n_edges == 0) and passes the
 * same n_edges back, fill writes them sorted by (dst, src).
 * box, pbc: host arrays of 3.  EGNN_EBOX if a periodic edge is shorter than 2*r_cut.
 * ws: with a workspace of egnn_nlist_workspace_bytes (256-byte aligned) and at most 262,144 atoms the search
 * goes through a cell list (cells of edge >= r_cut, at most 64 per axis); count builds the cells, fill reuses
 * them, so fill must follow count with the same atoms and the same, untouched workspace (a different pos or ws
 * pointer is rejected with EGNN_EINVAL; a workspace overwritten in between gives a wrong list but no access outside
 * the buffers).  With ws == NULL
 * every destination sweeps all atoms (O(n_owned * n_total), fine for a few thousand atoms).  Both give the
 * same edge list.  count synchronises the stream (twice with a workspace: bounding box, edge count). */
int egnn_nlist_workspace_bytes(const egnn_ctx* ctx, int32_t n_total, size_t* bytes);
int egnn_nlist_count(egnn_ctx* ctx, const float* pos, int32_t n_owned, int32_t n_total,
                     const float box[3], const uint8_t pbc[3], int32_t* row_ptr, int64_t* n_edges,
                     void* ws, size_t ws_bytes, void* stream);
int egnn_nlist_fill(egnn_ctx* ctx, const float* pos, int32_t n_owned, int32_t n_total,
                    const float box[3], const uint8_t pbc[3], const int32_t* row_ptr, int64_t n_edges,
                    int32_t* src, int32_t* dst, int8_t* shift /* may be NULL */, void* ws, size_t ws_bytes,
                    void* stream);

/* ---- shared rows of radial weights (Sec. 3 "Initialization": an edge enters the message transform through the
 *      Gaussian expansion of its length, so an edge and its reverse have the same radial weights) ----
 * Gives every edge the row of the weight tensor it reads, one row per unordered pair of owned atoms: edge k = (i -> j)
 * owns a row if i is a halo atom (its reverse is not in the list), if i < j, or if the list holds no reverse (j -> i)
 * with the opposite image shift; otherwise it reads the row of its reverse.  Rows are numbered in ascending order of
 * the owning edges' ids.  w_row [n_edges] in the encoding of egnn_graph.w_row; n_rows (host) the number of rows.
 * A graph with w_row / n_w_rows set makes egnn_layer_forward, egnn_readout_hij, their _save forms and the reverse
 * pass evaluate and store one row of radial weights per row index instead of one per edge (w_save then has n_w_rows
 * rows); results are the same numbers as without (the two lengths are bit-identical).  Caller-supplied w_edge and the
 * stage calls egnn_radial_weights / egnn_tp_segsum stay per edge unless stated.  Needs the list sorted by (dst, src)
 * with at most one edge per ordered pair (what egnn_nlist_fill produces).  Synchronises the stream (row count).
 * ws: egnn_edge_pairs_workspace_bytes, 256-byte aligned. */
int egnn_edge_pairs_workspace_bytes(const egnn_ctx* ctx, int32_t n_owned, size_t* bytes);
int egnn_edge_pairs(egnn_ctx* ctx, const egnn_graph* g, int32_t* w_row, int64_t* n_rows, void* ws, size_t ws_bytes,
                    void* stream);

/* ---- edges grouped by length (an index of the reverse pass, like egnn_graph_transpose) ----
 * Interval m of EGNN_LENGTH_BINS holds the edges with |r_k| in [m, m+1) * r_cut / EGNN_LENGTH_BINS; len_perm lists
 * the edge ids interval by interval (len_ptr[m] .. len_ptr[m+1]), ascending inside an interval.  The reverse pass of
 * the radial MLP in its grid form (EGNN_OPT_RADIAL_BWD) adds the rows of dw in this order; a graph that carries the
 * two arrays saves every backward call from building them (they depend on the geometry only).
 * ws: egnn_length_bins_workspace_bytes, 256-byte aligned. */
#define EGNN_LENGTH_BINS 2048
int egnn_length_bins_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, size_t* bytes);
int egnn_length_bins(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3], int32_t* len_ptr,
                     int32_t* len_perm, void* ws, size_t ws_bytes, void* stream);

/* ---- node initialisation (Sec. 3: the L=0 plane carries the atomic species) ----
 * x[i][0][c] += table[species[i]][c]. */
int egnn_species_embed(egnn_ctx* ctx, const int32_t* species, const float* table, int32_t n_species,
                       float* x, int32_t n_nodes, void* stream);

/* ---- S2  edge geometry (Sec. 3: distances in a Gaussian basis; Sec. 2.2: Y^l_m of the direction) ----
 * rhat_d[k] = (r_k / |r_k|, |r_k|) as 4 floats.  Optional outputs (NULL to skip):
 * Y [n_edges][(lmax_sh+1)^2] component-normalised real harmonics; rbf [n_edges][n_rbf] with
 * B_b(d) = exp(-(d - b*r_cut/(n_rbf-1))^2 / (2 (r_cut/(n_rbf-1))^2)); fc [n_edges] = (1+cos(pi d/r_cut))/2. */
int egnn_edge_geometry(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                       float* rhat_d, float* Y, float* rbf, float* fc, void* stream);

/* ---- S3  radial weights ----
 * w[k][p][c] = fc(d_k) * alpha_p * (W_r2 SiLU(W_r1 B(d_k)))[p*channels + c], alpha_p = 1/sqrt(#paths
 * with the same l3).  which = 0 (layer paths) or 1 (readout paths).  W_r1 [64][n_rbf], W_r2 [P*channels][64].
 * ws: scratch of at least 384 * P * channels bytes, 256-byte aligned. */
int egnn_radial_weights(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges,
                        const float* W_r1, const float* W_r2, float* w, void* ws, size_t ws_bytes, void* stream);

/* egnn_radial_weights without a workspace argument, for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation): the scratch that egnn_radial_weights
 * takes from the caller (scalings and half-precision pieces of W_r2) lives in a device array built into the
 * library, 2,064,384 bytes per GPU (the largest supported shape: 42 paths x 128 channels), held until the process
 * ends.  The call allocates and frees nothing and enqueues kernels only; it computes exactly what
 * egnn_radial_weights computes (bit-identical).  Shapes with paths * channels > 5,376 are rejected with EGNN_EWS.
 * All calls on one GPU share that array: calls that overlap in time on one GPU (different streams or threads) race;
 * calls on one stream are safe.  The array's address is looked up per device in egnn_create (or on the first call
 * on a device, which should then not be under capture).  rhat_d and w may be NULL when n_edges is 0. */
int egnn_radial_weights_static(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges, const float* W_r1,
                               const float* W_r2, float* w, void* stream);

/* ---- S4  tensor-product messages summed over incoming edges (Sec. 3 "Message passing";
 *          Sec. 2.1, 2.2, Eq. 1 for the coupling) ----
 * a[j][(l3,m3)][c] = agg_norm^-1/2 * sum_{k: dst(k)=j} sum_p w[k][p][c] *
 *                    sum_{m1,m2} C_p[m1][m2][m3] h[src(k)][(l1,m1)][c] Yhat_{l2,m2}(rhat_k),   j < n_owned.
 * h [n_total][...], w [n_edges][P][channels], a [n_owned][...].  Deterministic (sorted segments). */
int egnn_tp_segsum(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* h,
                   const float* w, float* a, void* stream);

/* ---- S3 / S4 with the weights stored in half precision (storage only: the weights are evaluated in fp32 as in
 *      egnn_radial_weights, rounded to nearest even once, and converted back to fp32 before use; half-precision
 *      values with fp32 sums are the arithmetic of the paper's own runs, Sec. 4.1) ----
 * w16 [n_edges][row_words] 32-bit words, row_words = 32 * ceil(P * channels / 64): word m (0..31) of group j of a
 * row holds column n = 64 j + m in its low 16 bits and column n + 32 in its high 16 bits, n = p * channels + c
 * (halves whose column is >= P * channels are unspecified).  Other arguments as in the fp32 calls. */
int egnn_radial_weights_f16(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges,
                            const float* W_r1, const float* W_r2, uint32_t* w16, void* ws, size_t ws_bytes,
                            void* stream);
int egnn_tp_segsum_f16(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* h,
                       const uint32_t* w16, float* a, void* stream);
/* The same with the gathered features in half precision as well (Sec. 4.1: the paper's runs keep embeddings and
 * communication buffers in half precision and aggregate in fp32): h16 [n_total][(lmax+1)^2][channels] IEEE half
 * precision, e.g. written by egnn_pack_rows with half != 0 and the identity index list.  Sums and output in fp32. */
int egnn_tp_segsum_f16h(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const uint16_t* h16,
                        const uint32_t* w16, float* a, void* stream);

/* ---- S5  per-degree channel mix (the per-l linear of Fig. 2(d)) ----
 * y[n][(l,m)][c] = sum_c' W1[l][c][c'] x1[n][(l,m)][c'] (+ sum_c' W2[l][c][c'] x2[n][(l,m)][c'] if W2 != NULL). */
int egnn_node_mix(egnn_ctx* ctx, const float* x1, const float* W1, const float* x2, const float* W2,
                  float* y, int32_t n_nodes, void* stream);

/* Options.  EGNN_OPT_FUSED (default 0): when 1 or 2, egnn_layer_forward with its own radial MLP, a power of two >= 8
 * channels and at most 32 radial bases produces and consumes the radial weights inside one kernel (they are never
 * written to memory); when 0 it goes through the materialised weight tensor (S3 then S4), as it always does for
 * caller-supplied weights, for the _save calls and for shapes the chosen kernel does not support.  All routes compute
 * the same function.  1: producer and consumer waves hand the weights over through LDS (needs lmax >= 1).
 * 2: transposed matrix-core tiles put the weights of one (edge, channel) into the registers of the lane that consumes
 * them (needs its LDS tiles to fit: up to 128 channels at lmax 4); its contraction cuts the operands into two
 * half-precision pieces with scalings taken from W_r1 and W_r2 on the device, as accurate as the default route for
 * any finite weights.  At 32 channels route 2 takes about 8 % less time than the two kernels of the default route, at
 * 64 channels about 10-15 % less; route 1 is slower than both. */
#define EGNN_OPT_FUSED 1
/* EGNN_OPT_W_FP16 (default 0): when 1, the radial weights that egnn_layer_forward (two-kernel route, own radial MLP)
 * and egnn_readout_hij pass from S3 to S4 / S6 inside their workspace are stored in half precision, as by
 * egnn_radial_weights_f16; all products and sums stay in fp32.  This halves the dominant memory traffic of both
 * calls at a relative rounding error of 2^-12 per weight: a reduced-precision mode, not covered by the fp32 accuracy
 * statement of the default.  Caller-supplied w_edge and the reverse pass always use fp32 weights. */
#define EGNN_OPT_W_FP16 2
/* EGNN_OPT_RADIAL_BWD (default 0): how egnn_layer_backward / egnn_readout_backward (and their _saved forms) turn the
 * gradient dw of the radial weights into dW_r1 and dW_r2.  1: two contractions on the matrix cores, each streaming dw.
 * 2: one pass over dw that bins its rows on a grid of 2,048 distances with six-point Lagrange weights, followed by two
 * small dense products over the grid points (everything but dw depends on the edge through its length only);
 * interpolation error below 1e-8 of the result while the absolute row sums of W_r1 stay below 100, 1e-6 at 256.
 * 0: decided on the device per call: route 2 if max_j sum_b |W_r1[j][b]| <= 256, else route 1.  Both are
 * deterministic. */
#define EGNN_OPT_RADIAL_BWD 3
int egnn_set_option(egnn_ctx* ctx, int32_t option, int32_t value);

/* ---- one message-passing layer, forward: S2 -> S5(pre) -> S3+S4 fused (or S3 -> S4) -> S5(post) ----
 * x_out[j] = W_post a_j + W_self x_in[j] for j < n_owned, with h = W_pre x_in.  x_in has n_total rows;
 * x_out has n_owned rows (may be NULL if n_owned is 0) and must not alias x_in.  If w_edge != NULL ([n_edges][P][channels]) it is used as
 * the radial weights (W_r1, W_r2 ignored).  ws: at least egnn_workspace_bytes(...) bytes, 256-byte aligned.
 * The call enqueues kernels only (no copies, no memsets, no host synchronisation; box is read on the host at call
 * time), so a stack of layers may be recorded into a graph by stream capture and replayed (tested); egnn_readout_hij
 * uploads its index tables with asynchronous copies from context memory and is not meant to be recorded. */
int egnn_layer_forward(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                       const float* x_in, const float* W_pre, const float* W_post, const float* W_self,
                       const float* W_r1, const float* W_r2, const float* w_edge, float* x_out,
                       void* ws, size_t ws_bytes, void* stream);

/* ---- S6  readout of the orbital blocks (Fig. 2(e); Sec. 2.2; Sec. 3) ----
 * z_k = (W_s x)[src] + (W_t x)[dst];  u_k = tensor product of z_k with Yhat(rhat_k) over P(lmax, lmax_sh, 4)
 * with its own radial weights;  q_k[o][M] = sum_c V_L[o][c] u_k[(L,M)][c];
 * H_k[(a,m_a)][(b,m_b)] = sum_{L,M} C^{(L,M)}_{(l_a m_a)(l_b m_b)} q_k[o(a,b,L)][M], rows = source-atom
 * orbitals, columns = destination-atom orbitals, o(a,b,L) counting ordered shell pairs in row-major
 * shell order with L ascending, separately per L.  V packs V_0 .. V_4, each [n_out(L)][channels].
 * H [n_edges][n_orb][n_orb] (may be NULL for a graph without edges). */
int egnn_readout_hij(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                     const float* x, const float* W_s, const float* W_t, const float* W_r1,
                     const float* W_r2, const float* V, float* H, void* ws, size_t ws_bytes, void* stream);

/* ---- S7  training step: loss and reverse pass (Sec. 4.1: gradients of the forward pass; the loss is the
 *          mean squared error over the elements of the H blocks) ----
 * Gradient outputs are overwritten, not accumulated.  Forward quantities are recomputed from the inputs of
 * the call; nothing has to be saved by the caller except each layer's input x_in.  All sums over edges and
 * nodes are taken in a fixed order (no floating-point atomics): results are bit-reproducible.
 *
 * egnn_graph_transpose: source-sorted index of the edge list.  col_ptr [n_total+1]; perm [n_edges] lists, for
 * each source node i, the ids of its outgoing edges in ascending order (= ascending destination).
 * ws: at least egnn_backward_workspace_bytes. */
int egnn_backward_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, int32_t n_total,
                                  size_t* bytes);
int egnn_graph_transpose(egnn_ctx* ctx, const egnn_graph* g, int32_t* col_ptr, int32_t* perm, void* ws,
                         size_t ws_bytes, void* stream);

/* loss[0] = mean_i (H[i] - T[i])^2 over n_values entries (device scalar); if dH != NULL,
 * dH[i] = 2 (H[i] - T[i]) / n_values.  ws: at least 8 * ceil(n_values / 4096) bytes. */
int egnn_loss_mse(egnn_ctx* ctx, const float* H, const float* T, int64_t n_values, float* loss, float* dH,
                  void* ws, size_t ws_bytes, void* stream);

/* Adjoint of egnn_layer_forward.  dx_out [n_owned][...] is the gradient w.r.t. the layer output; dx_in
 * [n_total][...] receives the gradient w.r.t. the layer input (halo rows included); dW_* have the shapes of
 * the corresponding weights. */
int egnn_layer_backward(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                        const float* pos, const float box[3], const float* x_in, const float* W_pre,
                        const float* W_post, const float* W_self, const float* W_r1, const float* W_r2,
                        const float* dx_out, float* dx_in, float* dW_pre, float* dW_post, float* dW_self,
                        float* dW_r1, float* dW_r2, void* ws, size_t ws_bytes, void* stream);

/* Keeping forward quantities instead of recomputing them (a trade of memory for time: at 3,000 atoms the weight
 * tensors of three layers and the readout are 13.5 GB, a few per cent of this GPU's memory; the paper reports 115 GB
 * of saved activations for its training runs at that size, Sec. 4).  egnn_layer_forward_save / egnn_readout_hij_save
 * compute exactly what egnn_layer_forward (own radial MLP, route through the materialised fp32 weight tensor) /
 * egnn_readout_hij compute and leave the radial weights w_save [n_edges][P][channels] and, for the layer, the summed
 * messages a_save [n_owned][(lmax+1)^2][channels] in caller buffers; egnn_layer_backward_saved /
 * egnn_readout_backward_saved take them back (either may be NULL: then it is recomputed) and give bit-identical
 * gradients to the recomputing calls.  Workspaces as for the recomputing calls. */
int egnn_layer_forward_save(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                            const float* x_in, const float* W_pre, const float* W_post, const float* W_self,
                            const float* W_r1, const float* W_r2, float* x_out, float* w_save, float* a_save,
                            void* ws, size_t ws_bytes, void* stream);
int egnn_readout_hij_save(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3], const float* x,
                          const float* W_s, const float* W_t, const float* W_r1, const float* W_r2, const float* V,
                          float* H, float* w_save, void* ws, size_t ws_bytes, void* stream);
int egnn_layer_backward_saved(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                              const float* pos, const float box[3], const float* x_in, const float* W_pre,
                              const float* W_post, const float* W_self, const float* W_r1, const float* W_r2,
                              const float* w_saved, const float* a_saved, const float* dx_out, float* dx_in,
                              float* dW_pre, float* dW_post, float* dW_self, float* dW_r1, float* dW_r2, void* ws,
                              size_t ws_bytes, void* stream);
int egnn_readout_backward_saved(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                                const float* pos, const float box[3], const float* x, const float* W_s,
                                const float* W_t, const float* W_r1, const float* W_r2, const float* V,
                                const float* w_saved, const float* dH, float* dx, float* dW_s, float* dW_t,
                                float* dW_r1, float* dW_r2, float* dV, void* ws, size_t ws_bytes, void* stream);

/* Adjoint of egnn_readout_hij.  dH [n_edges][n_orb][n_orb]; dx [n_total][...]; dV packed like V.
 * EGNN_EINVAL if the orbital basis is so large that the kernel's tiles (per wavefront one partial dV, per edge in
 * flight its block of dH and the collapsed gradients) exceed the 160 KB of LDS of a compute unit: the default basis
 * needs 37-54 KB, eight shells (s, s, s, p, p, p, d, d) 103-149 KB. */
int egnn_readout_backward(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                          const float* pos, const float box[3], const float* x, const float* W_s,
                          const float* W_t, const float* W_r1, const float* W_r2, const float* V,
                          const float* dH, float* dx, float* dW_s, float* dW_t, float* dW_r1, float* dW_r2,
                          float* dV, void* ws, size_t ws_bytes, void* stream);

/* ---- the message transform in its bond-aligned SO(2) form (Fig. 2(a) bottom, Fig. 2(d); Sec. 3 "Message passing";
 *      Sec. 2.1, last paragraph), summed over incoming edges ----
 * Per directed edge k = (i -> j) the message is [x_i | x_j | e_k] along the channel axis (3 * channels), e_k zero
 * except for its L = 0 plane W_e B(d_k) (B the Gaussian basis of S2).  It is rotated so that the bond lies on z,
 * every order m goes through its own linear layer over (degree l >= |m|, channel), 3 * channels -> channels,
 *     y_0 = W_0 x_0;   y_{+m} = Wr_m x_{+m} - Wi_m x_{-m},   y_{-m} = Wi_m x_{+m} + Wr_m x_{-m}   (m > 0 <-> cos, m < 0 <-> sin),
 * rotated back, multiplied by the cutoff envelope f_c(d_k), and
 *     a[j] = agg_norm^-1/2 sum_{k: dst(k) = j} y_k        for the owned nodes j.
 * W_so2: W_0, then Wr_1, Wi_1, ..., Wr_lmax, Wi_lmax, each row-major [(lmax+1-m) * channels][(lmax+1-m) * 3 * channels]
 * with row = (l_out - m) * channels + c_out and column = (l_in - m) * 3 * channels + g * channels + c_in, g = 0 source
 * node, 1 destination node, 2 edge (egnn_so2_weight_count floats in all).  W_e [channels][n_rbf].
 * x [n_total][(lmax+1)^2][channels], a [n_owned][(lmax+1)^2][channels] (a must not alias x).  Needs >= 8 channels.
 * The same function as the tensor-product messages of S4 when the weights are the coupling coefficients of the
 * bond direction (no channel mixing); in general a dense contraction shared by all edges. */
int egnn_so2_weight_count(const egnn_ctx* ctx, int64_t* n_floats);
int egnn_so2_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, size_t* bytes);
int egnn_so2_message_sum(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3], const float* x,
                         const float* W_e, const float* W_so2, float* a, void* ws, size_t ws_bytes, void* stream);

/* Adjoint of egnn_so2_message_sum with respect to the node embeddings and the weights (Sec. 4.1: training needs the
 * gradients of the forward pass; positions are data).  da [n_owned][(lmax+1)^2][channels] is the gradient with respect
 * to a.  Outputs are overwritten, not accumulated: dx [n_total][(lmax+1)^2][channels] (halo rows included: they
 * receive the source side of their outgoing edges), dW_e [channels][n_rbf], dW_so2 in the layout of W_so2 (the
 * columns g = 2 of l_in > 0, which multiply planes of the edge embedding that are zero on this path, get zero).
 * col_ptr, perm: the source-sorted index of egnn_graph_transpose.  The forward operands are recomputed from the inputs;
 * all sums over edges are taken in a fixed order (no floating-point atomics).  ws: at least
 * egnn_so2_backward_workspace_bytes, 256-byte aligned; EGNN_EWS if too small.  Needs 8 .. 128 channels, n_rbf <= 32. */
int egnn_so2_backward_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, size_t* bytes);
int egnn_so2_message_sum_backward(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                                  const float* pos, const float box[3], const float* x, const float* W_e,
                                  const float* W_so2, const float* da, float* dx, float* dW_e, float* dW_so2, void* ws,
                                  size_t ws_bytes, void* stream);

/* ---- the two blocks of a layer with the full message content (Sec. 3 "Message passing"; Fig. 2(b), 2(c)) ----
 * Edge embeddings T_edge [n_edges][(lmax+1)^2][channels] are persistent tensors that rotate like node embeddings;
 * the message of edge k is [x_src | x_dst | T_edge_k] in every degree (3 * channels), transformed as in
 * egnn_so2_message_sum (W_so2 in the same layout; all of its columns are used now).
 * egnn_edge_embed_init: the initial embeddings (Sec. 3 "Initialization"): L = 0 plane W_e B(d_k), zeros elsewhere.
 * egnn_so2_node_block (Fig. 2(b)): a[j] = sum_{k: dst(k) = j} alpha_k f_c(d_k) y_k for owned j, with the attention
 *   weights alpha = softmax over the incoming edges of j of s_k = sum_c w_att[c] LeakyReLU_0.2(y_k[L = 0][c]) (one
 *   head; the score uses the rotation-invariant plane of the transformed message before the envelope).
 * egnn_so2_edge_block (Fig. 2(c)): T_edge_out[k] = T_edge_in[k] + f_c(d_k) y_k, no sum; T_edge_out may alias T_edge_in.
 * egnn_gate: y[n][L = 0][c] = SiLU(x[n][L = 0][c]); for l >= 1, y[n][(l,m)][c] = x[n][(l,m)][c] *
 *   sigmoid(sum_c' W_g[l-1][c][c'] x[n][L = 0][c']);  W_g [lmax][channels][channels]; y may alias x.
 * ws: egnn_so2_blocks_workspace_bytes, 256-byte aligned. */
int egnn_so2_blocks_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, size_t* bytes);
int egnn_edge_embed_init(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3], const float* W_e,
                         float* T_edge, void* ws, size_t ws_bytes, void* stream);
int egnn_so2_node_block(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3], const float* x,
                        const float* T_edge, const float* W_so2, const float* w_att, float* a, void* ws,
                        size_t ws_bytes, void* stream);
int egnn_so2_edge_block(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3], const float* x,
                        const float* T_edge_in, const float* W_so2, float* T_edge_out, void* ws, size_t ws_bytes,
                        void* stream);
int egnn_gate(egnn_ctx* ctx, const float* x, const float* W_g, float* y, int32_t n_nodes, void* stream);

/* Adjoints of the two blocks and of the gate with respect to node embeddings, edge embeddings and weights (Sec. 4.1:
 * training needs the gradients of the forward pass; positions are data).  Outputs are overwritten, not accumulated;
 * forward quantities are recomputed from the inputs; all sums are taken in a fixed order (no floating-point atomics).
 * col_ptr, perm: the source-sorted index of egnn_graph_transpose.  dx [n_total][(lmax+1)^2][channels] (halo rows
 * included), dW_so2 in the layout of W_so2.
 * egnn_so2_node_block_backward: da [n_owned][...] is the gradient with respect to a; dT_edge [n_edges][...] the gradient
 *   with respect to the edge embeddings; dw_att [channels].  The attention weights are differentiated through (softmax
 *   over the incoming edges, LeakyReLU score; at a score input of exactly zero the slope 0.2 is taken).
 * egnn_so2_edge_block_backward: dT_out [n_edges][...] is the gradient with respect to T_edge_out; dT_in receives
 *   dT_out + the part through the messages and may alias dT_out.
 * egnn_gate_backward: dy, dx [n_nodes][...]; dW_g [lmax][channels][channels]; ws: egnn_gate_backward_workspace_bytes
 *   (not needed for lmax = 0).
 * ws of the block calls: at least egnn_so2_blocks_backward_workspace_bytes, 256-byte aligned; EGNN_EWS if too small.
 * 8 .. 128 channels. */
int egnn_so2_blocks_backward_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, size_t* bytes);
int egnn_so2_node_block_backward(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                                 const float* pos, const float box[3], const float* x, const float* T_edge,
                                 const float* W_so2, const float* w_att, const float* da, float* dx, float* dT_edge,
                                 float* dW_so2, float* dw_att, void* ws, size_t ws_bytes, void* stream);
int egnn_so2_edge_block_backward(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                                 const float* pos, const float box[3], const float* x, const float* T_edge_in,
                                 const float* W_so2, const float* dT_out, float* dx, float* dT_in, float* dW_so2,
                                 void* ws, size_t ws_bytes, void* stream);
int egnn_gate_backward_workspace_bytes(const egnn_ctx* ctx, int32_t n_nodes, size_t* bytes);
int egnn_gate_backward(egnn_ctx* ctx, const float* x, const float* W_g, const float* dy, float* dx, float* dW_g,
                       int32_t n_nodes, void* ws, size_t ws_bytes, void* stream);

/* ---- assembly of the predicted Hamiltonian (Sec. 3, end of "Message passing": nodes give the diagonal blocks, edges the
 *      off-diagonal ones; Fig. 2(e): collapse E -> 1, padded outputs; Sec. 2.2 / Eq. 1: the coupled basis and its
 *      inverse; Sec. 6: combined L1 + L2 loss over the elements of H) ----
 * Orbital sets: the model's shell list (egnn_model_desc.orb_l) is the global one; species s owns the orbitals whose
 * bit is set in orb_bits[s] (bit o = o-th orbital of the global list; device array of n_species words).  species is a
 * device array over all n_total atoms (values clamped to 0 .. n_species-1).  An entry of a block whose row orbital is
 * absent on the row atom or whose column orbital is absent on the column atom is padding.
 * Blocks: float [n_blocks][n_orb][n_orb]; row_atom / col_atom [n_blocks] give the atoms of a block's rows and
 * columns (for edge blocks g->src and g->dst; NULL = the block index itself, i.e. on-site blocks).
 *
 * egnn_onsite_hii: H_ii[i][(a,m_a)][(b,m_b)] = sum_{L <= lmax, M} C^{(L,M)}_{(l_a m_a)(l_b m_b)} q_i[o(a,b,L)][M],
 *   q_i[o][M] = sum_c V_node[L][o][c] x[i][(L,M)][c]; V_node packed like V of egnn_readout_hij (rows of degrees above
 *   lmax are not read).  x [n_nodes][(lmax+1)^2][channels].
 * egnn_apply_padding: sets the padding entries of H to zero in place.
 * egnn_loss_l1l2: loss[0] = mean |H - T| + mean (H - T)^2 over the entries that are not padding, loss[1], loss[2] the
 *   two terms (device, 3 floats); if dH != NULL, dH = (sign(H - T) + 2 (H - T)) / (number of such entries), 0 on padding.
 * egnn_hamiltonian_structure / egnn_hamiltonian_fill: the matrix with columns = orbitals of the owned atoms and rows =
 *   orbitals of all atoms (atom-major, each atom's own orbitals in the order of the global list), column-compressed:
 *   orb_off [n_total+1] first row/column of every atom; col_ptr [n_cols+1] (the caller provides n_owned * n_orb + 1
 *   entries); per column the rows ascend: the blocks of the sources of the atom's incoming edges and its own on-site
 *   block, every entry of a block stored.  structure computes orb_off, col_ptr and the placement of every block
 *   (kept in `plan`, an opaque device buffer of plan_bytes from egnn_hamiltonian_workspace_bytes) and returns
 *   n_cols and nnz (host; synchronises the stream); fill writes values [nnz] and, if not NULL, row_idx [nnz] from
 *   H_edge [n_edges][n_orb][n_orb] (rows = source orbitals) and H_node [>= n_owned][n_orb][n_orb].
 * ws / plan: 256-byte aligned, sizes from egnn_hamiltonian_workspace_bytes. */
int egnn_hamiltonian_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, int32_t n_total,
                                     size_t* ws_bytes, size_t* plan_bytes);
int egnn_onsite_hii(egnn_ctx* ctx, const float* x, const float* V_node, float* H_ii, int32_t n_nodes,
                    void* ws, size_t ws_bytes, void* stream);
/* Adjoint of egnn_onsite_hii: dx [n_nodes][(lmax+1)^2][channels] and dV_node (packed like V_node; rows of degrees
 * above lmax are set to zero) from dH_ii; both overwritten.  Nodes are added in a fixed order.  ws: egnn_onsite_backward_workspace_bytes, 256-byte aligned. */
int egnn_onsite_backward_workspace_bytes(const egnn_ctx* ctx, int32_t n_nodes, size_t* bytes);
int egnn_onsite_backward(egnn_ctx* ctx, const float* x, const float* V_node, const float* dH_ii, float* dx,
                         float* dV_node, int32_t n_nodes, void* ws, size_t ws_bytes, void* stream);
int egnn_apply_padding(egnn_ctx* ctx, float* H, int64_t n_blocks, const int32_t* row_atom, const int32_t* col_atom,
                       const int32_t* species, const uint32_t* orb_bits, int32_t n_species, void* stream);
int egnn_loss_l1l2(egnn_ctx* ctx, const float* H, const float* T, int64_t n_blocks, const int32_t* row_atom,
                   const int32_t* col_atom, const int32_t* species, const uint32_t* orb_bits, int32_t n_species,
                   float* loss, float* dH, void* ws, size_t ws_bytes, void* stream);
int egnn_hamiltonian_structure(egnn_ctx* ctx, const egnn_graph* g, const int32_t* species, const uint32_t* orb_bits,
                               int32_t n_species, int32_t* orb_off, int64_t* col_ptr, void* plan, size_t plan_bytes,
                               int64_t* n_cols, int64_t* nnz, void* stream);
int egnn_hamiltonian_fill(egnn_ctx* ctx, const egnn_graph* g, const int32_t* species, const uint32_t* orb_bits,
                          int32_t n_species, const int32_t* orb_off, const void* plan, size_t plan_bytes,
                          const float* H_edge, const float* H_node, int32_t* row_idx, float* values, void* stream);

/* ---- Low-NN partitioner (Sec. 4.4; Appendix A, Algorithm 1) and pack / unpack of halo rows (Sec. 4.3, Fig. 4(b)) ----
 * egnn_partition_low_nn: HOST function, all pointers are host pointers; needs no context and no GPU.  Recursive
 *   bisection of n_atoms atoms into 2^levels parts: a dimension that has no cut yet is first "opened" at its balanced
 *   position (one cut through a periodic ring divides nothing, it fixes the origin; non-periodic dimensions start
 *   opened at their smallest coordinate); then, at every level, NN[d] = 1 for a dimension with one cut and
 *   ceil(2 r_cut / L[d]) otherwise (L = extent of the sub-domain), the dimension with the lowest NN is cut (the highest
 *   index among equals) at the position that splits the atoms, ordered along it, into the two groups whose summed
 *   degree differs least (fewest atoms on the left among equals; atoms at equal coordinate keep their order of
 *   arrival), and both halves are cut further with their own copy of the cut counts.
 *   pos [n_atoms][3], degree [n_atoms] (edges of each atom), box / pbc [3], part [n_atoms] out: 0 .. 2^levels - 1 in
 *   the order the parts are finished (left before right).  cut_log (may be NULL): [2^levels - 1][4] = (level,
 *   dimension, atoms in the sub-domain, atoms on the left) for every bisection in depth-first order; n_cuts (may be
 *   NULL): how many were made (empty sub-domains make none).  levels <= 20.
 * egnn_spatial_order: HOST function, host pointers, needs no context and no GPU.  A numbering of the atoms that keeps
 *   neighbours in space close in index, for callers whose atoms come in no particular order (the kernels that gather
 *   node rows process destination nodes in index order and re-use the rows that neighbouring destinations share: with
 *   atoms in random order the message kernel of this library runs a quarter slower at the largest configuration).
 *   pos [n_total][3]; atoms are binned into cubes of edge cell > 0 (a good choice: half the cutoff) counted from the
 *   smallest coordinates, at most 1024 cubes per axis, the cubes are walked along a Morton curve, atoms of a cube
 *   keep their order; perm [n_total] out: perm[new index] = old index, the owned atoms (old indices < n_owned) first,
 *   then the halo atoms, each group in that order.  The caller permutes positions, species and features with it
 *   before building the graph.  This changes no result beyond the numbering (and the order of floating-point sums).
 * egnn_pack_rows: out[r] = x[idx[r]] for r < n_idx (rows of (lmax+1)^2 * channels floats; idx clamped to
 *   0 .. n_rows_x - 1); half != 0: the buffer holds IEEE half precision (round to nearest even), else fp32.
 * egnn_unpack_rows: x_full[first_row + r] = buf[r] for r < n_rows (converted back to fp32 if half != 0). */
int egnn_spatial_order(const float* pos, int32_t n_owned, int32_t n_total, float cell, int32_t* perm);
int egnn_partition_low_nn(const float* pos, const int32_t* degree, int32_t n_atoms, const float box[3],
                          const uint8_t pbc[3], double r_cut, int32_t levels, int32_t* part, int32_t* cut_log,
                          int32_t* n_cuts);
int egnn_pack_rows(egnn_ctx* ctx, const float* x, int32_t n_rows_x, const int32_t* idx, int32_t n_idx, int32_t half,
                   void* out, void* stream);
int egnn_unpack_rows(egnn_ctx* ctx, const void* buf, int32_t n_rows, int32_t half, float* x_full, int32_t first_row,
                     void* stream);

/* ---- stage timing (measurement aid; follows the paper's protocol of timing the blocks of the forward
 *      pass separately, Sec. 4.4 / Fig. 6(c)) ----
 * egnn_timing_enable(ctx, max_calls > 0) creates HIP events; from then on every egnn_layer_forward /
 * egnn_readout_hij / egnn_layer_backward / egnn_readout_backward (and their _save / _saved forms) records one event
 * per stage on the caller's stream, for at most max_calls calls (further calls are not recorded).  max_calls = 0
 * turns it off.  egnn_timing_read waits for the recorded calls, sums the elapsed milliseconds per stage and clears
 * the record:
 *   ms[0..4]    layer:           geometry, radial weights, pre mix, tensor-product + segmented sum, post mix
 *   ms[5..9]    readout:         geometry, radial weights, source mix, destination mix, product + collapse + uncoupling
 *   ms[10..14]  layer adjoint:   forward quantities (what is not supplied), adjoint of the post mix + weight
 *                                gradients, adjoint of the messages, adjoint of the pre mix + weight gradient,
 *                                radial MLP
 *   ms[15..19]  readout adjoint: forward quantities, adjoint of uncoupling + collapse + product, row sums + adjoints
 *                                of the two mixes + weight gradients, radial MLP, (unused)
 *   n_calls[0..3]: recorded calls of each kind (host arrays). */
int egnn_timing_enable(egnn_ctx* ctx, int32_t max_calls);
int egnn_timing_read(egnn_ctx* ctx, float ms[20], int32_t n_calls[4]);

#ifdef __cplusplus
}
#endif
#endif /* EGNN_H */
