// Composite entry points of the reverse pass (training step): egnn_layer_backward, egnn_readout_backward.
// Forward quantities are recomputed from the layer input rather than saved (the radial weights alone are
// 3.4 GB per layer at 3,000 atoms; Sec. 3 "Implementation" quotes 115 GB of saved activations for that size).
#include <math.h>
#include "egnn_internal.h"

static size_t a256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Carver2 {
  char* base;
  size_t used;
  void* take(size_t bytes) {
    void* p = base ? base + used : nullptr;
    used += a256(bytes);
    return p;
  }
};

static size_t row_bytes(const egnn_ctx* ctx) {
  return (size_t)(ctx->desc.lmax + 1) * (ctx->desc.lmax + 1) * ctx->desc.channels * sizeof(float);
}

static int vrows(const egnn_ctx* ctx) {
  int n = 0;
  for (int L = 0; L <= EGNN_L_READOUT; ++L) n += ctx->n_out[L];
  return n;
}

struct LayerBwdBufs {
  float *rhat_d, *rd_rows, *h, *a, *w, *da, *dh, *dw, *wgrad_partial;
  void *radial, *w2s;
};

static size_t carve_layer_bwd(const egnn_ctx* ctx, const egnn_graph* g, char* base, LayerBwdBufs* b) {
  const size_t row = row_bytes(ctx);
  const size_t wbytes = (size_t)g->n_edges * ctx->n_paths[0] * ctx->desc.channels * sizeof(float);
  Carver2 c{base, 0};
  b->rhat_d = (float*)c.take((size_t)g->n_edges * 16);
  b->rd_rows = (float*)c.take((size_t)g->n_edges * 16);   // records of the row-owning edges (graphs with shared rows)
  b->h = (float*)c.take((size_t)g->n_total * row);
  b->a = (float*)c.take((size_t)g->n_owned * row);
  b->da = (float*)c.take((size_t)g->n_owned * row);
  b->dh = (float*)c.take((size_t)g->n_total * row);
  b->w = (float*)c.take(wbytes);
  b->dw = (float*)c.take(wbytes);
  b->wgrad_partial = (float*)c.take(egnn_mix_wgrad_ws_bytes(ctx));
  b->radial = c.take(egnn_radial_backward_ws_bytes(ctx, 0, g->n_edges));
  b->w2s = c.take(egnn_radial_ws_bytes(ctx, 0));
  return c.used;
}

struct ReadoutBwdBufs {
  float *rhat_d, *rd_rows, *zs, *zt, *dzs, *dzt, *w, *dw, *dz, *wgrad_partial, *dV_partial, *tab_f;
  int* tab_i;
  void *radial, *w2s;
};

static size_t readout_bwd_tab_ints(const egnn_ctx* ctx) {
  const int nq = ctx->n_orb * ctx->n_orb;
  int q_off[EGNN_L_READOUT + 2], nqp;
  egnn_readout_backward_q_layout(ctx, q_off, &nqp);
  return (size_t)(nqp > nq ? nqp : nq) + 1 + ctx->unc_q.size();
}

static size_t carve_readout_bwd(const egnn_ctx* ctx, const egnn_graph* g, char* base, ReadoutBwdBufs* b) {
  const size_t row = row_bytes(ctx);
  const size_t wbytes = (size_t)g->n_edges * ctx->n_paths[1] * ctx->desc.channels * sizeof(float);
  Carver2 c{base, 0};
  b->rhat_d = (float*)c.take((size_t)g->n_edges * 16);
  b->rd_rows = (float*)c.take((size_t)g->n_edges * 16);   // records of the row-owning edges (graphs with shared rows)
  b->zs = (float*)c.take((size_t)g->n_total * row);
  b->zt = (float*)c.take((size_t)g->n_total * row);
  b->dzs = (float*)c.take((size_t)g->n_total * row);
  b->dzt = (float*)c.take((size_t)g->n_total * row);
  b->w = (float*)c.take(wbytes);
  b->dw = (float*)c.take(wbytes);
  b->dz = (float*)c.take((size_t)g->n_edges * row);
  b->wgrad_partial = (float*)c.take(egnn_mix_wgrad_ws_bytes(ctx));
  b->dV_partial = (float*)c.take(egnn_readout_backward_partial_bytes(ctx, g->n_edges));
  b->tab_i = (int*)c.take(readout_bwd_tab_ints(ctx) * sizeof(int));
  b->tab_f = (float*)c.take(ctx->unc_c.size() * sizeof(float));
  b->radial = c.take(egnn_radial_backward_ws_bytes(ctx, 1, g->n_edges));
  b->w2s = c.take(egnn_radial_ws_bytes(ctx, 1));
  return c.used;
}

extern "C" int egnn_backward_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, int32_t n_total,
                                             size_t* bytes) {
  if (!ctx || !bytes || n_edges < 0 || n_owned < 0 || n_total < n_owned) return EGNN_EINVAL;
  egnn_graph g = {nullptr, nullptr, nullptr, nullptr, n_edges, n_owned, n_total};
  LayerBwdBufs lb;
  ReadoutBwdBufs rb;
  size_t a = carve_layer_bwd(ctx, &g, nullptr, &lb);
  size_t b = ctx->n_orb > 0 ? carve_readout_bwd(ctx, &g, nullptr, &rb) : 0;
  size_t c = egnn_transpose_ws_bytes(n_edges, n_total);
  size_t m = a > b ? a : b;
  *bytes = (m > c ? m : c) + 256;
  return EGNN_OK;
}

static int check_bwd_graph(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                           const char* who) {
  if (!g) return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": null graph");
  if (g->n_edges < 0 || g->n_edges > 2147483647LL || g->n_owned < 0 || g->n_total < g->n_owned)
    return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": bad graph sizes");
  if (!g->row_ptr || !col_ptr || (g->n_edges > 0 && (!g->src || !g->dst || !perm)))
    return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": null graph arrays");
  if (g->w_row && (g->n_w_rows < 0 || g->n_w_rows > g->n_edges || (g->n_edges > 0 && g->n_w_rows == 0)))
    return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": n_w_rows does not fit the edge count");
  return EGNN_OK;
}

// w_saved / a_saved (may be NULL): the weight tensor and the summed messages of the forward pass, if the caller kept
// them (egnn_layer_forward_save); what is missing is recomputed
static int layer_backward_impl(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                               const float* pos, const float box[3], const float* x_in, const float* W_pre,
                               const float* W_post, const float* W_self, const float* W_r1, const float* W_r2,
                               const float* w_saved, const float* a_saved, const float* dx_out, float* dx_in,
                               float* dW_pre, float* dW_post, float* dW_self, float* dW_r1, float* dW_r2, void* ws,
                               size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_bwd_graph(ctx, g, col_ptr, perm, "layer_backward");
  if (rc) return rc;
  // (without owned nodes there is no output row: dx_out may then be NULL)
  if (!pos || !box || !x_in || !W_pre || !W_post || !W_self || !W_r1 || !W_r2 || (!dx_out && g->n_owned > 0) || !dx_in ||
      !dW_pre || !dW_post || !dW_self || !dW_r1 || !dW_r2 || !ws)
    return egnn_fail(ctx, EGNN_EINVAL, "layer_backward: null pointer");
  if (((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "layer_backward: workspace not 256-byte aligned");
  LayerBwdBufs b;
  if (ws_bytes < carve_layer_bwd(ctx, g, nullptr, &b)) return egnn_fail(ctx, EGNN_EWS, "layer_backward: workspace too small");
  carve_layer_bwd(ctx, g, (char*)ws, &b);
  hipStream_t st = (hipStream_t)stream;
  const size_t row_f = row_bytes(ctx) / sizeof(float);
  const int n_o = g->n_owned, n_t = g->n_total;

  // forward quantities
  // (graphs with shared rows: the forward weights, recomputed or kept, have one row per row index; dw one per edge)
  const bool shared = g->w_row != nullptr;
  StageTimer tm(ctx, st, 2);
  if ((rc = egnn_launch_geometry(ctx, g, pos, box, b.rhat_d, nullptr, nullptr, nullptr, st, shared ? b.rd_rows : nullptr)))
    return rc;
  const float* w = w_saved ? w_saved : b.w;
  const float* a = a_saved ? a_saved : b.a;
  if (!w_saved && (rc = egnn_launch_radial(ctx, 0, shared ? b.rd_rows : b.rhat_d, shared ? g->n_w_rows : g->n_edges, W_r1,
                                           W_r2, b.w, b.w2s, st)))
    return rc;
  if ((rc = egnn_launch_node_mix(ctx, x_in, W_pre, nullptr, nullptr, b.h, n_t, st))) return rc;
  if (!a_saved && (rc = egnn_launch_tp_segsum(ctx, g, b.rhat_d, b.h, w, b.a, st, false, shared))) return rc;
  tm.mark(0);
  // x_out = W_post a + W_self x_in[:n_owned]
  if ((rc = egnn_launch_node_mix(ctx, dx_out, W_post, nullptr, nullptr, b.da, n_o, st, 1))) return rc;
  if ((rc = egnn_launch_mix_wgrad(ctx, dx_out, a, dW_post, b.wgrad_partial, n_o, st))) return rc;
  if ((rc = egnn_launch_mix_wgrad(ctx, dx_out, x_in, dW_self, b.wgrad_partial, n_o, st))) return rc;
  tm.mark(1);
  // messages
  // (the largest |dw|, kept by the kernel that writes dw, scales the contractions that read it)
  unsigned* dw_max = egnn_radial_backward_dw_max(b.radial);
  if ((rc = egnn_launch_fill_int(ctx, (int*)dw_max, 64, 0, st))) return rc;
  if ((rc = egnn_launch_tp_backward(ctx, g, col_ptr, perm, b.rhat_d, b.h, w, b.da, b.dh, b.dw, dw_max, st, shared)))
    return rc;
  tm.mark(2);
  // h = W_pre x_in ; owned rows also receive the self term
  if ((rc = egnn_launch_node_mix(ctx, b.dh, W_pre, dx_out, W_self, dx_in, n_o, st, 1))) return rc;
  if (n_t > n_o &&
      (rc = egnn_launch_node_mix(ctx, b.dh + (size_t)n_o * row_f, W_pre, nullptr, nullptr, dx_in + (size_t)n_o * row_f,
                                 n_t - n_o, st, 1)))
    return rc;
  if ((rc = egnn_launch_mix_wgrad(ctx, b.dh, x_in, dW_pre, b.wgrad_partial, n_t, st))) return rc;
  tm.mark(3);
  // radial MLP
  rc = egnn_launch_radial_backward(ctx, 0, b.rhat_d, g->n_edges, W_r1, W_r2, b.dw, dW_r1, dW_r2, b.radial, true, st,
                                   g->len_ptr, g->len_perm);
  tm.mark(4);
  return rc;
}

extern "C" int egnn_layer_backward(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                                   const float* pos, const float box[3], const float* x_in, const float* W_pre,
                                   const float* W_post, const float* W_self, const float* W_r1, const float* W_r2,
                                   const float* dx_out, float* dx_in, float* dW_pre, float* dW_post, float* dW_self,
                                   float* dW_r1, float* dW_r2, void* ws, size_t ws_bytes, void* stream) {
  return layer_backward_impl(ctx, g, col_ptr, perm, pos, box, x_in, W_pre, W_post, W_self, W_r1, W_r2, nullptr, nullptr,
                             dx_out, dx_in, dW_pre, dW_post, dW_self, dW_r1, dW_r2, ws, ws_bytes, stream);
}

extern "C" int egnn_layer_backward_saved(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr,
                                         const int32_t* perm, const float* pos, const float box[3], const float* x_in,
                                         const float* W_pre, const float* W_post, const float* W_self,
                                         const float* W_r1, const float* W_r2, const float* w_saved,
                                         const float* a_saved, const float* dx_out, float* dx_in, float* dW_pre,
                                         float* dW_post, float* dW_self, float* dW_r1, float* dW_r2, void* ws,
                                         size_t ws_bytes, void* stream) {
  return layer_backward_impl(ctx, g, col_ptr, perm, pos, box, x_in, W_pre, W_post, W_self, W_r1, W_r2, w_saved, a_saved,
                             dx_out, dx_in, dW_pre, dW_post, dW_self, dW_r1, dW_r2, ws, ws_bytes, stream);
}

static int readout_backward_impl(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                                 const float* pos, const float box[3], const float* x, const float* W_s,
                                 const float* W_t, const float* W_r1, const float* W_r2, const float* V,
                                 const float* w_saved, const float* dH, float* dx, float* dW_s, float* dW_t,
                                 float* dW_r1, float* dW_r2, float* dV, void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_bwd_graph(ctx, g, col_ptr, perm, "readout_backward");
  if (rc) return rc;
  if (ctx->n_orb <= 0 || ctx->n_orb > 32) return egnn_fail(ctx, EGNN_EINVAL, "readout_backward: need 1..32 orbitals per atom");
  // (a graph without edges has no blocks: dH may then be NULL; every gradient is zero)
  if (!pos || !box || !x || !W_s || !W_t || !W_r1 || !W_r2 || !V || (!dH && g->n_edges > 0) || !dx || !dW_s || !dW_t ||
      !dW_r1 || !dW_r2 || !dV || !ws)
    return egnn_fail(ctx, EGNN_EINVAL, "readout_backward: null pointer");
  if (((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "readout_backward: workspace not 256-byte aligned");
  const int nq = ctx->n_orb * ctx->n_orb;
  if (egnn_readout_backward_lds_bytes(ctx) > 160 * 1024)
    return egnn_fail(ctx, EGNN_EINVAL, "readout_backward: orbital basis too large for the LDS tiles");
  ReadoutBwdBufs b;
  if (ws_bytes < carve_readout_bwd(ctx, g, nullptr, &b)) return egnn_fail(ctx, EGNN_EWS, "readout_backward: workspace too small");
  carve_readout_bwd(ctx, g, (char*)ws, &b);
  hipStream_t st = (hipStream_t)stream;
  const int n_t = g->n_total;
  const int row_len = (int)(row_bytes(ctx) / sizeof(float));

  // table: transposed uncoupling (q <- H).  The collapsed values are numbered by the row of V that produces
  // them, as egnn_readout_backward_q_layout lays them out (rows of one coupled degree consecutive, so the kernel finds
  // the values of a row without a table); the numbers that stand for no value have an empty list.
  std::vector<int>& ti = ctx->tab_rob_i;
  std::vector<float>& tf = ctx->tab_rob_f;
  if (ti.empty()) {
    std::vector<std::vector<std::pair<int, float>>> byq(nq);
    for (int hidx = 0; hidx < nq; ++hidx)
      for (int n = ctx->unc_ptr[hidx]; n < ctx->unc_ptr[hidx + 1]; ++n) byq[ctx->unc_q[n]].push_back({hidx, ctx->unc_c[n]});
    int v_off[EGNN_L_READOUT + 2] = {0}, q_off[EGNN_L_READOUT + 2], nqp;
    for (int L = 0; L <= EGNN_L_READOUT; ++L) v_off[L + 1] = v_off[L] + ctx->n_out[L];
    egnn_readout_backward_q_layout(ctx, q_off, &nqp);
    std::vector<int> by_row(nqp, -1);   // by_row[new number] = number of the value in the forward pass
    for (int s = 0; s < ctx->n_slots; ++s) {
      const int L = ctx->slot_L[s];
      for (int M = 0; M < 2 * L + 1; ++M)
        by_row[q_off[L] + (ctx->slot_vrow[s] - v_off[L]) * (2 * L + 1) + M] = ctx->slot_qoff[s] + M;
    }
    int run = 0;
    ti.push_back(0);
    for (int q = 0; q < nqp; ++q) {
      if (by_row[q] >= 0) run += (int)byq[by_row[q]].size();
      ti.push_back(run);
    }
    for (int q = 0; q < nqp; ++q)
      if (by_row[q] >= 0)
        for (auto& e : byq[by_row[q]]) {
          ti.push_back(e.first);
          tf.push_back(e.second);
        }
  }
  // (sources owned by the context: no need to wait for the copies)
  EGNN_HIP(ctx, hipMemcpyAsync(b.tab_i, ti.data(), ti.size() * sizeof(int), hipMemcpyHostToDevice, st));
  EGNN_HIP(ctx, hipMemcpyAsync(b.tab_f, tf.data(), tf.size() * sizeof(float), hipMemcpyHostToDevice, st));

  const bool shared = g->w_row != nullptr;
  StageTimer tm(ctx, st, 3);
  if ((rc = egnn_launch_geometry(ctx, g, pos, box, b.rhat_d, nullptr, nullptr, nullptr, st, shared ? b.rd_rows : nullptr)))
    return rc;
  const float* w = w_saved ? w_saved : b.w;
  if (!w_saved && (rc = egnn_launch_radial(ctx, 1, shared ? b.rd_rows : b.rhat_d, shared ? g->n_w_rows : g->n_edges, W_r1,
                                           W_r2, b.w, b.w2s, st)))
    return rc;
  if ((rc = egnn_launch_node_mix(ctx, x, W_s, nullptr, nullptr, b.zs, n_t, st))) return rc;
  if ((rc = egnn_launch_node_mix(ctx, x, W_t, nullptr, nullptr, b.zt, n_t, st))) return rc;
  tm.mark(0);
  if ((rc = egnn_launch_readout_backward(ctx, g, b.rhat_d, b.zs, b.zt, w, V, b.tab_i, b.tab_f, dH, b.dz, b.dw, dV,
                                         b.dV_partial, st, shared)))
    return rc;
  tm.mark(1);
  // dz_k feeds the source row (zs) and the destination row (zt, owned nodes only)
  if ((rc = egnn_launch_segsum_rows(ctx, b.dz, col_ptr, perm, b.dzs, n_t, row_len, st))) return rc;
  if ((rc = egnn_launch_segsum_rows(ctx, b.dz, g->row_ptr, nullptr, b.dzt, g->n_owned, row_len, st))) return rc;
  if (n_t > g->n_owned) {
    const long tail = (long)(n_t - g->n_owned) * row_len;
    // halo nodes are never destinations: their dzt rows are zero
    if ((rc = egnn_launch_reduce_partials(ctx, nullptr, 0, tail, b.dzt + (size_t)g->n_owned * row_len, 1.0f, st))) return rc;
  }
  if ((rc = egnn_launch_node_mix(ctx, b.dzs, W_s, b.dzt, W_t, dx, n_t, st, 1))) return rc;
  if ((rc = egnn_launch_mix_wgrad(ctx, b.dzs, x, dW_s, b.wgrad_partial, n_t, st))) return rc;
  if ((rc = egnn_launch_mix_wgrad(ctx, b.dzt, x, dW_t, b.wgrad_partial, n_t, st))) return rc;
  tm.mark(2);
  rc = egnn_launch_radial_backward(ctx, 1, b.rhat_d, g->n_edges, W_r1, W_r2, b.dw, dW_r1, dW_r2, b.radial, false, st,
                                   g->len_ptr, g->len_perm);   // (no running maximum of this dw: bf16 pieces on the exact route)
  tm.mark(3);
  tm.mark(4);
  return rc;
}

extern "C" int egnn_readout_backward(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm,
                                     const float* pos, const float box[3], const float* x, const float* W_s,
                                     const float* W_t, const float* W_r1, const float* W_r2, const float* V,
                                     const float* dH, float* dx, float* dW_s, float* dW_t, float* dW_r1,
                                     float* dW_r2, float* dV, void* ws, size_t ws_bytes, void* stream) {
  return readout_backward_impl(ctx, g, col_ptr, perm, pos, box, x, W_s, W_t, W_r1, W_r2, V, nullptr, dH, dx, dW_s, dW_t,
                               dW_r1, dW_r2, dV, ws, ws_bytes, stream);
}

extern "C" int egnn_readout_backward_saved(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr,
                                           const int32_t* perm, const float* pos, const float box[3], const float* x,
                                           const float* W_s, const float* W_t, const float* W_r1, const float* W_r2,
                                           const float* V, const float* w_saved, const float* dH, float* dx,
                                           float* dW_s, float* dW_t, float* dW_r1, float* dW_r2, float* dV, void* ws,
                                           size_t ws_bytes, void* stream) {
  return readout_backward_impl(ctx, g, col_ptr, perm, pos, box, x, W_s, W_t, W_r1, W_r2, V, w_saved, dH, dx, dW_s, dW_t,
                               dW_r1, dW_r2, dV, ws, ws_bytes, stream);
}
