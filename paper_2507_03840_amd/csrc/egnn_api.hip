// Context, argument checks, workspace carving and the composite entry points of the C ABI.
#include <math.h>
#include <string.h>
#include "egnn_internal.h"
#include "w_half.h"
#define EGNN_GEN_HOST_TABLES
#include "egnn_gen.inc"

static thread_local std::string g_create_error;

int egnn_fail(egnn_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->err = msg; else g_create_error = msg;
  return code;
}

int egnn_check_hip(egnn_ctx* ctx, hipError_t e, const char* what) {
  return egnn_fail(ctx, EGNN_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

static const EgnnPathList* find_paths(int l_in, int l_sh, int l_out) {
  for (int i = 0; i < egnn_n_path_lists; ++i) {
    const EgnnPathList& p = egnn_path_lists[i];
    if (p.l_in == l_in && p.l_sh == l_sh && p.l_out == l_out) return &p;
  }
  return nullptr;
}

static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

extern "C" int egnn_create(const egnn_model_desc* d, egnn_ctx** out) {
  if (!d || !out) return egnn_fail(nullptr, EGNN_EINVAL, "create: null pointer");
  *out = nullptr;
  if (d->size != sizeof(egnn_model_desc)) return egnn_fail(nullptr, EGNN_EINVAL, "create: desc.size mismatch");
  if (d->lmax < 0 || d->lmax > 4 || d->lmax_sh != d->lmax)
    return egnn_fail(nullptr, EGNN_EINVAL, "create: need 0 <= lmax == lmax_sh <= 4");
  int log2E = -1;
  for (int s = 3; s <= 7; ++s)
    if (d->channels == (1 << s)) log2E = s;
  if (log2E < 0) return egnn_fail(nullptr, EGNN_EINVAL, "create: channels must be 8, 16, 32, 64 or 128");
  if (d->n_rbf < 2 || d->n_rbf > 32) return egnn_fail(nullptr, EGNN_EINVAL, "create: n_rbf must be in 2..32");
  if (d->n_radial_hidden != EGNN_HIDDEN) return egnn_fail(nullptr, EGNN_EINVAL, "create: n_radial_hidden must be 64");
  if (!(d->r_cut > 0.0f) || !(d->agg_norm > 0.0f)) return egnn_fail(nullptr, EGNN_EINVAL, "create: r_cut, agg_norm must be > 0");
  if (d->n_orb_shells < 0 || d->n_orb_shells > EGNN_MAX_SHELLS)
    return egnn_fail(nullptr, EGNN_EINVAL, "create: n_orb_shells out of range");
  for (int s = 0; s < d->n_orb_shells; ++s)
    if (d->orb_l[s] < 0 || d->orb_l[s] > 2) return egnn_fail(nullptr, EGNN_EINVAL, "create: orbital shells need l <= 2");

  egnn_ctx* ctx = new egnn_ctx();
  ctx->desc = *d;
  ctx->log2_channels = log2E;
  const int l_outs[2] = {d->lmax, EGNN_L_READOUT};
  for (int which = 0; which < 2; ++which) {
    const EgnnPathList* pl = find_paths(d->lmax, d->lmax_sh, l_outs[which]);
    if (!pl || pl->n > EGNN_MAX_PATHS) {
      delete ctx;
      return egnn_fail(nullptr, EGNN_EINVAL, "create: no path table for this (lmax, lmax_sh)");
    }
    ctx->n_paths[which] = pl->n;
    int per_l3[16] = {0};
    for (int p = 0; p < pl->n; ++p) {
      for (int t = 0; t < 3; ++t) ctx->paths[which][p][t] = pl->l[p][t];
      per_l3[pl->l[p][2]]++;
    }
    for (int p = 0; p < pl->n; ++p) ctx->alpha[which][p] = (float)(1.0 / sqrt((double)per_l3[pl->l[p][2]]));
  }

  // readout tables
  const int ns = d->n_orb_shells;
  int orb_off[EGNN_MAX_SHELLS + 1] = {0};
  for (int s = 0; s < ns; ++s) orb_off[s + 1] = orb_off[s] + 2 * d->orb_l[s] + 1;
  ctx->n_orb = orb_off[ns];
  for (int L = 0; L <= EGNN_L_READOUT; ++L) ctx->n_out[L] = 0;
  for (int a = 0; a < ns; ++a)
    for (int b = 0; b < ns; ++b)
      for (int L = abs(d->orb_l[a] - d->orb_l[b]); L <= d->orb_l[a] + d->orb_l[b]; ++L) ctx->n_out[L]++;
  int v_off[EGNN_L_READOUT + 2] = {0};
  for (int L = 0; L <= EGNN_L_READOUT; ++L) v_off[L + 1] = v_off[L] + ctx->n_out[L];
  const int nq = ctx->n_orb * ctx->n_orb;
  std::vector<std::vector<std::pair<int, float>>> unc(nq);
  int running[EGNN_L_READOUT + 1] = {0};
  int qoff = 0;
  for (int a = 0; a < ns; ++a) {
    for (int b = 0; b < ns; ++b) {
      const int la = d->orb_l[a], lb = d->orb_l[b];
      for (int L = abs(la - lb); L <= la + lb; ++L) {
        ctx->slot_L.push_back(L);
        ctx->slot_vrow.push_back(v_off[L] + running[L]++);
        ctx->slot_qoff.push_back(qoff);
        const double* C = egnn_cg_values + egnn_cg_offset[la][lb][L];
        for (int ma = 0; ma < 2 * la + 1; ++ma)
          for (int mb = 0; mb < 2 * lb + 1; ++mb)
            for (int M = 0; M < 2 * L + 1; ++M) {
              const double cv = C[(ma * (2 * lb + 1) + mb) * (2 * L + 1) + M];
              if (cv != 0.0) unc[(orb_off[a] + ma) * ctx->n_orb + orb_off[b] + mb].push_back({qoff + M, (float)cv});
            }
        qoff += 2 * L + 1;
      }
    }
  }
  ctx->n_slots = (int)ctx->slot_L.size();
  ctx->unc_ptr.assign(nq + 1, 0);
  for (int q = 0; q < nq; ++q) {
    ctx->unc_ptr[q + 1] = ctx->unc_ptr[q] + (int)unc[q].size();
    for (auto& e : unc[q]) {
      ctx->unc_q.push_back(e.first);
      ctx->unc_c.push_back(e.second);
    }
  }
  egnn_static_scratch_prepare();   // set-up step of egnn_radial_weights_static (does nothing without a GPU)
  *out = ctx;
  return EGNN_OK;
}

extern "C" void egnn_destroy(egnn_ctx* ctx) {
  if (!ctx) return;
  // uploads of the context's index tables may still be queued: they read host memory that is freed below
  if (!ctx->tab_ro_i.empty() || !ctx->tab_rob_i.empty() || !ctx->tab_on_i.empty() || !ctx->tab_onb_i.empty())
    (void)hipDeviceSynchronize();
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  delete ctx;
}

// ---- stage timing ------------------------------------------------------------------------------
StageTimer::StageTimer(egnn_ctx* c, hipStream_t s, int kind) : ctx(c), st(s), slot(-1) {
  if (c->ev_max_calls > 0 && (int)c->ev_kind.size() < c->ev_max_calls) {
    slot = (int)c->ev_kind.size();
    c->ev_kind.push_back(kind);
    (void)hipEventRecord(c->ev[(size_t)slot * (EGNN_STAGES + 1)], st);
  }
}

void StageTimer::mark(int stage) {
  if (slot >= 0) (void)hipEventRecord(ctx->ev[(size_t)slot * (EGNN_STAGES + 1) + stage + 1], st);
}

extern "C" int egnn_timing_enable(egnn_ctx* ctx, int32_t max_calls) {
  if (!ctx || max_calls < 0 || max_calls > 65536) return EGNN_EINVAL;
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  ctx->ev.clear();
  ctx->ev_kind.clear();
  ctx->ev_max_calls = 0;
  for (int i = 0; i < max_calls * (EGNN_STAGES + 1); ++i) {
    hipEvent_t e;
    EGNN_HIP(ctx, hipEventCreate(&e));
    ctx->ev.push_back(e);
  }
  ctx->ev_max_calls = max_calls;
  return EGNN_OK;
}

extern "C" int egnn_timing_read(egnn_ctx* ctx, float ms[EGNN_TIMED_KINDS * EGNN_STAGES],
                                int32_t n_calls[EGNN_TIMED_KINDS]) {
  if (!ctx || !ms || !n_calls) return EGNN_EINVAL;
  for (int i = 0; i < EGNN_TIMED_KINDS * EGNN_STAGES; ++i) ms[i] = 0.0f;
  for (int i = 0; i < EGNN_TIMED_KINDS; ++i) n_calls[i] = 0;
  for (size_t c = 0; c < ctx->ev_kind.size(); ++c) {
    const int kind = ctx->ev_kind[c];
    hipEvent_t* e = &ctx->ev[c * (EGNN_STAGES + 1)];
    EGNN_HIP(ctx, hipEventSynchronize(e[EGNN_STAGES]));
    for (int s = 0; s < EGNN_STAGES; ++s) {
      float t = 0.0f;
      EGNN_HIP(ctx, hipEventElapsedTime(&t, e[s], e[s + 1]));
      ms[kind * EGNN_STAGES + s] += t;
    }
    n_calls[kind]++;
  }
  ctx->ev_kind.clear();
  return EGNN_OK;
}

extern "C" int egnn_set_option(egnn_ctx* ctx, int32_t option, int32_t value) {
  if (!ctx) return EGNN_EINVAL;
  if (option == EGNN_OPT_FUSED) {
    if (value < 0 || value > 2) return egnn_fail(ctx, EGNN_EINVAL, "set_option: EGNN_OPT_FUSED takes 0, 1 or 2");
    ctx->use_fused = value;
    return EGNN_OK;
  }
  if (option == EGNN_OPT_W_FP16) {
    ctx->w_half = value != 0;
    return EGNN_OK;
  }
  if (option == EGNN_OPT_RADIAL_BWD) {
    if (value < 0 || value > 2) return egnn_fail(ctx, EGNN_EINVAL, "set_option: EGNN_OPT_RADIAL_BWD takes 0, 1 or 2");
    ctx->radial_bwd_route = value;
    return EGNN_OK;
  }
  return egnn_fail(ctx, EGNN_EINVAL, "set_option: unknown option");
}

extern "C" const char* egnn_last_error(const egnn_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

extern "C" int egnn_path_count(const egnn_ctx* ctx, int which, int32_t* n_paths, int32_t* paths) {
  if (!ctx || !n_paths || which < 0 || which > 1) return EGNN_EINVAL;
  *n_paths = ctx->n_paths[which];
  if (paths)
    for (int p = 0; p < ctx->n_paths[which]; ++p)
      for (int t = 0; t < 3; ++t) paths[3 * p + t] = ctx->paths[which][p][t];
  return EGNN_OK;
}

extern "C" int egnn_readout_widths(const egnn_ctx* ctx, int32_t n_out[5]) {
  if (!ctx || !n_out) return EGNN_EINVAL;
  for (int L = 0; L <= EGNN_L_READOUT; ++L) n_out[L] = ctx->n_out[L];
  return EGNN_OK;
}

// ---- workspace carving -------------------------------------------------------------------------
struct Carver {
  char* base;
  size_t used;
  void* take(size_t bytes) {
    void* p = base ? base + used : nullptr;
    used += align256(bytes);
    return p;
  }
};

static size_t readout_tab_ints(const egnn_ctx* ctx) {
  const int nq = ctx->n_orb * ctx->n_orb;
  return (size_t)2 * nq + 2 * ctx->n_slots + nq + 1 + ctx->unc_q.size();
}

// the weight tensor of a layer, or the (much smaller, except for tiny models) scratch of the fused route in its place
size_t egnn_w_bytes(const egnn_ctx* ctx, int which, int64_t n_edges) {
  const int PE = ctx->n_paths[which] * ctx->desc.channels;
  const size_t full = (size_t)n_edges * PE * sizeof(float);
  const size_t half = (size_t)n_edges * w_half_row_words(PE) * sizeof(uint32_t);   // larger only for PE < 64
  return full > half ? full : half;
}

static size_t layer_w_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_total) {
  const size_t w = egnn_w_bytes(ctx, 0, n_edges);
  const size_t f = egnn_fused_supported(ctx) ? egnn_fused_scratch_bytes(ctx, n_edges) : 0;
  const size_t f2 = egnn_fused_lane_supported(ctx) ? egnn_fused_lane_scratch_bytes(ctx, n_total) : 0;
  const size_t m = w > f ? w : f;
  return m > f2 ? m : f2;
}

static size_t layer_ws(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, int32_t n_total, int with_w) {
  const size_t row = (size_t)(ctx->desc.lmax + 1) * (ctx->desc.lmax + 1) * ctx->desc.channels * sizeof(float);
  Carver c{nullptr, 0};
  c.take((size_t)n_edges * 16);
  c.take((size_t)n_total * row);
  c.take((size_t)n_owned * row);
  if (with_w) c.take(layer_w_bytes(ctx, n_edges, n_total));
  if (with_w) c.take(egnn_radial_ws_bytes(ctx, 0));
  if (with_w) c.take((size_t)n_edges * 16);   // records of the row-owning edges (graphs with shared rows)
  return c.used;
}

static size_t readout_ws(const egnn_ctx* ctx, int64_t n_edges, int32_t n_total) {
  const size_t row = (size_t)(ctx->desc.lmax + 1) * (ctx->desc.lmax + 1) * ctx->desc.channels * sizeof(float);
  Carver c{nullptr, 0};
  c.take((size_t)n_edges * 16);
  c.take((size_t)n_total * row);
  c.take((size_t)n_total * row);
  c.take(readout_tab_ints(ctx) * sizeof(int));
  c.take(ctx->unc_c.size() * sizeof(float));
  c.take(egnn_w_bytes(ctx, 1, n_edges));
  c.take(egnn_radial_ws_bytes(ctx, 1));
  c.take((size_t)n_edges * 16);               // records of the row-owning edges (graphs with shared rows)
  return c.used;
}

extern "C" int egnn_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, int32_t n_total,
                                    int with_weights, size_t* bytes) {
  if (!ctx || !bytes || n_edges < 0 || n_owned < 0 || n_total < n_owned) return EGNN_EINVAL;
  size_t a = layer_ws(ctx, n_edges, n_owned, n_total, with_weights);
  size_t b = ctx->n_orb > 0 ? readout_ws(ctx, n_edges, n_total) : 0;
  *bytes = (a > b ? a : b) + 256;
  return EGNN_OK;
}

static int check_graph(egnn_ctx* ctx, const egnn_graph* g, const char* who) {
  if (!g) return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": null graph");
  if (g->n_edges < 0 || g->n_edges > 2147483647LL || g->n_owned < 0 || g->n_total < g->n_owned)
    return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": bad graph sizes");
  if (!g->row_ptr || (g->n_edges > 0 && (!g->src || !g->dst)))
    return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": null graph arrays");
  if (g->w_row && (g->n_w_rows < 0 || g->n_w_rows > g->n_edges || (g->n_edges > 0 && g->n_w_rows == 0)))
    return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": n_w_rows does not fit the edge count");
  return EGNN_OK;
}

// ---- stage entry points ------------------------------------------------------------------------
extern "C" int egnn_edge_geometry(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                  float* rhat_d, float* Y, float* rbf, float* fc, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_graph(ctx, g, "edge_geometry");
  if (rc) return rc;
  if (!pos || !box || !rhat_d) return egnn_fail(ctx, EGNN_EINVAL, "edge_geometry: null pointer");
  return egnn_launch_geometry(ctx, g, pos, box, rhat_d, Y, rbf, fc, (hipStream_t)stream);
}

extern "C" int egnn_radial_weights(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges,
                                   const float* W_r1, const float* W_r2, float* w, void* ws, size_t ws_bytes,
                                   void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (which < 0 || which > 1 || n_edges < 0 || !rhat_d || !W_r1 || !W_r2 || !w || !ws)
    return egnn_fail(ctx, EGNN_EINVAL, "radial_weights: bad argument");
  if (((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "radial_weights: workspace not 256-byte aligned");
  if (ws_bytes < egnn_radial_ws_bytes(ctx, which)) return egnn_fail(ctx, EGNN_EWS, "radial_weights: workspace too small");
  return egnn_launch_radial(ctx, which, rhat_d, n_edges, W_r1, W_r2, w, ws, (hipStream_t)stream);
}

extern "C" int egnn_tp_segsum(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* h,
                              const float* w, float* a, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_graph(ctx, g, "tp_segsum");
  if (rc) return rc;
  if (!rhat_d || !h || !w || !a) return egnn_fail(ctx, EGNN_EINVAL, "tp_segsum: null pointer");
  return egnn_launch_tp_segsum(ctx, g, rhat_d, h, w, a, (hipStream_t)stream);
}

// the same two stages with w in half precision
extern "C" int egnn_radial_weights_f16(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges,
                                       const float* W_r1, const float* W_r2, uint32_t* w16, void* ws, size_t ws_bytes,
                                       void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (which < 0 || which > 1 || n_edges < 0 || !rhat_d || !W_r1 || !W_r2 || !w16 || !ws)
    return egnn_fail(ctx, EGNN_EINVAL, "radial_weights_f16: bad argument");
  if (((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "radial_weights_f16: workspace not 256-byte aligned");
  if (ws_bytes < egnn_radial_ws_bytes(ctx, which)) return egnn_fail(ctx, EGNN_EWS, "radial_weights_f16: workspace too small");
  return egnn_launch_radial(ctx, which, rhat_d, n_edges, W_r1, W_r2, reinterpret_cast<float*>(w16), ws,
                            (hipStream_t)stream, true);
}

extern "C" int egnn_tp_segsum_f16(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* h,
                                  const uint32_t* w16, float* a, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_graph(ctx, g, "tp_segsum_f16");
  if (rc) return rc;
  if (!rhat_d || !h || !w16 || !a) return egnn_fail(ctx, EGNN_EINVAL, "tp_segsum_f16: null pointer");
  return egnn_launch_tp_segsum(ctx, g, rhat_d, h, reinterpret_cast<const float*>(w16), a, (hipStream_t)stream, true);
}

extern "C" int egnn_tp_segsum_f16h(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const uint16_t* h16,
                                   const uint32_t* w16, float* a, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_graph(ctx, g, "tp_segsum_f16h");
  if (rc) return rc;
  if (!rhat_d || !h16 || !w16 || !a) return egnn_fail(ctx, EGNN_EINVAL, "tp_segsum_f16h: null pointer");
  return egnn_launch_tp_segsum(ctx, g, rhat_d, reinterpret_cast<const float*>(h16), reinterpret_cast<const float*>(w16), a,
                               (hipStream_t)stream, true, false, true);
}

extern "C" int egnn_node_mix(egnn_ctx* ctx, const float* x1, const float* W1, const float* x2, const float* W2,
                             float* y, int32_t n_nodes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!x1 || !W1 || !y || n_nodes < 0 || ((x2 == nullptr) != (W2 == nullptr)))
    return egnn_fail(ctx, EGNN_EINVAL, "node_mix: bad argument");
  return egnn_launch_node_mix(ctx, x1, W1, x2, W2, y, n_nodes, (hipStream_t)stream);
}

// ---- composite entry points ----------------------------------------------------------------------
// w_save / a_save (may be NULL): caller buffers that receive the weight tensor and the summed messages instead of the
// workspace (then the route through the materialised fp32 weights is taken whatever the options say)
static int layer_forward_impl(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                              const float* x_in, const float* W_pre, const float* W_post, const float* W_self,
                              const float* W_r1, const float* W_r2, const float* w_edge, float* x_out, float* w_save,
                              float* a_save, void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_graph(ctx, g, "layer_forward");
  if (rc) return rc;
  // (without owned nodes there is no output row: x_out may then be NULL)
  if (!pos || !box || !x_in || !W_pre || !W_post || !W_self || (!x_out && g->n_owned > 0) || !ws ||
      (!w_edge && (!W_r1 || !W_r2)))
    return egnn_fail(ctx, EGNN_EINVAL, "layer_forward: null pointer");
  if (x_in == x_out) return egnn_fail(ctx, EGNN_EINVAL, "layer_forward: x_out must not alias x_in");
  if (((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "layer_forward: workspace not 256-byte aligned");
  const int with_w = w_edge ? 0 : 1;
  if (ws_bytes < layer_ws(ctx, g->n_edges, g->n_owned, g->n_total, with_w))
    return egnn_fail(ctx, EGNN_EWS, "layer_forward: workspace too small");
  hipStream_t st = (hipStream_t)stream;
  const size_t row = (size_t)(ctx->desc.lmax + 1) * (ctx->desc.lmax + 1) * ctx->desc.channels * sizeof(float);
  Carver c{(char*)ws, 0};
  float* rhat_d = (float*)c.take((size_t)g->n_edges * 16);
  float* h = (float*)c.take((size_t)g->n_total * row);
  float* a = (float*)c.take((size_t)g->n_owned * row);
  const size_t w_bytes = with_w ? layer_w_bytes(ctx, g->n_edges, g->n_total) : 0;
  float* w = with_w ? (float*)c.take(w_bytes) : nullptr;
  const bool saving = w_save || a_save;
  if (w_save && with_w) w = w_save;
  if (a_save) a = a_save;
  void* w2s = with_w ? c.take(egnn_radial_ws_bytes(ctx, 0)) : nullptr;
  // shared rows (egnn_edge_pairs): S3 writes one row per row index, from the records of the row-owning edges
  const bool shared = with_w && g->w_row != nullptr;
  float* rd_rows = shared ? (float*)c.take((size_t)g->n_edges * 16) : nullptr;
  StageTimer tm(ctx, st, 0);
  if ((rc = egnn_launch_geometry(ctx, g, pos, box, rhat_d, nullptr, nullptr, nullptr, st, rd_rows))) return rc;
  tm.mark(0);
  // Default: S3 writes the weight tensor, S4 reads it.  Opt-in (EGNN_OPT_FUSED): the weights are produced and
  // consumed inside one kernel and never leave the chip.
  // (the scratch of the fused route lives where the weight tensor would be)
  const bool fused_lane = with_w && !saving && ctx->use_fused == 2 && egnn_fused_lane_supported(ctx);
  const bool fused = fused_lane || (with_w && !saving && ctx->use_fused == 1 && egnn_fused_supported(ctx));
  const bool half = with_w && !saving && !fused && ctx->w_half;   // storage precision of the weight tensor between S3 and S4
  if (fused) {
    if (g->n_edges > 0 && (rc = egnn_launch_split_w2(ctx, 0, W_r2, w2s, st))) return rc;
  } else if (with_w) {
    if ((rc = egnn_launch_radial(ctx, 0, shared ? rd_rows : rhat_d, shared ? g->n_w_rows : g->n_edges, W_r1, W_r2, w,
                                 w2s, st, half)))
      return rc;
  }
  tm.mark(1);
  if ((rc = egnn_launch_node_mix(ctx, x_in, W_pre, nullptr, nullptr, h, g->n_total, st))) return rc;
  tm.mark(2);
  if (fused_lane) {
    if ((rc = egnn_launch_layer_fused_lane(ctx, g, rhat_d, h, W_r1, W_r2, w, w_bytes, a, st))) return rc;
  } else if (fused) {
    if ((rc = egnn_launch_layer_fused(ctx, g, rhat_d, h, W_r1, w2s, w, w_bytes, a, st))) return rc;
  } else {
    if ((rc = egnn_launch_tp_segsum(ctx, g, rhat_d, h, with_w ? w : w_edge, a, st, half, shared))) return rc;
  }
  tm.mark(3);
  rc = egnn_launch_node_mix(ctx, a, W_post, x_in, W_self, x_out, g->n_owned, st);
  tm.mark(4);
  return rc;
}

extern "C" int egnn_layer_forward(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                  const float* x_in, const float* W_pre, const float* W_post, const float* W_self,
                                  const float* W_r1, const float* W_r2, const float* w_edge, float* x_out,
                                  void* ws, size_t ws_bytes, void* stream) {
  return layer_forward_impl(ctx, g, pos, box, x_in, W_pre, W_post, W_self, W_r1, W_r2, w_edge, x_out, nullptr, nullptr,
                            ws, ws_bytes, stream);
}

extern "C" int egnn_layer_forward_save(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                       const float* x_in, const float* W_pre, const float* W_post, const float* W_self,
                                       const float* W_r1, const float* W_r2, float* x_out, float* w_save, float* a_save,
                                       void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!w_save || !a_save || !W_r1 || !W_r2) return egnn_fail(ctx, EGNN_EINVAL, "layer_forward_save: null pointer");
  return layer_forward_impl(ctx, g, pos, box, x_in, W_pre, W_post, W_self, W_r1, W_r2, nullptr, x_out, w_save, a_save, ws,
                            ws_bytes, stream);
}

static int readout_hij_impl(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                            const float* x, const float* W_s, const float* W_t, const float* W_r1,
                            const float* W_r2, const float* V, float* H, float* w_save, void* ws, size_t ws_bytes,
                            void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_graph(ctx, g, "readout_hij");
  if (rc) return rc;
  if (ctx->n_orb <= 0 || ctx->n_orb > 32) return egnn_fail(ctx, EGNN_EINVAL, "readout_hij: need 1..32 orbitals per atom");
  // (a graph without edges has no blocks: H may then be NULL)
  if (!pos || !box || !x || !W_s || !W_t || !W_r1 || !W_r2 || !V || (!H && g->n_edges > 0) || !ws)
    return egnn_fail(ctx, EGNN_EINVAL, "readout_hij: null pointer");
  if (((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "readout_hij: workspace not 256-byte aligned");
  if (ws_bytes < readout_ws(ctx, g->n_edges, g->n_total)) return egnn_fail(ctx, EGNN_EWS, "readout_hij: workspace too small");
  hipStream_t st = (hipStream_t)stream;
  const size_t row = (size_t)(ctx->desc.lmax + 1) * (ctx->desc.lmax + 1) * ctx->desc.channels * sizeof(float);
  Carver c{(char*)ws, 0};
  float* rhat_d = (float*)c.take((size_t)g->n_edges * 16);
  float* zs = (float*)c.take((size_t)g->n_total * row);
  float* zt = (float*)c.take((size_t)g->n_total * row);
  int* tab_i = (int*)c.take(readout_tab_ints(ctx) * sizeof(int));
  float* tab_f = (float*)c.take(ctx->unc_c.size() * sizeof(float));
  float* w = (float*)c.take(egnn_w_bytes(ctx, 1, g->n_edges));
  void* w2s = c.take(egnn_radial_ws_bytes(ctx, 1));
  const bool shared = g->w_row != nullptr;
  float* rd_rows = shared ? (float*)c.take((size_t)g->n_edges * 16) : nullptr;
  const bool half = ctx->w_half && !w_save;
  if (w_save) w = w_save;

  // integer table: q_row[nq] q_vrow[nq] slot_L[n_slots] slot_qoff[n_slots] unc_ptr[nq+1] unc_q[nnz]
  const int nq = ctx->n_orb * ctx->n_orb;
  std::vector<int>& ti = ctx->tab_ro_i;
  if (ti.empty()) {
    ti.reserve(readout_tab_ints(ctx));
    std::vector<int> q_row(nq), q_vrow(nq);
    for (int s = 0; s < ctx->n_slots; ++s) {
      const int L = ctx->slot_L[s];
      for (int M = 0; M < 2 * L + 1; ++M) {
        q_row[ctx->slot_qoff[s] + M] = L * L + M;
        q_vrow[ctx->slot_qoff[s] + M] = ctx->slot_vrow[s];
      }
    }
    ti.insert(ti.end(), q_row.begin(), q_row.end());
    ti.insert(ti.end(), q_vrow.begin(), q_vrow.end());
    ti.insert(ti.end(), ctx->slot_L.begin(), ctx->slot_L.end());
    ti.insert(ti.end(), ctx->slot_qoff.begin(), ctx->slot_qoff.end());
    ti.insert(ti.end(), ctx->unc_ptr.begin(), ctx->unc_ptr.end());
    ti.insert(ti.end(), ctx->unc_q.begin(), ctx->unc_q.end());
  }
  // (sources owned by the context: no need to wait for the copies)
  EGNN_HIP(ctx, hipMemcpyAsync(tab_i, ti.data(), ti.size() * sizeof(int), hipMemcpyHostToDevice, st));
  EGNN_HIP(ctx, hipMemcpyAsync(tab_f, ctx->unc_c.data(), ctx->unc_c.size() * sizeof(float), hipMemcpyHostToDevice, st));

  StageTimer tm(ctx, st, 1);
  if ((rc = egnn_launch_geometry(ctx, g, pos, box, rhat_d, nullptr, nullptr, nullptr, st, rd_rows))) return rc;
  tm.mark(0);
  if ((rc = egnn_launch_radial(ctx, 1, shared ? rd_rows : rhat_d, shared ? g->n_w_rows : g->n_edges, W_r1, W_r2, w, w2s,
                               st, half)))
    return rc;
  tm.mark(1);
  if ((rc = egnn_launch_node_mix(ctx, x, W_s, nullptr, nullptr, zs, g->n_total, st))) return rc;
  tm.mark(2);
  if ((rc = egnn_launch_node_mix(ctx, x, W_t, nullptr, nullptr, zt, g->n_total, st))) return rc;
  tm.mark(3);
  rc = egnn_launch_readout(ctx, g, rhat_d, zs, zt, w, V, tab_i, tab_f, H, st, half, shared);
  tm.mark(4);
  return rc;
}

extern "C" int egnn_readout_hij(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                const float* x, const float* W_s, const float* W_t, const float* W_r1,
                                const float* W_r2, const float* V, float* H, void* ws, size_t ws_bytes,
                                void* stream) {
  return readout_hij_impl(ctx, g, pos, box, x, W_s, W_t, W_r1, W_r2, V, H, nullptr, ws, ws_bytes, stream);
}

extern "C" int egnn_readout_hij_save(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                     const float* x, const float* W_s, const float* W_t, const float* W_r1,
                                     const float* W_r2, const float* V, float* H, float* w_save, void* ws,
                                     size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!w_save && g && g->n_edges > 0) return egnn_fail(ctx, EGNN_EINVAL, "readout_hij_save: null pointer");
  return readout_hij_impl(ctx, g, pos, box, x, W_s, W_t, W_r1, W_r2, V, H, w_save, ws, ws_bytes, stream);
}
