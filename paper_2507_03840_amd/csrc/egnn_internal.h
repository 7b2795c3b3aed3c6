// Internal declarations shared by the translation units of libegnn_hip.so (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>
#include "../../include/egnn.h"

#define EGNN_MAX_PATHS 64
#define EGNN_HIDDEN 64
#define EGNN_L_READOUT 4

// Cell grid of the neighbour search: periodic axes span the box, open axes the bounding box of the atoms.
struct CellGrid {
  double lo[3], inv_cell[3], box[3];
  int n[3], pbc[3];
  int n_cells;
};

struct egnn_ctx {
  egnn_model_desc desc;
  int n_paths[2];                        // 0: layers, 1: readout
  int paths[2][EGNN_MAX_PATHS][3];
  float alpha[2][EGNN_MAX_PATHS];        // 1/sqrt(#paths ending in the same l3)
  int log2_channels;
  // readout tables (host copies; uploaded into the workspace by egnn_readout_hij)
  int n_orb;
  int n_out[EGNN_L_READOUT + 1];         // rows of V per coupled degree
  int n_slots;                           // number of (alpha, beta, L) triples
  std::vector<int> slot_L, slot_vrow, slot_qoff;   // per slot: degree, row in packed V, offset of its 2L+1 values
  std::vector<int> unc_ptr, unc_q;       // CSR over the n_orb^2 outputs: indices into q
  std::vector<float> unc_c;              //   and coupling coefficients
  // optional stage timing (egnn_timing_enable): EGNN_STAGES+1 events per recorded composite call
  std::vector<hipEvent_t> ev;
  std::vector<int> ev_kind;              // per recorded call: 0 = layer, 1 = readout, 2 = layer adjoint, 3 = readout adjoint
  int ev_max_calls = 0;
  CellGrid nl_grid;                      // grid of the last egnn_nlist_count that used the cell list
  int nl_grid_atoms = -1;                //   and the atom count, workspace and positions it was built for
  const void* nl_grid_ws = nullptr;
  const void* nl_grid_pos = nullptr;
  int use_fused = 0;                     // egnn_set_option(EGNN_OPT_FUSED): 0 two kernels, 1 / 2 the fused designs
  bool w_half = false;                   // egnn_set_option(EGNN_OPT_W_FP16)
  int radial_bwd_route = 0;              // egnn_set_option(EGNN_OPT_RADIAL_BWD): 0 decided on the device, 1 exact, 2 grid
  // index tables of the readout / on-site kernels in the order the kernels read them, built on first use and kept:
  // the asynchronous uploads into the caller's workspace read this memory, which lives as long as the context
  std::vector<int> tab_ro_i, tab_rob_i, tab_on_i, tab_onb_i;
  std::vector<float> tab_rob_f, tab_onb_f;
  std::string err;
};

#define EGNN_CUS 256    // compute units of the GPU this library is written for
#define EGNN_STAGES 5   // stages per composite call
#define EGNN_TIMED_KINDS 4

// Records the event that closes stage `stage` (or opens the call for stage = -1) if timing is on.
struct StageTimer {
  egnn_ctx* ctx; hipStream_t st; int slot;
  StageTimer(egnn_ctx* c, hipStream_t s, int kind);
  void mark(int stage);
};

struct PathAlpha { float a[EGNN_MAX_PATHS]; };

int egnn_fail(egnn_ctx* ctx, int code, const std::string& msg);
int egnn_check_hip(egnn_ctx* ctx, hipError_t e, const char* what);

// A running maximum of non-negative floats kept in a word of device memory as a bit pattern (such floats order like
// their bit patterns): the atomic is issued only when it would raise the value -- atomics on one address run one
// after the other, and after the first few thousand wavefronts almost none is needed.
#ifdef __HIPCC__
// Row of the radial-weight tensor that edge k reads: k itself without shared rows, else the decoded entry of
// egnn_graph.w_row (r >= 0: the edge owns row r; r < 0: it reads row ~r, which belongs to its reverse).
__device__ __forceinline__ long egnn_weight_row(const int* __restrict__ w_row, long k) {
  if (!w_row) return k;
  const int r = w_row[k];
  return r < 0 ? ~r : r;
}
// Cosine cutoff f_c(d) = (1 + cos(pi d / r_cut)) / 2, evaluated as sin^2(pi (r_cut - d) / (2 r_cut)): the same function,
// but near the cutoff, where it tends to zero, 1 + cos(...) loses its relative accuracy to rounding (an absolute error
// of 6e-8 on a value of 1e-5), while r_cut - d is exact there and the square of a small sine is not.
__device__ __forceinline__ float egnn_envelope(float d, float r_cut) {
  const float s = sinf(1.57079632679489662f * (r_cut - d) / r_cut);
  return s * s;
}
__device__ __forceinline__ void egnn_raise_max(unsigned* target, float v) {
  const unsigned bits = __float_as_uint(v);
  if (bits > __atomic_load_n(target, __ATOMIC_RELAXED)) atomicMax(target, bits);
}
#endif

#define EGNN_HIP(ctx, call)                                              \
  do {                                                                   \
    hipError_t e__ = (call);                                             \
    if (e__ != hipSuccess) return egnn_check_hip(ctx, e__, #call);       \
  } while (0)

#define EGNN_LAUNCH_CHECK(ctx, name)                                     \
  do {                                                                   \
    hipError_t e__ = hipGetLastError();                                  \
    if (e__ != hipSuccess) return egnn_check_hip(ctx, e__, name);        \
  } while (0)

// stage launchers (one per translation unit)
int egnn_launch_node_mix(egnn_ctx*, const float* x1, const float* W1, const float* x2, const float* W2,
                         float* y, int n_nodes, hipStream_t, int transpose = 0);
int egnn_launch_mix_wgrad(egnn_ctx*, const float* dy, const float* x, float* dW, float* partial, int n_nodes,
                          hipStream_t);
size_t egnn_mix_wgrad_ws_bytes(const egnn_ctx*);
int egnn_launch_row_scan(egnn_ctx*, int* row_ptr, int n, hipStream_t);
int egnn_launch_fill_int(egnn_ctx*, int* p, long n, int v, hipStream_t);
int egnn_launch_segsum_rows(egnn_ctx*, const float* rows, const int* ptr, const int* perm, float* out, int n_segments,
                            int row_len, hipStream_t);
// skip (may be NULL): a device word; the kernels return at once if it is non-zero
int egnn_launch_reduce_partials(egnn_ctx*, float* partial /* scratch, may be overwritten */, int n_partials, long n, float* out, float scale,
                                hipStream_t, const int* skip = nullptr);
// the radial MLP's reverse pass by interpolation on a grid of distances (radial_grid.hip)
size_t egnn_radial_grid_ws_bytes(const egnn_ctx*, int which, int64_t n_edges);
int egnn_launch_radial_route(egnn_ctx*, const float* W_r1, int* route, hipStream_t);
int egnn_launch_length_bins(egnn_ctx*, const float4* rd, int64_t n_edges, int* bin_ptr, int* perm, int* key, int* bucket,
                            int* cursor, const int* route, hipStream_t);
int egnn_launch_radial_grid(egnn_ctx*, int which, const float* rhat_d, int64_t n_edges, const int* len_ptr,
                            const int* len_perm, const float* W_r1,
                            const float* W_r2, const float* dw, float* dW_r1, float* dW_r2, void* ws, const int* route,
                            int (*hidden_launch)(egnn_ctx*, const float*, long, const float*, float*, float*, hipStream_t),
                            hipStream_t);
size_t egnn_transpose_ws_bytes(int64_t n_edges, int32_t n_total);
// dw_max (may be NULL): a word the caller has set to zero; raised to the bit pattern of the largest |dw| written
int egnn_launch_tp_backward(egnn_ctx*, const egnn_graph*, const int* col_ptr, const int* perm, const float* rhat_d,
                            const float* h, const float* w, const float* da, float* dh, float* dw, unsigned* dw_max,
                            hipStream_t, bool shared_rows = false);
size_t egnn_radial_backward_ws_bytes(const egnn_ctx*, int which, int64_t n_edges);
// dw_max_valid: the first word of ws (egnn_radial_backward_dw_max) holds the bit pattern of the largest |dw|; the
// two large contractions then run on half-precision pieces, otherwise on bf16 pieces (which need no scaling)
// len_ptr / len_perm (may be NULL): the edges grouped by length interval (egnn_length_bins), for the grid route
int egnn_launch_radial_backward(egnn_ctx*, int which, const float* rhat_d, int64_t n_edges, const float* W_r1,
                                const float* W_r2, const float* dw, float* dW_r1, float* dW_r2, void* ws,
                                bool dw_max_valid, hipStream_t, const int* len_ptr = nullptr,
                                const int* len_perm = nullptr);
static inline unsigned* egnn_radial_backward_dw_max(void* ws) { return reinterpret_cast<unsigned*>(ws); }
size_t egnn_readout_backward_partial_bytes(const egnn_ctx*, int64_t n_edges);
size_t egnn_readout_backward_lds_bytes(const egnn_ctx*);
void egnn_readout_backward_q_layout(const egnn_ctx*, int* q_off, int* nqp);   // q_off[EGNN_L_READOUT + 2]
int egnn_launch_readout_backward(egnn_ctx*, const egnn_graph*, const float* rhat_d, const float* zs, const float* zt,
                                 const float* w, const float* V, const int* tab_i, const float* tab_f,
                                 const float* dH, float* dz, float* dw, float* dV, float* partial, hipStream_t,
                                 bool shared_rows = false);
// half = true: `w` holds half-precision weights in the layout of w_half.h (egnn_w_bytes sizes it)
// shared_rows = true: `w` has one row per entry of g->w_row (egnn_edge_pairs), else one per edge
// h_half = true (needs half): `h` holds half-precision values
int egnn_launch_tp_segsum(egnn_ctx*, const egnn_graph*, const float* rhat_d, const float* h, const float* w,
                          float* a, hipStream_t, bool half = false, bool shared_rows = false, bool h_half = false);
int egnn_launch_radial(egnn_ctx*, int which, const float* rhat_d, int64_t n_edges, const float* W_r1,
                       const float* W_r2, float* w, void* scratch, hipStream_t, bool half = false);
// looks up the address of the built-in scratch array of egnn_radial_weights_static on the current device, if there is one
void egnn_static_scratch_prepare();
size_t egnn_w_bytes(const egnn_ctx*, int which, int64_t n_edges);   // room for w in either precision
size_t egnn_radial_ws_bytes(const egnn_ctx*, int which);
int egnn_launch_split_w2(egnn_ctx*, int which, const float* W_r2, void* scratch, hipStream_t);
// scales[0..2] = s_w, s_g, 1 / (s_w s_g): the power-of-two scalings of the half-precision operand pieces
int egnn_launch_half_scales(egnn_ctx*, int which, const float* W_r1, const float* W_r2, float* scales, hipStream_t);
bool egnn_fused_supported(const egnn_ctx*);
bool egnn_fused_lane_supported(const egnn_ctx*);
size_t egnn_fused_lane_scratch_bytes(const egnn_ctx*, int32_t n_total);
int egnn_launch_layer_fused_lane(egnn_ctx*, const egnn_graph*, const float* rhat_d, const float* h, const float* W_r1,
                                 const float* W_r2, void* scratch, size_t scratch_bytes, float* a, hipStream_t);
size_t egnn_fused_scratch_bytes(const egnn_ctx*, int64_t n_edges);
int egnn_launch_layer_fused(egnn_ctx*, const egnn_graph*, const float* rhat_d, const float* h, const float* W_r1,
                            const void* W2s, void* scratch, size_t scratch_bytes, float* a, hipStream_t);
int egnn_launch_geometry(egnn_ctx*, const egnn_graph*, const float* pos, const float box[3], float* rhat_d,
                         float* Y, float* rbf, float* fc, hipStream_t, float* rd_rows = nullptr);
int egnn_launch_readout(egnn_ctx*, const egnn_graph*, const float* rhat_d, const float* zs, const float* zt,
                        const float* w, const float* V, const int* tab_i, const float* tab_f, float* H, hipStream_t,
                        bool half = false, bool shared_rows = false);
