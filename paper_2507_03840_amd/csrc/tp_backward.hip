// Reverse pass of S4 (tensor-product messages + segmented sum).
//
// Forward, per edge k = (i -> j):  o_k = D_k^T Mid(D_k h_i ; w_k),  a_j = scale * sum_k o_k, with D_k the rotation
// into the bond frame.  Given da (gradient w.r.t. a):
//     go_k = scale * da_j,   (gv', gw_k) = Mid^T(D_k h_i, w_k ; D_k go_k),   dh_i = sum_{k: src(k)=i} D_k^T gv'.
// The sum over the outgoing edges of a source is what the forward pass does not have: edges are walked in
// source-sorted order (col_ptr / perm from egnn_graph_transpose), one workgroup per source node, partial sums
// in registers, slots added in fixed order -- the same shape as the forward kernel, no atomics.
// dw_k is written per edge (it feeds the radial-MLP gradients).
#include "egnn_internal.h"
#include "bond_frame.h"

// The adjoint of the bond-frame product, one input degree l1 at a time: the paths of a degree use one contiguous
// run of weights, so a run is loaded, turned into its part of the feature gradient and its own gradient, and stored
// before the next one is touched -- at most ten weights and ten weight gradients are live at once instead of 42 + 42,
// which is what lets two waves share a SIMD.
template <int LMAX, int L1>
struct TpBwdDegree {
  using Mid = typename LayerMid<LMAX>::T;
  __device__ __forceinline__ static void run(const float* v, const float* go, float* gv, const float* wr,
                                             float* __restrict__ dwp, int log2E, float& mx) {
    constexpr int first = Mid::CHUNK_FIRST[L1], count = Mid::CHUNK_COUNT[L1];
    float gw[count];
    Mid::template run_bwd_l1<L1>(v + L1 * L1, wr + first, go, gv + L1 * L1, gw);
#pragma unroll
    for (int p = 0; p < count; ++p) {
      __builtin_nontemporal_store(gw[p], dwp + ((size_t)(first + p) << log2E));
      mx = fmaxf(mx, fabsf(gw[p]));
    }
    if constexpr (L1 < LMAX) TpBwdDegree<LMAX, L1 + 1>::run(v, go, gv, wr, dwp, log2E, mx);
  }
};

// LE = log2(channels): a template parameter so that the row offsets of w, dw, h and da are immediates.
template <int LMAX, int LE>
__global__ __launch_bounds__(256, 2) void tp_backward_kernel(const int* __restrict__ col_ptr, const int* __restrict__ perm,
                                                             const int* __restrict__ dst,
                                                             const float4* __restrict__ rhat_d,
                                                             const float* __restrict__ h, const float* __restrict__ w,
                                                             const int* __restrict__ w_row,
                                                             const float* __restrict__ da, float* __restrict__ dh,
                                                             float* __restrict__ dw, unsigned* __restrict__ dw_max,
                                                             int n_total, int nodes_per_xcd, float scale) {
  constexpr int log2E = LE;
  using Mid = typename LayerMid<LMAX>::T;
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  constexpr int P = Mid::P;
  __shared__ float red[256 * D];

  const int i = (blockIdx.x & 7) * nodes_per_xcd + (blockIdx.x >> 3);
  if (i >= n_total) return;
  const int E = 1 << log2E;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1);
  const int slot = tid >> log2E;
  const int n_slots = 256 >> log2E;
  const int c0 = col_ptr[i], c1 = col_ptr[i + 1];

  float v0[D], acc[D];
  float mx = 0.0f;      // largest |dw| this thread writes (scaling of the contractions that read dw)
  const float* hp = h + ((size_t)i * D << log2E) + c;
#pragma unroll
  for (int q = 0; q < D; ++q) {
    v0[q] = hp[(size_t)q << log2E];
    acc[q] = 0.0f;
  }

  // The edge id, its destination, weight row and unit vector are fetched one edge ahead (a chain of three dependent
  // loads: position in the source's list -> edge -> destination / weight row), so that the row loads of an edge start
  // as soon as its turn comes.
  int k_nx = 0, j_nx = 0;
  size_t kw_nx = 0;
  float4 g_nx = make_float4(0.0f, 0.0f, 1.0f, 1.0f);
  if (c0 + slot < c1) {
    k_nx = perm[c0 + slot];
    j_nx = dst[k_nx];
    g_nx = rhat_d[k_nx];
    kw_nx = (size_t)egnn_weight_row(w_row, k_nx);
  }
  for (int idx = c0 + slot; idx < c1; idx += n_slots) {
    const int k = k_nx;
    const int j = j_nx;
    const float4 g = g_nx;
    const float* gp = da + ((size_t)j * D << log2E) + c;
    const float* wp = w + (kw_nx * P << log2E) + c;   // (dw stays one row per edge)
    float* dwp = dw + ((size_t)k * P << log2E) + c;
    float v[D], go[D], gv[D], wr[P];
#pragma unroll
    for (int p = 0; p < P; ++p) wr[p] = __builtin_nontemporal_load(wp + ((size_t)p << log2E));
#pragma unroll
    for (int q = 0; q < D; ++q) {
      v[q] = v0[q];
      go[q] = scale * gp[(size_t)q << log2E];
    }
    if (idx + n_slots < c1) {
      k_nx = perm[idx + n_slots];
      j_nx = dst[k_nx];
      g_nx = rhat_d[k_nx];
      kw_nx = (size_t)egnn_weight_row(w_row, k_nx);
    }
    BondTrig t;
    egnn_bond_trig<LMAX>(g.x, g.y, g.z, t);
    egnn_to_bond_frame<LMAX>(v, t);
    egnn_to_bond_frame<LMAX>(go, t);
    TpBwdDegree<LMAX, 0>::run(v, go, gv, wr, dwp, log2E, mx);
    egnn_from_bond_frame<LMAX>(gv, t);
#pragma unroll
    for (int q = 0; q < D; ++q) acc[q] += gv[q];
  }

  if (dw_max) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if ((tid & 63) == 0) egnn_raise_max(dw_max, mx);
  }
#pragma unroll
  for (int q = 0; q < D; ++q) red[((slot * D + q) << log2E) + c] = acc[q];
  __syncthreads();
  const int row = D << log2E;
  float* out = dh + (size_t)i * row;
  for (int idx = tid; idx < row; idx += 256) {
    float sum = 0.0f;
    for (int s = 0; s < n_slots; ++s) sum += red[s * row + idx];
    out[idx] = sum;
  }
}

int egnn_launch_tp_backward(egnn_ctx* ctx, const egnn_graph* g, const int* col_ptr, const int* perm,
                            const float* rhat_d, const float* h, const float* w, const float* da, float* dh,
                            float* dw, unsigned* dw_max, hipStream_t stream, bool shared_rows) {
  const int n = g->n_total;
  const int* w_row = shared_rows ? g->w_row : nullptr;
  if (n == 0) return EGNN_OK;
  const int per_xcd = (n + 7) / 8;
  dim3 grid(per_xcd * 8), block(256);
  const float scale = 1.0f / sqrtf(ctx->desc.agg_norm);
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
#define LAUNCH(L, LE_)                                                                                          \
  hipLaunchKernelGGL((tp_backward_kernel<L, LE_>), grid, block, 0, stream, col_ptr, perm, g->dst, rd, h, w, w_row, da, \
                     dh, dw, dw_max, n, per_xcd, scale)
#define CASES(L)                                                                        \
  switch (ctx->log2_channels) {                                                         \
    case 3: LAUNCH(L, 3); break;                                                        \
    case 4: LAUNCH(L, 4); break;                                                        \
    case 5: LAUNCH(L, 5); break;                                                        \
    case 6: LAUNCH(L, 6); break;                                                        \
    case 7: LAUNCH(L, 7); break;                                                        \
    default: return egnn_fail(ctx, EGNN_EINVAL, "tp_backward: channels out of range"); \
  }
  switch (ctx->desc.lmax) {
    case 0: CASES(0); break;
    case 1: CASES(1); break;
    case 2: CASES(2); break;
    case 3: CASES(3); break;
    case 4: CASES(4); break;
    default: return egnn_fail(ctx, EGNN_EINVAL, "tp_backward: lmax out of range");
  }
#undef CASES
#undef LAUNCH
  EGNN_LAUNCH_CHECK(ctx, "tp_backward_kernel");
  return EGNN_OK;
}
