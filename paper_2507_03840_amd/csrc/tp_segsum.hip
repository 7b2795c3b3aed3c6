// S4: tensor-product messages summed over the incoming edges of every owned node.
//
//   a[j][(l3,m3)][c] = nbar^-1/2 * sum_{k: dst(k)=j} sum_p w[k][p][c] sum_{m1,m2} C_p[m1][m2][m3]
//                      h[src(k)][(l1,m1)][c] Yhat_{l2,m2}(rhat_k)
//
// (message passing and aggregation of Sec. 3, with the coupling of Sec. 2.2 / Eq. 1 evaluated in the
// bond-aligned frame of Sec. 2.1 / Fig. 2(d)).
//
// Mapping: one workgroup per destination node; a lane owns one channel of one edge "slot"
// (256 / channels slots per workgroup), walks the node's edges with stride = #slots, and keeps the
// (lmax+1)^2 partial sums of its channel in registers.  Both streams it reads -- the weight row
// w[k][:][c] and the gathered source row h[src][:][c] -- are contiguous over the lanes of a slot.
// The slots are then added in a fixed order through LDS and the node row is written once, so the
// result does not depend on scheduling (no atomics).
#include "egnn_internal.h"
#include "bond_frame.h"
#include "w_half.h"

// HLE = 0: w in fp32, any channel count (log2E at run time).  HLE > 0: w in half precision (layout of w_half.h)
// for 2^HLE channels.  H16 (with HLE > 0): h holds IEEE half-precision values, same [node][(l,m)][channel] order
// (the paper's mixed-precision mode keeps the embeddings in half precision and the sums in fp32, Sec. 4.1).
template <int LMAX, int HLE, bool H16 = false>
__global__ __launch_bounds__(256) void tp_segsum_kernel(const int* __restrict__ row_ptr,
                                                        const int* __restrict__ src,
                                                        const float4* __restrict__ rhat_d,
                                                        const float* __restrict__ h,
                                                        const float* __restrict__ w,
                                                        const int* __restrict__ w_row,
                                                        float* __restrict__ a, int n_owned, int log2E,
                                                        int nodes_per_xcd, float scale) {
  using Mid = typename LayerMid<LMAX>::T;
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  constexpr int P = Mid::P;
  __shared__ float red[256 * D];

  // consecutive nodes (which share most of their sources) go to the same XCD, i.e. the same L2
  const int j = (blockIdx.x & 7) * nodes_per_xcd + (blockIdx.x >> 3);
  if (j >= n_owned || (int)(blockIdx.x >> 3) >= nodes_per_xcd) return;

  if (HLE) log2E = HLE;
  const int E = 1 << log2E;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1);
  const int slot = tid >> log2E;
  const int n_slots = 256 >> log2E;
  const int k0 = row_ptr[j], k1 = row_ptr[j + 1];

  float acc[D];
#pragma unroll
  for (int i = 0; i < D; ++i) acc[i] = 0.0f;

  // The indices of an edge (source, weight row) and its unit vector are fetched one edge ahead: the loads of the rows
  // they address then start at once instead of waiting out a second memory round trip per edge.
  int k = k0 + slot;
  int s = 0;
  size_t kw = 0;
  float4 g = make_float4(0.0f, 0.0f, 1.0f, 1.0f);
  if (k < k1) {
    s = src[k];
    g = rhat_d[k];
    kw = (size_t)egnn_weight_row(w_row, k);
  }
  for (; k < k1; k += n_slots) {
    float v[D], wr[P], o[D];
    if constexpr (HLE == 0) {
      const float* wp = w + (kw * P << log2E) + c;
#pragma unroll
      for (int p = 0; p < P; ++p) wr[p] = __builtin_nontemporal_load(wp + ((size_t)p << log2E));   // streamed once
    } else {
      w_half_load<P, HLE>(reinterpret_cast<const uint32_t*>(w) + kw * w_half_row_words(P << HLE), c, wr);
    }
    if constexpr (H16) {
      const _Float16* hp = reinterpret_cast<const _Float16*>(h) + ((size_t)s * D << log2E) + c;
#pragma unroll
      for (int i = 0; i < D; ++i) v[i] = (float)hp[(size_t)i << log2E];
    } else {
      const float* hp = h + ((size_t)s * D << log2E) + c;
#pragma unroll
      for (int i = 0; i < D; ++i) v[i] = hp[(size_t)i << log2E];
    }
    const float4 g_now = g;
    const int kn = k + n_slots;
    if (kn < k1) {
      s = src[kn];
      g = rhat_d[kn];
      kw = (size_t)egnn_weight_row(w_row, kn);
    }
    BondTrig t;
    egnn_bond_trig<LMAX>(g_now.x, g_now.y, g_now.z, t);
    egnn_to_bond_frame<LMAX>(v, t);
    Mid::run(v, wr, o);
    egnn_from_bond_frame<LMAX>(o, t);
#pragma unroll
    for (int i = 0; i < D; ++i) acc[i] += o[i];
  }

#pragma unroll
  for (int i = 0; i < D; ++i) red[((slot * D + i) << log2E) + c] = acc[i];
  __syncthreads();
  const int row = D << log2E;
  float* out = a + (size_t)j * row;
  for (int idx = tid; idx < row; idx += 256) {
    float sum = 0.0f;
    for (int s = 0; s < n_slots; ++s) sum += red[s * row + idx];
    out[idx] = sum * scale;
  }
}

int egnn_launch_tp_segsum(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* h,
                          const float* w, float* a, hipStream_t stream, bool half, bool shared_rows, bool h_half) {
  const int n = g->n_owned;
  if (n == 0) return EGNN_OK;
  const int per_xcd = (n + 7) / 8;
  dim3 grid(per_xcd * 8), block(256);
  const float scale = 1.0f / sqrtf(ctx->desc.agg_norm);
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
  const int* w_row = shared_rows ? g->w_row : nullptr;
  if (h_half && !half) return egnn_fail(ctx, EGNN_EINVAL, "tp_segsum: half-precision features need half-precision weights");
#define LAUNCH(L, H)                                                                                                  \
  do {                                                                                                                \
    if (h_half && H > 0)                                                                                              \
      hipLaunchKernelGGL((tp_segsum_kernel<L, H, (H > 0)>), grid, block, 0, stream, g->row_ptr, g->src, rd, h, w, w_row, \
                         a, n, ctx->log2_channels, per_xcd, scale);                                                   \
    else                                                                                                              \
      hipLaunchKernelGGL((tp_segsum_kernel<L, H, false>), grid, block, 0, stream, g->row_ptr, g->src, rd, h, w, w_row, \
                         a, n, ctx->log2_channels, per_xcd, scale);                                                   \
  } while (0)
#define CASE(L)                                                                                  \
  case L:                                                                                        \
    switch (half ? ctx->log2_channels : 0) {                                                     \
      case 0: LAUNCH(L, 0); break;                                                               \
      case 3: LAUNCH(L, 3); break;                                                               \
      case 4: LAUNCH(L, 4); break;                                                               \
      case 5: LAUNCH(L, 5); break;                                                               \
      case 6: LAUNCH(L, 6); break;                                                               \
      case 7: LAUNCH(L, 7); break;                                                               \
      default: return egnn_fail(ctx, EGNN_EINVAL, "tp_segsum: half-precision weights need 8..128 channels"); \
    }                                                                                            \
    break;
  switch (ctx->desc.lmax) {
    CASE(0) CASE(1) CASE(2) CASE(3) CASE(4)
    default: return egnn_fail(ctx, EGNN_EINVAL, "tp_segsum: lmax out of range");
  }
#undef CASE
#undef LAUNCH
  EGNN_LAUNCH_CHECK(ctx, "tp_segsum_kernel");
  return EGNN_OK;
}
