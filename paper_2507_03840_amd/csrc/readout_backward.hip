// Reverse pass of S6 (H_ij readout), per edge.
//
// Forward (' = in the bond frame, rotated by D_k):  u = D^T Mid(D z ; w),  q[o][M] = sum_c V[o][c] u[(L,M)][c],
// H = C q.  Given dH:
//     dq = C^T dH,
//     dV[o][c]  += sum_M dq[o][M] u[(L,M)][c]              (summed over all edges)
//     du[(L,M)][c] = sum_o V[o][c] dq[o][M],   du' = D du
//     (gv', gw) = Mid^T(D z, w ; du'),   dz = D^T gv'   (per edge row; summed by source and by destination later)
// A group of E lanes works on one edge, lane = channel: every rotation runs per lane on all lanes alike.  The
// collapsed quantities are shared through LDS; the loops over the rows o of V run per coupled degree L with the
// (L, M) register index fixed at compile time.
#include "egnn_internal.h"
#include "bond_frame.h"

#define ROB_MAX_WG 1024   // workgroups (= partial results of dV)
#define ROB_D 25

struct ReadoutBwdTabs {
  const int* uncT_ptr;   // [nq+1]  CSR over collapsed values q: which H entries they feed
  const int* uncT_h;     // [nnz]
  const float* uncT_c;   // [nnz]
  const int* slot_L;     // [n_slots]
  const int* slot_qoff;  // [n_slots]
  const int* vrow_qoff;  // [n_vrows] offset of the (2L+1) values of the slot that uses row o of V
  int nq, n_slots, n_vrows, nnz;
  int v_off[EGNN_L_READOUT + 2];
};

// Synchronisation among the lanes of a slot: up to 64 channels the slot lies inside one wavefront, whose LDS accesses
// execute in program order, so a wave-level fence suffices and the waves of the workgroup run free of each other.
__device__ __forceinline__ void rob_slot_sync(int log2E) {
  if (log2E <= 6) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
  } else {
    __syncthreads();
  }
}

template <int L>
__device__ __forceinline__ void collapse_adjoint(const ReadoutBwdTabs& tb, const float* __restrict__ V,
                                                 const float* sq, const int* s_vq, float* sdV, const float* u,
                                                 float* du, int c, int log2E) {
  for (int o = tb.v_off[L]; o < tb.v_off[L + 1]; ++o) {
    const float* q = sq + s_vq[o];
    const float vv = V[((size_t)o << log2E) + c];
    float dot = 0.0f;
#pragma unroll
    for (int M = 0; M < 2 * L + 1; ++M) {
      const float qv = q[M];
      dot += qv * u[L * L + M];
      du[L * L + M] += vv * qv;
    }
    sdV[(o << log2E) + c] += dot;
  }
}

template <int LMAX>
__global__ __launch_bounds__(256) void readout_backward_kernel(
    const int* __restrict__ src, const int* __restrict__ dst, const float4* __restrict__ rhat_d,
    const float* __restrict__ zs, const float* __restrict__ zt, const float* __restrict__ w,
    const float* __restrict__ V, ReadoutBwdTabs tb, const float* __restrict__ dH, float* __restrict__ dz,
    float* __restrict__ dw, float* __restrict__ dV_partial, long n_edges, int log2E, int iters) {
  using Mid = typename ReadoutMid<LMAX>::T;
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  constexpr int P = Mid::P;
  extern __shared__ float smem[];
  const int E = 1 << log2E;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1), slot = tid >> log2E;
  const int n_slots = 256 >> log2E;
  float* sq = smem + (size_t)slot * tb.nq;                                           // [nq] per slot
  float* sdV = smem + (size_t)n_slots * tb.nq + ((size_t)slot * tb.n_vrows << log2E);  // [n_vrows][E] per slot
  for (int o = 0; o < tb.n_vrows; ++o) sdV[(o << log2E) + c] = 0.0f;
  // the index tables, once per workgroup
  int* s_ptr = reinterpret_cast<int*>(smem + (size_t)n_slots * tb.nq + ((size_t)n_slots * tb.n_vrows << log2E));  // [nq + 1]
  int* s_h = s_ptr + tb.nq + 1;                            // [nnz]
  float* s_c = reinterpret_cast<float*>(s_h + tb.nnz);     // [nnz]
  int* s_vq = reinterpret_cast<int*>(s_c + tb.nnz);        // [n_vrows]
  for (int i = tid; i <= tb.nq; i += 256) s_ptr[i] = tb.uncT_ptr[i];
  for (int i = tid; i < tb.nnz; i += 256) {
    s_h[i] = tb.uncT_h[i];
    s_c[i] = tb.uncT_c[i];
  }
  for (int i = tid; i < tb.n_vrows; i += 256) s_vq[i] = tb.vrow_qoff[i];
  __syncthreads();

  const long k_base = (long)blockIdx.x * n_slots * iters;
  for (int it = 0; it < iters; ++it) {
    const long k = k_base + (long)it * n_slots + slot;
    const bool live = k < n_edges;
    BondTrig t;
    float4 g = make_float4(0.f, 0.f, 1.f, 1.f);
    if (live) {
      g = rhat_d[k];
      egnn_bond_trig<4>(g.x, g.y, g.z, t);
      const float* hrow = dH + (size_t)k * tb.nq;
      for (int q = c; q < tb.nq; q += E) {
        float sum = 0.0f;
        for (int n = s_ptr[q]; n < s_ptr[q + 1]; ++n) sum += s_c[n] * hrow[s_h[n]];
        sq[q] = sum;
      }
    }
    rob_slot_sync(log2E);
    if (live) {
      const int s = src[k], d = dst[k];
      const float* zsp = zs + ((size_t)s * D << log2E) + c;
      const float* ztp = zt + ((size_t)d * D << log2E) + c;
      const float* wp = w + ((size_t)k * P << log2E) + c;
      float v[D], wr[P], u[ROB_D], du[ROB_D];
#pragma unroll
      for (int p = 0; p < P; ++p) wr[p] = wp[(size_t)p << log2E];
#pragma unroll
      for (int i = 0; i < D; ++i) v[i] = zsp[(size_t)i << log2E] + ztp[(size_t)i << log2E];
      egnn_to_bond_frame<LMAX>(v, t);
      Mid::run(v, wr, u);
      egnn_from_bond_frame<4>(u, t);
#pragma unroll
      for (int i = 0; i < ROB_D; ++i) du[i] = 0.0f;
      collapse_adjoint<0>(tb, V, sq, s_vq, sdV, u, du, c, log2E);
      collapse_adjoint<1>(tb, V, sq, s_vq, sdV, u, du, c, log2E);
      collapse_adjoint<2>(tb, V, sq, s_vq, sdV, u, du, c, log2E);
      collapse_adjoint<3>(tb, V, sq, s_vq, sdV, u, du, c, log2E);
      collapse_adjoint<4>(tb, V, sq, s_vq, sdV, u, du, c, log2E);
      egnn_to_bond_frame<4>(du, t);
      float gv[D], gw[P];
      Mid::run_bwd(v, wr, du, gv, gw);
      egnn_from_bond_frame<LMAX>(gv, t);
      float* dzp = dz + ((size_t)k * D << log2E) + c;
      float* dwp = dw + ((size_t)k * P << log2E) + c;
#pragma unroll
      for (int i = 0; i < D; ++i) __builtin_nontemporal_store(gv[i], dzp + ((size_t)i << log2E));
#pragma unroll
      for (int p = 0; p < P; ++p) __builtin_nontemporal_store(gw[p], dwp + ((size_t)p << log2E));
    }
    __syncthreads();
  }
  // one partial [n_vrows][E] per workgroup: its slots added in fixed order
  const int nv = tb.n_vrows << log2E;
  const float* all = smem + (size_t)n_slots * tb.nq;
  float* out = dV_partial + (size_t)blockIdx.x * nv;
  for (int idx = tid; idx < nv; idx += 256) {
    float sum = 0.0f;
    for (int sidx = 0; sidx < n_slots; ++sidx) sum += all[(size_t)sidx * nv + idx];
    out[idx] = sum;
  }
}

// edges are dealt to at most ROB_MAX_WG workgroups, `iters` rounds of (256 / channels) edges each
static int rob_iters(const egnn_ctx* ctx, int64_t n_edges) {
  const long n_slots = 256 / ctx->desc.channels;
  const long rounds = (n_edges + n_slots - 1) / n_slots;
  return (int)((rounds + ROB_MAX_WG - 1) / ROB_MAX_WG);
}

static long rob_grid(const egnn_ctx* ctx, int64_t n_edges) {
  if (n_edges == 0) return 0;
  const long per_wg = (long)(256 / ctx->desc.channels) * rob_iters(ctx, n_edges);
  return (n_edges + per_wg - 1) / per_wg;
}

static int rob_vrows(const egnn_ctx* ctx) {
  int n = 0;
  for (int L = 0; L <= EGNN_L_READOUT; ++L) n += ctx->n_out[L];
  return n;
}

size_t egnn_readout_backward_partial_bytes(const egnn_ctx* ctx, int64_t n_edges) {
  return (size_t)rob_grid(ctx, n_edges) * rob_vrows(ctx) * ctx->desc.channels * sizeof(float);
}

// tab_i layout: uncT_ptr[nq+1] uncT_h[nnz] slot_L[n_slots] slot_qoff[n_slots] vrow_qoff[n_vrows]; tab_f: uncT_c[nnz]
int egnn_launch_readout_backward(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* zs,
                                 const float* zt, const float* w, const float* V, const int* tab_i,
                                 const float* tab_f, const float* dH, float* dz, float* dw, float* dV,
                                 float* partial, hipStream_t stream) {
  const long n = g->n_edges;
  const int E = ctx->desc.channels;
  const int n_vrows = rob_vrows(ctx);
  if (n == 0) return egnn_launch_reduce_partials(ctx, partial, 0, (long)n_vrows * E, dV, 1.0f, stream);
  const int nq = ctx->n_orb * ctx->n_orb;
  const int nnz = (int)ctx->unc_q.size();
  ReadoutBwdTabs tb;
  tb.nq = nq;
  tb.n_slots = ctx->n_slots;
  tb.n_vrows = n_vrows;
  tb.nnz = nnz;
  tb.v_off[0] = 0;
  for (int L = 0; L <= EGNN_L_READOUT; ++L) tb.v_off[L + 1] = tb.v_off[L] + ctx->n_out[L];
  tb.uncT_ptr = tab_i;
  tb.uncT_h = tab_i + nq + 1;
  tb.slot_L = tb.uncT_h + nnz;
  tb.slot_qoff = tb.slot_L + ctx->n_slots;
  tb.vrow_qoff = tb.slot_qoff + ctx->n_slots;
  tb.uncT_c = tab_f;
  const int n_slots = 256 / E;
  const size_t shmem = ((size_t)n_slots * nq + (size_t)n_slots * n_vrows * E) * sizeof(float) +
                       ((size_t)nq + 1 + 2 * (size_t)nnz + n_vrows) * sizeof(int);
  const long grid_x = rob_grid(ctx, n);
  dim3 grid((unsigned)grid_x), block(256);
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
#define LAUNCH(L)                                                                                                 \
  do {                                                                                                            \
    if (shmem > 64 * 1024) {                                                                                      \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(readout_backward_kernel<L>),               \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);                 \
      if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(readout_backward_kernel)");         \
    }                                                                                                             \
    hipLaunchKernelGGL(readout_backward_kernel<L>, grid, block, shmem, stream, g->src, g->dst, rd, zs, zt, w, V, \
                       tb, dH, dz, dw, partial, n, ctx->log2_channels, rob_iters(ctx, n));                        \
  } while (0)
  switch (ctx->desc.lmax) {
    case 0: LAUNCH(0); break;
    case 1: LAUNCH(1); break;
    case 2: LAUNCH(2); break;
    case 3: LAUNCH(3); break;
    case 4: LAUNCH(4); break;
    default: return egnn_fail(ctx, EGNN_EINVAL, "readout_backward: lmax out of range");
  }
#undef LAUNCH
  EGNN_LAUNCH_CHECK(ctx, "readout_backward_kernel");
  return egnn_launch_reduce_partials(ctx, partial, (int)grid_x, (long)n_vrows * E, dV, 1.0f, stream);
}
