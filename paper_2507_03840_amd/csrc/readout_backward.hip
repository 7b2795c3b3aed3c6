// Reverse pass of S6 (H_ij readout), per edge.
//
// Forward (' = in the bond frame, rotated by D_k):  u = D^T Mid(D z ; w),  q[o][M] = sum_c V[o][c] u[(L,M)][c],
// H = C q.  Given dH:
//     dq = C^T dH,
//     dV[o][c]  += sum_M dq[o][M] u[(L,M)][c]              (summed over all edges)
//     du[(L,M)][c] = sum_o V[o][c] dq[o][M],   du' = D du
//     (gv', gw) = Mid^T(D z, w ; du'),   dz = D^T gv'   (per edge row; summed by source and by destination later)
// A group of E lanes (a slot) works on one edge, lane = channel: every rotation runs per lane on all lanes alike.
// The edge's block of dH is staged in LDS (coalesced), dq is shared through LDS; the loops over the rows o of V run
// per coupled degree L with the (L, M) register index fixed at compile time.
#include "egnn_internal.h"
#include "bond_frame.h"

#define ROB_MAX_WG 8192   // workgroups (= partial results of dV): many short ones, so that the last round of
                          // resident workgroups is nearly as full as the others
#define ROB_D 25
#define ROB_R 4            // rows of V per group of the collapse adjoint

struct ReadoutBwdTabs {
  const int* uncT_ptr;   // [nq+1]  CSR over collapsed values q: which H entries they feed
  const int* uncT_h;     // [nnz]
  const float* uncT_c;   // [nnz]
  int nq, n_vrows, nnz;
  int nqp;                         // length of the array of collapsed values (= nq)
  int v_off[EGNN_L_READOUT + 2];   // first row of V of every coupled degree
  int q_off[EGNN_L_READOUT + 2];   // first collapsed value of every coupled degree: the values are numbered by row of
                                   // V, (row o of degree L, M) at q_off[L] + (o - v_off[L]) (2L+1) + M
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

// Adjoint of the collapse for the rows o of V that belong to coupled degree L.  V (when it fits: the kernel's VLDS),
// the collapsed gradients dq of the slot's edge (numbered by row of V) and the partial dV of the wavefront (one value
// per (row, channel)) sit in LDS, and every address is the lane's base plus a scalar: no look-up stands between a
// row and its values.  Up to 32
// channels a wavefront holds several edges of the same channel: their contributions to dV are added first (a
// butterfly below 32 lanes, then one exchange of the wavefront's halves that leaves the total of one row in the lower
// half and the total of the next row in the upper half), and both halves update the sum, each its own row.  Rows are
// taken four at a time; rows past the end of the degree repeat its last row with weight zero and are not written.
template <int L>
__device__ __forceinline__ void collapse_adjoint(const ReadoutBwdTabs& tb, const float* __restrict__ Vrows,
                                                 const float* __restrict__ sq, float* __restrict__ sdVw,
                                                 const float* u, float* du, int c, int wl, int log2E) {
  constexpr int W = 2 * L + 1;
  constexpr int R = ROB_R;
  const int E = 1 << log2E;
  const int log2Ew = log2E < 6 ? log2E : 6;
  const bool paired = log2E < 6;
  const int n = tb.v_off[L + 1] - tb.v_off[L];
  const float* q0 = sq + tb.q_off[L];
  const float* Vp = Vrows + (tb.v_off[L] << log2E) + c;
  // the lane's own element of the partial sum: its channel, and for the halves of a wavefront that share channels
  // the row that half ends up with
  const int half = paired ? wl >> 5 : 0;
  const bool writer = paired ? (wl & 31) < E : true;
  float* dvp = sdVw + (tb.v_off[L] << log2Ew) + (paired ? (wl & 31) : wl);
  for (int r0 = 0; r0 < n; r0 += R) {
    float dot[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const bool ok = r0 + r < n;
      const int rr = ok ? r0 + r : n - 1;
      const float* q = q0 + rr * W;
      const float vl = Vp[rr << log2E];
      const float v = ok ? vl : 0.0f;
      float dsum = 0.0f;
#pragma unroll
      for (int M = 0; M < W; ++M) {
        const float qv = q[M];
        dsum += qv * u[L * L + M];
        du[L * L + M] += v * qv;
      }
      dot[r] = dsum;
    }
    if (paired) {
      for (int off = E; off < 32; off <<= 1) {
#pragma unroll
        for (int r = 0; r < R; ++r) dot[r] += __shfl_xor(dot[r], off);
      }
#pragma unroll
      for (int r = 0; r < R; r += 2) {
        // lower half: dot[r] of both halves; upper half: dot[r + 1] of both halves
        const auto x = __builtin_amdgcn_permlane32_swap(__float_as_uint(dot[r]), __float_as_uint(dot[r + 1]), false, false);
        const float sum = __uint_as_float(x[0]) + __uint_as_float(x[1]);
        const int row = r0 + r + half;
        if (writer && row < n) dvp[row << log2Ew] += sum;
      }
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r)
        if (r0 + r < n) dvp[(r0 + r) << log2Ew] += dot[r];
    }
  }
}

// Numbering of the collapsed values of one edge in LDS and in the transposed uncoupling table: by row of V.
void egnn_readout_backward_q_layout(const egnn_ctx* ctx, int* q_off, int* nqp) {
  q_off[0] = 0;
  for (int L = 0; L <= EGNN_L_READOUT; ++L) q_off[L + 1] = q_off[L] + ctx->n_out[L] * (2 * L + 1);
  *nqp = q_off[EGNN_L_READOUT + 1];
}

// The bond-frame product and its adjoint, one input degree at a time.  The rows of z of a degree, of the rotated
// input and of the input gradient are its own, and its weight gradients are one contiguous run, so a degree is
// loaded, rotated, used and (in the adjoint) rotated back and stored before the next one is touched: the weights
// stay in registers throughout (a second read would come from HBM), but at most two nine-component rows and ten
// weight gradients are live next to them instead of everything at once.  The price is a second read of z (from
// cache) and a second rotation; the gain is that three waves share a SIMD and hide each other's latency.
template <int L1>
__device__ __forceinline__ void rob_load_rotate(const float* __restrict__ zsp, const float* __restrict__ ztp,
                                                const BondTrig& t, float* vl, int log2E) {
#pragma unroll
  for (int i = 0; i < 2 * L1 + 1; ++i)
    vl[i] = zsp[(size_t)(L1 * L1 + i) << log2E] + ztp[(size_t)(L1 * L1 + i) << log2E];
  egnn_to_bond_frame_l<L1>(vl, t);
}
template <int LMAX, int L1>
struct RobFwdDegree {
  using Mid = typename ReadoutMid<LMAX>::T;
  __device__ __forceinline__ static void run(const float* __restrict__ zsp, const float* __restrict__ ztp,
                                             const BondTrig& t, float* u, const float* wr, int log2E) {
    constexpr int first = Mid::CHUNK_FIRST[L1];
    float vl[2 * L1 + 1];
    rob_load_rotate<L1>(zsp, ztp, t, vl, log2E);
    Mid::template run_l1<L1>(vl, wr + first, u);
    if constexpr (L1 < LMAX) RobFwdDegree<LMAX, L1 + 1>::run(zsp, ztp, t, u, wr, log2E);
  }
};
template <int LMAX, int L1>
struct RobBwdDegree {
  using Mid = typename ReadoutMid<LMAX>::T;
  __device__ __forceinline__ static void run(const float* __restrict__ zsp, const float* __restrict__ ztp,
                                             const BondTrig& t, const float* du, const float* wr,
                                             float* __restrict__ dwp, float* __restrict__ dzp, bool live, int log2E) {
    constexpr int first = Mid::CHUNK_FIRST[L1], count = Mid::CHUNK_COUNT[L1];
    float vl[2 * L1 + 1], gvl[2 * L1 + 1], gw[count];
    rob_load_rotate<L1>(zsp, ztp, t, vl, log2E);
    Mid::template run_bwd_l1<L1>(vl, wr + first, du, gvl, gw);
    egnn_from_bond_frame_l<L1>(gvl, t);
    if (live) {
#pragma unroll
      for (int p = 0; p < count; ++p) __builtin_nontemporal_store(gw[p], dwp + ((size_t)(first + p) << log2E));
#pragma unroll
      for (int i = 0; i < 2 * L1 + 1; ++i) __builtin_nontemporal_store(gvl[i], dzp + ((size_t)(L1 * L1 + i) << log2E));
    }
    if constexpr (L1 < LMAX) RobBwdDegree<LMAX, L1 + 1>::run(zsp, ztp, t, du, wr, dwp, dzp, live, log2E);
  }
};

// LE = log2(channels): a template parameter so that the row offsets of w, z, dw and dz are immediates.
// VLDS: V staged in LDS (whenever it fits beside the other tiles); otherwise its rows are read through the cache.
template <int LMAX, int LE, bool VLDS>
__global__ __launch_bounds__(256, 3) void readout_backward_kernel(
    const int* __restrict__ src, const int* __restrict__ dst, const float4* __restrict__ rhat_d,
    const float* __restrict__ zs, const float* __restrict__ zt, const float* __restrict__ w,
    const int* __restrict__ w_row, const float* __restrict__ V, ReadoutBwdTabs tb, const float* __restrict__ dH, float* __restrict__ dz,
    float* __restrict__ dw, float* __restrict__ dV_partial, long n_edges, int iters) {
  constexpr int log2E = LE;
  using Mid = typename ReadoutMid<LMAX>::T;
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  constexpr int P = Mid::P;
  extern __shared__ float smem[];
  const int E = 1 << log2E;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1), slot = tid >> log2E;
  const int wl = tid & 63, wave = tid >> 6;
  const int n_slots = 256 >> log2E;
  const int log2Ew = log2E < 6 ? log2E : 6;                  // channels of a slot that one wavefront covers
  const int nvw = tb.n_vrows << log2Ew;
  float* sq = smem + (size_t)slot * tb.nqp;                                  // [nqp] per slot: dq
  float* sh = smem + (size_t)n_slots * tb.nqp + (size_t)slot * tb.nq;        // [nq] per slot: the edge's block of dH
  float* sdV_all = smem + (size_t)n_slots * (tb.nqp + tb.nq);                // [4 waves][n_vrows][2^log2Ew]
  float* sdVw = sdV_all + (size_t)wave * nvw;
  for (int i = wl; i < nvw; i += 64) sdVw[i] = 0.0f;
  // the index tables, once per workgroup
  int* s_ptr = reinterpret_cast<int*>(sdV_all + (size_t)4 * nvw);  // [nqp + 1]
  int* s_h = s_ptr + tb.nqp + 1;                           // [nnz]
  float* s_c = reinterpret_cast<float*>(s_h + tb.nnz);     // [nnz]
  for (int i = tid; i <= tb.nqp; i += 256) s_ptr[i] = tb.uncT_ptr[i];
  for (int i = tid; i < tb.nnz; i += 256) {
    s_h[i] = tb.uncT_h[i];
    s_c[i] = tb.uncT_c[i];
  }
  // V too: read from memory inside the loop over its rows, every group of rows would wait for a round trip to the
  // cache behind the stores of the edge before
  float* sV = s_c + tb.nnz;                                // [n_vrows][E]
  if (VLDS)
    for (int i = tid; i < (tb.n_vrows << log2E); i += 256) sV[i] = V[i];
  __syncthreads();

  const long k_base = (long)blockIdx.x * n_slots * iters;
  // (the weight row of an edge is looked up one edge ahead: its loads then do not wait for the index)
  size_t kw_nx;
  {
    const long k_first = k_base + slot;
    kw_nx = (size_t)egnn_weight_row(w_row, k_first < n_edges ? k_first : n_edges - 1);
  }
  for (int it = 0; it < iters; ++it) {
    // A slot past the end works on the last edge with dH = 0 (every lane takes part in the butterflies) and
    // stores nothing.
    const long k_own = k_base + (long)it * n_slots + slot;
    const bool live = k_own < n_edges;
    const long k = live ? k_own : n_edges - 1;
    // Every load of the edge that comes from HBM is issued here, ahead of the first wait: a wave's memory counter
    // retires loads and stores in issue order, so that wait also sits out the stores of the previous edge -- one
    // round trip per edge instead of one for dH and another for the weights.
    const float4 g = rhat_d[k];
    const int s = src[k], d = dst[k];
    const float* wp = w + (kw_nx * P << log2E) + c;   // (dw stays one row per edge)
    float wr[P];
#pragma unroll
    for (int p = 0; p < P; ++p) wr[p] = __builtin_nontemporal_load(wp + ((size_t)p << log2E));
    {
      const long k_next = k_own + n_slots;
      kw_nx = (size_t)egnn_weight_row(w_row, k_next < n_edges ? k_next : n_edges - 1);
    }
    {
      const float* hrow = dH + (size_t)k * tb.nq;
      for (int q = c; q < tb.nq; q += E) sh[q] = live ? hrow[q] : 0.0f;
    }
    rob_slot_sync(log2E);
    for (int q = c; q < tb.nqp; q += E) {
      float sum = 0.0f;
      for (int n = s_ptr[q]; n < s_ptr[q + 1]; ++n) sum += s_c[n] * sh[s_h[n]];
      sq[q] = sum;
    }
    rob_slot_sync(log2E);
    {
      BondTrig t;
      egnn_bond_trig<4>(g.x, g.y, g.z, t);
      const float* zsp = zs + ((size_t)s * D << log2E) + c;
      const float* ztp = zt + ((size_t)d * D << log2E) + c;
      float u[ROB_D], du[ROB_D];
#pragma unroll
      for (int i = 0; i < ROB_D; ++i) u[i] = 0.0f;
      RobFwdDegree<LMAX, 0>::run(zsp, ztp, t, u, wr, log2E);
      egnn_from_bond_frame<4>(u, t);
#pragma unroll
      for (int i = 0; i < ROB_D; ++i) du[i] = 0.0f;
      collapse_adjoint<0>(tb, VLDS ? sV : V, sq, sdVw, u, du, c, wl, log2E);
      collapse_adjoint<1>(tb, VLDS ? sV : V, sq, sdVw, u, du, c, wl, log2E);
      collapse_adjoint<2>(tb, VLDS ? sV : V, sq, sdVw, u, du, c, wl, log2E);
      collapse_adjoint<3>(tb, VLDS ? sV : V, sq, sdVw, u, du, c, wl, log2E);
      collapse_adjoint<4>(tb, VLDS ? sV : V, sq, sdVw, u, du, c, wl, log2E);
      egnn_to_bond_frame<4>(du, t);
      RobBwdDegree<LMAX, 0>::run(zsp, ztp, t, du, wr, dw + ((size_t)k * P << log2E) + c,
                                 dz + ((size_t)k * D << log2E) + c, live, log2E);
    }
    rob_slot_sync(log2E);   // sq and sh are rewritten by the next edge
  }
  __syncthreads();
  // one partial [n_vrows][E] per workgroup: the wavefronts that cover a channel added in fixed order
  const int nv = tb.n_vrows << log2E;
  const int waves_per_slot = E > 64 ? E >> 6 : 1;
  float* out = dV_partial + (size_t)blockIdx.x * nv;
  for (int idx = tid; idx < nv; idx += 256) {
    const int o = idx >> log2E, cc = idx & (E - 1);
    const int part = cc >> 6, cl = cc & ((1 << log2Ew) - 1);
    float sum = 0.0f;
    for (int wv = 0; wv < 4; ++wv)
      if ((wv & (waves_per_slot - 1)) == part) sum += sdV_all[(size_t)wv * nvw + (o << log2Ew) + cl];
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

// dynamic LDS of the kernel: dq and the block of dH per slot, one partial dV per wavefront, the index tables, and V
// if it is staged
static size_t rob_lds_bytes(const egnn_ctx* ctx, bool with_v) {
  const int E = ctx->desc.channels, n_slots = 256 / E, Ew = E < 64 ? E : 64;
  const size_t nq = (size_t)ctx->n_orb * ctx->n_orb, nnz = ctx->unc_q.size(), n_vrows = (size_t)rob_vrows(ctx);
  int q_off[EGNN_L_READOUT + 2], nqp;
  egnn_readout_backward_q_layout(ctx, q_off, &nqp);
  return (n_slots * (nqp + nq) + 4 * n_vrows * Ew + (with_v ? n_vrows * E : 0)) * sizeof(float) +
         ((size_t)nqp + 1 + 2 * nnz) * sizeof(int);
}

// what the kernel needs at least (a basis that needs more than a compute unit has cannot be served)
size_t egnn_readout_backward_lds_bytes(const egnn_ctx* ctx) { return rob_lds_bytes(ctx, false); }

size_t egnn_readout_backward_partial_bytes(const egnn_ctx* ctx, int64_t n_edges) {
  return (size_t)rob_grid(ctx, n_edges) * rob_vrows(ctx) * ctx->desc.channels * sizeof(float);
}

// tab_i layout: uncT_ptr[nqp+1] uncT_h[nnz]; tab_f: uncT_c[nnz]; the collapsed
// values are numbered as egnn_readout_backward_q_layout lays them out
int egnn_launch_readout_backward(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* zs,
                                 const float* zt, const float* w, const float* V, const int* tab_i,
                                 const float* tab_f, const float* dH, float* dz, float* dw, float* dV,
                                 float* partial, hipStream_t stream, bool shared_rows) {
  const long n = g->n_edges;
  const int* w_row = shared_rows ? g->w_row : nullptr;
  const int E = ctx->desc.channels;
  const int n_vrows = rob_vrows(ctx);
  if (n == 0) return egnn_launch_reduce_partials(ctx, partial, 0, (long)n_vrows * E, dV, 1.0f, stream);
  const int nq = ctx->n_orb * ctx->n_orb;
  const int nnz = (int)ctx->unc_q.size();
  ReadoutBwdTabs tb;
  tb.nq = nq;
  tb.n_vrows = n_vrows;
  tb.nnz = nnz;
  tb.v_off[0] = 0;
  for (int L = 0; L <= EGNN_L_READOUT; ++L) tb.v_off[L + 1] = tb.v_off[L] + ctx->n_out[L];
  egnn_readout_backward_q_layout(ctx, tb.q_off, &tb.nqp);
  tb.uncT_ptr = tab_i;
  tb.uncT_h = tab_i + tb.nqp + 1;
  tb.uncT_c = tab_f;
  const bool vlds = rob_lds_bytes(ctx, true) <= 160 * 1024;
  const size_t shmem = rob_lds_bytes(ctx, vlds);
  const long grid_x = rob_grid(ctx, n);
  dim3 grid((unsigned)grid_x), block(256);
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
#define LAUNCH(L, LE_)                                                                                            \
  do {                                                                                                            \
    auto kern = vlds ? readout_backward_kernel<L, LE_, true> : readout_backward_kernel<L, LE_, false>;            \
    if (shmem > 64 * 1024) {                                                                                      \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                     \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);                 \
      if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(readout_backward_kernel)");         \
    }                                                                                                             \
    hipLaunchKernelGGL(kern, grid, block, shmem, stream, g->src, g->dst, rd, zs, zt, w, w_row, V, tb, dH, dz, dw, \
                       partial, n, rob_iters(ctx, n));                                                            \
  } while (0)
#define CASES(L)                                                                \
  switch (ctx->log2_channels) {                                                 \
    case 3: LAUNCH(L, 3); break;                                                \
    case 4: LAUNCH(L, 4); break;                                                \
    case 5: LAUNCH(L, 5); break;                                                \
    case 6: LAUNCH(L, 6); break;                                                \
    case 7: LAUNCH(L, 7); break;                                                \
    default: return egnn_fail(ctx, EGNN_EINVAL, "readout_backward: channels out of range"); \
  }
  switch (ctx->desc.lmax) {
    case 0: CASES(0); break;
    case 1: CASES(1); break;
    case 2: CASES(2); break;
    case 3: CASES(3); break;
    case 4: CASES(4); break;
    default: return egnn_fail(ctx, EGNN_EINVAL, "readout_backward: lmax out of range");
  }
#undef CASES
#undef LAUNCH
  EGNN_LAUNCH_CHECK(ctx, "readout_backward_kernel");
  return egnn_launch_reduce_partials(ctx, partial, (int)grid_x, (long)n_vrows * E, dV, 1.0f, stream);
}
