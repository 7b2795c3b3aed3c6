// The message transform in its bond-aligned SO(2) form, summed over incoming edges
// (Fig. 2(a) bottom, Fig. 2(d); Sec. 3 "Message passing"; Sec. 2.1, last paragraph).
//
// Per directed edge k = (i -> j): the message is the concatenation [x_i | x_j | e_k] along the channel axis (3E
// channels), e_k being zero except for its L = 0 plane W_e B(d_k); it is rotated so that the bond lies on z, every
// order m goes through its own linear layer over (degree l >= |m|, channel),
//     y_0 = W_0 x_0;    y_{+m} = Wr_m x_{+m} - Wi_m x_{-m},   y_{-m} = Wi_m x_{+m} + Wr_m x_{-m}    (3E -> E channels),
// the result is rotated back, multiplied by the cutoff envelope and summed into the destination node (times
// agg_norm^-1/2).  Unlike the tensor-product route of the layer (per-edge weights, no channel mixing) this is a
// dense contraction shared by all edges, so it runs as five GEMMs, one per |m|:
//   1. so2_gather_kernel   lane = (edge, channel): both node rows rotated into the bond frame in registers, written
//                          m-major: A_0[k] = (x_{l,0} of both nodes for all l, then e_k), A_m[k] = [x_{+m} | x_{-m}];
//   2. so2_pack_kernel     the weights of order m as one matrix B_m = [[Wr^T, Wi^T], [-Wi^T, Wr^T]], scaled and cut
//                          into two half-precision pieces, stored in the operand order of the streaming GEMM
//                          (stream_gemm.h);
//   3. so2_gemmw_kernel    Y_m = A_m B_m on half-precision MFMA (three products per fp32 product), 256 edges x up to
//                          192 columns per workgroup: a row of A is fetched and cut once for all its column blocks;
//   4. so2_scatter_kernel  one workgroup per destination node, lane = (edge slot, channel): m-major rows of Y back to
//                          (l, m) order, rotated back, times f_c, summed; slots added in fixed order (no atomics).
#include <type_traits>
#include "egnn_internal.h"
#include "bond_frame.h"
#include "stream_gemm.h"

struct So2Bufs {
  float* A[5];
  float* Y[5];
  int K[5], N[5];       // columns of A_m and of Y_m
  int ldA[5], ldY[5];   // floats from one row to the next (so2_ld)
};

// Row pitch of the per-edge operands: the rows lie back to back.  (A pitch padded to an odd number of 128-byte lines,
// so that the same columns of consecutive rows fall into different channels of the L2 where the shapes of this layer
// give pitches of 8 or 16 lines, was measured: no gain for the weight gradient, 3-4 % slower forward.)
__host__ __device__ inline int so2_ld(int cols) { return cols; }

// columns of A_m: without persistent edge embeddings the edge slot exists only for l = 0 (its other planes are zero);
// with them (full) every degree carries [source | destination | edge]
__host__ __device__ inline int so2_K(int lmax, int E, int m, bool full = false) {
  if (full) return (m == 0 ? 1 : 2) * (lmax + 1 - m) * 3 * E;
  return m == 0 ? (lmax + 1) * 2 * E + E : 2 * (lmax + 1 - m) * 2 * E;
}
__host__ __device__ inline int so2_N(int lmax, int E, int m) { return m == 0 ? (lmax + 1) * E : 2 * (lmax + 1 - m) * E; }
// first float of order m in the packed weights: W_0, then (Wr_m, Wi_m) for m = 1..lmax
static size_t so2_w_offset(int lmax, int E, int m) {
  size_t off = 0;
  for (int q = 0; q < m; ++q) {
    const size_t nl = lmax + 1 - q;
    off += (q == 0 ? 1 : 2) * (nl * E) * (nl * 3 * E);
  }
  return off;
}

__device__ __forceinline__ void so2_raise_max(unsigned* target, float v) {
  const unsigned bits = __float_as_uint(v);
  if (bits > __atomic_load_n(target, __ATOMIC_RELAXED)) atomicMax(target, bits);
}

// ---------------------------------------------------------------------------------------------- 1. gather
// FULL: edge_in is the edge embedding tensor [n_edges][(LMAX+1)^2][E]; otherwise it is W_e [E][n_rbf]
template <int LMAX, bool FULL>
__global__ __launch_bounds__(256) void so2_gather_kernel(const int* __restrict__ src, const int* __restrict__ dst,
                                                         const float4* __restrict__ rhat_d, const float* __restrict__ x,
                                                         const float* __restrict__ edge_in, So2Bufs b, long n_edges,
                                                         int log2E, int n_rbf, float r_cut,
                                                         unsigned* __restrict__ a_max) {
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  const int E = 1 << log2E;
  const int c = threadIdx.x & (E - 1);
  const long k_own = (long)blockIdx.x * (256 >> log2E) + (threadIdx.x >> log2E);
  // (threads past the last edge repeat it and store nothing: every lane takes part in the reduction at the end)
  const bool live = k_own < n_edges;
  const long k = live ? k_own : n_edges - 1;
  float amax = 0.0f;     // largest magnitude this thread writes into the operands A_m (scaling of the GEMMs)
  const float4 g = rhat_d[k];
  const float* xs = x + (((size_t)src[k] * D) << log2E) + c;
  const float* xd = x + (((size_t)dst[k] * D) << log2E) + c;
  float vs[D], vd[D];
#pragma unroll
  for (int i = 0; i < D; ++i) {
    vs[i] = xs[(size_t)i << log2E];
    vd[i] = xd[(size_t)i << log2E];
  }
  BondTrig t;
  egnn_bond_trig<LMAX>(g.x, g.y, g.z, t);
  egnn_to_bond_frame<LMAX>(vs, t);
  egnn_to_bond_frame<LMAX>(vd, t);
#pragma unroll
  for (int i = 0; i < D; ++i) amax = fmaxf(amax, fmaxf(fabsf(vs[i]), fabsf(vd[i])));
  if constexpr (FULL) {
    float ve[D];
    const float* te = edge_in + (((size_t)k * D) << log2E) + c;
#pragma unroll
    for (int i = 0; i < D; ++i) ve[i] = __builtin_nontemporal_load(te + ((size_t)i << log2E));
    egnn_to_bond_frame<LMAX>(ve, t);
#pragma unroll
    for (int i = 0; i < D; ++i) amax = fmaxf(amax, fabsf(ve[i]));
    if (live) {
      float* a0 = b.A[0] + (size_t)k * b.ldA[0] + c;
#pragma unroll
      for (int l = 0; l <= LMAX; ++l) {
        __builtin_nontemporal_store(vs[l * l + l], a0 + ((3 * l) << log2E));
        __builtin_nontemporal_store(vd[l * l + l], a0 + ((3 * l + 1) << log2E));
        __builtin_nontemporal_store(ve[l * l + l], a0 + ((3 * l + 2) << log2E));
      }
#pragma unroll
      for (int m = 1; m <= LMAX; ++m) {
        const int nl = LMAX + 1 - m;
        float* am = b.A[m] + (size_t)k * b.ldA[m] + c;
#pragma unroll
        for (int l = m; l <= LMAX; ++l) {
          const int col = (3 * (l - m)) << log2E, neg = (3 * nl) << log2E;
          __builtin_nontemporal_store(vs[l * l + l + m], am + col);
          __builtin_nontemporal_store(vd[l * l + l + m], am + col + E);
          __builtin_nontemporal_store(ve[l * l + l + m], am + col + 2 * E);
          __builtin_nontemporal_store(vs[l * l + l - m], am + neg + col);
          __builtin_nontemporal_store(vd[l * l + l - m], am + neg + col + E);
          __builtin_nontemporal_store(ve[l * l + l - m], am + neg + col + 2 * E);
        }
      }
    }
  } else {
    // L = 0 plane of the edge embedding: a linear map of the Gaussian expansion of the length
    const float step = r_cut / (float)(n_rbf - 1);
    const float inv2s2 = 0.5f / (step * step);
    float e0 = 0.0f;
    for (int q = 0; q < n_rbf; ++q) {
      const float u = g.w - (float)q * step;
      e0 += edge_in[c * n_rbf + q] * __expf(-u * u * inv2s2);
    }
    amax = fmaxf(amax, fabsf(e0));
    if (live) {
      float* a0 = b.A[0] + (size_t)k * b.ldA[0] + c;
#pragma unroll
      for (int l = 0; l <= LMAX; ++l) {
        __builtin_nontemporal_store(vs[l * l + l], a0 + ((2 * l) << log2E));
        __builtin_nontemporal_store(vd[l * l + l], a0 + ((2 * l + 1) << log2E));
      }
      __builtin_nontemporal_store(e0, a0 + ((2 * (LMAX + 1)) << log2E));
#pragma unroll
      for (int m = 1; m <= LMAX; ++m) {
        const int nl = LMAX + 1 - m;
        float* am = b.A[m] + (size_t)k * b.ldA[m] + c;
#pragma unroll
        for (int l = m; l <= LMAX; ++l) {
          const int col = (2 * (l - m)) << log2E;
          __builtin_nontemporal_store(vs[l * l + l + m], am + col);
          __builtin_nontemporal_store(vd[l * l + l + m], am + col + E);
          __builtin_nontemporal_store(vs[l * l + l - m], am + ((2 * nl) << log2E) + col);
          __builtin_nontemporal_store(vd[l * l + l - m], am + ((2 * nl) << log2E) + col + E);
        }
      }
    }
  }
  // the wavefront's largest value raises the global one with an integer atomic (non-negative floats order like their
  // bit patterns) -- only if it is larger than what is there already, which after the first few thousand wavefronts
  // it almost never is: atomics on one address run one after the other
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
  if ((threadIdx.x & 63) == 0) so2_raise_max(a_max, amax);
}

// largest magnitude of the weights of all orders (they share one scaling), by integer atomics as above
__global__ __launch_bounds__(256) void so2_wmax_kernel(const float* __restrict__ W, long n_w, unsigned* __restrict__ w_max) {
  float mx = 0.0f;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n_w; i += (long)gridDim.x * 256) mx = fmaxf(mx, fabsf(W[i]));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if ((threadIdx.x & 63) == 0) so2_raise_max(w_max, mx);
}

// The initial edge embedding (Sec. 3 "Initialization"): L = 0 plane = W_e B(d_k), zeros elsewhere.
__global__ __launch_bounds__(256) void so2_edge_init_kernel(const float4* __restrict__ rhat_d, const float* __restrict__ W_e,
                                                            float* __restrict__ T_edge, long n_edges, int D, int log2E,
                                                            int n_rbf, float r_cut) {
  const int E = 1 << log2E;
  const int c = threadIdx.x & (E - 1);
  const long k = (long)blockIdx.x * (256 >> log2E) + (threadIdx.x >> log2E);
  if (k >= n_edges) return;
  const float d = rhat_d[k].w;
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
  float e0 = 0.0f;
  for (int q = 0; q < n_rbf; ++q) {
    const float u = d - (float)q * step;
    e0 += W_e[c * n_rbf + q] * __expf(-u * u * inv2s2);
  }
  float* te = T_edge + (((size_t)k * D) << log2E) + c;
  te[0] = e0;
  for (int i = 1; i < D; ++i) te[(size_t)i << log2E] = 0.0f;
}

// ---------------------------------------------------------------------------------------------- 2. weights
// B_m[k][n] for the column order of A_m (k) and of Y_m (n); W points at W_0 (m = 0) or at Wr_m (Wi_m follows it)
__device__ __forceinline__ float so2_b_value(const float* __restrict__ W, int m, int lmax, int E, int k, int n, int K, int N,
                                             bool full) {
  if (k >= K || n >= N) return 0.0f;
  if (full) {
    // the columns of A_m are in the column order of the weights: (l_in - m) 3E + g E + c, +m half then -m half
    const int nl = lmax + 1 - m;
    const int half_k = nl * 3 * E, half_n = nl * E;
    if (m == 0) return W[(size_t)n * half_k + k];
    const int s_in = k / half_k, col = k - s_in * half_k;
    const int s_out = n / half_n, row = n - s_out * half_n;
    const size_t at = (size_t)row * half_k + col, sz = (size_t)half_n * half_k;
    if (s_in == s_out) return W[at];
    return s_in == 0 ? W[sz + at] : -W[sz + at];
  }
  if (m == 0) {
    const int edge0 = (lmax + 1) * 2 * E;
    int col;
    if (k < edge0) {
      const int l = k / (2 * E);
      col = l * 3 * E + (k - l * 2 * E);     // g E + c with g in {0, 1}
    } else {
      col = 2 * E + (k - edge0);             // l = 0, g = 2: the edge embedding
    }
    return W[(size_t)n * ((lmax + 1) * 3 * E) + col];
  }
  const int nl = lmax + 1 - m;
  const int half_k = nl * 2 * E, half_n = nl * E;
  const int s_in = k / half_k, kr = k - s_in * half_k;
  const int li = kr / (2 * E);
  const int col = li * 3 * E + (kr - li * 2 * E);
  const int s_out = n / half_n, row = n - s_out * half_n;
  const size_t at = (size_t)row * (nl * 3 * E) + col;
  const size_t sz = (size_t)half_n * (nl * 3 * E);
  if (s_in == s_out) return W[at];                     // Wr
  return s_in == 0 ? W[sz + at] : -W[sz + at];         // x_{+m} -> y_{-m}: +Wi;  x_{-m} -> y_{+m}: -Wi
}

// T[ct][step][j][piece][64] halves (two pieces: see stream_gemm.h): thread -> (ct, step, j, pair of contraction indices)
__global__ __launch_bounds__(256) void so2_pack_kernel(const float* __restrict__ W, uint16_t* __restrict__ T, int m, int lmax,
                                                       int E, int K, int N, int n_steps, int n_ct, bool full,
                                                       const unsigned* __restrict__ w_max, bool transposed) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  const long total = (long)n_ct * n_steps * 64 * 32;
  if (i >= total) return;
  const int rp = (int)(i & 31), j = (int)((i >> 5) & 63);
  const long blk = i >> 11;                    // ct * n_steps + step
  const int step = (int)(blk % n_steps), ct = (int)(blk / n_steps);
  const int n = ct * 64 + j, k = step * 64 + 2 * rp;
  const float sc = ldexpf(1.0f, sgh_scale_exp(*w_max));
  // transposed: the operand is B_m^T (contraction over the columns of Y_m, one output column per column of A_m)
  const float xv[8] = {transposed ? so2_b_value(W, m, lmax, E, n, k, K, N, full) : so2_b_value(W, m, lmax, E, k, n, K, N, full),
                       transposed ? so2_b_value(W, m, lmax, E, n, k + 1, K, N, full)
                                  : so2_b_value(W, m, lmax, E, k + 1, n, K, N, full),
                       0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
  uint4 hi, lo;
  sgh_split8(xv, sc, hi, lo);
  uint32_t* o = reinterpret_cast<uint32_t*>(T) + blk * (64 * 64) + j * 64 + rp;
  o[0] = hi.x;
  o[32] = lo.x;
}

// ---------------------------------------------------------------------------------------------- 3. GEMM
// C[e][n] = sum_k A[e][k] B[k][n] with wide column tiles (sghw_contract of stream_gemm.h): a workgroup = (block of
// 32 * SG_WAVES rows, wide tile of NCB / 2 packed 64-column tiles); a wave owns 32 rows, whose 32 x 64 tile of A per
// step is fetched in memory order, turned to operand order through a private LDS tile and cut into pieces once for
// all column blocks.  Workgroup ids go round-robin over the 8 XCDs, each with its own L2, so the id is decoded such
// that the wide tiles of one block of rows (there is more than one only beyond 192 columns) sit on the same XCD with
// consecutive dispatch slots: they read the same rows of A, once from HBM and then from that L2.
template <int NCB>
__global__ __launch_bounds__(SG_THREADS) void so2_gemmw_kernel(const float* __restrict__ A, long M, int K, int lda,
                                                               const uint16_t* __restrict__ T, int n_steps,
                                                               float* __restrict__ C, int N, int ldc, int n_ct, int n_wt,
                                                               int n_row_blocks, const unsigned* __restrict__ maxima) {
  extern __shared__ uint4 so2_smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
  const int wt = idx % n_wt;
  const int row_block = (idx / n_wt) * 8 + xcd;
  if (row_block >= n_row_blocks) return;   // (whole workgroup: the grid is rounded up to a multiple of 8 row blocks)
  const long e_base = ((long)row_block * SG_WAVES + wave) * 32;
  const int ct0 = wt * (NCB / 2);
  const int ea = sgh_scale_exp(maxima[0]), eb = sgh_scale_exp(maxima[1]);
  const float a_scale = ldexpf(1.0f, ea), unscale = ldexpf(1.0f, -ea - eb);
  float16v acc[NCB];
  const long tile_stride = (long)n_steps * (64 * 16);
  sghw_contract<NCB>(A, M, K, lda, reinterpret_cast<const uint4*>(T) + (long)ct0 * tile_stride, tile_stride, n_ct - ct0,
                     n_steps, so2_smem, e_base, a_scale, acc);
  const int m = lane & 31, hh = lane >> 5;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int col = ct0 * 64 + cb * 32 + m;
    if (col < N) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const long e = e_base + 8 * (i >> 2) + 4 * hh + (i & 3);
        if (e < M) C[(size_t)e * ldc + col] = unscale * acc[cb][i];
      }
    }
  }
}

// launches the wide-tile product: NCB from the number of 64-column tiles (at most 6 column blocks per wave)
static int so2_launch_gemm(egnn_ctx* ctx, const float* A, long n, int K, int lda, const uint16_t* T, float* C, int N,
                           int ldc, const unsigned* maxima, hipStream_t st) {
  const int n_steps = (K + 63) / 64, n_ct = (N + 63) / 64;
  const int n_wt = (n_ct + 2) / 3;                // wide tiles of at most three 64-column tiles, evenly filled
  const int nt = (n_ct + n_wt - 1) / n_wt;
  const long rows_per_wg = 32L * SG_WAVES;
  const int n_row_blocks = (int)((n + rows_per_wg - 1) / rows_per_wg);
  const unsigned grid_x = (unsigned)(((n_row_blocks + 7) / 8) * 8 * n_wt);
#define SO2_GEMMW(NCB)                                                                                               \
  do {                                                                                                               \
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(so2_gemmw_kernel<NCB>),                         \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)SGHW_LDS_BYTES(NCB));        \
    if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(so2_gemmw_kernel)");                     \
    hipLaunchKernelGGL(so2_gemmw_kernel<NCB>, dim3(grid_x), dim3(SG_THREADS), SGHW_LDS_BYTES(NCB), st, A, n, K, lda,  \
                       T, n_steps, C, N, ldc, n_ct, n_wt, n_row_blocks, maxima);                                     \
  } while (0)
  switch (nt) {
    case 1: SO2_GEMMW(2); break;
    case 2: SO2_GEMMW(4); break;
    default: SO2_GEMMW(6); break;
  }
#undef SO2_GEMMW
  EGNN_LAUNCH_CHECK(ctx, "so2_gemmw_kernel");
  return EGNN_OK;
}

// ---------------------------------------------------------------------------------------------- 4. scatter
// bond-frame rows of Y (m-major) of edge k, channel c -> o[(l, m)] in the lab frame
template <int LMAX>
__device__ __forceinline__ void so2_load_rotate_back(const So2Bufs& b, long k, int c, int log2E, const float4& g, float* o) {
  const float* y0 = b.Y[0] + (size_t)k * b.ldY[0] + c;
#pragma unroll
  for (int l = 0; l <= LMAX; ++l) o[l * l + l] = __builtin_nontemporal_load(y0 + (l << log2E));
#pragma unroll
  for (int m = 1; m <= LMAX; ++m) {
    const int nl = LMAX + 1 - m;
    const float* ym = b.Y[m] + (size_t)k * b.ldY[m] + c;
#pragma unroll
    for (int l = m; l <= LMAX; ++l) {
      o[l * l + l + m] = __builtin_nontemporal_load(ym + ((l - m) << log2E));
      o[l * l + l - m] = __builtin_nontemporal_load(ym + ((nl + l - m) << log2E));
    }
  }
  BondTrig t;
  egnn_bond_trig<LMAX>(g.x, g.y, g.z, t);
  egnn_from_bond_frame<LMAX>(o, t);
}

// alpha != NULL: every message is weighted by its attention weight as well
template <int LMAX>
__global__ __launch_bounds__(256) void so2_scatter_kernel(const int* __restrict__ row_ptr, const float4* __restrict__ rhat_d,
                                                          So2Bufs b, const float* __restrict__ alpha,
                                                          float* __restrict__ a, int n_owned, int log2E,
                                                          int nodes_per_xcd, float scale, float r_cut) {
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  __shared__ float red[256 * D];
  const int j = (blockIdx.x & 7) * nodes_per_xcd + (blockIdx.x >> 3);
  if (j >= n_owned || (int)(blockIdx.x >> 3) >= nodes_per_xcd) return;
  const int E = 1 << log2E;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1), slot = tid >> log2E, n_slots = 256 >> log2E;
  const int k0 = row_ptr[j], k1 = row_ptr[j + 1];
  float acc[D];
#pragma unroll
  for (int i = 0; i < D; ++i) acc[i] = 0.0f;
  for (int k = k0 + slot; k < k1; k += n_slots) {
    const float4 g = rhat_d[k];
    float o[D];
    so2_load_rotate_back<LMAX>(b, k, c, log2E, g, o);
    float fc = egnn_envelope(g.w, r_cut);
    if (alpha) fc *= alpha[k];
#pragma unroll
    for (int i = 0; i < D; ++i) acc[i] += fc * o[i];
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

// ---------------------------------------------------------------------------------------------- 5. attention
// One wavefront per destination node: score of an incoming edge from the L = 0 plane of its transformed message (the
// first E columns of Y_0; that plane is the same in the bond frame and in the lab frame), softmax over the node's edges.
__global__ __launch_bounds__(256) void so2_attention_kernel(const int* __restrict__ row_ptr, const float* __restrict__ Y0,
                                                            int N0, const float* __restrict__ w_att,
                                                            float* __restrict__ alpha, int n_owned, int E) {
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= n_owned) return;
  const int k0 = row_ptr[j], k1 = row_ptr[j + 1];
  float mx = -3.0e38f;
  for (int k = k0 + lane; k < k1; k += 64) {
    const float* y = Y0 + (size_t)k * N0;
    float sc = 0.0f;
    for (int c = 0; c < E; ++c) {
      const float v = y[c];
      sc += w_att[c] * (v > 0.0f ? v : 0.2f * v);
    }
    alpha[k] = sc;
    mx = fmaxf(mx, sc);
  }
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  float sum = 0.0f;
  for (int k = k0 + lane; k < k1; k += 64) {
    const float e = __expf(alpha[k] - mx);     // written by this lane above
    alpha[k] = e;
    sum += e;
  }
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  const float inv = 1.0f / sum;
  for (int k = k0 + lane; k < k1; k += 64) alpha[k] *= inv;
}

// ---------------------------------------------------------------------------------------------- 6. edge update
// lane = (edge, channel): T_out = T_in + f_c(d) * (transformed message, rotated back); no sum over edges.
template <int LMAX>
__global__ __launch_bounds__(256) void so2_edge_update_kernel(const float4* __restrict__ rhat_d, So2Bufs b,
                                                              const float* __restrict__ T_in, float* __restrict__ T_out,
                                                              long n_edges, int log2E, float r_cut) {
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  const int E = 1 << log2E;
  const int c = threadIdx.x & (E - 1);
  const long k = (long)blockIdx.x * (256 >> log2E) + (threadIdx.x >> log2E);
  if (k >= n_edges) return;
  const float4 g = rhat_d[k];
  float o[D];
  so2_load_rotate_back<LMAX>(b, k, c, log2E, g, o);
  const float fc = egnn_envelope(g.w, r_cut);
  const float* ti = T_in + (((size_t)k * D) << log2E) + c;
  float* to = T_out + (((size_t)k * D) << log2E) + c;
#pragma unroll
  for (int i = 0; i < D; ++i)
    __builtin_nontemporal_store(__builtin_nontemporal_load(ti + ((size_t)i << log2E)) + fc * o[i], to + ((size_t)i << log2E));
}

// ---------------------------------------------------------------------------------------------- 7. gate
// One workgroup per node: y[L=0] = SiLU(x[L=0]); y[(l,m)][c] = x[(l,m)][c] * sigmoid(sum_c' W_g[l-1][c][c'] x[L=0][c']).
__global__ __launch_bounds__(256) void so2_gate_kernel(const float* __restrict__ x, const float* __restrict__ W_g,
                                                       float* __restrict__ y, int lmax, int log2E) {
  __shared__ float s_x0[128];
  __shared__ float s_gate[4 * 128];
  const int E = 1 << log2E, D = (lmax + 1) * (lmax + 1), tid = threadIdx.x;
  const float* xi = x + (((size_t)blockIdx.x * D) << log2E);
  float* yi = y + (((size_t)blockIdx.x * D) << log2E);
  if (tid < E) s_x0[tid] = xi[tid];
  __syncthreads();
  for (int t = tid; t < (lmax << log2E); t += 256) {
    const float* wrow = W_g + ((size_t)t << log2E);     // row (l-1) * E + c
    float sc = 0.0f;
    for (int cc = 0; cc < E; ++cc) sc += wrow[cc] * s_x0[cc];
    s_gate[t] = 1.0f / (1.0f + __expf(-sc));
  }
  __syncthreads();
  for (int idx = tid; idx < (D << log2E); idx += 256) {
    const int q = idx >> log2E, c = idx & (E - 1);
    const float v = xi[idx];
    if (q == 0) {
      yi[idx] = v / (1.0f + __expf(-v));
    } else {
      int l = 1;
      while ((l + 1) * (l + 1) <= q) ++l;
      yi[idx] = v * s_gate[((l - 1) << log2E) + c];
    }
  }
}

// ---------------------------------------------------------------------------------------------- host side
static size_t so2_a256(size_t n) { return (n + 255) & ~(size_t)255; }
static int so2_steps(int K) { return (K + 63) / 64; }
static int so2_tiles(int N) { return (N + 63) / 64; }

extern "C" int egnn_so2_weight_count(const egnn_ctx* ctx, int64_t* n_floats) {
  if (!ctx || !n_floats) return EGNN_EINVAL;
  *n_floats = (int64_t)so2_w_offset(ctx->desc.lmax, ctx->desc.channels, ctx->desc.lmax + 1);
  return EGNN_OK;
}

// rhat_d, the operands A_m, the results Y_m, the packed weights, and (blocks only) one float per edge
static size_t so2_ws(const egnn_ctx* ctx, int64_t n_edges, bool full, bool carve, char* base, float** rhat_d, So2Bufs* b,
                     uint16_t** T, float** alpha, unsigned** maxima = nullptr) {
  const int lmax = ctx->desc.lmax, E = ctx->desc.channels;
  size_t used = 0;
  auto take = [&](size_t bytes) { char* p = carve ? base + used : nullptr; used += so2_a256(bytes); return p; };
  float* rd = (float*)take((size_t)n_edges * 16);
  if (rhat_d) *rhat_d = rd;
  unsigned* mx = (unsigned*)take(256);     // largest magnitudes of the GEMM operands (bit patterns), see so2_transform
  if (maxima) *maxima = mx;
  for (int m = 0; m <= lmax; ++m) {
    const int K = so2_K(lmax, E, m, full), N = so2_N(lmax, E, m);
    float* A = (float*)take((size_t)n_edges * so2_ld(K) * sizeof(float));
    float* Y = (float*)take((size_t)n_edges * so2_ld(N) * sizeof(float));
    uint16_t* t = (uint16_t*)take((size_t)so2_tiles(N) * so2_steps(K) * 64 * 3 * 64 * sizeof(uint16_t));
    if (b) { b->A[m] = A; b->Y[m] = Y; b->K[m] = K; b->N[m] = N; b->ldA[m] = so2_ld(K); b->ldY[m] = so2_ld(N); }
    if (T) T[m] = t;
  }
  if (full) {
    float* al = (float*)take((size_t)n_edges * sizeof(float));
    if (alpha) *alpha = al;
  }
  return used;
}

extern "C" int egnn_so2_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, size_t* bytes) {
  if (!ctx || !bytes || n_edges < 0) return EGNN_EINVAL;
  *bytes = so2_ws(ctx, n_edges, false, false, nullptr, nullptr, nullptr, nullptr, nullptr) + 256;
  return EGNN_OK;
}

extern "C" int egnn_so2_blocks_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, size_t* bytes) {
  if (!ctx || !bytes || n_edges < 0) return EGNN_EINVAL;
  *bytes = so2_ws(ctx, n_edges, true, false, nullptr, nullptr, nullptr, nullptr, nullptr) + 256;
  return EGNN_OK;
}

struct So2Call {
  float* rhat_d;
  float* alpha;
  unsigned* maxima;
  So2Bufs b;
  uint16_t* T[5];
};

static int so2_check(egnn_ctx* ctx, const egnn_graph* g, const void* ws, size_t ws_bytes, bool full, const char* who) {
  if (!g || g->n_edges < 0 || g->n_edges > 2147483647LL || g->n_owned < 0 || g->n_total < g->n_owned || !g->row_ptr ||
      (g->n_edges > 0 && (!g->src || !g->dst)))
    return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": bad graph");
  if (!ws || ((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": workspace missing or not 256-byte aligned");
  if (ctx->desc.channels < 8 || ctx->desc.n_rbf < 2)
    return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": needs >= 8 channels and >= 2 radial bases");
  if (ctx->desc.lmax < 0 || ctx->desc.lmax > 4) return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": lmax out of range");
  if (ws_bytes < so2_ws(ctx, g->n_edges, full, false, nullptr, nullptr, nullptr, nullptr, nullptr))
    return egnn_fail(ctx, EGNN_EWS, std::string(who) + ": workspace too small");
  return EGNN_OK;
}

// geometry, gather into the m-major operands, weight packing and the GEMMs: Y_m of every edge in the workspace
// (gemms = false: operands only -- the reverse passes that do not need Y)
static int so2_transform(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3], const float* x,
                         const float* edge_in, bool full, const float* W_so2, void* ws, So2Call* call, hipStream_t st,
                         bool gemms = true) {
  const int lmax = ctx->desc.lmax, E = ctx->desc.channels;
  for (int m = 0; m < 5; ++m) { call->b.A[m] = call->b.Y[m] = nullptr; call->b.K[m] = call->b.N[m] = call->b.ldA[m] = call->b.ldY[m] = 0; call->T[m] = nullptr; }
  call->alpha = nullptr;
  so2_ws(ctx, g->n_edges, full, true, (char*)ws, &call->rhat_d, &call->b, call->T, &call->alpha, &call->maxima);
  const long n = g->n_edges;
  if (n == 0) return EGNN_OK;
  int rc;
  // the two largest magnitudes start at zero; the gather kernel and so2_wmax_kernel raise them
  if ((rc = egnn_launch_fill_int(ctx, (int*)call->maxima, 64, 0, st))) return rc;
  if ((rc = egnn_launch_geometry(ctx, g, pos, box, call->rhat_d, nullptr, nullptr, nullptr, st))) return rc;
  const float4* rd = reinterpret_cast<const float4*>(call->rhat_d);
  const int per_wg = 256 / E;
  dim3 grid((unsigned)((n + per_wg - 1) / per_wg)), block(256);
#define GATHER(L)                                                                                                      \
  do {                                                                                                                 \
    if (full)                                                                                                          \
      hipLaunchKernelGGL((so2_gather_kernel<L, true>), grid, block, 0, st, g->src, g->dst, rd, x, edge_in, call->b, n, \
                         ctx->log2_channels, ctx->desc.n_rbf, ctx->desc.r_cut, call->maxima);                          \
    else                                                                                                               \
      hipLaunchKernelGGL((so2_gather_kernel<L, false>), grid, block, 0, st, g->src, g->dst, rd, x, edge_in, call->b, n, \
                         ctx->log2_channels, ctx->desc.n_rbf, ctx->desc.r_cut, call->maxima);                          \
  } while (0)
  switch (lmax) {
    case 0: GATHER(0); break;
    case 1: GATHER(1); break;
    case 2: GATHER(2); break;
    case 3: GATHER(3); break;
    default: GATHER(4); break;
  }
#undef GATHER
  EGNN_LAUNCH_CHECK(ctx, "so2_gather_kernel");
  {
    const long n_w = (long)so2_w_offset(lmax, E, lmax + 1);
    const unsigned wg = (unsigned)((n_w + 255) / 256 < 256 ? (n_w + 255) / 256 : 256);
    hipLaunchKernelGGL(so2_wmax_kernel, dim3(wg), dim3(256), 0, st, W_so2, n_w, call->maxima + 1);
    EGNN_LAUNCH_CHECK(ctx, "so2_wmax_kernel");
  }
  for (int m = 0; gemms && m <= lmax; ++m) {
    const int K = call->b.K[m], N = call->b.N[m], n_steps = so2_steps(K), n_ct = so2_tiles(N);
    const long total = (long)n_ct * n_steps * 64 * 32;
    hipLaunchKernelGGL(so2_pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       W_so2 + so2_w_offset(lmax, E, m), call->T[m], m, lmax, E, K, N, n_steps, n_ct, full, call->maxima + 1,
                       false);
    EGNN_LAUNCH_CHECK(ctx, "so2_pack_kernel");
    if ((rc = so2_launch_gemm(ctx, call->b.A[m], n, K, call->b.ldA[m], call->T[m], call->b.Y[m], N, call->b.ldY[m],
                              call->maxima, st)))
      return rc;
  }
  return EGNN_OK;
}

static int so2_scatter(egnn_ctx* ctx, const egnn_graph* g, const So2Call& call, const float* alpha, float scale, float* a,
                       hipStream_t st) {
  if (g->n_owned == 0) return EGNN_OK;
  const int per_xcd = (g->n_owned + 7) / 8;
  const float4* rd = reinterpret_cast<const float4*>(call.rhat_d);
#define SCATTER(L)                                                                                                  \
  hipLaunchKernelGGL(so2_scatter_kernel<L>, dim3(per_xcd * 8), dim3(256), 0, st, g->row_ptr, rd, call.b, alpha, a,    \
                     g->n_owned, ctx->log2_channels, per_xcd, scale, ctx->desc.r_cut)
  switch (ctx->desc.lmax) {
    case 0: SCATTER(0); break;
    case 1: SCATTER(1); break;
    case 2: SCATTER(2); break;
    case 3: SCATTER(3); break;
    default: SCATTER(4); break;
  }
#undef SCATTER
  EGNN_LAUNCH_CHECK(ctx, "so2_scatter_kernel");
  return EGNN_OK;
}

extern "C" int egnn_so2_message_sum(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                    const float* x, const float* W_e, const float* W_so2, float* a, void* ws,
                                    size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!pos || !box || !x || !W_e || !W_so2 || !a) return egnn_fail(ctx, EGNN_EINVAL, "so2_message_sum: null pointer");
  int rc = so2_check(ctx, g, ws, ws_bytes, false, "so2_message_sum");
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  So2Call call;
  if ((rc = so2_transform(ctx, g, pos, box, x, W_e, false, W_so2, ws, &call, st))) return rc;
  return so2_scatter(ctx, g, call, nullptr, 1.0f / sqrtf(ctx->desc.agg_norm), a, st);
}

extern "C" int egnn_edge_embed_init(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                    const float* W_e, float* T_edge, void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!pos || !box || !W_e) return egnn_fail(ctx, EGNN_EINVAL, "edge_embed_init: null pointer");
  int rc = so2_check(ctx, g, ws, ws_bytes, true, "edge_embed_init");
  if (rc) return rc;
  const long n = g->n_edges;
  if (n == 0) return EGNN_OK;
  if (!T_edge) return egnn_fail(ctx, EGNN_EINVAL, "edge_embed_init: null pointer");
  hipStream_t st = (hipStream_t)stream;
  float* rhat_d = (float*)ws;
  if ((rc = egnn_launch_geometry(ctx, g, pos, box, rhat_d, nullptr, nullptr, nullptr, st))) return rc;
  const int E = ctx->desc.channels, per_wg = 256 / E, D = (ctx->desc.lmax + 1) * (ctx->desc.lmax + 1);
  hipLaunchKernelGGL(so2_edge_init_kernel, dim3((unsigned)((n + per_wg - 1) / per_wg)), dim3(256), 0, st,
                     reinterpret_cast<const float4*>(rhat_d), W_e, T_edge, n, D, ctx->log2_channels, ctx->desc.n_rbf,
                     ctx->desc.r_cut);
  EGNN_LAUNCH_CHECK(ctx, "so2_edge_init_kernel");
  return EGNN_OK;
}

extern "C" int egnn_so2_node_block(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                   const float* x, const float* T_edge, const float* W_so2, const float* w_att, float* a,
                                   void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!pos || !box || !x || !W_so2 || !w_att || !a) return egnn_fail(ctx, EGNN_EINVAL, "so2_node_block: null pointer");
  int rc = so2_check(ctx, g, ws, ws_bytes, true, "so2_node_block");
  if (rc) return rc;
  if (g->n_edges > 0 && !T_edge) return egnn_fail(ctx, EGNN_EINVAL, "so2_node_block: null edge embeddings");
  hipStream_t st = (hipStream_t)stream;
  So2Call call;
  if ((rc = so2_transform(ctx, g, pos, box, x, T_edge, true, W_so2, ws, &call, st))) return rc;
  if (g->n_owned == 0) return EGNN_OK;
  if (g->n_edges > 0) {
    hipLaunchKernelGGL(so2_attention_kernel, dim3((g->n_owned + 3) / 4), dim3(256), 0, st, g->row_ptr, call.b.Y[0],
                       call.b.ldY[0], w_att, call.alpha, g->n_owned, ctx->desc.channels);
    EGNN_LAUNCH_CHECK(ctx, "so2_attention_kernel");
  }
  return so2_scatter(ctx, g, call, call.alpha, 1.0f, a, st);
}

extern "C" int egnn_so2_edge_block(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                   const float* x, const float* T_edge_in, const float* W_so2, float* T_edge_out,
                                   void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!pos || !box || !x || !W_so2) return egnn_fail(ctx, EGNN_EINVAL, "so2_edge_block: null pointer");
  int rc = so2_check(ctx, g, ws, ws_bytes, true, "so2_edge_block");
  if (rc) return rc;
  const long n = g->n_edges;
  if (n == 0) return EGNN_OK;
  if (!T_edge_in || !T_edge_out) return egnn_fail(ctx, EGNN_EINVAL, "so2_edge_block: null edge embeddings");
  hipStream_t st = (hipStream_t)stream;
  So2Call call;
  if ((rc = so2_transform(ctx, g, pos, box, x, T_edge_in, true, W_so2, ws, &call, st))) return rc;
  const float4* rd = reinterpret_cast<const float4*>(call.rhat_d);
  const int per_wg = 256 / ctx->desc.channels;
  dim3 grid((unsigned)((n + per_wg - 1) / per_wg)), block(256);
#define UPDATE(L)                                                                                              \
  hipLaunchKernelGGL(so2_edge_update_kernel<L>, grid, block, 0, st, rd, call.b, T_edge_in, T_edge_out, n,        \
                     ctx->log2_channels, ctx->desc.r_cut)
  switch (ctx->desc.lmax) {
    case 0: UPDATE(0); break;
    case 1: UPDATE(1); break;
    case 2: UPDATE(2); break;
    case 3: UPDATE(3); break;
    default: UPDATE(4); break;
  }
#undef UPDATE
  EGNN_LAUNCH_CHECK(ctx, "so2_edge_update_kernel");
  return EGNN_OK;
}

extern "C" int egnn_gate(egnn_ctx* ctx, const float* x, const float* W_g, float* y, int32_t n_nodes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (n_nodes < 0 || (n_nodes > 0 && (!x || !y || (ctx->desc.lmax > 0 && !W_g))))
    return egnn_fail(ctx, EGNN_EINVAL, "gate: bad argument");
  if (ctx->desc.channels > 128 || ctx->desc.lmax > 4) return egnn_fail(ctx, EGNN_EINVAL, "gate: unsupported shape");
  if (n_nodes == 0) return EGNN_OK;
  hipLaunchKernelGGL(so2_gate_kernel, dim3(n_nodes), dim3(256), 0, (hipStream_t)stream, x, W_g, y, ctx->desc.lmax,
                     ctx->log2_channels);
  EGNN_LAUNCH_CHECK(ctx, "so2_gate_kernel");
  return EGNN_OK;
}

// =====================================================================================================================
// Reverse pass of egnn_so2_message_sum (adjoint with respect to the node embeddings and the weights; positions are
// data).  Every step of the forward pass is linear in (x, W_e) for fixed weights and linear in the weights for fixed
// inputs, so the reverse pass is the same chain read backwards:
//   1. so2_gather_kernel       the operands A_m of the forward pass again (they are the inputs of the weight gradient);
//   2. so2_dy_kernel           dY_m[k] = bond-frame rotation of  agg_norm^-1/2 f_c(d_k) da[dst(k)], m-major like Y_m;
//   3. so2_wgrad_kernel        dB_m = A_m^T dY_m, a contraction over the edges on half-precision pieces (three
//                              products per fp32 product); both operands are read in memory order: the contraction
//                              index is the row index of both; partial sums per chunk of edges added in a fixed order;
//      so2_unpack_wgrad_kernel dB_m = [[dWr^T, dWi^T], [-dWi^T, dWr^T]] folded back into the layout of the weights;
//   4. so2_gemmw_kernel        dA_m = dY_m B_m^T with the packed operand transposed, written over A_m;
//   5. so2_dx_edge_kernel      lane = (edge, channel): the source part of dA_m[k] rotated back to the lab frame, to a
//                              per-edge row that a segmented sum over the source-sorted index adds up;
//      so2_dx_kernel           one workgroup per destination node: the destination part rotated back and summed over
//                              the node's incoming edges;
//      so2_dwe_kernel          dW_e[c][q] = sum_k dA_0[k][edge column c] B_q(d_k).
// ---------------------------------------------------------------------------------------------------------------------
// Gradient of the bond-frame results, written m-major over Y_m.  The lab-frame gradient of edge k is
//   scale f_c(d_k) [alpha_k] rows[per_edge ? k : dst(k)]      (the sum over incoming edges, weighted if alpha != NULL, or
//                                                              the edge update)
// plus, for the node block (ds != NULL), ds_k w_att[c] LeakyReLU'(y_k[L = 0][c]) in the L = 0 plane -- the part that
// reaches the messages through the attention scores; y_k[L = 0] is read from Y_0 before it is overwritten.
template <int LMAX>
__global__ __launch_bounds__(256) void so2_dy_kernel(const int* __restrict__ dst, const float4* __restrict__ rhat_d,
                                                     const float* __restrict__ rows, bool per_edge,
                                                     const float* __restrict__ alpha, const float* __restrict__ ds,
                                                     const float* __restrict__ w_att, So2Bufs b, long n_edges, int log2E,
                                                     float scale, float r_cut, unsigned* __restrict__ y_max) {
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  const int E = 1 << log2E;
  const int c = threadIdx.x & (E - 1);
  const long k_own = (long)blockIdx.x * (256 >> log2E) + (threadIdx.x >> log2E);
  const bool live = k_own < n_edges;
  const long k = live ? k_own : n_edges - 1;   // (as in the gather kernel: every lane takes part in the reduction)
  const float4 g = rhat_d[k];
  float f = scale * egnn_envelope(g.w, r_cut);
  if (alpha) f *= alpha[k];
  const float* dj = rows + (((size_t)(per_edge ? k : (long)dst[k]) * D) << log2E) + c;
  float v[D];
#pragma unroll
  for (int i = 0; i < D; ++i) v[i] = f * dj[(size_t)i << log2E];
  float* y0 = b.Y[0] + (size_t)k * b.ldY[0] + c;
  if (ds) {
    const float y = y0[0];                     // L = 0 plane of the transformed message (the same in both frames)
    v[0] += ds[k] * w_att[c] * (y > 0.0f ? 1.0f : 0.2f);
  }
  BondTrig t;
  egnn_bond_trig<LMAX>(g.x, g.y, g.z, t);
  egnn_to_bond_frame<LMAX>(v, t);            // Y = D^T Y' in the forward pass, so dY' = D dY
  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < D; ++i) amax = fmaxf(amax, fabsf(v[i]));
  if (live) {
#pragma unroll
    for (int l = 0; l <= LMAX; ++l) __builtin_nontemporal_store(v[l * l + l], y0 + (l << log2E));
#pragma unroll
    for (int m = 1; m <= LMAX; ++m) {
      const int nl = LMAX + 1 - m;
      float* ym = b.Y[m] + (size_t)k * b.ldY[m] + c;
#pragma unroll
      for (int l = m; l <= LMAX; ++l) {
        __builtin_nontemporal_store(v[l * l + l + m], ym + ((l - m) << log2E));
        __builtin_nontemporal_store(v[l * l + l - m], ym + ((nl + l - m) << log2E));
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
  if ((threadIdx.x & 63) == 0) so2_raise_max(y_max, amax);
}

// Adjoint of the attention weights of the node block, one workgroup per destination node j (lane = (edge slot,
// channel)):  t_k = f_c(d_k) <da_j, y_k> is the gradient of alpha_k; the softmax gives ds_k = alpha_k (t_k - sum alpha t)
// (written over t); the score s_k = w_att . LeakyReLU(y_k[L = 0]) gives dw_att += ds_k LeakyReLU(y_k[L = 0]), kept per
// node in dwatt_part[j][E] and added up afterwards.  All sums in a fixed order.
template <int LMAX>
__global__ __launch_bounds__(256) void so2_attention_adjoint_kernel(const int* __restrict__ row_ptr,
                                                                    const float4* __restrict__ rhat_d, So2Bufs b,
                                                                    const float* __restrict__ alpha,
                                                                    const float* __restrict__ da, float* __restrict__ tds,
                                                                    float* __restrict__ dwatt_part, int n_owned, int log2E,
                                                                    float r_cut) {
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  __shared__ float red[256];
  __shared__ float s_sum;
  const int j = blockIdx.x;
  if (j >= n_owned) return;
  const int E = 1 << log2E;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1), slot = tid >> log2E, n_slots = 256 >> log2E;
  const int k0 = row_ptr[j], k1 = row_ptr[j + 1];
  float daj[D];
#pragma unroll
  for (int i = 0; i < D; ++i) daj[i] = da[(((size_t)j * D + i) << log2E) + c];
  // pass 1: t_k (every thread runs the same number of rounds: there is a barrier in each)
  const int rounds = (k1 - k0 + n_slots - 1) / n_slots;
  for (int r = 0; r < rounds; ++r) {
    const int k = k0 + r * n_slots + slot;
    float p = 0.0f;
    float fc = 0.0f;
    if (k < k1) {
      const float4 g = rhat_d[k];
      float o[D];
      so2_load_rotate_back<LMAX>(b, k, c, log2E, g, o);
#pragma unroll
      for (int i = 0; i < D; ++i) p += daj[i] * o[i];
      fc = egnn_envelope(g.w, r_cut);
    }
    red[tid] = p;
    __syncthreads();
    if (c == 0 && k < k1) {
      float sum = 0.0f;
      for (int q = 0; q < E; ++q) sum += red[(slot << log2E) + q];
      tds[k] = fc * sum;
    }
    __syncthreads();
  }
  // pass 2: sum_k alpha_k t_k (this workgroup wrote t itself: visible after the barrier above)
  float part = 0.0f;
  for (int k = k0 + tid; k < k1; k += 256) part += alpha[k] * tds[k];
  red[tid] = part;
  __syncthreads();
  if (tid == 0) {
    float sum = 0.0f;
    for (int q = 0; q < 256; ++q) sum += red[q];
    s_sum = sum;
  }
  __syncthreads();
  const float mean = s_sum;
  for (int k = k0 + tid; k < k1; k += 256) tds[k] = alpha[k] * (tds[k] - mean);
  __syncthreads();
  // pass 3: this node's part of dw_att
  float acc = 0.0f;
  for (int k = k0 + slot; k < k1; k += n_slots) {
    const float y = b.Y[0][(size_t)k * b.ldY[0] + c];
    acc += tds[k] * (y > 0.0f ? y : 0.2f * y);
  }
  red[tid] = acc;
  __syncthreads();
  if (tid < E) {
    float sum = 0.0f;
    for (int q = 0; q < n_slots; ++q) sum += red[(q << log2E) + tid];
    dwatt_part[((size_t)j << log2E) + tid] = sum;
  }
}

// partial[chunk][k][n] = sum over the edges e of the chunk of A[e][k] Y[e][n].  Workgroup = (chunk of edges, four
// neighbouring 128 x 64 quarters of the result), one quarter per wave as 4 x 2 accumulators of 32 x 32.  The products
// run on half-precision pieces like the GEMMs (two pieces per operand after a power-of-two scaling from its largest
// magnitude, three products per fp32 product: v_mfma_f32_32x32x16_f16 contracts 16 edges per instruction; the first
// version used exact fp32 products, v_mfma_f32_32x32x2_f32, at a sixteenth of the rate).  Both operands are read
// in memory order, because the contraction index is the row index of both: per block of 16 edges a lane fetches, for
// the eight edges of its half-wave, 16 bytes of A and 8 bytes of Y each -- a half-wave reads 512 and 256 contiguous
// bytes of a row -- and finds the eight consecutive edges that one operand register wants, for each of its 4 + 2
// columns, in one component of those eight registers: lane (i, h) holds A[e + 8 h + r][k0 + 4 i + a] and
// Y[e + 8 h + r][n0 + 2 i + q], so accumulator (a, q) holds the rows k0 + 4 r' + a and the columns n0 + 2 i + q of the
// result -- a permutation that only the final store has to know.  Columns past the last one are clamped (K and N are
// multiples of 8: a lane's group is valid or not as a whole; invalid ones are not stored).
#define SW_BLOCK 16
typedef float sw_f4 __attribute__((ext_vector_type(4)));
typedef float sw_f2 __attribute__((ext_vector_type(2)));
__global__ __launch_bounds__(256, 2) void so2_wgrad_kernel(const float* __restrict__ A, int K, int lda,
                                                           const float* __restrict__ Y, int N, int ldy, long n_edges,
                                                           long per_chunk, int quarters_n, float* __restrict__ partial,
                                                           const unsigned* __restrict__ a_max,
                                                           const unsigned* __restrict__ y_max) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i32 = lane & 31, hh = lane >> 5;
  // (tiles of one chunk of edges are neighbours in the grid and land on different XCDs: putting them on one XCD, so
  // that its L2 serves the rows they share, was measured slower)
  const int chunk = blockIdx.y;
  // the 128 x 64 quarters of the result are numbered row by row and dealt out four to a workgroup: only the last
  // workgroup of a chunk can have waves without work (a wave that ends early does not make room for another one
  // in practice)
  const int quarter = blockIdx.x * (blockDim.x >> 6) + wave;   // (a result of fewer than four quarters: smaller workgroups)
  const int kq = quarter / quarters_n, nq = quarter - kq * quarters_n;
  const int k0 = kq * 128, n0 = nq * 64;
  if (k0 >= K) return;                       // (no barrier in this kernel)
  const long e_begin = (long)chunk * per_chunk;
  long e_end = e_begin + per_chunk;
  if (e_end > n_edges) e_end = n_edges;
  const int ca = k0 + 4 * i32, cy = n0 + 2 * i32;
  const bool a_ok = ca < K, y_ok = cy < N;
  const int ea = sgh_scale_exp(*a_max), ey = sgh_scale_exp(*y_max);
  const float a_scale = ldexpf(1.0f, ea), y_scale = ldexpf(1.0f, ey), unscale = ldexpf(1.0f, -ea - ey);
  // addresses: a row pointer that is the same for the whole wave (scalar arithmetic) plus a per-lane byte offset that
  // never changes (its half-wave's first row and its columns) -- no vector arithmetic per load
  const unsigned oa = (unsigned)(8 * hh * lda + (a_ok ? ca : K - 4)) * 4u;
  const unsigned oy = (unsigned)(8 * hh * ldy + (y_ok ? cy : N - 2)) * 4u;
  float16v acc[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][q][i] = 0.0f;
  sw_f4 ra[8];
  sw_f2 ry[8];
  // a full block: rows e .. e + 15 exist; no mask and no branch around a load
  auto fetch = [&](long e) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      ra[r] = *reinterpret_cast<const sw_f4*>(reinterpret_cast<const char*>(A + (size_t)(e + r) * lda) + oa);
      ry[r] = *reinterpret_cast<const sw_f2*>(reinterpret_cast<const char*>(Y + (size_t)(e + r) * ldy) + oy);
    }
  };
  uint4 ah[4], al[4], yh[2], yl[2];
  auto cut = [&]() {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const float x[8] = {ra[0][a], ra[1][a], ra[2][a], ra[3][a], ra[4][a], ra[5][a], ra[6][a], ra[7][a]};
      sgh_split8(x, a_scale, ah[a], al[a]);
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const float x[8] = {ry[0][q], ry[1][q], ry[2][q], ry[3][q], ry[4][q], ry[5][q], ry[6][q], ry[7][q]};
      sgh_split8(x, y_scale, yh[q], yl[q]);
    }
  };
  auto products = [&]() {
    // smallest terms first; the eight accumulation chains are independent
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int q = 0; q < 2; ++q)
        acc[a][q] = __builtin_amdgcn_mfma_f32_32x32x16_f16(sgh_as_h8(al[a]), sgh_as_h8(yh[q]), acc[a][q], 0, 0, 0);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int q = 0; q < 2; ++q)
        acc[a][q] = __builtin_amdgcn_mfma_f32_32x32x16_f16(sgh_as_h8(ah[a]), sgh_as_h8(yl[q]), acc[a][q], 0, 0, 0);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int q = 0; q < 2; ++q)
        acc[a][q] = __builtin_amdgcn_mfma_f32_32x32x16_f16(sgh_as_h8(ah[a]), sgh_as_h8(yh[q]), acc[a][q], 0, 0, 0);
  };
  // The full blocks of the chunk: the block's registers are cut into pieces, then refilled with the next block while
  // the products of this one run (the block after the last one is the last one again, loaded and not used).
  const long n_blocks = (e_end - e_begin) / SW_BLOCK;
  if (n_blocks > 0) {
    const long last = e_begin + (n_blocks - 1) * SW_BLOCK;
    fetch(e_begin);
    for (long blk = 0; blk < n_blocks; ++blk) {
      cut();
      const long e1 = e_begin + (blk + 1) * SW_BLOCK;
      fetch(e1 < last ? e1 : last);
      products();
    }
  }
  {
    // the ragged end of the last chunk: fewer than 16 edges, zeros past the end
    const long e = e_begin + n_blocks * SW_BLOCK;
    if (e < e_end) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const long ee = e + 8 * hh + r;
        const bool ok = ee < e_end;
        // a row whose lane offset (8 hh rows further) stays inside the matrix: e_end - 1 at most
        const long er = ok ? e + r : e_end - 1 - 8 * hh;
        const sw_f4 a4 = *reinterpret_cast<const sw_f4*>(reinterpret_cast<const char*>(A + (size_t)er * lda) + oa);
        const sw_f2 y2 = *reinterpret_cast<const sw_f2*>(reinterpret_cast<const char*>(Y + (size_t)er * ldy) + oy);
        const sw_f4 z4 = {0.0f, 0.0f, 0.0f, 0.0f};
        const sw_f2 z2 = {0.0f, 0.0f};
        ra[r] = ok ? a4 : z4;
        ry[r] = ok ? y2 : z2;
      }
      cut();
      products();
    }
  }
  float* out = partial + (size_t)chunk * K * N;
  if (y_ok) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int kk = k0 + 4 * (8 * (i >> 2) + 4 * hh + (i & 3)) + a;
        if (kk < K) {
          const sw_f2 v = {unscale * acc[a][0][i], unscale * acc[a][1][i]};
          *reinterpret_cast<sw_f2*>(out + (size_t)kk * N + cy) = v;
        }
      }
  }
}

// dB_m [K][N] (column orders of A_m and Y_m) -> gradient of W_0 (m = 0) or of (Wr_m, Wi_m), row-major like the weights.
// Without persistent edge embeddings (full = false) the weight columns that multiply the planes l > 0 of the edge
// embedding, which are zero on that path, have gradient zero; with them the columns of A_m are in the column order of
// the weights.  One thread per weight element of W_0 / Wr_m.
__global__ __launch_bounds__(256) void so2_unpack_wgrad_kernel(const float* __restrict__ dB, float* __restrict__ dW, int m,
                                                               int lmax, int E, int N, bool full) {
  const int nl = lmax + 1 - m;
  const int rows = nl * E, cols = nl * 3 * E;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)rows * cols) return;
  const int row = (int)(idx / cols), col = (int)(idx - (long)row * cols);
  const int li = col / (3 * E), rem = col - li * 3 * E;
  const int gsel = rem / E, c = rem - gsel * E;
  // column of A_m (its +m half) that this weight column multiplies, -1: none
  int kr = -1;
  if (full) kr = col;
  else if (gsel < 2) kr = li * 2 * E + gsel * E + c;
  else if (m == 0 && li == 0) kr = (lmax + 1) * 2 * E + c;
  if (m == 0) {
    dW[idx] = kr >= 0 ? dB[(size_t)kr * N + row] : 0.0f;
    return;
  }
  float gr = 0.0f, gi = 0.0f;
  if (kr >= 0) {
    const int half_k = full ? nl * 3 * E : nl * 2 * E, half_n = nl * E;
    const float pp = dB[(size_t)kr * N + row], mm = dB[(size_t)(half_k + kr) * N + half_n + row];
    const float pm = dB[(size_t)kr * N + half_n + row], mp = dB[(size_t)(half_k + kr) * N + row];
    gr = pp + mm;     // Wr takes x_{+m} to y_{+m} and x_{-m} to y_{-m}
    gi = pm - mp;     // Wi takes x_{+m} to y_{-m} and, with a minus sign, x_{-m} to y_{+m}
  }
  dW[idx] = gr;
  dW[(size_t)rows * cols + idx] = gi;
}

// Column group grp (0 source, 1 destination, 2 edge) of dA_m[k], channel c, back in (l, m) order (bond frame);
// G = column groups per degree (3 with persistent edge embeddings, else 2).
template <int LMAX, int G>
__device__ __forceinline__ void so2_load_group(const So2Bufs& b, long k, int c, int log2E, int grp, float* v) {
  const float* a0 = b.A[0] + (size_t)k * b.ldA[0] + c;
#pragma unroll
  for (int l = 0; l <= LMAX; ++l) v[l * l + l] = __builtin_nontemporal_load(a0 + ((G * l + grp) << log2E));
#pragma unroll
  for (int m = 1; m <= LMAX; ++m) {
    const int nl = LMAX + 1 - m;
    const float* am = b.A[m] + (size_t)k * b.ldA[m] + c;
#pragma unroll
    for (int l = m; l <= LMAX; ++l) {
      const int col = (G * (l - m) + grp) << log2E, neg = (G * nl) << log2E;
      v[l * l + l + m] = __builtin_nontemporal_load(am + col);
      v[l * l + l - m] = __builtin_nontemporal_load(am + neg + col);
    }
  }
}

// The per-edge parts of the gradient of the messages, lane = (edge, channel): the source part of dA_m[k] rotated back
// to the lab frame (X' = D M in the forward pass, so dM = D^T dX') -> rows[k], which a segmented sum over the
// source-sorted index adds up afterwards; FULL (persistent edge embeddings): the edge part -> dT[k], plus dT_add[k] if
// that is given (the identity term of the edge update; dT may be dT_add).
template <int LMAX, bool FULL>
__global__ __launch_bounds__(256) void so2_dx_edge_kernel(const float4* __restrict__ rhat_d, So2Bufs b,
                                                          float* __restrict__ rows, float* dT, const float* dT_add,
                                                          long n_edges, int log2E) {
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  constexpr int G = FULL ? 3 : 2;
  const int E = 1 << log2E;
  const int c = threadIdx.x & (E - 1);
  const long k = (long)blockIdx.x * (256 >> log2E) + (threadIdx.x >> log2E);
  if (k >= n_edges) return;
  const float4 g = rhat_d[k];
  BondTrig t;
  egnn_bond_trig<LMAX>(g.x, g.y, g.z, t);
  float v[D];
  so2_load_group<LMAX, G>(b, k, c, log2E, 0, v);
  egnn_from_bond_frame<LMAX>(v, t);
  float* rk = rows + (((size_t)k * D) << log2E) + c;
#pragma unroll
  for (int i = 0; i < D; ++i) __builtin_nontemporal_store(v[i], rk + ((size_t)i << log2E));
  if constexpr (FULL) {
    so2_load_group<LMAX, G>(b, k, c, log2E, 2, v);
    egnn_from_bond_frame<LMAX>(v, t);
    float* tk = dT + (((size_t)k * D) << log2E) + c;
    const float* ta = dT_add ? dT_add + (((size_t)k * D) << log2E) + c : nullptr;
#pragma unroll
    for (int i = 0; i < D; ++i) {
      const float add = ta ? ta[(size_t)i << log2E] : 0.0f;
      tk[(size_t)i << log2E] = v[i] + add;
    }
  }
}

// One workgroup per destination node j, lane = (edge slot, channel): the destination part of dA_m[k] rotated back and
// summed over the incoming edges of j in a fixed order -> dxd[j].
template <int LMAX, bool FULL>
__global__ __launch_bounds__(256) void so2_dx_kernel(const int* __restrict__ row_ptr, const float4* __restrict__ rhat_d,
                                                     So2Bufs b, float* __restrict__ dxd, int n_owned, int log2E,
                                                     int nodes_per_xcd) {
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  constexpr int G = FULL ? 3 : 2;            // column groups per degree
  __shared__ float red[256 * D];
  const int j = (blockIdx.x & 7) * nodes_per_xcd + (blockIdx.x >> 3);
  if (j >= n_owned || (int)(blockIdx.x >> 3) >= nodes_per_xcd) return;
  const int E = 1 << log2E;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1), slot = tid >> log2E, n_slots = 256 >> log2E;
  const int k0 = row_ptr[j], k1 = row_ptr[j + 1];
  float acc[D];
#pragma unroll
  for (int i = 0; i < D; ++i) acc[i] = 0.0f;
  for (int k = k0 + slot; k < k1; k += n_slots) {
    const float4 g = rhat_d[k];
    BondTrig t;
    egnn_bond_trig<LMAX>(g.x, g.y, g.z, t);
    float v[D];
    so2_load_group<LMAX, G>(b, k, c, log2E, 1, v);
    egnn_from_bond_frame<LMAX>(v, t);
#pragma unroll
    for (int i = 0; i < D; ++i) acc[i] += v[i];
  }
#pragma unroll
  for (int i = 0; i < D; ++i) red[((slot * D + i) << log2E) + c] = acc[i];
  __syncthreads();
  const int row = D << log2E;
  float* out = dxd + (size_t)j * row;
  for (int idx = tid; idx < row; idx += 256) {
    float sum = 0.0f;
    for (int s = 0; s < n_slots; ++s) sum += red[s * row + idx];
    out[idx] = sum;
  }
}

// dx[i] += dxd[i] for the owned nodes (dx holds the sums over outgoing edges of all nodes)
__global__ __launch_bounds__(256) void so2_add_kernel(float* __restrict__ dx, const float* __restrict__ dxd, long n) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dx[i] += dxd[i];
}

// partial[chunk][c][q] = sum over the edges k of the chunk of de[k][c] B_q(d_k), de = the edge columns of dA_0.
// A thread owns the outputs o = tid + 256 s (c = o mod E: neighbouring threads read neighbouring columns).
#define SO2_DWE_CHUNKS 2048
__global__ __launch_bounds__(256) void so2_dwe_kernel(const float4* __restrict__ rhat_d, const float* __restrict__ A0, int K0,
                                                      int edge_col0, long n_edges, long per_chunk, int log2E, int n_rbf,
                                                      float r_cut, float* __restrict__ partial) {
  const int E = 1 << log2E, n_out = n_rbf << log2E;
  const long e_begin = (long)blockIdx.x * per_chunk;
  long e_end = e_begin + per_chunk;
  if (e_end > n_edges) e_end = n_edges;
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
  float acc[16];    // E n_rbf <= 128 * 32 = 16 * 256
#pragma unroll
  for (int s = 0; s < 16; ++s) acc[s] = 0.0f;
  for (long k = e_begin; k < e_end; k += 4) {
    // four edges at a time: their loads are independent (edges past the chunk repeat its last edge with weight zero)
    float d[4], live[4];
    const float* de[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long ku = k + u < e_end ? k + u : e_end - 1;
      live[u] = k + u < e_end ? 1.0f : 0.0f;
      d[u] = rhat_d[ku].w;
      de[u] = A0 + (size_t)ku * K0 + edge_col0;
    }
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      const int o = threadIdx.x + 256 * s;
      if (o < n_out) {
        const float centre = (float)(o >> log2E) * step;
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = live[u] * de[u][o & (E - 1)];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float t = d[u] - centre;
          acc[s] += v[u] * __expf(-t * t * inv2s2);
        }
      }
    }
  }
  float* out = partial + (size_t)blockIdx.x * n_out;
#pragma unroll
  for (int s = 0; s < 16; ++s) {
    const int o = threadIdx.x + 256 * s;
    if (o < n_out) out[(o & (E - 1)) * n_rbf + (o >> log2E)] = acc[s];
  }
}

// chunks of edges of the weight gradient of one order.  All waves of a launch take the same time, so their number
// should fill the chip's places once (256 compute units x 4 SIMDs x 2 waves, what the kernel's registers allow), not
// one and a third times.  Every chunk is a multiple of 2 * SW_UNROLL edges.
#define SW_UNROLL 8   // (chunks are multiples of 2 * SW_UNROLL = SW_BLOCK edges)
#define SW_WAVE_SLOTS 2048
static int so2_wgrad_quarters(int K, int N) { return ((K + 127) / 128) * ((N + 63) / 64); }
static int so2_wgrad_waves(int K, int N) { const int q = so2_wgrad_quarters(K, N); return q < 4 ? q : 4; }   // per workgroup
static int so2_wgrad_groups(int K, int N) {                                                                  // workgroups per chunk
  return (so2_wgrad_quarters(K, N) + so2_wgrad_waves(K, N) - 1) / so2_wgrad_waves(K, N);
}
static void so2_wgrad_split(long n, int K, int N, int* chunks, long* per_chunk) {
  long c = SW_WAVE_SLOTS / (so2_wgrad_waves(K, N) * so2_wgrad_groups(K, N));
  if (c < 1) c = 1;
  long per = (n + c - 1) / c;
  per = (per + 2 * SW_UNROLL - 1) / (2 * SW_UNROLL) * (2 * SW_UNROLL);
  if (per < 2 * SW_UNROLL) per = 2 * SW_UNROLL;
  *per_chunk = per;
  *chunks = (int)((n + per - 1) / per);
}

struct So2Bwd {
  float* rows;      // [n_edges][D][E] source parts of dM
  float* dxd;       // [n_owned][D][E]
  float* partial;   // partial weight gradients of one order
  float* dB;        // [K_m][N_m] of one order
  float* dwe;       // [SO2_DWE_CHUNKS][E][n_rbf]   (message sum)
  float* tds;       // [n_edges] gradient of the attention weights, then of the scores   (node block)
  float* dwatt;     // [n_owned][E] per-node parts of dw_att                             (node block)
};

static size_t so2_bwd_ws(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, bool full, bool carve, char* base,
                         So2Bwd* out) {
  const int lmax = ctx->desc.lmax, E = ctx->desc.channels, D = (lmax + 1) * (lmax + 1);
  size_t used = so2_ws(ctx, n_edges, full, false, nullptr, nullptr, nullptr, nullptr, nullptr);
  auto take = [&](size_t bytes) { char* p = carve ? base + used : nullptr; used += so2_a256(bytes); return p; };
  size_t part = 0, db = 0;
  for (int m = 0; m <= lmax; ++m) {
    const int K = so2_K(lmax, E, m, full), N = so2_N(lmax, E, m);
    int chunks;
    long per;
    so2_wgrad_split(n_edges > 0 ? n_edges : 1, K, N, &chunks, &per);
    part = std::max(part, (size_t)chunks * K * N);
    db = std::max(db, (size_t)K * N);
  }
  So2Bwd w;
  w.rows = (float*)take((size_t)n_edges * D * E * sizeof(float));
  w.dxd = (float*)take((size_t)n_owned * D * E * sizeof(float));
  w.partial = (float*)take(part * sizeof(float));
  w.dB = (float*)take(db * sizeof(float));
  w.dwe = full ? nullptr : (float*)take((size_t)SO2_DWE_CHUNKS * E * ctx->desc.n_rbf * sizeof(float));
  w.tds = full ? (float*)take((size_t)n_edges * sizeof(float)) : nullptr;
  w.dwatt = full ? (float*)take((size_t)n_owned * E * sizeof(float)) : nullptr;
  if (out) *out = w;
  return used;
}

extern "C" int egnn_so2_backward_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, size_t* bytes) {
  if (!ctx || !bytes || n_edges < 0 || n_owned < 0) return EGNN_EINVAL;
  *bytes = so2_bwd_ws(ctx, n_edges, n_owned, false, false, nullptr, nullptr) + 256;
  return EGNN_OK;
}

extern "C" int egnn_so2_blocks_backward_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned,
                                                        size_t* bytes) {
  if (!ctx || !bytes || n_edges < 0 || n_owned < 0) return EGNN_EINVAL;
  *bytes = so2_bwd_ws(ctx, n_edges, n_owned, true, false, nullptr, nullptr) + 256;
  return EGNN_OK;
}

#define SO2_BY_LMAX(lmax, STMT)    \
  switch (lmax) {                  \
    case 0: { STMT(0); } break;    \
    case 1: { STMT(1); } break;    \
    case 2: { STMT(2); } break;    \
    case 3: { STMT(3); } break;    \
    default: { STMT(4); } break;   \
  }

// what the lab-frame gradient of the transformed messages is made of (so2_dy_kernel)
struct So2Grad {
  const float* rows;     // da [n_owned][D][E] (read at dst(k)) or, per_edge, dT_out [n_edges][D][E]
  bool per_edge;
  float scale;           // factor besides f_c
  const float* alpha;    // node block: attention weights, gradient of the scores, attention vector
  const float* ds;
  const float* w_att;
};

// The part every reverse pass shares, after the operands A_m are in the workspace (so2_transform): dY_m over Y_m, then
// per order the weight gradient and dA_m over A_m, then the rotation back with the sums over the two node roles.
// dT / dT_add: gradient of the edge embeddings (full only).  maxima[2], [3] must be zero on entry.
static int so2_backward_tail(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr, const int32_t* perm, bool full,
                             const float* W_so2, const So2Grad& grad, So2Call& call, So2Bwd& w, float* dx,
                             float* dW_so2, float* dT, const float* dT_add, hipStream_t st) {
  const int lmax = ctx->desc.lmax, E = ctx->desc.channels, D = (lmax + 1) * (lmax + 1);
  const long n = g->n_edges;
  const long n_w = (long)so2_w_offset(lmax, E, lmax + 1);
  int rc;
  const float4* rd = reinterpret_cast<const float4*>(call.rhat_d);
  const int per_wg = 256 / E;
  const dim3 egrid((unsigned)((n + per_wg - 1) / per_wg)), block(256);
  unsigned* bmax = call.maxima + 2;   // [0]: largest |dY| (operand of the GEMMs below), [1]: largest weight
#define DY(L)                                                                                                          \
  hipLaunchKernelGGL(so2_dy_kernel<L>, egrid, block, 0, st, g->dst, rd, grad.rows, grad.per_edge, grad.alpha, grad.ds, \
                     grad.w_att, call.b, n, ctx->log2_channels, grad.scale, ctx->desc.r_cut, bmax)
  SO2_BY_LMAX(lmax, DY)
#undef DY
  EGNN_LAUNCH_CHECK(ctx, "so2_dy_kernel");
  {
    const unsigned wg = (unsigned)((n_w + 255) / 256 < 256 ? (n_w + 255) / 256 : 256);
    hipLaunchKernelGGL(so2_wmax_kernel, dim3(wg), dim3(256), 0, st, W_so2, n_w, bmax + 1);
    EGNN_LAUNCH_CHECK(ctx, "so2_wmax_kernel");
  }
  for (int m = 0; m <= lmax; ++m) {
    const int K = call.b.K[m], N = call.b.N[m];
    int chunks;
    long per;
    so2_wgrad_split(n, K, N, &chunks, &per);
    hipLaunchKernelGGL(so2_wgrad_kernel, dim3(so2_wgrad_groups(K, N), chunks), dim3(64 * so2_wgrad_waves(K, N)), 0, st,
                       call.b.A[m], K, call.b.ldA[m], call.b.Y[m], N, call.b.ldY[m], n, per, (N + 63) / 64, w.partial,
                       call.maxima, bmax);
    EGNN_LAUNCH_CHECK(ctx, "so2_wgrad_kernel");
    if ((rc = egnn_launch_reduce_partials(ctx, w.partial, chunks, (long)K * N, w.dB, 1.0f, st))) return rc;
    const int nl = lmax + 1 - m;
    const long n_el = (long)nl * E * nl * 3 * E;
    hipLaunchKernelGGL(so2_unpack_wgrad_kernel, dim3((unsigned)((n_el + 255) / 256)), dim3(256), 0, st, w.dB,
                       dW_so2 + so2_w_offset(lmax, E, m), m, lmax, E, N, full);
    EGNN_LAUNCH_CHECK(ctx, "so2_unpack_wgrad_kernel");
    // dA_m = dY_m B_m^T over A_m: contraction over the N columns of Y_m, one output column per column of A_m
    const int n_steps = so2_steps(N), n_ct = so2_tiles(K);
    const long total = (long)n_ct * n_steps * 64 * 32;
    hipLaunchKernelGGL(so2_pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       W_so2 + so2_w_offset(lmax, E, m), call.T[m], m, lmax, E, K, N, n_steps, n_ct, full, bmax + 1, true);
    EGNN_LAUNCH_CHECK(ctx, "so2_pack_kernel");
    if ((rc = so2_launch_gemm(ctx, call.b.Y[m], n, N, call.b.ldY[m], call.T[m], call.b.A[m], K, call.b.ldA[m], bmax, st)))
      return rc;
  }
  {
#define DXE(L)                                                                                                       \
  do {                                                                                                               \
    if (full)                                                                                                        \
      hipLaunchKernelGGL((so2_dx_edge_kernel<L, true>), egrid, block, 0, st, rd, call.b, w.rows, dT, dT_add, n,      \
                         ctx->log2_channels);                                                                        \
    else                                                                                                             \
      hipLaunchKernelGGL((so2_dx_edge_kernel<L, false>), egrid, block, 0, st, rd, call.b, w.rows, dT, dT_add, n,     \
                         ctx->log2_channels);                                                                        \
  } while (0)
    SO2_BY_LMAX(lmax, DXE)
#undef DXE
    EGNN_LAUNCH_CHECK(ctx, "so2_dx_edge_kernel");
  }
  if (g->n_owned > 0) {
    const int per_xcd = (g->n_owned + 7) / 8;
#define DX(L)                                                                                                        \
  do {                                                                                                               \
    if (full)                                                                                                        \
      hipLaunchKernelGGL((so2_dx_kernel<L, true>), dim3(per_xcd * 8), dim3(256), 0, st, g->row_ptr, rd, call.b,      \
                         w.dxd, g->n_owned, ctx->log2_channels, per_xcd);                                            \
    else                                                                                                             \
      hipLaunchKernelGGL((so2_dx_kernel<L, false>), dim3(per_xcd * 8), dim3(256), 0, st, g->row_ptr, rd, call.b,     \
                         w.dxd, g->n_owned, ctx->log2_channels, per_xcd);                                            \
  } while (0)
    SO2_BY_LMAX(lmax, DX)
#undef DX
    EGNN_LAUNCH_CHECK(ctx, "so2_dx_kernel");
  }
  if ((rc = egnn_launch_segsum_rows(ctx, w.rows, col_ptr, perm, dx, g->n_total, D * E, st))) return rc;
  const long n_own = (long)g->n_owned * D * E;
  if (n_own > 0) {
    hipLaunchKernelGGL(so2_add_kernel, dim3((unsigned)((n_own + 255) / 256)), dim3(256), 0, st, dx, w.dxd, n_own);
    EGNN_LAUNCH_CHECK(ctx, "so2_add_kernel");
  }
  return EGNN_OK;
}

static int so2_backward_check(egnn_ctx* ctx, const egnn_graph* g, const void* ws, size_t ws_bytes, bool full,
                              const char* who) {
  int rc = so2_check(ctx, g, ws, ws_bytes, full, who);
  if (rc) return rc;
  if (ctx->desc.channels > 128 || ctx->desc.n_rbf > 32)
    return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": needs <= 128 channels and <= 32 radial bases");
  if (ws_bytes < so2_bwd_ws(ctx, g->n_edges, g->n_owned, full, false, nullptr, nullptr))
    return egnn_fail(ctx, EGNN_EWS, std::string(who) + ": workspace too small");
  return EGNN_OK;
}

extern "C" int egnn_so2_message_sum_backward(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr,
                                             const int32_t* perm, const float* pos, const float box[3], const float* x,
                                             const float* W_e, const float* W_so2, const float* da, float* dx,
                                             float* dW_e, float* dW_so2, void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!pos || !box || !x || !W_e || !W_so2 || !dW_e || !dW_so2 || !col_ptr)
    return egnn_fail(ctx, EGNN_EINVAL, "so2_message_sum_backward: null pointer");
  int rc = so2_backward_check(ctx, g, ws, ws_bytes, false, "so2_message_sum_backward");
  if (rc) return rc;
  if ((g->n_total > 0 && !dx) || (g->n_owned > 0 && !da) || (g->n_edges > 0 && !perm))
    return egnn_fail(ctx, EGNN_EINVAL, "so2_message_sum_backward: null pointer");
  hipStream_t st = (hipStream_t)stream;
  const int lmax = ctx->desc.lmax, E = ctx->desc.channels, D = (lmax + 1) * (lmax + 1), n_rbf = ctx->desc.n_rbf;
  const long n = g->n_edges;
  if (n == 0) {
    // no message: every gradient is zero (a float zero is the integer zero)
    if ((rc = egnn_launch_fill_int(ctx, (int*)dx, (long)g->n_total * D * E, 0, st))) return rc;
    if ((rc = egnn_launch_fill_int(ctx, (int*)dW_e, (long)E * n_rbf, 0, st))) return rc;
    return egnn_launch_fill_int(ctx, (int*)dW_so2, (long)so2_w_offset(lmax, E, lmax + 1), 0, st);
  }
  So2Call call;
  if ((rc = so2_transform(ctx, g, pos, box, x, W_e, false, W_so2, ws, &call, st, false))) return rc;
  So2Bwd w;
  so2_bwd_ws(ctx, n, g->n_owned, false, true, (char*)ws, &w);
  const So2Grad grad = {da, false, 1.0f / sqrtf(ctx->desc.agg_norm), nullptr, nullptr, nullptr};
  if ((rc = so2_backward_tail(ctx, g, col_ptr, perm, false, W_so2, grad, call, w, dx, dW_so2, nullptr, nullptr, st)))
    return rc;
  // (the edge columns of dA_0 are still in place: the rotation back reads the node columns only)
  const long per = (n + SO2_DWE_CHUNKS - 1) / SO2_DWE_CHUNKS;
  const int chunks = (int)((n + per - 1) / per);
  hipLaunchKernelGGL(so2_dwe_kernel, dim3(chunks), dim3(256), 0, st, reinterpret_cast<const float4*>(call.rhat_d),
                     call.b.A[0], call.b.ldA[0], (lmax + 1) * 2 * E, n, per, ctx->log2_channels, n_rbf, ctx->desc.r_cut,
                     w.dwe);
  EGNN_LAUNCH_CHECK(ctx, "so2_dwe_kernel");
  return egnn_launch_reduce_partials(ctx, w.dwe, chunks, (long)E * n_rbf, dW_e, 1.0f, st);
}

extern "C" int egnn_so2_edge_block_backward(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr,
                                            const int32_t* perm, const float* pos, const float box[3], const float* x,
                                            const float* T_edge_in, const float* W_so2, const float* dT_out, float* dx,
                                            float* dT_in, float* dW_so2, void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!pos || !box || !x || !W_so2 || !dW_so2 || !col_ptr)
    return egnn_fail(ctx, EGNN_EINVAL, "so2_edge_block_backward: null pointer");
  int rc = so2_backward_check(ctx, g, ws, ws_bytes, true, "so2_edge_block_backward");
  if (rc) return rc;
  if ((g->n_total > 0 && !dx) || (g->n_edges > 0 && (!perm || !T_edge_in || !dT_out || !dT_in)))
    return egnn_fail(ctx, EGNN_EINVAL, "so2_edge_block_backward: null pointer");
  hipStream_t st = (hipStream_t)stream;
  const int lmax = ctx->desc.lmax, E = ctx->desc.channels, D = (lmax + 1) * (lmax + 1);
  const long n = g->n_edges;
  if (n == 0) {
    if ((rc = egnn_launch_fill_int(ctx, (int*)dx, (long)g->n_total * D * E, 0, st))) return rc;
    return egnn_launch_fill_int(ctx, (int*)dW_so2, (long)so2_w_offset(lmax, E, lmax + 1), 0, st);
  }
  So2Call call;
  if ((rc = so2_transform(ctx, g, pos, box, x, T_edge_in, true, W_so2, ws, &call, st, false))) return rc;
  So2Bwd w;
  so2_bwd_ws(ctx, n, g->n_owned, true, true, (char*)ws, &w);
  // T' = T + f_c y: the message term has gradient f_c dT', the identity term passes dT' on (added by so2_dx_kernel)
  const So2Grad grad = {dT_out, true, 1.0f, nullptr, nullptr, nullptr};
  return so2_backward_tail(ctx, g, col_ptr, perm, true, W_so2, grad, call, w, dx, dW_so2, dT_in, dT_out, st);
}

extern "C" int egnn_so2_node_block_backward(egnn_ctx* ctx, const egnn_graph* g, const int32_t* col_ptr,
                                            const int32_t* perm, const float* pos, const float box[3], const float* x,
                                            const float* T_edge, const float* W_so2, const float* w_att, const float* da,
                                            float* dx, float* dT_edge, float* dW_so2, float* dw_att, void* ws,
                                            size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!pos || !box || !x || !W_so2 || !w_att || !dW_so2 || !dw_att || !col_ptr)
    return egnn_fail(ctx, EGNN_EINVAL, "so2_node_block_backward: null pointer");
  int rc = so2_backward_check(ctx, g, ws, ws_bytes, true, "so2_node_block_backward");
  if (rc) return rc;
  if ((g->n_total > 0 && !dx) || (g->n_owned > 0 && !da) || (g->n_edges > 0 && (!perm || !T_edge || !dT_edge)))
    return egnn_fail(ctx, EGNN_EINVAL, "so2_node_block_backward: null pointer");
  hipStream_t st = (hipStream_t)stream;
  const int lmax = ctx->desc.lmax, E = ctx->desc.channels, D = (lmax + 1) * (lmax + 1);
  const long n = g->n_edges;
  if (n == 0) {
    if ((rc = egnn_launch_fill_int(ctx, (int*)dx, (long)g->n_total * D * E, 0, st))) return rc;
    if ((rc = egnn_launch_fill_int(ctx, (int*)dw_att, E, 0, st))) return rc;
    return egnn_launch_fill_int(ctx, (int*)dW_so2, (long)so2_w_offset(lmax, E, lmax + 1), 0, st);
  }
  // the forward pass up to the attention weights: Y_m and alpha in the workspace
  So2Call call;
  if ((rc = so2_transform(ctx, g, pos, box, x, T_edge, true, W_so2, ws, &call, st))) return rc;
  hipLaunchKernelGGL(so2_attention_kernel, dim3((g->n_owned + 3) / 4), dim3(256), 0, st, g->row_ptr, call.b.Y[0],
                     call.b.ldY[0], w_att, call.alpha, g->n_owned, E);
  EGNN_LAUNCH_CHECK(ctx, "so2_attention_kernel");
  So2Bwd w;
  so2_bwd_ws(ctx, n, g->n_owned, true, true, (char*)ws, &w);
  const float4* rd = reinterpret_cast<const float4*>(call.rhat_d);
#define ATT(L)                                                                                                     \
  hipLaunchKernelGGL(so2_attention_adjoint_kernel<L>, dim3(g->n_owned), dim3(256), 0, st, g->row_ptr, rd, call.b,  \
                     call.alpha, da, w.tds, w.dwatt, g->n_owned, ctx->log2_channels, ctx->desc.r_cut)
  SO2_BY_LMAX(lmax, ATT)
#undef ATT
  EGNN_LAUNCH_CHECK(ctx, "so2_attention_adjoint_kernel");
  if ((rc = egnn_launch_reduce_partials(ctx, w.dwatt, g->n_owned, (long)E, dw_att, 1.0f, st))) return rc;
  const So2Grad grad = {da, false, 1.0f, call.alpha, w.tds, w_att};
  return so2_backward_tail(ctx, g, col_ptr, perm, true, W_so2, grad, call, w, dx, dW_so2, dT_edge, nullptr, st);
}

// ---------------------------------------------------------------------------------------------- gate, reverse pass
// One workgroup per node.  With g_l = sigmoid(W_g[l-1] x0):  dx_l = dy_l g_l;  dz_l[c] = g_l (1 - g_l) sum_m dy_l[m][c]
// x_l[m][c] (kept in dz [n][lmax][E] for the weight gradient);  dx0 = dy0 SiLU'(x0) + sum_l W_g[l-1]^T dz_l.
__global__ __launch_bounds__(256) void so2_gate_backward_kernel(const float* __restrict__ x, const float* __restrict__ W_g,
                                                                const float* __restrict__ dy, float* __restrict__ dx,
                                                                float* __restrict__ dz, int lmax, int log2E) {
  __shared__ float s_x0[128];
  __shared__ float s_gate[4 * 128];
  __shared__ float s_dz[4 * 128];
  const int E = 1 << log2E, D = (lmax + 1) * (lmax + 1), tid = threadIdx.x;
  const float* xi = x + (((size_t)blockIdx.x * D) << log2E);
  const float* dyi = dy + (((size_t)blockIdx.x * D) << log2E);
  float* dxi = dx + (((size_t)blockIdx.x * D) << log2E);
  if (tid < E) s_x0[tid] = xi[tid];
  __syncthreads();
  for (int t = tid; t < (lmax << log2E); t += 256) {
    const float* wrow = W_g + ((size_t)t << log2E);     // row (l-1) * E + c
    float sc = 0.0f;
    for (int cc = 0; cc < E; ++cc) sc += wrow[cc] * s_x0[cc];
    const float gt = 1.0f / (1.0f + __expf(-sc));
    const int l = (t >> log2E) + 1, c = t & (E - 1);
    float dot = 0.0f;
    for (int q = l * l; q < (l + 1) * (l + 1); ++q) dot += dyi[(q << log2E) + c] * xi[(q << log2E) + c];
    const float v = dot * gt * (1.0f - gt);
    s_gate[t] = gt;
    s_dz[t] = v;
    dz[(((size_t)blockIdx.x * lmax) << log2E) + t] = v;
  }
  __syncthreads();
  for (int idx = tid; idx < (D << log2E); idx += 256) {
    const int q = idx >> log2E, c = idx & (E - 1);
    if (q == 0) {
      const float v = xi[idx];
      const float sg = 1.0f / (1.0f + __expf(-v));
      float sum = dyi[idx] * (sg * (1.0f + v * (1.0f - sg)));
      for (int t = 0; t < (lmax << log2E); ++t) sum += W_g[((size_t)t << log2E) + c] * s_dz[t];
      dxi[idx] = sum;
    } else {
      int l = 1;
      while ((l + 1) * (l + 1) <= q) ++l;
      dxi[idx] = dyi[idx] * s_gate[((l - 1) << log2E) + c];
    }
  }
}

// partial[chunk][l-1][c][c'] = sum over the nodes n of the chunk of dz[n][l-1][c] x[n][L = 0][c'].  grid = (chunks, lmax);
// a thread owns the outputs o = tid + 256 s (c' = o mod E: neighbouring threads, neighbouring columns).
#define GATE_WGRAD_CHUNKS 64
#define GATE_WGRAD_BATCH 8
__global__ __launch_bounds__(256) void so2_gate_wgrad_kernel(const float* __restrict__ dz, const float* __restrict__ x,
                                                             float* __restrict__ partial, int n_nodes, int per_chunk,
                                                             int lmax, int D, int log2E) {
  __shared__ float s_dz[GATE_WGRAD_BATCH * 128];
  __shared__ float s_x0[GATE_WGRAD_BATCH * 128];
  const int E = 1 << log2E, l1 = blockIdx.y, tid = threadIdx.x;
  const int n_begin = blockIdx.x * per_chunk;
  const int n_end = n_begin + per_chunk < n_nodes ? n_begin + per_chunk : n_nodes;
  float acc[64];     // E * E <= 128 * 128 = 64 * 256
#pragma unroll
  for (int s = 0; s < 64; ++s) acc[s] = 0.0f;
  for (int n0 = n_begin; n0 < n_end; n0 += GATE_WGRAD_BATCH) {
    __syncthreads();
    for (int i = tid; i < (GATE_WGRAD_BATCH << log2E); i += 256) {
      const int nn = n0 + (i >> log2E), c = i & (E - 1);
      const bool ok = nn < n_end;
      s_dz[i] = ok ? dz[((((size_t)nn * lmax) + l1) << log2E) + c] : 0.0f;
      s_x0[i] = ok ? x[(((size_t)nn * D) << log2E) + c] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 64; ++s) {
      const int o = tid + 256 * s;
      if (o < (E << log2E)) {
        const int c = o >> log2E, cp = o & (E - 1);
        float sum = acc[s];
#pragma unroll
        for (int b = 0; b < GATE_WGRAD_BATCH; ++b) sum += s_dz[(b << log2E) + c] * s_x0[(b << log2E) + cp];
        acc[s] = sum;
      }
    }
  }
  float* out = partial + (((size_t)blockIdx.x * lmax + l1) << (2 * log2E));
#pragma unroll
  for (int s = 0; s < 64; ++s) {
    const int o = tid + 256 * s;
    if (o < (E << log2E)) out[o] = acc[s];
  }
}

static size_t so2_gate_bwd_ws(const egnn_ctx* ctx, int32_t n_nodes) {
  const size_t E = ctx->desc.channels, lmax = ctx->desc.lmax;
  return so2_a256((size_t)n_nodes * lmax * E * sizeof(float)) + so2_a256((size_t)GATE_WGRAD_CHUNKS * lmax * E * E * sizeof(float));
}

extern "C" int egnn_gate_backward_workspace_bytes(const egnn_ctx* ctx, int32_t n_nodes, size_t* bytes) {
  if (!ctx || !bytes || n_nodes < 0) return EGNN_EINVAL;
  *bytes = so2_gate_bwd_ws(ctx, n_nodes) + 256;
  return EGNN_OK;
}

extern "C" int egnn_gate_backward(egnn_ctx* ctx, const float* x, const float* W_g, const float* dy, float* dx, float* dW_g,
                                  int32_t n_nodes, void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  const int lmax = ctx->desc.lmax, E = ctx->desc.channels;
  if (n_nodes < 0 || (n_nodes > 0 && (!x || !dy || !dx)) || (lmax > 0 && (!W_g || !dW_g)))
    return egnn_fail(ctx, EGNN_EINVAL, "gate_backward: bad argument");
  if (E > 128 || lmax > 4) return egnn_fail(ctx, EGNN_EINVAL, "gate_backward: unsupported shape");
  if (lmax > 0 && (!ws || ((uintptr_t)ws & 255) != 0 || ws_bytes < so2_gate_bwd_ws(ctx, n_nodes)))
    return egnn_fail(ctx, EGNN_EWS, "gate_backward: workspace missing, misaligned or too small");
  hipStream_t st = (hipStream_t)stream;
  const long n_w = (long)lmax * E * E;
  if (n_nodes == 0) return egnn_launch_fill_int(ctx, (int*)dW_g, n_w, 0, st);
  float* dz = (float*)ws;
  float* partial = (float*)((char*)ws + so2_a256((size_t)n_nodes * lmax * E * sizeof(float)));
  hipLaunchKernelGGL(so2_gate_backward_kernel, dim3(n_nodes), dim3(256), 0, st, x, W_g, dy, dx, dz, lmax,
                     ctx->log2_channels);
  EGNN_LAUNCH_CHECK(ctx, "so2_gate_backward_kernel");
  if (lmax == 0) return EGNN_OK;
  int chunks = n_nodes < GATE_WGRAD_CHUNKS ? n_nodes : GATE_WGRAD_CHUNKS;
  const int per = (n_nodes + chunks - 1) / chunks;
  chunks = (n_nodes + per - 1) / per;
  hipLaunchKernelGGL(so2_gate_wgrad_kernel, dim3(chunks, lmax), dim3(256), 0, st, dz, x, partial, n_nodes, per, lmax,
                     (lmax + 1) * (lmax + 1), ctx->log2_channels);
  EGNN_LAUNCH_CHECK(ctx, "so2_gate_wgrad_kernel");
  return egnn_launch_reduce_partials(ctx, partial, chunks, n_w, dW_g, 1.0f, st);
}
