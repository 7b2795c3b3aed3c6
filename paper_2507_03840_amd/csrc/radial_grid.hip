// Reverse pass of the radial MLP (S3) in one pass over dw, by interpolation on a grid of distances.
//
//   dW_r2[n][j] = alpha_n sum_k dw[k][n] G_j(d_k),                              G_j(d) = f_c(d) SiLU(pre_j(d))
//   dW_r1[j][b] = sum_k S_j(d_k) B_b(d_k) sum_n dw[k][n] alpha_n W_r2[n][j],    S_j(d) = f_c(d) SiLU'(pre_j(d))
//
// Everything the edge contributes besides its row dw[k][:] is a smooth function of its length alone (the radial
// basis, the envelope and the hidden layer act on d_k: Sec. 3 "Initialization").  A smooth f is reproduced from its
// values on a grid d_i = i h by six-point Lagrange interpolation, f(d_k) = sum_i phi_i(d_k) f(d_i) up to
// O(h^6 f^(6)), so with  Z[i][n] = alpha_n sum_k phi_i(d_k) dw[k][n]  (six non-zero phi per edge)
//   dW_r2[n][j] = sum_i Z[i][n] G_j(d_i),      dW_r1[j][b] = sum_i S_j(d_i) B_b(d_i) sum_n Z[i][n] W_r2[n][j].
// Z is a weighted binning of the rows of dw -- one streaming pass over dw, four multiply-adds per value and no
// contraction at all -- and what follows are two small dense products over the ~2,000 grid points.  The exact route
// (radial_backward.hip) streams dw twice through the matrix cores; this one reads it once.
//
// Grid: RG_BINS intervals over [0, r_cut), h = r_cut / RG_BINS; an edge in interval m (d in [m h, (m+1) h)) uses the
// grid points m-2 .. m+3, stored as nodes m .. m+5 (node i <-> distance (i - 2) h; the functions are evaluated a little
// outside [0, r_cut] by the same analytic formulas).  Interpolation error, measured against fp64 on this layer's
// functions: 1e-12 of the result for weights of the size the model is initialised with, 5e-9 when the rows of W_r1
// have an absolute sum of 100; it grows like the 4.7th power of that sum, so a device-side switch (rg_route_kernel)
// leaves the work to the exact route beyond 256, where it would pass 1e-6.
//
// Determinism: the edges of an interval are visited in ascending edge id (a counting sort by interval with integer
// atomics, then a rank sort inside each interval), every sum has a fixed order, no floating-point atomics.
#include "egnn_internal.h"

#define RG_BINS 2048
#define RG_PTS 6
#define RG_NODES (RG_BINS + RG_PTS - 1)
#define RG_COLS 1024          // columns of dw per workgroup of the binning pass (256 threads x float4)
#define RG_L1_LIMIT 256.0f    // largest absolute row sum of W_r1 this route accepts (at 16 radial bases; scaled with
                              // the inverse width of the Gaussians, n_rbf - 1, otherwise)
typedef float rg_f4 __attribute__((ext_vector_type(4)));

static size_t rg_a256(size_t n) { return (n + 255) & ~(size_t)255; }

// route[0] = 1: this route computes the gradients, 0: the exact route does.  forced: 0 decide from W_r1, 1 exact, 2 grid.
__global__ __launch_bounds__(64) void rg_route_kernel(const float* __restrict__ W_r1, int n_rbf, int forced,
                                                      int* __restrict__ route) {
  float s = 0.0f;
  for (int b = 0; b < n_rbf; ++b) s += fabsf(W_r1[threadIdx.x * n_rbf + b]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s = fmaxf(s, __shfl_xor(s, off));
  // the hidden layer's input varies with d at a rate ~ (row sum) / (width of a Gaussian) = s (n_rbf - 1) / r_cut
  const bool smooth = s * (float)(n_rbf - 1) <= RG_L1_LIMIT * 15.0f;                                   // (NaN: exact route)
  if (threadIdx.x == 0) route[0] = forced == 2 ? 1 : (forced == 1 ? 0 : (smooth ? 1 : 0));
}

__device__ __forceinline__ int rg_bin(float d, float inv_h) {
  const int m = (int)floorf(d * inv_h);
  return m < 0 ? 0 : (m > RG_BINS - 1 ? RG_BINS - 1 : m);
}

// key[k] = interval of edge k; cnt[m + 1] += 1
__global__ __launch_bounds__(256) void rg_key_kernel(const float4* __restrict__ rhat_d, long n_edges, float inv_h,
                                                     int* __restrict__ key, int* __restrict__ cnt,
                                                     const int* __restrict__ route) {
  if (route && !route[0]) return;
  const long k = (long)blockIdx.x * 256 + threadIdx.x;
  if (k >= n_edges) return;
  const int m = rg_bin(rhat_d[k].w, inv_h);
  key[k] = m;
  atomicAdd(&cnt[m + 1], 1);    // integer: the result does not depend on the order
}

__global__ __launch_bounds__(256) void rg_fill_kernel(const int* __restrict__ key, long n_edges,
                                                      const int* __restrict__ bin_ptr, int* __restrict__ cursor,
                                                      int* __restrict__ bucket, const int* __restrict__ route) {
  if (route && !route[0]) return;
  const long k = (long)blockIdx.x * 256 + threadIdx.x;
  if (k >= n_edges) return;
  const int m = key[k];
  bucket[bin_ptr[m] + atomicAdd(&cursor[m], 1)] = (int)k;
}

// One workgroup per interval: rank sort of its edges (ascending id), so that the binning pass adds them in a fixed order.
__global__ __launch_bounds__(256) void rg_sort_kernel(const int* __restrict__ bin_ptr, const int* __restrict__ bucket,
                                                      int* __restrict__ perm, const int* __restrict__ route) {
  if (route && !route[0]) return;
  const int m = blockIdx.x;
  const int c0 = bin_ptr[m], c1 = bin_ptr[m + 1];
  for (int a = c0 + threadIdx.x; a < c1; a += 256) {
    const int e = bucket[a];
    int rank = 0;
    for (int b = c0; b < c1; ++b) rank += bucket[b] < e ? 1 : 0;
    perm[c0 + rank] = e;
  }
}

// Lagrange weights of the six grid points -2 .. 3 around an interval, at position t in [0, 1) inside it
__device__ __forceinline__ void rg_weights(float t, float (&phi)[RG_PTS]) {
  const float a = t + 2.0f, b = t + 1.0f, c = t, d = t - 1.0f, e = t - 2.0f, f = t - 3.0f;
  phi[0] = b * c * d * e * f * (-1.0f / 120.0f);
  phi[1] = a * c * d * e * f * (1.0f / 24.0f);
  phi[2] = a * b * d * e * f * (-1.0f / 12.0f);
  phi[3] = a * b * c * e * f * (1.0f / 12.0f);
  phi[4] = a * b * c * d * f * (-1.0f / 24.0f);
  phi[5] = a * b * c * d * e * (1.0f / 120.0f);
}

// The binning pass.  grid = (interval, column tile); a thread owns four consecutive columns of dw and adds the rows
// of the interval's edges, in ascending edge id, into six running sums (one per grid point the interval touches):
// Zp[m][i][n] = sum_{k in interval m} phi_i(d_k) dw[k][n].  RG_UNROLL rows are requested before the first is used.
#define RG_UNROLL 8
__global__ __launch_bounds__(256) void rg_bin_kernel(const float* __restrict__ dw, const float4* __restrict__ rhat_d,
                                                     const int* __restrict__ bin_ptr, const int* __restrict__ perm,
                                                     float* __restrict__ Zp, int n_edges, int PE, int cols_per_wg,
                                                     float inv_h, const int* __restrict__ route) {
  if (!route[0]) return;
  // (the number of edges grows with the square of the distance: the longest intervals are started first)
  const int m = RG_BINS - 1 - (int)blockIdx.x;
  const int col = blockIdx.y * cols_per_wg + threadIdx.x * 4;
  if (threadIdx.x * 4 >= cols_per_wg || col >= PE) return;
  const int c0 = bin_ptr[m], c1 = bin_ptr[m + 1];
  float4 acc[RG_PTS];
#pragma unroll
  for (int i = 0; i < RG_PTS; ++i) acc[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  int a = c0;
  for (; a + RG_UNROLL <= c1; a += RG_UNROLL) {
    int e[RG_UNROLL];
    float4 x[RG_UNROLL];
    float dd[RG_UNROLL];
#pragma unroll
    for (int u = 0; u < RG_UNROLL; ++u) e[u] = min(max(perm[a + u], 0), n_edges - 1);
#pragma unroll
    for (int u = 0; u < RG_UNROLL; ++u) {
      const rg_f4 v = __builtin_nontemporal_load(reinterpret_cast<const rg_f4*>(dw + (size_t)e[u] * PE + col));
      x[u] = make_float4(v.x, v.y, v.z, v.w);
      dd[u] = rhat_d[e[u]].w;
    }
#pragma unroll
    for (int u = 0; u < RG_UNROLL; ++u) {
      float phi[RG_PTS];
      rg_weights(dd[u] * inv_h - (float)m, phi);
#pragma unroll
      for (int i = 0; i < RG_PTS; ++i) {
        acc[i].x += phi[i] * x[u].x;
        acc[i].y += phi[i] * x[u].y;
        acc[i].z += phi[i] * x[u].z;
        acc[i].w += phi[i] * x[u].w;
      }
    }
  }
  for (; a < c1; ++a) {
    const int e = min(max(perm[a], 0), n_edges - 1);
    const float4 x = *reinterpret_cast<const float4*>(dw + (size_t)e * PE + col);
    float phi[RG_PTS];
    rg_weights(rhat_d[e].w * inv_h - (float)m, phi);
#pragma unroll
    for (int i = 0; i < RG_PTS; ++i) {
      acc[i].x += phi[i] * x.x;
      acc[i].y += phi[i] * x.y;
      acc[i].z += phi[i] * x.z;
      acc[i].w += phi[i] * x.w;
    }
  }
  float* out = Zp + ((size_t)m * RG_PTS) * PE + col;
#pragma unroll
  for (int i = 0; i < RG_PTS; ++i) *reinterpret_cast<float4*>(out + (size_t)i * PE) = acc[i];
}

// Z[node][n] = alpha_n * sum over the (at most six) intervals m = node - i that touch the node of Zp[m][i][n]
__global__ __launch_bounds__(256) void rg_assemble_kernel(const float* __restrict__ Zp, float* __restrict__ Z, int PE,
                                                          int log2E, PathAlpha alpha, const int* __restrict__ route) {
  if (!route[0]) return;
  const int node = blockIdx.x;
  for (int n = threadIdx.x; n < PE; n += 256) {
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < RG_PTS; ++i) {
      const int m = node - i;
      if (m >= 0 && m < RG_BINS) s += Zp[((size_t)m * RG_PTS + i) * PE + n];
    }
    Z[(size_t)node * PE + n] = alpha.a[n >> log2E] * s;
  }
}

// the grid points as edge records (only the length is read), so that radial_hidden_kernel can evaluate G and S there
__global__ __launch_bounds__(256) void rg_nodes_kernel(float4* __restrict__ rd_nodes, float h) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < RG_NODES) rd_nodes[i] = make_float4(0.0f, 0.0f, 1.0f, (float)(i - 2) * h);
}

// C_partial[chunk][m][0..63] = sum_{k in chunk} A(m, k) B[k][0..63], plain fp32.  A_KMAJOR: A(m, k) = A[k * lda + m],
// else A[m * lda + k].  64 x 64 output tile per workgroup, a thread owns 4 x 4 of it; grid = (row tiles, k chunks).
template <bool A_KMAJOR>
__global__ __launch_bounds__(256) void rg_gemm64_kernel(const float* __restrict__ A, long lda,
                                                        const float* __restrict__ B, float* __restrict__ C_partial,
                                                        int M, int K, int k_chunk, const int* __restrict__ route) {
  if (!route[0]) return;
  __shared__ float As[16][68];
  __shared__ float Bs[16][64];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.x * 64;
  const int k_begin = blockIdx.y * k_chunk;
  const int k_end = k_begin + k_chunk < K ? k_begin + k_chunk : K;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;
  for (int k0 = k_begin; k0 < k_end; k0 += 16) {
    if (A_KMAJOR) {
      const int k = k0 + (tid >> 4), m = m0 + (tid & 15) * 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) As[tid >> 4][(tid & 15) * 4 + i] = (k < k_end && m + i < M) ? A[(size_t)k * lda + m + i] : 0.0f;
    } else {
      const int m = m0 + (tid >> 2), k = k0 + (tid & 3) * 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) As[(tid & 3) * 4 + i][tid >> 2] = (m < M && k + i < k_end) ? A[(size_t)m * lda + k + i] : 0.0f;
    }
    {
      const int k = k0 + (tid >> 4);
      const float4 v = k < k_end ? *reinterpret_cast<const float4*>(B + (size_t)k * 64 + (tid & 15) * 4)
                                 : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      *reinterpret_cast<float4*>(&Bs[tid >> 4][(tid & 15) * 4]) = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      const float4 a = *reinterpret_cast<const float4*>(&As[kk][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&Bs[kk][tx * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
    }
    __syncthreads();
  }
  float* out = C_partial + (size_t)blockIdx.y * M * 64;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m < M) *reinterpret_cast<float4*>(out + (size_t)m * 64 + tx * 4) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
  }
}

// out[i] = sum_c partial[c][i] in ascending c (route-gated: the shared reduction kernels are not)
__global__ __launch_bounds__(256) void rg_sum_kernel(const float* __restrict__ partial, int n_partials, long n,
                                                     float* __restrict__ out, const int* __restrict__ route) {
  if (!route[0]) return;
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float s = 0.0f;
  for (int c = 0; c < n_partials; ++c) s += partial[(size_t)c * n + i];
  out[i] = s;
}

// Partial dW_r1 over a chunk of RG_DW1_NODES grid points: partial[chunk][j][b] = sum_node S_j(d_node) U[node][j] B_b(d_node);
// grid = (basis b, chunk), the four waves split the chunk's nodes, lane = j
#define RG_DW1_NODES 128
__global__ __launch_bounds__(256) void rg_dw1_kernel(const float* __restrict__ Sn, const float* __restrict__ U,
                                                     float* __restrict__ partial, int n_rbf, float r_cut, float h,
                                                     const int* __restrict__ route) {
  if (!route[0]) return;
  __shared__ float red[4][64];
  const int b = blockIdx.x, j = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
  const int n0 = blockIdx.y * RG_DW1_NODES;
  const int n1 = n0 + RG_DW1_NODES < RG_NODES ? n0 + RG_DW1_NODES : RG_NODES;
  float acc = 0.0f;
  for (int node = n0 + wv; node < n1; node += 4) {
    const float u = (float)(node - 2) * h - (float)b * step;
    acc += Sn[(size_t)node * 64 + j] * U[(size_t)node * 64 + j] * __expf(-u * u * inv2s2);
  }
  red[wv][j] = acc;
  __syncthreads();
  if (wv == 0) partial[((size_t)blockIdx.y * 64 + j) * n_rbf + b] = (red[0][j] + red[1][j]) + (red[2][j] + red[3][j]);
}

#define RG_KCHUNK_NODES 128   // grid points per partial of dW_r2
#define RG_KCHUNK_COLS 128    // columns per partial of U

size_t egnn_radial_grid_ws_bytes(const egnn_ctx* ctx, int which, int64_t n_edges) {
  const size_t PE = (size_t)ctx->n_paths[which] * ctx->desc.channels;
  const size_t c2 = (RG_NODES + RG_KCHUNK_NODES - 1) / RG_KCHUNK_NODES, cu = (PE + RG_KCHUNK_COLS - 1) / RG_KCHUNK_COLS;
  const size_t part = (c2 * PE > cu * RG_NODES ? c2 * PE : cu * RG_NODES) * 64 * sizeof(float);
  return 3 * rg_a256((size_t)n_edges * sizeof(int)) + 2 * rg_a256(((size_t)RG_BINS + 1) * sizeof(int)) +
         rg_a256((size_t)RG_NODES * sizeof(float4)) + 3 * rg_a256((size_t)RG_NODES * 64 * sizeof(float)) +
         rg_a256((size_t)RG_BINS * RG_PTS * PE * sizeof(float)) + rg_a256((size_t)RG_NODES * PE * sizeof(float)) +
         rg_a256(part);
}

// Enqueues the grid route; every kernel returns at once unless route[0] is 1 (set on the device by rg_route_kernel).
// hidden_launch: evaluates G and S at given edge records (radial_hidden_kernel of the exact route, not gated).
int egnn_launch_radial_grid(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges, const int* len_ptr,
                            const int* len_perm, const float* W_r1,
                            const float* W_r2, const float* dw, float* dW_r1, float* dW_r2, void* ws, const int* route,
                            int (*hidden_launch)(egnn_ctx*, const float*, long, const float*, float*, float*, hipStream_t),
                            hipStream_t st) {
  const int P = ctx->n_paths[which];
  const int PE = P * ctx->desc.channels, n_rbf = ctx->desc.n_rbf;
  PathAlpha al;
  for (int p = 0; p < EGNN_MAX_PATHS; ++p) al.a[p] = p < P ? ctx->alpha[which][p] : 0.0f;
  const float h = ctx->desc.r_cut / (float)RG_BINS, inv_h = (float)RG_BINS / ctx->desc.r_cut;
  char* p = (char*)ws;
  auto take = [&](size_t bytes) { char* q = p; p += rg_a256(bytes); return q; };
  int* key = (int*)take((size_t)n_edges * sizeof(int));
  int* bucket = (int*)take((size_t)n_edges * sizeof(int));
  int* perm = (int*)take((size_t)n_edges * sizeof(int));
  int* bin_ptr = (int*)take(((size_t)RG_BINS + 1) * sizeof(int));
  int* cursor = (int*)take(((size_t)RG_BINS + 1) * sizeof(int));
  float* rd_nodes = (float*)take((size_t)RG_NODES * sizeof(float4));
  float* Gn = (float*)take((size_t)RG_NODES * 64 * sizeof(float));
  float* Sn = (float*)take((size_t)RG_NODES * 64 * sizeof(float));
  float* U = (float*)take((size_t)RG_NODES * 64 * sizeof(float));
  float* Zp = (float*)take((size_t)RG_BINS * RG_PTS * PE * sizeof(float));
  float* Z = (float*)take((size_t)RG_NODES * PE * sizeof(float));
  float* part = (float*)p;
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
  int rc;
  const dim3 b256(256);
  // the edges grouped by length interval: given with the graph (egnn_length_bins, once per graph), else built here
  if (len_ptr && len_perm) {
    bin_ptr = const_cast<int*>(len_ptr);
    perm = const_cast<int*>(len_perm);
  } else if ((rc = egnn_launch_length_bins(ctx, rd, n_edges, bin_ptr, perm, key, bucket, cursor, route, st))) {
    return rc;
  }
  // the one pass over dw
  // column tiles of equal width (a multiple of four columns, at most RG_COLS)
  const int n_tiles = (PE + RG_COLS - 1) / RG_COLS;
  const int cols_per_wg = ((PE + n_tiles - 1) / n_tiles + 3) & ~3;
  hipLaunchKernelGGL(rg_bin_kernel, dim3(RG_BINS, n_tiles), b256, 0, st, dw, rd, bin_ptr, perm, Zp, (int)n_edges, PE,
                     cols_per_wg, inv_h, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_bin_kernel");
  hipLaunchKernelGGL(rg_assemble_kernel, dim3(RG_NODES), b256, 0, st, Zp, Z, PE, ctx->log2_channels, al, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_assemble_kernel");
  // G and S at the grid points
  hipLaunchKernelGGL(rg_nodes_kernel, dim3((RG_NODES + 255) / 256), b256, 0, st, reinterpret_cast<float4*>(rd_nodes), h);
  EGNN_LAUNCH_CHECK(ctx, "rg_nodes_kernel");
  if ((rc = hidden_launch(ctx, rd_nodes, RG_NODES, W_r1, Gn, Sn, st))) return rc;
  // dW_r2 = Z^T G
  const int c2 = (RG_NODES + RG_KCHUNK_NODES - 1) / RG_KCHUNK_NODES;
  hipLaunchKernelGGL(rg_gemm64_kernel<true>, dim3((PE + 63) / 64, c2), b256, 0, st, Z, (long)PE, Gn, part, PE, RG_NODES,
                     RG_KCHUNK_NODES, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_gemm64_kernel<dW_r2>");
  hipLaunchKernelGGL(rg_sum_kernel, dim3((unsigned)(((long)PE * 64 + 255) / 256)), b256, 0, st, part, c2, (long)PE * 64,
                     dW_r2, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_sum_kernel<dW_r2>");
  // U = Z W_r2, then dW_r1
  const int cu = (PE + RG_KCHUNK_COLS - 1) / RG_KCHUNK_COLS;
  hipLaunchKernelGGL(rg_gemm64_kernel<false>, dim3((RG_NODES + 63) / 64, cu), b256, 0, st, Z, (long)PE, W_r2, part, RG_NODES,
                     PE, RG_KCHUNK_COLS, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_gemm64_kernel<U>");
  hipLaunchKernelGGL(rg_sum_kernel, dim3((unsigned)(((long)RG_NODES * 64 + 255) / 256)), b256, 0, st, part, cu,
                     (long)RG_NODES * 64, U, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_sum_kernel<U>");
  const int c1 = (RG_NODES + RG_DW1_NODES - 1) / RG_DW1_NODES;     // (64 * n_rbf floats each: far inside `part`)
  hipLaunchKernelGGL(rg_dw1_kernel, dim3(n_rbf, c1), b256, 0, st, Sn, U, part, n_rbf, ctx->desc.r_cut, h, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_dw1_kernel");
  hipLaunchKernelGGL(rg_sum_kernel, dim3((64 * n_rbf + 255) / 256), b256, 0, st, part, c1, (long)64 * n_rbf, dW_r1, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_sum_kernel<dW_r1>");
  return EGNN_OK;
}

// bin_ptr [RG_BINS + 1], perm [n_edges]: edge ids grouped by length interval, ascending inside an interval.
// key, bucket [n_edges], cursor [RG_BINS]: scratch.  route (may be NULL): device word that gates the kernels.
int egnn_launch_length_bins(egnn_ctx* ctx, const float4* rd, int64_t n_edges, int* bin_ptr, int* perm, int* key,
                            int* bucket, int* cursor, const int* route, hipStream_t st) {
  const float inv_h = (float)RG_BINS / ctx->desc.r_cut;
  int rc;
  if ((rc = egnn_launch_fill_int(ctx, bin_ptr, RG_BINS + 1, 0, st))) return rc;
  if ((rc = egnn_launch_fill_int(ctx, cursor, RG_BINS, 0, st))) return rc;
  if (n_edges == 0) return EGNN_OK;
  const dim3 ge((unsigned)((n_edges + 255) / 256)), b256(256);
  hipLaunchKernelGGL(rg_key_kernel, ge, b256, 0, st, rd, (long)n_edges, inv_h, key, bin_ptr, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_key_kernel");
  if ((rc = egnn_launch_row_scan(ctx, bin_ptr, RG_BINS, st))) return rc;
  hipLaunchKernelGGL(rg_fill_kernel, ge, b256, 0, st, key, (long)n_edges, bin_ptr, cursor, bucket, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_fill_kernel");
  hipLaunchKernelGGL(rg_sort_kernel, dim3(RG_BINS), b256, 0, st, bin_ptr, bucket, perm, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_sort_kernel");
  return EGNN_OK;
}

size_t egnn_length_bins_ws_bytes(int64_t n_edges) {
  return rg_a256((size_t)n_edges * 16) + 2 * rg_a256((size_t)n_edges * sizeof(int)) + rg_a256((size_t)RG_BINS * sizeof(int));
}

extern "C" int egnn_length_bins_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, size_t* bytes) {
  if (!ctx || !bytes || n_edges < 0) return EGNN_EINVAL;
  *bytes = egnn_length_bins_ws_bytes(n_edges);
  return EGNN_OK;
}

extern "C" int egnn_length_bins(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                int32_t* len_ptr, int32_t* len_perm, void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!g || !pos || !box || !len_ptr || g->n_edges < 0 || g->n_edges > 2147483647LL ||
      (g->n_edges > 0 && (!g->src || !g->dst || !len_perm)))
    return egnn_fail(ctx, EGNN_EINVAL, "length_bins: null pointer or bad sizes");
  if (g->n_edges > 0 && (!ws || ((uintptr_t)ws & 255) != 0 || ws_bytes < egnn_length_bins_ws_bytes(g->n_edges)))
    return egnn_fail(ctx, EGNN_EWS, "length_bins: workspace missing, misaligned or too small");
  hipStream_t st = (hipStream_t)stream;
  char* p = (char*)ws;
  float* rhat_d = (float*)p;
  p += rg_a256((size_t)g->n_edges * 16);
  int* key = (int*)p;
  p += rg_a256((size_t)g->n_edges * sizeof(int));
  int* bucket = (int*)p;
  p += rg_a256((size_t)g->n_edges * sizeof(int));
  int* cursor = (int*)p;
  int rc;
  if (g->n_edges == 0) return egnn_launch_fill_int(ctx, len_ptr, RG_BINS + 1, 0, st);
  if ((rc = egnn_launch_geometry(ctx, g, pos, box, rhat_d, nullptr, nullptr, nullptr, st))) return rc;
  return egnn_launch_length_bins(ctx, reinterpret_cast<const float4*>(rhat_d), g->n_edges, len_ptr, len_perm, key, bucket,
                                 cursor, nullptr, st);
}

int egnn_launch_radial_route(egnn_ctx* ctx, const float* W_r1, int* route, hipStream_t st) {
  hipLaunchKernelGGL(rg_route_kernel, dim3(1), dim3(64), 0, st, W_r1, ctx->desc.n_rbf, ctx->radial_bwd_route, route);
  EGNN_LAUNCH_CHECK(ctx, "rg_route_kernel");
  return EGNN_OK;
}
