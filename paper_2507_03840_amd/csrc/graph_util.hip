// Small graph / reduction utilities of the reverse pass:
//   * source-sorted ("transposed") edge index: col_ptr over sources and the permutation of edge ids,
//     so that gradients w.r.t. source rows are summed in a fixed order without floating-point atomics;
//   * segmented sum of per-edge rows; sum of per-workgroup partial results; MSE loss.
#include "egnn_internal.h"

__global__ void fill_int_kernel(int* p, long n, int v) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ void count_src_kernel(const int* __restrict__ src, long n_edges, int* __restrict__ cnt) {
  const long k = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n_edges) atomicAdd(&cnt[src[k] + 1], 1);  // integer atomics: the result does not depend on order
}

__global__ void fill_src_kernel(const int* __restrict__ src, long n_edges, const int* __restrict__ col_ptr,
                                int* __restrict__ cursor, int* __restrict__ bucket) {
  const long k = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n_edges) return;
  const int s = src[k];
  bucket[col_ptr[s] + atomicAdd(&cursor[s], 1)] = (int)k;
}

// One wavefront per source: rank sort of its bucket (ascending edge id = ascending destination), so the
// order in which the reverse pass adds up the edges of a source is fixed.
__global__ __launch_bounds__(256) void sort_bucket_kernel(const int* __restrict__ col_ptr,
                                                          const int* __restrict__ bucket, int* __restrict__ perm,
                                                          int n_total) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= n_total) return;
  const int c0 = col_ptr[i], c1 = col_ptr[i + 1];
  for (int a = c0 + lane; a < c1; a += 64) {
    const int e = bucket[a];
    int rank = 0;
    for (int b = c0; b < c1; ++b) rank += bucket[b] < e ? 1 : 0;
    perm[c0 + rank] = e;
  }
}

// out[i][:] = sum over idx in ptr[i]..ptr[i+1] of rows[perm ? perm[idx] : idx][:], fixed order.
__global__ __launch_bounds__(256) void edge_rows_segsum_kernel(const float* __restrict__ rows,
                                                               const int* __restrict__ ptr,
                                                               const int* __restrict__ perm, float* __restrict__ out,
                                                               int row_len) {
  const int i = blockIdx.x;
  const int p0 = ptr[i], p1 = ptr[i + 1];
  // four interleaved running sums (position in the segment mod 4): four row loads in flight per thread, fixed order
  for (int q = threadIdx.x; q < row_len; q += 256) {
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    int idx = p0;
    for (; idx + 4 <= p1; idx += 4) {
      float v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const long k = perm ? perm[idx + u] : idx + u;
        v[u] = __builtin_nontemporal_load(rows + k * row_len + q);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] += v[u];
    }
    for (int u = 0; idx < p1; ++idx, ++u) {
      const long k = perm ? perm[idx] : idx;
      acc[u] += rows[k * row_len + q];
    }
    out[(long)i * row_len + q] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  }
}

// out[i] = scale * sum_b partial[b * stride][i] in a fixed order: eight interleaved running sums (b mod 8), so that
// eight loads are in flight per thread, combined pairwise at the end.
__global__ void reduce_partials_kernel(const float* __restrict__ partial, int n_partials, long stride, long n,
                                       float* __restrict__ out, float scale, const int* __restrict__ skip) {
  if (skip && skip[0]) return;   // (a caller whose result another route computes: radial_grid.hip)
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
  const long step = stride * n;
  int b = 0;
  for (; b + 8 <= n_partials; b += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(partial + (long)(b + u) * step + i);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] += v[u];
  }
  for (int u = 0; b < n_partials; ++b, ++u) acc[u] += partial[(long)b * step + i];
  out[i] = (((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]))) * scale;
}

// First level for long lists of partials: blockIdx.y takes RP_CHUNK consecutive rows and leaves their sum in the
// first of them (every element of the buffer is read and written by one thread only).
#define RP_CHUNK 32
__global__ void reduce_partials_chunk_kernel(float* __restrict__ partial, int n_partials, long n,
                                             const int* __restrict__ skip) {
  if (skip && skip[0]) return;
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int b0 = blockIdx.y * RP_CHUNK;
  const int cnt = n_partials - b0 < RP_CHUNK ? n_partials - b0 : RP_CHUNK;
  float* base = partial + (long)b0 * n + i;
  float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
  int b = 0;
  for (; b + 8 <= cnt; b += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = base[(long)(b + u) * n];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] += v[u];
  }
  for (int u = 0; b < cnt; ++b, ++u) acc[u] += base[(long)b * n];
  base[0] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
}

#define LOSS_PER_BLOCK 4096
__global__ __launch_bounds__(256) void loss_mse_partial_kernel(const float* __restrict__ H, const float* __restrict__ T,
                                                               long n, float* __restrict__ dH,
                                                               double* __restrict__ partial, float grad_scale) {
  __shared__ double red[256];
  const long base = (long)blockIdx.x * LOSS_PER_BLOCK;
  double acc = 0.0;
  for (int q = 0; q < LOSS_PER_BLOCK / 256; ++q) {
    const long i = base + q * 256 + threadIdx.x;
    if (i < n) {
      const float diff = H[i] - T[i];
      acc += (double)diff * (double)diff;
      if (dH) dH[i] = grad_scale * diff;
    }
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

__global__ __launch_bounds__(256) void loss_mse_final_kernel(const double* __restrict__ partial, int n_partials,
                                                             double inv_n, float* __restrict__ loss) {
  __shared__ double red[256];
  double acc = 0.0;
  for (int b = threadIdx.x; b < n_partials; b += 256) acc += partial[b];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = (float)(red[0] * inv_n);
}

int egnn_launch_fill_int(egnn_ctx* ctx, int* p, long n, int v, hipStream_t st) {
  if (n <= 0) return EGNN_OK;
  hipLaunchKernelGGL(fill_int_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, v);
  EGNN_LAUNCH_CHECK(ctx, "fill_int_kernel");
  return EGNN_OK;
}

int egnn_launch_segsum_rows(egnn_ctx* ctx, const float* rows, const int* ptr, const int* perm, float* out,
                            int n_segments, int row_len, hipStream_t st) {
  if (n_segments <= 0) return EGNN_OK;
  hipLaunchKernelGGL(edge_rows_segsum_kernel, dim3(n_segments), dim3(256), 0, st, rows, ptr, perm, out, row_len);
  EGNN_LAUNCH_CHECK(ctx, "edge_rows_segsum_kernel");
  return EGNN_OK;
}

// `partial` is scratch: long lists are summed in two levels, the first one in place.
int egnn_launch_reduce_partials(egnn_ctx* ctx, float* partial, int n_partials, long n, float* out, float scale,
                                hipStream_t st, const int* skip) {
  if (n <= 0) return EGNN_OK;
  const unsigned gx = (unsigned)((n + 255) / 256);
  long stride = 1;
  if (n_partials > 8 * RP_CHUNK) {
    const int n_chunks = (n_partials + RP_CHUNK - 1) / RP_CHUNK;
    if (n_chunks > 65535) return egnn_fail(ctx, EGNN_EINVAL, "reduce_partials: too many partial results");
    hipLaunchKernelGGL(reduce_partials_chunk_kernel, dim3(gx, (unsigned)n_chunks), dim3(256), 0, st, partial,
                       n_partials, n, skip);
    EGNN_LAUNCH_CHECK(ctx, "reduce_partials_chunk_kernel");
    n_partials = n_chunks;
    stride = RP_CHUNK;
  }
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(gx), dim3(256), 0, st, partial, n_partials, stride, n, out, scale,
                     skip);
  EGNN_LAUNCH_CHECK(ctx, "reduce_partials_kernel");
  return EGNN_OK;
}

size_t egnn_transpose_ws_bytes(int64_t n_edges, int32_t n_total) {
  return (((size_t)n_total * sizeof(int) + 255) & ~(size_t)255) + (((size_t)n_edges * sizeof(int) + 255) & ~(size_t)255);
}

extern "C" int egnn_graph_transpose(egnn_ctx* ctx, const egnn_graph* g, int32_t* col_ptr, int32_t* perm, void* ws,
                                    size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!g || !col_ptr || g->n_edges < 0 || g->n_total < 0 || (g->n_edges > 0 && (!g->src || !perm || !ws)))
    return egnn_fail(ctx, EGNN_EINVAL, "graph_transpose: null pointer or bad sizes");
  if (g->n_edges > 0 && ws_bytes < egnn_transpose_ws_bytes(g->n_edges, g->n_total))
    return egnn_fail(ctx, EGNN_EWS, "graph_transpose: workspace too small");
  hipStream_t st = (hipStream_t)stream;
  const long n_e = g->n_edges;
  int rc;
  if ((rc = egnn_launch_fill_int(ctx, col_ptr, (long)g->n_total + 1, 0, st))) return rc;
  if (n_e == 0) return EGNN_OK;
  int* cursor = (int*)ws;
  int* bucket = (int*)((char*)ws + (((size_t)g->n_total * sizeof(int) + 255) & ~(size_t)255));
  if ((rc = egnn_launch_fill_int(ctx, cursor, g->n_total, 0, st))) return rc;
  const dim3 ge((unsigned)((n_e + 255) / 256)), b(256);
  hipLaunchKernelGGL(count_src_kernel, ge, b, 0, st, g->src, n_e, col_ptr);
  EGNN_LAUNCH_CHECK(ctx, "count_src_kernel");
  if ((rc = egnn_launch_row_scan(ctx, col_ptr, g->n_total, st))) return rc;
  hipLaunchKernelGGL(fill_src_kernel, ge, b, 0, st, g->src, n_e, col_ptr, cursor, bucket);
  EGNN_LAUNCH_CHECK(ctx, "fill_src_kernel");
  hipLaunchKernelGGL(sort_bucket_kernel, dim3((g->n_total + 3) / 4), b, 0, st, col_ptr, bucket, perm, g->n_total);
  EGNN_LAUNCH_CHECK(ctx, "sort_bucket_kernel");
  return EGNN_OK;
}

extern "C" int egnn_loss_mse(egnn_ctx* ctx, const float* H, const float* T, int64_t n_values, float* loss,
                             float* dH, void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!H || !T || !loss || n_values <= 0 || !ws) return egnn_fail(ctx, EGNN_EINVAL, "loss_mse: bad argument");
  const long nb = (n_values + LOSS_PER_BLOCK - 1) / LOSS_PER_BLOCK;
  if (ws_bytes < (size_t)nb * sizeof(double)) return egnn_fail(ctx, EGNN_EWS, "loss_mse: workspace too small");
  hipStream_t st = (hipStream_t)stream;
  double* partial = (double*)ws;
  hipLaunchKernelGGL(loss_mse_partial_kernel, dim3((unsigned)nb), dim3(256), 0, st, H, T, (long)n_values, dH, partial,
                     (float)(2.0 / (double)n_values));
  EGNN_LAUNCH_CHECK(ctx, "loss_mse_partial_kernel");
  hipLaunchKernelGGL(loss_mse_final_kernel, dim3(1), dim3(256), 0, st, partial, (int)nb, 1.0 / (double)n_values, loss);
  EGNN_LAUNCH_CHECK(ctx, "loss_mse_final_kernel");
  return EGNN_OK;
}
