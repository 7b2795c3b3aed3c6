// Shared rows of radial weights: one row per unordered pair of owned atoms.
//
// The radial weights of an edge depend on the edge only through its length (Sec. 3 "Initialization": the edge enters
// through the Gaussian expansion of its distance), and between two owned atoms every edge i -> j has its reverse
// j -> i with the same length.  egnn_edge_pairs gives every edge the index of the row of radial weights it reads:
// an edge is "canonical" and owns a row if its source is a halo atom (its reverse is not in the list: destinations are
// owned atoms only), if src < dst, or if its reverse cannot be found; the other edges (src > dst, both owned) take the
// row of their reverse.  Rows are numbered in ascending order of the canonical edges' ids, so that the rows of one
// destination are contiguous and ascending, like the edges themselves.
//
// The list is sorted by (dst, src) with at most one edge per ordered pair (the periodic box is at least 2 r_cut
// wide), so the reverse of (i -> j) is found by a binary search for src = j in row i; when the list carries image
// shifts the match must have the opposite shift.
#include "egnn_internal.h"

// index of the edge (j -> i) in row i, or -1
__device__ __forceinline__ int find_reverse(const int* __restrict__ row_ptr, const int* __restrict__ src,
                                            const int8_t* __restrict__ shift, int k, int i, int j) {
  int lo = row_ptr[i], hi = row_ptr[i + 1];   // row of destination i, ascending sources
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (src[mid] < j) lo = mid + 1; else hi = mid;
  }
  if (lo >= row_ptr[i + 1] || src[lo] != j) return -1;
  if (shift) {
    const int8_t* a = shift + 3 * (long)k;
    const int8_t* b = shift + 3 * (long)lo;
    if (a[0] != -b[0] || a[1] != -b[1] || a[2] != -b[2]) return -1;
  }
  return lo;
}

__device__ __forceinline__ bool owns_row(const int* __restrict__ row_ptr, const int* __restrict__ src,
                                         const int8_t* __restrict__ shift, int n_owned, int k, int j) {
  const int i = src[k];
  if (i >= n_owned || i < j) return true;
  return find_reverse(row_ptr, src, shift, k, i, j) < 0;
}

// One wavefront per destination.  ASSIGN = false: cnt[j + 1] = number of canonical edges of row j.
// ASSIGN = true: w_row[k] = first[j] + rank of k among the canonical edges of row j, -1 for the others.
template <bool ASSIGN>
__global__ __launch_bounds__(256) void pair_rows_kernel(const int* __restrict__ row_ptr, const int* __restrict__ src,
                                                        const int8_t* __restrict__ shift, int n_owned,
                                                        int* __restrict__ cnt, int* __restrict__ w_row) {
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= n_owned) return;
  const int k0 = row_ptr[j], k1 = row_ptr[j + 1];
  int done = ASSIGN ? cnt[j] : 0;
  for (int kb = k0; kb < k1; kb += 64) {
    const int k = kb + lane;
    const bool own = k < k1 && owns_row(row_ptr, src, shift, n_owned, k, j);
    const unsigned long long mask = __ballot(own);
    if (ASSIGN && k < k1) w_row[k] = own ? done + __popcll(mask & ((1ull << lane) - 1ull)) : -1;
    done += __popcll(mask);
  }
  if (!ASSIGN && lane == 0) cnt[j + 1] = done;
}

// One thread per edge: an edge without a row of its own takes the row of its reverse.
__global__ __launch_bounds__(256) void pair_link_kernel(const int* __restrict__ row_ptr, const int* __restrict__ src,
                                                        const int* __restrict__ dst, const int8_t* __restrict__ shift,
                                                        long n_edges, int* __restrict__ w_row) {
  const long k = (long)blockIdx.x * 256 + threadIdx.x;
  if (k >= n_edges) return;
  const int i = src[k], j = dst[k];
  if (i < j) return;                      // canonical (a halo source has i >= n_owned > j and kept its own row: w_row >= 0)
  if (w_row[k] >= 0) return;
  const int r = find_reverse(row_ptr, src, shift, (int)k, i, j);
  // (r >= 0: otherwise the edge would own a row.  The reverse has src j < dst i: it is canonical, its row is final.)
  w_row[k] = ~w_row[r];                 // negative: the row is read, not owned
}

size_t egnn_edge_pairs_ws_bytes(int32_t n_owned) { return (((size_t)n_owned + 1) * sizeof(int) + 255) & ~(size_t)255; }

extern "C" int egnn_edge_pairs_workspace_bytes(const egnn_ctx* ctx, int32_t n_owned, size_t* bytes) {
  if (!ctx || !bytes || n_owned < 0) return EGNN_EINVAL;
  *bytes = egnn_edge_pairs_ws_bytes(n_owned);
  return EGNN_OK;
}

extern "C" int egnn_edge_pairs(egnn_ctx* ctx, const egnn_graph* g, int32_t* w_row, int64_t* n_rows, void* ws,
                               size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!g || !n_rows || g->n_edges < 0 || g->n_edges > 2147483647LL || g->n_owned < 0 || g->n_total < g->n_owned ||
      !g->row_ptr || (g->n_edges > 0 && (!g->src || !g->dst || !w_row)))
    return egnn_fail(ctx, EGNN_EINVAL, "edge_pairs: null pointer or bad sizes");
  *n_rows = 0;
  if (g->n_edges == 0 || g->n_owned == 0) return EGNN_OK;
  if (!ws || ((uintptr_t)ws & 255) != 0 || ws_bytes < egnn_edge_pairs_ws_bytes(g->n_owned))
    return egnn_fail(ctx, EGNN_EWS, "edge_pairs: workspace missing, misaligned or too small");
  hipStream_t st = (hipStream_t)stream;
  int* cnt = (int*)ws;
  const dim3 gw((g->n_owned + 3) / 4), b(256);
  hipLaunchKernelGGL(pair_rows_kernel<false>, gw, b, 0, st, g->row_ptr, g->src, g->shift, g->n_owned, cnt, (int*)nullptr);
  EGNN_LAUNCH_CHECK(ctx, "pair_rows_kernel<count>");
  int rc = egnn_launch_row_scan(ctx, cnt, g->n_owned, st);   // cnt[j] = first row of destination j, cnt[n_owned] = total
  if (rc) return rc;
  hipLaunchKernelGGL(pair_rows_kernel<true>, gw, b, 0, st, g->row_ptr, g->src, g->shift, g->n_owned, cnt, w_row);
  EGNN_LAUNCH_CHECK(ctx, "pair_rows_kernel<assign>");
  hipLaunchKernelGGL(pair_link_kernel, dim3((unsigned)((g->n_edges + 255) / 256)), b, 0, st, g->row_ptr, g->src, g->dst,
                     g->shift, (long)g->n_edges, w_row);
  EGNN_LAUNCH_CHECK(ctx, "pair_link_kernel");
  int32_t total = 0;
  EGNN_HIP(ctx, hipMemcpyAsync(&total, cnt + g->n_owned, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  EGNN_HIP(ctx, hipStreamSynchronize(st));
  *n_rows = total;
  return EGNN_OK;
}
