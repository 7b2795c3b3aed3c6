// S1: radius graph (Sec. 3 "Initialization": edges i -> j within r_cut; Sec. 4.4: periodic structures).
//
// One wavefront per destination atom j.  It sweeps the source atoms in index order, 64 at a time; a
// lane evaluates the fp64 minimum-image predicate for its source, a ballot gathers the 64 outcomes
// and the prefix popcount of the ballot gives every accepted source its place.  Sources are visited
// in ascending order, so the row of j comes out sorted by src with no sort pass, and rows are
// stored in ascending j: the edge list is sorted by (dst, src).
//
// Two sweeps: the first one only counts (row lengths -> exclusive scan -> row_ptr), the second writes.
#include "egnn_internal.h"

struct NlistGeom {
  double box[3];
  double rc2;
  int pbc[3];
};

__device__ __forceinline__ bool pair_inside(const double pj[3], const float* __restrict__ pos, int i,
                                            const NlistGeom& g, int sh[3]) {
  double d2 = 0.0;
#pragma unroll
  for (int a = 0; a < 3; ++a) {
    double d = (double)pos[3 * i + a] - pj[a];
    sh[a] = 0;
    if (g.pbc[a]) {
      const double n = rint(d / g.box[a]);
      d -= n * g.box[a];
      sh[a] = -(int)n;
    }
    d2 += d * d;
  }
  return d2 < g.rc2;
}

template <bool FILL>
__global__ __launch_bounds__(256) void nlist_sweep_kernel(const float* __restrict__ pos, int n_owned, int n_total,
                                                          NlistGeom g, int* __restrict__ row_ptr,
                                                          int* __restrict__ src, int* __restrict__ dst,
                                                          int8_t* __restrict__ shift) {
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= n_owned) return;
  const double pj[3] = {(double)pos[3 * j], (double)pos[3 * j + 1], (double)pos[3 * j + 2]};
  const long base = FILL ? row_ptr[j] : 0;
  int count = 0;
  for (int i0 = 0; i0 < n_total; i0 += 64) {
    const int i = i0 + lane;
    int sh[3] = {0, 0, 0};
    const bool inside = (i < n_total) && (i != j) && pair_inside(pj, pos, i, g, sh);
    const unsigned long long mask = __ballot(inside);
    if (FILL && inside) {
      const long at = base + count + __popcll(mask & ((1ull << lane) - 1ull));
      src[at] = i;
      dst[at] = j;
      if (shift) {
        shift[3 * at + 0] = (int8_t)sh[0];
        shift[3 * at + 1] = (int8_t)sh[1];
        shift[3 * at + 2] = (int8_t)sh[2];
      }
    }
    count += __popcll(mask);
  }
  if (!FILL && lane == 0) row_ptr[j + 1] = count;
}

// In-place inclusive scan of row_ptr[1..n] (row lengths) by one workgroup; row_ptr[0] = 0.
// If the total does not fit in int32 the last entry is set to -1.
__global__ __launch_bounds__(1024) void row_scan_kernel(int* __restrict__ row_ptr, int n) {
  __shared__ long part[1024];
  __shared__ long carry;
  const int tid = threadIdx.x;
  if (tid == 0) { carry = 0; row_ptr[0] = 0; }
  __syncthreads();
  for (int base = 0; base < n; base += 1024) {
    const int idx = base + tid;
    long v = idx < n ? (long)row_ptr[idx + 1] : 0;
    part[tid] = v;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      const long add = tid >= off ? part[tid - off] : 0;
      __syncthreads();
      part[tid] += add;
      __syncthreads();
    }
    const long incl = part[tid] + carry;
    if (idx < n) row_ptr[idx + 1] = incl > 2147483647L ? -1 : (int)incl;
    __syncthreads();
    if (tid == 1023) carry = incl;
    __syncthreads();
  }
}

int egnn_launch_row_scan(egnn_ctx* ctx, int* row_ptr, int n, hipStream_t st) {
  hipLaunchKernelGGL(row_scan_kernel, dim3(1), dim3(1024), 0, st, row_ptr, n);
  EGNN_LAUNCH_CHECK(ctx, "row_scan_kernel");
  return EGNN_OK;
}

static int nlist_geom(egnn_ctx* ctx, const float* pos, int32_t n_owned, int32_t n_total, const float box[3],
                      const uint8_t pbc[3], NlistGeom* g) {
  if (!pos || !box || !pbc || n_owned < 0 || n_total < n_owned)
    return egnn_fail(ctx, EGNN_EINVAL, "nlist: null pointer or n_owned/n_total out of range");
  const double rc = (double)ctx->desc.r_cut;
  for (int a = 0; a < 3; ++a) {
    g->box[a] = (double)box[a];
    g->pbc[a] = pbc[a] ? 1 : 0;
    if (pbc[a] && !((double)box[a] >= 2.0 * rc))
      return egnn_fail(ctx, EGNN_EBOX, "nlist: periodic box edge shorter than 2*r_cut");
  }
  g->rc2 = rc * rc;
  return EGNN_OK;
}

extern "C" int egnn_nlist_count(egnn_ctx* ctx, const float* pos, int32_t n_owned, int32_t n_total,
                                const float box[3], const uint8_t pbc[3], int32_t* row_ptr, int64_t* n_edges,
                                void* stream) {
  if (!ctx) return EGNN_EINVAL;
  NlistGeom g;
  int rc = nlist_geom(ctx, pos, n_owned, n_total, box, pbc, &g);
  if (rc) return rc;
  if (!row_ptr || !n_edges) return egnn_fail(ctx, EGNN_EINVAL, "nlist_count: null output pointer");
  hipStream_t st = (hipStream_t)stream;
  if (n_owned > 0) {
    hipLaunchKernelGGL(nlist_sweep_kernel<false>, dim3((n_owned + 3) / 4), dim3(256), 0, st, pos, n_owned, n_total,
                       g, row_ptr, (int*)nullptr, (int*)nullptr, (int8_t*)nullptr);
    EGNN_LAUNCH_CHECK(ctx, "nlist_sweep_kernel<count>");
  }
  hipLaunchKernelGGL(row_scan_kernel, dim3(1), dim3(1024), 0, st, row_ptr, n_owned);
  EGNN_LAUNCH_CHECK(ctx, "row_scan_kernel");
  int32_t total = 0;
  EGNN_HIP(ctx, hipMemcpyAsync(&total, row_ptr + n_owned, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  EGNN_HIP(ctx, hipStreamSynchronize(st));
  if (total < 0) return egnn_fail(ctx, EGNN_EINVAL, "nlist_count: more than 2^31-1 edges");
  *n_edges = total;
  return EGNN_OK;
}

extern "C" int egnn_nlist_fill(egnn_ctx* ctx, const float* pos, int32_t n_owned, int32_t n_total,
                               const float box[3], const uint8_t pbc[3], const int32_t* row_ptr, int64_t n_edges,
                               int32_t* src, int32_t* dst, int8_t* shift, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  NlistGeom g;
  int rc = nlist_geom(ctx, pos, n_owned, n_total, box, pbc, &g);
  if (rc) return rc;
  if (!row_ptr || n_edges < 0 || (n_edges > 0 && (!src || !dst)))
    return egnn_fail(ctx, EGNN_EINVAL, "nlist_fill: null pointer");
  if (n_owned == 0 || n_edges == 0) return EGNN_OK;
  hipLaunchKernelGGL(nlist_sweep_kernel<true>, dim3((n_owned + 3) / 4), dim3(256), 0, (hipStream_t)stream, pos,
                     n_owned, n_total, g, const_cast<int*>(row_ptr), src, dst, shift);
  EGNN_LAUNCH_CHECK(ctx, "nlist_sweep_kernel<fill>");
  return EGNN_OK;
}
