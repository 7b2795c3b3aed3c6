// S1: radius graph (Sec. 3 "Initialization": edges i -> j within r_cut; Sec. 4.4: periodic structures).
//
// Output: all ordered pairs (src i, dst j), i != j, j owned, inside the cutoff (fp64 minimum-image predicate on
// the fp32 data, strict '<'), sorted by (dst, src), with the CSR index over destinations.
//
// Two search strategies feed the same compaction:
//   * cell list (when the caller supplies a workspace): atoms are binned into cells of edge >= r_cut; one wavefront
//     per destination atom visits the atoms of the <= 27 neighbouring cells, evaluates the predicate and sets a
//     bit per accepted source in an LDS bitmap.  Scanning the bitmap in word order -- popcount per lane, wave prefix
//     sum -- yields the accepted sources in ascending order whatever order the cells delivered them in, so no sort
//     pass is needed and the order inside a cell (filled with integer atomics) does not matter.
//   * full sweep (no workspace, or more atoms than the bitmap holds): the wavefront sweeps all sources in index
//     order, 64 per step; a ballot collects the outcomes and its prefix popcount places the accepted ones.
// Each runs twice: a counting pass (row lengths -> exclusive scan -> row_ptr) and a filling pass.
#include "egnn_internal.h"

#define NL_MAX_CELLS_AXIS 64
#define NL_MAX_BITMAP_ATOMS 262144   // 8192 words = 32 KB of LDS per wavefront

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

// ------------------------------------------------------------------------------------------------ full sweep
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
  const long row_end = FILL ? row_ptr[j + 1] : 0;   // the fill pass never writes past the row the count pass sized
  int count = 0;
  for (int i0 = 0; i0 < n_total; i0 += 64) {
    const int i = i0 + lane;
    int sh[3] = {0, 0, 0};
    const bool inside = (i < n_total) && (i != j) && pair_inside(pj, pos, i, g, sh);
    const unsigned long long mask = __ballot(inside);
    const long at = base + count + __popcll(mask & ((1ull << lane) - 1ull));
    if (FILL && inside && at < row_end) {
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

// ------------------------------------------------------------------------------------------------ cell list
// bounding box of all atoms: one workgroup, result as 6 floats (min xyz, max xyz)
__global__ __launch_bounds__(1024) void bbox_kernel(const float* __restrict__ pos, int n_total, float* __restrict__ out) {
  __shared__ float smin[3][1024], smax[3][1024];
  const int tid = threadIdx.x;
  float mn[3] = {3.0e38f, 3.0e38f, 3.0e38f}, mx[3] = {-3.0e38f, -3.0e38f, -3.0e38f};
  for (int i = tid; i < n_total; i += 1024)
#pragma unroll
    for (int a = 0; a < 3; ++a) {
      const float v = pos[3 * i + a];
      mn[a] = fminf(mn[a], v);
      mx[a] = fmaxf(mx[a], v);
    }
#pragma unroll
  for (int a = 0; a < 3; ++a) {
    smin[a][tid] = mn[a];
    smax[a][tid] = mx[a];
  }
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (tid < off)
#pragma unroll
      for (int a = 0; a < 3; ++a) {
        smin[a][tid] = fminf(smin[a][tid], smin[a][tid + off]);
        smax[a][tid] = fmaxf(smax[a][tid], smax[a][tid + off]);
      }
    __syncthreads();
  }
  if (tid < 3) {
    out[tid] = smin[tid][0];
    out[3 + tid] = smax[tid][0];
  }
}

__device__ __forceinline__ int cell_coord(double x, int a, const CellGrid& cg) {
  double u = x - cg.lo[a];
  if (cg.pbc[a]) u -= floor(u / cg.box[a]) * cg.box[a];
  int ci = (int)floor(u * cg.inv_cell[a]);
  return ci < 0 ? 0 : (ci >= cg.n[a] ? cg.n[a] - 1 : ci);
}

__global__ void cell_count_kernel(const float* __restrict__ pos, int n_total, CellGrid cg, int* __restrict__ cell_of,
                                  int* __restrict__ cell_ptr) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_total) return;
  const int cx = cell_coord((double)pos[3 * i], 0, cg), cy = cell_coord((double)pos[3 * i + 1], 1, cg),
            cz = cell_coord((double)pos[3 * i + 2], 2, cg);
  const int cell = (cx * cg.n[1] + cy) * cg.n[2] + cz;
  cell_of[i] = cell;
  atomicAdd(&cell_ptr[cell + 1], 1);   // integer count: independent of order
}

__global__ void cell_fill_kernel(int n_total, const int* __restrict__ cell_of, const int* __restrict__ cell_ptr,
                                 int* __restrict__ cursor, int* __restrict__ cell_atoms) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_total) return;
  const int cell = cell_of[i];
  cell_atoms[cell_ptr[cell] + atomicAdd(&cursor[cell], 1)] = i;   // order inside a cell is irrelevant (bitmap)
}

// neighbour cell coordinates along one axis (without duplicates): returns the count, fills out[3]
__device__ __forceinline__ int axis_neighbours(int c, int a, const CellGrid& cg, int out[3]) {
  const int n = cg.n[a];
  if (n == 1) { out[0] = 0; return 1; }
  if (n == 2) { out[0] = 0; out[1] = 1; return 2; }
  int k = 0;
  for (int d = -1; d <= 1; ++d) {
    int v = c + d;
    if (cg.pbc[a]) v = (v + n) % n;
    else if (v < 0 || v >= n) continue;
    out[k++] = v;
  }
  return k;
}

template <bool FILL>
__global__ __launch_bounds__(256) void nlist_cells_kernel(const float* __restrict__ pos, int n_owned, int n_total,
                                                          NlistGeom g, CellGrid cg, const int* __restrict__ cell_of,
                                                          const int* __restrict__ cell_ptr,
                                                          const int* __restrict__ cell_atoms, int* __restrict__ row_ptr,
                                                          int* __restrict__ src, int* __restrict__ dst,
                                                          int8_t* __restrict__ shift, int words, int waves_per_wg) {
  extern __shared__ unsigned int bitmap_all[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * waves_per_wg + wave;
  if (wave >= waves_per_wg || j >= n_owned) return;
  unsigned int* bitmap = bitmap_all + (size_t)wave * words;
  for (int wi = lane; wi < words; wi += 64) bitmap[wi] = 0u;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_wave_barrier();

  const double pj[3] = {(double)pos[3 * j], (double)pos[3 * j + 1], (double)pos[3 * j + 2]};
  // indices read back from the workspace are clamped: a workspace overwritten between the count and the fill call
  // then gives a wrong list, never an access outside the buffers
  const int cj = min(max(cell_of[j], 0), cg.n_cells - 1);
  const int cz = cj % cg.n[2], cy = (cj / cg.n[2]) % cg.n[1], cx = cj / (cg.n[2] * cg.n[1]);
  int nx[3], ny[3], nz[3];
  const int kx = axis_neighbours(cx, 0, cg, nx), ky = axis_neighbours(cy, 1, cg, ny), kz = axis_neighbours(cz, 2, cg, nz);
  for (int ix = 0; ix < kx; ++ix)
    for (int iy = 0; iy < ky; ++iy)
      for (int iz = 0; iz < kz; ++iz) {
        const int cell = (nx[ix] * cg.n[1] + ny[iy]) * cg.n[2] + nz[iz];
        const int a0 = max(cell_ptr[cell], 0), a1 = min(cell_ptr[cell + 1], n_total);
        for (int a = a0 + lane; a < a1; a += 64) {
          const int i = cell_atoms[a];
          int sh[3];
          if ((unsigned)i < (unsigned)n_total && i != j && pair_inside(pj, pos, i, g, sh))
            atomicOr(&bitmap[i >> 5], 1u << (i & 31));
        }
      }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");

  // bitmap -> sorted sources
  const long base = FILL ? row_ptr[j] : 0;
  const long row_end = FILL ? row_ptr[j + 1] : 0;   // the fill pass never writes past the row the count pass sized
  int count = 0;
  for (int w0 = 0; w0 < words; w0 += 64) {
    const int wi = w0 + lane;
    unsigned int bits = wi < words ? bitmap[wi] : 0u;
    const int mine = __popc(bits);
    int incl = mine;   // inclusive prefix sum over the wave
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    if (FILL) {
      long at = base + count + incl - mine;
      while (bits) {
        const int b = __ffs(bits) - 1;
        bits &= bits - 1;
        const int i = wi * 32 + b;
        int sh[3];
        pair_inside(pj, pos, i, g, sh);
        if (at < row_end) {
          src[at] = i;
          dst[at] = j;
          if (shift) {
            shift[3 * at + 0] = (int8_t)sh[0];
            shift[3 * at + 1] = (int8_t)sh[1];
            shift[3 * at + 2] = (int8_t)sh[2];
          }
        }
        ++at;
      }
    }
    count += __shfl(incl, 63);
  }
  if (!FILL && lane == 0) row_ptr[j + 1] = count;
}

// ------------------------------------------------------------------------------------------------ row scan
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

// ------------------------------------------------------------------------------------------------ host side
static size_t a256(size_t n) { return (n + 255) & ~(size_t)255; }
static const int kMaxCells = NL_MAX_CELLS_AXIS * NL_MAX_CELLS_AXIS * NL_MAX_CELLS_AXIS;

struct CellWs {
  float* bbox;       // [6]
  int* cell_of;      // [n_total]
  int* cell_ptr;     // [max cells + 1]
  int* cursor;       // [max cells]
  int* cell_atoms;   // [n_total]
};

static size_t carve_cells(char* base, int n_total, CellWs* w) {
  size_t used = 0;
  auto take = [&](size_t bytes) { char* p = base ? base + used : nullptr; used += a256(bytes); return p; };
  w->bbox = (float*)take(6 * sizeof(float));
  w->cell_of = (int*)take((size_t)n_total * sizeof(int));
  w->cell_ptr = (int*)take(((size_t)kMaxCells + 1) * sizeof(int));
  w->cursor = (int*)take((size_t)kMaxCells * sizeof(int));
  w->cell_atoms = (int*)take((size_t)n_total * sizeof(int));
  return used;
}

extern "C" int egnn_nlist_workspace_bytes(const egnn_ctx* ctx, int32_t n_total, size_t* bytes) {
  if (!ctx || !bytes || n_total < 0) return EGNN_EINVAL;
  CellWs w;
  *bytes = carve_cells(nullptr, n_total, &w);
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

static bool use_cells(const void* ws, size_t ws_bytes, int n_total) {
  CellWs w;
  return ws && n_total > 0 && n_total <= NL_MAX_BITMAP_ATOMS && ws_bytes >= carve_cells(nullptr, n_total, &w);
}

template <bool FILL>
static int launch_cells(egnn_ctx* ctx, const float* pos, int n_owned, int n_total, const NlistGeom& g, const CellGrid& cg,
                        const CellWs& w, int* row_ptr, int* src, int* dst, int8_t* shift, hipStream_t st) {
  const int words = (n_total + 31) / 32;
  const int waves = words <= 2048 ? 4 : 1;
  const size_t shmem = (size_t)waves * words * sizeof(unsigned int);
  hipLaunchKernelGGL(nlist_cells_kernel<FILL>, dim3((n_owned + waves - 1) / waves), dim3(256), shmem, st, pos, n_owned,
                     n_total, g, cg, w.cell_of, w.cell_ptr, w.cell_atoms, row_ptr, src, dst, shift, words, waves);
  EGNN_LAUNCH_CHECK(ctx, "nlist_cells_kernel");
  return EGNN_OK;
}

extern "C" int egnn_nlist_count(egnn_ctx* ctx, const float* pos, int32_t n_owned, int32_t n_total,
                                const float box[3], const uint8_t pbc[3], int32_t* row_ptr, int64_t* n_edges,
                                void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  NlistGeom g;
  int rc = nlist_geom(ctx, pos, n_owned, n_total, box, pbc, &g);
  if (rc) return rc;
  if (!row_ptr || !n_edges) return egnn_fail(ctx, EGNN_EINVAL, "nlist_count: null output pointer");
  if (ws && ((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "nlist_count: workspace not 256-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  if (n_owned > 0 && use_cells(ws, ws_bytes, n_total)) {
    CellWs w;
    carve_cells((char*)ws, n_total, &w);
    // grid: periodic axes span the box, open axes the bounding box of the atoms; cell edge >= r_cut (1 + 1e-6)
    float bb[6];
    hipLaunchKernelGGL(bbox_kernel, dim3(1), dim3(1024), 0, st, pos, n_total, w.bbox);
    EGNN_LAUNCH_CHECK(ctx, "bbox_kernel");
    EGNN_HIP(ctx, hipMemcpyAsync(bb, w.bbox, sizeof(bb), hipMemcpyDeviceToHost, st));
    EGNN_HIP(ctx, hipStreamSynchronize(st));
    CellGrid cg;
    const double rc_pad = (double)ctx->desc.r_cut * (1.0 + 1e-6);
    cg.n_cells = 1;
    for (int a = 0; a < 3; ++a) {
      cg.pbc[a] = g.pbc[a];
      cg.box[a] = g.box[a];
      const double lo = g.pbc[a] ? 0.0 : (double)bb[a];
      double extent = g.pbc[a] ? g.box[a] : (double)bb[3 + a] - (double)bb[a];
      if (!(extent > 0.0)) extent = rc_pad;
      int n = (int)floor(extent / rc_pad);
      n = n < 1 ? 1 : (n > NL_MAX_CELLS_AXIS ? NL_MAX_CELLS_AXIS : n);
      cg.lo[a] = lo;
      cg.n[a] = n;
      cg.inv_cell[a] = (double)n / extent;
      cg.n_cells *= n;
    }
    ctx->nl_grid = cg;          // egnn_nlist_fill walks the same cells
    ctx->nl_grid_atoms = n_total;
    ctx->nl_grid_ws = ws;
    ctx->nl_grid_pos = pos;
    if ((rc = egnn_launch_fill_int(ctx, w.cell_ptr, (long)cg.n_cells + 1, 0, st))) return rc;
    if ((rc = egnn_launch_fill_int(ctx, w.cursor, cg.n_cells, 0, st))) return rc;
    const dim3 ga((n_total + 255) / 256), b(256);
    hipLaunchKernelGGL(cell_count_kernel, ga, b, 0, st, pos, n_total, cg, w.cell_of, w.cell_ptr);
    EGNN_LAUNCH_CHECK(ctx, "cell_count_kernel");
    if ((rc = egnn_launch_row_scan(ctx, w.cell_ptr, cg.n_cells, st))) return rc;
    hipLaunchKernelGGL(cell_fill_kernel, ga, b, 0, st, n_total, w.cell_of, w.cell_ptr, w.cursor, w.cell_atoms);
    EGNN_LAUNCH_CHECK(ctx, "cell_fill_kernel");
    if ((rc = launch_cells<false>(ctx, pos, n_owned, n_total, g, cg, w, row_ptr, nullptr, nullptr, nullptr, st))) return rc;
  } else if (n_owned > 0) {
    hipLaunchKernelGGL(nlist_sweep_kernel<false>, dim3((n_owned + 3) / 4), dim3(256), 0, st, pos, n_owned, n_total,
                       g, row_ptr, (int*)nullptr, (int*)nullptr, (int8_t*)nullptr);
    EGNN_LAUNCH_CHECK(ctx, "nlist_sweep_kernel<count>");
  }
  if ((rc = egnn_launch_row_scan(ctx, row_ptr, n_owned, st))) return rc;
  int32_t total = 0;
  EGNN_HIP(ctx, hipMemcpyAsync(&total, row_ptr + n_owned, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  EGNN_HIP(ctx, hipStreamSynchronize(st));
  if (total < 0) return egnn_fail(ctx, EGNN_EINVAL, "nlist_count: more than 2^31-1 edges");
  *n_edges = total;
  return EGNN_OK;
}

extern "C" int egnn_nlist_fill(egnn_ctx* ctx, const float* pos, int32_t n_owned, int32_t n_total,
                               const float box[3], const uint8_t pbc[3], const int32_t* row_ptr, int64_t n_edges,
                               int32_t* src, int32_t* dst, int8_t* shift, void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  NlistGeom g;
  int rc = nlist_geom(ctx, pos, n_owned, n_total, box, pbc, &g);
  if (rc) return rc;
  if (!row_ptr || n_edges < 0 || (n_edges > 0 && (!src || !dst)))
    return egnn_fail(ctx, EGNN_EINVAL, "nlist_fill: null pointer");
  if (ws && ((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "nlist_fill: workspace not 256-byte aligned");
  if (n_owned == 0 || n_edges == 0) return EGNN_OK;
  hipStream_t st = (hipStream_t)stream;
  if (use_cells(ws, ws_bytes, n_total)) {
    // the cell lists built by egnn_nlist_count are still in the workspace; their grid is kept in the context
    CellWs w;
    carve_cells((char*)ws, n_total, &w);
    if (ctx->nl_grid_atoms != n_total || ctx->nl_grid_ws != ws || ctx->nl_grid_pos != pos)
      return egnn_fail(ctx, EGNN_EINVAL, "nlist_fill: call egnn_nlist_count with the same atoms and workspace first");
    const CellGrid cg = ctx->nl_grid;
    return launch_cells<true>(ctx, pos, n_owned, n_total, g, cg, w, const_cast<int*>(row_ptr), src, dst, shift, st);
  }
  hipLaunchKernelGGL(nlist_sweep_kernel<true>, dim3((n_owned + 3) / 4), dim3(256), 0, st, pos, n_owned, n_total, g,
                     const_cast<int*>(row_ptr), src, dst, shift);
  EGNN_LAUNCH_CHECK(ctx, "nlist_sweep_kernel<fill>");
  return EGNN_OK;
}
