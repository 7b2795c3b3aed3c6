// Assembly of the predicted Hamiltonian (Sec. 3, end of "Message passing"; Fig. 2(e); Sec. 2.2; Sec. 6):
//   * on-site blocks H_ii from the node features (collapse E -> 1 per coupled slot, inverse coupling of Eq. 1);
//   * species-dependent orbital sets: every block is predicted in the global shell list, an orbital that a species
//     does not own is padding (zero, no loss, no gradient, no place in the assembled matrix);
//   * combined L1 + L2 loss over the entries that are not padding;
//   * the column-compressed matrix: columns = orbitals of the owned atoms, rows = orbitals of all atoms, block (i, j)
//     from the edge i -> j, block (j, j) from node j.
// Everything here is memory-bound bookkeeping around the blocks; sums are taken in a fixed order (no float atomics).
#include "egnn_internal.h"

#define HAM_TILE_FLOATS 10240   // floats of block data staged per tile (40 KB)
#define HAM_MAX_TILE 64         // blocks per tile at most

__device__ __forceinline__ uint32_t ham_bits(const int* __restrict__ species, const uint32_t* __restrict__ orb_bits,
                                             int n_species, int atom, uint32_t all) {
  int s = species[atom];
  s = s < 0 ? 0 : (s >= n_species ? n_species - 1 : s);
  return orb_bits[s] & all;
}

// ------------------------------------------------------------------------------------------------ on-site blocks
// One workgroup per node: the node row goes to LDS, a thread collapses one coupled component (a dot product over the
// channels with its row of V), then a thread uncouples one entry of the block.
__global__ __launch_bounds__(256) void onsite_kernel(const float* __restrict__ x, const float* __restrict__ V,
                                                     const int* __restrict__ q_row, const int* __restrict__ q_vrow,
                                                     const int* __restrict__ unc_ptr, const int* __restrict__ unc_q,
                                                     const float* __restrict__ unc_c, float* __restrict__ H,
                                                     int D, int log2E, int nq) {
  extern __shared__ float sm[];
  float* sx = sm;                      // [D][E]
  float* sq = sm + (D << log2E);       // [nq]
  const int i = blockIdx.x, tid = threadIdx.x, E = 1 << log2E;
  const float* xi = x + ((size_t)i * D << log2E);
  for (int t = tid; t < (D << log2E); t += 256) sx[t] = xi[t];
  __syncthreads();
  for (int t = tid; t < nq; t += 256) {
    const int r = q_row[t];
    float s = 0.0f;
    if (r < D) {                       // coupled degrees above l_max have no feature to read
      const float* v = V + ((size_t)q_vrow[t] << log2E);
      const float* xr = sx + (r << log2E);
      for (int c = 0; c < E; ++c) s += v[c] * xr[c];
    }
    sq[t] = s;
  }
  __syncthreads();
  for (int e = tid; e < nq; e += 256) {
    float sum = 0.0f;
    for (int n = unc_ptr[e]; n < unc_ptr[e + 1]; ++n) sum += unc_c[n] * sq[unc_q[n]];
    H[(size_t)i * nq + e] = sum;
  }
}

// ---- adjoint of the on-site blocks: dq = C^T dH per node, dx[i][(L,M)][c] = sum_o V[o][c] dq[o][M],
//      dV[o][c] = sum_i sum_M dq_i[o][M] x[i][(L,M)][c] (nodes added in a fixed order)
__global__ __launch_bounds__(256) void onsite_bwd_node_kernel(const float* __restrict__ V,
                                                              const float* __restrict__ dH,
                                                              const int* __restrict__ uncT_ptr,
                                                              const int* __restrict__ uncT_h,
                                                              const float* __restrict__ uncT_c,
                                                              const int* __restrict__ rowT_ptr,
                                                              const int* __restrict__ rowT_t,
                                                              const int* __restrict__ q_vrow, float* __restrict__ dx,
                                                              float* __restrict__ dq_all, int D, int log2E, int nq) {
  extern __shared__ float sm[];
  float* sdH = sm;         // [nq]
  float* sq = sm + nq;     // [nq]
  const int i = blockIdx.x, tid = threadIdx.x, E = 1 << log2E;
  for (int e = tid; e < nq; e += 256) sdH[e] = dH[(size_t)i * nq + e];
  __syncthreads();
  for (int t = tid; t < nq; t += 256) {
    float s = 0.0f;
    for (int n = uncT_ptr[t]; n < uncT_ptr[t + 1]; ++n) s += uncT_c[n] * sdH[uncT_h[n]];
    sq[t] = s;
    dq_all[(size_t)i * nq + t] = s;
  }
  __syncthreads();
  float* dxi = dx + ((size_t)i * D << log2E);
  for (int idx = tid; idx < (D << log2E); idx += 256) {
    const int r = idx >> log2E, c = idx & (E - 1);
    float s = 0.0f;
    for (int n = rowT_ptr[r]; n < rowT_ptr[r + 1]; ++n) {
      const int t = rowT_t[n];
      s += V[((size_t)q_vrow[t] << log2E) + c] * sq[t];
    }
    dxi[idx] = s;
  }
}

// One workgroup per row o of V: lane = (channel, part); a part walks the nodes i = part, part + n_parts, ...
__global__ __launch_bounds__(256) void onsite_bwd_dV_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ dq_all,
                                                            const int* __restrict__ vrow_L,
                                                            const int* __restrict__ vrow_qoff, float* __restrict__ dV,
                                                            int n_nodes, int D, int log2E, int nq, int lmax) {
  __shared__ float red[256];
  const int o = blockIdx.x, tid = threadIdx.x, E = 1 << log2E;
  const int c = tid & (E - 1), part = tid >> log2E, n_parts = 256 >> log2E;
  const int L = vrow_L[o], qoff = vrow_qoff[o];
  float acc = 0.0f;
  if (L <= lmax) {
    for (int i = part; i < n_nodes; i += n_parts) {
      const float* xi = x + (((size_t)i * D + L * L) << log2E) + c;
      const float* dq = dq_all + (size_t)i * nq + qoff;
      for (int M = 0; M < 2 * L + 1; ++M) acc += dq[M] * xi[(size_t)M << log2E];
    }
  }
  red[tid] = acc;
  __syncthreads();
  if (part == 0) {
    float s = 0.0f;
    for (int p = 0; p < n_parts; ++p) s += red[(p << log2E) + c];
    dV[((size_t)o << log2E) + c] = s;
  }
}

// ------------------------------------------------------------------------------------------------ padding
// A workgroup takes `bpw` whole blocks (about 4096 values): the orbital masks of its blocks go to LDS once, then
// the values are walked in memory order.  Index arithmetic by multiplication with a float reciprocal: exact here,
// the quotients are at least 0.5 / n_orb^2 away from an integer and the indices stay below 2^13.
#define HAM_MAX_BPW 1024
__host__ __device__ inline int ham_bpw(int nq) {
  const int b = 4096 / nq;
  return b < 1 ? 1 : (b > HAM_MAX_BPW ? HAM_MAX_BPW : b);
}

__device__ __forceinline__ void ham_stage_masks(long blk0, int nb, const int* __restrict__ row_atom,
                                                const int* __restrict__ col_atom, const int* __restrict__ species,
                                                const uint32_t* __restrict__ orb_bits, int n_species, uint32_t all,
                                                uint32_t* s_rb, uint32_t* s_cb) {
  for (int t = threadIdx.x; t < nb; t += 256) {
    const long blk = blk0 + t;
    s_rb[t] = ham_bits(species, orb_bits, n_species, row_atom ? row_atom[blk] : (int)blk, all);
    s_cb[t] = ham_bits(species, orb_bits, n_species, col_atom ? col_atom[blk] : (int)blk, all);
  }
  __syncthreads();
}

__global__ __launch_bounds__(256) void padding_kernel(float* __restrict__ H, long n_blocks, int n_orb, int bpw,
                                                      const int* __restrict__ row_atom,
                                                      const int* __restrict__ col_atom,
                                                      const int* __restrict__ species,
                                                      const uint32_t* __restrict__ orb_bits, int n_species) {
  __shared__ uint32_t s_rb[HAM_MAX_BPW], s_cb[HAM_MAX_BPW];
  const int nq = n_orb * n_orb;
  const uint32_t all = n_orb >= 32 ? 0xffffffffu : ((1u << n_orb) - 1u);
  const long blk0 = (long)blockIdx.x * bpw;
  const int nb = (int)min((long)bpw, n_blocks - blk0);
  ham_stage_masks(blk0, nb, row_atom, col_atom, species, orb_bits, n_species, all, s_rb, s_cb);
  const float inv_nq = 1.0f / (float)nq, inv_no = 1.0f / (float)n_orb;
  float* Hb = H + blk0 * nq;
  const int n_local = nb * nq;
  for (int idx = threadIdx.x; idx < n_local; idx += 256) {
    const int bl = (int)(((float)idx + 0.5f) * inv_nq);
    const int r = idx - bl * nq;
    const int a = (int)(((float)r + 0.5f) * inv_no), b = r - a * n_orb;
    if (!(((s_rb[bl] >> a) & 1u) && ((s_cb[bl] >> b) & 1u))) Hb[idx] = 0.0f;   // the entry itself is never read
  }
}

// ------------------------------------------------------------------------------------------------ L1 + L2 loss
#define HL_PER_WG 4096
__device__ __forceinline__ double wg_sum(double v, double* red) {
  red[threadIdx.x] = v;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  const double r = red[0];
  __syncthreads();
  return r;
}

// number of entries that are not padding: per block popcount(rows) * popcount(columns)
__global__ __launch_bounds__(256) void present_partial_kernel(long n_blocks, int n_orb,
                                                              const int* __restrict__ row_atom,
                                                              const int* __restrict__ col_atom,
                                                              const int* __restrict__ species,
                                                              const uint32_t* __restrict__ orb_bits, int n_species,
                                                              double* __restrict__ partial) {
  __shared__ double red[256];
  const uint32_t all = n_orb >= 32 ? 0xffffffffu : ((1u << n_orb) - 1u);
  double acc = 0.0;
  for (int q = 0; q < HL_PER_WG / 256; ++q) {
    const long blk = (long)blockIdx.x * HL_PER_WG + q * 256 + threadIdx.x;
    if (blk < n_blocks) {
      const uint32_t rb = ham_bits(species, orb_bits, n_species, row_atom ? row_atom[blk] : (int)blk, all);
      const uint32_t cb = ham_bits(species, orb_bits, n_species, col_atom ? col_atom[blk] : (int)blk, all);
      acc += (double)(__popc(rb) * __popc(cb));
    }
  }
  const double s = wg_sum(acc, red);
  if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// out[0] = sum of the partials (exact: integers below 2^53)
__global__ __launch_bounds__(256) void sum_partials_kernel(const double* __restrict__ partial, int n_partials,
                                                           double* __restrict__ out) {
  __shared__ double red[256];
  double acc = 0.0;
  for (int b = threadIdx.x; b < n_partials; b += 256) acc += partial[b];
  const double s = wg_sum(acc, red);
  if (threadIdx.x == 0) out[0] = s;
}

__global__ __launch_bounds__(256) void l1l2_partial_kernel(const float* __restrict__ H, const float* __restrict__ T,
                                                           long n_blocks, int n_orb, int bpw,
                                                           const int* __restrict__ row_atom,
                                                           const int* __restrict__ col_atom,
                                                           const int* __restrict__ species,
                                                           const uint32_t* __restrict__ orb_bits, int n_species,
                                                           const double* __restrict__ n_present,
                                                           float* __restrict__ dH, double* __restrict__ partial1,
                                                           double* __restrict__ partial2) {
  __shared__ double red[256];
  __shared__ uint32_t s_rb[HAM_MAX_BPW], s_cb[HAM_MAX_BPW];
  const int nq = n_orb * n_orb;
  const uint32_t all = n_orb >= 32 ? 0xffffffffu : ((1u << n_orb) - 1u);
  const long blk0 = (long)blockIdx.x * bpw;
  const int nb = (int)min((long)bpw, n_blocks - blk0);
  ham_stage_masks(blk0, nb, row_atom, col_atom, species, orb_bits, n_species, all, s_rb, s_cb);
  const double cnt = n_present[0];
  const float inv_n = cnt > 0.0 ? (float)(1.0 / cnt) : 0.0f;
  const float inv_nq = 1.0f / (float)nq, inv_no = 1.0f / (float)n_orb;
  const float* Hb = H + blk0 * nq;
  const float* Tb = T + blk0 * nq;
  float* gb = dH ? dH + blk0 * nq : nullptr;
  const int n_local = nb * nq;
  double a1 = 0.0, a2 = 0.0;
#pragma unroll 4
  for (int idx = threadIdx.x; idx < n_local; idx += 256) {
    const float d = Hb[idx] - Tb[idx];
    const int bl = (int)(((float)idx + 0.5f) * inv_nq);
    const int r = idx - bl * nq;
    const int a = (int)(((float)r + 0.5f) * inv_no), b = r - a * n_orb;
    float g = 0.0f;
    if (((s_rb[bl] >> a) & 1u) && ((s_cb[bl] >> b) & 1u)) {
      a1 += (double)fabsf(d);
      a2 += (double)d * (double)d;
      g = ((d > 0.0f ? 1.0f : (d < 0.0f ? -1.0f : 0.0f)) + 2.0f * d) * inv_n;
    }
    if (gb) gb[idx] = g;
  }
  const double s1 = wg_sum(a1, red);
  const double s2 = wg_sum(a2, red);
  if (threadIdx.x == 0) {
    partial1[blockIdx.x] = s1;
    partial2[blockIdx.x] = s2;
  }
}

__global__ __launch_bounds__(256) void l1l2_final_kernel(const double* __restrict__ partial1,
                                                         const double* __restrict__ partial2, int n_partials,
                                                         const double* __restrict__ n_present,
                                                         float* __restrict__ loss) {
  __shared__ double red[256];
  double a1 = 0.0, a2 = 0.0;
  for (int b = threadIdx.x; b < n_partials; b += 256) {
    a1 += partial1[b];
    a2 += partial2[b];
  }
  const double s1 = wg_sum(a1, red);
  const double s2 = wg_sum(a2, red);
  if (threadIdx.x == 0) {
    const double cnt = n_present[0];
    const double inv = cnt > 0.0 ? 1.0 / cnt : 0.0;
    loss[0] = (float)((s1 + s2) * inv);
    loss[1] = (float)(s1 * inv);
    loss[2] = (float)(s2 * inv);
  }
}

// ------------------------------------------------------------------------------------------------ structure
__global__ __launch_bounds__(256) void orb_count_kernel(const int* __restrict__ species,
                                                        const uint32_t* __restrict__ orb_bits, int n_species,
                                                        int n_total, int n_orb, int* __restrict__ orb_off) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n_total) return;
  const uint32_t all = n_orb >= 32 ? 0xffffffffu : ((1u << n_orb) - 1u);
  orb_off[i + 1] = __popc(ham_bits(species, orb_bits, n_species, i, all));
}

// Per owned atom j: the blocks of its columns are its incoming edges (sources ascending) with its own on-site block
// inserted where j falls among the sources.  Row offset of every block inside a column, the column length, and the
// number of stored entries of the atom's columns.
__global__ __launch_bounds__(256) void column_layout_kernel(const int* __restrict__ row_ptr,
                                                            const int* __restrict__ src,
                                                            const int* __restrict__ species,
                                                            const uint32_t* __restrict__ orb_bits, int n_species,
                                                            uint32_t all, const int* __restrict__ orb_off,
                                                            int n_owned, int* __restrict__ edge_pos,
                                                            uint32_t* __restrict__ edge_bits,
                                                            int* __restrict__ edge_off, int* __restrict__ self_pos,
                                                            int* __restrict__ self_idx, int* __restrict__ col_len,
                                                            long* __restrict__ col_start) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n_owned) return;
  const int k0 = row_ptr[j], k1 = row_ptr[j + 1];
  const int n_j = orb_off[j + 1] - orb_off[j];
  int run = 0, sidx = -1;
  for (int k = k0; k < k1; ++k) {
    const int i = src[k];
    if (sidx < 0 && i > j) {
      sidx = k - k0;
      self_pos[j] = run;
      run += n_j;
    }
    edge_pos[k] = run;
    edge_bits[k] = ham_bits(species, orb_bits, n_species, i, all);
    edge_off[k] = orb_off[i];
    run += orb_off[i + 1] - orb_off[i];
  }
  if (sidx < 0) {
    sidx = k1 - k0;
    self_pos[j] = run;
    run += n_j;
  }
  self_idx[j] = sidx;
  col_len[j] = run;
  col_start[j + 1] = (long)n_j * (long)run;
}

// In-place inclusive scan of v[1..n] by one workgroup; v[0] = 0.
__global__ __launch_bounds__(1024) void scan_i64_kernel(long* __restrict__ v, int n) {
  __shared__ long part[1024];
  __shared__ long carry;
  const int tid = threadIdx.x;
  if (tid == 0) { carry = 0; v[0] = 0; }
  __syncthreads();
  for (int base = 0; base < n; base += 1024) {
    const int idx = base + tid;
    part[tid] = idx < n ? v[idx + 1] : 0;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      const long add = tid >= off ? part[tid - off] : 0;
      __syncthreads();
      part[tid] += add;
      __syncthreads();
    }
    const long incl = part[tid] + carry;
    if (idx < n) v[idx + 1] = incl;
    __syncthreads();
    if (tid == 1023) carry = incl;
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void col_ptr_kernel(const int* __restrict__ orb_off,
                                                      const long* __restrict__ col_start,
                                                      const int* __restrict__ col_len, int n_owned,
                                                      long* __restrict__ col_ptr) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j > n_owned) return;
  if (j == n_owned) {
    col_ptr[orb_off[n_owned]] = col_start[n_owned];
    return;
  }
  const int n_j = orb_off[j + 1] - orb_off[j];
  for (int b = 0; b < n_j; ++b) col_ptr[orb_off[j] + b] = col_start[j] + (long)b * col_len[j];
}

// ------------------------------------------------------------------------------------------------ values
// One workgroup per owned atom.  A tile of consecutive blocks of its columns is staged in LDS: the edge blocks of a
// tile are one contiguous stretch of H_edge (edges are sorted by destination) and are copied flat, eight loads in
// flight per thread; the on-site block, if it falls into the tile, goes to a slot of its own.  Then, column by
// column, consecutive threads write consecutive rows of the column.
#define HAM_COPY_UNROLL 8
__global__ __launch_bounds__(256) void csc_fill_kernel(const int* __restrict__ row_ptr, const int* __restrict__ species,
                                                       const uint32_t* __restrict__ orb_bits, int n_species,
                                                       const int* __restrict__ orb_off,
                                                       const int* __restrict__ edge_pos,
                                                       const uint32_t* __restrict__ edge_bits,
                                                       const int* __restrict__ edge_off,
                                                       const int* __restrict__ self_pos,
                                                       const int* __restrict__ self_idx,
                                                       const int* __restrict__ col_len,
                                                       const long* __restrict__ col_start,
                                                       const float* __restrict__ H_edge,
                                                       const float* __restrict__ H_node, int n_orb, int tile_blocks,
                                                       int* __restrict__ row_idx, float* __restrict__ values) {
  extern __shared__ float ham_lds[];
  const int nq = n_orb * n_orb;
  float* tile = ham_lds;                                               // [tile_blocks + 1][nq], last slot: on-site block
  int* s_pos = reinterpret_cast<int*>(tile + (tile_blocks + 1) * nq);  // [tile_blocks + 1] first row of each block
  int* s_off = s_pos + tile_blocks + 1;                                // [tile_blocks] first global row of the source
  int* s_base = s_off + tile_blocks;                                   // [tile_blocks] where the block sits in `tile`
  unsigned char* s_map = reinterpret_cast<unsigned char*>(s_base + tile_blocks);   // [tile_blocks][32] a' -> a
  __shared__ unsigned char s_colmap[32];
  const int j = blockIdx.x, tid = threadIdx.x;
  const uint32_t all = n_orb >= 32 ? 0xffffffffu : ((1u << n_orb) - 1u);
  const int k0 = row_ptr[j], k1 = row_ptr[j + 1];
  const int n_blk = k1 - k0 + 1, sidx = self_idx[j];
  const int len = col_len[j];
  const long cstart = col_start[j];
  const uint32_t bits_j = ham_bits(species, orb_bits, n_species, j, all);
  const int n_j = __popc(bits_j);
  if (tid == 0) {
    int c = 0;
    for (int o = 0; o < n_orb; ++o)
      if ((bits_j >> o) & 1u) s_colmap[c++] = (unsigned char)o;
  }
  for (int t0 = 0; t0 < n_blk; t0 += tile_blocks) {
    const int nt = min(tile_blocks, n_blk - t0);
    const bool self_here = sidx >= t0 && sidx < t0 + nt;
    const int eA = t0 - (t0 > sidx ? 1 : 0);          // first edge of the tile (offset from k0)
    const int ne = nt - (self_here ? 1 : 0);          // edges in the tile
    __syncthreads();                                  // the previous tile has been written out (and s_colmap is set)
    if (tid < nt) {
      const int tt = t0 + tid;
      int pos, off, base;
      uint32_t bits;
      if (tt == sidx) {
        pos = self_pos[j]; off = orb_off[j]; bits = bits_j; base = tile_blocks * nq;
      } else {
        const int e = tt - (tt > sidx ? 1 : 0);
        const int k = k0 + e;
        pos = edge_pos[k]; off = edge_off[k]; bits = edge_bits[k]; base = (e - eA) * nq;
      }
      s_pos[tid] = pos;
      s_off[tid] = off;
      s_base[tid] = base;
      int c = 0;
      for (int o = 0; o < n_orb; ++o)
        if ((bits >> o) & 1u) s_map[tid * 32 + c++] = (unsigned char)o;
      if (tid == nt - 1) s_pos[nt] = pos + c;
    }
    {
      const int n = ne * nq;
      const float* gsrc = H_edge + (size_t)(k0 + eA) * nq;     // (not dereferenced when n == 0)
      for (int base = 0; base < n; base += 256 * HAM_COPY_UNROLL) {
        float v[HAM_COPY_UNROLL];
#pragma unroll
        for (int u = 0; u < HAM_COPY_UNROLL; ++u) {
          const int idx = base + u * 256 + tid;
          v[u] = idx < n ? __builtin_nontemporal_load(gsrc + idx) : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < HAM_COPY_UNROLL; ++u) {
          const int idx = base + u * 256 + tid;
          if (idx < n) tile[idx] = v[u];
        }
      }
      if (self_here)
        for (int e = tid; e < nq; e += 256) tile[tile_blocks * nq + e] = H_node[(size_t)j * nq + e];
    }
    __syncthreads();
    const int r0 = s_pos[0], r1 = s_pos[nt];
    for (int r = r0 + tid; r < r1; r += 256) {
      int lo = 0, hi = nt - 1;            // largest t with s_pos[t] <= r (blocks without orbitals are skipped over)
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (s_pos[mid] <= r) lo = mid; else hi = mid - 1;
      }
      const int ap = r - s_pos[lo];
      const int a = s_map[lo * 32 + ap];
      const float* trow = tile + s_base[lo] + a * n_orb;
      const int grow = s_off[lo] + ap;
      for (int b = 0; b < n_j; ++b) {
        const long at = cstart + (long)b * len + r;
        __builtin_nontemporal_store(trow[s_colmap[b]], values + at);
        if (row_idx) __builtin_nontemporal_store(grow, row_idx + at);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------ host side
static size_t h256(size_t n) { return (n + 255) & ~(size_t)255; }

struct HamPlan {
  int* edge_pos;    // [n_edges] row of the edge's block inside a column of its destination
  uint32_t* edge_bits;   // [n_edges] orbitals of the source atom
  int* edge_off;    // [n_edges] first global row of the source atom
  int* self_pos;    // [n_owned]
  int* self_idx;    // [n_owned]
  int* col_len;     // [n_owned]
  long* col_start;  // [n_owned + 1]
};

static size_t carve_plan(char* base, int64_t n_edges, int32_t n_owned, HamPlan* p) {
  size_t used = 0;
  auto take = [&](size_t bytes) { char* q = base ? base + used : nullptr; used += h256(bytes); return q; };
  p->edge_pos = (int*)take((size_t)n_edges * sizeof(int));
  p->edge_bits = (uint32_t*)take((size_t)n_edges * sizeof(uint32_t));
  p->edge_off = (int*)take((size_t)n_edges * sizeof(int));
  p->self_pos = (int*)take((size_t)n_owned * sizeof(int));
  p->self_idx = (int*)take((size_t)n_owned * sizeof(int));
  p->col_len = (int*)take((size_t)n_owned * sizeof(int));
  p->col_start = (long*)take(((size_t)n_owned + 1) * sizeof(long));
  return used;
}

static size_t tab_ints(const egnn_ctx* ctx) {
  const int nq = ctx->n_orb * ctx->n_orb;
  return (size_t)2 * nq + (size_t)nq + 1 + ctx->unc_q.size();
}

extern "C" int egnn_hamiltonian_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, int32_t n_owned, int32_t n_total,
                                                size_t* ws_bytes, size_t* plan_bytes) {
  if (!ctx || !ws_bytes || !plan_bytes || n_edges < 0 || n_owned < 0 || n_total < n_owned) return EGNN_EINVAL;
  const size_t nq = (size_t)ctx->n_orb * ctx->n_orb;
  const size_t n_blocks = (size_t)n_edges + (size_t)n_total;
  const size_t partials = (n_blocks + ham_bpw((int)nq) - 1) / ham_bpw((int)nq) + 1;   // >= the count of either launch
  const size_t loss = h256(sizeof(double)) + 3 * h256(partials * sizeof(double));
  const size_t tabs = h256(tab_ints(ctx) * sizeof(int)) + h256(ctx->unc_c.size() * sizeof(float));
  *ws_bytes = (loss > tabs ? loss : tabs) + 256;
  HamPlan p;
  *plan_bytes = carve_plan(nullptr, n_edges, n_owned, &p) + 256;
  return EGNN_OK;
}

static int check_orbitals(egnn_ctx* ctx, const char* who) {
  if (ctx->n_orb <= 0 || ctx->n_orb > 32) return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": need 1..32 orbitals per atom");
  return EGNN_OK;
}

extern "C" int egnn_onsite_hii(egnn_ctx* ctx, const float* x, const float* V_node, float* H_ii, int32_t n_nodes,
                               void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_orbitals(ctx, "onsite_hii");
  if (rc) return rc;
  if (n_nodes < 0 || !ws || (n_nodes > 0 && (!x || !V_node || !H_ii))) return egnn_fail(ctx, EGNN_EINVAL, "onsite_hii: bad argument");
  if (((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "onsite_hii: workspace not 256-byte aligned");
  const size_t ni = tab_ints(ctx), nf = ctx->unc_c.size();
  if (ws_bytes < h256(ni * sizeof(int)) + h256(nf * sizeof(float))) return egnn_fail(ctx, EGNN_EWS, "onsite_hii: workspace too small");
  if (n_nodes == 0) return EGNN_OK;
  hipStream_t st = (hipStream_t)stream;
  const int nq = ctx->n_orb * ctx->n_orb;
  // integer table: q_row[nq] q_vrow[nq] unc_ptr[nq+1] unc_q[nnz]
  std::vector<int>& ti = ctx->tab_on_i;
  if (ti.empty()) {
    ti.resize(ni);
    for (int s = 0; s < ctx->n_slots; ++s) {
      const int L = ctx->slot_L[s];
      for (int M = 0; M < 2 * L + 1; ++M) {
        ti[ctx->slot_qoff[s] + M] = L * L + M;
        ti[nq + ctx->slot_qoff[s] + M] = ctx->slot_vrow[s];
      }
    }
    std::copy(ctx->unc_ptr.begin(), ctx->unc_ptr.end(), ti.begin() + 2 * nq);
    std::copy(ctx->unc_q.begin(), ctx->unc_q.end(), ti.begin() + 3 * nq + 1);
  }
  int* tab_i = (int*)ws;
  float* tab_f = (float*)((char*)ws + h256(ni * sizeof(int)));
  // (sources owned by the context: no need to wait for the copies)
  EGNN_HIP(ctx, hipMemcpyAsync(tab_i, ti.data(), ni * sizeof(int), hipMemcpyHostToDevice, st));
  EGNN_HIP(ctx, hipMemcpyAsync(tab_f, ctx->unc_c.data(), nf * sizeof(float), hipMemcpyHostToDevice, st));
  const int D = (ctx->desc.lmax + 1) * (ctx->desc.lmax + 1);
  const size_t shmem = ((size_t)D * ctx->desc.channels + nq) * sizeof(float);
  hipLaunchKernelGGL(onsite_kernel, dim3(n_nodes), dim3(256), shmem, st, x, V_node, tab_i, tab_i + nq, tab_i + 2 * nq,
                     tab_i + 3 * nq + 1, tab_f, H_ii, D, ctx->log2_channels, nq);
  EGNN_LAUNCH_CHECK(ctx, "onsite_kernel");
  return EGNN_OK;
}

static size_t onsite_bwd_tab_ints(const egnn_ctx* ctx) {
  const int nq = ctx->n_orb * ctx->n_orb;
  int nv = 0;
  for (int L = 0; L <= EGNN_L_READOUT; ++L) nv += ctx->n_out[L];
  const int D = (ctx->desc.lmax + 1) * (ctx->desc.lmax + 1);
  return (size_t)(nq + 1) + ctx->unc_q.size() + (size_t)(D + 1) + nq + nq + 2 * (size_t)nv;
}

extern "C" int egnn_onsite_backward_workspace_bytes(const egnn_ctx* ctx, int32_t n_nodes, size_t* bytes) {
  if (!ctx || !bytes || n_nodes < 0) return EGNN_EINVAL;
  const size_t nq = (size_t)ctx->n_orb * ctx->n_orb;
  *bytes = h256(onsite_bwd_tab_ints(ctx) * sizeof(int)) + h256(ctx->unc_c.size() * sizeof(float)) +
           h256((size_t)n_nodes * nq * sizeof(float)) + 256;
  return EGNN_OK;
}

extern "C" int egnn_onsite_backward(egnn_ctx* ctx, const float* x, const float* V_node, const float* dH_ii,
                                    float* dx, float* dV_node, int32_t n_nodes, void* ws, size_t ws_bytes,
                                    void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_orbitals(ctx, "onsite_backward");
  if (rc) return rc;
  if (n_nodes <= 0 || !x || !V_node || !dH_ii || !dx || !dV_node || !ws)
    return egnn_fail(ctx, EGNN_EINVAL, "onsite_backward: bad argument");
  if (((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "onsite_backward: workspace not 256-byte aligned");
  const int nq = ctx->n_orb * ctx->n_orb;
  const size_t ni = onsite_bwd_tab_ints(ctx), nf = ctx->unc_c.size();
  const size_t need = h256(ni * sizeof(int)) + h256(nf * sizeof(float)) + h256((size_t)n_nodes * nq * sizeof(float));
  if (ws_bytes < need) return egnn_fail(ctx, EGNN_EWS, "onsite_backward: workspace too small");
  hipStream_t st = (hipStream_t)stream;
  const int D = (ctx->desc.lmax + 1) * (ctx->desc.lmax + 1);
  int nv = 0;
  for (int L = 0; L <= EGNN_L_READOUT; ++L) nv += ctx->n_out[L];
  // host tables (built once, kept in the context): transposed uncoupling (q <- H), the collapsed components that
  // read each feature row, rows of V
  const size_t o_rowptr = (size_t)(nq + 1) + nf, o_rowt = o_rowptr + D + 1, o_vrow = o_rowt + nq, o_vL = o_vrow + nq,
               o_vq = o_vL + nv;
  std::vector<int>& ti = ctx->tab_onb_i;
  std::vector<float>& tf = ctx->tab_onb_f;
  if (ti.empty()) {
    std::vector<std::vector<std::pair<int, float>>> byq(nq);
    for (int e = 0; e < nq; ++e)
      for (int n = ctx->unc_ptr[e]; n < ctx->unc_ptr[e + 1]; ++n) byq[ctx->unc_q[n]].push_back({e, ctx->unc_c[n]});
    std::vector<int> q_row(nq), q_vrow(nq), vrow_L(nv, 0), vrow_qoff(nv, 0);
    for (int s = 0; s < ctx->n_slots; ++s) {
      const int L = ctx->slot_L[s];
      vrow_L[ctx->slot_vrow[s]] = L;
      vrow_qoff[ctx->slot_vrow[s]] = ctx->slot_qoff[s];
      for (int M = 0; M < 2 * L + 1; ++M) {
        q_row[ctx->slot_qoff[s] + M] = L * L + M;
        q_vrow[ctx->slot_qoff[s] + M] = ctx->slot_vrow[s];
      }
    }
    ti.reserve(ni);
    int run = 0;
    ti.push_back(0);
    for (int q = 0; q < nq; ++q) ti.push_back(run += (int)byq[q].size());
    for (int q = 0; q < nq; ++q)
      for (auto& e : byq[q]) {
        ti.push_back(e.first);
        tf.push_back(e.second);
      }
    std::vector<std::vector<int>> byrow(D);
    for (int t = 0; t < nq; ++t)
      if (q_row[t] < D) byrow[q_row[t]].push_back(t);
    run = 0;
    ti.push_back(0);
    for (int r = 0; r < D; ++r) ti.push_back(run += (int)byrow[r].size());
    for (int r = 0; r < D; ++r) ti.insert(ti.end(), byrow[r].begin(), byrow[r].end());
    ti.resize(o_rowt + nq, 0);
    ti.insert(ti.end(), q_vrow.begin(), q_vrow.end());
    ti.insert(ti.end(), vrow_L.begin(), vrow_L.end());
    ti.insert(ti.end(), vrow_qoff.begin(), vrow_qoff.end());
  }
  if (ti.size() != ni || tf.size() != nf) return egnn_fail(ctx, EGNN_EINVAL, "onsite_backward: table size mismatch");
  int* tab_i = (int*)ws;
  float* tab_f = (float*)((char*)ws + h256(ni * sizeof(int)));
  float* dq_all = (float*)((char*)tab_f + h256(nf * sizeof(float)));
  // (sources owned by the context: no need to wait for the copies)
  EGNN_HIP(ctx, hipMemcpyAsync(tab_i, ti.data(), ni * sizeof(int), hipMemcpyHostToDevice, st));
  EGNN_HIP(ctx, hipMemcpyAsync(tab_f, tf.data(), nf * sizeof(float), hipMemcpyHostToDevice, st));
  hipLaunchKernelGGL(onsite_bwd_node_kernel, dim3(n_nodes), dim3(256), 2 * (size_t)nq * sizeof(float), st, V_node, dH_ii,
                     tab_i, tab_i + nq + 1, tab_f, tab_i + o_rowptr, tab_i + o_rowt, tab_i + o_vrow, dx, dq_all, D,
                     ctx->log2_channels, nq);
  EGNN_LAUNCH_CHECK(ctx, "onsite_bwd_node_kernel");
  hipLaunchKernelGGL(onsite_bwd_dV_kernel, dim3(nv), dim3(256), 0, st, x, dq_all, tab_i + o_vL, tab_i + o_vq, dV_node,
                     n_nodes, D, ctx->log2_channels, nq, ctx->desc.lmax);
  EGNN_LAUNCH_CHECK(ctx, "onsite_bwd_dV_kernel");
  return EGNN_OK;
}

extern "C" int egnn_apply_padding(egnn_ctx* ctx, float* H, int64_t n_blocks, const int32_t* row_atom,
                                  const int32_t* col_atom, const int32_t* species, const uint32_t* orb_bits,
                                  int32_t n_species, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_orbitals(ctx, "apply_padding");
  if (rc) return rc;
  if (n_blocks < 0 || n_species <= 0 || !species || !orb_bits || (n_blocks > 0 && !H))
    return egnn_fail(ctx, EGNN_EINVAL, "apply_padding: bad argument");
  if (n_blocks == 0) return EGNN_OK;
  const int bpw = ham_bpw(ctx->n_orb * ctx->n_orb);
  const long n_wg = ((long)n_blocks + bpw - 1) / bpw;
  if (n_wg > 2147483647L) return egnn_fail(ctx, EGNN_EINVAL, "apply_padding: too many blocks");
  hipLaunchKernelGGL(padding_kernel, dim3((unsigned)n_wg), dim3(256), 0, (hipStream_t)stream, H, (long)n_blocks,
                     ctx->n_orb, bpw, row_atom, col_atom, species, orb_bits, n_species);
  EGNN_LAUNCH_CHECK(ctx, "padding_kernel");
  return EGNN_OK;
}

extern "C" int egnn_loss_l1l2(egnn_ctx* ctx, const float* H, const float* T, int64_t n_blocks,
                              const int32_t* row_atom, const int32_t* col_atom, const int32_t* species,
                              const uint32_t* orb_bits, int32_t n_species, float* loss, float* dH, void* ws,
                              size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_orbitals(ctx, "loss_l1l2");
  if (rc) return rc;
  if (n_blocks <= 0 || n_species <= 0 || !H || !T || !species || !orb_bits || !loss || !ws)
    return egnn_fail(ctx, EGNN_EINVAL, "loss_l1l2: bad argument");
  if (((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "loss_l1l2: workspace not 256-byte aligned");
  const int bpw = ham_bpw(ctx->n_orb * ctx->n_orb);
  const long nb_v = ((long)n_blocks + bpw - 1) / bpw;                       // workgroups of the loss kernel
  const long nb_b = ((long)n_blocks + HL_PER_WG - 1) / HL_PER_WG;           // workgroups of the counting kernel (<= nb_v)
  const size_t need = h256(sizeof(double)) + 3 * h256((size_t)(nb_v + 1) * sizeof(double));
  if (ws_bytes < need) return egnn_fail(ctx, EGNN_EWS, "loss_l1l2: workspace too small");
  if (nb_v > 2147483647L) return egnn_fail(ctx, EGNN_EINVAL, "loss_l1l2: too many blocks");
  hipStream_t st = (hipStream_t)stream;
  double* count = (double*)ws;
  double* p0 = (double*)((char*)ws + h256(sizeof(double)));
  double* p1 = (double*)((char*)p0 + h256((size_t)(nb_v + 1) * sizeof(double)));
  double* p2 = (double*)((char*)p1 + h256((size_t)(nb_v + 1) * sizeof(double)));
  hipLaunchKernelGGL(present_partial_kernel, dim3((unsigned)nb_b), dim3(256), 0, st, (long)n_blocks, ctx->n_orb,
                     row_atom, col_atom, species, orb_bits, n_species, p0);
  EGNN_LAUNCH_CHECK(ctx, "present_partial_kernel");
  hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, p0, (int)nb_b, count);
  EGNN_LAUNCH_CHECK(ctx, "sum_partials_kernel");
  hipLaunchKernelGGL(l1l2_partial_kernel, dim3((unsigned)nb_v), dim3(256), 0, st, H, T, (long)n_blocks, ctx->n_orb, bpw,
                     row_atom, col_atom, species, orb_bits, n_species, count, dH, p1, p2);
  EGNN_LAUNCH_CHECK(ctx, "l1l2_partial_kernel");
  hipLaunchKernelGGL(l1l2_final_kernel, dim3(1), dim3(256), 0, st, p1, p2, (int)nb_v, count, loss);
  EGNN_LAUNCH_CHECK(ctx, "l1l2_final_kernel");
  return EGNN_OK;
}

static int check_ham_graph(egnn_ctx* ctx, const egnn_graph* g, const char* who) {
  if (!g) return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": null graph");
  if (g->n_edges < 0 || g->n_edges > 2147483647LL || g->n_owned < 0 || g->n_total < g->n_owned)
    return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": bad graph sizes");
  if (!g->row_ptr || (g->n_edges > 0 && !g->src)) return egnn_fail(ctx, EGNN_EINVAL, std::string(who) + ": null graph arrays");
  return EGNN_OK;
}

extern "C" int egnn_hamiltonian_structure(egnn_ctx* ctx, const egnn_graph* g, const int32_t* species,
                                          const uint32_t* orb_bits, int32_t n_species, int32_t* orb_off,
                                          int64_t* col_ptr, void* plan, size_t plan_bytes, int64_t* n_cols,
                                          int64_t* nnz, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_orbitals(ctx, "hamiltonian_structure");
  if (rc) return rc;
  if ((rc = check_ham_graph(ctx, g, "hamiltonian_structure"))) return rc;
  if (!species || !orb_bits || n_species <= 0 || !orb_off || !col_ptr || !plan || !n_cols || !nnz)
    return egnn_fail(ctx, EGNN_EINVAL, "hamiltonian_structure: null pointer");
  if (((uintptr_t)plan & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "hamiltonian_structure: plan not 256-byte aligned");
  HamPlan p;
  if (plan_bytes < carve_plan((char*)plan, g->n_edges, g->n_owned, &p))
    return egnn_fail(ctx, EGNN_EWS, "hamiltonian_structure: plan buffer too small");
  hipStream_t st = (hipStream_t)stream;
  const int n_total = g->n_total, n_owned = g->n_owned;
  if ((rc = egnn_launch_fill_int(ctx, orb_off, 1, 0, st))) return rc;
  if (n_total > 0) {
    hipLaunchKernelGGL(orb_count_kernel, dim3((n_total + 255) / 256), dim3(256), 0, st, species, orb_bits, n_species,
                       n_total, ctx->n_orb, orb_off);
    EGNN_LAUNCH_CHECK(ctx, "orb_count_kernel");
  }
  if ((rc = egnn_launch_row_scan(ctx, orb_off, n_total, st))) return rc;
  if (n_owned > 0) {
    const uint32_t all = ctx->n_orb >= 32 ? 0xffffffffu : ((1u << ctx->n_orb) - 1u);
    hipLaunchKernelGGL(column_layout_kernel, dim3((n_owned + 255) / 256), dim3(256), 0, st, g->row_ptr, g->src, species,
                       orb_bits, n_species, all, orb_off, n_owned, p.edge_pos, p.edge_bits, p.edge_off, p.self_pos,
                       p.self_idx, p.col_len, p.col_start);
    EGNN_LAUNCH_CHECK(ctx, "column_layout_kernel");
  }
  hipLaunchKernelGGL(scan_i64_kernel, dim3(1), dim3(1024), 0, st, p.col_start, n_owned);
  EGNN_LAUNCH_CHECK(ctx, "scan_i64_kernel");
  hipLaunchKernelGGL(col_ptr_kernel, dim3((n_owned + 1 + 255) / 256), dim3(256), 0, st, orb_off, p.col_start, p.col_len,
                     n_owned, reinterpret_cast<long*>(col_ptr));
  EGNN_LAUNCH_CHECK(ctx, "col_ptr_kernel");
  int32_t nc = 0;
  long nz = 0;
  EGNN_HIP(ctx, hipMemcpyAsync(&nc, orb_off + n_owned, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  EGNN_HIP(ctx, hipMemcpyAsync(&nz, p.col_start + n_owned, sizeof(long), hipMemcpyDeviceToHost, st));
  EGNN_HIP(ctx, hipStreamSynchronize(st));
  *n_cols = nc;
  *nnz = nz;
  return EGNN_OK;
}

extern "C" int egnn_hamiltonian_fill(egnn_ctx* ctx, const egnn_graph* g, const int32_t* species,
                                     const uint32_t* orb_bits, int32_t n_species, const int32_t* orb_off,
                                     const void* plan, size_t plan_bytes, const float* H_edge, const float* H_node,
                                     int32_t* row_idx, float* values, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  int rc = check_orbitals(ctx, "hamiltonian_fill");
  if (rc) return rc;
  if ((rc = check_ham_graph(ctx, g, "hamiltonian_fill"))) return rc;
  if (!species || !orb_bits || n_species <= 0 || !orb_off || !plan || !H_node || (g->n_edges > 0 && !H_edge) ||
      (g->n_owned > 0 && !values))
    return egnn_fail(ctx, EGNN_EINVAL, "hamiltonian_fill: null pointer");
  HamPlan p;
  if (plan_bytes < carve_plan((char*)plan, g->n_edges, g->n_owned, &p))
    return egnn_fail(ctx, EGNN_EWS, "hamiltonian_fill: plan buffer too small");
  if (g->n_owned == 0) return EGNN_OK;
  const int nq = ctx->n_orb * ctx->n_orb;
  int tile_blocks = HAM_TILE_FLOATS / nq;
  tile_blocks = tile_blocks < 1 ? 1 : (tile_blocks > HAM_MAX_TILE ? HAM_MAX_TILE : tile_blocks);
  // tile [tile+1][nq], s_pos [tile+1], s_off [tile], s_base [tile], s_map [tile][32]
  const size_t shmem = (size_t)(tile_blocks + 1) * nq * sizeof(float) + (size_t)(3 * tile_blocks + 1) * sizeof(int) +
                       (size_t)tile_blocks * 32;
  hipLaunchKernelGGL(csc_fill_kernel, dim3(g->n_owned), dim3(256), shmem, (hipStream_t)stream, g->row_ptr, species,
                     orb_bits, n_species, orb_off, p.edge_pos, p.edge_bits, p.edge_off, p.self_pos, p.self_idx,
                     p.col_len, p.col_start, H_edge, H_node, ctx->n_orb, tile_blocks, row_idx, values);
  EGNN_LAUNCH_CHECK(ctx, "csc_fill_kernel");
  return EGNN_OK;
}
