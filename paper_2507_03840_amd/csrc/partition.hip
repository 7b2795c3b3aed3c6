// Low-NN partitioner (host) and the pack / unpack of node embeddings that cross a partition boundary.
//
// Sec. 4.4 and Appendix A (Algorithm 1): recursive bisection of the atoms into 2^l parts that balances the summed node
// degree of the two sides of every cut, treats the structure as periodic, and cuts the dimension in which a cut is
// expected to add the fewest neighbouring parts.  Sec. 4.3 / Fig. 4(b): per neighbouring part the rows a rank has to
// send are gathered by index into one contiguous buffer (pack), the received rows are put behind the rank's own rows
// (unpack); the payload may be half precision (Sec. 4.1).
//
// The partitioner is host code: it runs once per structure on a few 10^4 atoms (a sort per cut).
#include "egnn_internal.h"
#include <algorithm>
#include <array>
#include <cmath>
#include <numeric>

namespace {

// a mod b with the sign of b (b > 0): the coordinate of a point on a ring of length b
double ring_mod(double a, double b) {
  double m = std::fmod(a, b);
  if (m != 0.0 && m < 0.0) m += b;
  return m;
}

struct Partitioner {
  const std::vector<double>& x;   // [n][3]
  const std::vector<double>& nd;  // [n]
  double box[3];
  bool pbc[3];
  double r_cut;
  int32_t* part;
  int32_t* cut_log;   // [max][4] (level, dimension, atoms, atoms on the left) or NULL
  int n_cuts = 0, max_cuts = 0, counter = 0;

  double coord(int atom, int d, double origin) const {
    const double v = x[3 * (size_t)atom + d] - origin;
    return pbc[d] ? ring_mod(v, box[d]) : v;
  }

  // Orders `idx` along dimension d; returns the number of atoms on the left of the balanced cut and its position.
  int get_cut(std::vector<int>& idx, int d, double origin, double* p) const {
    const size_t n = idx.size();
    std::vector<double> c(n);
    for (size_t t = 0; t < n; ++t) c[t] = coord(idx[t], d, origin);
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return c[a] < c[b]; });
    std::vector<int> sorted(n);
    for (size_t t = 0; t < n; ++t) sorted[t] = idx[order[t]];
    if (n < 2) {
      *p = n ? c[order[0]] : 0.0;
      idx.swap(sorted);
      return (int)n;
    }
    double total = 0.0;
    for (size_t t = 0; t < n; ++t) total += nd[sorted[t]];
    double run = 0.0, best = 0.0;
    int n_left = 1;
    for (size_t t = 0; t + 1 < n; ++t) {
      run += nd[sorted[t]];
      const double diff = std::fabs(2.0 * run - total);
      if (t == 0 || diff < best) { best = diff; n_left = (int)t + 1; }
    }
    *p = c[order[n_left]];
    idx.swap(sorted);
    return n_left;
  }

  void cut_domain(int l, std::vector<int> idx, std::array<int, 3> cuts, std::array<double, 3> origin) {
    if (l == 0) {
      for (int a : idx) part[a] = counter;
      ++counter;
      return;
    }
    if (idx.empty()) {
      counter += 1 << l;
      return;
    }
    // a dimension without a cut: open the ring at the balanced position, the atoms stay together
    for (;;) {
      int dim = -1;
      for (int d = 0; d < 3; ++d)
        if (cuts[d] == 0) { dim = d; break; }
      if (dim < 0) break;
      double p;
      std::vector<int> tmp = idx;
      get_cut(tmp, dim, origin[dim], &p);
      origin[dim] += p;
      cuts[dim] += 1;
    }
    int nn[3];
    for (int d = 0; d < 3; ++d) {
      if (cuts[d] == 1) {
        nn[d] = 1;
      } else {
        double lo = 0.0, hi = 0.0;
        for (size_t t = 0; t < idx.size(); ++t) {
          const double v = coord(idx[t], d, origin[d]);
          if (t == 0 || v < lo) lo = v;
          if (t == 0 || v > hi) hi = v;
        }
        const double L = hi - lo;
        nn[d] = L > 0.0 ? (int)std::min(std::ceil(2.0 * r_cut / L), 1073741824.0) : (1 << 30);
      }
    }
    int dim = 0;
    for (int d = 1; d < 3; ++d)
      if (nn[d] <= nn[dim]) dim = d;          // lowest count, highest index among equals
    double p;
    const int n_left = get_cut(idx, dim, origin[dim], &p);
    if (cut_log && n_cuts < max_cuts) {
      int32_t* e = cut_log + 4 * (size_t)n_cuts;
      e[0] = l; e[1] = dim; e[2] = (int32_t)idx.size(); e[3] = n_left;
    }
    ++n_cuts;
    cuts[dim] += 1;
    std::vector<int> left(idx.begin(), idx.begin() + n_left), right(idx.begin() + n_left, idx.end());
    std::vector<int>().swap(idx);
    cut_domain(l - 1, std::move(left), cuts, origin);
    cut_domain(l - 1, std::move(right), cuts, origin);
  }
};

}  // namespace

extern "C" int egnn_partition_low_nn(const float* pos, const int32_t* degree, int32_t n_atoms, const float box[3],
                                     const uint8_t pbc[3], double r_cut, int32_t levels, int32_t* part,
                                     int32_t* cut_log, int32_t* n_cuts) {
  if (n_atoms < 0 || levels < 0 || levels > 20 || !box || !pbc || !(r_cut > 0.0) || (n_atoms > 0 && (!pos || !degree || !part)))
    return EGNN_EINVAL;
  for (int d = 0; d < 3; ++d)
    if (pbc[d] && !(box[d] > 0.0f)) return EGNN_EINVAL;
  std::vector<double> x((size_t)n_atoms * 3), nd(n_atoms);
  for (size_t i = 0; i < x.size(); ++i) x[i] = (double)pos[i];
  for (int i = 0; i < n_atoms; ++i) nd[i] = (double)degree[i];
  Partitioner P{x, nd, {(double)box[0], (double)box[1], (double)box[2]}, {pbc[0] != 0, pbc[1] != 0, pbc[2] != 0}, r_cut, part,
                cut_log};
  P.max_cuts = (1 << levels) - 1;
  std::array<int, 3> cuts;
  std::array<double, 3> origin;
  for (int d = 0; d < 3; ++d) {
    cuts[d] = pbc[d] ? 0 : 1;
    origin[d] = 0.0;
    if (!pbc[d] && n_atoms > 0) {
      double lo = x[d];
      for (int i = 1; i < n_atoms; ++i) lo = std::min(lo, x[3 * (size_t)i + d]);
      origin[d] = lo;
    }
  }
  std::vector<int> idx(n_atoms);
  std::iota(idx.begin(), idx.end(), 0);
  P.cut_domain(levels, std::move(idx), cuts, origin);
  if (n_cuts) *n_cuts = P.n_cuts;
  return EGNN_OK;
}

// ------------------------------------------------------------------------------------------------ pack / unpack
// One workgroup per row, four floats per thread and step.  HALF: the buffer holds IEEE half precision (nearest even).
template <bool HALF>
__global__ __launch_bounds__(256) void pack_rows_kernel(const float* __restrict__ x, const int* __restrict__ idx,
                                                        int n_rows_x, int row_len, void* __restrict__ out) {
  const int r = blockIdx.x;
  int i = idx[r];
  i = i < 0 ? 0 : (i >= n_rows_x ? n_rows_x - 1 : i);
  const float4* src = reinterpret_cast<const float4*>(x + (size_t)i * row_len);
  for (int q = threadIdx.x; q < row_len / 4; q += 256) {
    const float4 v = src[q];
    if constexpr (HALF) {
      typedef _Float16 half4 __attribute__((ext_vector_type(4)));
      half4 h = {(_Float16)v.x, (_Float16)v.y, (_Float16)v.z, (_Float16)v.w};
      __builtin_nontemporal_store(__builtin_bit_cast(uint2, h).x, reinterpret_cast<uint32_t*>(out) + ((size_t)r * row_len / 2) + 2 * q);
      __builtin_nontemporal_store(__builtin_bit_cast(uint2, h).y, reinterpret_cast<uint32_t*>(out) + ((size_t)r * row_len / 2) + 2 * q + 1);
    } else {
      reinterpret_cast<float4*>(out)[(size_t)r * (row_len / 4) + q] = v;
    }
  }
}

template <bool HALF>
__global__ __launch_bounds__(256) void unpack_rows_kernel(const void* __restrict__ buf, int row_len,
                                                          float* __restrict__ x_rows) {
  const int r = blockIdx.x;
  float4* dst = reinterpret_cast<float4*>(x_rows + (size_t)r * row_len);
  for (int q = threadIdx.x; q < row_len / 4; q += 256) {
    if constexpr (HALF) {
      typedef _Float16 half4 __attribute__((ext_vector_type(4)));
      const uint2 u = reinterpret_cast<const uint2*>(buf)[(size_t)r * (row_len / 4) + q];
      const half4 h = __builtin_bit_cast(half4, u);
      dst[q] = make_float4((float)h.x, (float)h.y, (float)h.z, (float)h.w);
    } else {
      dst[q] = reinterpret_cast<const float4*>(buf)[(size_t)r * (row_len / 4) + q];
    }
  }
}

extern "C" int egnn_pack_rows(egnn_ctx* ctx, const float* x, int32_t n_rows_x, const int32_t* idx, int32_t n_idx,
                              int32_t half, void* out, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (n_idx < 0 || n_rows_x < 0 || (n_idx > 0 && (!x || !idx || !out || n_rows_x == 0)))
    return egnn_fail(ctx, EGNN_EINVAL, "pack_rows: bad argument");
  if (n_idx == 0) return EGNN_OK;
  const int row_len = (ctx->desc.lmax + 1) * (ctx->desc.lmax + 1) * ctx->desc.channels;   // a multiple of 8
  if (half)
    hipLaunchKernelGGL(pack_rows_kernel<true>, dim3(n_idx), dim3(256), 0, (hipStream_t)stream, x, idx, n_rows_x, row_len, out);
  else
    hipLaunchKernelGGL(pack_rows_kernel<false>, dim3(n_idx), dim3(256), 0, (hipStream_t)stream, x, idx, n_rows_x, row_len, out);
  EGNN_LAUNCH_CHECK(ctx, "pack_rows_kernel");
  return EGNN_OK;
}

extern "C" int egnn_unpack_rows(egnn_ctx* ctx, const void* buf, int32_t n_rows, int32_t half, float* x_full,
                                int32_t first_row, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (n_rows < 0 || first_row < 0 || (n_rows > 0 && (!buf || !x_full))) return egnn_fail(ctx, EGNN_EINVAL, "unpack_rows: bad argument");
  if (n_rows == 0) return EGNN_OK;
  const int row_len = (ctx->desc.lmax + 1) * (ctx->desc.lmax + 1) * ctx->desc.channels;
  float* rows = x_full + (size_t)first_row * row_len;
  if (half)
    hipLaunchKernelGGL(unpack_rows_kernel<true>, dim3(n_rows), dim3(256), 0, (hipStream_t)stream, buf, row_len, rows);
  else
    hipLaunchKernelGGL(unpack_rows_kernel<false>, dim3(n_rows), dim3(256), 0, (hipStream_t)stream, buf, row_len, rows);
  EGNN_LAUNCH_CHECK(ctx, "unpack_rows_kernel");
  return EGNN_OK;
}
