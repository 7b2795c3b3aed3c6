// Low-NN partitioner (host) and the pack / unpack of node embeddings that cross a partition boundary.
//
// Sec. 4.4 and Appendix A (Algorithm 1): bisection of the atoms into 2^l parts that balances the summed node degree
// of the two sides of every cut, treats the structure as periodic, and cuts the dimension in which a cut is expected
// to add the fewest neighbouring parts.  Here: one permutation of the atoms in which every sub-domain is a contiguous
// range, a work stack of sub-domains (range + cut state) in place of recursion, the opening of periodic rings as a
// pre-pass of its own, and a scored choice of the axis.  Sec. 4.3 / Fig. 4(b): per neighbouring part the rows a rank has to
// send are gathered by index into one contiguous buffer (pack), the received rows are put behind the rank's own rows
// (unpack); the payload may be half precision (Sec. 4.1).
//
// The partitioner is host code: it runs once per structure on a few 10^4 atoms (a sort per cut).
#include "egnn_internal.h"
#include <algorithm>
#include <array>
#include <cmath>
#include <numeric>
#include <vector>

namespace {

// One sub-domain waiting to be bisected: a contiguous range of the atom permutation plus its cut state.
struct SubDomain {
  int begin, end;     // range of `order_`
  int levels_left;    // bisections still to make below this sub-domain (2^levels_left parts)
  int n_cuts[3];      // cuts made so far along each axis (an axis that is not periodic starts with one)
  double origin[3];   // where the coordinate along each axis starts (for a periodic axis: where its ring was opened)
};

class LowNNBisection {
 public:
  LowNNBisection(const float* pos, const int32_t* degree, int n_atoms, const float box[3], const uint8_t pbc[3],
                 double r_cut, int32_t* part, int32_t* cut_log, int max_log)
      : n_(n_atoms), r_cut_(r_cut), part_(part), cut_log_(cut_log), max_log_(max_log) {
    xyz_.resize((size_t)n_ * 3);
    weight_.resize(n_);
    for (size_t i = 0; i < xyz_.size(); ++i) xyz_[i] = (double)pos[i];
    for (int i = 0; i < n_; ++i) weight_[i] = (double)degree[i];
    for (int a = 0; a < 3; ++a) {
      box_[a] = (double)box[a];
      periodic_[a] = pbc[a] != 0;
    }
    order_.resize(n_);
    std::iota(order_.begin(), order_.end(), 0);
  }

  int cuts_made() const { return cuts_made_; }

  // Depth first, left half before right half: an explicit stack instead of recursion (the right half is pushed first).
  void run(int levels) {
    SubDomain root{0, n_, levels, {0, 0, 0}, {0.0, 0.0, 0.0}};
    for (int a = 0; a < 3; ++a) {
      if (periodic_[a]) continue;
      root.n_cuts[a] = 1;   // an open axis needs no ring opening: it starts at its smallest coordinate
      if (n_ > 0) {
        double lo = xyz_[a];
        for (int i = 1; i < n_; ++i) lo = std::min(lo, xyz_[3 * (size_t)i + a]);
        root.origin[a] = lo;
      }
    }
    std::vector<SubDomain> todo{root};
    while (!todo.empty()) {
      SubDomain dom = todo.back();
      todo.pop_back();
      if (dom.levels_left == 0) {           // a finished part
        for (int t = dom.begin; t < dom.end; ++t) part_[order_[t]] = next_part_;
        ++next_part_;
        continue;
      }
      if (dom.begin == dom.end) {           // nothing to divide: its parts stay empty but keep their numbers
        next_part_ += 1 << dom.levels_left;
        continue;
      }
      open_rings(dom);
      const int axis = axis_with_fewest_neighbours(dom);
      double where;
      const int n_left = balanced_split(dom.begin, dom.end, axis, dom.origin[axis], /*reorder=*/true, &where);
      if (cut_log_ && cuts_made_ < max_log_) {
        int32_t* e = cut_log_ + 4 * (size_t)cuts_made_;
        e[0] = dom.levels_left;
        e[1] = axis;
        e[2] = dom.end - dom.begin;
        e[3] = n_left;
      }
      ++cuts_made_;
      SubDomain left = dom, right = dom;
      left.n_cuts[axis] = right.n_cuts[axis] = dom.n_cuts[axis] + 1;
      left.levels_left = right.levels_left = dom.levels_left - 1;
      left.end = right.begin = dom.begin + n_left;
      todo.push_back(right);
      todo.push_back(left);
    }
  }

 private:
  // coordinate of an atom along an axis, measured from `origin` (on a ring for a periodic axis)
  double along(int atom, int axis, double origin) const {
    const double v = xyz_[3 * (size_t)atom + axis] - origin;
    if (!periodic_[axis]) return v;
    double m = std::fmod(v, box_[axis]);
    if (m < 0.0) m += box_[axis];
    return m;
  }

  // Orders the atoms of [begin, end) along `axis` (atoms at equal coordinate keep their order) and finds the split
  // into a left and a right group whose summed weights differ least (fewest atoms on the left among equals; both
  // groups non-empty).  Returns the size of the left group and, in *where, the coordinate of the first atom on the
  // right.  reorder = false leaves the range as it was (ring opening only asks where the split would be).
  int balanced_split(int begin, int end, int axis, double origin, bool reorder, double* where) {
    const int n = end - begin;
    key_.resize(n);
    rank_.resize(n);
    for (int t = 0; t < n; ++t) key_[t] = along(order_[begin + t], axis, origin);
    std::iota(rank_.begin(), rank_.end(), 0);
    std::stable_sort(rank_.begin(), rank_.end(), [&](int a, int b) { return key_[a] < key_[b]; });
    int n_left = n;
    *where = n ? key_[rank_[0]] : 0.0;
    if (n >= 2) {
      double total = 0.0;
      for (int t = 0; t < n; ++t) total += weight_[order_[begin + t]];
      double left_sum = 0.0, least = 0.0;
      n_left = 1;
      for (int t = 0; t + 1 < n; ++t) {
        left_sum += weight_[order_[begin + rank_[t]]];
        const double imbalance = std::fabs(2.0 * left_sum - total);
        if (t == 0 || imbalance < least) {
          least = imbalance;
          n_left = t + 1;
        }
      }
      *where = key_[rank_[n_left]];
    }
    if (reorder) {
      moved_.resize(n);
      for (int t = 0; t < n; ++t) moved_[t] = order_[begin + rank_[t]];
      std::copy(moved_.begin(), moved_.end(), order_.begin() + begin);
    }
    return n_left;
  }

  // Pre-pass: one cut through a periodic ring divides nothing, it only fixes where the ring is opened.  Every axis
  // of the sub-domain that has no cut yet is opened at its balanced position; the atoms stay together.
  void open_rings(SubDomain& dom) {
    for (int a = 0; a < 3; ++a) {
      if (dom.n_cuts[a] != 0) continue;
      double where;
      balanced_split(dom.begin, dom.end, a, dom.origin[a], /*reorder=*/false, &where);
      dom.origin[a] += where;
      dom.n_cuts[a] = 1;
    }
  }

  // Score of an axis = neighbouring parts a cut along it is expected to add: 1 while the axis has been cut once
  // (two slabs of a ring see each other and nothing else), else the number of slabs of the sub-domain's extent that
  // the interaction range 2 r_cut spans.  Lowest score wins, the highest axis among equals.
  int axis_with_fewest_neighbours(const SubDomain& dom) const {
    int best_axis = 0, best_score = 0;
    for (int a = 0; a < 3; ++a) {
      int score = 1;
      if (dom.n_cuts[a] != 1) {
        double lo = 0.0, hi = 0.0;
        for (int t = dom.begin; t < dom.end; ++t) {
          const double v = along(order_[t], a, dom.origin[a]);
          if (t == dom.begin || v < lo) lo = v;
          if (t == dom.begin || v > hi) hi = v;
        }
        const double extent = hi - lo;
        score = extent > 0.0 ? (int)std::min(std::ceil(2.0 * r_cut_ / extent), 1073741824.0) : (1 << 30);
      }
      if (a == 0 || score <= best_score) {
        best_axis = a;
        best_score = score;
      }
    }
    return best_axis;
  }

  int n_;
  double r_cut_, box_[3];
  bool periodic_[3];
  std::vector<double> xyz_, weight_, key_;
  std::vector<int> order_, rank_, moved_;
  int32_t* part_;
  int32_t* cut_log_;
  int max_log_, cuts_made_ = 0, next_part_ = 0;
};

}  // namespace

extern "C" int egnn_partition_low_nn(const float* pos, const int32_t* degree, int32_t n_atoms, const float box[3],
                                     const uint8_t pbc[3], double r_cut, int32_t levels, int32_t* part,
                                     int32_t* cut_log, int32_t* n_cuts) {
  if (n_atoms < 0 || levels < 0 || levels > 20 || !box || !pbc || !(r_cut > 0.0) || (n_atoms > 0 && (!pos || !degree || !part)))
    return EGNN_EINVAL;
  for (int d = 0; d < 3; ++d)
    if (pbc[d] && !(box[d] > 0.0f)) return EGNN_EINVAL;
  LowNNBisection bisection(pos, degree, n_atoms, box, pbc, r_cut, part, cut_log, (1 << levels) - 1);
  bisection.run(levels);
  if (n_cuts) *n_cuts = bisection.cuts_made();
  return EGNN_OK;
}

// A spatially coherent numbering of the atoms, for callers whose atoms come in no particular order: the gathering
// kernels process destination nodes in index order and re-use the node rows that neighbouring destinations share,
// which works as far as consecutive indices are close in space.  Atoms are binned into cubes of edge `cell` (counted
// from the smallest coordinate of all atoms, at most 1024 per axis: the last cube takes the rest), the cubes are
// walked along a Morton (Z-order) curve, atoms of a cube stay in their order of arrival; the owned atoms come first,
// then the halo atoms, each group ordered in this way.
extern "C" int egnn_spatial_order(const float* pos, int32_t n_owned, int32_t n_total, float cell, int32_t* perm) {
  if (n_owned < 0 || n_total < n_owned || !(cell > 0.0f) || (n_total > 0 && (!pos || !perm))) return EGNN_EINVAL;
  if (n_total == 0) return EGNN_OK;
  double lo[3];
  for (int a = 0; a < 3; ++a) {
    lo[a] = pos[a];
    for (int i = 1; i < n_total; ++i) lo[a] = std::min(lo[a], (double)pos[3 * (size_t)i + a]);
  }
  std::vector<uint32_t> key(n_total);
  for (int i = 0; i < n_total; ++i) {
    uint32_t k = 0;
    for (int a = 0; a < 3; ++a) {
      const double q = std::floor(((double)pos[3 * (size_t)i + a] - lo[a]) / (double)cell);
      const uint32_t c = !(q >= 0.0) ? 0u : (q > 1023.0 ? 1023u : (uint32_t)q);   // (a NaN coordinate lands in cube 0)
      for (int b = 0; b < 10; ++b) k |= ((c >> b) & 1u) << (3 * b + a);
    }
    key[i] = k;
  }
  std::iota(perm, perm + n_total, 0);
  auto by_key = [&](int32_t x, int32_t y) { return key[x] < key[y]; };
  std::stable_sort(perm, perm + n_owned, by_key);
  std::stable_sort(perm + n_owned, perm + n_total, by_key);
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
