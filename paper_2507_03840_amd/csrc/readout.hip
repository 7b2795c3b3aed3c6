// S6: readout of the orbital blocks H_ij (Fig. 2(e); Sec. 2.2; Sec. 3 "Message passing", last paragraph).
//
// Per edge k: z = zs[src] + zt[dst] (already channel-mixed), tensor product with the harmonics of the
// edge direction up to coupled degree 4, collapse of the channel axis by V_L (E -> 1), and the inverse
// Clebsch-Gordan transform (Eq. 1 read backwards) from the coupled components q[o][M] to the orbital
// block H[(a,m_a)][(b,m_b)].
//
// As in the message kernel the product is evaluated in the bond frame and rotated back per lane (lane = channel:
// all lanes run the same rotation code; rotating the collapsed numbers instead -- fewer of them, since the collapse
// commutes with the rotation -- needs one rotation per coupled slot with the degree varying from lane to lane,
// which a wavefront executes one degree after the other and which costs more than it saves).
//
// A group of E lanes works on one edge: lane = channel for the product, then the lanes share the n_orb^2 collapsed
// outputs among themselves through LDS.  The small index tables of the collapse and of the uncoupling live in LDS.
#include "egnn_internal.h"
#include "bond_frame.h"
#include "w_half.h"

#define RO_ITERS 8   // edges per slot per workgroup
#define RO_D 25      // (L_READOUT+1)^2

struct ReadoutTabs {
  const int* q_row;     // [nq]  row (L^2+L+M) of the bond-frame product feeding collapsed value t
  const int* q_vrow;    // [nq]  row of the packed V used for it
  const int* slot_L;    // [n_slots]
  const int* slot_qoff; // [n_slots]
  const int* unc_ptr;   // [nq+1]
  const int* unc_q;     // [nnz]
  const float* unc_c;   // [nnz]
  int nq, n_slots, n_vrows, nnz;
};

// The lanes of a slot exchange data through LDS.  Up to 64 channels a slot lies inside one wavefront, whose LDS
// accesses execute in program order: a wave-level fence is all the synchronisation needed, and the waves of the
// workgroup run free of each other (their memory phases and their arithmetic phases overlap).  Wider slots span
// wavefronts and need the workgroup barrier.
template <int log2E>
__device__ __forceinline__ void readout_slot_sync() {
  if constexpr (log2E <= 6) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
  } else {
    __syncthreads();
  }
}

// HALF: w in half precision (layout of w_half.h)
template <int LMAX, int log2E, bool HALF>
__global__ __launch_bounds__(256) void readout_kernel(const int* __restrict__ src, const int* __restrict__ dst,
                                                      const float4* __restrict__ rhat_d,
                                                      const float* __restrict__ zs, const float* __restrict__ zt,
                                                      const float* __restrict__ w, const int* __restrict__ w_row,
                                                      const float* __restrict__ V,
                                                      ReadoutTabs tb, float* __restrict__ H, long n_edges,
                                                      int tiles_per_xcd) {
  using Mid = typename ReadoutMid<LMAX>::T;
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  constexpr int P = Mid::P;
  extern __shared__ float smem[];
  constexpr int E = 1 << log2E;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1), slot = tid >> log2E;
  constexpr int n_slots = 256 >> log2E;
  constexpr int us = E + 4;             // padded row of su and sV: 16-byte aligned, rows 4 banks apart
  float* sV = smem;                                      // [n_vrows][E+4]
  float* su = sV + (size_t)tb.n_vrows * us + (size_t)slot * RO_D * us;    // this slot: [25][E+4]
  float* sq = smem + (size_t)tb.n_vrows * us + (size_t)n_slots * RO_D * us + (size_t)slot * tb.nq;  // this slot: [nq]
  // tables: offsets of the two rows of each collapsed value, CSR of the uncoupling
  int* s_urow = reinterpret_cast<int*>(smem + (size_t)tb.n_vrows * us + (size_t)n_slots * RO_D * us + (size_t)n_slots * tb.nq);
  int* s_vrow = s_urow + tb.nq;
  int* s_ptr = s_vrow + tb.nq;          // [nq + 1]
  int* s_uq = s_ptr + tb.nq + 1;        // [nnz]
  float* s_uc = reinterpret_cast<float*>(s_uq + tb.nnz);   // [nnz]

  for (int i = tid; i < tb.n_vrows * E; i += 256) {
    const int r = i >> log2E, cc = i & (E - 1);
    sV[r * us + cc] = V[i];
  }
  for (int i = tid; i < tb.nq; i += 256) {
    s_urow[i] = tb.q_row[i] * us;
    s_vrow[i] = tb.q_vrow[i] * us;
  }
  for (int i = tid; i <= tb.nq; i += 256) s_ptr[i] = tb.unc_ptr[i];
  for (int i = tid; i < tb.nnz; i += 256) {
    s_uq[i] = tb.unc_q[i];
    s_uc[i] = tb.unc_c[i];
  }
  __syncthreads();

  // consecutive groups of edges (the same destinations, neighbouring sources) go to the same XCD, so that its L2
  // serves their rows of zs and zt
  const long tile = (long)(blockIdx.x & 7) * tiles_per_xcd + (blockIdx.x >> 3);
  const long k_base = tile * n_slots * RO_ITERS;
  // The indices of an edge (source, destination, weight row) and its unit vector are fetched one edge ahead, so that
  // the loads of the rows they address start at once.
  int s_nx = 0, d_nx = 0;
  size_t kw_nx = 0;
  float4 g_nx = make_float4(0.0f, 0.0f, 1.0f, 1.0f);
  if (k_base + slot < n_edges) {
    const long k = k_base + slot;
    s_nx = src[k];
    d_nx = dst[k];
    g_nx = rhat_d[k];
    kw_nx = (size_t)egnn_weight_row(w_row, k);
  }
  for (int it = 0; it < RO_ITERS; ++it) {
    const long k = k_base + (long)it * n_slots + slot;
    const bool live = k < n_edges;
    if (live) {
      const int s = s_nx, d = d_nx;
      const float4 g = g_nx;
      const size_t kw = kw_nx;
      const float* zsp = zs + ((size_t)s * D << log2E) + c;
      const float* ztp = zt + ((size_t)d * D << log2E) + c;
      float v[D], wr[P], o[RO_D];
      if constexpr (!HALF) {
        const float* wp = w + (kw * P << log2E) + c;
#pragma unroll
        for (int p = 0; p < P; ++p) wr[p] = __builtin_nontemporal_load(wp + ((size_t)p << log2E));
      } else {
        w_half_load<P, log2E>(reinterpret_cast<const uint32_t*>(w) + kw * w_half_row_words(P << log2E), c, wr);
      }
#pragma unroll
      for (int i = 0; i < D; ++i) v[i] = zsp[(size_t)i << log2E] + ztp[(size_t)i << log2E];
      const long kn = k + n_slots;
      if (it + 1 < RO_ITERS && kn < n_edges) {
        s_nx = src[kn];
        d_nx = dst[kn];
        g_nx = rhat_d[kn];
        kw_nx = (size_t)egnn_weight_row(w_row, kn);
      }
      BondTrig t;
      egnn_bond_trig<4>(g.x, g.y, g.z, t);
      egnn_to_bond_frame<LMAX>(v, t);
      Mid::run(v, wr, o);
      egnn_from_bond_frame<4>(o, t);
#pragma unroll
      for (int i = 0; i < RO_D; ++i) su[i * us + c] = o[i];
    }
    readout_slot_sync<log2E>();
    if (live) {
      for (int q = c; q < tb.nq; q += E) {
        const float4* ur = reinterpret_cast<const float4*>(su + s_urow[q]);
        const float4* vr = reinterpret_cast<const float4*>(sV + s_vrow[q]);
        float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
#pragma unroll
        for (int cc = 0; cc < E / 4; ++cc) {
          const float4 a = ur[cc], b = vr[cc];
          s0 += a.x * b.x;
          s1 += a.y * b.y;
          s2 += a.z * b.z;
          s3 += a.w * b.w;
        }
        sq[q] = (s0 + s1) + (s2 + s3);
      }
    }
    readout_slot_sync<log2E>();
    if (live) {
      float* out = H + (size_t)k * tb.nq;
      for (int q = c; q < tb.nq; q += E) {
        float sum = 0.0f;
        for (int n = s_ptr[q]; n < s_ptr[q + 1]; ++n) sum += s_uc[n] * sq[s_uq[n]];
        __builtin_nontemporal_store(sum, out + q);
      }
    }
    // the next iteration overwrites su before its first synchronisation and sq after it: sq is safe (a
    // synchronisation in between), su needs the collapse of this iteration to be over -- it is, by the one above
  }
}

template <int L, int LE, bool HALF>
static int launch_readout(egnn_ctx* ctx, const egnn_graph* g, const float4* rd, const float* zs, const float* zt,
                          const float* w, const int* w_row, const float* V, const ReadoutTabs& tb, float* H,
                          hipStream_t stream) {
  constexpr int E = 1 << LE, n_slots = 256 / E;
  const size_t shmem = ((size_t)tb.n_vrows * (E + 4) + (size_t)n_slots * RO_D * (E + 4) + (size_t)n_slots * tb.nq) *
                           sizeof(float) +
                       ((size_t)3 * tb.nq + 1 + 2 * (size_t)tb.nnz) * sizeof(int);
  const long per_wg = (long)n_slots * RO_ITERS;
  const int tiles_per_xcd = (int)(((g->n_edges + per_wg - 1) / per_wg + 7) / 8);
  dim3 grid((unsigned)(8 * tiles_per_xcd)), block(256);   // (a tile past the end finds no live edge)
  auto kern = readout_kernel<L, LE, HALF>;
  if (shmem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)shmem);
    if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(readout_kernel)");
  }
  hipLaunchKernelGGL(kern, grid, block, shmem, stream, g->src, g->dst, rd, zs, zt, w, w_row, V, tb, H,
                     (long)g->n_edges, tiles_per_xcd);
  EGNN_LAUNCH_CHECK(ctx, "readout_kernel");
  return EGNN_OK;
}

int egnn_launch_readout(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* zs, const float* zt,
                        const float* w, const float* V, const int* tab_i, const float* tab_f, float* H,
                        hipStream_t stream, bool half, bool shared_rows) {
  const long n = g->n_edges;
  const int* w_row = shared_rows ? g->w_row : nullptr;
  if (n == 0) return EGNN_OK;
  const int nq = ctx->n_orb * ctx->n_orb;
  ReadoutTabs tb;
  tb.nq = nq;
  tb.n_slots = ctx->n_slots;
  tb.n_vrows = 0;
  for (int L = 0; L <= EGNN_L_READOUT; ++L) tb.n_vrows += ctx->n_out[L];
  // layout of the integer table: q_row[nq] q_vrow[nq] slot_L[n_slots] slot_qoff[n_slots] unc_ptr[nq+1] unc_q[nnz]
  tb.q_row = tab_i;
  tb.q_vrow = tab_i + nq;
  tb.slot_L = tab_i + 2 * nq;
  tb.slot_qoff = tb.slot_L + ctx->n_slots;
  tb.unc_ptr = tb.slot_qoff + ctx->n_slots;
  tb.unc_q = tb.unc_ptr + nq + 1;
  tb.unc_c = tab_f;
  tb.nnz = (int)ctx->unc_c.size();
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
#define CASE(L, LE)                                                                         \
  if (ctx->desc.lmax == L && ctx->log2_channels == LE)                                      \
    return half ? launch_readout<L, LE, true>(ctx, g, rd, zs, zt, w, w_row, V, tb, H, stream)      \
                : launch_readout<L, LE, false>(ctx, g, rd, zs, zt, w, w_row, V, tb, H, stream);
#define CASES(L) CASE(L, 3) CASE(L, 4) CASE(L, 5) CASE(L, 6) CASE(L, 7)
  CASES(0) CASES(1) CASES(2) CASES(3) CASES(4)
#undef CASES
#undef CASE
  return egnn_fail(ctx, EGNN_EINVAL, "readout: unsupported (lmax, channels)");
}
