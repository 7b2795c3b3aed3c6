// S6: readout of the orbital blocks H_ij (Fig. 2(e); Sec. 2.2; Sec. 3 "Message passing", last paragraph).
//
// Per edge k: z = zs[src] + zt[dst] (already channel-mixed), tensor product with the harmonics of the
// edge direction up to coupled degree 4, collapse of the channel axis by V_L (E -> 1), and the inverse
// Clebsch-Gordan transform (Eq. 1 read backwards) from the coupled components q[o][M] to the orbital
// block H[(a,m_a)][(b,m_b)].
//
// As in the message kernel the product is evaluated in the bond frame.  The collapse acts on the channel
// axis only, so it commutes with the rotation: the E-channel result is collapsed while still in the bond
// frame and only the n_orb^2 collapsed numbers are rotated back (one (2L+1)-vector per coupled slot).
//
// A group of E lanes (a "slot") works on one edge: lane = channel for the product, then the lanes share
// the n_orb^2 collapsed outputs among themselves through LDS.
#include "egnn_internal.h"
#include "bond_frame.h"

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
  int nq, n_slots, n_vrows;
};

template <int L>
__device__ __forceinline__ void rotate_slot_back(float* q, const BondTrig& t) {
  float v[2 * L + 1];
#pragma unroll
  for (int i = 0; i < 2 * L + 1; ++i) v[i] = q[i];
  egnn_from_bond_frame_l<L>(v, t);
#pragma unroll
  for (int i = 0; i < 2 * L + 1; ++i) q[i] = v[i];
}

template <int LMAX, int log2E>
__global__ __launch_bounds__(256) void readout_kernel(const int* __restrict__ src, const int* __restrict__ dst,
                                                      const float4* __restrict__ rhat_d,
                                                      const float* __restrict__ zs, const float* __restrict__ zt,
                                                      const float* __restrict__ w, const float* __restrict__ V,
                                                      ReadoutTabs tb, float* __restrict__ H, long n_edges) {
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

  for (int i = tid; i < tb.n_vrows * E; i += 256) {
    const int r = i >> log2E, cc = i & (E - 1);
    sV[r * us + cc] = V[i];
  }

  const long k_base = (long)blockIdx.x * n_slots * RO_ITERS;
  for (int it = 0; it < RO_ITERS; ++it) {
    const long k = k_base + (long)it * n_slots + slot;
    const bool live = k < n_edges;
    BondTrig t;
    if (live) {
      const int s = src[k], d = dst[k];
      const float4 g = rhat_d[k];
      const float* zsp = zs + ((size_t)s * D << log2E) + c;
      const float* ztp = zt + ((size_t)d * D << log2E) + c;
      const float* wp = w + ((size_t)k * P << log2E) + c;
      float v[D], wr[P], o[RO_D];
#pragma unroll
      for (int p = 0; p < P; ++p) wr[p] = __builtin_nontemporal_load(wp + ((size_t)p << log2E));
#pragma unroll
      for (int i = 0; i < D; ++i) v[i] = zsp[(size_t)i << log2E] + ztp[(size_t)i << log2E];
      egnn_bond_trig<4>(g.x, g.y, g.z, t);
      egnn_to_bond_frame<LMAX>(v, t);
      Mid::run(v, wr, o);
#pragma unroll
      for (int i = 0; i < RO_D; ++i) su[i * us + c] = o[i];
    }
    __syncthreads();
    if (live) {
      for (int q = c; q < tb.nq; q += E) {
        const float4* ur = reinterpret_cast<const float4*>(su + tb.q_row[q] * us);
        const float4* vr = reinterpret_cast<const float4*>(sV + tb.q_vrow[q] * us);
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
    __syncthreads();
    if (live) {
      for (int sl = c; sl < tb.n_slots; sl += E) {
        float* q = sq + tb.slot_qoff[sl];
        switch (tb.slot_L[sl]) {
          case 1: rotate_slot_back<1>(q, t); break;
          case 2: rotate_slot_back<2>(q, t); break;
          case 3: rotate_slot_back<3>(q, t); break;
          case 4: rotate_slot_back<4>(q, t); break;
          default: break;
        }
      }
    }
    __syncthreads();
    if (live) {
      float* out = H + (size_t)k * tb.nq;
      for (int q = c; q < tb.nq; q += E) {
        float sum = 0.0f;
        for (int n = tb.unc_ptr[q]; n < tb.unc_ptr[q + 1]; ++n) sum += tb.unc_c[n] * sq[tb.unc_q[n]];
        __builtin_nontemporal_store(sum, out + q);
      }
    }
  }
}

template <int L, int LE>
static int launch_readout(egnn_ctx* ctx, const egnn_graph* g, const float4* rd, const float* zs, const float* zt,
                          const float* w, const float* V, const ReadoutTabs& tb, float* H, hipStream_t stream) {
  constexpr int E = 1 << LE, n_slots = 256 / E;
  const size_t shmem = ((size_t)tb.n_vrows * (E + 4) + (size_t)n_slots * RO_D * (E + 4) + (size_t)n_slots * tb.nq) *
                       sizeof(float);
  const long per_wg = (long)n_slots * RO_ITERS;
  dim3 grid((unsigned)((g->n_edges + per_wg - 1) / per_wg)), block(256);
  auto kern = readout_kernel<L, LE>;
  if (shmem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)shmem);
    if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(readout_kernel)");
  }
  hipLaunchKernelGGL(kern, grid, block, shmem, stream, g->src, g->dst, rd, zs, zt, w, V, tb, H, (long)g->n_edges);
  EGNN_LAUNCH_CHECK(ctx, "readout_kernel");
  return EGNN_OK;
}

int egnn_launch_readout(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* zs, const float* zt,
                        const float* w, const float* V, const int* tab_i, const float* tab_f, float* H,
                        hipStream_t stream) {
  const long n = g->n_edges;
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
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
#define CASE(L, LE) \
  if (ctx->desc.lmax == L && ctx->log2_channels == LE) return launch_readout<L, LE>(ctx, g, rd, zs, zt, w, V, tb, H, stream);
#define CASES(L) CASE(L, 3) CASE(L, 4) CASE(L, 5) CASE(L, 6) CASE(L, 7)
  CASES(0) CASES(1) CASES(2) CASES(3) CASES(4)
#undef CASES
#undef CASE
  return egnn_fail(ctx, EGNN_EINVAL, "readout: unsupported (lmax, channels)");
}
