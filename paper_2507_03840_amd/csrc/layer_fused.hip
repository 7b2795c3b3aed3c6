// S3 + S4 fused: radial weights are produced on the matrix cores and consumed by the tensor-product messages
// without ever being written to HBM.
//
//   a[j] = nbar^-1/2 sum_{k: dst(k)=j} sum_p w_k[p][c] (C_p . h_src(k) . Yhat(rhat_k)),
//   w_k[p][c] = fc(d_k) alpha_p (W_r2 SiLU(W_r1 B(d_k)))[p*E + c]
// (Sec. 3 "Message passing"; coupling of Sec. 2.2 / Eq. 1 in the bond frame of Sec. 2.1 / Fig. 2(d)).
//
// One workgroup per destination node, its edges taken in tiles of 32 (one MFMA row block).  Per tile:
//   1. the hidden activations of the 32 edges (times fc) are computed once, cut into bf16 pieces and put in LDS
//      (the A operand of every contraction of the tile);
//   2. the coupling paths are ordered by input degree l1, so the product splits into l_max+1 chunks that use
//      disjoint, contiguous runs of weights.  For each chunk the waves contract A with the matching rows of the
//      pre-split W_r2 (split-bf16 MFMA, six products per fp32 product) and leave the 32 x (paths of the chunk) x E
//      weights in an LDS tile; then every lane -- one channel of PAIRS edges -- rotates the degree-l1 block of its
//      source rows into the bond frame, runs the chunk of the product with the weights read from LDS and
//      accumulates the bond-frame result of each of its edges in registers;
//   3. after the last chunk each edge's result is rotated back and added to the lane's partial sum of the node.
// Slots are added in fixed order through LDS at the end: deterministic, no atomics.
// HBM traffic per edge: the gathered source row and 20 bytes of indices / geometry; W_r2 (pre-split, a few hundred
// KB) is re-read from L2 once per tile.
//
// Status: correct (parity-tested at every supported shape) but latency-bound -- each chunk phase is a few thousand
// cycles between two barriers with an L2 round trip at its start, the matrix pipe is 17 % busy -- and at 3,000
// atoms / 32 channels it takes 1.70 ms against 0.82 + 0.69 ms for the two-kernel route.  It is therefore opt-in
// (EGNN_OPT_FUSED); the next step for it is a producer / consumer split of the waves so that both phases run
// continuously.
#include "egnn_internal.h"
#include "bond_frame.h"
#include "split_bf16.h"

#define FU_TILE 32
#define FU_AROW4 25   // uint4 per row of the A tile: 24 of data (3 pieces x 64 bf16) + 1 of padding

template <int LMAX, int LOG2E>
struct FusedCfg {
  static constexpr int E = 1 << LOG2E;
  static constexpr int T = (E >= 64) ? 512 : 256;   // threads per workgroup
  static constexpr int NW = T / 64;
  static constexpr int NSLOT = T / E;               // edges worked on at once in the product phase
  static constexpr int PAIRS = FU_TILE / NSLOT;     // edges of a tile per lane
  static constexpr int D = (LMAX + 1) * (LMAX + 1);
  using Mid = typename LayerMid<LMAX>::T;
  static constexpr int SWLD = Mid::CHUNK_MAX * E;   // floats per edge row of the weight tile
  static_assert(PAIRS >= 1 && PAIRS <= 4, "tile / slot mismatch");
};

struct FusedArgs {
  const int* row_ptr;
  const int* src;
  const float4* rhat_d;
  const float* h;
  const float* W_r1;
  const uint16_t* W2s;
  float* a;
  int n_owned, nodes_per_xcd, n_rbf;
  float scale, r_cut;
};

// One chunk (input degree L1) of one tile: weights of the chunk -> LDS, then the product for this lane's edges.
template <int LMAX, int LOG2E, int L1>
__device__ __forceinline__ void fused_chunk(const FusedArgs& g, const uint4* sA, float* sw, const int* ssrc,
                                            const float* strig, int cnt, float (&o)[FusedCfg<LMAX, LOG2E>::PAIRS][FusedCfg<LMAX, LOG2E>::D]) {
  using Cfg = FusedCfg<LMAX, LOG2E>;
  using Mid = typename Cfg::Mid;
  constexpr int E = Cfg::E;
  constexpr int NCH = Mid::CHUNK_COUNT[L1];
  constexpr int n0 = Mid::CHUNK_FIRST[L1] * E, n1 = n0 + NCH * E;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = lane & 31, hh = lane >> 5;

  // ---- contraction: column blocks of the chunk are dealt to the waves
  for (int nb = (n0 >> 5) + wave; nb < ((n1 + 31) >> 5); nb += Cfg::NW) {
    const int n = nb * 32 + m;
    const bool ok = n >= n0 && n < n1;
    uint4 b_frag[3][4];
    {
      const uint4* row = reinterpret_cast<const uint4*>(g.W2s + ((size_t)(ok ? n : n0) * 3) * EGNN_HIDDEN + hh * 32);
#pragma unroll
      for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int t = 0; t < 4; ++t) b_frag[p][t] = row[p * 8 + t];
    }
    float16v acc = {0};
    const uint4* arow = sA + m * FU_AROW4 + hh * 4;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const uint4 a_hi = arow[t], a_mid = arow[8 + t], a_lo = arow[16 + t];
      // smallest terms first
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a_lo), as_bf16x8(b_frag[0][t]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a_hi), as_bf16x8(b_frag[2][t]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a_mid), as_bf16x8(b_frag[1][t]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a_mid), as_bf16x8(b_frag[0][t]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a_hi), as_bf16x8(b_frag[1][t]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a_hi), as_bf16x8(b_frag[0][t]), acc, 0, 0, 0);
    }
    if (ok) {
      float* col = sw + (n - n0);
#pragma unroll
      for (int i = 0; i < 16; ++i) col[(8 * (i >> 2) + 4 * hh + (i & 3)) * Cfg::SWLD] = acc[i];
    }
  }
  __syncthreads();

  // ---- product: lane = (edge slot, channel); its PAIRS edges of the tile one after the other
  const int c = tid & (E - 1), slot = tid >> LOG2E;
#pragma unroll
  for (int q = 0; q < Cfg::PAIRS; ++q) {
    const int r = slot + Cfg::NSLOT * q;
    if (r < cnt) {
      const float* hp = g.h + (((size_t)ssrc[r] * Cfg::D + L1 * L1) << LOG2E) + c;
      float v[2 * L1 + 1], wl[NCH];
#pragma unroll
      for (int i = 0; i < 2 * L1 + 1; ++i) v[i] = hp[(size_t)i << LOG2E];
#pragma unroll
      for (int i = 0; i < NCH; ++i) wl[i] = sw[r * Cfg::SWLD + (i << LOG2E) + c];
      if (L1 > 0) {
        BondTrig t;
        const float* tr = strig + r * 16;
#pragma unroll
        for (int mm = 1; mm <= L1; ++mm) {
          t.cp[mm] = tr[mm - 1];
          t.sp[mm] = tr[4 + mm - 1];
          t.ct[mm] = tr[8 + mm - 1];
          t.st[mm] = tr[12 + mm - 1];
        }
        egnn_to_bond_frame_l<L1>(v, t);
      }
      Mid::template run_l1<L1>(v, wl, o[q]);
    }
  }
  __syncthreads();
}

template <int LMAX, int LOG2E>
__global__ __launch_bounds__((FusedCfg<LMAX, LOG2E>::T)) void layer_fused_kernel(FusedArgs g) {
  using Cfg = FusedCfg<LMAX, LOG2E>;
  constexpr int E = Cfg::E, D = Cfg::D, T = Cfg::T;
  extern __shared__ uint4 smem4[];
  uint4* sA = smem4;                                              // [32][FU_AROW4]
  float* sw = reinterpret_cast<float*>(sA + FU_TILE * FU_AROW4);   // [32][SWLD], reused for the final reduction
  constexpr int SW_FLOATS = (FU_TILE * Cfg::SWLD > T * D) ? FU_TILE * Cfg::SWLD : T * D;
  float* sW1 = sw + SW_FLOATS;                                    // [n_rbf][64]
  float* strig = sW1 + 32 * EGNN_HIDDEN;                          // [32][16]
  float* sd = strig + FU_TILE * 16;                               // [32] edge lengths
  int* ssrc = reinterpret_cast<int*>(sd + FU_TILE);               // [32]

  const int j = (blockIdx.x & 7) * g.nodes_per_xcd + (blockIdx.x >> 3);
  if (j >= g.n_owned) return;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1), slot = tid >> LOG2E;
  for (int i = tid; i < g.n_rbf * EGNN_HIDDEN; i += T) sW1[i] = g.W_r1[(i & 63) * g.n_rbf + (i >> 6)];

  const int k0 = g.row_ptr[j], k1 = g.row_ptr[j + 1];
  float acc[D];
#pragma unroll
  for (int i = 0; i < D; ++i) acc[i] = 0.0f;
  const float step = g.r_cut / (float)(g.n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);

  for (int tile0 = k0; tile0 < k1; tile0 += FU_TILE) {
    const int cnt = (k1 - tile0 < FU_TILE) ? (k1 - tile0) : FU_TILE;
    __syncthreads();   // previous tile finished with the staged data
    if (tid < FU_TILE) {
      const int k = tile0 + (tid < cnt ? tid : cnt - 1);
      const float4 rd = g.rhat_d[k];
      ssrc[tid] = g.src[k];
      sd[tid] = rd.w;
      BondTrig t;
      egnn_bond_trig<4>(rd.x, rd.y, rd.z, t);
#pragma unroll
      for (int mm = 1; mm <= 4; ++mm) {
        strig[tid * 16 + mm - 1] = t.cp[mm];
        strig[tid * 16 + 4 + mm - 1] = t.sp[mm];
        strig[tid * 16 + 8 + mm - 1] = t.ct[mm];
        strig[tid * 16 + 12 + mm - 1] = t.st[mm];
      }
    }
    __syncthreads();
    // A tile: thread (edge r, group of 8 hidden units); fc * SiLU(W_r1 B(d)) cut into three bf16 pieces
    if (tid < 256) {
      const int r = tid & 31, ug = tid >> 5;
      const float d = sd[r];
      float pre[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) pre[i] = 0.0f;
      for (int b = 0; b < g.n_rbf; ++b) {
        const float u = d - (float)b * step;
        const float B = __expf(-u * u * inv2s2);
        const float* wrow = sW1 + b * EGNN_HIDDEN + ug * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) pre[i] += wrow[i] * B;
      }
      const float fc = 0.5f * (1.0f + cosf(3.14159265358979323846f * d / g.r_cut));
      uint32_t ph[4], pm[4], pl[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float x0 = pre[2 * q], x1 = pre[2 * q + 1];
        const Split3 s0 = split3(fc * x0 / (1.0f + __expf(-x0)));
        const Split3 s1 = split3(fc * x1 / (1.0f + __expf(-x1)));
        ph[q] = pack2(s0.hi, s1.hi);
        pm[q] = pack2(s0.mid, s1.mid);
        pl[q] = pack2(s0.lo, s1.lo);
      }
      uint4* row = sA + r * FU_AROW4 + ug;
      row[0] = make_uint4(ph[0], ph[1], ph[2], ph[3]);
      row[8] = make_uint4(pm[0], pm[1], pm[2], pm[3]);
      row[16] = make_uint4(pl[0], pl[1], pl[2], pl[3]);
    }
    __syncthreads();

    float o[Cfg::PAIRS][D];
#pragma unroll
    for (int q = 0; q < Cfg::PAIRS; ++q)
#pragma unroll
      for (int i = 0; i < D; ++i) o[q][i] = 0.0f;
    fused_chunk<LMAX, LOG2E, 0>(g, sA, sw, ssrc, strig, cnt, o);
    if constexpr (LMAX >= 1) fused_chunk<LMAX, LOG2E, 1>(g, sA, sw, ssrc, strig, cnt, o);
    if constexpr (LMAX >= 2) fused_chunk<LMAX, LOG2E, 2>(g, sA, sw, ssrc, strig, cnt, o);
    if constexpr (LMAX >= 3) fused_chunk<LMAX, LOG2E, 3>(g, sA, sw, ssrc, strig, cnt, o);
    if constexpr (LMAX >= 4) fused_chunk<LMAX, LOG2E, 4>(g, sA, sw, ssrc, strig, cnt, o);

    // back to the lab frame, into the node's partial sums
#pragma unroll
    for (int q = 0; q < Cfg::PAIRS; ++q) {
      const int r = slot + Cfg::NSLOT * q;
      if (r < cnt) {
        BondTrig t;
        const float* tr = strig + r * 16;
#pragma unroll
        for (int mm = 1; mm <= 4; ++mm) {
          t.cp[mm] = tr[mm - 1];
          t.sp[mm] = tr[4 + mm - 1];
          t.ct[mm] = tr[8 + mm - 1];
          t.st[mm] = tr[12 + mm - 1];
        }
        egnn_from_bond_frame<LMAX>(o[q], t);
#pragma unroll
        for (int i = 0; i < D; ++i) acc[i] += o[q][i];
      }
    }
  }

  __syncthreads();
  float* red = sw;
#pragma unroll
  for (int i = 0; i < D; ++i) red[((slot * D + i) << LOG2E) + c] = acc[i];
  __syncthreads();
  const int row = D << LOG2E;
  float* out = g.a + (size_t)j * row;
  for (int idx = tid; idx < row; idx += T) {
    float sum = 0.0f;
    for (int s = 0; s < Cfg::NSLOT; ++s) sum += red[s * row + idx];
    out[idx] = sum * g.scale;
  }
}

template <int LMAX, int LOG2E>
static int launch_fused(egnn_ctx* ctx, const FusedArgs& args, int grid, hipStream_t stream) {
  using Cfg = FusedCfg<LMAX, LOG2E>;
  constexpr int SW_FLOATS = (FU_TILE * Cfg::SWLD > Cfg::T * Cfg::D) ? FU_TILE * Cfg::SWLD : Cfg::T * Cfg::D;
  const size_t shmem = (size_t)FU_TILE * FU_AROW4 * sizeof(uint4) +
                       ((size_t)SW_FLOATS + 32 * EGNN_HIDDEN + FU_TILE * 16 + FU_TILE) * sizeof(float) +
                       FU_TILE * sizeof(int);
  auto kern = layer_fused_kernel<LMAX, LOG2E>;
  if (shmem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)shmem);
    if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(layer_fused_kernel)");
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(Cfg::T), shmem, stream, args);
  EGNN_LAUNCH_CHECK(ctx, "layer_fused_kernel");
  return EGNN_OK;
}

bool egnn_fused_supported(const egnn_ctx* ctx) {
  const int E = ctx->desc.channels;
  return E == 16 || E == 32 || E == 64;
}

// W2s: the pre-split W_r2 (egnn_launch_split_w2).  a [n_owned][D][E].
int egnn_launch_layer_fused(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* h,
                            const float* W_r1, const void* W2s, float* a, hipStream_t stream) {
  const int n = g->n_owned;
  if (n == 0) return EGNN_OK;
  FusedArgs args;
  args.row_ptr = g->row_ptr;
  args.src = g->src;
  args.rhat_d = reinterpret_cast<const float4*>(rhat_d);
  args.h = h;
  args.W_r1 = W_r1;
  args.W2s = reinterpret_cast<const uint16_t*>(W2s);
  args.a = a;
  args.n_owned = n;
  args.nodes_per_xcd = (n + 7) / 8;
  args.n_rbf = ctx->desc.n_rbf;
  args.scale = 1.0f / sqrtf(ctx->desc.agg_norm);
  args.r_cut = ctx->desc.r_cut;
  const int grid = args.nodes_per_xcd * 8;
#define CASE(L, LE) if (ctx->desc.lmax == L && ctx->log2_channels == LE) return launch_fused<L, LE>(ctx, args, grid, stream);
  CASE(0, 4) CASE(1, 4) CASE(2, 4) CASE(3, 4) CASE(4, 4)
  CASE(0, 5) CASE(1, 5) CASE(2, 5) CASE(3, 5) CASE(4, 5)
  CASE(0, 6) CASE(1, 6) CASE(2, 6) CASE(3, 6) CASE(4, 6)
#undef CASE
  return egnn_fail(ctx, EGNN_EINVAL, "layer_fused: unsupported (lmax, channels)");
}
