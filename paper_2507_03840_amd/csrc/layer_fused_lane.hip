// S3 + S4 fused, second design (EGNN_OPT_FUSED = 2): the radial weights of an (edge, channel) are produced on the
// matrix cores straight into the registers of the lane that consumes them -- no weight tensor in memory, no hand-over
// through LDS.
//
//   a[j] = nbar^-1/2 sum_{k: dst(k)=j} sum_p w_k[p][c] (C_p . h_src(k) . Yhat(rhat_k)),
//   w_k[p][c] = fc(d_k) alpha_p (W_r2 SiLU(W_r1 B(d_k)))[p*E + c]
// (Sec. 3 "Message passing"; coupling of Sec. 2.2 / Eq. 1 in the bond frame of Sec. 2.1 / Fig. 2(d)).
//
// The contraction runs transposed: the matrix-core tile has 32 rows of W_r2 and 32 edges as columns.  Its result
// register i of lane (edge = lane % 32, hh = lane / 32) is row 8 (i / 4) + 4 hh + (i % 4); the rows of W_r2 are packed
// so that this row is (path 16 pt + i, channel 2 cp + hh) -- one tile gives every lane 16 path weights of ONE
// (edge, channel), ceil(P / 16) tiles ("pt") give it all of them, and a pass over the E / 2 channel pairs ("cp")
// covers the channels.  The lane then runs the bond-frame product for its (edge, channel) exactly as the two-kernel
// route does, the 32 edges of a wave are added with a butterfly, and the wave keeps one partial row of the node sum
// per channel in LDS.
//
// One workgroup per destination node: seven waves of 32 edges each per round (nodes with more than 224 incoming edges
// take more rounds), an eighth wave streams the packed tiles of W_r2 (12 KB each, the tiles of a channel pair together)
// from L2 into two LDS buffers, one barrier per channel pair with LDS-only fences.  The hidden activations of a wave's 32 edges stay in registers as the other
// matrix-core operand for the whole round.  Source rows are read from a copy of h in which the two channels of a
// pair are adjacent ([node][cp][(l,m)][2]), so that the 25 values a lane gathers share two or three cache lines.
#include "egnn_internal.h"
#include "bond_frame.h"
#include "split_bf16.h"

#define F2_WAVES 7                       // compute waves = blocks of 32 edges per round
#define F2_THREADS ((F2_WAVES + 1) * 64)
#define F2_ROUND (32 * F2_WAVES)         // edges of a node per round
#define F2_BROW4 17                      // uint4 per staged row of W_r2: 16 of data (two pieces of 64 halves) + 1 of padding
// Operands of the radial contraction are cut into two half-precision pieces (11 significant bits each) after a scaling
// by a power of two: x * 2^s = hi + lo exactly to 22 bits, and a product is hi*hi + hi*lo + lo*hi (the lo*lo term is
// 2^-22 of the product, the size of the representation error).  Against fp64 the contraction is as accurate as the
// three-piece bf16 form with six products (1e-7 of the largest result, rms 1.5e-8) at half the matrix-core work.
// Half precision has a narrow exponent range, so the two scalings are taken from the weights on the device, once per
// call: alpha W_r2 by its largest magnitude, the hidden activations by the bound |SiLU(pre)| <= |pre| <=
// max_j sum_b |W_r1[j][b]| (basis values lie in [0, 1]); the largest piece then sits in [2^13, 2^14), and elements
// more than 2^-17 below it lose low bits that are below 2^-28 of the largest one.
typedef unsigned int f2_u4 __attribute__((ext_vector_type(4)));
typedef _Float16 f2_h8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ f2_h8 f2_as_h8(uint4 v) { return __builtin_bit_cast(f2_h8, v); }
// x -> (hi, lo) half-precision pieces, as raw bits
__device__ __forceinline__ void f2_split(float x, uint32_t& hi, uint32_t& lo) {
  const _Float16 h = (_Float16)x;
  const _Float16 l = (_Float16)(x - (float)h);
  hi = __builtin_bit_cast(unsigned short, h);
  lo = __builtin_bit_cast(unsigned short, l);
}

__device__ __forceinline__ void f2_release_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
}
__device__ __forceinline__ void f2_barrier_acquire() {
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// W_r2 [n = path * E + channel][64 units] fp32 -> W2p[tile = cp * npt + pt][R][2 pieces][64 halves] (16 uint4 per row),
// values alpha_p * W_r2 * s_w cut into pieces; R = result row of the tile:
// (i, hh) = (4 (R / 8) + R % 4, (R / 4) % 2) <-> (path 16 pt + i, channel 2 cp + hh).
// Paths past the last one repeat path 0 (their weights are computed and never used).
__global__ __launch_bounds__(256) void f2_pack_kernel(const float* __restrict__ W_r2, uint4* __restrict__ W2p, int P,
                                                      int log2E, int npt, int n_tiles, PathAlpha alpha,
                                                      const float* __restrict__ scales) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= n_tiles * 32 * 16) return;
  const int c16 = idx % 16, R = (idx / 16) % 32, tile = idx / (16 * 32);
  const int cp = tile / npt, pt = tile - cp * npt;
  const int i = 4 * (R >> 3) + (R & 3), hh = (R >> 2) & 1;
  int p = 16 * pt + i;
  if (p >= P) p = 0;
  const int n = (p << log2E) + 2 * cp + hh;
  const int piece = c16 >> 3, k0 = (c16 & 7) * 8;
  const float sc = alpha.a[p] * scales[0];
  uint32_t w[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    uint32_t h0, l0, h1, l1;
    f2_split(sc * W_r2[(size_t)n * EGNN_HIDDEN + k0 + 2 * q], h0, l0);
    f2_split(sc * W_r2[(size_t)n * EGNN_HIDDEN + k0 + 2 * q + 1], h1, l1);
    w[q] = piece == 0 ? (h0 | (h1 << 16)) : (l0 | (l1 << 16));
  }
  W2p[idx] = make_uint4(w[0], w[1], w[2], w[3]);
}

// h [node][(l,m)][E] -> h2 [node][cp][(l,m)][2]
__global__ __launch_bounds__(256) void f2_pair_kernel(const float* __restrict__ h, float* __restrict__ h2, long n_values,
                                                      int D, int log2E) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n_values) return;
  const int row = D << log2E;
  const long node = idx / row;
  const int rem = (int)(idx - node * row);
  const int cp = rem / (2 * D), r2 = rem - cp * 2 * D;
  const int i = r2 >> 1, hh = r2 & 1;
  h2[idx] = h[node * row + ((long)i << log2E) + 2 * cp + hh];
}

// Sum over the 32 lanes of a half wavefront with data-parallel-primitive moves (vector ALU only, no LDS): four steps
// inside the rows of 16 lanes, then lane 15 of every row is added into the row after it: the lanes of rows 1 and 3
// hold the sum of their half (rows 0 and 2 hold other things and are not read).  Each step is applied to all N values before the next one, so that no instruction waits for its
// predecessor.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float f2_dpp(float x) {
  return __builtin_bit_cast(float,
                            __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROW_MASK, 0xF, false));
}
template <int N>
__device__ __forceinline__ void f2_sum32(float (&x)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i) x[i] += f2_dpp<0xB1, 0xF>(x[i]);    // quad_perm [1,0,3,2]: lane ^ 1
#pragma unroll
  for (int i = 0; i < N; ++i) x[i] += f2_dpp<0x4E, 0xF>(x[i]);    // quad_perm [2,3,0,1]: lane ^ 2
#pragma unroll
  for (int i = 0; i < N; ++i) x[i] += f2_dpp<0x141, 0xF>(x[i]);   // row_half_mirror: the other quad of the group of 8
#pragma unroll
  for (int i = 0; i < N; ++i) x[i] += f2_dpp<0x140, 0xF>(x[i]);   // row_mirror: the other group of 8 of the row
#pragma unroll
  for (int i = 0; i < N; ++i) x[i] += f2_dpp<0x142, 0xF>(x[i]);   // row_bcast 15: every row adds the row before it
}

template <int LMAX>
__global__ __launch_bounds__(F2_THREADS) void f2_kernel(const int* __restrict__ row_ptr, const int* __restrict__ src,
                                                        const float4* __restrict__ rhat_d,
                                                        const float* __restrict__ h2, const float* __restrict__ W_r1,
                                                        const uint4* __restrict__ W2p,
                                                        const float* __restrict__ scales, float* __restrict__ a,
                                                        int n_owned, int nodes_per_xcd, int n_rbf, int log2E,
                                                        float scale, float r_cut) {
  using Mid = typename LayerMid<LMAX>::T;
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  constexpr int P = Mid::P;
  constexpr int NPT = (P + 15) / 16;
  __shared__ float sW1[32 * EGNN_HIDDEN];          // [b][j]
  __shared__ uint4 sB[2][NPT * 32 * F2_BROW4];     // the NPT tiles of a channel pair, double-buffered
  extern __shared__ float sP[];                    // [F2_WAVES][E / 2][2][D]: per wave, partial rows of the node sum

  const int j = (blockIdx.x & 7) * nodes_per_xcd + (blockIdx.x >> 3);
  if (j >= n_owned || (int)(blockIdx.x >> 3) >= nodes_per_xcd) return;
  const int E = 1 << log2E, ncp = E >> 1;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int i = tid; i < n_rbf * EGNN_HIDDEN; i += F2_THREADS) {
    const int jj = i & (EGNN_HIDDEN - 1), b = i >> 6;
    sW1[i] = W_r1[jj * n_rbf + b];
  }
  for (int i = tid; i < F2_WAVES * D * E; i += F2_THREADS) sP[i] = 0.0f;
  __syncthreads();

  const int k0 = row_ptr[j], deg = row_ptr[j + 1] - k0;
  const int rounds = (deg + F2_ROUND - 1) / F2_ROUND;
  const float s_g = scales[1];

  if (wave == F2_WAVES) {
    // ---- loader: the NPT tiles of channel pair s (all rounds in sequence) -> sB[s & 1].  The loads of a group are
    // issued a whole group time before they are written to LDS, so that their latency does not show.
    const int n_groups = rounds * ncp;
    constexpr int NV = NPT * 8;
    f2_u4 v[NV];                   // (native vectors: an array of them that lives across iterations stays in registers)
    auto fetch = [&](int s) {
      const int cp = s % ncp;
      const f2_u4* tsrc = reinterpret_cast<const f2_u4*>(W2p) + (size_t)cp * NPT * (32 * 16);
#pragma unroll
      for (int i = 0; i < NV; ++i) v[i] = tsrc[i * 64 + lane];
    };
    if (n_groups > 0) fetch(0);
    for (int s = 0; s < n_groups; ++s) {
      f2_u4* dstb = reinterpret_cast<f2_u4*>(sB[s & 1]);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int u = i * 64 + lane, row = u >> 4, c16 = u & 15;            // row counts through the NPT tiles
        dstb[row * F2_BROW4 + c16] = v[i];
      }
      if (s + 1 < n_groups) fetch(s + 1);
      f2_release_barrier();
    }
  } else {
    const int m = lane & 31, hh = lane >> 5;
    float* sPw = sP + (size_t)wave * D * E;
    int step = 0;
    for (int r = 0; r < rounds; ++r) {
      const int e = r * F2_ROUND + wave * 32 + m;
      const bool valid = e < deg;
      const bool wave_active = r * F2_ROUND + wave * 32 < deg;      // the same for all lanes
      const long k = k0 + (valid ? e : deg - 1);
      if (!wave_active) {                                           // nothing to do this round: keep the barriers in step
        for (int cp = 0; cp < ncp; ++cp, ++step) f2_barrier_acquire();
        continue;
      }
      const float4 g = rhat_d[k];
      const int srcn = src[k];
      // hidden activations (times the cutoff envelope) of the lane's edge, units 32 hh .. 32 hh + 31, in pieces
      uint4 gf[2][4];
      {
        const float step_r = r_cut / (float)(n_rbf - 1);
        const float inv2s2 = 0.5f / (step_r * step_r);
        float pre[32];
#pragma unroll
        for (int s = 0; s < 32; ++s) pre[s] = 0.0f;
        for (int b = 0; b < n_rbf; ++b) {
          const float u = g.w - (float)b * step_r;
          const float Bv = __expf(-u * u * inv2s2);
          const float* wrow = sW1 + b * EGNN_HIDDEN + hh * 32;
#pragma unroll
          for (int s = 0; s < 32; ++s) pre[s] += wrow[s] * Bv;
        }
        // (a lane past the node's last edge gets a zero envelope: zero weights, a zero message, nothing to mask later)
        const float fc = valid ? s_g * egnn_envelope(g.w, r_cut) : 0.0f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          uint32_t ph[4], pl[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const float x0 = pre[8 * t + 2 * q], x1 = pre[8 * t + 2 * q + 1];
            uint32_t h0, l0, h1, l1;
            f2_split(fc * x0 / (1.0f + __expf(-x0)), h0, l0);
            f2_split(fc * x1 / (1.0f + __expf(-x1)), h1, l1);
            ph[q] = h0 | (h1 << 16);
            pl[q] = l0 | (l1 << 16);
          }
          gf[0][t] = make_uint4(ph[0], ph[1], ph[2], ph[3]);
          gf[1][t] = make_uint4(pl[0], pl[1], pl[2], pl[3]);
        }
      }
      BondTrig trig;
      egnn_bond_trig<LMAX>(g.x, g.y, g.z, trig);

      // the source row of the lane's (edge, channel) is requested one channel pair ahead, before the matrix-core
      // phase, so that the gather has that phase to arrive
      const float* hsrc = h2 + (size_t)srcn * ncp * (2 * D) + hh;
      float vn[D];
#pragma unroll
      for (int i = 0; i < D; ++i) vn[i] = hsrc[2 * i];
      for (int cp = 0; cp < ncp; ++cp) {
        float v[D];
#pragma unroll
        for (int i = 0; i < D; ++i) v[i] = vn[i];
        {
          const float* hn = hsrc + (size_t)(cp + 1 < ncp ? cp + 1 : cp) * (2 * D);
#pragma unroll
          for (int i = 0; i < D; ++i) vn[i] = hn[2 * i];
        }
        // ---- the weights of (edge, channel 2 cp + hh): NPT tiles, three piece products per fp32 product
        float wr[NPT * 16];
        f2_barrier_acquire();
        const uint4* gbase = sB[step & 1] + m * F2_BROW4 + hh * 4;
        ++step;
        {
          // the pieces of W_r2 of contraction step u = 4 pt + t are read from LDS one step ahead of their products
          uint4 wf[2][2];
          auto lds_step = [&](int u, uint4 (&dstw)[2]) {
            const uint4* row = gbase + (u >> 2) * (32 * F2_BROW4) + (u & 3);
            dstw[0] = row[0];
            dstw[1] = row[8];
          };
          lds_step(0, wf[0]);
          float16v acc;
#pragma unroll
          for (int u = 0; u < 4 * NPT; ++u) {
            const int pt = u >> 2, t = u & 3;
            if (u + 1 < 4 * NPT) lds_step(u + 1, wf[(u + 1) & 1]);
            if (t == 0) {
#pragma unroll
              for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
            }
            // smallest terms first: (lo,hi) (hi,lo) (hi,hi)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(f2_as_h8(wf[u & 1][1]), f2_as_h8(gf[0][t]), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(f2_as_h8(wf[u & 1][0]), f2_as_h8(gf[1][t]), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(f2_as_h8(wf[u & 1][0]), f2_as_h8(gf[0][t]), acc, 0, 0, 0);
            if (t == 3) {
#pragma unroll
              for (int i = 0; i < 16; ++i) wr[16 * pt + i] = acc[i];
            }
          }
        }
        // ---- the message of this (edge, channel) in the bond frame, rotated back
        float o[D];
        egnn_to_bond_frame<LMAX>(v, trig);
        Mid::run(v, wr, o);
        egnn_from_bond_frame<LMAX>(o, trig);
        // ---- sum over the 32 edges of the wave (fixed order), one partial row per channel
        float* prow = sPw + (size_t)(cp * 2 + hh) * D;
        f2_sum32<D>(o);
        if (m == 16) {
          if (r == 0) {
#pragma unroll
            for (int i = 0; i < D; ++i) prow[i] = o[i];
          } else {
#pragma unroll
            for (int i = 0; i < D; ++i) prow[i] += o[i];
          }
        }
      }
    }
  }
  __syncthreads();
  // a[j][(l,m)][c] = scale * sum over the waves, in fixed order (the operand scalings are undone here)
  const float out_scale = scale * scales[2];
  float* out = a + ((size_t)j * D << log2E);
  for (int idx = tid; idx < (D << log2E); idx += F2_THREADS) {
    const int i = idx >> log2E, c = idx & (E - 1);
    float sum = 0.0f;
#pragma unroll
    for (int w = 0; w < F2_WAVES; ++w) sum += sP[(size_t)w * D * E + (size_t)((c >> 1) * 2 + (c & 1)) * D + i];
    out[idx] = out_scale * sum;
  }
}

static int f2_npt(const egnn_ctx* ctx) { return (ctx->n_paths[0] + 15) / 16; }

// LDS of the kernel: W_r1, two groups of tiles, one partial node row per compute wave
static size_t f2_lds_bytes(const egnn_ctx* ctx) {
  const size_t D = (size_t)(ctx->desc.lmax + 1) * (ctx->desc.lmax + 1);
  return 32 * EGNN_HIDDEN * sizeof(float) + (size_t)2 * f2_npt(ctx) * 32 * F2_BROW4 * sizeof(uint4) +
         (size_t)F2_WAVES * D * ctx->desc.channels * sizeof(float);
}

bool egnn_fused_lane_supported(const egnn_ctx* ctx) {
  const int E = ctx->desc.channels;
  return E >= 8 && (E & (E - 1)) == 0 && ctx->desc.n_rbf <= 32 && f2_lds_bytes(ctx) <= 160 * 1024;
}

static size_t f2_pack_bytes(const egnn_ctx* ctx) {
  return 256 + (size_t)(ctx->desc.channels / 2) * f2_npt(ctx) * 32 * 16 * sizeof(uint4);   // scales, then tiles
}
static size_t f2_align(size_t b) { return (b + 255) & ~(size_t)255; }

// Scratch: the packed tiles of W_r2, then the pair-interleaved copy of h.
size_t egnn_fused_lane_scratch_bytes(const egnn_ctx* ctx, int32_t n_total) {
  const size_t row = (size_t)(ctx->desc.lmax + 1) * (ctx->desc.lmax + 1) * ctx->desc.channels * sizeof(float);
  return f2_align(f2_pack_bytes(ctx)) + f2_align((size_t)n_total * row);
}

// scratch: egnn_fused_lane_scratch_bytes.  a [n_owned][D][E].
int egnn_launch_layer_fused_lane(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* h,
                                 const float* W_r1, const float* W_r2, void* scratch, size_t scratch_bytes, float* a,
                                 hipStream_t stream) {
  const int n = g->n_owned;
  if (n == 0) return EGNN_OK;
  if (!egnn_fused_lane_supported(ctx)) return egnn_fail(ctx, EGNN_EINVAL, "layer_fused_lane: unsupported channel count");
  if (scratch_bytes < egnn_fused_lane_scratch_bytes(ctx, g->n_total))
    return egnn_fail(ctx, EGNN_EWS, "layer_fused_lane: scratch too small");
  const int E = ctx->desc.channels, D = (ctx->desc.lmax + 1) * (ctx->desc.lmax + 1);
  const int npt = f2_npt(ctx), n_tiles = (E / 2) * npt;
  float* scales = reinterpret_cast<float*>(scratch);
  uint4* W2p = reinterpret_cast<uint4*>((char*)scratch + 256);
  float* h2 = reinterpret_cast<float*>((char*)scratch + f2_align(f2_pack_bytes(ctx)));
  PathAlpha al;
  for (int p = 0; p < EGNN_MAX_PATHS; ++p) al.a[p] = p < ctx->n_paths[0] ? ctx->alpha[0][p] : 0.0f;
  {
    const int rc = egnn_launch_half_scales(ctx, 0, W_r1, W_r2, scales, stream);
    if (rc) return rc;
  }
  hipLaunchKernelGGL(f2_pack_kernel, dim3((n_tiles * 32 * 16 + 255) / 256), dim3(256), 0, stream, W_r2, W2p,
                     ctx->n_paths[0], ctx->log2_channels, npt, n_tiles, al, scales);
  EGNN_LAUNCH_CHECK(ctx, "f2_pack_kernel");
  const long n_values = (long)g->n_total * D * E;
  if (n_values > 0) {
    hipLaunchKernelGGL(f2_pair_kernel, dim3((unsigned)((n_values + 255) / 256)), dim3(256), 0, stream, h, h2, n_values, D,
                       ctx->log2_channels);
    EGNN_LAUNCH_CHECK(ctx, "f2_pair_kernel");
  }
  const int per_xcd = (n + 7) / 8;
  const size_t shmem = (size_t)F2_WAVES * D * E * sizeof(float);
  const float scale = 1.0f / sqrtf(ctx->desc.agg_norm);
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
#define LAUNCH(L)                                                                                                   \
  do {                                                                                                              \
    auto kern = f2_kernel<L>;                                                                                       \
    {   /* static + dynamic LDS of this kernel exceed 64 KB */                                                      \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                       \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);                   \
      if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(f2_kernel)");                         \
    }                                                                                                               \
    hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(F2_THREADS), shmem, stream, g->row_ptr, g->src, rd, h2, W_r1,  \
                       W2p, scales, a, n, per_xcd, ctx->desc.n_rbf, ctx->log2_channels, scale, ctx->desc.r_cut);            \
  } while (0)
  switch (ctx->desc.lmax) {
    case 0: LAUNCH(0); break;
    case 1: LAUNCH(1); break;
    case 2: LAUNCH(2); break;
    case 3: LAUNCH(3); break;
    case 4: LAUNCH(4); break;
    default: return egnn_fail(ctx, EGNN_EINVAL, "layer_fused_lane: lmax out of range");
  }
#undef LAUNCH
  EGNN_LAUNCH_CHECK(ctx, "f2_kernel");
  return EGNN_OK;
}
