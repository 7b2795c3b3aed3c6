// Reverse pass of S3 (radial weights): gradients of the two MLP matrices from dw[k][p][c].
//
//   w[k][n] = fc_k alpha_n (W_r2 g_k)[n],  g_k = SiLU(pre_k),  pre_k = W_r1 B(d_k),   n = p*E + c
//   dW_r2[n][j] = alpha_n sum_k dw[k][n] G[k][j],                 G = fc * g
//   dpre[k][j]  = S[k][j] * sum_n dw[k][n] alpha_n W_r2[n][j],     S = fc * SiLU'(pre)
//   dW_r1[j][b] = sum_k dpre[k][j] B_b(d_k)
//
// The two large contractions run on the matrix cores with split-bf16 operands like the forward one; sums over edges
// are split into fixed chunks whose partial results are added in a second pass, so the result does not depend on
// scheduling.
#include "egnn_internal.h"
#include "split_bf16.h"
#include "stream_gemm.h"

#define RB_KCHUNK 4096   // edges per partial of dW_r2
#define RB_R1CHUNK 256   // edges per partial of dW_r1 (many short workgroups; the partials are summed in two levels)

__device__ __forceinline__ float rb_basis(float d, int b, float step, float inv2s2) {
  const float u = d - (float)b * step;
  return __expf(-u * u * inv2s2);
}

// G[k][j], S[k][j] for all edges.  Tiles of 64 edges per workgroup: the basis values and the envelope of the tile
// are computed once into LDS, lane j keeps column j of W_r1 in registers and each wave takes 16 of the edges.
// NB8 = number of bases rounded up to a multiple of 8, in eighths: the loops over the bases have compile-time bounds
// (columns past n_rbf hold zeros), so that no branch sits between the LDS reads.
#define RH_EDGES 64
template <int NB8>
__global__ __launch_bounds__(256) void radial_hidden_kernel(const float4* __restrict__ rhat_d, long n_edges,
                                                            const float* __restrict__ W_r1, float* __restrict__ G,
                                                            float* __restrict__ S, int n_rbf, float r_cut,
                                                            const int* __restrict__ skip) {
  if (skip && skip[0]) return;   // (the grid route has taken the call: radial_grid.hip)
  __shared__ float sBas[RH_EDGES][33];
  __shared__ float sFc[RH_EDGES];
  const int tid = threadIdx.x;
  const int j = tid & 63, w = tid >> 6;
  const long k0 = (long)blockIdx.x * RH_EDGES;
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
  constexpr int NB = 8 * NB8;
  for (int i = tid; i < RH_EDGES * NB; i += 256) {
    const int e = i / NB, b = i - e * NB;
    const long k = k0 + e < n_edges ? k0 + e : n_edges - 1;
    sBas[e][b] = b < n_rbf ? rb_basis(rhat_d[k].w, b, step, inv2s2) : 0.0f;
  }
  if (tid < RH_EDGES) {
    const long k = k0 + tid < n_edges ? k0 + tid : n_edges - 1;
    sFc[tid] = egnn_envelope(rhat_d[k].w, r_cut);
  }
  float w1[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) w1[b] = b < n_rbf ? W_r1[j * n_rbf + b] : 0.0f;
  __syncthreads();
#pragma unroll 4
  for (int ee = 0; ee < RH_EDGES / 4; ++ee) {
    const int e = 4 * ee + w;
    const long k = k0 + e;
    float pre = 0.0f;
#pragma unroll
    for (int b = 0; b < NB; ++b) pre += w1[b] * sBas[e][b];
    const float fc = sFc[e];
    const float sig = 1.0f / (1.0f + __expf(-pre));
    if (k < n_edges) {
      G[k * EGNN_HIDDEN + j] = fc * pre * sig;
      S[k * EGNN_HIDDEN + j] = fc * sig * (1.0f + pre * (1.0f - sig));
    }
  }
}

// ---- the two large contractions ------------------------------------------------------------------------------
// Both stream dw (the big operand, read once) against a small operand that every wave needs.  The small operand is
// cut into bf16 pieces beforehand and stored transposed in blocks of 64 contraction indices,
//   T[step][j][piece][64]  (step = contraction index / 64, j = hidden unit),
// which is the order an MFMA B operand is read in; one wave of each workgroup copies the next 24 KB block into one of
// two LDS buffers while the other seven contract (same scheme as the forward kernel: a wave that only computes never
// waits on a store, and the barriers carry LDS-only fences).  dw is cut into pieces on the fly, in registers.
// Six piece products per fp32 product, smallest first: fp32-level accuracy at 6/16 of the fp32-MFMA cost.
// src[r][64] (r < n_rows, times scale[r >> log2E] if scale_on) -> T[r / 64][j][piece][r % 64]; rows past n_rows are 0.
// One workgroup per block of 64 rows; the 64 x 64 tile is turned in LDS so that both sides are contiguous.
__global__ __launch_bounds__(256) void rb_split_transpose_kernel(const float* __restrict__ src, long n_rows,
                                                                 uint16_t* __restrict__ T, int log2E, PathAlpha alpha,
                                                                 int scale_on, const int* __restrict__ skip) {
  if (skip && skip[0]) return;
  __shared__ float tile[64][65];
  const long r0 = (long)blockIdx.x * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int rr = i >> 6, j = i & 63;
    const long r = r0 + rr;
    tile[rr][j] = r < n_rows ? src[r * EGNN_HIDDEN + j] * (scale_on ? alpha.a[r >> log2E] : 1.0f) : 0.0f;
  }
  __syncthreads();
  uint32_t* out = reinterpret_cast<uint32_t*>(T + (size_t)blockIdx.x * 64 * 3 * 64);
  // thread -> (j, pair of rows): three 4-byte stores, consecutive threads write consecutive words of a piece row
  for (int i = threadIdx.x; i < 64 * 32; i += 256) {
    const int j = i >> 5, rp = i & 31;
    const Split3 s0 = split3(tile[2 * rp][j]), s1 = split3(tile[2 * rp + 1][j]);
    uint32_t* o = out + j * 96 + rp;
    o[0] = pack2(s0.hi, s1.hi);
    o[32] = pack2(s0.mid, s1.mid);
    o[64] = pack2(s0.lo, s1.lo);
  }
}

// The same for the half-precision form of the contractions: src[r][64] times scale[0] (a power of two kept in device
// memory) -> T[r / 64][j][piece][r % 64] halves, two pieces (stream_gemm.h).
__global__ __launch_bounds__(256) void rb_split_transpose_half_kernel(const float* __restrict__ src, long n_rows,
                                                                      uint16_t* __restrict__ T, int log2E, PathAlpha alpha,
                                                                      int alpha_on, const float* __restrict__ scale,
                                                                      const int* __restrict__ skip) {
  if (skip && skip[0]) return;
  __shared__ float tile[64][65];
  const long r0 = (long)blockIdx.x * 64;
  const float sc = scale[0];
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int rr = i >> 6, j = i & 63;
    const long r = r0 + rr;
    tile[rr][j] = r < n_rows ? src[r * EGNN_HIDDEN + j] * (alpha_on ? alpha.a[r >> log2E] : 1.0f) : 0.0f;
  }
  __syncthreads();
  uint32_t* out = reinterpret_cast<uint32_t*>(T) + (size_t)blockIdx.x * 64 * 64;
  for (int i = threadIdx.x; i < 64 * 32; i += 256) {
    const int j = i >> 5, rp = i & 31;
    const float xv[8] = {tile[2 * rp][j], tile[2 * rp + 1][j], 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    uint4 hi, lo;
    sgh_split8(xv, sc, hi, lo);
    uint32_t* o = out + j * 64 + rp;
    o[0] = hi.x;
    o[32] = lo.x;
  }
}

// dpre on half-precision pieces: W2T = packed (alpha W_r2 s_w), scales = {s_w, s_g, .}, dw_max = bit pattern of the
// largest |dw|
__global__ __launch_bounds__(SG_THREADS) void radial_dpre_half_kernel(const float* __restrict__ dw, long n_edges,
                                                                      const uint16_t* __restrict__ W2T,
                                                                      float* __restrict__ S, int PE, int n_steps,
                                                                      const float* __restrict__ scales,
                                                                      const unsigned* __restrict__ dw_max,
                                                                      const int* __restrict__ skip) {
  if (skip && skip[0]) return;
  extern __shared__ uint4 rb_smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = lane & 31, hh = lane >> 5;
  const long e_base = ((long)blockIdx.x * SG_WAVES + wave) * 64;
  const int ea = sgh_scale_exp(*dw_max);
  const float a_scale = ldexpf(1.0f, ea), unscale = ldexpf(1.0f, -ea) / scales[0];
  float16v acc[2][2];
  sgh_contract(dw, n_edges, PE, reinterpret_cast<const uint4*>(W2T), n_steps, rb_smem, e_base, a_scale, acc);
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const long e = e_base + rb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
        if (e < n_edges) {
          const size_t at = (size_t)e * EGNN_HIDDEN + cb * 32 + m;
          S[at] = S[at] * (unscale * acc[rb][cb][i]);
        }
      }
}

// dpre[k][j] = S[k][j] * sum_n dw[k][n] alpha_n W_r2[n][j]  (in place over S).  W2T = T of (alpha W_r2), contraction
// index n; the contraction is sg_contract of stream_gemm.h (rows = edges, one 64-column tile = the 64 hidden units).
__global__ __launch_bounds__(SG_THREADS) void radial_dpre_kernel(const float* __restrict__ dw, long n_edges,
                                                                 const uint16_t* __restrict__ W2T,
                                                                 float* __restrict__ S, int PE, int n_steps,
                                                                 const int* __restrict__ skip) {
  if (skip && skip[0]) return;
  extern __shared__ uint4 rb_smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = lane & 31, hh = lane >> 5;
  const long e_base = ((long)blockIdx.x * SG_WAVES + wave) * 64;
  float16v acc[2][2];
  sg_contract(dw, n_edges, PE, reinterpret_cast<const uint4*>(W2T), n_steps, rb_smem, e_base, acc);
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const long e = e_base + rb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
        if (e < n_edges) {
          const size_t at = (size_t)e * EGNN_HIDDEN + cb * 32 + m;
          S[at] = S[at] * acc[rb][cb][i];
        }
      }
}

// Partial dW_r2 over one chunk of RB_KCHUNK edges: partial[chunk][n][j] = alpha_n sum_{k in chunk} dw[k][n] G[k][j].
// GT = T of G, contraction index k.  grid = (tiles of 32 * RB_WAVES rows n, edge chunks); a compute wave owns 32 rows n
// and all 64 units; MFMA step t of a 64-edge step contracts k = 64 s + 32 hh + 8 t .. + 7.
// HALF: GT holds two half-precision pieces of G s_g (scales[1] = s_g), dw is scaled by the power of two that dw_max
// gives before it is cut into two pieces, three products per fp32 product.
template <bool HALF>
__global__ __launch_bounds__(RB_THREADS) void radial_dw2_kernel(const float* __restrict__ dw, long n_edges,
                                                                const uint16_t* __restrict__ GT,
                                                                float* __restrict__ partial, int PE, int log2E,
                                                                PathAlpha alpha, const float* __restrict__ scales,
                                                                const unsigned* __restrict__ dw_max,
                                                                const int* __restrict__ skip) {
  if (skip && skip[0]) return;   // (whole workgroup, before any barrier)
  constexpr int BROW4 = HALF ? SGH_BROW4 : RB_BROW4;
  __shared__ uint4 sB[2 * 64 * BROW4];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  // blockIdx.x = tile of rows n (fastest: the workgroups that read the other columns of the same edges run at the
  // same time, so the rows of dw are fetched whole), blockIdx.y = edge chunk
  const long k_begin = (long)blockIdx.y * RB_KCHUNK;
  long k_end = k_begin + RB_KCHUNK;
  if (k_end > n_edges) k_end = n_edges;
  const int n_steps = (int)((k_end - k_begin + 63) / 64);
  if (wave == RB_WAVES) {
    if constexpr (HALF) rbh_loader(GT, k_begin / 64, n_steps, sB, lane);
    else rb_loader(GT, k_begin / 64, n_steps, sB, lane);
    return;
  }
  float a_scale = 1.0f, unscale = 1.0f;
  if constexpr (HALF) {
    const int ea = sgh_scale_exp(*dw_max);
    a_scale = ldexpf(1.0f, ea);
    unscale = ldexpf(1.0f, -ea) / scales[1];
  }
  const int m = lane & 31, hh = lane >> 5;
  const int n_tile = (blockIdx.x * RB_WAVES + wave) * 32;
  const int n_row = n_tile + m;                       // row of dW_r2 this lane feeds as the A operand
  const bool row_ok = n_row < PE;
  float16v acc[2];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[0][i] = acc[1][i] = 0.0f;

  // The 32 values a lane needs for a step (its half of the 64 edges, one per load) are requested one step ahead
  // into the registers the step before has just cut into pieces: no copy, nothing touched in the step that issues
  // the load.  Row addresses are a uniform part (edge * PE, scalar arithmetic) plus a per-lane offset that never
  // changes.  No masks: rows past the last edge are clamped to it and meet zero rows of GT, rows n >= PE read
  // column 0 and are not stored.
  const unsigned lane_off = (unsigned)(hh * 32) * (unsigned)PE + (unsigned)(row_ok ? n_row : 0);
  const long k_last = n_edges - 1;
  // (a chunk is at most RB_KCHUNK rows of PE floats: far below the 4 GB a descriptor spans)
  const __amdgpu_buffer_rsrc_t chunk_rows = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(dw + (size_t)k_begin * PE), 0, (int)((k_end - k_begin) * PE * 4), 0x00020000);
  float nxt[32];
  auto fetch8 = [&](int s, int t) {
    const long k0 = k_begin + (long)s * 64 + 8 * t;          // (+ 32 hh through lane_off)
    if (k0 + 32 + 7 <= k_last) {                             // the same for all lanes
      // buffer loads: descriptor (the chunk's rows of dw) and row offset in scalar registers, the lane's own
      // offset in one vector register -- no vector arithmetic per load
      const int row0 = s * 64 + 8 * t;
#pragma unroll
      for (int q = 0; q < 8; ++q)
        nxt[8 * t + q] = __builtin_bit_cast(
            float, __builtin_amdgcn_raw_buffer_load_b32(chunk_rows, (int)(lane_off * 4u), (row0 + q) * PE * 4, 0));
    } else {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const long k = k0 + hh * 32 + q;
        nxt[8 * t + q] = dw[(size_t)(k < k_last ? k : k_last) * PE + (row_ok ? n_row : 0)];
      }
    }
  };
#pragma unroll
  for (int t = 0; t < 4; ++t) fetch8(0, t);
  for (int s = 0; s < n_steps; ++s) {
    const int s_next = s + 1 < n_steps ? s + 1 : s;          // (the last step fetches itself again: no branch)
    rb_barrier_acquire();
    const uint4* bbase = sB + (s & 1) * (64 * BROW4) + hh * 4;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      float x[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) x[q] = nxt[8 * t + q];
      if constexpr (HALF) {
        uint4 ah, al;
        sgh_split8(x, a_scale, ah, al);
        fetch8(s_next, t);
        const uint4* brow0 = bbase + m * BROW4 + t;
        const uint4* brow1 = brow0 + 32 * BROW4;
        const uint4 b0[2] = {brow0[0], brow0[8]};
        const uint4 b1[2] = {brow1[0], brow1[8]};
        sgh_mma3x2(ah, al, b0, b1, acc[0], acc[1]);
      } else {
        uint4 ah, am, al;
        rb_split8(x, ah, am, al);
        fetch8(s_next, t);
        const uint4* brow0 = bbase + m * BROW4 + t;
        const uint4* brow1 = brow0 + 32 * BROW4;
        const uint4 b0[3] = {brow0[0], brow0[8], brow0[16]};
        const uint4 b1[3] = {brow1[0], brow1[8], brow1[16]};
        rb_mma6x2(ah, am, al, b0, b1, acc[0], acc[1]);
      }
    }
  }
  float* out = partial + (size_t)blockIdx.y * PE * EGNN_HIDDEN;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int n = n_tile + 8 * (i >> 2) + 4 * hh + (i & 3);
    if (n < PE) {
      const float al = alpha.a[n >> log2E] * unscale;
      out[(size_t)n * EGNN_HIDDEN + m] = al * acc[0][i];
      out[(size_t)n * EGNN_HIDDEN + 32 + m] = al * acc[1][i];
    }
  }
}

// Partial dW_r1: one partial per wavefront and chunk of RB_R1CHUNK edges, the waves of a workgroup independent of
// each other (no workgroup barrier).  Tiles of 32 edges: the basis values of the tile are computed once into the
// wave's own LDS tile (two lanes per edge, half of the bases each), then lane j accumulates hidden unit j against all
// bases, its 32 values of dpre loaded ahead.
#define RB_R1TILE 32
template <int NB8>
__global__ __launch_bounds__(256) void radial_dw1_kernel(const float4* __restrict__ rhat_d, long n_edges,
                                                         const float* __restrict__ dpre, float* __restrict__ partial,
                                                         int n_rbf, float r_cut, const int* __restrict__ skip) {
  if (skip && skip[0]) return;
  __shared__ float sBas_all[4][RB_R1TILE][33];
  const int tid = threadIdx.x;
  const int j = tid & 63, w = tid >> 6;
  float (*sBas)[33] = sBas_all[w];
  const long chunk = (long)blockIdx.x * 4 + w;
  const long k_begin = chunk * RB_R1CHUNK;
  if (k_begin >= n_edges) return;                    // (whole wave; no workgroup barrier below)
  long k_end = k_begin + RB_R1CHUNK;
  if (k_end > n_edges) k_end = n_edges;
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
  constexpr int NB = 8 * NB8;
  const int be = j & 31, bhalf = j >> 5;
  float acc[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) acc[b] = 0.0f;
  for (long k0 = k_begin; k0 < k_end; k0 += RB_R1TILE) {
    float dp[RB_R1TILE];
#pragma unroll
    for (int e = 0; e < RB_R1TILE; ++e) dp[e] = k0 + e < k_end ? dpre[(k0 + e) * EGNN_HIDDEN + j] : 0.0f;
    {
      const long k = k0 + be;
      const float d = rhat_d[k < k_end ? k : k_end - 1].w;
#pragma unroll
      for (int bb = 0; bb < NB / 2; ++bb) {
        const int b = bhalf * (NB / 2) + bb;
        sBas[be][b] = (k < k_end && b < n_rbf) ? rb_basis(d, b, step, inv2s2) : 0.0f;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
#pragma unroll
    for (int e = 0; e < RB_R1TILE; ++e) {
#pragma unroll
      for (int b = 0; b < NB; ++b) acc[b] += dp[e] * sBas[e][b];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();                 // reads of the tile are over before the next one is written
  }
  float* out = partial + (size_t)chunk * EGNN_HIDDEN * n_rbf + (size_t)j * n_rbf;
#pragma unroll
  for (int b = 0; b < NB; ++b)
    if (b < n_rbf) out[b] = acc[b];
}

static size_t a256(size_t n) { return (n + 255) & ~(size_t)255; }
static size_t rb_pad64(size_t n) { return (n + 63) & ~(size_t)63; }

static size_t rb_exact_ws_bytes(const egnn_ctx* ctx, int which, int64_t n_edges) {
  const size_t PE = (size_t)ctx->n_paths[which] * ctx->desc.channels;
  const size_t kc = (size_t)((n_edges + RB_KCHUNK - 1) / RB_KCHUNK), rc = (size_t)((n_edges + RB_R1CHUNK - 1) / RB_R1CHUNK);
  // (the first 512 bytes: the running maximum of |dw| and the scalings of the half-precision form)
  return 512 + 2 * a256((size_t)n_edges * EGNN_HIDDEN * 4) + a256(kc * PE * EGNN_HIDDEN * 4) +
         a256(rc * EGNN_HIDDEN * ctx->desc.n_rbf * 4) + a256(rb_pad64(PE) * EGNN_HIDDEN * 6) +
         a256(rb_pad64(n_edges) * EGNN_HIDDEN * 6);
}

// the exact route's buffers, then the grid route's (radial_grid.hip): which of the two runs is decided on the device
size_t egnn_radial_backward_ws_bytes(const egnn_ctx* ctx, int which, int64_t n_edges) {
  return rb_exact_ws_bytes(ctx, which, n_edges) + egnn_radial_grid_ws_bytes(ctx, which, n_edges);
}

// G and S at the given edge records (for the grid route: the records of its grid points)
static int rb_launch_hidden(egnn_ctx* ctx, const float* rhat_d, long n, const float* W_r1, float* G, float* S,
                            hipStream_t st) {
  const int n_rbf = ctx->desc.n_rbf, nb8 = (n_rbf + 7) / 8;
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
  const dim3 grid((unsigned)((n + RH_EDGES - 1) / RH_EDGES));
  const int* never = nullptr;
  switch (nb8) {
    case 1: hipLaunchKernelGGL(radial_hidden_kernel<1>, grid, dim3(256), 0, st, rd, n, W_r1, G, S, n_rbf, ctx->desc.r_cut, never); break;
    case 2: hipLaunchKernelGGL(radial_hidden_kernel<2>, grid, dim3(256), 0, st, rd, n, W_r1, G, S, n_rbf, ctx->desc.r_cut, never); break;
    case 3: hipLaunchKernelGGL(radial_hidden_kernel<3>, grid, dim3(256), 0, st, rd, n, W_r1, G, S, n_rbf, ctx->desc.r_cut, never); break;
    default: hipLaunchKernelGGL(radial_hidden_kernel<4>, grid, dim3(256), 0, st, rd, n, W_r1, G, S, n_rbf, ctx->desc.r_cut, never); break;
  }
  EGNN_LAUNCH_CHECK(ctx, "radial_hidden_kernel(grid points)");
  return EGNN_OK;
}

int egnn_launch_radial_backward(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges, const float* W_r1,
                                const float* W_r2, const float* dw, float* dW_r1, float* dW_r2, void* ws,
                                bool dw_max_valid, hipStream_t st, const int* len_ptr, const int* len_perm) {
  const int P = ctx->n_paths[which];
  const int PE = P * ctx->desc.channels, n_rbf = ctx->desc.n_rbf;
  int rc;
  if (n_edges == 0) {
    if ((rc = egnn_launch_reduce_partials(ctx, nullptr, 0, (long)PE * EGNN_HIDDEN, dW_r2, 1.0f, st))) return rc;
    return egnn_launch_reduce_partials(ctx, nullptr, 0, (long)EGNN_HIDDEN * n_rbf, dW_r1, 1.0f, st);
  }
  PathAlpha al;
  for (int p = 0; p < EGNN_MAX_PATHS; ++p) al.a[p] = p < P ? ctx->alpha[which][p] : 0.0f;
  const int kc = (int)((n_edges + RB_KCHUNK - 1) / RB_KCHUNK), r1c = (int)((n_edges + RB_R1CHUNK - 1) / RB_R1CHUNK);
  const unsigned* dw_max = egnn_radial_backward_dw_max(ws);
  float* scales = (float*)((char*)ws + 256);
  // Which route computes the gradients is decided on the device from W_r1 (or forced by EGNN_OPT_RADIAL_BWD): the
  // kernels of both are enqueued, those of the route that is not taken return at once.
  int* route = (int*)((char*)ws + 384);
  if ((rc = egnn_launch_radial_route(ctx, W_r1, route, st))) return rc;
  const int* skip = route;
  const bool half = dw_max_valid;
  char* base = (char*)ws + 512;
  float* G = (float*)base;
  float* S = (float*)(base + a256((size_t)n_edges * EGNN_HIDDEN * 4));
  float* part2 = (float*)(base + 2 * a256((size_t)n_edges * EGNN_HIDDEN * 4));
  float* part1 = (float*)((char*)part2 + a256((size_t)kc * PE * EGNN_HIDDEN * 4));
  uint16_t* W2T = (uint16_t*)((char*)part1 + a256((size_t)r1c * EGNN_HIDDEN * n_rbf * 4));
  uint16_t* GT = (uint16_t*)((char*)W2T + a256(rb_pad64(PE) * EGNN_HIDDEN * 6));
  const long pe_pad = (long)rb_pad64(PE), ne_pad = (long)rb_pad64(n_edges);
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
  const int nb8 = (n_rbf + 7) / 8;   // 1 .. 4 (n_rbf <= 32)
#define RB_BY_NB8(KERNEL, GRID, ...)                                                                 \
  switch (nb8) {                                                                                     \
    case 1: hipLaunchKernelGGL(KERNEL<1>, GRID, dim3(256), 0, st, __VA_ARGS__); break;               \
    case 2: hipLaunchKernelGGL(KERNEL<2>, GRID, dim3(256), 0, st, __VA_ARGS__); break;               \
    case 3: hipLaunchKernelGGL(KERNEL<3>, GRID, dim3(256), 0, st, __VA_ARGS__); break;               \
    default: hipLaunchKernelGGL(KERNEL<4>, GRID, dim3(256), 0, st, __VA_ARGS__); break;              \
  }
  RB_BY_NB8(radial_hidden_kernel, dim3((unsigned)((n_edges + RH_EDGES - 1) / RH_EDGES)), rd, (long)n_edges, W_r1, G, S,
            n_rbf, ctx->desc.r_cut, skip);
  EGNN_LAUNCH_CHECK(ctx, "radial_hidden_kernel");
  const int n_tile = 32 * RB_WAVES;
  const long per_wg = 64L * SG_WAVES;
  const dim3 dw2_grid((PE + n_tile - 1) / n_tile, kc), dpre_grid((unsigned)((n_edges + per_wg - 1) / per_wg));
  if (half) {
    // two half-precision pieces per operand, three products: G and alpha W_r2 are scaled by the powers of two that
    // egnn_launch_half_scales derives from the weights, dw by the one its running maximum gives
    if ((rc = egnn_launch_half_scales(ctx, which, W_r1, W_r2, scales, st))) return rc;
    hipLaunchKernelGGL(rb_split_transpose_half_kernel, dim3((unsigned)(ne_pad / 64)), dim3(256), 0, st, G, (long)n_edges,
                       GT, 0, al, 0, scales + 1, skip);
    EGNN_LAUNCH_CHECK(ctx, "rb_split_transpose_half_kernel(G)");
    hipLaunchKernelGGL(rb_split_transpose_half_kernel, dim3((unsigned)(pe_pad / 64)), dim3(256), 0, st, W_r2, (long)PE,
                       W2T, ctx->log2_channels, al, 1, scales, skip);
    EGNN_LAUNCH_CHECK(ctx, "rb_split_transpose_half_kernel(W_r2)");
    hipLaunchKernelGGL(radial_dw2_kernel<true>, dw2_grid, dim3(RB_THREADS), 0, st, dw, (long)n_edges, GT, part2, PE,
                       ctx->log2_channels, al, scales, dw_max, skip);
    EGNN_LAUNCH_CHECK(ctx, "radial_dw2_kernel");
    if ((rc = egnn_launch_reduce_partials(ctx, part2, kc, (long)PE * EGNN_HIDDEN, dW_r2, 1.0f, st, skip))) return rc;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(radial_dpre_half_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)SGH_LDS_BYTES);
    if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(radial_dpre_half_kernel)");
    hipLaunchKernelGGL(radial_dpre_half_kernel, dpre_grid, dim3(SG_THREADS), SGH_LDS_BYTES, st, dw, (long)n_edges, W2T, S,
                       PE, (int)(pe_pad / 64), scales, dw_max, skip);
    EGNN_LAUNCH_CHECK(ctx, "radial_dpre_half_kernel");
  } else {
    hipLaunchKernelGGL(rb_split_transpose_kernel, dim3((unsigned)(ne_pad / 64)), dim3(256), 0, st, G, (long)n_edges, GT, 0,
                       al, 0, skip);
    EGNN_LAUNCH_CHECK(ctx, "rb_split_transpose_kernel(G)");
    hipLaunchKernelGGL(rb_split_transpose_kernel, dim3((unsigned)(pe_pad / 64)), dim3(256), 0, st, W_r2, (long)PE, W2T,
                       ctx->log2_channels, al, 1, skip);
    EGNN_LAUNCH_CHECK(ctx, "rb_split_transpose_kernel(W_r2)");
    hipLaunchKernelGGL(radial_dw2_kernel<false>, dw2_grid, dim3(RB_THREADS), 0, st, dw, (long)n_edges, GT, part2, PE,
                       ctx->log2_channels, al, scales, dw_max, skip);
    EGNN_LAUNCH_CHECK(ctx, "radial_dw2_kernel");
    if ((rc = egnn_launch_reduce_partials(ctx, part2, kc, (long)PE * EGNN_HIDDEN, dW_r2, 1.0f, st, skip))) return rc;
    const size_t dpre_lds = SG_LDS_BYTES;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(radial_dpre_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)dpre_lds);
    if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(radial_dpre_kernel)");
    hipLaunchKernelGGL(radial_dpre_kernel, dpre_grid, dim3(SG_THREADS), dpre_lds, st, dw, (long)n_edges, W2T, S, PE,
                       (int)(pe_pad / 64), skip);
    EGNN_LAUNCH_CHECK(ctx, "radial_dpre_kernel");
  }
  RB_BY_NB8(radial_dw1_kernel, dim3((r1c + 3) / 4), rd, (long)n_edges, S, part1, n_rbf, ctx->desc.r_cut, skip);
#undef RB_BY_NB8
  EGNN_LAUNCH_CHECK(ctx, "radial_dw1_kernel");
  if ((rc = egnn_launch_reduce_partials(ctx, part1, r1c, (long)EGNN_HIDDEN * n_rbf, dW_r1, 1.0f, st, skip))) return rc;
  // the grid route (its kernels run only if route[0] is 1)
  return egnn_launch_radial_grid(ctx, which, rhat_d, n_edges, len_ptr, len_perm, W_r1, W_r2, dw, dW_r1, dW_r2,
                                 (char*)ws + rb_exact_ws_bytes(ctx, which, n_edges), route, rb_launch_hidden, st);
}
