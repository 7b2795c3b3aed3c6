// S2 (edge geometry) and S3 (radial weights).
//
// S2: r_k = pos[src] + shift*box - pos[dst] evaluated in fp64 from the fp32 inputs, then rounded once;
//     unit vector and length; optionally the real spherical harmonics of the direction (Sec. 2.2), the
//     Gaussian expansion of the length (Sec. 3 "Initialization") and the cosine cutoff.
// S3: w[k][p][c] = fc(d_k) alpha_p (W_r2 SiLU(W_r1 B(d_k)))[p*E + c] -- a dense [n_edges x 64] x [64 x P*E]
//     contraction on the matrix cores, with the 64-wide hidden activation of 64 edges per wavefront held in
//     registers as the A operand for the whole row.
#include "egnn_internal.h"

// ------------------------------------------------------------------------------------------------ S2
template <int LSH>
__device__ __forceinline__ void real_sph_harm_component(float x, float y, float z, float* Y) {
  // Yhat_{l,+-m} = sqrt(2 - delta_m0) sqrt((2l+1)(l-m)!/(l+m)!) Q_l^m(z) {Re,Im}(x+iy)^m,
  // Q_l^m = d^m P_l/dz^m by the three-term recurrence in l.
  float cm = 1.0f, sm = 0.0f;  // Re, Im of (x+iy)^m
  float qmm = 1.0f;            // Q_m^m = (2m-1)!!
#pragma unroll
  for (int m = 0; m <= LSH; ++m) {
    if (m > 0) {
      const float c2 = cm * x - sm * y;
      sm = sm * x + cm * y;
      cm = c2;
      qmm *= (float)(2 * m - 1);
    }
    float q_prev = 0.0f, q = qmm;
#pragma unroll
    for (int l = m; l <= LSH; ++l) {
      if (l > m) {
        const float q_next = ((float)(2 * l - 1) * z * q - (float)(l + m - 1) * q_prev) / (float)(l - m);
        q_prev = q;
        q = q_next;
      }
      // (l-m)!/(l+m)!
      float ratio = 1.0f;
#pragma unroll
      for (int t = l - m + 1; t <= l + m; ++t) ratio /= (float)t;
      const float n = sqrtf((float)(2 * l + 1) * ratio) * (m ? 1.41421356237309515f : 1.0f);
      if (m == 0) {
        Y[l * l + l] = n * q;
      } else {
        Y[l * l + l + m] = n * q * cm;
        Y[l * l + l - m] = n * q * sm;
      }
    }
  }
}

template <int LSH>
__global__ __launch_bounds__(256) void edge_geometry_kernel(const int* __restrict__ src,
                                                            const int* __restrict__ dst,
                                                            const int8_t* __restrict__ shift,
                                                            const float* __restrict__ pos, double bx,
                                                            double by, double bz, long n_edges,
                                                            float4* __restrict__ rhat_d,
                                                            float* __restrict__ Y, float* __restrict__ rbf,
                                                            float* __restrict__ fc, int n_rbf, float r_cut,
                                                            const int* __restrict__ w_row,
                                                            float4* __restrict__ rd_rows) {
  const long k = (long)blockIdx.x * 256 + threadIdx.x;
  if (k >= n_edges) return;
  const int i = src[k], j = dst[k];
  double dx = (double)pos[3 * i + 0] - (double)pos[3 * j + 0];
  double dy = (double)pos[3 * i + 1] - (double)pos[3 * j + 1];
  double dz = (double)pos[3 * i + 2] - (double)pos[3 * j + 2];
  if (shift) {
    dx += (double)shift[3 * k + 0] * bx;
    dy += (double)shift[3 * k + 1] * by;
    dz += (double)shift[3 * k + 2] * bz;
  }
  const double d = sqrt(dx * dx + dy * dy + dz * dz);
  const double inv = 1.0 / d;
  const float x = (float)(dx * inv), y = (float)(dy * inv), z = (float)(dz * inv);
  const float df = (float)d;
  rhat_d[k] = make_float4(x, y, z, df);
  // shared rows of radial weights: the edge that owns a row leaves its record (of which only the length is used) there
  if (rd_rows) {
    const int r = w_row[k];
    if (r >= 0) rd_rows[r] = make_float4(x, y, z, df);
  }
  if (Y) {
    constexpr int NY = (LSH + 1) * (LSH + 1);
    float yy[NY];
    real_sph_harm_component<LSH>(x, y, z, yy);
#pragma unroll
    for (int t = 0; t < NY; ++t) Y[k * NY + t] = yy[t];
  }
  if (rbf) {
    const float step = r_cut / (float)(n_rbf - 1);
    const float inv2s2 = 0.5f / (step * step);
    for (int b = 0; b < n_rbf; ++b) {
      const float u = df - (float)b * step;
      rbf[k * n_rbf + b] = __expf(-u * u * inv2s2);
    }
  }
  if (fc) fc[k] = egnn_envelope(df, r_cut);
}

// rd_rows (may be NULL): [g->n_w_rows] records of the edges that own a row of radial weights (needs g->w_row)
int egnn_launch_geometry(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                         float* rhat_d, float* Y, float* rbf, float* fc, hipStream_t stream, float* rd_rows) {
  const long n = g->n_edges;
  if (n == 0) return EGNN_OK;
  dim3 grid((unsigned)((n + 255) / 256)), block(256);
  float4* rd = reinterpret_cast<float4*>(rhat_d);
  float4* rr = g->w_row ? reinterpret_cast<float4*>(rd_rows) : nullptr;
#define LAUNCH(L)                                                                                          \
  hipLaunchKernelGGL(edge_geometry_kernel<L>, grid, block, 0, stream, g->src, g->dst, g->shift, pos,      \
                     (double)box[0], (double)box[1], (double)box[2], n, rd, Y, rbf, fc, ctx->desc.n_rbf, \
                     ctx->desc.r_cut, g->w_row, rr)
  switch (ctx->desc.lmax_sh) {
    case 0: LAUNCH(0); break;
    case 1: LAUNCH(1); break;
    case 2: LAUNCH(2); break;
    case 3: LAUNCH(3); break;
    case 4: LAUNCH(4); break;
    default: return egnn_fail(ctx, EGNN_EINVAL, "edge_geometry: lmax_sh out of range");
  }
#undef LAUNCH
  EGNN_LAUNCH_CHECK(ctx, "edge_geometry_kernel");
  return EGNN_OK;
}

// ------------------------------------------------------------------------------------------------ S3
// The contraction runs on the half-precision matrix cores with fp32-level accuracy.  Both operands are scaled by a
// power of two and cut into two half-precision pieces of 11 significant bits each (x 2^s = hi + lo to 22 bits, by
// rounding and exact subtraction); a product is hi*hi + hi*lo + lo*hi, accumulated in fp32 -- the dropped lo*lo term
// is 2^-22 of the product, the size of the representation error.  Against fp64 this is as accurate as three bf16
// pieces with six products (largest error 1e-7 of the largest result) and better than a plain fp32 dot product, at
// half the matrix-core work of the former: three v_mfma_f32_32x32x16_f16 replace eight v_mfma_f32_32x32x2_f32 at 1/16
// of their cost each.  Half precision has a narrow exponent range, so the scalings are taken from the weights, on
// the device, once per call (egnn_launch_half_scales): alpha W_r2 by its largest magnitude, the hidden activations by
// the bound |fc SiLU(pre)| <= |pre| <= max_j sum_b |W_r1[j][b]| (basis values and envelope lie in [0, 1]); the
// largest piece then sits in [2^13, 2^14), and the scalings are undone exactly when the result is stored.
#include "split_bf16.h"
#include "w_half.h"

typedef _Float16 rw_h8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ rw_h8 rw_as_h8(uint4 v) { return __builtin_bit_cast(rw_h8, v); }
// x -> (hi, lo) half-precision pieces, as raw bits
__device__ __forceinline__ void rw_split(float x, uint32_t& hi, uint32_t& lo) {
  const _Float16 h = (_Float16)x;
  const _Float16 l = (_Float16)(x - (float)h);
  hi = __builtin_bit_cast(unsigned short, h);
  lo = __builtin_bit_cast(unsigned short, l);
}

// scales[0] = s_w, scales[1] = s_g (powers of two, see above), scales[2] = 1 / (s_w s_g).  One workgroup of 1,024
// threads, 16-byte loads: a few microseconds for the 10^5 values of W_r2.
#define HS_THREADS 1024
__global__ __launch_bounds__(HS_THREADS) void half_scales_kernel(const float* __restrict__ W_r1,
                                                                 const float* __restrict__ W_r2, int n_rbf, int PE,
                                                                 int log2E, PathAlpha alpha, float* __restrict__ scales) {
  __shared__ float red[HS_THREADS];
  float mw = 0.0f;
  const float4* W4 = reinterpret_cast<const float4*>(W_r2);
#pragma unroll 4   // (several loads in flight: the kernel is one workgroup, its time is load latency)
  for (int i = threadIdx.x; i < PE * (EGNN_HIDDEN / 4); i += HS_THREADS) {
    const float4 v = W4[i];
    const float al = fabsf(alpha.a[(i / (EGNN_HIDDEN / 4)) >> log2E]);
    mw = fmaxf(mw, al * fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
  }
  float mg = 0.0f;
  if (threadIdx.x < EGNN_HIDDEN) {
    for (int b = 0; b < n_rbf; ++b) mg += fabsf(W_r1[threadIdx.x * n_rbf + b]);
  }
  auto block_max = [&](float v) {
    red[threadIdx.x] = v;
    __syncthreads();
    for (int st = HS_THREADS / 2; st > 0; st >>= 1) {
      if ((int)threadIdx.x < st) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + st]);
      __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
  };
  mw = block_max(mw);
  mg = block_max(mg);
  if (threadIdx.x == 0) {
    // (zero, infinite or NaN weights: no scaling; the result then shows them as it would without)
    auto exp_of = [](float m) { return (m > 0.0f && m < 3.0e38f) ? ilogbf(m) : 13; };
    int ew = 13 - exp_of(mw), eg = 13 - exp_of(mg);
    ew = ew < -60 ? -60 : (ew > 60 ? 60 : ew);
    eg = eg < -60 ? -60 : (eg > 60 ? 60 : eg);
    scales[0] = ldexpf(1.0f, ew);
    scales[1] = ldexpf(1.0f, eg);
    scales[2] = ldexpf(1.0f, -ew - eg);
  }
}

int egnn_launch_half_scales(egnn_ctx* ctx, int which, const float* W_r1, const float* W_r2, float* scales,
                            hipStream_t stream) {
  const int P = ctx->n_paths[which];
  PathAlpha al;
  for (int p = 0; p < EGNN_MAX_PATHS; ++p) al.a[p] = p < P ? ctx->alpha[which][p] : 0.0f;
  hipLaunchKernelGGL(half_scales_kernel, dim3(1), dim3(HS_THREADS), 0, stream, W_r1, W_r2, ctx->desc.n_rbf,
                     P * ctx->desc.channels, ctx->log2_channels, al, scales);
  EGNN_LAUNCH_CHECK(ctx, "half_scales_kernel");
  return EGNN_OK;
}

// W_r2 (times alpha_p) cut into three bf16 pieces once per call: out[n][piece][64] (operand of the first fused design).
__global__ __launch_bounds__(256) void split_w2_kernel(const float* __restrict__ W_r2, uint16_t* __restrict__ out,
                                                       int PE, int log2E, PathAlpha alpha) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= PE * EGNN_HIDDEN) return;
  const int n = i >> 6, j = i & 63;
  const Split3 s = split3(W_r2[i] * alpha.a[n >> log2E]);
  uint16_t* o = out + (size_t)n * 3 * EGNN_HIDDEN + j;
  o[0] = (uint16_t)(s.hi >> 16);
  o[EGNN_HIDDEN] = (uint16_t)(s.mid >> 16);
  o[2 * EGNN_HIDDEN] = (uint16_t)(s.lo >> 16);
}

// W_r2 times alpha_p times s_w cut into two half-precision pieces: out[n][piece][64].
__global__ __launch_bounds__(256) void split_w2_half_kernel(const float* __restrict__ W_r2, uint16_t* __restrict__ out,
                                                            int PE, int log2E, PathAlpha alpha,
                                                            const float* __restrict__ scales) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= PE * EGNN_HIDDEN) return;
  const int n = i >> 6, j = i & 63;
  uint32_t hi, lo;
  rw_split(W_r2[i] * alpha.a[n >> log2E] * scales[0], hi, lo);
  uint16_t* o = out + (size_t)n * 2 * EGNN_HIDDEN + j;
  o[0] = (uint16_t)hi;
  o[EGNN_HIDDEN] = (uint16_t)lo;
}

// Workgroup = 8 wavefronts (one per register-file slot of a CU at this kernel's register count).  Waves 0-6 each
// own 64 consecutive edges (two 32-row MFMA blocks): lane l serves
// matrix row/column (l & 31) and the half hh = l >> 5 of the 64-long contraction index; MFMA step t contracts
// hidden units 32*hh + 8*t .. +7 on both operands.  Wave 7 only moves data: it copies the pieces of the next
// 32 rows of W_r2 (8 KB, contiguous) from global memory into one of two LDS buffers.
// Why a separate loader: the memory counter of a wave retires loads and stores in issue order, so a wave that
// both loads its next operand and stores its results has to sit out a full HBM write round trip per block.
// The compute waves here never wait on global memory inside the loop -- their operand comes from LDS and their
// stores are fire-and-forget -- and the barriers carry LDS-only fences.
// The output block of 32 columns is contiguous along the channel/path axis of w, i.e. each accumulator
// register is stored as two full 128-byte lines.
#define RW_MB 2                 // 32-row MFMA blocks per compute wave
#define RW_ROWS (32 * RW_MB)
#ifndef RW_COMPUTE_WAVES
#define RW_COMPUTE_WAVES 7
#endif
#ifndef RW_PIPELINE
#define RW_PIPELINE 1
#endif
#ifndef RW_MIN_WG
#define RW_MIN_WG 1
#endif
#define RW_THREADS ((RW_COMPUTE_WAVES + 1) * 64)
#define RW_BROW4 17   // uint4 per staged W_r2 row: 16 of data (2 pieces x 64 halves) + 1 of padding (bank spread)

__device__ __forceinline__ void lds_release_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
}
__device__ __forceinline__ void lds_barrier_acquire() {
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// One 32-column block: wait for its rows of W_r2 in LDS, then 4 steps x 3 piece products per 32-row block.
// STORE: after each step a quarter of the previous block's results (prev, times `unscale`) goes to memory: out_prev
// describes the wave's rows of w, col_prev is the block's first column, lane_off the lane's own offset, ld the row
// stride (w is written once and read once by another kernel: non-temporal stores).
template <bool STORE>
__device__ __forceinline__ void rw_block(const uint4* __restrict__ sB_nb, const uint4 (&a_frag)[RW_MB][2][4], int m,
                                         int hh, float16v (&acc)[RW_MB], const float16v (&prev)[RW_MB],
                                         __amdgpu_buffer_rsrc_t out_prev, int col_prev, unsigned lane_off, size_t ld,
                                         float unscale) {
  lds_barrier_acquire();
  const uint4* row = sB_nb + m * RW_BROW4 + hh * 4;
#pragma unroll
  for (int mb = 0; mb < RW_MB; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[mb][i] = 0.0f;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    // the pieces of W_r2 of this step only (8 registers; the next step's are read while these are multiplied)
    const uint4 b_frag[2] = {row[t], row[8 + t]};
    // smallest terms first: (lo,hi) (hi,lo) (hi,hi)
    const int pa[3] = {1, 0, 0};
    const int pb[3] = {0, 1, 0};
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
      for (int mb = 0; mb < RW_MB; ++mb)
        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rw_as_h8(a_frag[mb][pa[q]][t]), rw_as_h8(b_frag[pb[q]]),
                                                         acc[mb], 0, 0, 0);
    if constexpr (STORE) {
      static_assert(RW_MB == 2, "a quarter of the previous block per contraction step");
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int idx = 8 * t + j, mb = idx >> 4, i = idx & 15;
        // row and block offset (the same for all lanes) added to the lane's own offset: one vector add per store, and
        // the whole offset is what the range check of the buffer sees (rows the wave does not own are discarded)
        const int row_off = ((32 * mb + 8 * (i >> 2) + (i & 3)) * (int)ld + col_prev) * 4;
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, unscale * (float)prev[mb][i]), out_prev,
                                              (int)(lane_off * 4u) + row_off, 0, 2 /* non-temporal */);
      }
    }
  }
  if constexpr (STORE) {
    // keep the stores spread between the matrix-core instructions (the scheduler would otherwise bunch them up)
#ifndef RW_SG_M
#define RW_SG_M 3
#define RW_SG_S 4
#endif
#pragma unroll
    for (int g = 0; g < 24 / RW_SG_M; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x008, RW_SG_M, 0);   // MFMA
      __builtin_amdgcn_sched_group_barrier(0x040, RW_SG_S, 0);   // global stores
    }
  }
}

// HALF: w is stored in half precision (layout of w_half.h), two column blocks per 32-bit word.
template <bool HALF>
__global__ __launch_bounds__(RW_THREADS, RW_MIN_WG) void radial_weights_kernel(const float4* __restrict__ rhat_d, long n_edges,
                                                             const float* __restrict__ W_r1,
                                                             const uint16_t* __restrict__ W2s,
                                                             const float* __restrict__ scales,
                                                             float* __restrict__ w, int n_rbf, int PE,
                                                             float r_cut, int rows_per_wave) {
  __shared__ float sW1[32 * EGNN_HIDDEN];  // [b][j], n_rbf <= 32
  __shared__ uint4 sB[2][32 * RW_BROW4];
  const int tid = threadIdx.x;
  for (int i = tid; i < n_rbf * EGNN_HIDDEN; i += RW_THREADS) {
    const int jj = i & (EGNN_HIDDEN - 1), b = i >> 6;
    sW1[i] = W_r1[jj * n_rbf + b];
  }
  __syncthreads();

  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_blocks = (PE + 31) >> 5;

  if (wave == RW_COMPUTE_WAVES) {
    // ---- loader: block nb -> sB[nb & 1]; rows past the end repeat row 0 (their columns are never stored)
    const uint4* src = reinterpret_cast<const uint4*>(W2s);
    for (int nb = 0; nb < n_blocks; ++nb) {
      uint4 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int u = i * 64 + lane, row = u >> 4, c16 = u & 15;
        const int n = nb * 32 + row;
        v[i] = src[(size_t)(n < PE ? n : 0) * 16 + c16];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int u = i * 64 + lane, row = u >> 4, c16 = u & 15;
        sB[nb & 1][row * RW_BROW4 + c16] = v[i];
      }
      lds_release_barrier();
    }
    return;
  }

  const int m = lane & 31, hh = lane >> 5;
  // a wave owns rows_per_wave <= RW_ROWS consecutive edges (the launch spreads the edges evenly over a whole number
  // of rounds of workgroups); it computes RW_ROWS rows, the surplus ones are its neighbour's and are not stored
  const long e_base = ((long)blockIdx.x * RW_COMPUTE_WAVES + wave) * rows_per_wave;
  const long rows_left = n_edges - e_base;
  const int rows_here = rows_left <= 0 ? 0 : (rows_left < rows_per_wave ? (int)rows_left : rows_per_wave);
  const bool any_row = rows_here > 0;
  const bool all_rows = rows_here == RW_ROWS;

  // A operand: hidden activations (times the cutoff envelope and s_g) of RW_MB x 32 edges, this lane's 32 units, in
  // pieces
  uint4 a_frag[RW_MB][2][4];
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
  const float s_g = scales[1], unscale = scales[2];
#pragma unroll
  for (int mb = 0; mb < RW_MB; ++mb) {
    long e = e_base + mb * 32 + m;
    if (e >= n_edges) e = n_edges - 1;
    const float d = rhat_d[e].w;
    float pre[32];
#pragma unroll
    for (int s = 0; s < 32; ++s) pre[s] = 0.0f;
    for (int b = 0; b < n_rbf; ++b) {
      const float u = d - (float)b * step;
      const float B = __expf(-u * u * inv2s2);
      const float* wrow = sW1 + b * EGNN_HIDDEN + hh * 32;
#pragma unroll
      for (int s = 0; s < 32; ++s) pre[s] += wrow[s] * B;
    }
    const float fc = s_g * egnn_envelope(d, r_cut);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      uint32_t ph[4], pl[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float x0 = pre[8 * t + 2 * q], x1 = pre[8 * t + 2 * q + 1];
        uint32_t h0, l0, h1, l1;
        rw_split(fc * x0 / (1.0f + __expf(-x0)), h0, l0);
        rw_split(fc * x1 / (1.0f + __expf(-x1)), h1, l1);
        ph[q] = h0 | (h1 << 16);
        pl[q] = l0 | (l1 << 16);
      }
      a_frag[mb][0][t] = make_uint4(ph[0], ph[1], ph[2], ph[3]);
      a_frag[mb][1][t] = make_uint4(pl[0], pl[1], pl[2], pl[3]);
    }
  }

  if constexpr (!HALF) {
    // Software-pipelined over column blocks: while the matrix cores work on block nb, the wave stores block nb - 1
    // from a second set of accumulators, a quarter of it after each of the four contraction steps.  Without this all
    // waves of the workgroup (kept in step by the barriers) store at the same time and compute at the same time, and
    // neither the matrix pipes nor the memory pipeline are fed evenly.
    float* const wave_base = w + (size_t)e_base * PE;                    // the same for all lanes
    const unsigned lane_off = (unsigned)(4 * hh * PE + m);
    // The wave's own rows of w as a buffer: a store to a row past them is out of range and discarded by the
    // hardware's range check, so no store needs a per-row test.
    const __amdgpu_buffer_rsrc_t wave_rows =
        __builtin_amdgcn_make_buffer_rsrc((void*)wave_base, 0, rows_here * PE * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t no_rows = wave_rows;
    auto store_block = [&](const float16v (&acc)[RW_MB], int nb) {      // general case: ragged rows / last columns
      if (nb * 32 + m >= PE) return;
#pragma unroll
      for (int mb = 0; mb < RW_MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int r = 32 * mb + 8 * (i >> 2) + (i & 3);               // row relative to e_base + 4*hh
          // (the whole offset in the vector register: that is the part the range check looks at)
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, unscale * (float)acc[mb][i]), wave_rows,
                                                (int)((lane_off + (unsigned)(r * PE + nb * 32)) * 4u), 0, 2);
        }
    };
    // block nb -> acc, block nb - 1 (in prev) -> memory
    auto step = [&](float16v (&acc)[RW_MB], const float16v (&prev)[RW_MB], int nb) {
      const bool fast = nb * 32 <= PE;                                  // block nb - 1 lies wholly inside the row
      if (fast)
        rw_block<true>(sB[nb & 1], a_frag, m, hh, acc, prev, wave_rows, (nb - 1) * 32, lane_off, (size_t)PE, unscale);
      else {
        rw_block<false>(sB[nb & 1], a_frag, m, hh, acc, prev, no_rows, 0, 0, 0, unscale);
        store_block(prev, nb - 1);
      }
    };
#if RW_PIPELINE
    float16v acc0[RW_MB], acc1[RW_MB];
    rw_block<false>(sB[0], a_frag, m, hh, acc0, acc0, no_rows, 0, 0, 0, unscale);
    int nb = 1;
    for (; nb + 1 < n_blocks; nb += 2) {
      step(acc1, acc0, nb);
      step(acc0, acc1, nb + 1);
    }
    if (nb < n_blocks) {
      step(acc1, acc0, nb);
      store_block(acc1, nb);
    } else {
      store_block(acc0, n_blocks - 1);
    }
#else
    (void)step;
    for (int nb = 0; nb < n_blocks; ++nb) {
      float16v acc[RW_MB];
      rw_block<false>(sB[nb & 1], a_frag, m, hh, acc, acc, no_rows, 0, 0, 0, unscale);
      if ((nb + 1) * 32 <= PE) {
#pragma unroll
        for (int mb = 0; mb < RW_MB; ++mb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int row_off = ((32 * mb + 8 * (i >> 2) + (i & 3)) * PE + nb * 32) * 4;
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, unscale * (float)acc[mb][i]), wave_rows,
                                                  (int)(lane_off * 4u) + row_off, 0, 2);
          }
      } else {
        store_block(acc, nb);
      }
    }
#endif
  } else {
    const __amdgpu_buffer_rsrc_t no_rows = __builtin_amdgcn_make_buffer_rsrc((void*)w, 0, 0, 0x00020000);
    const int row_words = w_half_row_words(PE);
    uint32_t* const out_base = reinterpret_cast<uint32_t*>(w) + (size_t)(e_base + 4 * hh) * row_words + m;
    for (int nb = 0; nb < n_blocks; nb += 2) {
      float16v acc[RW_MB];
      uint32_t word[RW_MB][16];
      rw_block<false>(sB[0], a_frag, m, hh, acc, acc, no_rows, 0, 0, 0, unscale);   // nb is even
#pragma unroll
      for (int mb = 0; mb < RW_MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) word[mb][i] = w_half_bits(unscale * acc[mb][i]);
      if (nb + 1 < n_blocks) {                      // (the same for every wave of the workgroup, loader included)
        rw_block<false>(sB[1], a_frag, m, hh, acc, acc, no_rows, 0, 0, 0, unscale);
#pragma unroll
        for (int mb = 0; mb < RW_MB; ++mb)
#pragma unroll
          for (int i = 0; i < 16; ++i) word[mb][i] |= w_half_bits(unscale * acc[mb][i]) << 16;
      }
      // the low half decides: if its column exists the word does (a high half past the end is never read)
      if (nb * 32 + m < PE) {
        uint32_t* out = out_base + (nb >> 1) * 32;
        if (all_rows) {
#pragma unroll
          for (int mb = 0; mb < RW_MB; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i)
              __builtin_nontemporal_store(word[mb][i], out + (size_t)(32 * mb + 8 * (i >> 2) + (i & 3)) * row_words);
        } else if (any_row) {
#pragma unroll
          for (int mb = 0; mb < RW_MB; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int r = 32 * mb + 8 * (i >> 2) + (i & 3);
              if (e_base + 4 * hh + r < n_edges) __builtin_nontemporal_store(word[mb][i], out + (size_t)r * row_words);
            }
        }
      }
    }
  }
}

// room for the pieces of W_r2 in either form: three bf16 pieces per value (384 bytes per row), or 256 bytes of
// scalings and two half-precision pieces (256 bytes per row; P * channels is at least 2)
size_t egnn_radial_ws_bytes(const egnn_ctx* ctx, int which) {
  return (size_t)ctx->n_paths[which] * ctx->desc.channels * 3 * EGNN_HIDDEN * sizeof(uint16_t);
}

// W_r2 * alpha_p -> bf16 pieces [n][3][64] in `scratch` (egnn_radial_ws_bytes).
int egnn_launch_split_w2(egnn_ctx* ctx, int which, const float* W_r2, void* scratch, hipStream_t stream) {
  const int P = ctx->n_paths[which];
  const int PE = P * ctx->desc.channels;
  PathAlpha al;
  for (int p = 0; p < EGNN_MAX_PATHS; ++p) al.a[p] = p < P ? ctx->alpha[which][p] : 0.0f;
  hipLaunchKernelGGL(split_w2_kernel, dim3((PE * EGNN_HIDDEN + 255) / 256), dim3(256), 0, stream, W_r2,
                     (uint16_t*)scratch, PE, ctx->log2_channels, al);
  EGNN_LAUNCH_CHECK(ctx, "split_w2_kernel");
  return EGNN_OK;
}

// `scratch` holds egnn_radial_ws_bytes: the three scalings (256 bytes), then the half-precision pieces of W_r2.
int egnn_launch_radial(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges, const float* W_r1,
                       const float* W_r2, float* w, void* scratch, hipStream_t stream, bool half) {
  if (n_edges == 0) return EGNN_OK;
  const int P = ctx->n_paths[which];
  const int PE = P * ctx->desc.channels;
  float* scales = (float*)scratch;
  uint16_t* W2s = (uint16_t*)((char*)scratch + 256);
  int rc = egnn_launch_half_scales(ctx, which, W_r1, W_r2, scales, stream);
  if (rc) return rc;
  {
    PathAlpha al;
    for (int p = 0; p < EGNN_MAX_PATHS; ++p) al.a[p] = p < P ? ctx->alpha[which][p] : 0.0f;
    hipLaunchKernelGGL(split_w2_half_kernel, dim3((PE * EGNN_HIDDEN + 255) / 256), dim3(256), 0, stream, W_r2, W2s, PE,
                       ctx->log2_channels, al, scales);
    EGNN_LAUNCH_CHECK(ctx, "split_w2_half_kernel");
  }
  // Workgroups: enough for RW_ROWS rows per wave; beyond one round of the 256 CUs their number is rounded up to whole
  // rounds and the edges are spread evenly, so that the last round is as full as the others.
  const long per_wg = (long)RW_ROWS * RW_COMPUTE_WAVES;
  long n_wg = (n_edges + per_wg - 1) / per_wg;
  int rows_per_wave = RW_ROWS;
  if (!half && n_wg > EGNN_CUS) {
    n_wg = (n_wg + EGNN_CUS - 1) / EGNN_CUS * EGNN_CUS;
    rows_per_wave = (int)((n_edges + n_wg * RW_COMPUTE_WAVES - 1) / (n_wg * RW_COMPUTE_WAVES));
  }
  dim3 grid((unsigned)n_wg), block(RW_THREADS);
  if (half)
    hipLaunchKernelGGL(radial_weights_kernel<true>, grid, block, 0, stream, reinterpret_cast<const float4*>(rhat_d),
                       (long)n_edges, W_r1, W2s, scales, w, ctx->desc.n_rbf, PE, ctx->desc.r_cut, rows_per_wave);
  else
    hipLaunchKernelGGL(radial_weights_kernel<false>, grid, block, 0, stream, reinterpret_cast<const float4*>(rhat_d),
                       (long)n_edges, W_r1, W2s, scales, w, ctx->desc.n_rbf, PE, ctx->desc.r_cut, rows_per_wave);
  EGNN_LAUNCH_CHECK(ctx, "radial_weights_kernel");
  return EGNN_OK;
}
