// S2 (edge geometry) and S3 (radial weights).
//
// S2: r_k = pos[src] + shift*box - pos[dst] evaluated in fp64 from the fp32 inputs, then rounded once;
//     unit vector and length; optionally the real spherical harmonics of the direction (Sec. 2.2), the
//     Gaussian expansion of the length (Sec. 3 "Initialization") and the cosine cutoff.
// S3: w[k][p][c] = fc(d_k) alpha_p (W_r2 SiLU(W_r1 B(d_k)))[p*E + c] -- a dense [n_edges x 64] x [64 x P*E]
//     contraction, done on the fp32 matrix cores (v_mfma_f32_32x32x2_f32) with the 64-wide hidden
//     activation of 64 edges per wavefront held in registers as the A operand for the whole row.
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
                                                            float* __restrict__ fc, int n_rbf, float r_cut) {
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
  if (fc) fc[k] = 0.5f * (1.0f + cosf(3.14159265358979323846f * df / r_cut));
}

int egnn_launch_geometry(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                         float* rhat_d, float* Y, float* rbf, float* fc, hipStream_t stream) {
  const long n = g->n_edges;
  if (n == 0) return EGNN_OK;
  dim3 grid((unsigned)((n + 255) / 256)), block(256);
  float4* rd = reinterpret_cast<float4*>(rhat_d);
#define LAUNCH(L)                                                                                          \
  hipLaunchKernelGGL(edge_geometry_kernel<L>, grid, block, 0, stream, g->src, g->dst, g->shift, pos,      \
                     (double)box[0], (double)box[1], (double)box[2], n, rd, Y, rbf, fc, ctx->desc.n_rbf, \
                     ctx->desc.r_cut)
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
typedef float float16v __attribute__((ext_vector_type(16)));

// Workgroup = 4 wavefronts, each owning 64 consecutive edges (two 32-row MFMA blocks).  Lane l serves
// matrix row/column (l & 31) and the half hh = l >> 5 of the 64-long contraction index: the k-th
// MFMA of a block contracts hidden units {s, 32 + s}, so a lane reads 32 consecutive floats of a W_r2
// row.  The output block of 32 columns is contiguous along the channel/path axis of w, i.e. each
// accumulator register is stored as two full 128-byte lines.
__global__ __launch_bounds__(256) void radial_weights_kernel(const float4* __restrict__ rhat_d, long n_edges,
                                                             const float* __restrict__ W_r1,
                                                             const float* __restrict__ W_r2,
                                                             float* __restrict__ w, int n_rbf, int PE,
                                                             int log2E, float r_cut, PathAlpha alpha) {
  __shared__ float sW1[32 * EGNN_HIDDEN];  // [b][j], n_rbf <= 32
  const int tid = threadIdx.x;
  for (int i = tid; i < n_rbf * EGNN_HIDDEN; i += 256) {
    const int jj = i & (EGNN_HIDDEN - 1), b = i >> 6;
    sW1[i] = W_r1[jj * n_rbf + b];
  }
  __syncthreads();

  const int lane = tid & 63, wave = tid >> 6;
  const int m = lane & 31, hh = lane >> 5;
  const long e_base = ((long)blockIdx.x * 4 + wave) * 64;
  if (e_base >= n_edges) return;

  // A operand: hidden activations (times the cutoff envelope) of 2 x 32 edges, this lane's 32 units
  float a_frag[2][32];
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
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
    const float fc = 0.5f * (1.0f + cosf(3.14159265358979323846f * d / r_cut));
#pragma unroll
    for (int s = 0; s < 32; ++s) a_frag[mb][s] = fc * pre[s] / (1.0f + __expf(-pre[s]));
  }

  const int n_blocks = (PE + 31) >> 5;
  for (int nb = 0; nb < n_blocks; ++nb) {
    const int n = nb * 32 + m;
    const bool col_ok = n < PE;
    float b_frag[32];
    if (col_ok) {
      const float al = alpha.a[n >> log2E];
      const float4* row = reinterpret_cast<const float4*>(W_r2 + (size_t)n * EGNN_HIDDEN + hh * 32);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float4 t = row[q];
        b_frag[4 * q + 0] = t.x * al;
        b_frag[4 * q + 1] = t.y * al;
        b_frag[4 * q + 2] = t.z * al;
        b_frag[4 * q + 3] = t.w * al;
      }
    } else {
#pragma unroll
      for (int s = 0; s < 32; ++s) b_frag[s] = 0.0f;
    }
    float16v acc0 = {0}, acc1 = {0};
#pragma unroll
    for (int s = 0; s < 32; ++s) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a_frag[0][s], b_frag[s], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a_frag[1][s], b_frag[s], acc1, 0, 0, 0);
    }
    if (col_ok) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int r = 8 * (i >> 2) + 4 * hh + (i & 3);
        const long e0 = e_base + r, e1 = e_base + 32 + r;
        if (e0 < n_edges) w[(size_t)e0 * PE + n] = acc0[i];
        if (e1 < n_edges) w[(size_t)e1 * PE + n] = acc1[i];
      }
    }
  }
}

int egnn_launch_radial(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges, const float* W_r1,
                       const float* W_r2, float* w, hipStream_t stream) {
  if (n_edges == 0) return EGNN_OK;
  const int P = ctx->n_paths[which];
  const int PE = P * ctx->desc.channels;
  PathAlpha al;
  for (int p = 0; p < EGNN_MAX_PATHS; ++p) al.a[p] = p < P ? ctx->alpha[which][p] : 0.0f;
  dim3 grid((unsigned)((n_edges + 255) / 256)), block(256);
  hipLaunchKernelGGL(radial_weights_kernel, grid, block, 0, stream, reinterpret_cast<const float4*>(rhat_d),
                     (long)n_edges, W_r1, W_r2, w, ctx->desc.n_rbf, PE, ctx->log2_channels, ctx->desc.r_cut, al);
  EGNN_LAUNCH_CHECK(ctx, "radial_weights_kernel");
  return EGNN_OK;
}
