// Reverse pass of S3 (radial weights): gradients of the two MLP matrices from dw[k][p][c].
//
//   w[k][n] = fc_k alpha_n (W_r2 g_k)[n],  g_k = SiLU(pre_k),  pre_k = W_r1 B(d_k),   n = p*E + c
//   dW_r2[n][j] = alpha_n sum_k dw[k][n] G[k][j],                 G = fc * g
//   dpre[k][j]  = S[k][j] * sum_n dw[k][n] alpha_n W_r2[n][j],     S = fc * SiLU'(pre)
//   dW_r1[j][b] = sum_k dpre[k][j] B_b(d_k)
//
// The two large contractions run on the fp32 matrix cores like the forward one; sums over edges are split into
// fixed chunks whose partial results are added in a second pass, so the result does not depend on scheduling.
#include "egnn_internal.h"

typedef float float16v __attribute__((ext_vector_type(16)));
#define RB_KCHUNK 4096   // edges per partial of dW_r2
#define RB_R1CHUNK 1024  // edges per partial of dW_r1

__device__ __forceinline__ float rb_basis(float d, int b, float step, float inv2s2) {
  const float u = d - (float)b * step;
  return __expf(-u * u * inv2s2);
}

// G[k][j], S[k][j] for all edges: 4 edges per workgroup, one hidden unit per lane.
__global__ __launch_bounds__(256) void radial_hidden_kernel(const float4* __restrict__ rhat_d, long n_edges,
                                                            const float* __restrict__ W_r1, float* __restrict__ G,
                                                            float* __restrict__ S, int n_rbf, float r_cut) {
  __shared__ float sW1[32 * EGNN_HIDDEN];
  const int tid = threadIdx.x;
  for (int i = tid; i < n_rbf * EGNN_HIDDEN; i += 256) sW1[(i % n_rbf) * EGNN_HIDDEN + i / n_rbf] = W_r1[i];
  __syncthreads();
  const long k = (long)blockIdx.x * 4 + (tid >> 6);
  if (k >= n_edges) return;
  const int j = tid & 63;
  const float d = rhat_d[k].w;
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
  float pre = 0.0f;
  for (int b = 0; b < n_rbf; ++b) pre += sW1[b * EGNN_HIDDEN + j] * rb_basis(d, b, step, inv2s2);
  const float fc = 0.5f * (1.0f + cosf(3.14159265358979323846f * d / r_cut));
  const float sig = 1.0f / (1.0f + __expf(-pre));
  G[k * EGNN_HIDDEN + j] = fc * pre * sig;
  S[k * EGNN_HIDDEN + j] = fc * sig * (1.0f + pre * (1.0f - sig));
}

// dpre[k][j] = S[k][j] * sum_n dw[k][n] alpha_n W_r2[n][j]  (in place over S).  One wavefront: 64 edges x 64 units.
__global__ __launch_bounds__(256) void radial_dpre_kernel(const float* __restrict__ dw, long n_edges,
                                                          const float* __restrict__ W_r2, float* __restrict__ S,
                                                          int PE, int log2E, PathAlpha alpha) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int m = lane & 31, hh = lane >> 5;
  const long e_base = ((long)blockIdx.x * 4 + wave) * 64;
  if (e_base >= n_edges) return;
  long e_row[2];
  e_row[0] = e_base + m < n_edges ? e_base + m : n_edges - 1;
  e_row[1] = e_base + 32 + m < n_edges ? e_base + 32 + m : n_edges - 1;
  float16v acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

  for (int n0 = 0; n0 < PE; n0 += 64) {
    float a_frag[2][32], b_frag[2][32];
    const int nl = n0 + 32 * hh;   // first contraction index of this lane half
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const float4* row = reinterpret_cast<const float4*>(dw + (size_t)e_row[mb] * PE + nl);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (nl + 4 * q < PE) t = row[q];
        a_frag[mb][4 * q + 0] = t.x;
        a_frag[mb][4 * q + 1] = t.y;
        a_frag[mb][4 * q + 2] = t.z;
        a_frag[mb][4 * q + 3] = t.w;
      }
    }
#pragma unroll
    for (int s = 0; s < 32; ++s) {
      const int n = nl + s;
      float b0 = 0.0f, b1 = 0.0f;
      if (n < PE) {
        const float al = alpha.a[n >> log2E];
        b0 = al * W_r2[(size_t)n * EGNN_HIDDEN + m];
        b1 = al * W_r2[(size_t)n * EGNN_HIDDEN + 32 + m];
      }
      b_frag[0][s] = b0;
      b_frag[1][s] = b1;
    }
#pragma unroll
    for (int s = 0; s < 32; ++s) {
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_frag[0][s], b_frag[0][s], acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_frag[0][s], b_frag[1][s], acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_frag[1][s], b_frag[0][s], acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_frag[1][s], b_frag[1][s], acc[1][1], 0, 0, 0);
    }
  }
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const long e = e_base + mb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
        if (e < n_edges) {
          const size_t at = (size_t)e * EGNN_HIDDEN + nb * 32 + m;
          S[at] = S[at] * acc[mb][nb][i];
        }
      }
}

// Partial dW_r2 over one chunk of edges: grid = (edge chunks, tiles of 128 rows n); wave = 32 rows x 64 units.
__global__ __launch_bounds__(256) void radial_dw2_kernel(const float* __restrict__ dw, long n_edges,
                                                         const float* __restrict__ G, float* __restrict__ partial,
                                                         int PE, int log2E, PathAlpha alpha) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int m = lane & 31, hh = lane >> 5;
  const int n_row = (blockIdx.y * 4 + wave) * 32 + m;     // row of dW_r2 this lane feeds as the A operand
  if ((blockIdx.y * 4 + wave) * 32 >= PE) return;
  const bool row_ok = n_row < PE;
  const long k_begin = (long)blockIdx.x * RB_KCHUNK;
  long k_end = k_begin + RB_KCHUNK;
  if (k_end > n_edges) k_end = n_edges;
  float16v acc0, acc1;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc0[i] = acc1[i] = 0.0f;
  for (long k0 = k_begin; k0 < k_end; k0 += 64) {
    float a_frag[32], b0[32], b1[32];
#pragma unroll
    for (int s = 0; s < 32; ++s) {
      const long k = k0 + 32 * hh + s;
      const bool ok = k < k_end;
      a_frag[s] = (ok && row_ok) ? dw[(size_t)k * PE + n_row] : 0.0f;
      b0[s] = ok ? G[(size_t)k * EGNN_HIDDEN + m] : 0.0f;
      b1[s] = ok ? G[(size_t)k * EGNN_HIDDEN + 32 + m] : 0.0f;
    }
#pragma unroll
    for (int s = 0; s < 32; ++s) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a_frag[s], b0[s], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a_frag[s], b1[s], acc1, 0, 0, 0);
    }
  }
  float* out = partial + (size_t)blockIdx.x * PE * EGNN_HIDDEN;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int n = (blockIdx.y * 4 + wave) * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
    if (n < PE) {
      const float al = alpha.a[n >> log2E];
      out[(size_t)n * EGNN_HIDDEN + m] = al * acc0[i];
      out[(size_t)n * EGNN_HIDDEN + 32 + m] = al * acc1[i];
    }
  }
}

// Partial dW_r1 over one chunk of edges: thread = (hidden unit j, group of 8 basis functions).
__global__ __launch_bounds__(256) void radial_dw1_kernel(const float4* __restrict__ rhat_d, long n_edges,
                                                         const float* __restrict__ dpre, float* __restrict__ partial,
                                                         int n_rbf, float r_cut) {
  const int tid = threadIdx.x;
  const int j = tid & 63, bg = tid >> 6;
  const long k_begin = (long)blockIdx.x * RB_R1CHUNK;
  long k_end = k_begin + RB_R1CHUNK;
  if (k_end > n_edges) k_end = n_edges;
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
  float acc[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) acc[q] = 0.0f;
  for (long k = k_begin; k < k_end; ++k) {
    const float d = rhat_d[k].w;
    const float dp = dpre[k * EGNN_HIDDEN + j];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int b = bg * 8 + q;
      if (b < n_rbf) acc[q] += dp * rb_basis(d, b, step, inv2s2);
    }
  }
  float* out = partial + (size_t)blockIdx.x * EGNN_HIDDEN * n_rbf;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int b = bg * 8 + q;
    if (b < n_rbf) out[j * n_rbf + b] = acc[q];
  }
}

static size_t a256(size_t n) { return (n + 255) & ~(size_t)255; }

size_t egnn_radial_backward_ws_bytes(const egnn_ctx* ctx, int which, int64_t n_edges) {
  const size_t PE = (size_t)ctx->n_paths[which] * ctx->desc.channels;
  const size_t kc = (size_t)((n_edges + RB_KCHUNK - 1) / RB_KCHUNK), rc = (size_t)((n_edges + RB_R1CHUNK - 1) / RB_R1CHUNK);
  return 2 * a256((size_t)n_edges * EGNN_HIDDEN * 4) + a256(kc * PE * EGNN_HIDDEN * 4) +
         a256(rc * EGNN_HIDDEN * ctx->desc.n_rbf * 4);
}

int egnn_launch_radial_backward(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges, const float* W_r1,
                                const float* W_r2, const float* dw, float* dW_r1, float* dW_r2, void* ws,
                                hipStream_t st) {
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
  char* base = (char*)ws;
  float* G = (float*)base;
  float* S = (float*)(base + a256((size_t)n_edges * EGNN_HIDDEN * 4));
  float* part2 = (float*)(base + 2 * a256((size_t)n_edges * EGNN_HIDDEN * 4));
  float* part1 = (float*)((char*)part2 + a256((size_t)kc * PE * EGNN_HIDDEN * 4));
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
  hipLaunchKernelGGL(radial_hidden_kernel, dim3((unsigned)((n_edges + 3) / 4)), dim3(256), 0, st, rd, (long)n_edges,
                     W_r1, G, S, n_rbf, ctx->desc.r_cut);
  EGNN_LAUNCH_CHECK(ctx, "radial_hidden_kernel");
  hipLaunchKernelGGL(radial_dw2_kernel, dim3(kc, (PE + 127) / 128), dim3(256), 0, st, dw, (long)n_edges, G, part2, PE,
                     ctx->log2_channels, al);
  EGNN_LAUNCH_CHECK(ctx, "radial_dw2_kernel");
  if ((rc = egnn_launch_reduce_partials(ctx, part2, kc, (long)PE * EGNN_HIDDEN, dW_r2, 1.0f, st))) return rc;
  hipLaunchKernelGGL(radial_dpre_kernel, dim3((unsigned)((n_edges + 255) / 256)), dim3(256), 0, st, dw, (long)n_edges,
                     W_r2, S, PE, ctx->log2_channels, al);
  EGNN_LAUNCH_CHECK(ctx, "radial_dpre_kernel");
  hipLaunchKernelGGL(radial_dw1_kernel, dim3(r1c), dim3(256), 0, st, rd, (long)n_edges, S, part1, n_rbf,
                     ctx->desc.r_cut);
  EGNN_LAUNCH_CHECK(ctx, "radial_dw1_kernel");
  return egnn_launch_reduce_partials(ctx, part1, r1c, (long)EGNN_HIDDEN * n_rbf, dW_r1, 1.0f, st);
}
