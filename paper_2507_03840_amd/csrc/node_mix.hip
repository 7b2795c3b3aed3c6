// S5: per-degree channel mix  y[n][(l,m)][:] = W1[l] x1[n][(l,m)][:] (+ W2[l] x2[n][(l,m)][:])
// (the linear layer of Fig. 2(d), one E x E matrix per degree l), and the species embedding of Sec. 3.
//
// Workgroup = (one degree l, a run of rows (node, m)).  W^T sits in LDS so that lanes of consecutive
// output channels read consecutive words; a thread produces ROWS_PER_THREAD rows of one output channel
// and reads the inputs of its rows as LDS broadcasts.
#include "egnn_internal.h"

#define MIX_RPT 4      // rows per thread
#define MIX_TILES 8    // row tiles per workgroup

__global__ __launch_bounds__(256) void node_mix_kernel(const float* __restrict__ x1, const float* __restrict__ W1,
                                                       const float* __restrict__ x2, const float* __restrict__ W2,
                                                       float* __restrict__ y, int n_nodes, int lmax, int log2E) {
  extern __shared__ float smem[];
  const int E = 1 << log2E;
  const int l = blockIdx.y;
  const int D = (lmax + 1) * (lmax + 1);
  const int nm = 2 * l + 1;
  const long n_rows = (long)n_nodes * nm;
  const int rows_per_tile = MIX_RPT * (256 >> log2E);
  const int n_in = W2 ? 2 : 1;
  float* sWt = smem;                              // [n_in][c'][c]
  float* sx = smem + (size_t)n_in * E * E;        // [n_in][rows_per_tile][c'] (+1 padding per row)
  const int xs = E + 1;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1), rg = tid >> log2E;

  for (int i = tid; i < E * E; i += 256) {
    const int co = i >> log2E, ci = i & (E - 1);  // W[l][co][ci]
    sWt[ci * E + co] = W1[(size_t)l * E * E + i];
    if (W2) sWt[E * E + ci * E + co] = W2[(size_t)l * E * E + i];
  }

  for (int t = 0; t < MIX_TILES; ++t) {
    const long r0 = ((long)blockIdx.x * MIX_TILES + t) * rows_per_tile;
    if (r0 >= n_rows) break;
    __syncthreads();
    for (int i = tid; i < rows_per_tile * E; i += 256) {
      const int rr = i >> log2E, ci = i & (E - 1);
      const long r = r0 + rr;
      float v1 = 0.0f, v2 = 0.0f;
      if (r < n_rows) {
        const long node = r / nm;
        const int mm = (int)(r - node * nm);
        const size_t off = (((size_t)node * D + l * l + mm) << log2E) + ci;
        v1 = x1[off];
        if (W2) v2 = x2[off];
      }
      sx[rr * xs + ci] = v1;
      if (W2) sx[(rows_per_tile + rr) * xs + ci] = v2;
    }
    __syncthreads();
    float acc[MIX_RPT];
#pragma unroll
    for (int q = 0; q < MIX_RPT; ++q) acc[q] = 0.0f;
    for (int in = 0; in < n_in; ++in) {
      const float* wt = sWt + (size_t)in * E * E + c;
      const float* xr = sx + (size_t)(in * rows_per_tile + rg * MIX_RPT) * xs;
      for (int ci = 0; ci < E; ++ci) {
        const float wv = wt[ci * E];
#pragma unroll
        for (int q = 0; q < MIX_RPT; ++q) acc[q] += wv * xr[q * xs + ci];
      }
    }
#pragma unroll
    for (int q = 0; q < MIX_RPT; ++q) {
      const long r = r0 + rg * MIX_RPT + q;
      if (r < n_rows) {
        const long node = r / nm;
        const int mm = (int)(r - node * nm);
        y[(((size_t)node * D + l * l + mm) << log2E) + c] = acc[q];
      }
    }
  }
}

int egnn_launch_node_mix(egnn_ctx* ctx, const float* x1, const float* W1, const float* x2, const float* W2,
                         float* y, int n_nodes, hipStream_t stream) {
  if (n_nodes == 0) return EGNN_OK;
  const int E = ctx->desc.channels, lmax = ctx->desc.lmax;
  const int rows_per_tile = MIX_RPT * (256 / E);
  const long max_rows = (long)n_nodes * (2 * lmax + 1);
  const long per_wg = (long)rows_per_tile * MIX_TILES;
  dim3 grid((unsigned)((max_rows + per_wg - 1) / per_wg), lmax + 1), block(256);
  const int n_in = W2 ? 2 : 1;
  const size_t shmem = ((size_t)n_in * E * E + (size_t)n_in * rows_per_tile * (E + 1)) * sizeof(float);
  if (shmem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(node_mix_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(node_mix_kernel)");
  }
  hipLaunchKernelGGL(node_mix_kernel, grid, block, shmem, stream, x1, W1, x2, W2, y, n_nodes, lmax,
                     ctx->log2_channels);
  EGNN_LAUNCH_CHECK(ctx, "node_mix_kernel");
  return EGNN_OK;
}

__global__ void species_embed_kernel(const int* __restrict__ species, const float* __restrict__ table,
                                     float* __restrict__ x, int n_nodes, int n_species, int E, int D) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)n_nodes * E) return;
  const int node = (int)(i / E), c = (int)(i - (long)node * E);
  const int s = species[node];
  if (s >= 0 && s < n_species) x[(size_t)node * D * E + c] += table[s * E + c];
}

extern "C" int egnn_species_embed(egnn_ctx* ctx, const int32_t* species, const float* table, int32_t n_species,
                                  float* x, int32_t n_nodes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!species || !table || !x || n_nodes < 0 || n_species <= 0)
    return egnn_fail(ctx, EGNN_EINVAL, "species_embed: null pointer or bad size");
  if (n_nodes == 0) return EGNN_OK;
  const int E = ctx->desc.channels, D = (ctx->desc.lmax + 1) * (ctx->desc.lmax + 1);
  const long n = (long)n_nodes * E;
  hipLaunchKernelGGL(species_embed_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     species, table, x, n_nodes, n_species, E, D);
  EGNN_LAUNCH_CHECK(ctx, "species_embed_kernel");
  return EGNN_OK;
}
