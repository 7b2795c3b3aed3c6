// S5: per-degree channel mix  y[n][(l,m)][:] = W1[l] x1[n][(l,m)][:] (+ W2[l] x2[n][(l,m)][:])
// (the linear layer of Fig. 2(d), one E x E matrix per degree l), and the species embedding of Sec. 3.
//
// Two implementations.  32 and 64 channels: fp32 MFMA (node_mix_mfma_kernel below).  Other channel counts: a vector
// kernel -- workgroup = (one degree l, a run of rows (node, m)), W^T in LDS so that lanes of consecutive output channels
// read consecutive words; a thread produces ROWS_PER_THREAD rows of one output channel and reads the inputs of its
// rows as LDS broadcasts.
#include "egnn_internal.h"

#define MIX_RPT 4      // rows per thread
#define MIX_TILES 8    // row tiles per workgroup at most (fewer on small inputs, to have enough workgroups in flight)

__global__ __launch_bounds__(256) void node_mix_kernel(const float* __restrict__ x1, const float* __restrict__ W1,
                                                       const float* __restrict__ x2, const float* __restrict__ W2,
                                                       float* __restrict__ y, int n_nodes, int lmax, int log2E,
                                                       int transpose, int tiles) {
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
    // forward: y[co] = sum_ci W[l][co][ci] x[ci]; transposed (reverse pass): y[co] = sum_ci W[l][ci][co] x[ci]
    const int r = i >> log2E, q = i & (E - 1);
    const int at = transpose ? i : q * E + r;
    sWt[at] = W1[(size_t)l * E * E + i];
    if (W2) sWt[E * E + at] = W2[(size_t)l * E * E + i];
  }

  for (int t = 0; t < tiles; ++t) {
    const long r0 = ((long)blockIdx.x * tiles + t) * rows_per_tile;
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

// The same mix on the matrix cores, for 32 and 64 channels (a 32 x 32 MFMA block is one block of output channels):
// workgroup = (degree l, run of 32-row tiles), W^T in LDS, one tile per wave at a time.  v_mfma_f32_32x32x2_f32 takes
// plain fp32 operands, so the products are exact fp32 as in the vector version.  Lane l serves row / output channel
// l & 31; the contraction index of MFMA step s on lane half hh is c' = hh * E/2 + s (any order will do as long as
// both operands use it; this one lets a lane fetch its half row as contiguous 16-byte loads).
typedef float mix_float16v __attribute__((ext_vector_type(16)));

template <int LOG2E>
__global__ __launch_bounds__(256) void node_mix_mfma_kernel(const float* __restrict__ x1, const float* __restrict__ W1,
                                                            const float* __restrict__ x2, const float* __restrict__ W2,
                                                            float* __restrict__ y, int n_nodes, int lmax, int transpose,
                                                            int tiles) {
  constexpr int E = 1 << LOG2E, KH = E / 2, NCB = E / 32;
  extern __shared__ float smem[];   // [n_in][c'][c]
  const int l = blockIdx.y;
  const int D = (lmax + 1) * (lmax + 1);
  const int nm = 2 * l + 1;
  const long n_rows = (long)n_nodes * nm;
  const int n_in = W2 ? 2 : 1;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = lane & 31, hh = lane >> 5;
  for (int i = tid; i < E * E; i += 256) {
    // forward: y[co] = sum_ci W[l][co][ci] x[ci]; transposed (reverse pass): y[co] = sum_ci W[l][ci][co] x[ci]
    const int r = i >> LOG2E, q = i & (E - 1);
    const int at = transpose ? i : q * E + r;
    smem[at] = W1[(size_t)l * E * E + i];
    if (W2) smem[E * E + at] = W2[(size_t)l * E * E + i];
  }
  __syncthreads();
  // Items = (row tile, input) pairs in order; the half row of the next item is requested before the matrix-core
  // instructions of the current one are issued, so that a wave's loads and its arithmetic overlap.
  auto row_offset = [&](int t, bool& valid) -> size_t {
    const long r0 = (((long)blockIdx.x * tiles + t) * 4 + wave) * 32;
    valid = t < tiles && r0 < n_rows;
    long r = r0 + m;
    if (r >= n_rows) r = n_rows - 1;
    if (!valid) r = 0;
    const long node = r / nm;
    return (((size_t)node * D + l * l + (int)(r - node * nm)) << LOG2E) + hh * KH;
  };
  auto fetch = [&](const float* x, size_t off, float* a) {
    const float4* xr = reinterpret_cast<const float4*>(x + off);
#pragma unroll
    for (int q = 0; q < KH / 4; ++q) {
      const float4 v = xr[q];
      a[4 * q] = v.x; a[4 * q + 1] = v.y; a[4 * q + 2] = v.z; a[4 * q + 3] = v.w;
    }
  };
  bool valid;
  size_t off = row_offset(0, valid);
  if (!valid) return;
  float a[KH], an[KH];
  fetch(x1, off, a);
  for (int t = 0; t < tiles; ++t) {
    const long r0 = (((long)blockIdx.x * tiles + t) * 4 + wave) * 32;
    bool valid_next;
    const size_t off_next = row_offset(t + 1, valid_next);
    mix_float16v acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[cb][i] = 0.0f;
    for (int in = 0; in < n_in; ++in) {
      // next item: the second input of this tile, or the first input of the next tile
      const bool more = in + 1 < n_in || valid_next;
      if (more) fetch(in + 1 < n_in ? x2 : x1, in + 1 < n_in ? off : off_next, an);
      const float* wt = smem + (size_t)in * E * E + (size_t)(hh * KH) * E + m;
#pragma unroll
      for (int s = 0; s < KH; ++s)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
          acc[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], wt[s * E + 32 * cb], acc[cb], 0, 0, 0);
#pragma unroll
      for (int s = 0; s < KH; ++s) a[s] = an[s];
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const long ro = r0 + 8 * (i >> 2) + 4 * hh + (i & 3);
      if (ro < n_rows) {
        const long no = ro / nm;
        float* out = y + (((size_t)no * D + l * l + (int)(ro - no * nm)) << LOG2E) + m;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) out[32 * cb] = acc[cb][i];
      }
    }
    if (!valid_next) break;
    off = off_next;
  }
}

template <int LOG2E>
static int launch_node_mix_mfma(egnn_ctx* ctx, const float* x1, const float* W1, const float* x2, const float* W2,
                                float* y, int n_nodes, hipStream_t stream, int transpose) {
  constexpr int E = 1 << LOG2E;
  const int lmax = ctx->desc.lmax;
  const long max_rows = (long)n_nodes * (2 * lmax + 1);
  const long n_tiles = (max_rows + 127) / 128;                 // 4 waves x 32 rows
  // several tiles per workgroup once there are enough of them to fill the chip (the next tile's rows are in flight
  // while the current one is multiplied; measured at 500,000 rows of 64 channels: 0.120 -> 0.103 ms)
  long tiles = n_tiles / 256;
  tiles = tiles < 1 ? 1 : (tiles > 8 ? 8 : tiles);
  dim3 grid((unsigned)((n_tiles + tiles - 1) / tiles), lmax + 1), block(256);
  const size_t shmem = (size_t)(W2 ? 2 : 1) * E * E * sizeof(float);
  hipLaunchKernelGGL(node_mix_mfma_kernel<LOG2E>, grid, block, shmem, stream, x1, W1, x2, W2, y, n_nodes, lmax, transpose,
                     (int)tiles);
  EGNN_LAUNCH_CHECK(ctx, "node_mix_mfma_kernel");
  return EGNN_OK;
}

int egnn_launch_node_mix(egnn_ctx* ctx, const float* x1, const float* W1, const float* x2, const float* W2,
                         float* y, int n_nodes, hipStream_t stream, int transpose) {
  if (n_nodes == 0) return EGNN_OK;
  if (ctx->desc.channels == 32) return launch_node_mix_mfma<5>(ctx, x1, W1, x2, W2, y, n_nodes, stream, transpose);
  if (ctx->desc.channels == 64) return launch_node_mix_mfma<6>(ctx, x1, W1, x2, W2, y, n_nodes, stream, transpose);
  const int E = ctx->desc.channels, lmax = ctx->desc.lmax;
  const int rows_per_tile = MIX_RPT * (256 / E);
  const long max_rows = (long)n_nodes * (2 * lmax + 1);
  // each workgroup loads W once: several tiles per workgroup amortise that, but only once the grid is large enough
  const long n_tiles = (max_rows + rows_per_tile - 1) / rows_per_tile;
  long tiles = n_tiles / 2048;
  tiles = tiles < 1 ? 1 : (tiles > MIX_TILES ? MIX_TILES : tiles);
  const long per_wg = (long)rows_per_tile * tiles;
  dim3 grid((unsigned)((max_rows + per_wg - 1) / per_wg), lmax + 1), block(256);
  const int n_in = W2 ? 2 : 1;
  const size_t shmem = ((size_t)n_in * E * E + (size_t)n_in * rows_per_tile * (E + 1)) * sizeof(float);
  if (shmem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(node_mix_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(node_mix_kernel)");
  }
  hipLaunchKernelGGL(node_mix_kernel, grid, block, shmem, stream, x1, W1, x2, W2, y, n_nodes, lmax,
                     ctx->log2_channels, transpose, (int)tiles);
  EGNN_LAUNCH_CHECK(ctx, "node_mix_kernel");
  return EGNN_OK;
}

// Weight gradient of the mix: dW[l][d][c] = sum over rows (node, m) of dy[row][d] x[row][c].
// grid = (row chunks, degrees); each workgroup writes one partial [E][E] block; a second pass adds the
// partials in fixed order.
#define WG_ROWS 16
// PT = outputs per thread = max(1, E*E/256).  A thread owns input channel c = tid % E and the output channels
// d = tid / E + q * (256 / E), q < PT.
template <int PT>
__global__ __launch_bounds__(256) void mix_wgrad_kernel(const float* __restrict__ dy, const float* __restrict__ x,
                                                        float* __restrict__ partial, int n_nodes, int lmax, int log2E,
                                                        int nodes_per_chunk) {
  extern __shared__ float smem[];
  const int E = 1 << log2E;
  const int l = blockIdx.y;
  const int D = (lmax + 1) * (lmax + 1);
  const int nm = 2 * l + 1;
  float* sdy = smem;                  // [WG_ROWS][E]
  float* sx = smem + WG_ROWS * E;     // [WG_ROWS][E]
  const int tid = threadIdx.x;
  const int c = tid & (E - 1), d0 = tid >> log2E, dstep = 256 >> log2E;
  const bool active = d0 < E;         // E = 8: only the first 64 threads own an output
  float acc[PT];
#pragma unroll
  for (int q = 0; q < PT; ++q) acc[q] = 0.0f;
  const long r_begin = (long)blockIdx.x * nodes_per_chunk * nm;
  long r_end = r_begin + (long)nodes_per_chunk * nm;
  const long n_rows = (long)n_nodes * nm;
  if (r_end > n_rows) r_end = n_rows;
  for (long r0 = r_begin; r0 < r_end; r0 += WG_ROWS) {
    __syncthreads();
    for (int i = tid; i < WG_ROWS * E; i += 256) {
      const int rr = i >> log2E, cc = i & (E - 1);
      const long r = r0 + rr;
      float a = 0.0f, b = 0.0f;
      if (r < r_end) {
        const long node = r / nm;
        const int mm = (int)(r - node * nm);
        const size_t off = (((size_t)node * D + l * l + mm) << log2E) + cc;
        a = dy[off];
        b = x[off];
      }
      sdy[i] = a;
      sx[i] = b;
    }
    __syncthreads();
    if (active) {
      for (int rr = 0; rr < WG_ROWS; ++rr) {
        const float xv = sx[(rr << log2E) + c];
        const float* dr = sdy + (rr << log2E) + d0;
#pragma unroll
        for (int q = 0; q < PT; ++q) acc[q] += dr[q * dstep] * xv;
      }
    }
  }
  if (active) {
    float* out = partial + ((size_t)blockIdx.x * (lmax + 1) + l) * E * E;
#pragma unroll
    for (int q = 0; q < PT; ++q) out[((d0 + q * dstep) << log2E) + c] = acc[q];
  }
}

#define WGRAD_MAX_CHUNKS 256
size_t egnn_mix_wgrad_ws_bytes(const egnn_ctx* ctx) {
  const size_t E = ctx->desc.channels;
  return (size_t)WGRAD_MAX_CHUNKS * (ctx->desc.lmax + 1) * E * E * sizeof(float);
}

// dW[lmax+1][E][E] = sum_rows dy (x) x; `partial` must hold egnn_mix_wgrad_ws_bytes.
int egnn_launch_mix_wgrad(egnn_ctx* ctx, const float* dy, const float* x, float* dW, float* partial, int n_nodes,
                          hipStream_t stream) {
  const int E = ctx->desc.channels, lmax = ctx->desc.lmax;
  const long n_w = (long)(lmax + 1) * E * E;
  if (n_nodes == 0) return egnn_launch_reduce_partials(ctx, partial, 0, n_w, dW, 1.0f, stream);
  int chunks = n_nodes < WGRAD_MAX_CHUNKS ? n_nodes : WGRAD_MAX_CHUNKS;
  const int per = (n_nodes + chunks - 1) / chunks;
  chunks = (n_nodes + per - 1) / per;
  const dim3 grid(chunks, lmax + 1), block(256);
  const size_t shmem = 2 * WG_ROWS * E * sizeof(float);
#define LAUNCH(PT)                                                                                             \
  hipLaunchKernelGGL(mix_wgrad_kernel<PT>, grid, block, shmem, stream, dy, x, partial, n_nodes, lmax,          \
                     ctx->log2_channels, per)
  switch (E) {
    case 8: case 16: LAUNCH(1); break;
    case 32: LAUNCH(4); break;
    case 64: LAUNCH(16); break;
    case 128: LAUNCH(64); break;
    default: return egnn_fail(ctx, EGNN_EINVAL, "mix_wgrad: unsupported channel count");
  }
#undef LAUNCH
  EGNN_LAUNCH_CHECK(ctx, "mix_wgrad_kernel");
  return egnn_launch_reduce_partials(ctx, partial, chunks, n_w, dW, 1.0f, stream);
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
