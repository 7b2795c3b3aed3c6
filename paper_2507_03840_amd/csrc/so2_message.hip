// The message transform in its bond-aligned SO(2) form, summed over incoming edges
// (Fig. 2(a) bottom, Fig. 2(d); Sec. 3 "Message passing"; Sec. 2.1, last paragraph).
//
// Per directed edge k = (i -> j): the message is the concatenation [x_i | x_j | e_k] along the channel axis (3E
// channels), e_k being zero except for its L = 0 plane W_e B(d_k); it is rotated so that the bond lies on z, every
// order m goes through its own linear layer over (degree l >= |m|, channel),
//     y_0 = W_0 x_0;    y_{+m} = Wr_m x_{+m} - Wi_m x_{-m},   y_{-m} = Wi_m x_{+m} + Wr_m x_{-m}    (3E -> E channels),
// the result is rotated back, multiplied by the cutoff envelope and summed into the destination node (times
// agg_norm^-1/2).  Unlike the tensor-product route of the layer (per-edge weights, no channel mixing) this is a
// dense contraction shared by all edges, so it runs as five GEMMs, one per |m|:
//   1. so2_gather_kernel   lane = (edge, channel): both node rows rotated into the bond frame in registers, written
//                          m-major: A_0[k] = (x_{l,0} of both nodes for all l, then e_k), A_m[k] = [x_{+m} | x_{-m}];
//   2. so2_pack_kernel     the weights of order m as one matrix B_m = [[Wr^T, Wi^T], [-Wi^T, Wr^T]], cut into bf16
//                          pieces and stored in the operand order of the streaming GEMM (stream_gemm.h);
//   3. so2_gemm_kernel     Y_m = A_m B_m on split-bf16 MFMA (six products per fp32 product), 448 edges x 64 columns per
//                          workgroup, the 64-column tiles of an edge block running side by side;
//   4. so2_scatter_kernel  one workgroup per destination node, lane = (edge slot, channel): m-major rows of Y back to
//                          (l, m) order, rotated back, times f_c, summed; slots added in fixed order (no atomics).
#include "egnn_internal.h"
#include "bond_frame.h"
#include "stream_gemm.h"

struct So2Bufs {
  float* A[5];
  float* Y[5];
  int K[5], N[5];   // columns of A_m and of Y_m
};

__host__ __device__ inline int so2_K(int lmax, int E, int m) { return m == 0 ? (lmax + 1) * 2 * E + E : 2 * (lmax + 1 - m) * 2 * E; }
__host__ __device__ inline int so2_N(int lmax, int E, int m) { return m == 0 ? (lmax + 1) * E : 2 * (lmax + 1 - m) * E; }
// first float of order m in the packed weights: W_0, then (Wr_m, Wi_m) for m = 1..lmax
static size_t so2_w_offset(int lmax, int E, int m) {
  size_t off = 0;
  for (int q = 0; q < m; ++q) {
    const size_t nl = lmax + 1 - q;
    off += (q == 0 ? 1 : 2) * (nl * E) * (nl * 3 * E);
  }
  return off;
}

// ---------------------------------------------------------------------------------------------- 1. gather
template <int LMAX>
__global__ __launch_bounds__(256) void so2_gather_kernel(const int* __restrict__ src, const int* __restrict__ dst,
                                                         const float4* __restrict__ rhat_d, const float* __restrict__ x,
                                                         const float* __restrict__ W_e, So2Bufs b, long n_edges,
                                                         int log2E, int n_rbf, float r_cut) {
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  const int E = 1 << log2E;
  const int c = threadIdx.x & (E - 1);
  const long k = (long)blockIdx.x * (256 >> log2E) + (threadIdx.x >> log2E);
  if (k >= n_edges) return;
  const float4 g = rhat_d[k];
  const float* xs = x + (((size_t)src[k] * D) << log2E) + c;
  const float* xd = x + (((size_t)dst[k] * D) << log2E) + c;
  float vs[D], vd[D];
#pragma unroll
  for (int i = 0; i < D; ++i) {
    vs[i] = xs[(size_t)i << log2E];
    vd[i] = xd[(size_t)i << log2E];
  }
  BondTrig t;
  egnn_bond_trig<LMAX>(g.x, g.y, g.z, t);
  egnn_to_bond_frame<LMAX>(vs, t);
  egnn_to_bond_frame<LMAX>(vd, t);
  // L = 0 plane of the edge embedding: a linear map of the Gaussian expansion of the length
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
  float e0 = 0.0f;
  for (int q = 0; q < n_rbf; ++q) {
    const float u = g.w - (float)q * step;
    e0 += W_e[c * n_rbf + q] * __expf(-u * u * inv2s2);
  }
  float* a0 = b.A[0] + (size_t)k * b.K[0] + c;
#pragma unroll
  for (int l = 0; l <= LMAX; ++l) {
    __builtin_nontemporal_store(vs[l * l + l], a0 + ((2 * l) << log2E));
    __builtin_nontemporal_store(vd[l * l + l], a0 + ((2 * l + 1) << log2E));
  }
  __builtin_nontemporal_store(e0, a0 + ((2 * (LMAX + 1)) << log2E));
#pragma unroll
  for (int m = 1; m <= LMAX; ++m) {
    constexpr int dummy = 0;
    (void)dummy;
    const int nl = LMAX + 1 - m;
    float* am = b.A[m] + (size_t)k * b.K[m] + c;
#pragma unroll
    for (int l = m; l <= LMAX; ++l) {
      const int col = (2 * (l - m)) << log2E;
      __builtin_nontemporal_store(vs[l * l + l + m], am + col);
      __builtin_nontemporal_store(vd[l * l + l + m], am + col + E);
      __builtin_nontemporal_store(vs[l * l + l - m], am + ((2 * nl) << log2E) + col);
      __builtin_nontemporal_store(vd[l * l + l - m], am + ((2 * nl) << log2E) + col + E);
    }
  }
}

// ---------------------------------------------------------------------------------------------- 2. weights
// B_m[k][n] for the column order of A_m (k) and of Y_m (n); W points at W_0 (m = 0) or at Wr_m (Wi_m follows it)
__device__ __forceinline__ float so2_b_value(const float* __restrict__ W, int m, int lmax, int E, int k, int n, int K, int N) {
  if (k >= K || n >= N) return 0.0f;
  if (m == 0) {
    const int edge0 = (lmax + 1) * 2 * E;
    int col;
    if (k < edge0) {
      const int l = k / (2 * E);
      col = l * 3 * E + (k - l * 2 * E);     // g E + c with g in {0, 1}
    } else {
      col = 2 * E + (k - edge0);             // l = 0, g = 2: the edge embedding
    }
    return W[(size_t)n * ((lmax + 1) * 3 * E) + col];
  }
  const int nl = lmax + 1 - m;
  const int half_k = nl * 2 * E, half_n = nl * E;
  const int s_in = k / half_k, kr = k - s_in * half_k;
  const int li = kr / (2 * E);
  const int col = li * 3 * E + (kr - li * 2 * E);
  const int s_out = n / half_n, row = n - s_out * half_n;
  const size_t at = (size_t)row * (nl * 3 * E) + col;
  const size_t sz = (size_t)half_n * (nl * 3 * E);
  if (s_in == s_out) return W[at];                     // Wr
  return s_in == 0 ? W[sz + at] : -W[sz + at];         // x_{+m} -> y_{-m}: +Wi;  x_{-m} -> y_{+m}: -Wi
}

// T[ct][step][j][piece][64]: thread -> (ct, step, j, pair of contraction indices)
__global__ __launch_bounds__(256) void so2_pack_kernel(const float* __restrict__ W, uint16_t* __restrict__ T, int m, int lmax,
                                                       int E, int K, int N, int n_steps, int n_ct) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  const long total = (long)n_ct * n_steps * 64 * 32;
  if (i >= total) return;
  const int rp = (int)(i & 31), j = (int)((i >> 5) & 63);
  const long blk = i >> 11;                    // ct * n_steps + step
  const int step = (int)(blk % n_steps), ct = (int)(blk / n_steps);
  const int n = ct * 64 + j, k = step * 64 + 2 * rp;
  const Split3 s0 = split3(so2_b_value(W, m, lmax, E, k, n, K, N)), s1 = split3(so2_b_value(W, m, lmax, E, k + 1, n, K, N));
  uint32_t* o = reinterpret_cast<uint32_t*>(T) + blk * (64 * 96) + j * 96 + rp;
  o[0] = pack2(s0.hi, s1.hi);
  o[32] = pack2(s0.mid, s1.mid);
  o[64] = pack2(s0.lo, s1.lo);
}

// ---------------------------------------------------------------------------------------------- 3. GEMM
// C[e][ct*64 + j] = sum_k A[e][k] B[k][ct*64 + j].  A workgroup = (block of 64 * RB_WAVES rows, 64-column tile ct).
// Workgroup ids go round-robin over the 8 XCDs, each with its own L2, so the id is decoded such that the column tiles
// of one block of rows sit on the same XCD with consecutive dispatch slots: they read the same rows of A, once from
// HBM and then from that L2.  A compute wave owns 64 rows; its 64 x 64 tile of A is fetched in memory order and turned
// to operand order through a private LDS tile.
#define SO2_AROW 68
__global__ __launch_bounds__(RB_THREADS) void so2_gemm_kernel(const float* __restrict__ A, long M, int K, const uint16_t* __restrict__ T,
                                                              int n_steps, float* __restrict__ C, int N, int n_ct,
                                                              int n_row_blocks) {
  extern __shared__ uint4 so2_smem[];
  uint4* sB = so2_smem;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
  const int ct = idx % n_ct;
  const int row_block = (idx / n_ct) * 8 + xcd;
  if (row_block >= n_row_blocks) return;   // (whole workgroup: the grid is rounded up to a multiple of 8 row blocks)
  if (wave == RB_WAVES) {
    rb_loader(T, (long)ct * n_steps, n_steps, sB, lane);
    return;
  }
  float* sA = reinterpret_cast<float*>(sB + 2 * 64 * RB_BROW4) + (size_t)wave * 32 * SO2_AROW;
  const int m = lane & 31, hh = lane >> 5;
  const long e_base = ((long)row_block * RB_WAVES + wave) * 64;
  const int frow = lane >> 4, fcol = (lane & 15) * 4;
  const float* fptr[2][8];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      long e = e_base + rb * 32 + 4 * i + frow;
      if (e >= M) e = M - 1;
      fptr[rb][i] = A + (size_t)e * K;
    }
  float16v acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;
  // rows of the next step in flight while this one is contracted; columns past the row are clamped here and
  // zeroed where the value is used (touching it here would make the wave wait for the load it has just issued)
  float4 nxt[2][8];
  auto fetch = [&](int s) {
    const int n = s * 64 + fcol;
    const int nc = n < K ? n : K - 4;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int i = 0; i < 8; ++i) nxt[rb][i] = *reinterpret_cast<const float4*>(fptr[rb][i] + nc);
  };
  fetch(0);
  for (int s = 0; s < n_steps; ++s) {
    float4 cur[2][8];
    const bool col_ok = s * 64 + fcol < K;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int i = 0; i < 8; ++i) cur[rb][i] = col_ok ? nxt[rb][i] : make_float4(0.f, 0.f, 0.f, 0.f);
    if (s + 1 < n_steps) fetch(s + 1);
    rb_barrier_acquire();
    const uint4* bbase = sB + (s & 1) * (64 * RB_BROW4) + hh * 4;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<float4*>(sA + (4 * i + frow) * SO2_AROW + fcol) = cur[rb][i];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
      const float4* arow = reinterpret_cast<const float4*>(sA + m * SO2_AROW + hh * 32);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float4 u = arow[2 * t], v = arow[2 * t + 1];
        const float xv[8] = {u.x, u.y, u.z, u.w, v.x, v.y, v.z, v.w};
        uint4 ah, am, al;
        rb_split8(xv, ah, am, al);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          const uint4* brow = bbase + (m + 32 * cb) * RB_BROW4 + t;
          const uint4 bq[3] = {brow[0], brow[8], brow[16]};
          acc[rb][cb] = rb_mma6(ah, am, al, bq, acc[rb][cb]);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
      __builtin_amdgcn_wave_barrier();
    }
  }
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      const int col = ct * 64 + cb * 32 + m;
      if (col < N) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const long e = e_base + rb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
          if (e < M) C[(size_t)e * N + col] = acc[rb][cb][i];
        }
      }
    }
}

// ---------------------------------------------------------------------------------------------- 4. scatter
template <int LMAX>
__global__ __launch_bounds__(256) void so2_scatter_kernel(const int* __restrict__ row_ptr, const float4* __restrict__ rhat_d,
                                                          So2Bufs b, float* __restrict__ a, int n_owned, int log2E,
                                                          int nodes_per_xcd, float scale, float r_cut) {
  constexpr int D = (LMAX + 1) * (LMAX + 1);
  __shared__ float red[256 * D];
  const int j = (blockIdx.x & 7) * nodes_per_xcd + (blockIdx.x >> 3);
  if (j >= n_owned || (int)(blockIdx.x >> 3) >= nodes_per_xcd) return;
  const int E = 1 << log2E;
  const int tid = threadIdx.x;
  const int c = tid & (E - 1), slot = tid >> log2E, n_slots = 256 >> log2E;
  const int k0 = row_ptr[j], k1 = row_ptr[j + 1];
  float acc[D];
#pragma unroll
  for (int i = 0; i < D; ++i) acc[i] = 0.0f;
  for (int k = k0 + slot; k < k1; k += n_slots) {
    const float4 g = rhat_d[k];
    float o[D];
    const float* y0 = b.Y[0] + (size_t)k * b.N[0] + c;
#pragma unroll
    for (int l = 0; l <= LMAX; ++l) o[l * l + l] = __builtin_nontemporal_load(y0 + (l << log2E));
#pragma unroll
    for (int m = 1; m <= LMAX; ++m) {
      const int nl = LMAX + 1 - m;
      const float* ym = b.Y[m] + (size_t)k * b.N[m] + c;
#pragma unroll
      for (int l = m; l <= LMAX; ++l) {
        o[l * l + l + m] = __builtin_nontemporal_load(ym + ((l - m) << log2E));
        o[l * l + l - m] = __builtin_nontemporal_load(ym + ((nl + l - m) << log2E));
      }
    }
    BondTrig t;
    egnn_bond_trig<LMAX>(g.x, g.y, g.z, t);
    egnn_from_bond_frame<LMAX>(o, t);
    const float fc = 0.5f * (1.0f + cosf(3.14159265358979323846f * g.w / r_cut));
#pragma unroll
    for (int i = 0; i < D; ++i) acc[i] += fc * o[i];
  }
#pragma unroll
  for (int i = 0; i < D; ++i) red[((slot * D + i) << log2E) + c] = acc[i];
  __syncthreads();
  const int row = D << log2E;
  float* out = a + (size_t)j * row;
  for (int idx = tid; idx < row; idx += 256) {
    float sum = 0.0f;
    for (int s = 0; s < n_slots; ++s) sum += red[s * row + idx];
    out[idx] = sum * scale;
  }
}

// ---------------------------------------------------------------------------------------------- host side
static size_t so2_a256(size_t n) { return (n + 255) & ~(size_t)255; }
static int so2_steps(int K) { return (K + 63) / 64; }
static int so2_tiles(int N) { return (N + 63) / 64; }

extern "C" int egnn_so2_weight_count(const egnn_ctx* ctx, int64_t* n_floats) {
  if (!ctx || !n_floats) return EGNN_EINVAL;
  *n_floats = (int64_t)so2_w_offset(ctx->desc.lmax, ctx->desc.channels, ctx->desc.lmax + 1);
  return EGNN_OK;
}

static size_t so2_ws(const egnn_ctx* ctx, int64_t n_edges, bool carve, char* base, float** rhat_d, So2Bufs* b, uint16_t** T) {
  const int lmax = ctx->desc.lmax, E = ctx->desc.channels;
  size_t used = 0;
  auto take = [&](size_t bytes) { char* p = carve ? base + used : nullptr; used += so2_a256(bytes); return p; };
  float* rd = (float*)take((size_t)n_edges * 16);
  if (rhat_d) *rhat_d = rd;
  for (int m = 0; m <= lmax; ++m) {
    const int K = so2_K(lmax, E, m), N = so2_N(lmax, E, m);
    float* A = (float*)take((size_t)n_edges * K * sizeof(float));
    float* Y = (float*)take((size_t)n_edges * N * sizeof(float));
    uint16_t* t = (uint16_t*)take((size_t)so2_tiles(N) * so2_steps(K) * 64 * 3 * 64 * sizeof(uint16_t));
    if (b) { b->A[m] = A; b->Y[m] = Y; b->K[m] = K; b->N[m] = N; }
    if (T) T[m] = t;
  }
  return used;
}

extern "C" int egnn_so2_workspace_bytes(const egnn_ctx* ctx, int64_t n_edges, size_t* bytes) {
  if (!ctx || !bytes || n_edges < 0) return EGNN_EINVAL;
  *bytes = so2_ws(ctx, n_edges, false, nullptr, nullptr, nullptr, nullptr) + 256;
  return EGNN_OK;
}

extern "C" int egnn_so2_message_sum(egnn_ctx* ctx, const egnn_graph* g, const float* pos, const float box[3],
                                    const float* x, const float* W_e, const float* W_so2, float* a, void* ws,
                                    size_t ws_bytes, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (!g || !pos || !box || !x || !W_e || !W_so2 || !a || !ws)
    return egnn_fail(ctx, EGNN_EINVAL, "so2_message_sum: null pointer");
  if (g->n_edges < 0 || g->n_edges > 2147483647LL || g->n_owned < 0 || g->n_total < g->n_owned || !g->row_ptr ||
      (g->n_edges > 0 && (!g->src || !g->dst)))
    return egnn_fail(ctx, EGNN_EINVAL, "so2_message_sum: bad graph");
  if (((uintptr_t)ws & 255) != 0) return egnn_fail(ctx, EGNN_EINVAL, "so2_message_sum: workspace not 256-byte aligned");
  const int lmax = ctx->desc.lmax, E = ctx->desc.channels;
  if (E < 8 || ctx->desc.n_rbf < 2) return egnn_fail(ctx, EGNN_EINVAL, "so2_message_sum: needs >= 8 channels and >= 2 radial bases");
  if (ws_bytes < so2_ws(ctx, g->n_edges, false, nullptr, nullptr, nullptr, nullptr))
    return egnn_fail(ctx, EGNN_EWS, "so2_message_sum: workspace too small");
  hipStream_t st = (hipStream_t)stream;
  float* rhat_d;
  So2Bufs b;
  uint16_t* T[5];
  for (int m = 0; m < 5; ++m) { b.A[m] = b.Y[m] = nullptr; b.K[m] = b.N[m] = 0; T[m] = nullptr; }
  so2_ws(ctx, g->n_edges, true, (char*)ws, &rhat_d, &b, T);
  const long n = g->n_edges;
  int rc;
  if (n > 0) {
    if ((rc = egnn_launch_geometry(ctx, g, pos, box, rhat_d, nullptr, nullptr, nullptr, st))) return rc;
    const float4* rd = reinterpret_cast<const float4*>(rhat_d);
    const int per_wg = 256 / E;
    dim3 grid((unsigned)((n + per_wg - 1) / per_wg)), block(256);
#define GATHER(L)                                                                                                    \
  hipLaunchKernelGGL(so2_gather_kernel<L>, grid, block, 0, st, g->src, g->dst, rd, x, W_e, b, n, ctx->log2_channels, \
                     ctx->desc.n_rbf, ctx->desc.r_cut)
    switch (lmax) {
      case 0: GATHER(0); break;
      case 1: GATHER(1); break;
      case 2: GATHER(2); break;
      case 3: GATHER(3); break;
      case 4: GATHER(4); break;
      default: return egnn_fail(ctx, EGNN_EINVAL, "so2_message_sum: lmax out of range");
    }
#undef GATHER
    EGNN_LAUNCH_CHECK(ctx, "so2_gather_kernel");
    const size_t lds = (size_t)2 * 64 * RB_BROW4 * sizeof(uint4) + (size_t)RB_WAVES * 32 * SO2_AROW * sizeof(float);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(so2_gemm_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(so2_gemm_kernel)");
    for (int m = 0; m <= lmax; ++m) {
      const int K = b.K[m], N = b.N[m], n_steps = so2_steps(K), n_ct = so2_tiles(N);
      const long total = (long)n_ct * n_steps * 64 * 32;
      hipLaunchKernelGGL(so2_pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                         W_so2 + so2_w_offset(lmax, E, m), T[m], m, lmax, E, K, N, n_steps, n_ct);
      EGNN_LAUNCH_CHECK(ctx, "so2_pack_kernel");
      const long rows_per_wg = 64L * RB_WAVES;
      const int n_row_blocks = (int)((n + rows_per_wg - 1) / rows_per_wg);
      const unsigned grid_x = (unsigned)(((n_row_blocks + 7) / 8) * 8 * n_ct);
      hipLaunchKernelGGL(so2_gemm_kernel, dim3(grid_x), dim3(RB_THREADS), lds, st, b.A[m], n, K, T[m], n_steps, b.Y[m], N,
                         n_ct, n_row_blocks);
      EGNN_LAUNCH_CHECK(ctx, "so2_gemm_kernel");
    }
  }
  if (g->n_owned == 0) return EGNN_OK;
  const int per_xcd = (g->n_owned + 7) / 8;
  const float scale = 1.0f / sqrtf(ctx->desc.agg_norm);
  const float4* rd = reinterpret_cast<const float4*>(rhat_d);
#define SCATTER(L)                                                                                               \
  hipLaunchKernelGGL(so2_scatter_kernel<L>, dim3(per_xcd * 8), dim3(256), 0, st, g->row_ptr, rd, b, a, g->n_owned, \
                     ctx->log2_channels, per_xcd, scale, ctx->desc.r_cut)
  switch (lmax) {
    case 0: SCATTER(0); break;
    case 1: SCATTER(1); break;
    case 2: SCATTER(2); break;
    case 3: SCATTER(3); break;
    case 4: SCATTER(4); break;
    default: return egnn_fail(ctx, EGNN_EINVAL, "so2_message_sum: lmax out of range");
  }
#undef SCATTER
  EGNN_LAUNCH_CHECK(ctx, "so2_scatter_kernel");
  return EGNN_OK;
}
