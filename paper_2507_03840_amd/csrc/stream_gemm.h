// Device helpers shared by the kernels that stream a large fp32 operand against a small, pre-split one on the matrix
// cores (reverse pass of the radial MLP, per-m linear layers of the SO(2) message transform).
//
// The small operand is cut into bf16 pieces beforehand and stored transposed in blocks of 64 contraction indices,
//   T[step][j][piece][64]   (step = contraction index / 64, j = output column of a 64-column tile),
// the order an MFMA B operand is read in; one wave of each workgroup (the loader) copies the next 24 KB block into
// one of two LDS buffers while the other seven contract.  A wave that only computes never waits on a store, and the
// barriers carry LDS-only fences.  The large operand is cut into pieces on the fly, in registers.  Six piece products
// per fp32 product, smallest first: fp32-level accuracy at 6/16 of the fp32-MFMA cost.
#pragma once
#include "split_bf16.h"

#define RB_WAVES 7                    // compute waves per workgroup
#define RB_THREADS ((RB_WAVES + 1) * 64)
#define RB_BROW4 25                   // uint4 per staged row: 24 of data (3 pieces x 64 bf16) + 1 of padding

__device__ __forceinline__ void rb_release_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
}
__device__ __forceinline__ void rb_barrier_acquire() {
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// the loader wave: block `step` of T -> sB[step & 1], one barrier per block (the loads of block s + 1 overlap the
// compute waves' work on block s)
__device__ __forceinline__ void rb_loader(const uint16_t* __restrict__ T, long first_step, int n_steps, uint4* sB, int lane) {
  const uint4* src = reinterpret_cast<const uint4*>(T) + first_step * (64 * 24);
  for (int s = 0; s < n_steps; ++s) {
    uint4 v[24];
#pragma unroll
    for (int i = 0; i < 24; ++i) v[i] = src[(size_t)s * (64 * 24) + i * 64 + lane];
    uint4* dst = sB + (s & 1) * (64 * RB_BROW4);
#pragma unroll
    for (int i = 0; i < 24; ++i) {
      const int u = i * 64 + lane, row = u / 24, c16 = u - row * 24;
      dst[row * RB_BROW4 + c16] = v[i];
    }
    rb_release_barrier();
  }
}

// eight fp32 values -> the three bf16 pieces of an MFMA operand register
__device__ __forceinline__ void rb_split8(const float (&x)[8], uint4& hi, uint4& mid, uint4& lo) {
  uint32_t h[4], m[4], l[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const Split3 s0 = split3(x[2 * q]), s1 = split3(x[2 * q + 1]);
    h[q] = pack2(s0.hi, s1.hi);
    m[q] = pack2(s0.mid, s1.mid);
    l[q] = pack2(s0.lo, s1.lo);
  }
  hi = make_uint4(h[0], h[1], h[2], h[3]);
  mid = make_uint4(m[0], m[1], m[2], m[3]);
  lo = make_uint4(l[0], l[1], l[2], l[3]);
}

// acc += A (pieces ah, am, al) x B (pieces b[0..2]) for one 16-wide contraction step
__device__ __forceinline__ float16v rb_mma6(uint4 ah, uint4 am, uint4 al, const uint4 (&b)[3], float16v acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(al), as_bf16x8(b[0]), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ah), as_bf16x8(b[2]), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(am), as_bf16x8(b[1]), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(am), as_bf16x8(b[0]), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ah), as_bf16x8(b[1]), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ah), as_bf16x8(b[0]), acc, 0, 0, 0);
  return acc;
}


// the same for two independent column blocks, the two accumulation chains interleaved (a matrix-core instruction that
// continues the chain of the one before it has to wait for its result)
__device__ __forceinline__ void rb_mma6x2(uint4 ah, uint4 am, uint4 al, const uint4 (&b0)[3], const uint4 (&b1)[3],
                                          float16v& acc0, float16v& acc1) {
#define RB_STEP(A, P)                                                                                  \
  acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(A), as_bf16x8(b0[P]), acc0, 0, 0, 0);       \
  acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(A), as_bf16x8(b1[P]), acc1, 0, 0, 0);
  RB_STEP(al, 0) RB_STEP(ah, 2) RB_STEP(am, 1) RB_STEP(am, 0) RB_STEP(ah, 1) RB_STEP(ah, 0)
#undef RB_STEP
}

// ---------------------------------------------------------------------------------------------------------------
// The streaming contraction as a whole: acc[rb][cb] = rows (e_base + 32 rb ..+31) of A [M][K] times the 64-column
// tile of the small operand whose packed blocks start at `tsrc` (n_steps blocks of 64 contraction indices).
// A workgroup is SG_WAVES = 8 identical waves of 64 rows each (two per SIMD: the matrix cores of the four SIMDs carry
// equal loads).  The wave's 64 x 64 tile of A is fetched in memory order, one step ahead (the registers of step s are
// refilled with step s + 1 as soon as they have been copied to LDS, row block by row block: no register copies), and
// turned to operand order through a private LDS tile.  The 24 KB block of the small operand of a step is brought in
// by all waves together, three 16-byte pieces per thread: loaded into registers at the top of step s, written to the
// other LDS buffer after the step's arithmetic, published by the barrier that opens step s + 1 (no wave stores to
// global memory inside the loop, so these loads cost no waiting).  Columns past the end of a row of A are clamped to
// the row's last four: the packed operand is zero for contraction indices >= K and what is read in their place is
// finite, so those products vanish.  Rows past M repeat row M - 1; the caller does not store them.
// Dynamic LDS: SG_LDS_BYTES.
#define SG_WAVES 8
#define SG_THREADS (SG_WAVES * 64)
#define SG_AROW 68   // floats per row of the private tile: 64 + 4 (16-byte aligned, rows 4 banks apart)
#define SG_LDS_BYTES ((size_t)2 * 64 * RB_BROW4 * sizeof(uint4) + (size_t)SG_WAVES * 32 * SG_AROW * sizeof(float))
typedef float sg_f4 __attribute__((ext_vector_type(4)));
typedef unsigned int sg_u4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void sg_fetch8(sg_f4 (&dst)[8], const float* const (&row)[8], int col) {
#pragma unroll
  for (int i = 0; i < 8; ++i) dst[i] = *reinterpret_cast<const sg_f4*>(row[i] + col);
}
__device__ __forceinline__ void sg_store8(float* tile, const sg_f4 (&v)[8]) {   // rows 4 apart
#pragma unroll
  for (int i = 0; i < 8; ++i) *reinterpret_cast<sg_f4*>(tile + 4 * i * SG_AROW) = v[i];
}

// one 32-row block of a step: registers -> private tile, refill, tile -> operand order, 4 x (cut, 12 products)
__device__ __forceinline__ void sg_row_block(float* sA, const uint4* bbase, sg_f4 (&nxt)[8], const float* const (&fptr)[8],
                                             int next_col, int frow, int fcol, int m, int hh, float16v& acc0,
                                             float16v& acc1) {
  sg_store8(sA + frow * SG_AROW + fcol, nxt);
  sg_fetch8(nxt, fptr, next_col);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
  const float4* arow = reinterpret_cast<const float4*>(sA + m * SG_AROW + hh * 32);
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    // both column blocks' pieces of the small operand first: their LDS latency passes while A is cut into pieces
    const uint4* brow0 = bbase + m * RB_BROW4 + t;
    const uint4* brow1 = brow0 + 32 * RB_BROW4;
    const uint4 b0[3] = {brow0[0], brow0[8], brow0[16]};
    const uint4 b1[3] = {brow1[0], brow1[8], brow1[16]};
    const float4 u = arow[2 * t], v = arow[2 * t + 1];
    const float xv[8] = {u.x, u.y, u.z, u.w, v.x, v.y, v.z, v.w};
    uint4 ah, am, al;
    rb_split8(xv, ah, am, al);
    rb_mma6x2(ah, am, al, b0, b1, acc0, acc1);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_wave_barrier();   // reads of the tile are done before the next block overwrites it
}

__device__ __forceinline__ void sg_contract(const float* __restrict__ A, long M, int K, const uint4* __restrict__ tsrc,
                                            int n_steps, uint4* smem, long e_base, float16v (&acc)[2][2]) {
  uint4* sB = smem;                                  // [2][64][RB_BROW4]
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  float* sA = reinterpret_cast<float*>(sB + 2 * 64 * RB_BROW4) + (size_t)wave * 32 * SG_AROW;
  const int m = lane & 31, hh = lane >> 5;
  const int frow = lane >> 4, fcol = (lane & 15) * 4;
  const float* fptr0[8];
  const float* fptr1[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    long e0 = e_base + 4 * i + frow, e1 = e0 + 32;
    if (e0 >= M) e0 = M - 1;
    if (e1 >= M) e1 = M - 1;
    fptr0[i] = A + (size_t)e0 * K;
    fptr1[i] = A + (size_t)e1 * K;
  }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;
  sg_u4 bnext[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) bnext[i] = *reinterpret_cast<const sg_u4*>(tsrc + i * SG_THREADS + tid);
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int u = i * SG_THREADS + tid, row = u / 24, c16 = u - row * 24;
    *reinterpret_cast<sg_u4*>(sB + row * RB_BROW4 + c16) = bnext[i];
  }
  sg_f4 nxt0[8], nxt1[8];
  sg_fetch8(nxt0, fptr0, fcol < K ? fcol : K - 4);
  sg_fetch8(nxt1, fptr1, fcol < K ? fcol : K - 4);
  for (int s = 0; s < n_steps; ++s) {
    rb_release_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    const uint4* bbase = sB + (s & 1) * (64 * RB_BROW4) + hh * 4;
    const int s_next = s + 1 < n_steps ? s + 1 : s;   // (the last step fetches itself again: no branch around loads)
    const int n_next = s_next * 64 + fcol;
    const int next_col = n_next < K ? n_next : K - 4;
#pragma unroll
    for (int i = 0; i < 3; ++i)
      bnext[i] = *reinterpret_cast<const sg_u4*>(tsrc + (size_t)s_next * (64 * 24) + i * SG_THREADS + tid);
    sg_row_block(sA, bbase, nxt0, fptr0, next_col, frow, fcol, m, hh, acc[0][0], acc[0][1]);
    sg_row_block(sA, bbase, nxt1, fptr1, next_col, frow, fcol, m, hh, acc[1][0], acc[1][1]);
    // (after the last step this rewrites a buffer that nobody reads any more)
    uint4* bdst = sB + ((s + 1) & 1) * (64 * RB_BROW4);
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int u = i * SG_THREADS + tid, row = u / 24, c16 = u - row * 24;
      *reinterpret_cast<sg_u4*>(bdst + row * RB_BROW4 + c16) = bnext[i];
    }
  }
}

// ---------------------------------------------------------------------------------------------------------------
// The same streaming contraction on two half-precision pieces per operand and three products per fp32 product
// (hi*hi + hi*lo + lo*hi; the lo*lo term is 2^-22 of the product).  Half precision has a narrow exponent range, so
// both operands carry a power-of-two scaling chosen from their largest magnitude (largest piece in [2^13, 2^14)):
// the small operand is scaled when it is packed, the large one (times a_scale) when it is cut, and the caller undoes
// both on the accumulators.  Packed small operand: T[step][j][piece][64] halves, 16 uint4 per row j.
// Dynamic LDS: SGH_LDS_BYTES.
#define SGH_BROW4 17   // uint4 per staged row: 16 of data (2 pieces x 64 halves) + 1 of padding
#define SGH_LDS_BYTES ((size_t)2 * 64 * SGH_BROW4 * sizeof(uint4) + (size_t)SG_WAVES * 32 * SG_AROW * sizeof(float))
typedef _Float16 sgh_h8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ sgh_h8 sgh_as_h8(uint4 v) { return __builtin_bit_cast(sgh_h8, v); }

// the power of two that brings a largest magnitude (given as the bits of a non-negative float) into [2^13, 2^14):
// returned as its exponent; 0 for zero, infinite or NaN input
__device__ __forceinline__ int sgh_scale_exp(unsigned max_bits) {
  const float m = __uint_as_float(max_bits);
  if (!(m > 0.0f && m < 3.0e38f)) return 0;
  const int e = 13 - ilogbf(m);
  return e < -60 ? -60 : (e > 60 ? 60 : e);
}

// eight fp32 values times `scale` -> the two half-precision pieces of an MFMA operand register
__device__ __forceinline__ void sgh_split8(const float (&x)[8], float scale, uint4& hi, uint4& lo) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float a0 = x[2 * q] * scale, a1 = x[2 * q + 1] * scale;
    const _Float16 h0 = (_Float16)a0, h1 = (_Float16)a1;
    const _Float16 l0 = (_Float16)(a0 - (float)h0), l1 = (_Float16)(a1 - (float)h1);
    h[q] = (uint32_t)__builtin_bit_cast(unsigned short, h0) | ((uint32_t)__builtin_bit_cast(unsigned short, h1) << 16);
    l[q] = (uint32_t)__builtin_bit_cast(unsigned short, l0) | ((uint32_t)__builtin_bit_cast(unsigned short, l1) << 16);
  }
  hi = make_uint4(h[0], h[1], h[2], h[3]);
  lo = make_uint4(l[0], l[1], l[2], l[3]);
}

// acc0 / acc1 += A (pieces ah, al) x B (pieces b0 / b1) for one 16-wide contraction step, two column blocks, the two
// accumulation chains interleaved; smallest terms first
__device__ __forceinline__ void sgh_mma3x2(uint4 ah, uint4 al, const uint4 (&b0)[2], const uint4 (&b1)[2],
                                           float16v& acc0, float16v& acc1) {
#define SGH_STEP(A, P)                                                                                  \
  acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(sgh_as_h8(A), sgh_as_h8(b0[P]), acc0, 0, 0, 0);         \
  acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(sgh_as_h8(A), sgh_as_h8(b1[P]), acc1, 0, 0, 0);
  SGH_STEP(al, 0) SGH_STEP(ah, 1) SGH_STEP(ah, 0)
#undef SGH_STEP
}

__device__ __forceinline__ void sgh_row_block(float* sA, const uint4* bbase, sg_f4 (&nxt)[8], const float* const (&fptr)[8],
                                              int next_col, int frow, int fcol, int m, int hh, float a_scale,
                                              float16v& acc0, float16v& acc1) {
  sg_store8(sA + frow * SG_AROW + fcol, nxt);
  sg_fetch8(nxt, fptr, next_col);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
  const float4* arow = reinterpret_cast<const float4*>(sA + m * SG_AROW + hh * 32);
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const uint4* brow0 = bbase + m * SGH_BROW4 + t;
    const uint4* brow1 = brow0 + 32 * SGH_BROW4;
    const uint4 b0[2] = {brow0[0], brow0[8]};
    const uint4 b1[2] = {brow1[0], brow1[8]};
    const float4 u = arow[2 * t], v = arow[2 * t + 1];
    const float xv[8] = {u.x, u.y, u.z, u.w, v.x, v.y, v.z, v.w};
    uint4 ah, al;
    sgh_split8(xv, a_scale, ah, al);
    sgh_mma3x2(ah, al, b0, b1, acc0, acc1);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_wave_barrier();   // reads of the tile are done before the next block overwrites it
}

// the loader wave of a kernel that keeps one (see rb_loader): block `step` of T (64 rows of 16 uint4) -> sB[step & 1]
__device__ __forceinline__ void rbh_loader(const uint16_t* __restrict__ T, long first_step, int n_steps, uint4* sB, int lane) {
  const uint4* src = reinterpret_cast<const uint4*>(T) + first_step * (64 * 16);
  for (int s = 0; s < n_steps; ++s) {
    uint4 v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = src[(size_t)s * (64 * 16) + i * 64 + lane];
    uint4* dst = sB + (s & 1) * (64 * SGH_BROW4);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int u = i * 64 + lane, row = u >> 4, c16 = u & 15;
      dst[row * SGH_BROW4 + c16] = v[i];
    }
    rb_release_barrier();
  }
}

// as sg_contract; tsrc: n_steps blocks of 64 x 16 uint4; the accumulators hold a_scale * (scale of the packed operand)
// times the result
// lda: floats from one row of A to the next (0: K, rows back to back)
__device__ __forceinline__ void sgh_contract(const float* __restrict__ A, long M, int K, const uint4* __restrict__ tsrc,
                                             int n_steps, uint4* smem, long e_base, float a_scale, float16v (&acc)[2][2],
                                             int lda = 0) {
  if (lda == 0) lda = K;
  uint4* sB = smem;                                  // [2][64][SGH_BROW4]
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  float* sA = reinterpret_cast<float*>(sB + 2 * 64 * SGH_BROW4) + (size_t)wave * 32 * SG_AROW;
  const int m = lane & 31, hh = lane >> 5;
  const int frow = lane >> 4, fcol = (lane & 15) * 4;
  const float* fptr0[8];
  const float* fptr1[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    long e0 = e_base + 4 * i + frow, e1 = e0 + 32;
    if (e0 >= M) e0 = M - 1;
    if (e1 >= M) e1 = M - 1;
    fptr0[i] = A + (size_t)e0 * lda;
    fptr1[i] = A + (size_t)e1 * lda;
  }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;
  // the 16 KB block of the small operand of a step: two 16-byte pieces per thread
  sg_u4 bnext[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) bnext[i] = *reinterpret_cast<const sg_u4*>(tsrc + i * SG_THREADS + tid);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int u = i * SG_THREADS + tid, row = u >> 4, c16 = u & 15;
    *reinterpret_cast<sg_u4*>(sB + row * SGH_BROW4 + c16) = bnext[i];
  }
  sg_f4 nxt0[8], nxt1[8];
  sg_fetch8(nxt0, fptr0, fcol < K ? fcol : K - 4);
  sg_fetch8(nxt1, fptr1, fcol < K ? fcol : K - 4);
  for (int s = 0; s < n_steps; ++s) {
    rb_release_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    const uint4* bbase = sB + (s & 1) * (64 * SGH_BROW4) + hh * 4;
    const int s_next = s + 1 < n_steps ? s + 1 : s;   // (the last step fetches itself again: no branch around loads)
    const int n_next = s_next * 64 + fcol;
    const int next_col = n_next < K ? n_next : K - 4;
#pragma unroll
    for (int i = 0; i < 2; ++i)
      bnext[i] = *reinterpret_cast<const sg_u4*>(tsrc + (size_t)s_next * (64 * 16) + i * SG_THREADS + tid);
    sgh_row_block(sA, bbase, nxt0, fptr0, next_col, frow, fcol, m, hh, a_scale, acc[0][0], acc[0][1]);
    sgh_row_block(sA, bbase, nxt1, fptr1, next_col, frow, fcol, m, hh, a_scale, acc[1][0], acc[1][1]);
    // (after the last step this rewrites a buffer that nobody reads any more)
    uint4* bdst = sB + ((s + 1) & 1) * (64 * SGH_BROW4);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int u = i * SG_THREADS + tid, row = u >> 4, c16 = u & 15;
      *reinterpret_cast<sg_u4*>(bdst + row * SGH_BROW4 + c16) = bnext[i];
    }
  }
}

// ---------------------------------------------------------------------------------------------------------------
// The streaming contraction with wide column tiles: a wave owns one 32-row block of A and NCB column blocks of 32
// (NCB = 2, 4 or 6: up to 192 columns; 8 would not fit the register file), so that a row of A is fetched, turned and cut into pieces once for all of
// them.  With 64-column tiles every tile's workgroup fetched the rows again (from L2, at the same moment as its
// neighbours) and cut them again.  acc[cb] = rows (e_base ..+31) x columns (32 cb ..+31) of the wide tile.
// tsrc: packed blocks of the wide tile's first 64-column tile; the blocks of the next tiles follow at distances of
// tile_stride uint4 (tiles past the last one are read from the last one: the caller does not store their columns).
// The block of the small operand of a step (NCB / 2 tiles of 16 KB) is single-buffered in LDS: loaded into registers
// during step s - 1, written between two barriers at the top of step s.  SG_WAVES waves per workgroup.
// Dynamic LDS: SGHW_LDS_BYTES(NCB).
#define SGHW_LDS_BYTES(NCB) ((size_t)((NCB) / 2) * 64 * SGH_BROW4 * sizeof(uint4) + (size_t)SG_WAVES * 32 * SG_AROW * sizeof(float))
template <int NCB>
__device__ __forceinline__ void sghw_contract(const float* __restrict__ A, long M, int K, int lda,
                                              const uint4* __restrict__ tsrc, long tile_stride, int n_tiles_left,
                                              int n_steps, uint4* smem, long e_base, float a_scale,
                                              float16v (&acc)[NCB]) {
  constexpr int NT = NCB / 2;
  uint4* sB = smem;                                  // [NT * 64][SGH_BROW4]
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  float* sA = reinterpret_cast<float*>(sB + NT * 64 * SGH_BROW4) + (size_t)wave * 32 * SG_AROW;
  const int m = lane & 31, hh = lane >> 5;
  const int frow = lane >> 4, fcol = (lane & 15) * 4;
  const float* fptr[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    long e0 = e_base + 4 * i + frow;
    if (e0 >= M) e0 = M - 1;
    fptr[i] = A + (size_t)e0 * lda;
  }
#pragma unroll
  for (int b = 0; b < NCB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;
  // the 64-column tiles of this wide tile (clamped to the last existing one)
  const uint4* tile[NT];
#pragma unroll
  for (int c = 0; c < NT; ++c) tile[c] = tsrc + (long)(c < n_tiles_left ? c : n_tiles_left - 1) * tile_stride;
  sg_u4 bnext[NT][2];
#pragma unroll
  for (int c = 0; c < NT; ++c)
#pragma unroll
    for (int i = 0; i < 2; ++i) bnext[c][i] = *reinterpret_cast<const sg_u4*>(tile[c] + i * SG_THREADS + tid);
  sg_f4 nxt[8];
  sg_fetch8(nxt, fptr, fcol < K ? fcol : K - 4);
  for (int s = 0; s < n_steps; ++s) {
    rb_release_barrier();                            // every wave has finished reading the block of step s - 1
#pragma unroll
    for (int c = 0; c < NT; ++c)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int u = i * SG_THREADS + tid, row = c * 64 + (u >> 4), c16 = u & 15;
        *reinterpret_cast<sg_u4*>(sB + row * SGH_BROW4 + c16) = bnext[c][i];
      }
    rb_release_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    const int s_next = s + 1 < n_steps ? s + 1 : s;   // (the last step fetches itself again: no branch around loads)
    const int n_next = s_next * 64 + fcol;
    const int next_col = n_next < K ? n_next : K - 4;
    sg_store8(sA + frow * SG_AROW + fcol, nxt);
    sg_fetch8(nxt, fptr, next_col);
#pragma unroll
    for (int c = 0; c < NT; ++c)
#pragma unroll
      for (int i = 0; i < 2; ++i)
        bnext[c][i] = *reinterpret_cast<const sg_u4*>(tile[c] + (size_t)s_next * (64 * 16) + i * SG_THREADS + tid);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
    const float4* arow = reinterpret_cast<const float4*>(sA + m * SG_AROW + hh * 32);
    const uint4* bbase = sB + hh * 4;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float4 u = arow[2 * t], v = arow[2 * t + 1];
      const float xv[8] = {u.x, u.y, u.z, u.w, v.x, v.y, v.z, v.w};
      // the first pair of column blocks' pieces of the small operand are requested before A is cut, every further
      // pair before the products of the pair in front of it: their LDS latency passes behind other work
      uint4 b0[2], b1[2];
      {
        const uint4* brow0 = bbase + m * SGH_BROW4 + t;
        const uint4* brow1 = brow0 + 32 * SGH_BROW4;
        b0[0] = brow0[0]; b0[1] = brow0[8]; b1[0] = brow1[0]; b1[1] = brow1[8];
      }
      uint4 ah, al;
      sgh_split8(xv, a_scale, ah, al);
#pragma unroll
      for (int cb = 0; cb < NCB; cb += 2) {
        uint4 n0[2], n1[2];
        if (cb + 2 < NCB) {
          const uint4* brow0 = bbase + ((cb + 2) * 32 + m) * SGH_BROW4 + t;
          const uint4* brow1 = brow0 + 32 * SGH_BROW4;
          n0[0] = brow0[0]; n0[1] = brow0[8]; n1[0] = brow1[0]; n1[1] = brow1[8];
        }
        sgh_mma3x2(ah, al, b0, b1, acc[cb], acc[cb + 1]);
        if (cb + 2 < NCB) { b0[0] = n0[0]; b0[1] = n0[1]; b1[0] = n1[0]; b1[1] = n1[1]; }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();   // reads of the tile are done before the next step overwrites it
  }
}
