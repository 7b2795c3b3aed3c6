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
