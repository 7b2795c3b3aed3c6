// Exact three-piece bf16 splitting of fp32 values for the matrix cores.
//
// x = hi + mid + lo with every piece a bf16 (8 significant bits): hi = x truncated, mid = (x - hi) truncated,
// lo = (x - hi - mid) truncated; the subtractions are exact.  A product a*b is then the sum of nine piece
// products, of which the six with weight >= 2^-16 are kept (error ~3 * 2^-24 relative).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float float16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct Split3 { uint32_t hi, mid, lo; };   // each: a bf16 in the upper 16 bits

__device__ __forceinline__ Split3 split3(float x) {
  Split3 r;
  r.hi = __float_as_uint(x) & 0xffff0000u;
  const float r1 = x - __uint_as_float(r.hi);
  r.mid = __float_as_uint(r1) & 0xffff0000u;
  const float r2 = r1 - __uint_as_float(r.mid);
  r.lo = __float_as_uint(r2) & 0xffff0000u;
  return r;
}

__device__ __forceinline__ uint32_t pack2(uint32_t even, uint32_t odd) { return (even >> 16) | odd; }

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

