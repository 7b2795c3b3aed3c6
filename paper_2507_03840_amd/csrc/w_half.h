// Half-precision storage of the per-edge path weights w[k][p][c] (an option: storage only, every product and sum
// stays in fp32).
//
// The kernel that produces w holds, per matrix-core block, one output column n = p*E + c per lane (32 columns per
// block), so two neighbouring blocks give one full 32-bit word per lane.  Row k of the stored tensor is therefore a
// sequence of groups of 32 words, one group per 64 columns: word m of group j carries column 64j + m in its low
// half and column 64j + 32 + m in its high half.  Stores and loads are then whole 128-byte lines, as with fp32.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

__host__ __device__ inline int w_half_row_words(int PE) { return ((PE + 63) >> 6) * 32; }

__device__ __forceinline__ uint32_t w_half_bits(float x) {   // round to nearest even
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
}
__device__ __forceinline__ float w_half_lo(uint32_t word) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)(word & 0xffffu));
}
__device__ __forceinline__ float w_half_hi(uint32_t word) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)(word >> 16));
}

// The P weights of channel c of one edge (row = first word of the edge's row), E = 2^LE channels.
template <int P, int LE>
__device__ __forceinline__ void w_half_load(const uint32_t* __restrict__ row, int c, float* wr) {
  constexpr int E = 1 << LE;
  if constexpr (LE <= 5) {
    // a group of 64 columns holds 64/E paths; paths q and q + 32/E of a group share their words
    constexpr int PG = 64 / E, Q = 32 / E;
    constexpr int NG = (P + PG - 1) / PG;
#pragma unroll
    for (int j = 0; j < NG; ++j)
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        const int p_lo = j * PG + q, p_hi = p_lo + Q;
        if (p_lo < P) {
          const uint32_t word = __builtin_nontemporal_load(row + j * 32 + q * E + c);
          wr[p_lo] = w_half_lo(word);
          if (p_hi < P) wr[p_hi] = w_half_hi(word);
        }
      }
  } else {
    // a path spans E/64 groups; lanes c and c + 32 of a 64-channel stretch share their words
    const int off = ((c >> 6) << 5) + (c & 31);
    const uint32_t sh = (c & 32) ? 16u : 0u;
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const uint32_t word = __builtin_nontemporal_load(row + p * (E / 2) + off);
      wr[p] = w_half_lo(word >> sh);
    }
  }
}
