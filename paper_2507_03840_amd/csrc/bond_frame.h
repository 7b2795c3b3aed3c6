// Device helpers: rotation of degree-l feature blocks into and out of the bond-aligned frame.
//
// The tensor product with the spherical harmonics of the edge direction (Sec. 2.1, 2.2, Eq. 1) is
// evaluated in a frame where the edge lies on the polar axis (the SO(2) reduction of Sec. 2.1 /
// Fig. 2(d)).  With r_hat = (sin t cos p, sin t sin p, cos t) the rotation R = R_y(-t) R_z(-p) takes
// r_hat to z_hat, and for every degree D(R) = J^T Z(-t) J Z(-p), where Z(a) mixes the (+m, -m)
// components by the angle m*a and J is a constant matrix (generated file).  Everything lives in
// registers: a lane handles one channel of one edge.
#pragma once
#include <hip/hip_runtime.h>
#include "egnn_gen.inc"

template <int L> __device__ __forceinline__ void egnn_apply_J(float* v);
template <int L> __device__ __forceinline__ void egnn_apply_Jt(float* v);
template <> __device__ __forceinline__ void egnn_apply_J<0>(float*) {}
template <> __device__ __forceinline__ void egnn_apply_Jt<0>(float*) {}
template <> __device__ __forceinline__ void egnn_apply_J<1>(float* v) { egnn_apply_J1(v); }
template <> __device__ __forceinline__ void egnn_apply_Jt<1>(float* v) { egnn_apply_Jt1(v); }
template <> __device__ __forceinline__ void egnn_apply_J<2>(float* v) { egnn_apply_J2(v); }
template <> __device__ __forceinline__ void egnn_apply_Jt<2>(float* v) { egnn_apply_Jt2(v); }
template <> __device__ __forceinline__ void egnn_apply_J<3>(float* v) { egnn_apply_J3(v); }
template <> __device__ __forceinline__ void egnn_apply_Jt<3>(float* v) { egnn_apply_Jt3(v); }
template <> __device__ __forceinline__ void egnn_apply_J<4>(float* v) { egnn_apply_J4(v); }
template <> __device__ __forceinline__ void egnn_apply_Jt<4>(float* v) { egnn_apply_Jt4(v); }

// cos(m a), sin(m a) for m = 1..4 of the azimuth (p) and polar (t) angle of a unit vector.
struct BondTrig {
  float cp[5], sp[5], ct[5], st[5];
};

template <int LMAX>
__device__ __forceinline__ void egnn_bond_trig(float x, float y, float z, BondTrig& t) {
  const float rho2 = x * x + y * y;
  const float rho = sqrtf(rho2);
  const float inv = rho2 > 1e-30f ? 1.0f / rho : 0.0f;
  const float c1 = rho2 > 1e-30f ? x * inv : 1.0f;
  const float s1 = y * inv;
  t.cp[0] = 1.0f; t.sp[0] = 0.0f; t.ct[0] = 1.0f; t.st[0] = 0.0f;
  if (LMAX >= 1) { t.cp[1] = c1; t.sp[1] = s1; t.ct[1] = z; t.st[1] = rho; }
#pragma unroll
  for (int m = 2; m <= LMAX; ++m) {
    t.cp[m] = t.cp[m - 1] * c1 - t.sp[m - 1] * s1;
    t.sp[m] = t.sp[m - 1] * c1 + t.cp[m - 1] * s1;
    t.ct[m] = t.ct[m - 1] * z - t.st[m - 1] * rho;
    t.st[m] = t.st[m - 1] * z + t.ct[m - 1] * rho;
  }
}

// v <- Z(a) v (NEG = false) or Z(-a) v (NEG = true) on one degree-L block, c[m] = cos(m a), s[m] = sin(m a).
template <int L, bool NEG>
__device__ __forceinline__ void egnn_zrot(float* v, const float* c, const float* s) {
#pragma unroll
  for (int m = 1; m <= L; ++m) {
    const float a = v[L + m], b = v[L - m];
    const float sm = NEG ? -s[m] : s[m];
    v[L + m] = c[m] * a - sm * b;
    v[L - m] = sm * a + c[m] * b;
  }
}

template <int L>
__device__ __forceinline__ void egnn_to_bond_frame_l(float* v, const BondTrig& t) {
  egnn_zrot<L, true>(v, t.cp, t.sp);
  egnn_apply_J<L>(v);
  egnn_zrot<L, true>(v, t.ct, t.st);
  egnn_apply_Jt<L>(v);
}

template <int L>
__device__ __forceinline__ void egnn_from_bond_frame_l(float* v, const BondTrig& t) {
  egnn_apply_J<L>(v);
  egnn_zrot<L, false>(v, t.ct, t.st);
  egnn_apply_Jt<L>(v);
  egnn_zrot<L, false>(v, t.cp, t.sp);
}

// all degrees 0..LMAX of a flattened (l, m) vector
template <int LMAX>
__device__ __forceinline__ void egnn_to_bond_frame(float* v, const BondTrig& t) {
  if (LMAX >= 1) egnn_to_bond_frame_l<1>(v + 1, t);
  if (LMAX >= 2) egnn_to_bond_frame_l<2>(v + 4, t);
  if (LMAX >= 3) egnn_to_bond_frame_l<3>(v + 9, t);
  if (LMAX >= 4) egnn_to_bond_frame_l<4>(v + 16, t);
}

template <int LMAX>
__device__ __forceinline__ void egnn_from_bond_frame(float* v, const BondTrig& t) {
  if (LMAX >= 1) egnn_from_bond_frame_l<1>(v + 1, t);
  if (LMAX >= 2) egnn_from_bond_frame_l<2>(v + 4, t);
  if (LMAX >= 3) egnn_from_bond_frame_l<3>(v + 9, t);
  if (LMAX >= 4) egnn_from_bond_frame_l<4>(v + 16, t);
}

template <int LMAX> struct LayerMid;
template <> struct LayerMid<0> { using T = TpMid_0_0_0; };
template <> struct LayerMid<1> { using T = TpMid_1_1_1; };
template <> struct LayerMid<2> { using T = TpMid_2_2_2; };
template <> struct LayerMid<3> { using T = TpMid_3_3_3; };
template <> struct LayerMid<4> { using T = TpMid_4_4_4; };
template <int LMAX> struct ReadoutMid;
template <> struct ReadoutMid<0> { using T = TpMid_0_0_4; };
template <> struct ReadoutMid<1> { using T = TpMid_1_1_4; };
template <> struct ReadoutMid<2> { using T = TpMid_2_2_4; };
template <> struct ReadoutMid<3> { using T = TpMid_3_3_4; };
template <> struct ReadoutMid<4> { using T = TpMid_4_4_4; };
