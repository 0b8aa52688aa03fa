// Device-side helpers shared by the picassomesh kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "picassomesh.h"

#define PM_MAX_K ((PM_MAX_L + 1) * (PM_MAX_L + 1))
#define PM_NLM ((PM_MAX_L + 1) * (PM_MAX_L + 2) / 2)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Normalisation constants of Eq. 3, N[l(l+1)/2 + m] for m >= 0 (times sqrt(2) for m > 0 in the
// orthonormal variant); filled on the host in double precision and passed by value to kernels.
struct ShTable {
  float N[PM_NLM];
  int L;
};

__device__ __forceinline__ bool pm_aligned16_dev(const void* p) { return (((uintptr_t)p) & 15u) == 0; }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
// round-to-nearest-even (inputs are finite)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

// Unit facet normal by the right-hand rule on the stored corner order, (x2-x1) x (x3-x1).
// A (near-)degenerate facet, squared cross-product length < 1e-30, takes (0,0,1).
// Cross product and squared length with their multiply-adds written out.  Directions and basis values are evaluated
// in several kernels (and in several copies of a kernel's code); left to the compiler's contraction, which products
// are fused differs from copy to copy, and the same facet gets basis values that differ in the last bit.  With the
// fused operations explicit (and contraction off in these functions) every copy computes the same bits.
__device__ __forceinline__ void cross_fixed(float ux, float uy, float uz, float wx, float wy, float wz, float& cx,
                                            float& cy, float& cz) {
#pragma clang fp contract(off)
  cx = fmaf(uy, wz, -(uz * wy));
  cy = fmaf(uz, wx, -(ux * wz));
  cz = fmaf(ux, wy, -(uy * wx));
}
// a - b rounded once, never contracted with a product that made a (which some copies of a code would do and others not)
__device__ __forceinline__ float sub_fixed(float a, float b) {
#pragma clang fp contract(off)
  return a - b;
}
__device__ __forceinline__ float norm2_fixed(float x, float y, float z) {
#pragma clang fp contract(off)
  return fmaf(x, x, fmaf(y, y, z * z));
}

__device__ __forceinline__ void facet_normal(const float* __restrict__ vert, int v0, int v1, int v2, float& nx,
                                             float& ny, float& nz) {
  const float* a = vert + 3 * (int64_t)v0;
  const float* b = vert + 3 * (int64_t)v1;
  const float* c = vert + 3 * (int64_t)v2;
  float ax = a[0], ay = a[1], az = a[2];
  float ux = b[0] - ax, uy = b[1] - ay, uz = b[2] - az;
  float wx = c[0] - ax, wy = c[1] - ay, wz = c[2] - az;
  float cx, cy, cz;
  cross_fixed(ux, uy, uz, wx, wy, wz, cx, cy, cz);
  float l2 = norm2_fixed(cx, cy, cz);
  if (l2 < 1e-30f) {
    nx = 0.f; ny = 0.f; nz = 1.f;
  } else {
    float r = 1.0f / sqrtf(l2);
    nx = cx * r; ny = cy * r; nz = cz * r;
  }
}

__device__ __forceinline__ void normalize_dir(float& x, float& y, float& z) {
  float l2 = norm2_fixed(x, y, z);
  float r = 1.0f / sqrtf(l2);
  x *= r; y *= r; z *= r;
}

// Real SH basis of Eq. 4 at a UNIT direction (x,y,z), in Cartesian form:
//   N_lm P_l^m(cos t) cos(m phi) = N_lm Q_l^m(z) Re (x+iy)^m,   sin part: Im (x+iy)^m,
// where Q_l^m(z) = d^m P_l / dz^m (the associated Legendre function without the Condon-Shortley
// phase is P_l^m = sin^m(t) Q_l^m).  Q obeys the same three-term recurrence in l as P_l^m.
// sink(k, value) receives every k = l(l+1)+m once; nothing is kept in an indexed array.
// LT >= 0 fixes the degree at compile time (loops unroll, k is a constant in every sink call);
// LT < 0 takes the degree from the table at run time.
template <int LT, class Sink>
__device__ __forceinline__ void sh_eval(float x, float y, float z, const ShTable& T, Sink sink) {
#pragma clang fp contract(off)
  // (the multiply-adds below are explicit: every copy of this code, in whichever kernel, gives the same bits)
  const int L = (LT >= 0) ? LT : T.L;
  float cm = 1.f, sm = 0.f;  // Re, Im of (x+iy)^m
  float qmm = 1.f;           // Q_m^m = (2m-1)!!
#pragma unroll
  for (int m = 0; m <= L; ++m) {
    if (m > 0) {
      float c2 = fmaf(cm, x, -(sm * y));
      sm = fmaf(cm, y, sm * x);
      cm = c2;
      qmm *= (float)(2 * m - 1);
    }
    float q0 = qmm, q1 = 0.f;
#pragma unroll
    for (int l = m; l <= L; ++l) {
      float q;
      if (l == m) {
        q = q0;
      } else if (l == m + 1) {
        q1 = (float)(2 * m + 1) * z * q0;
        q = q1;
      } else {
        q = fmaf(-(float)(l + m - 1), q0, (float)(2 * l - 1) * z * q1) / (float)(l - m);
        q0 = q1;
        q1 = q;
      }
      float v = T.N[l * (l + 1) / 2 + m] * q;
      sink(l * (l + 1) + m, v * cm);
      if (m > 0) sink(l * (l + 1) - m, v * sm);
    }
  }
}

// The degree taken from the table, evaluated by the unrolled code of that degree (a wave-uniform branch): the
// run-time-degree loops of sh_eval<-1> cost several times the instructions of the unrolled recurrence.
template <class Sink>
__device__ __forceinline__ void sh_eval_any(float x, float y, float z, const ShTable& T, Sink sink) {
  switch (T.L) {
    case 0: sh_eval<0>(x, y, z, T, sink); break;
    case 1: sh_eval<1>(x, y, z, T, sink); break;
    case 2: sh_eval<2>(x, y, z, T, sink); break;
    case 3: sh_eval<3>(x, y, z, T, sink); break;
    case 4: sh_eval<4>(x, y, z, T, sink); break;
    case 5: sh_eval<5>(x, y, z, T, sink); break;
    default: sh_eval<-1>(x, y, z, T, sink); break;
  }
}
