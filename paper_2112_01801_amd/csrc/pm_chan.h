// Channel-run access shared by the row-streaming kernels: a lane owns CPL consecutive channels of a row.
#pragma once
#include "pm_device.h"

// CPL consecutive channels of one row, as fp32.  VEC: one 8- or 16-byte access (the caller has checked that
// every run is whole and aligned); else element by element, channels past C read as zero / are not written.
template <bool BF16, int CPL, bool VEC>
__device__ __forceinline__ void chan_load(const void* base, int64_t off, int C, int c0, float (&v)[CPL]) {
  static_assert((BF16 && (CPL == 8 || CPL == 4)) || (!BF16 && CPL == 4), "run width");
  if constexpr (VEC) {
    if constexpr (BF16 && CPL == 8) {
      const uint4 u = *(const uint4*)((const uint16_t*)base + off + c0);
      v[0] = bf16lo_to_f32(u.x); v[1] = bf16hi_to_f32(u.x); v[2] = bf16lo_to_f32(u.y); v[3] = bf16hi_to_f32(u.y);
      v[4] = bf16lo_to_f32(u.z); v[5] = bf16hi_to_f32(u.z); v[6] = bf16lo_to_f32(u.w); v[7] = bf16hi_to_f32(u.w);
    } else if constexpr (BF16) {
      const uint2 u = *(const uint2*)((const uint16_t*)base + off + c0);
      v[0] = bf16lo_to_f32(u.x); v[1] = bf16hi_to_f32(u.x); v[2] = bf16lo_to_f32(u.y); v[3] = bf16hi_to_f32(u.y);
    } else {
      const float4 f = *(const float4*)((const float*)base + off + c0);
      v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      float t = 0.f;
      if (c0 + i < C) t = BF16 ? bf16_to_f32(((const uint16_t*)base)[off + c0 + i]) : ((const float*)base)[off + c0 + i];
      v[i] = t;
    }
  }
}

// CPL fp32 values of one row (the vertex rows dz and the corner scales stay fp32 in both feature dtypes)
template <int CPL, bool VEC>
__device__ __forceinline__ void chan_load_f32(const float* base, int64_t off, int C, int c0, float (&v)[CPL]) {
  if constexpr (VEC) {
#pragma unroll
    for (int q = 0; q < CPL / 4; ++q) {
      const float4 f = *(const float4*)(base + off + c0 + 4 * q);
      v[4 * q] = f.x; v[4 * q + 1] = f.y; v[4 * q + 2] = f.z; v[4 * q + 3] = f.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < CPL; ++i) v[i] = (c0 + i < C) ? base[off + c0 + i] : 0.f;
  }
}

template <bool BF16, int CPL, bool VEC>
__device__ __forceinline__ void chan_store(void* base, int64_t off, int C, int c0, const float (&v)[CPL]) {
  if constexpr (VEC) {
    if constexpr (BF16 && CPL == 8) {
      uint4 u;
      u.x = pack_bf16x2(v[0], v[1]); u.y = pack_bf16x2(v[2], v[3]);
      u.z = pack_bf16x2(v[4], v[5]); u.w = pack_bf16x2(v[6], v[7]);
      *(uint4*)((uint16_t*)base + off + c0) = u;
    } else if constexpr (BF16) {
      uint2 u;
      u.x = pack_bf16x2(v[0], v[1]); u.y = pack_bf16x2(v[2], v[3]);
      *(uint2*)((uint16_t*)base + off + c0) = u;
    } else {
      *(float4*)((float*)base + off + c0) = make_float4(v[0], v[1], v[2], v[3]);
    }
  } else {
#pragma unroll
    for (int i = 0; i < CPL; ++i)
      if (c0 + i < C) {
        if (BF16) ((uint16_t*)base)[off + c0 + i] = (uint16_t)f32_to_bf16_bits(v[i]);
        else ((float*)base)[off + c0 + i] = v[i];
      }
  }
}

// whole, 16-byte aligned channel runs: C a multiple of 8 (bf16) or 4 (fp32) and aligned bases
static inline bool chan_vec_ok(int C, int is_bf16, const void* a, const void* b, const void* c) {
  auto al = [](const void* q) { return (((uintptr_t)q) & 15) == 0; };
  return C % (is_bf16 ? 8 : 4) == 0 && al(a) && al(b) && al(c);
}

