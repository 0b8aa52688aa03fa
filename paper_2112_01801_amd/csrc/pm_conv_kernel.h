// conv_rows kernel template and its per-degree launcher (included by the pm_conv_i*.hip instance files).
#pragma once
#include "pm_rows.h"

#define STAGE_U4 (PM_STAGE_BYTES / 16) /* 512 uint4 per stage */

// ------------------------------------------------------------------------------------------------
// conv_rows
// ------------------------------------------------------------------------------------------------
struct ConvP {
  int64_t R;
  int Cc, Cn, NCH, NBG;
  int resident;          // all stages fit in LDS
  BasisSrc bs;
  RowSrc xs;
  const uint4* apack;
  void* out;
  int out_bf16;
};

template <int DT>
__device__ __forceinline__ uint4 pack_granule(const float* v) {
  uint4 o;
  if constexpr (DT == 1) {
    o.x = pack_bf16x2(v[0], v[1]); o.y = pack_bf16x2(v[2], v[3]);
    o.z = pack_bf16x2(v[4], v[5]); o.w = pack_bf16x2(v[6], v[7]);
  } else {
    o.x = __float_as_uint(v[0]); o.y = __float_as_uint(v[1]);
    o.z = __float_as_uint(v[2]); o.w = __float_as_uint(v[3]);
  }
  return o;
}

// one c-group of the contraction: 16 channels (bf16) or 8 channels (fp32, four k=2 steps)
template <int DT>
__device__ __forceinline__ floatx16 mma_group(uint4 a, uint4 x, floatx16 c) {
  if constexpr (DT == 1) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, x), c, 0,
                                                   0, 0);
  } else {
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(x.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(x.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(x.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(x.w), c, 0, 0, 0);
    return c;
  }
}

template <int DT, int BM, int XM, int LT, int NW, bool RES>
__global__ void __launch_bounds__(NW * 64) k_conv_rows(ConvP p) {
  extern __shared__ uint4 lds[];
  constexpr int K = (BM == B_ONE) ? 1 : (LT + 1) * (LT + 1);
  constexpr int NT = NW * 64;
  constexpr int EPG = (DT == 1) ? 8 : 4;       // channels per 16-byte granule
  constexpr int PER_T = STAGE_U4 / NT;         // uint4 per thread per stage copy
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int NCH = p.NCH, NBG = p.NBG;
  const int64_t S = (int64_t)NBG * NCH * K;
  const int64_t n_tiles = (p.R + NT - 1) / NT;
  // XCD-aware order: workgroup b runs on XCD b%8; give every XCD one contiguous band of tiles so rows
  // gathered by neighbouring tiles meet in the same L2.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, wg_per_xcd = gridDim.x >> 3;
  const int64_t tpx = (n_tiles + 7) / 8;

  if constexpr (RES) {
    for (int64_t i = tid; i < S * STAGE_U4; i += NT) lds[i] = p.apack[i];
    __syncthreads();
  }

  for (int64_t ti = slot; ti < tpx; ti += wg_per_xcd) {
    const int64_t tile = (int64_t)xcd * tpx + ti;
    const bool tile_ok = tile < n_tiles;
    const int64_t r0 = tile * NT + wave * 64;
    int64_t row[2];
    bool ok[2];
    RowMeta meta[2];
    float B[2][K];
#pragma unroll
    for (int fb = 0; fb < 2; ++fb) {
      row[fb] = r0 + fb * 32 + l32;
      ok[fb] = tile_ok && row[fb] < p.R;
      load_meta<XM>(p.xs, row[fb], ok[fb], meta[fb]);
      if constexpr (BM != B_ONE) {
        float x = 0.f, y = 0.f, z = 1.f;
        if (ok[fb]) row_direction<BM>(p.bs, row[fb], x, y, z);
        sh_eval<LT>(x, y, z, p.bs.sh, [&](int k, float v) { B[fb][k] = v; });
      } else {
        B[fb][0] = 1.f;
      }
    }

    if constexpr (!RES) {  // prologue of the weight stream for this tile
#pragma unroll
      for (int i = 0; i < PER_T; ++i) lds[i * NT + tid] = p.apack[i * NT + tid];
      __syncthreads();
    }
    int64_t q = 0;  // stage sequence number inside this tile
    for (int nbg = 0; nbg < NBG; ++nbg) {
      floatx16 y[PM_NBS][2];
#pragma unroll
      for (int a = 0; a < PM_NBS; ++a)
#pragma unroll
        for (int fb = 0; fb < 2; ++fb)
#pragma unroll
          for (int i = 0; i < 16; ++i) y[a][fb][i] = 0.f;

      for (int ch = 0; ch < NCH; ++ch) {
        uint4 X[2][PM_GC];
#pragma unroll
        for (int fb = 0; fb < 2; ++fb)
#pragma unroll
          for (int g = 0; g < PM_GC; ++g) {
            float v[EPG];
            fetch_vals<XM, EPG>(p.xs, row[fb], ok[fb], meta[fb], ((ch * PM_GC + g) * 2 + hh) * EPG, v);
            X[fb][g] = pack_granule<DT>(v);
          }
        // Software pipeline over the chains (k, nbi).  A wave issues in order, so the only way to keep the
        // matrix pipe busy while the SH weighting runs is to interleave, in program order, the MFMAs of
        // chain c with the FMA epilogue of chain c-1 (whose U tiles are "pending" in pu0/pu1): every MFMA
        // is followed by four of the pending FMAs, and sched_barrier keeps that written order.  The A
        // fragments of chain c+1 are read from LDS while chain c computes.
        floatx16 pu0, pu1;
        float pb0 = 0.f, pb1 = 0.f;
        uint4 afr[PM_GC];  // A fragments of the chain about to run
        if constexpr (RES) {
#pragma unroll
          for (int g = 0; g < PM_GC; ++g) afr[g] = lds[q * STAGE_U4 + g * 64 + lane];
        }
#pragma unroll
        for (int k = 0; k < K; ++k, ++q) {
          asm volatile("" ::: "memory");  // keep LDS reads of later stages from being hoisted up here
          const uint4* stage;
          uint4 pre[PER_T];
          if constexpr (RES) {
            stage = lds + q * STAGE_U4;
          } else {
            stage = lds + (q & 1) * STAGE_U4;
            if (q + 1 < S) {
#pragma unroll
              for (int i = 0; i < PER_T; ++i) pre[i] = p.apack[(q + 1) * STAGE_U4 + i * NT + tid];
            }
          }
#pragma unroll
          for (int nbi = 0; nbi < PM_NBS; ++nbi) {
            if constexpr (BM == B_ONE) {
#pragma unroll
              for (int g = 0; g < PM_GC; ++g) {
                uint4 a = stage[(nbi * PM_GC + g) * 64 + lane];
                y[nbi][0] = mma_group<DT>(a, X[0][g], y[nbi][0]);
                y[nbi][1] = mma_group<DT>(a, X[1][g], y[nbi][1]);
              }
            } else {
              uint4 ac[PM_GC];
              if constexpr (RES) {
#pragma unroll
                for (int g = 0; g < PM_GC; ++g) ac[g] = afr[g];
                // prefetch the fragments of the next chain (next n-block of this stage, or next stage)
                const bool last_chain = (k == K - 1) && (nbi == PM_NBS - 1);
                if (!last_chain) {
                  const uint4* nxt = (nbi + 1 < PM_NBS) ? stage + (nbi + 1) * PM_GC * 64 : stage + STAGE_U4;
#pragma unroll
                  for (int g = 0; g < PM_GC; ++g) afr[g] = nxt[g * 64 + lane];
                }
              } else {
#pragma unroll
                for (int g = 0; g < PM_GC; ++g) ac[g] = stage[(nbi * PM_GC + g) * 64 + lane];
              }
              const bool have_pending = (k > 0 || nbi > 0);
              const int pn = (nbi == 0) ? PM_NBS - 1 : nbi - 1;
              floatx16 u0, u1;
#pragma unroll
              for (int i = 0; i < 16; ++i) { u0[i] = 0.f; u1[i] = 0.f; }
              __builtin_amdgcn_sched_barrier(0);
#pragma unroll
              for (int g = 0; g < PM_GC; ++g) {
                u0 = mma_group<DT>(ac[g], X[0][g], u0);
                if (have_pending) {
#pragma unroll
                  for (int i = 4 * g; i < 4 * g + 4; ++i) y[pn][0][i] += pb0 * pu0[i];
                }
                __builtin_amdgcn_sched_barrier(0);
                u1 = mma_group<DT>(ac[g], X[1][g], u1);
                if (have_pending) {
#pragma unroll
                  for (int i = 4 * g; i < 4 * g + 4; ++i) y[pn][1][i] += pb1 * pu1[i];
                }
                __builtin_amdgcn_sched_barrier(0);
              }
              if (have_pending) asm volatile("" : "+v"(y[pn][0]), "+v"(y[pn][1]));
              pu0 = u0; pu1 = u1;
              pb0 = B[0][k]; pb1 = B[1][k];
            }
          }
          if constexpr (!RES) {
            if (q + 1 < S) {
#pragma unroll
              for (int i = 0; i < PER_T; ++i) lds[((q + 1) & 1) * STAGE_U4 + i * NT + tid] = pre[i];
            }
            __syncthreads();
          }
        }
        if constexpr (BM != B_ONE) {  // drain the pipeline
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            y[PM_NBS - 1][0][i] += pb0 * pu0[i];
            y[PM_NBS - 1][1][i] += pb1 * pu1[i];
          }
          asm volatile("" : "+v"(y[PM_NBS - 1][0]), "+v"(y[PM_NBS - 1][1]));
        }
      }

      // store the NBS x 32 output channels of this pass
#pragma unroll
      for (int nbi = 0; nbi < PM_NBS; ++nbi)
#pragma unroll
        for (int fb = 0; fb < 2; ++fb) {
          if (!ok[fb]) continue;
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int n0 = (nbg * PM_NBS + nbi) * 32 + q4 * 8 + hh * 4;
            if (n0 >= p.Cn) continue;
            const float v0 = y[nbi][fb][q4 * 4], v1 = y[nbi][fb][q4 * 4 + 1], v2 = y[nbi][fb][q4 * 4 + 2],
                        v3 = y[nbi][fb][q4 * 4 + 3];
            const int64_t o = row[fb] * (int64_t)p.Cn + n0;
            if (n0 + 4 <= p.Cn && (p.Cn & 3) == 0) {
              if (p.out_bf16) {
                uint2 w;
                w.x = pack_bf16x2(v0, v1); w.y = pack_bf16x2(v2, v3);
                *(uint2*)((uint16_t*)p.out + o) = w;
              } else {
                *(float4*)((float*)p.out + o) = make_float4(v0, v1, v2, v3);
              }
            } else {
              const float vv[4] = {v0, v1, v2, v3};
#pragma unroll
              for (int i = 0; i < 4; ++i)
                if (n0 + i < p.Cn) {
                  if (p.out_bf16) ((uint16_t*)p.out)[o + i] = (uint16_t)f32_to_bf16_bits(vv[i]);
                  else ((float*)p.out)[o + i] = vv[i];
                }
            }
          }
        }
    }
  }
}

template <int DT, int BM, int XM, int LT, int NW, bool RES>
static pm_status launch_conv_res(const ConvP& p, int64_t S, hipStream_t st) {
  auto kern = k_conv_rows<DT, BM, XM, LT, NW, RES>;
  size_t lds = RES ? (size_t)S * PM_STAGE_BYTES : 2 * (size_t)PM_STAGE_BYTES;
  PM_CHECK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const int NT = NW * 64;
  int64_t n_tiles = (p.R + NT - 1) / NT;
  int64_t grid = n_tiles < 256 ? (n_tiles + 7) / 8 * 8 : 256;
  { ProfScope ps__(st, "k_conv_rows");
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), lds, st, p); }
  PM_CHECK_LAUNCH("k_conv_rows");
  return PM_OK;
}

template <int DT, int BM, int XM, int LT, int NW>
static pm_status launch_conv_inst(const ConvP& p, int64_t S, hipStream_t st) {
  if (p.resident) return launch_conv_res<DT, BM, XM, LT, NW, true>(p, S, st);
  return launch_conv_res<DT, BM, XM, LT, NW, false>(p, S, st);
}

template <int DT, int BM, int XM>
static pm_status launch_conv_L(const ConvP& p, int L, int64_t S, hipStream_t st) {
  if constexpr (BM == B_ONE) {
    return launch_conv_inst<DT, BM, XM, 0, 8>(p, S, st);
  } else {
    switch (L) {
      case 0: return launch_conv_inst<DT, BM, XM, 0, 8>(p, S, st);
      case 1: return launch_conv_inst<DT, BM, XM, 1, 8>(p, S, st);
      case 2: return launch_conv_inst<DT, BM, XM, 2, 8>(p, S, st);
      case 3: return launch_conv_inst<DT, BM, XM, 3, 8>(p, S, st);
      case 4: return launch_conv_inst<DT, BM, XM, 4, 4>(p, S, st);
      case 5: return launch_conv_inst<DT, BM, XM, 5, 4>(p, S, st);
      default: return pm_fail(PM_ERR_UNSUPPORTED, "SH degree %d", L);
    }
  }
}


// One instance file defines one of these (both residency variants, all degrees).
#define PM_CONV_INSTANCE(DT, BM, XM)                                                                   \
  pm_status pm_conv_dispatch_##DT##_##BM##_##XM(const ConvP& p, int L, int64_t S, hipStream_t st) {    \
    return launch_conv_L<DT, BM, XM>(p, L, S, st);                                                     \
  }
#define PM_CONV_DECLARE(DT, BM, XM) \
  pm_status pm_conv_dispatch_##DT##_##BM##_##XM(const ConvP& p, int L, int64_t S, hipStream_t st);
