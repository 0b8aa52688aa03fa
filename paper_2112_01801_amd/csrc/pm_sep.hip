// Depth-wise stage of the separable facet2vertex convolution (Section "Mesh convolutions": Eq. 5 with one
// scalar SH coefficient set per channel), forward and backward:
//     y_f[c]  = h_f[c] * s_f[c],            s_f[c] = sum_k alpha[k][c] B_k(n_f)
//     dh_f[c] = dy_f[c] * s_f[c],           dy_f[c] = sum_j dz[v_j(f)][c] / deg(v_j(f))    (dz in fp32)
//     dalpha[k][c] = sum_f B_k(n_f) h_f[c] dy_f[c]
// Bound by HBM (one row read, one written per facet).  A group of lanes owns a facet row, each lane a run of
// channels; a block walks its rows four per group at a time so that a coefficient fetched from LDS serves
// four rows.  The SH basis of the block's rows is evaluated once per row (one thread each) into LDS.
// dalpha is reduced without atomics: every lane group accumulates its rows in registers (a fixed
// assignment of rows to groups) and writes its own slice; the slices are added in a fixed order.
// The tail of the file holds the small fold/unfold kernels of the separable vertex2facet form (Eq. 6).
#include "pm_rows.h"

#define SEP_RPG 4      /* rows a lane group handles per step */
#define SEP_KC 16      /* basis functions per pass of the backward kernel (register accumulators) */

struct SepP {
  int64_t F;
  int K, C, lpg;          // lanes per row group (power of two), each lane CPL channels per step
  int is_bf16;
  BasisSrc bs;            // vert / facet / sh table
  const void* h;          // [F][C]
  const float* alpha;     // [K][C]
  void* y;                // fwd: [F][C]   bwd: dh [F][C] (may be NULL)
  const float* dz;        // bwd: [V][C] fp32
  const int32_t* row_ptr; // bwd: vertex degrees
  float* partial;         // bwd: [slices][K][C]
  int kc0;                // bwd: first k of this pass
  int want_dalpha;
};

template <bool BF16>
__device__ __forceinline__ void sep_load(const void* base, int64_t off, int C, int c0, float (&v)[BF16 ? 8 : 4]) {
  constexpr int CPL = BF16 ? 8 : 4;
  if (c0 + CPL <= C && ((((uintptr_t)base) + (uint64_t)(off + c0) * (BF16 ? 2 : 4)) & 15) == 0) {
    if constexpr (BF16) {
      const uint4 u = *(const uint4*)((const uint16_t*)base + off + c0);
      v[0] = bf16lo_to_f32(u.x); v[1] = bf16hi_to_f32(u.x); v[2] = bf16lo_to_f32(u.y); v[3] = bf16hi_to_f32(u.y);
      v[4] = bf16lo_to_f32(u.z); v[5] = bf16hi_to_f32(u.z); v[6] = bf16lo_to_f32(u.w); v[7] = bf16hi_to_f32(u.w);
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

// CPL fp32 values of one row (the vertex rows dz stay fp32 in both feature dtypes)
template <int CPL>
__device__ __forceinline__ void sep_load_f32(const float* base, int64_t off, int C, int c0, float (&v)[CPL]) {
  if (c0 + CPL <= C && ((((uintptr_t)base) + (uint64_t)(off + c0) * 4) & 15) == 0) {
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

template <bool BF16>
__device__ __forceinline__ void sep_store(void* base, int64_t off, int C, int c0, const float (&v)[BF16 ? 8 : 4]) {
  constexpr int CPL = BF16 ? 8 : 4;
  if (c0 + CPL <= C && ((((uintptr_t)base) + (uint64_t)(off + c0) * (BF16 ? 2 : 4)) & 15) == 0) {
    if constexpr (BF16) {
      uint4 u;
      u.x = pack_bf16x2(v[0], v[1]); u.y = pack_bf16x2(v[2], v[3]);
      u.z = pack_bf16x2(v[4], v[5]); u.w = pack_bf16x2(v[6], v[7]);
      *(uint4*)((uint16_t*)base + off + c0) = u;
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

// LDS: alpha [kn][lanes per group * channels per lane] (this pass's k range, one channel run), basis [rows per step][kn]
template <bool BF16, bool BWD>
__global__ void __launch_bounds__(256) k_dw_f2v(SepP p) {
  extern __shared__ float sep_lds[];
  constexpr int CPL = BF16 ? 8 : 4;
  const int tid = threadIdx.x;
  const int G = 256 / p.lpg;                 // lane groups per block
  const int grp = tid / p.lpg, sub = tid % p.lpg;
  const int rows_step = G * SEP_RPG;         // rows per block step (<= 256)
  const int RW = p.lpg * CPL;                // channels per run: one run is resident in LDS at a time
  const int k0 = BWD ? p.kc0 : 0;
  // basis functions handled in this launch: all of them, or one chunk when dalpha accumulates in registers
  const int kn = (BWD && p.want_dalpha) ? min(SEP_KC, p.K - k0) : p.K;
  float* A = sep_lds;                        // [kn][RW]
  float* Bs = sep_lds + (size_t)kn * RW;     // [rows_step][kn]
  const int nchunk = (p.C + RW - 1) / RW;    // channel runs per lane (1 unless C > 64 * CPL)

  // backward: this group's dalpha accumulators for one channel run at a time
  for (int cr = 0; cr < nchunk; ++cr) {
    const int c0 = (cr * p.lpg + sub) * CPL;
    __syncthreads();                          // the previous run's coefficients are no longer needed
    for (int i = tid; i < kn * RW; i += 256) {
      const int k = i / RW, c = cr * RW + (i - k * RW);
      A[i] = (c < p.C) ? p.alpha[(int64_t)(k0 + k) * p.C + c] : 0.f;
    }
    float da[BWD ? SEP_KC : 1][CPL];
    if constexpr (BWD) {
#pragma unroll
      for (int k = 0; k < SEP_KC; ++k)
#pragma unroll
        for (int i = 0; i < CPL; ++i) da[k][i] = 0.f;
    }
    for (int64_t r0 = (int64_t)blockIdx.x * rows_step; r0 < p.F; r0 += (int64_t)gridDim.x * rows_step) {
      __syncthreads();                        // the previous step's basis rows are no longer needed
      if (tid < rows_step) {
        const int64_t r = r0 + tid;
        if (r < p.F) {
          float x, y, z;
          row_direction<B_NORMAL>(p.bs, r, x, y, z);
          sh_eval<-1>(x, y, z, p.bs.sh, [&](int k, float v) {
            const int kl = k - k0;
            if (kl >= 0 && kl < kn) Bs[tid * kn + kl] = v;
          });
        }
      }
      __syncthreads();
      // this group's rows of the step: grp * SEP_RPG + q
      float hv[SEP_RPG][CPL], s[SEP_RPG][CPL], dyv[SEP_RPG][CPL];
      bool ok[SEP_RPG];
#pragma unroll
      for (int q = 0; q < SEP_RPG; ++q) {
        const int64_t r = r0 + grp * SEP_RPG + q;
        ok[q] = r < p.F && c0 < p.C;
#pragma unroll
        for (int i = 0; i < CPL; ++i) { hv[q][i] = 0.f; s[q][i] = 0.f; dyv[q][i] = 0.f; }
        if (ok[q]) {
          sep_load<BF16>(p.h, r * p.C, p.C, c0, hv[q]);
          if constexpr (BWD) {
#pragma unroll
            for (int j = 0; j < 3; ++j) {
              const int32_t v = p.bs.facet[3 * r + j];
              const float w = 1.0f / (float)(p.row_ptr[v + 1] - p.row_ptr[v]);
              float t[CPL];
              sep_load_f32<CPL>(p.dz, (int64_t)v * p.C, p.C, c0, t);
#pragma unroll
              for (int i = 0; i < CPL; ++i) dyv[q][i] += t[i] * w;
            }
          }
        }
      }
      if (c0 < p.C) {
        for (int k = 0; k < kn; ++k) {
          float a[CPL];
#pragma unroll
          for (int i = 0; i < CPL; ++i) a[i] = A[k * RW + sub * CPL + i];
#pragma unroll
          for (int q = 0; q < SEP_RPG; ++q) {
            const float b = Bs[(grp * SEP_RPG + q) * kn + k];
#pragma unroll
            for (int i = 0; i < CPL; ++i) s[q][i] += a[i] * b;
          }
        }
      }
      if constexpr (BWD) {
        if (c0 < p.C && p.want_dalpha) {
#pragma unroll
          for (int k = 0; k < SEP_KC; ++k) {
            if (k < kn) {
#pragma unroll
              for (int q = 0; q < SEP_RPG; ++q) {
                const float b = ok[q] ? Bs[(grp * SEP_RPG + q) * kn + k] : 0.f;
#pragma unroll
                for (int i = 0; i < CPL; ++i) da[k][i] += b * (hv[q][i] * dyv[q][i]);
              }
            }
          }
        }
      }
#pragma unroll
      for (int q = 0; q < SEP_RPG; ++q) {
        if (!ok[q]) continue;
        const int64_t r = r0 + grp * SEP_RPG + q;
        float o[CPL];
        if constexpr (BWD) {
          // the whole filter value is needed for dh: only a launch that covers every k writes it
          if (p.y && kn == p.K) {
#pragma unroll
            for (int i = 0; i < CPL; ++i) o[i] = dyv[q][i] * s[q][i];
            sep_store<BF16>(p.y, r * p.C, p.C, c0, o);
          }
        } else {
#pragma unroll
          for (int i = 0; i < CPL; ++i) o[i] = hv[q][i] * s[q][i];
          sep_store<BF16>(p.y, r * p.C, p.C, c0, o);
        }
      }
    }
    if constexpr (BWD) {
      if (p.want_dalpha && c0 < p.C) {
        float* dst = p.partial + ((int64_t)blockIdx.x * G + grp) * p.K * p.C;
#pragma unroll
        for (int k = 0; k < SEP_KC; ++k)
          if (k < kn) {
#pragma unroll
            for (int i = 0; i < CPL; ++i)
              if (c0 + i < p.C) dst[(int64_t)(k0 + k) * p.C + c0 + i] = da[k][i];
          }
      }
    }
  }
}

static void sep_geom(int C, int is_bf16, int* lpg, int* grid, int64_t F) {
  const int cpl = is_bf16 ? 8 : 4;
  int need = (C + cpl - 1) / cpl, l = 1;
  while (l < need && l < 64) l <<= 1;
  if (l < 4) l = 4;      // one thread per row evaluates the basis: at most 256 rows per block step
  *lpg = l;
  const int rows_step = (256 / l) * SEP_RPG;
  int64_t nblk = (F + rows_step - 1) / rows_step;
  if (nblk > 512) nblk = 512;
  if (nblk < 1) nblk = 1;
  *grid = (int)nblk;
}

size_t pm_sep_dalpha_ws_bytes(int64_t F, int K, int C, int is_bf16) {
  int lpg, grid;
  sep_geom(C, is_bf16, &lpg, &grid, F);
  return pm_round_up((size_t)grid * (256 / lpg) * K * C * sizeof(float), 256);
}

static size_t sep_lds_bytes(int kn, int C, int is_bf16, int lpg) {
  (void)C;
  return ((size_t)kn * lpg * (is_bf16 ? 8 : 4) + (size_t)(256 / lpg) * SEP_RPG * kn) * sizeof(float);
}

pm_status pm_launch_dw_f2v(int64_t F, int K, int C, int is_bf16, const BasisSrc& bs, const void* h, const float* alpha,
                           void* y, hipStream_t st) {
  if (F == 0) return PM_OK;
  SepP p;
  p.F = F; p.K = K; p.C = C; p.is_bf16 = is_bf16; p.bs = bs; p.h = h; p.alpha = alpha; p.y = y;
  p.dz = nullptr; p.row_ptr = nullptr; p.partial = nullptr; p.kc0 = 0; p.want_dalpha = 0;
  int grid;
  sep_geom(C, is_bf16, &p.lpg, &grid, F);
  const size_t lds = sep_lds_bytes(K, C, is_bf16, p.lpg);
  auto kern = is_bf16 ? k_dw_f2v<true, false> : k_dw_f2v<false, false>;
  PM_CHECK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  { ProfScope ps__(st, "k_dw_f2v");
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p); }
  PM_CHECK_LAUNCH("k_dw_f2v");
  return PM_OK;
}

// dh [F][C] (may be NULL) and dalpha [K][C] (may be NULL; `partial` must then hold pm_sep_dalpha_ws_bytes)
pm_status pm_launch_dw_f2v_bwd(int64_t F, int K, int C, int is_bf16, const BasisSrc& bs, const void* h,
                               const float* alpha, const float* dz, const int32_t* row_ptr, void* dh, float* dalpha,
                               float* partial, hipStream_t st) {
  SepP p;
  p.F = F; p.K = K; p.C = C; p.is_bf16 = is_bf16; p.bs = bs; p.h = h; p.alpha = alpha; p.y = dh;
  p.dz = dz; p.row_ptr = row_ptr; p.partial = partial; p.want_dalpha = dalpha != nullptr;
  int grid;
  sep_geom(C, is_bf16, &p.lpg, &grid, F);
  auto kern = is_bf16 ? k_dw_f2v<true, true> : k_dw_f2v<false, true>;
  if (F == 0) {
    if (dalpha) return pm_launch_sum_slices(partial, (int64_t)K * C, 0, dalpha, st);   // no slices: zeros
    return PM_OK;
  }
  // dh needs the whole filter value: it comes from the dalpha launch when that covers every k (K <= SEP_KC),
  // else from a launch of its own without dalpha accumulators
  const bool fused = dalpha && K <= SEP_KC;
  if (dh && !fused) {
    p.kc0 = 0; p.want_dalpha = 0; p.y = dh;
    const size_t lds = sep_lds_bytes(K, C, is_bf16, p.lpg);
    PM_CHECK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    { ProfScope ps__(st, "k_dw_f2v_bwd");
      hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p); }
    PM_CHECK_LAUNCH("k_dw_f2v_bwd");
  }
  if (dalpha) {
    p.want_dalpha = 1;
    p.y = fused ? dh : nullptr;
    for (int k0 = 0; k0 < K; k0 += SEP_KC) {
      p.kc0 = k0;
      const int kn = K - k0 < SEP_KC ? K - k0 : SEP_KC;
      const size_t lds = sep_lds_bytes(kn, C, is_bf16, p.lpg);
      PM_CHECK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
      { ProfScope ps__(st, "k_dw_f2v_bwd");
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p); }
      PM_CHECK_LAUNCH("k_dw_f2v_bwd");
    }
    return pm_launch_sum_slices(partial, (int64_t)K * C, grid * (256 / p.lpg), dalpha, st);
  }
  return PM_OK;
}

// ---- separable vertex2facet, backward to the vertex features.  With T_f = dg_f P^T (one row per facet),
//   dh_v[c] = sum over the adjacency entries (f, j) of v of  s_j[c] T_f[c],     s_j[c] = sum_k fc[j][k] alpha[k][c]
// (fc[j][k] is the SH basis at the barycentric corner j, Eq. 6).  A group of lanes owns a vertex, each lane a
// run of channels whose three scales it keeps in registers; entries are taken two at a time in ascending
// order, the corner chosen by selects.
struct SlotP {
  int64_t V;
  int K, C, lpg, out_bf16;
  const void* T;            // [F][C] feature dtype
  const int32_t* row_ptr;   // [V+1]
  const int32_t* col;       // entries 3f + j
  const float* alpha;       // [K][C]
  FoldCoef fc;
  void* out;                // [V][C]
};

template <bool BF16>
__global__ void __launch_bounds__(256) k_slot_scale_sum(SlotP p) {
  constexpr int CPL = BF16 ? 8 : 4;
  const int gpb = 256 / p.lpg;
  const int sub = threadIdx.x % p.lpg;
  for (int c0 = sub * CPL; c0 < p.C; c0 += p.lpg * CPL) {
    float sc[3][CPL];
#pragma unroll
    for (int j = 0; j < 3; ++j)
#pragma unroll
      for (int i = 0; i < CPL; ++i) sc[j][i] = 0.f;
    for (int k = 0; k < p.K; ++k)
#pragma unroll
      for (int i = 0; i < CPL; ++i) {
        const float a = (c0 + i < p.C) ? p.alpha[(int64_t)k * p.C + c0 + i] : 0.f;
#pragma unroll
        for (int j = 0; j < 3; ++j) sc[j][i] += p.fc.c[j][k] * a;
      }
    for (int64_t seg = (int64_t)blockIdx.x * gpb + threadIdx.x / p.lpg; seg < p.V; seg += (int64_t)gridDim.x * gpb) {
      const int32_t b = p.row_ptr[seg], e = p.row_ptr[seg + 1];
      float acc[CPL];
#pragma unroll
      for (int i = 0; i < CPL; ++i) acc[i] = 0.f;
      for (int32_t i0 = b; i0 < e; i0 += 2) {
        int32_t cidx[2], row[2];
        float x[2][CPL];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          cidx[q] = p.col[min(i0 + q, e - 1)];
          row[q] = (int32_t)(((uint64_t)(uint32_t)cidx[q] * 0xAAAAAAABull) >> 33);   // / 3
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) sep_load<BF16>(p.T, (int64_t)row[q] * p.C, p.C, c0, x[q]);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int slot = cidx[q] - 3 * row[q];
          const bool live = i0 + q < e;
#pragma unroll
          for (int i = 0; i < CPL; ++i) {
            const float w = slot == 0 ? sc[0][i] : (slot == 1 ? sc[1][i] : sc[2][i]);
            acc[i] += live ? w * x[q][i] : 0.f;
          }
        }
      }
      if (p.out_bf16) {
        if constexpr (BF16) sep_store<true>(p.out, seg * p.C, p.C, c0, acc);
      } else {
        if constexpr (!BF16) sep_store<false>(p.out, seg * p.C, p.C, c0, acc);
      }
    }
  }
}

pm_status pm_launch_slot_scale_sum(int64_t V, int K, int C, int is_bf16, const void* T, const int32_t* row_ptr,
                                   const int32_t* col, const float* alpha, const FoldCoef* fc, void* out, hipStream_t st) {
  if (V == 0) return PM_OK;
  SlotP p;
  p.V = V; p.K = K; p.C = C; p.out_bf16 = is_bf16; p.T = T; p.row_ptr = row_ptr; p.col = col; p.alpha = alpha;
  p.fc = *fc; p.out = out;
  const int cpl = is_bf16 ? 8 : 4;
  int need = (C + cpl - 1) / cpl, l = 1;
  while (l < need && l < 64) l <<= 1;
  p.lpg = l;
  const int gpb = 256 / l;
  int64_t nblk = (V + gpb - 1) / gpb;
  if (nblk > 8192) nblk = 8192;
  { ProfScope ps__(st, "k_slot_scale_sum");
    if (is_bf16) hipLaunchKernelGGL(k_slot_scale_sum<true>, dim3((unsigned)nblk), dim3(256), 0, st, p);
    else hipLaunchKernelGGL(k_slot_scale_sum<false>, dim3((unsigned)nblk), dim3(256), 0, st, p); }
  PM_CHECK_LAUNCH("k_slot_scale_sum");
  return PM_OK;
}

// ---- separable vertex2facet: gradients of (alpha, P) from the three corner matrices M_j = sum_f h_{v_j(f)} (x) dg_f
//   dP[ci][co]    = sum_j s_j[ci] M_j[ci][co],        s_j[ci] = sum_k fc[j][k] alpha[k][ci]
//   dalpha[k][ci] = sum_j fc[j][k] sum_co P[ci][co] M_j[ci][co]
__global__ void __launch_bounds__(256) k_sep_unfold(int K, int cin, int cout, int p_bf16, const float* __restrict__ M,
                                                    const float* __restrict__ alpha, const void* __restrict__ P,
                                                    FoldCoef fc, float* __restrict__ dalpha, float* __restrict__ dP) {
  const int ci = blockIdx.x;
  __shared__ float red[3][256];
  float t[3] = {0.f, 0.f, 0.f};
  float sj[3] = {0.f, 0.f, 0.f};
  for (int k = 0; k < K; ++k) {
    const float a = alpha[(int64_t)k * cin + ci];
#pragma unroll
    for (int j = 0; j < 3; ++j) sj[j] += fc.c[j][k] * a;
  }
  for (int co = threadIdx.x; co < cout; co += 256) {
    const int64_t e = (int64_t)ci * cout + co;
    const float pv = p_bf16 ? bf16_to_f32(((const uint16_t*)P)[e]) : ((const float*)P)[e];
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const float m = M[(int64_t)j * cin * cout + e];
      acc += sj[j] * m;
      t[j] += pv * m;
    }
    if (dP) dP[e] = acc;
  }
#pragma unroll
  for (int j = 0; j < 3; ++j) red[j][threadIdx.x] = t[j];
  __syncthreads();
  if (dalpha && threadIdx.x < 3) {      // fixed-order sum over the 256 partial sums of corner j
    float sacc = 0.f;
    for (int i = 0; i < 256; ++i) sacc += red[threadIdx.x][i];
    red[threadIdx.x][0] = sacc;
  }
  __syncthreads();
  if (dalpha)
    for (int k = threadIdx.x; k < K; k += 256)
      dalpha[(int64_t)k * cin + ci] = fc.c[0][k] * red[0][0] + fc.c[1][k] * red[1][0] + fc.c[2][k] * red[2][0];
}

pm_status pm_launch_sep_unfold(int K, int cin, int cout, int p_bf16, const float* M, const float* alpha, const void* P,
                               const FoldCoef* fc, float* dalpha, float* dP, hipStream_t st) {
  { ProfScope ps__(st, "k_sep_unfold");
    hipLaunchKernelGGL(k_sep_unfold, dim3((unsigned)cin), dim3(256), 0, st, K, cin, cout, p_bf16, M, alpha, P, *fc, dalpha,
                       dP); }
  PM_CHECK_LAUNCH("k_sep_unfold");
  return PM_OK;
}
