// Depth-wise stage of the separable facet2vertex convolution (Section "Mesh convolutions": Eq. 5 with one
// scalar SH coefficient set per channel), forward and backward:
//     y_f[c]  = h_f[c] * s_f[c],            s_f[c] = sum_k alpha[k][c] B_k(n_f)
//     dh_f[c] = dy_f[c] * s_f[c],           dy_f[c] = sum_j dz[v_j(f)][c] / deg(v_j(f))    (dz in fp32)
//     dalpha[k][c] = sum_f B_k(n_f) h_f[c] dy_f[c]
// The backward kernel can also take dh through the epilogue that produced h (vertex2vertex block: h = relu(a u + b),
// so du = dh a [h > 0]): h is in registers anyway.
// Bound by HBM (one row read, one written per facet); the K multiply-adds per element run on the fp32
// matrix cores so that the vector ALU only loads, converts and stores.
// dalpha is reduced without atomics: every wave accumulates its rows in matrix-core tiles (a fixed assignment
// of rows to waves), a block adds its waves in LDS one after the other and writes its own slice; the slices
// are added in a fixed order.
// The tail of the file holds the small fold/unfold kernels of the separable vertex2facet form (Eq. 6).
#include "pm_rows.h"
#include "pm_chan.h"

#define SEP_KC 16      /* basis functions per pass of the backward kernel (rows of one matrix-core tile) */

struct SepP {
  int64_t F;
  int K, C, lpg;          // lanes per row group (16)
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
  const float* mask_scale; // bwd, optional: dh[c] *= mask_scale[c]          (the affine map that produced h)
  int mask_relu;           // bwd, optional: dh[c] = 0 where h[c] <= 0       (the ReLU that produced h)
};

// Lane layout (fixed): a wave holds 4 row groups of 16 lanes, lane `sub` of a group owns channels
// 4 sub .. 4 sub + 3 of a run of 64 channels, and each group handles four consecutive rows per sub-step, so a
// wave covers 16 rows x 64 channels per sub-step.  Both small contractions run on the fp32 matrix cores
// (16x16x4: A[i][kk] from lane (i = lane % 16, kk = lane / 16), B[kk][j] from lane (kk = lane / 16,
// j = lane % 16), D[4 (lane / 16) + reg][lane % 16]) in exactly this layout, with no data movement:
//   s = Basis alpha:      i = row of the sub-step, kk = basis function, column j of tile t = channel 4 j + t;
//                         register q of tile t is then s[row 4 g + q][channel 4 sub + t], the lane's own element
//   dalpha = Basis^T (h dy): i = basis function, kk = row group g (its q-th row), same columns; the lane's own
//                         products h dy are the B operand.
// A wave evaluates the SH basis of 64 rows at a time (one lane per row) into its own LDS rows, then walks
// them in four sub-steps; waves never wait for each other inside the row loop.
// LDS: alpha [4 ceil(kn/4)][64] (zero rows past kn), per wave basis [64][kn | 1], backward: block sum [16][64].
#define SEP_RW 64

template <bool BF16, bool BWD, bool VEC, bool MASK = false, bool PRE = false>
__global__ void __launch_bounds__(256) k_dw_f2v(SepP p) {
  extern __shared__ float sep_lds[];
  constexpr int CPL = 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, sub = lane & 15;
  const int k0 = BWD ? p.kc0 : 0;
  // basis functions handled in this launch: all of them, or one chunk of the dalpha rows
  const int kn = (BWD && p.want_dalpha) ? min(SEP_KC, p.K - k0) : p.K;
  const int nk4 = (kn + 3) >> 2;
  const int KP = kn | 1;                                   // odd row pitch: conflict-free column reads
  float* A = sep_lds;                                      // [4 nk4][64]
  float* Bw = sep_lds + nk4 * 4 * SEP_RW + wave * 64 * KP;  // this wave's [64][KP]
  float* red = sep_lds + nk4 * 4 * SEP_RW + 4 * 64 * KP;   // [SEP_KC][64] (backward)
  const bool want_s = !BWD || (p.y != nullptr && kn == p.K);   // dh needs the whole filter value
  const int nrun = (p.C + SEP_RW - 1) / SEP_RW;
  const int64_t n_ss = (p.F + 63) >> 6;

  for (int cr = 0; cr < nrun; ++cr) {
    const int c0 = cr * SEP_RW + sub * CPL;
    const bool cok = c0 < p.C;
    const int cl = VEC ? min(c0, p.C - CPL) : c0;
    __syncthreads();                          // the previous run's coefficients are no longer needed
    for (int i = tid; i < nk4 * 4 * SEP_RW; i += 256) {
      const int k = i >> 6, c = cr * SEP_RW + (i & 63);
      A[i] = (k < kn && c < p.C) ? p.alpha[(int64_t)(k0 + k) * p.C + c] : 0.f;
    }
    __syncthreads();
    float msc[CPL];                           // backward: the epilogue's scale for the lane's channels
#pragma unroll
    for (int i = 0; i < CPL; ++i) msc[i] = (MASK && p.mask_scale) ? p.mask_scale[min(c0 + i, p.C - 1)] : 1.f;
    floatx4 D[4];                             // backward: dalpha tiles of this wave
#pragma unroll
    for (int t = 0; t < 4; ++t) D[t] = floatx4{0.f, 0.f, 0.f, 0.f};

    for (int64_t ss = (int64_t)blockIdx.x * 4 + wave; ss < n_ss; ss += (int64_t)gridDim.x * 4) {
      const int64_t R0 = ss << 6;
      __builtin_amdgcn_wave_barrier();        // the previous rows' basis has been read
      {
        const int64_t r = R0 + lane;
        if (r < p.F) {
          float x, y, z;
          row_direction<B_NORMAL>(p.bs, r, x, y, z);
          sh_eval_any(x, y, z, p.bs.sh, [&](int k, float v) {
            const int kl = k - k0;
            if (kl >= 0 && kl < kn) Bw[lane * KP + kl] = v;
          });
        } else {
          for (int k = 0; k < kn; ++k) Bw[lane * KP + k] = 0.f;   // rows past the end add nothing to dalpha
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      for (int s4 = 0; s4 < 4; ++s4) {
        if (R0 + 16 * s4 >= p.F) break;       // the same for the whole wave
        const int64_t rb = R0 + 16 * s4 + 4 * g;
        float hv[4][CPL], dyv[BWD ? 4 : 1][CPL];
        bool ok[4];
        // With whole aligned runs every load is issued unconditionally at an in-range address (row and run
        // clamped) and masked afterwards, so that the loads of all four rows are in flight together.
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int64_t r = rb + q;
          ok[q] = r < p.F && cok;
          const int64_t rl = min(r, p.F - 1);
#pragma unroll
          for (int i = 0; i < CPL; ++i) hv[q][i] = 0.f;
          if constexpr (BWD) {
#pragma unroll
            for (int i = 0; i < CPL; ++i) dyv[q][i] = 0.f;
          }
          if (VEC || ok[q]) {
            chan_load<BF16, CPL, VEC>(p.h, rl * p.C, p.C, cl, hv[q]);
            if constexpr (BWD) {
#pragma unroll
              for (int j = 0; j < 3; ++j) {
                const int32_t v = p.bs.facet[3 * rl + j];
                float t[CPL];
                chan_load_f32<CPL, VEC>(p.dz, (int64_t)v * p.C, p.C, cl, t);
                if constexpr (PRE) {             // the rows of dz carry their 1/deg(v) already
#pragma unroll
                  for (int i = 0; i < CPL; ++i) dyv[q][i] += t[i];
                } else {
                  const float w = 1.0f / (float)(p.row_ptr[v + 1] - p.row_ptr[v]);
#pragma unroll
                  for (int i = 0; i < CPL; ++i) dyv[q][i] += t[i] * w;
                }
              }
            }
          }
          if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < CPL; ++i) hv[q][i] = ok[q] ? hv[q][i] : 0.f;
            if constexpr (BWD) {
#pragma unroll
              for (int i = 0; i < CPL; ++i) dyv[q][i] = ok[q] ? dyv[q][i] : 0.f;
            }
          }
        }
        floatx4 S[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) S[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (want_s) {
          for (int ks = 0; ks < nk4; ++ks) {
            const int k = 4 * ks + g;
            const float bv = Bw[(16 * s4 + sub) * KP + min(k, kn - 1)];
            const float a = k < kn ? bv : 0.f;
            const float4 w4 = *(const float4*)&A[k * SEP_RW + sub * CPL];
            S[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, w4.x, S[0], 0, 0, 0);
            S[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, w4.y, S[1], 0, 0, 0);
            S[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, w4.z, S[2], 0, 0, 0);
            S[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, w4.w, S[3], 0, 0, 0);
          }
        }
        if constexpr (BWD) {
          if (p.want_dalpha) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float bv = Bw[(16 * s4 + 4 * g + q) * KP + min(sub, kn - 1)];
              const float a = sub < kn ? bv : 0.f;
#pragma unroll
              for (int t = 0; t < 4; ++t)
                D[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, hv[q][t] * dyv[q][t], D[t], 0, 0, 0);
            }
          }
        }
        if (!BWD || (p.y != nullptr && want_s)) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float o[CPL];
#pragma unroll
            for (int t = 0; t < 4; ++t) o[t] = (BWD ? dyv[q][t] : hv[q][t]) * S[t][q];
            if constexpr (MASK) {
#pragma unroll
              for (int t = 0; t < 4; ++t) o[t] = (p.mask_relu && !(hv[q][t] > 0.f)) ? 0.f : o[t] * msc[t];
            }
            if (ok[q]) chan_store<BF16, CPL, VEC>(p.y, (rb + q) * p.C, p.C, c0, o);
          }
        }
      }
    }
    if constexpr (BWD) {
      if (p.want_dalpha) {
        // the block's sum over its four waves, one after the other (a fixed order), then one slice per block
        for (int w = 0; w < 4; ++w) {
          __syncthreads();
          if (wave == w) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const int o = (4 * g + r) * SEP_RW + sub * CPL + t;
                red[o] = (w == 0 ? 0.f : red[o]) + D[t][r];
              }
          }
        }
        __syncthreads();
        float* dst = p.partial + (int64_t)blockIdx.x * p.K * p.C;
        for (int i = tid; i < kn * SEP_RW; i += 256) {
          const int k = i >> 6, c = cr * SEP_RW + (i & 63);
          if (c < p.C) dst[(int64_t)(k0 + k) * p.C + c] = red[i];
        }
      }
    }
  }
}

#define SEP_GRID_FWD 2048
#define SEP_GRID_BWD 1024
static int sep_grid(int64_t F, int cap) {
  int64_t nblk = (((F + 63) >> 6) + 3) >> 2;      // four waves per block, 64 rows per wave step
  if (nblk > cap) nblk = cap;
  return nblk < 1 ? 1 : (int)nblk;
}

size_t pm_sep_dalpha_ws_bytes(int64_t F, int K, int C, int is_bf16) {
  (void)is_bf16;
  return pm_round_up((size_t)sep_grid(F, SEP_GRID_BWD) * K * C * sizeof(float), 256);
}

static size_t sep_lds_bytes(int kn, bool bwd) {
  const int nk4 = (kn + 3) / 4, KP = kn | 1;
  return ((size_t)nk4 * 4 * SEP_RW + (size_t)4 * 64 * KP + (bwd ? (size_t)SEP_KC * SEP_RW : 0)) * sizeof(float);
}

pm_status pm_launch_dw_f2v(int64_t F, int K, int C, int is_bf16, const BasisSrc& bs, const void* h, const float* alpha,
                           void* y, hipStream_t st) {
  if (F == 0) return PM_OK;
  SepP p;
  p.F = F; p.K = K; p.C = C; p.is_bf16 = is_bf16; p.bs = bs; p.h = h; p.alpha = alpha; p.y = y;
  p.dz = nullptr; p.row_ptr = nullptr; p.partial = nullptr; p.kc0 = 0; p.want_dalpha = 0; p.lpg = 16;
  p.mask_scale = nullptr; p.mask_relu = 0;
  const int grid = sep_grid(F, SEP_GRID_FWD);
  const size_t lds = sep_lds_bytes(K, false);
  const bool vec = chan_vec_ok(C, is_bf16, h, y, nullptr);
  auto kern = is_bf16 ? (vec ? k_dw_f2v<true, false, true> : k_dw_f2v<true, false, false>)
                      : (vec ? k_dw_f2v<false, false, true> : k_dw_f2v<false, false, false>);
  PM_TRY(pm_set_dyn_lds((const void*)kern, lds));
  { ProfScope ps__(st, "k_dw_f2v");
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p); }
  PM_CHECK_LAUNCH("k_dw_f2v");
  return PM_OK;
}

// dh [F][C] (may be NULL) and dalpha [K][C] (may be NULL; `partial` must then hold pm_sep_dalpha_ws_bytes).
// mask_scale [C] (may be NULL) / mask_relu: dh leaves as dh * mask_scale * [h > 0].
pm_status pm_launch_dw_f2v_bwd(int64_t F, int K, int C, int is_bf16, const BasisSrc& bs, const void* h,
                               const float* alpha, const float* dz, const int32_t* row_ptr, void* dh, float* dalpha,
                               float* partial, const float* mask_scale, int mask_relu, int dz_prescaled, hipStream_t st) {
  SepP p;
  p.mask_scale = mask_scale; p.mask_relu = mask_relu;
  p.F = F; p.K = K; p.C = C; p.is_bf16 = is_bf16; p.bs = bs; p.h = h; p.alpha = alpha; p.y = dh;
  p.dz = dz; p.row_ptr = row_ptr; p.partial = partial; p.want_dalpha = dalpha != nullptr; p.lpg = 16;
  const int grid = sep_grid(F, SEP_GRID_BWD);
  const bool vec = chan_vec_ok(C, is_bf16, h, dz, dh);
  const bool mask = mask_scale != nullptr || mask_relu != 0;
  auto kern = is_bf16 ? (vec ? k_dw_f2v<true, true, true> : k_dw_f2v<true, true, false>)
                      : (vec ? k_dw_f2v<false, true, true> : k_dw_f2v<false, true, false>);
  if (mask)
    kern = is_bf16 ? (vec ? k_dw_f2v<true, true, true, true> : k_dw_f2v<true, true, false, true>)
                   : (vec ? k_dw_f2v<false, true, true, true> : k_dw_f2v<false, true, false, true>);
  if (dz_prescaled) {   // only the staged point-wise pass (bf16 rows) prescales
    if (!is_bf16) return pm_fail(PM_ERR_UNSUPPORTED, "prescaled dz rows with fp32 features");
    kern = vec ? (mask ? k_dw_f2v<true, true, true, true, true> : k_dw_f2v<true, true, true, false, true>)
               : (mask ? k_dw_f2v<true, true, false, true, true> : k_dw_f2v<true, true, false, false, true>);
  }
  if (F == 0) {
    if (dalpha) return pm_launch_sum_slices(partial, (int64_t)K * C, 0, dalpha, st);   // no slices: zeros
    return PM_OK;
  }
  // dh needs the whole filter value: it comes from the dalpha launch when that covers every k (K <= SEP_KC),
  // else from a launch of its own without dalpha tiles
  const bool fused = dalpha && K <= SEP_KC;
  if (dh && !fused) {
    p.kc0 = 0; p.want_dalpha = 0; p.y = dh;
    const size_t lds = sep_lds_bytes(K, true);
    PM_TRY(pm_set_dyn_lds((const void*)kern, lds));
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
      const size_t lds = sep_lds_bytes(kn, true);
      PM_TRY(pm_set_dyn_lds((const void*)kern, lds));
      { ProfScope ps__(st, "k_dw_f2v_bwd");
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p); }
      PM_CHECK_LAUNCH("k_dw_f2v_bwd");
    }
    return pm_launch_sum_slices(partial, (int64_t)K * C, grid, dalpha, st);
  }
  return PM_OK;
}

// ---- separable vertex2facet, backward to the vertex features.  With T_f = dg_f P^T (one row per facet),
//   dh_v[c] = sum over the adjacency entries (f, j) of v of  s_j[c] T_f[c],     s_j[c] = sum_k fc[j][k] alpha[k][c]
// (fc[j][k] is the SH basis at the barycentric corner j, Eq. 6).  A group of lanes owns a vertex, each lane a
// run of channels whose three scales (from a small table built first) it keeps in registers; entries are
// taken two at a time in ascending order into per-corner sums (the corner chosen by selects), which are
// scaled and added at the end.
struct SlotP {
  int64_t V;
  int C, lpg, out_bf16;
  const void* T;            // [F][C] feature dtype
  const int32_t* row_ptr;   // [V+1]
  const int32_t* col;       // entries 3f + j
  const float* sc;          // [3][C] corner scales s_j[c]
  void* out;                // [V][C]
};

__global__ void __launch_bounds__(256) k_sep_slot_scales(int K, int C, const float* __restrict__ alpha, FoldCoef fc,
                                                         float* __restrict__ sc) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= 3 * C) return;
  const int j = i / C, c = i - j * C;
  float a = 0.f;
  for (int k = 0; k < K; ++k) a += fc.c[j][k] * alpha[(int64_t)k * C + c];
  sc[i] = a;
}

template <bool BF16, bool VEC>
__global__ void __launch_bounds__(256) k_slot_scale_sum(SlotP p) {
  constexpr int CPL = BF16 ? 8 : 4;
  const int gpb = 256 / p.lpg;
  const int sub = threadIdx.x % p.lpg;
  for (int c0 = sub * CPL; c0 < p.C; c0 += p.lpg * CPL) {
    float sc[3][CPL];
#pragma unroll
    for (int j = 0; j < 3; ++j) chan_load_f32<CPL, VEC>(p.sc, (int64_t)j * p.C, p.C, c0, sc[j]);
    for (int64_t seg = (int64_t)blockIdx.x * gpb + threadIdx.x / p.lpg; seg < p.V; seg += (int64_t)gridDim.x * gpb) {
      const int32_t b = p.row_ptr[seg], e = p.row_ptr[seg + 1];
      float a3[3][CPL];                      // per-corner sums; the scales are applied once at the end
#pragma unroll
      for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int i = 0; i < CPL; ++i) a3[j][i] = 0.f;
      for (int32_t i0 = b; i0 < e; i0 += 2) {
        int32_t cidx[2], row[2];
        float x[2][CPL];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          cidx[q] = p.col[min(i0 + q, e - 1)];
          row[q] = (int32_t)(((uint64_t)(uint32_t)cidx[q] * 0xAAAAAAABull) >> 33);   // / 3
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) chan_load<BF16, CPL, VEC>(p.T, (int64_t)row[q] * p.C, p.C, c0, x[q]);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int slot = (i0 + q < e) ? cidx[q] - 3 * row[q] : 3;
#pragma unroll
          for (int j = 0; j < 3; ++j)
#pragma unroll
            for (int i = 0; i < CPL; ++i) a3[j][i] += (slot == j) ? x[q][i] : 0.f;
        }
      }
      float acc[CPL];
#pragma unroll
      for (int i = 0; i < CPL; ++i) acc[i] = sc[0][i] * a3[0][i] + sc[1][i] * a3[1][i] + sc[2][i] * a3[2][i];
      chan_store<BF16, CPL, VEC>(p.out, seg * p.C, p.C, c0, acc);
    }
  }
}

// The same sum with the corner scales looked up in LDS (a table [4][C], row 3 = zeros for the masked entry of an
// odd-length list): one multiply-add per element, s_j[c] T[c] added in ascending entry order.  For whole aligned
// channel runs and tables that fit LDS.
#define SLOT_LDS_MAX_C 2048
template <bool BF16>
__global__ void __launch_bounds__(256) k_slot_scale_sum_lds(SlotP p) {
  extern __shared__ float slot_sc[];          // [4][C]
  constexpr int CPL = BF16 ? 8 : 4;
  for (int i = threadIdx.x; i < 4 * p.C; i += 256) slot_sc[i] = (i < 3 * p.C) ? p.sc[i] : 0.f;
  __syncthreads();
  const int gpb = 256 / p.lpg;
  const int sub = threadIdx.x % p.lpg;
  for (int c0 = sub * CPL; c0 < p.C; c0 += p.lpg * CPL) {
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
        for (int q = 0; q < 2; ++q) chan_load<BF16, CPL, true>(p.T, (int64_t)row[q] * p.C, p.C, c0, x[q]);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int slot = (i0 + q < e) ? cidx[q] - 3 * row[q] : 3;
          float w[CPL];
          chan_load_f32<CPL, true>(slot_sc, (int64_t)slot * p.C, p.C, c0, w);
#pragma unroll
          for (int i = 0; i < CPL; ++i) acc[i] += w[i] * x[q][i];
        }
      }
      chan_store<BF16, CPL, true>(p.out, seg * p.C, p.C, c0, acc);
    }
  }
}

// `sc` is a scratch table of 3 * C floats
pm_status pm_launch_slot_scale_sum(int64_t V, int K, int C, int is_bf16, const void* T, const int32_t* row_ptr,
                                   const int32_t* col, const float* alpha, const FoldCoef* fc, float* sc, void* out,
                                   hipStream_t st) {
  if (V == 0) return PM_OK;
  { ProfScope ps__(st, "k_sep_slot_scales");
    hipLaunchKernelGGL(k_sep_slot_scales, dim3((unsigned)((3 * C + 255) / 256)), dim3(256), 0, st, K, C, alpha, *fc, sc); }
  PM_CHECK_LAUNCH("k_sep_slot_scales");
  SlotP p;
  p.V = V; p.C = C; p.out_bf16 = is_bf16; p.T = T; p.row_ptr = row_ptr; p.col = col; p.sc = sc; p.out = out;
  const int cpl = is_bf16 ? 8 : 4;
  int need = (C + cpl - 1) / cpl, l = 1;
  while (l < need && l < 64) l <<= 1;
  p.lpg = l;
  const int gpb = 256 / l;
  int64_t nblk = (V + gpb - 1) / gpb;
  if (nblk > 0x7fffffff) nblk = 0x7fffffff;
  { ProfScope ps__(st, "k_slot_scale_sum");
    const bool vec = chan_vec_ok(C, is_bf16, T, out, sc);
    if (vec && C <= SLOT_LDS_MAX_C) {
      auto kern = is_bf16 ? k_slot_scale_sum_lds<true> : k_slot_scale_sum_lds<false>;
      hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(256), (size_t)4 * C * sizeof(float), st, p);
    } else {
      auto kern = is_bf16 ? (vec ? k_slot_scale_sum<true, true> : k_slot_scale_sum<true, false>)
                          : (vec ? k_slot_scale_sum<false, true> : k_slot_scale_sum<false, false>);
      hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(256), 0, st, p);
    } }
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
