// Depth-wise stage of the point-cloud convolution with the radial term (subsection "Extension to Point Cloud
// Convolution"): for the neighbours q_e of a query point i (lists supplied by the caller)
//     delta_e = xs[q_e] - xq[i],  r_e = |delta_e|,  Z_e = min(r_e / rho, 1),
//     s_e[c] = Z_e sum_k alpha[k][c] B_k(delta_e / r_e) + c0[c] (1 - Z_e),
//     y_i[c] = 1/|N(i)| sum_e s_e[c] h[q_e][c]
// and its transposed sums.  With B'_e = [Z_e B_0 .. Z_e B_{K-1}, 1 - Z_e] and alpha' = [alpha; c0] the filter is
// s_e = B'_e alpha', K + 1 numbers per channel, so the kernel is the mesh depth-wise kernel with one more basis row.
//
// One kernel walks a list of (row, entries) in three modes:
//   0  rows = queries, entries = neighbour ids:            y_i  = w_i sum_e s_e (.) h[q_e]
//   2  the same walk plus the coefficient gradients:       dalpha' += B'_e^T (h[q_e] (.) dy_i w_i)
//   1  rows = sources, entries = pair ids of the reverse lists:  dh_q = sum_e s_e (.) dy_{i_e} w_{i_e}
// (w_i = 1/|N(i)|).  Lane layout and matrix-core use as in the mesh kernel, with the wave's 64 LDS basis rows
// holding four entries of each of 16 rows: lane (row, slot) evaluates the basis of the row's (4 j + slot)-th
// entry, then the four sub-steps (one per slot) of 16 rows x 64 channels contract B' with alpha' (and B'^T with
// the products) in 16x16x4 fp32 tiles; the sums over a row's entries stay in 16 registers (j runs to the
// longest list of the 16 rows), so nothing per pair reaches memory.
#include "pm_rows.h"
#include "pm_chan.h"

#define PC_TRY(expr)                   \
  do {                                 \
    pm_status s__ = (expr);            \
    if (s__ != PM_OK) return s__;      \
  } while (0)

#define PC_KC 16       /* alpha rows per pass of the coefficient gradient (one matrix-core tile) */
#define PC_RW 64

struct PcP {
  int64_t R, n_other;
  int K, C, kc0;
  float inv_rho, sign;      // delta = sign * (x_other - x_row)
  ShTable sh;
  const float* x_row;       // [R][3]
  const float* x_other;     // [n_other][3]
  const int32_t* ptr;       // [R+1]
  const int32_t* ent;       // mode 0/2: neighbour ids; mode 1: pair ids
  const int32_t* owner;     // mode 1: query of every pair
  const int32_t* q_ptr;     // mode 1: neighbour list offsets of the queries (for w)
  const void* G;            // gathered rows: mode 0/2 h (feature dtype), mode 1 dy (fp32)
  const float* dy;          // mode 2: dy [R][C] fp32
  const float* alpha;       // [K][C]
  const float* c0;          // [C]
  void* out;                // [R][C] feature dtype (mode 2: may be NULL)
  float* partial;           // mode 2: [grid][K+1][C]
};

template <bool BF16, int MODE, bool VEC>
__global__ void __launch_bounds__(256) k_pc_dw(PcP p) {
  extern __shared__ float pc_lds[];
  constexpr int CPL = 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, sub = lane & 15;
  const int K1 = p.K + 1;
  const int nk4 = (K1 + 3) >> 2;
  const int KP = K1 | 1;
  const int kn = MODE == 2 ? min(PC_KC, p.K - p.kc0) : 0;
  const int per_wave = 64 * KP + 192;
  float* A = pc_lds;                                           // [4 nk4][64]: alpha rows, then c0, then zeros
  float* Bw = pc_lds + nk4 * 4 * PC_RW + wave * per_wave;      // this wave's [64][KP]
  int32_t* Oth = (int32_t*)(Bw + 64 * KP);                     // [64] gathered row of the current entry, -1 = none
  float* Wt = Bw + 64 * KP + 64;                               // [64] weight of the gathered row (mode 1)
  float* Wrow = Bw + 64 * KP + 128;                            // [64] 1/|N(row)|
  float* red = pc_lds + nk4 * 4 * PC_RW + 4 * per_wave;        // [PC_KC + 1][64] (mode 2)
  const bool want_s = MODE != 2 || p.out != nullptr;           // a coefficient pass without output needs no filter values
  const int nrun = (p.C + PC_RW - 1) / PC_RW;
  const int64_t n_ss = (p.R + 15) >> 4;                        // a wave step covers 16 rows, four entries of each

  for (int cr = 0; cr < nrun; ++cr) {
    const int c0 = cr * PC_RW + sub * CPL;
    const bool cok = c0 < p.C;
    const int cl = VEC ? min(c0, p.C - CPL) : c0;
    __syncthreads();
    for (int i = tid; i < nk4 * 4 * PC_RW; i += 256) {
      const int k = i >> 6, c = cr * PC_RW + (i & 63);
      float v = 0.f;
      if (c < p.C) {
        if (k < p.K) v = p.alpha[(int64_t)k * p.C + c];
        else if (k == p.K) v = p.c0[c];
      }
      A[i] = v;
    }
    __syncthreads();
    floatx4 D[4];
    float E[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t) D[t] = floatx4{0.f, 0.f, 0.f, 0.f};

    for (int64_t ss = (int64_t)blockIdx.x * 4 + wave; ss < n_ss; ss += (int64_t)gridDim.x * 4) {
      const int64_t R0 = ss << 4;
      const int64_t row_l = R0 + sub;          // basis evaluation: lane = (row sub, entry slot g) -> LDS slot `lane`
      int32_t b = 0, e = 0;
      float xr[3] = {0.f, 0.f, 0.f};
      if (row_l < p.R) {
        b = p.ptr[row_l]; e = p.ptr[row_l + 1];
        xr[0] = p.x_row[3 * row_l]; xr[1] = p.x_row[3 * row_l + 1]; xr[2] = p.x_row[3 * row_l + 2];
      }
      int maxdeg = e - b;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) maxdeg = max(maxdeg, __shfl_xor(maxdeg, o, 64));
      __builtin_amdgcn_wave_barrier();
      Wrow[sub] = 1.0f / (float)max(e - b, 1);     // (the four lanes of a row write the same value)
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      float acc[4][CPL], dyr[MODE == 2 ? 4 : 1][CPL];
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int t = 0; t < CPL; ++t) acc[q][t] = 0.f;
      if constexpr (MODE == 2) {
        // the rows' own gradient, weighted: (dy_i / |N(i)|)[c]
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int64_t row = min(R0 + 4 * g + q, p.R - 1);
          const int32_t d = p.ptr[row + 1] - p.ptr[row];
          if (VEC || cok) chan_load_f32<CPL, VEC>(p.dy, row * p.C, p.C, cl, dyr[q]);
          else {
#pragma unroll
            for (int t = 0; t < CPL; ++t) dyr[q][t] = 0.f;
          }
          const float wr = 1.0f / (float)max(d, 1);
#pragma unroll
          for (int t = 0; t < CPL; ++t) dyr[q][t] *= wr;
        }
      }

      for (int j4 = 0; j4 < maxdeg; j4 += 4) {
        __builtin_amdgcn_wave_barrier();        // the previous entries' basis rows have been read
        const int j = j4 + g;                   // this lane's entry of its row
        const bool has = b + j < e;
        if (has) {
          int32_t other = p.ent[b + j];
          if (MODE == 1) other = p.owner[other];
          other = min(max(other, 0), (int32_t)(p.n_other - 1));       // a bad id is never followed out of range
          const float* xo = p.x_other + 3 * (int64_t)other;
          const float dx = p.sign * (xo[0] - xr[0]), dyy = p.sign * (xo[1] - xr[1]), dz = p.sign * (xo[2] - xr[2]);
          const float r = sqrtf(dx * dx + dyy * dyy + dz * dz);
          const float Z = fminf(r * p.inv_rho, 1.0f);
          float ux = 0.f, uy = 0.f, uz = 1.f;
          if (r > 0.f) { const float ir = 1.0f / r; ux = dx * ir; uy = dyy * ir; uz = dz * ir; }
          sh_eval<-1>(ux, uy, uz, p.sh, [&](int k, float v) { Bw[lane * KP + k] = Z * v; });
          Bw[lane * KP + p.K] = 1.0f - Z;
          Oth[lane] = other;
          float wt = 1.f;
          if (MODE == 1) wt = 1.0f / (float)max(p.q_ptr[other + 1] - p.q_ptr[other], 1);
          Wt[lane] = wt;
        } else {
          for (int k = 0; k < K1; ++k) Bw[lane * KP + k] = 0.f;
          Oth[lane] = -1;
          Wt[lane] = 0.f;
        }
        const uint64_t live = __ballot(has);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          if (((live >> (16 * s4)) & 0xffffull) == 0) continue;     // the same for the whole wave
          float hv[4][CPL];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int rr = 16 * s4 + 4 * g + q;
            const int32_t o = Oth[rr];
            const bool ok = o >= 0 && cok;
#pragma unroll
            for (int t = 0; t < CPL; ++t) hv[q][t] = 0.f;
            if (VEC || ok) {
              const int64_t ol = max(o, 0);
              if (MODE == 1) chan_load_f32<CPL, VEC>((const float*)p.G, ol * p.C, p.C, cl, hv[q]);
              else chan_load<BF16, CPL, VEC>(p.G, ol * p.C, p.C, cl, hv[q]);
            }
            const float wv = MODE == 1 ? Wt[rr] : 1.f;
#pragma unroll
            for (int t = 0; t < CPL; ++t) hv[q][t] = ok ? hv[q][t] * wv : 0.f;
          }
          if (want_s) {
            floatx4 S[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) S[t] = floatx4{0.f, 0.f, 0.f, 0.f};
            for (int ks = 0; ks < nk4; ++ks) {
              const int k = 4 * ks + g;
              const float bv = Bw[(16 * s4 + sub) * KP + min(k, K1 - 1)];
              const float a = k < K1 ? bv : 0.f;
              const float4 w4 = *(const float4*)&A[k * PC_RW + sub * CPL];
              S[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, w4.x, S[0], 0, 0, 0);
              S[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, w4.y, S[1], 0, 0, 0);
              S[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, w4.z, S[2], 0, 0, 0);
              S[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, w4.w, S[3], 0, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
              for (int t = 0; t < 4; ++t) acc[q][t] += hv[q][t] * S[t][q];
          }
          if constexpr (MODE == 2) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int rr = 16 * s4 + 4 * g + q;
              float pe[CPL];
#pragma unroll
              for (int t = 0; t < CPL; ++t) pe[t] = hv[q][t] * dyr[q][t];      // hv is 0 where there is no pair
              const float bv = Bw[rr * KP + p.kc0 + min(sub, kn - 1)];
              const float a = sub < kn ? bv : 0.f;
#pragma unroll
              for (int t = 0; t < 4; ++t) D[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, pe[t], D[t], 0, 0, 0);
              if (p.kc0 == 0) {
                const float z1 = Bw[rr * KP + p.K];
#pragma unroll
                for (int t = 0; t < 4; ++t) E[t] += z1 * pe[t];
              }
            }
          }
        }
      }
      if (want_s) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int64_t row = R0 + 4 * g + q;
          const float w = MODE == 1 ? 1.f : Wrow[4 * g + q];
          float o[CPL];
#pragma unroll
          for (int t = 0; t < CPL; ++t) o[t] = acc[q][t] * w;
          if (row < p.R && cok) chan_store<BF16, CPL, VEC>(p.out, row * p.C, p.C, c0, o);
        }
      }
    }
    if constexpr (MODE == 2) {
      // the block's sums over its four waves (and, for c0, over the four row groups of a wave), one after the
      // other in a fixed order, then one slice per block
      for (int w = 0; w < 4; ++w) {
        __syncthreads();
        if (wave == w) {
#pragma unroll
          for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int o = (4 * g + r) * PC_RW + sub * CPL + t;
              red[o] = (w == 0 ? 0.f : red[o]) + D[t][r];
            }
        }
      }
      for (int w = 0; w < 16; ++w) {
        __syncthreads();
        if (wave == (w >> 2) && g == (w & 3)) {
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int o = PC_KC * PC_RW + sub * CPL + t;
            red[o] = (w == 0 ? 0.f : red[o]) + E[t];
          }
        }
      }
      __syncthreads();
      float* dst = p.partial + (int64_t)blockIdx.x * K1 * p.C;
      for (int i = tid; i < kn * PC_RW; i += 256) {
        const int k = i >> 6, c = cr * PC_RW + (i & 63);
        if (c < p.C) dst[(int64_t)(p.kc0 + k) * p.C + c] = red[i];
      }
      if (p.kc0 == 0)
        for (int i = tid; i < PC_RW; i += 256) {
          const int c = cr * PC_RW + i;
          if (c < p.C) dst[(int64_t)p.K * p.C + c] = red[PC_KC * PC_RW + i];
        }
    }
  }
}

#define PC_GRID 4096
#define PC_GRID_BWD 1024
static int pc_grid(int64_t R, int cap) {
  int64_t nblk = (((R + 15) >> 4) + 3) >> 2;      // four waves per block, 16 rows per wave step
  if (nblk > cap) nblk = cap;
  return nblk < 1 ? 1 : (int)nblk;
}

size_t pm_pc_coef_ws_bytes(int64_t M, int K, int C) {
  return pm_round_up((size_t)pc_grid(M, PC_GRID_BWD) * (K + 1) * C * sizeof(float), 256);
}

static size_t pc_lds_bytes(int K) {
  const int K1 = K + 1, nk4 = (K1 + 3) / 4, KP = K1 | 1;
  return ((size_t)nk4 * 4 * PC_RW + (size_t)4 * (64 * KP + 192) + (size_t)(PC_KC + 1) * PC_RW) * sizeof(float);
}

template <int MODE>
static pm_status pc_launch(const PcP& p, int is_bf16, bool vec, int grid, hipStream_t st) {
  auto kern = is_bf16 ? (vec ? k_pc_dw<true, MODE, true> : k_pc_dw<true, MODE, false>)
                      : (vec ? k_pc_dw<false, MODE, true> : k_pc_dw<false, MODE, false>);
  const size_t lds = pc_lds_bytes(p.K);
  PM_TRY(pm_set_dyn_lds((const void*)kern, lds));
  { ProfScope ps__(st, MODE == 0 ? "k_pc_dw" : (MODE == 1 ? "k_pc_dw_dh" : "k_pc_dw_coef"));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p); }
  PM_CHECK_LAUNCH("k_pc_dw");
  return PM_OK;
}

static PcP pc_params(int K, int C, float rho, const ShTable& sh, const float* alpha, const float* c0) {
  PcP p;
  p.K = K; p.C = C; p.kc0 = 0; p.inv_rho = 1.0f / rho; p.sign = 1.f; p.sh = sh; p.alpha = alpha; p.c0 = c0;
  p.owner = nullptr; p.q_ptr = nullptr; p.dy = nullptr; p.partial = nullptr; p.out = nullptr;
  return p;
}

// y [M][C] (feature dtype) = mean over the neighbours of s_e (.) h[q_e]
pm_status pm_launch_pc_dw(int64_t M, int64_t N, int K, int C, int is_bf16, float rho, const ShTable& sh, const float* xq,
                          const float* xs, const int32_t* nbr_ptr, const int32_t* nbr_idx, const void* h,
                          const float* alpha, const float* c0, void* y, hipStream_t st) {
  if (M == 0) return PM_OK;
  PcP p = pc_params(K, C, rho, sh, alpha, c0);
  p.R = M; p.n_other = N; p.x_row = xq; p.x_other = xs; p.ptr = nbr_ptr; p.ent = nbr_idx; p.G = h; p.out = y;
  return pc_launch<0>(p, is_bf16, chan_vec_ok(C, is_bf16, h, y, nullptr), pc_grid(M, PC_GRID), st);
}

// dalpha [K][C], dc0 [C] (through `partial`, pm_pc_coef_ws_bytes) and, in the same walk, y [M][C] (feature
// dtype, for dP); dy [M][C] fp32 is the gradient of the depth-wise output before the 1/|N(i)| weight
pm_status pm_launch_pc_dw_coef(int64_t M, int64_t N, int K, int C, int is_bf16, float rho, const ShTable& sh,
                               const float* xq, const float* xs, const int32_t* nbr_ptr, const int32_t* nbr_idx,
                               const void* h, const float* alpha, const float* c0, const float* dy, void* y,
                               float* dalpha, float* dc0, float* partial, hipStream_t st) {
  const int grid = pc_grid(M, PC_GRID_BWD);
  const int64_t slice = (int64_t)(K + 1) * C;
  if (M > 0) {
    PcP p = pc_params(K, C, rho, sh, alpha, c0);
    p.R = M; p.n_other = N; p.x_row = xq; p.x_other = xs; p.ptr = nbr_ptr; p.ent = nbr_idx; p.G = h; p.dy = dy;
    p.partial = partial;
    const bool vec = chan_vec_ok(C, is_bf16, h, dy, y);
    for (int k0 = 0; k0 < K; k0 += PC_KC) {
      p.kc0 = k0;
      p.out = k0 == 0 ? y : nullptr;
      PC_TRY(pc_launch<2>(p, is_bf16, vec, grid, st));
    }
  }
  const int n_slice = M > 0 ? grid : 0;
  PC_TRY(pm_launch_sum_slices_strided(partial, (int64_t)K * C, slice, n_slice, dalpha, st));
  return pm_launch_sum_slices_strided(partial + (int64_t)K * C, C, slice, n_slice, dc0, st);
}

// dh [N][C] (feature dtype) over the reverse lists: rev_ptr [N+1], rev_col = pair ids, owner = query of a pair
pm_status pm_launch_pc_dw_dh(int64_t M, int64_t N, int K, int C, int is_bf16, float rho, const ShTable& sh,
                             const float* xq, const float* xs, const int32_t* nbr_ptr, const int32_t* rev_ptr,
                             const int32_t* rev_col, const int32_t* owner, const float* alpha, const float* c0,
                             const float* dy, void* dh, hipStream_t st) {
  if (N == 0) return PM_OK;
  PcP p = pc_params(K, C, rho, sh, alpha, c0);
  p.R = N; p.n_other = M; p.x_row = xs; p.x_other = xq; p.sign = -1.f; p.ptr = rev_ptr; p.ent = rev_col;
  p.owner = owner; p.q_ptr = nbr_ptr; p.G = dy; p.out = dh;
  return pc_launch<1>(p, is_bf16, chan_vec_ok(C, is_bf16, dy, dh, nullptr), pc_grid(N, PC_GRID), st);
}

// flag bit 1: offsets not monotone / not spanning the list; bit 2: a neighbour id outside [0, N)
__global__ void __launch_bounds__(256) k_validate_nbr(int64_t M, int64_t N, int64_t nnz, const int32_t* __restrict__ ptr,
                                                      const int32_t* __restrict__ idx, int32_t* __restrict__ flag) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i <= M) {
    const int32_t a = ptr[i];
    bool bad = a < 0 || a > nnz;
    if (i == 0 && a != 0) bad = true;
    if (i == M && a != nnz) bad = true;
    if (i < M && ptr[i + 1] < a) bad = true;
    if (bad) atomicOr(flag, 1);
  }
  if (i < nnz && (idx[i] < 0 || idx[i] >= N)) atomicOr(flag, 2);
}

pm_status pm_launch_validate_nbr(int64_t M, int64_t N, int64_t nnz, const int32_t* ptr, const int32_t* idx,
                                 int32_t* flag, hipStream_t st) {
  PC_TRY(pm_launch_fill_i32(flag, 1, 0, st));
  const int64_t n = (M + 1 > nnz) ? M + 1 : nnz;
  { ProfScope ps__(st, "k_validate_nbr");
    hipLaunchKernelGGL(k_validate_nbr, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, M, N, nnz, ptr, idx, flag); }
  PM_CHECK_LAUNCH("k_validate_nbr");
  return PM_OK;
}
