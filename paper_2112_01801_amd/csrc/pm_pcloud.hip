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
// the products); the sums over a row's entries stay in 16 registers (j runs to the longest list of the 16 rows), so
// nothing per pair reaches memory.
//
// The two contractions run on the matrix cores.  fp32 features: 16x16x4 fp32 tiles on fp32 basis rows.  bf16 features
// with K + 1 <= 32 (SPLIT): 16x16x32 bf16 tiles, one of which holds all K + 1 basis rows.  The lane that evaluates a
// pair's basis writes it to LDS as a bf16 head and a bf16 remainder (x = hi + lo, |lo| <= 2^-8 |x|), so an operand is one
// 16-byte LDS read; the coefficients alpha' are split the same way once per channel run and stay in registers.  The
// filter is the three leading products hi hi + hi lo + lo hi accumulated in fp32 (the dropped lo lo term is below 2^-16
// of a product: fp32 accuracy at under a third of the fp32 tiles' matrix-core time).  For the coefficient gradient
// the 32-deep dimension runs over the 32 pairs a lane group holds per two entry slots: the heads of the basis rows are
// also kept transposed ([k][pair]), the products h (.) dy are rounded to bf16 once (a sum over all pairs of terms with
// unbiased 2^-9 errors), one tile per channel quarter.
#include "pm_rows.h"
#include "pm_chan.h"

#define PC_TRY(expr)                   \
  do {                                 \
    pm_status s__ = (expr);            \
    if (s__ != PM_OK) return s__;      \
  } while (0)

#define PC_KC 16       /* alpha rows per pass of the coefficient gradient (one matrix-core tile) */
#define PC_RW 64
#define PC_PP 40       /* SPLIT: bf16 values per pair row (32 + pad: 80-byte pitch, conflict-free 16-byte reads) */
#define PC_TP 72       /* SPLIT: bf16 values per row of the transposed heads (64 pairs + pad) */

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

// floats of LDS per wave: fp32 basis rows [64][KP], or the SPLIT arrays (heads and remainders [64][PC_PP] bf16 each,
// mode 2 also the transposed heads [PC_KC][PC_TP]), then four 64-entry side arrays
__host__ __device__ constexpr int pc_wave_floats(int KP, bool split, int mode) {
  return (split ? (2 * 64 * PC_PP + (mode == 2 ? PC_KC * PC_TP : 0)) / 2 : 64 * KP) + 256;
}

// head and remainder of eight fp32 values as two bf16x8 operands
__device__ __forceinline__ void pc_split8(const float (&v)[8], uint4& hi, uint4& lo) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    h[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    // a plain rounded subtraction: were it contracted with a product that made v, the remainder would come from the
    // unrounded product in some copies of this code and from the rounded one in others
    l[i] = pack_bf16x2(sub_fixed(v[2 * i], bf16lo_to_f32(h[i])), sub_fixed(v[2 * i + 1], bf16hi_to_f32(h[i])));
  }
  hi = make_uint4(h[0], h[1], h[2], h[3]);
  lo = make_uint4(l[0], l[1], l[2], l[3]);
}
__device__ __forceinline__ floatx4 pc_mfma_split(const uint4& ahi, const uint4& alo, const uint4& bhi, const uint4& blo,
                                                 floatx4 c) {
  c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, alo), __builtin_bit_cast(bf16x8, bhi), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ahi), __builtin_bit_cast(bf16x8, blo), c, 0, 0, 0);
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ahi), __builtin_bit_cast(bf16x8, bhi), c, 0, 0, 0);
}

// LT: 3 with SPLIT for the L = 3 basis evaluated in registers (unrolled), else -1 (any L, values written one by one)
template <bool BF16, int MODE, bool VEC, bool SPLIT, int LT>
__global__ void __launch_bounds__(256) k_pc_dw(PcP p) {
  static_assert(LT == -1 || (LT == 3 && SPLIT), "the unrolled evaluation belongs to the split form");
  extern __shared__ float pc_lds[];
  constexpr int CPL = 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, sub = lane & 15;
  const int K1 = p.K + 1;
  const int nk4 = (K1 + 3) >> 2;
  const int KP = K1 | 1;
  const int kn = MODE == 2 ? min(PC_KC, p.K - p.kc0) : 0;
  const int per_wave = pc_wave_floats(KP, SPLIT, MODE);
  float* A = pc_lds;                                           // [4 nk4][64]: alpha rows, then c0, then zeros
  float* Bw = pc_lds + nk4 * 4 * PC_RW + wave * per_wave;      // this wave's [64][KP] (fp32 tiles)
  uint16_t* Ph = (uint16_t*)Bw;                                // SPLIT: [64][PC_PP] heads of this wave's basis rows,
  uint16_t* Pl = Ph + 64 * PC_PP;                              //        [64][PC_PP] remainders,
  uint16_t* Th = Pl + 64 * PC_PP;                              //        mode 2: [PC_KC][PC_TP] heads of rows kc0.., transposed
  float* tail = Bw + per_wave - 256;
  int32_t* Oth = (int32_t*)tail;                               // [64] gathered row of the current entry, -1 = none
  float* Wt = tail + 64;                                       // [64] weight of the gathered row (mode 1)
  float* Wrow = tail + 128;                                    // [64] 1/|N(row)|
  float* Wz = tail + 192;                                      // [64] SPLIT, mode 2: 1 - Z of the pair (fp32)
  float* red = pc_lds + nk4 * 4 * PC_RW + 4 * per_wave;        // [PC_KC + 1][64] (mode 2)
  if constexpr (SPLIT) {
    // columns K + 1 .. 31 of the pair rows and the unused rows of the transposed heads stay zero
    for (int i = lane; i < (per_wave - 256) / 4; i += 64) ((uint4*)Bw)[i] = make_uint4(0, 0, 0, 0);
  }
  // a pair's basis value k: fp32 tiles keep it as it is, SPLIT as head + remainder
  auto put = [&](int k, float x) {
    if constexpr (SPLIT) {
      const uint16_t h = (uint16_t)f32_to_bf16_bits(x);
      Ph[lane * PC_PP + k] = h;
      Pl[lane * PC_PP + k] = (uint16_t)f32_to_bf16_bits(sub_fixed(x, bf16_to_f32(h)));   // (never contracted: see pc_split8)
      if constexpr (MODE == 2) {
        const int kl = k - p.kc0;
        if (kl >= 0 && kl < PC_KC && k < p.K) Th[kl * PC_TP + lane] = h;
      }
    } else {
      Bw[lane * KP + k] = x;
    }
  };
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
    // SPLIT: the coefficient operand of lane (g, sub) for channel c0 + t: alpha'[8 g + j][c0 + t], j = 0..7, head and
    // remainder, kept in registers for the whole channel run
    uint4 bhi[SPLIT ? 4 : 1], blo[SPLIT ? 4 : 1];
    if constexpr (SPLIT) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = A[min(8 * g + j, nk4 * 4 - 1) * PC_RW + sub * CPL + t] * (8 * g + j < K1 ? 1.f : 0.f);
        pc_split8(v, bhi[t], blo[t]);
      }
    }
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

      // The chain entry -> (mode 1: owner of the pair ->) position and weight of the other point is two or three
      // dependent global loads.  It runs as a pipeline over the steps of four entries: every stage reads what the
      // previous stage loaded one step earlier, so no step waits for a load it has just issued.  Loads are
      // unconditional; a lane without an entry reads a valid dummy location (the row offsets) instead.
      auto has_at = [&](int jj) { return b + jj + g < e; };
      auto st_ent = [&](int jj) -> int32_t {
        const int32_t* a = has_at(jj) ? p.ent + (b + jj + g) : p.ptr;
        return *a;
      };
      auto st_other = [&](int jj, int32_t v) -> int32_t {
        if constexpr (MODE == 1) {
          const int32_t* a = has_at(jj) ? p.owner + v : p.ptr;
          v = *a;
        }
        return min(max(v, 0), (int32_t)max(p.n_other - 1, (int64_t)0));       // a bad id is never followed out of range
      };
      struct Pt { float x, y, z, wt; };
      auto st_point = [&](int jj, int32_t o) -> Pt {
        const bool h = has_at(jj);
        const float* xo = h ? p.x_other + 3 * (int64_t)o : p.x_row;
        Pt r;
        r.x = xo[0]; r.y = xo[1]; r.z = xo[2];
        r.wt = 1.f;
        if constexpr (MODE == 1) {
          const int32_t* qa = h ? p.q_ptr + o : p.ptr;
          r.wt = 1.0f / (float)max(qa[1] - qa[0], 1);
        }
        return r;
      };
      int32_t e2 = st_ent(8), e1 = st_ent(4);
      int32_t o1, o0;
      { const int32_t e0 = st_ent(0); o0 = st_other(0, e0); }
      o1 = st_other(4, e1);
      Pt pt0 = st_point(0, o0);

      for (int j4 = 0; j4 < maxdeg; j4 += 4) {
        __builtin_amdgcn_wave_barrier();        // the previous entries' basis rows have been read
        const bool has = has_at(j4);
        const int32_t other = o0;
        const Pt pt = pt0;
        // next step's point, the step after's id, the one after that's entry
        pt0 = st_point(j4 + 4, o1);
        o0 = o1;
        o1 = st_other(j4 + 8, e2);
        e2 = st_ent(j4 + 12);
        if (has) {
          const float dx = p.sign * (pt.x - xr[0]), dyy = p.sign * (pt.y - xr[1]), dz = p.sign * (pt.z - xr[2]);
          const float r = sqrtf(norm2_fixed(dx, dyy, dz));
          const float Z = fminf(r * p.inv_rho, 1.0f);
          float ux = 0.f, uy = 0.f, uz = 1.f;
          if (r > 0.f) { const float ir = 1.0f / r; ux = dx * ir; uy = dyy * ir; uz = dz * ir; }
          if constexpr (LT == 3) {
            // the 16 values and 1 - Z in registers, split pairwise by the conversion instruction, three 16-byte stores
            // each for heads and remainders (columns 17 .. 23 zero; 24 .. 31 stay zero from the start)
            float bv[24];
#pragma unroll
            for (int k = 17; k < 24; ++k) bv[k] = 0.f;
            sh_eval<3>(ux, uy, uz, p.sh, [&](int k, float v) { bv[k] = Z * v; });
            bv[16] = 1.0f - Z;
#pragma unroll
            for (int o = 0; o < 3; ++o) {
              float x8[8];
#pragma unroll
              for (int i = 0; i < 8; ++i) x8[i] = bv[8 * o + i];
              uint4 hi, lo;
              pc_split8(x8, hi, lo);
              *(uint4*)(Ph + lane * PC_PP + 8 * o) = hi;
              *(uint4*)(Pl + lane * PC_PP + 8 * o) = lo;
              if constexpr (MODE == 2) {     // K = 16: one pass, kc0 = 0
                if (o < 2) {
                  const uint32_t w[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                  for (int i = 0; i < 8; ++i)
                    Th[(8 * o + i) * PC_TP + lane] = (uint16_t)((i & 1) ? (w[i >> 1] >> 16) : (w[i >> 1] & 0xffffu));
                }
              }
            }
          } else {
            sh_eval_any(ux, uy, uz, p.sh, [&](int k, float v) { put(k, Z * v); });
            put(p.K, 1.0f - Z);
          }
          if constexpr (SPLIT && MODE == 2) Wz[lane] = 1.0f - Z;
          Oth[lane] = other;
          Wt[lane] = pt.wt;
        } else {
          if constexpr (LT == 3) {
#pragma unroll
            for (int o = 0; o < 3; ++o) {
              *(uint4*)(Ph + lane * PC_PP + 8 * o) = make_uint4(0, 0, 0, 0);
              *(uint4*)(Pl + lane * PC_PP + 8 * o) = make_uint4(0, 0, 0, 0);
            }
            if constexpr (MODE == 2) {
#pragma unroll
              for (int k = 0; k < 16; ++k) Th[k * PC_TP + lane] = 0;
            }
          } else {
            for (int k = 0; k < K1; ++k) put(k, 0.f);
          }
          if constexpr (SPLIT && MODE == 2) Wz[lane] = 0.f;
          Oth[lane] = -1;
          Wt[lane] = 0.f;
        }
        const uint64_t live = __ballot(has);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        uint32_t dPk[(MODE == 2 && SPLIT) ? 4 : 1][4];   // bf16 products h (.) dy of the lane's eight pairs of a tile
        constexpr bool RAW16 = MODE == 1 || !BF16;        // the gathered rows are fp32 (16 bytes a lane), else bf16 (8)
        constexpr int SG = VEC ? (RAW16 ? 2 : 4) : 0;     // slots whose gathered rows are in flight together
        uint4 raw[SG > 0 ? SG : 1][4];
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          if constexpr (MODE == 2 && SPLIT) {
            if ((s4 & 1) == 0) {
#pragma unroll
              for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j) dPk[t][j] = 0u;
            }
          }
          if constexpr (SG > 0) {
            // whole aligned channel runs: the gathered rows of SG slots are requested together, ahead of the arithmetic
            // of the first (a slot without entries reads row 0, unused)
            if ((s4 % SG) == 0) {
#pragma unroll
              for (int u = 0; u < SG; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                  const int64_t ol = max(Oth[16 * (s4 + u) + 4 * g + q], 0);
                  if constexpr (RAW16) raw[u][q] = *(const uint4*)((const float*)p.G + ol * p.C + cl);
                  else {
                    const uint2 w = *(const uint2*)((const uint16_t*)p.G + ol * p.C + cl);
                    raw[u][q].x = w.x; raw[u][q].y = w.y;
                  }
                }
            }
          }
          if (((live >> (16 * s4)) & 0xffffull) != 0) {     // the same for the whole wave
          float hv[4][CPL];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int rr = 16 * s4 + 4 * g + q;
            const int32_t o = Oth[rr];
            const bool ok = o >= 0 && cok;
#pragma unroll
            for (int t = 0; t < CPL; ++t) hv[q][t] = 0.f;
            if constexpr (SG > 0) {
              const uint4 w = raw[s4 % SG][q];
              if constexpr (RAW16) {
                hv[q][0] = __uint_as_float(w.x); hv[q][1] = __uint_as_float(w.y);
                hv[q][2] = __uint_as_float(w.z); hv[q][3] = __uint_as_float(w.w);
              } else {
                hv[q][0] = bf16lo_to_f32(w.x); hv[q][1] = bf16hi_to_f32(w.x);
                hv[q][2] = bf16lo_to_f32(w.y); hv[q][3] = bf16hi_to_f32(w.y);
              }
            } else if (ok) {
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
            if constexpr (SPLIT) {
              // lane (g, sub): basis values 8 g .. 8 g + 7 of row sub's entry in slot s4
              const uint4 ahi = *(const uint4*)(Ph + (16 * s4 + sub) * PC_PP + 8 * g);
              const uint4 alo = *(const uint4*)(Pl + (16 * s4 + sub) * PC_PP + 8 * g);
#pragma unroll
              for (int t = 0; t < 4; ++t) S[t] = pc_mfma_split(ahi, alo, bhi[t], blo[t], S[t]);
            } else {
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
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
              for (int t = 0; t < 4; ++t) acc[q][t] = fmaf(hv[q][t], S[t][q], acc[q][t]);   // explicit: the three modes round alike
          }
          if constexpr (MODE == 2) {
            float pe[4][CPL];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int rr = 16 * s4 + 4 * g + q;
#pragma unroll
              for (int t = 0; t < CPL; ++t) pe[q][t] = hv[q][t] * dyr[q][t];      // hv is 0 where there is no pair
              if constexpr (!SPLIT) {
                const float bv = Bw[rr * KP + p.kc0 + min(sub, kn - 1)];
                const float a = sub < kn ? bv : 0.f;
#pragma unroll
                for (int t = 0; t < 4; ++t) D[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, pe[q][t], D[t], 0, 0, 0);
              }
              if (p.kc0 == 0) {
                const float z1 = SPLIT ? Wz[rr] : Bw[rr * KP + p.K];
#pragma unroll
                for (int t = 0; t < 4; ++t) E[t] = fmaf(z1, pe[q][t], E[t]);
              }
            }
            if constexpr (SPLIT) {
              // elements 4 (s4 % 2) + q of the lane's eight pairs of a tile
#pragma unroll
              for (int t = 0; t < 4; ++t) {
                dPk[t][(s4 & 1) * 2] = pack_bf16x2(pe[0][t], pe[1][t]);
                dPk[t][(s4 & 1) * 2 + 1] = pack_bf16x2(pe[2][t], pe[3][t]);
              }
            }
          }
          }
          if constexpr (MODE == 2 && SPLIT) {
            // two slots x four rows of each lane group = the 32 pairs of one tile:
            //   D[k][c] += sum_pairs B'[pair][kc0 + k] pe[pair][c],  lane (g, sub): k = sub, pairs (slot, row 4 g + q)
            if ((s4 & 1) == 1 && ((live >> (16 * (s4 - 1))) & 0xffffull) != 0) {
              const uint2 a0 = *(const uint2*)(Th + sub * PC_TP + 16 * (s4 - 1) + 4 * g);
              const uint2 a1 = *(const uint2*)(Th + sub * PC_TP + 16 * s4 + 4 * g);
              const uint4 av = make_uint4(a0.x, a0.y, a1.x, a1.y);
#pragma unroll
              for (int t = 0; t < 4; ++t)
                D[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    __builtin_bit_cast(bf16x8, av),
                    __builtin_bit_cast(bf16x8, make_uint4(dPk[t][0], dPk[t][1], dPk[t][2], dPk[t][3])), D[t], 0, 0, 0);
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

static size_t pc_lds_bytes(int K, bool split, int mode) {
  const int K1 = K + 1, nk4 = (K1 + 3) / 4, KP = K1 | 1;
  return ((size_t)nk4 * 4 * PC_RW + (size_t)4 * pc_wave_floats(KP, split, mode) + (size_t)(PC_KC + 1) * PC_RW) * sizeof(float);
}

template <int MODE>
static pm_status pc_launch(const PcP& p, int is_bf16, bool vec, int grid, hipStream_t st) {
  const bool split = is_bf16 && p.K + 1 <= 32;     // one 32-deep bf16 tile holds every basis row
  const bool l3 = split && p.sh.L == 3 && p.K == 16;
  auto kern = is_bf16 ? (split ? (l3 ? (vec ? k_pc_dw<true, MODE, true, true, 3> : k_pc_dw<true, MODE, false, true, 3>)
                                     : (vec ? k_pc_dw<true, MODE, true, true, -1> : k_pc_dw<true, MODE, false, true, -1>))
                               : (vec ? k_pc_dw<true, MODE, true, false, -1> : k_pc_dw<true, MODE, false, false, -1>))
                      : (vec ? k_pc_dw<false, MODE, true, false, -1> : k_pc_dw<false, MODE, false, false, -1>);
  const size_t lds = pc_lds_bytes(p.K, split, MODE);
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
