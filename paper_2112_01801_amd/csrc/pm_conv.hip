// Row-wise SH contraction on the matrix cores, weight packing, and the deterministic segmented reduction.
//
// conv_rows computes, for every row r (a facet or a texture point),
//     out[r][n] = sum_k B_r[k] * ( sum_c X_r[c] * Wp[k][c][n] )
// i.e. Eq. 5's summand F(theta_r, phi_r) h_r with dense coefficients, re-associated so that the SH
// weighting happens on the accumulators:  U_k = Wp[k]^T x_r  is a plain GEMM (matrix cores), and
// out = sum_k B_r[k] U_k is an fp32 FMA epilogue.  The Khatri-Rao operand B_r (x) x_r is never formed.
//
// The GEMM is laid out "transposed": MFMA rows = output channels n, MFMA columns = rows r.  Then every
// lane owns ONE row r (column l%32 of the 32x32 tile) and 16 output channels, so the basis values
// B_r[k] it multiplies with are the lane's own registers.
//
// Weights are pre-packed (pm_launch_pack) into the exact per-lane operand image: a "stage" is the
// 8 KiB block for one (n-block pair, c-chunk, k); a wave reads its A fragments as 16-byte LDS loads.
// If all stages fit in LDS they are loaded once per workgroup (which then loops over row tiles);
// otherwise they stream through a two-slot ring, one barrier per stage.
#include "pm_conv_kernel.h"

// ------------------------------------------------------------------------------------------------
// weight packing
// ------------------------------------------------------------------------------------------------
struct PackP {
  int mode, src_bf16, dst_bf16;
  int K, cin, cout;   // source W[K][cin][cout]
  int Kp, Cc, Cn;     // packed logical Wp[Kp][Cc][Cn]
  int NCH, NBG;
  const void* W;
  const float* alpha;   // SEP modes: per-channel SH coefficients [K][cin]; W is then the point-wise matrix [cin][cout]
  uint4* out;
  FoldCoef fc;
};

__device__ __forceinline__ float pack_src(const PackP& p, int k, int ci, int co) {
  int64_t o = ((int64_t)k * p.cin + ci) * p.cout + co;
  return p.src_bf16 ? bf16_to_f32(((const uint16_t*)p.W)[o]) : ((const float*)p.W)[o];
}

// logical Wp[k][c][n], N consecutive c starting at c0.  The folded forms sum over k in ascending order; the
// loads of all N elements for two k at a time are issued before the additions.
//   PLAIN: W[k][c][n]   TRANS: W[k][n][c]   FOLD: sum_k fc[j][k] W[k][ci][n], c = j*cin+ci
//   FOLD_TRANS: sum_k fc[j][k] W[k][ci][c], n = j*cin+ci      FOLD_BWD: sum_k fc[j][k] W[k][n][co], c = j*cout+co
template <int MODE, int N>
__device__ __forceinline__ void pack_values(const PackP& p, int k, int c0, int n, float (&v)[N]) {
  int j[N], ci[N], co[N];
  bool ok[N];
#pragma unroll
  for (int e = 0; e < N; ++e) {
    const int c = c0 + e;
    ok[e] = c < p.Cc && n < p.Cn;
    j[e] = 0;
    if (MODE == PACK_PLAIN) { ci[e] = c; co[e] = n; }
    else if (MODE == PACK_PLAIN_TWICE) { ci[e] = c & 63; co[e] = n; ok[e] = ok[e] && ci[e] < p.cin; }
    else if (MODE == PACK_TRANS) { ci[e] = n; co[e] = c; }
    else if (MODE == PACK_FOLD) { j[e] = c / p.cin; ci[e] = c - j[e] * p.cin; co[e] = n; }
    else if (MODE == PACK_FOLD_TRANS) { j[e] = n / p.cin; ci[e] = n - j[e] * p.cin; co[e] = c; }
    else if (MODE == PACK_FOLD_BWD) { j[e] = c / p.cout; ci[e] = n; co[e] = c - j[e] * p.cout; }
    else { j[e] = c / p.cin; ci[e] = c - j[e] * p.cin; co[e] = n; }   // PACK_SEP_FOLD
    if (!ok[e]) { j[e] = 0; ci[e] = 0; co[e] = 0; }   // in-bounds dummy, the value is dropped
    v[e] = 0.f;
  }
  if (MODE == PACK_PLAIN || MODE == PACK_TRANS || MODE == PACK_PLAIN_TWICE) {
#pragma unroll
    for (int e = 0; e < N; ++e) v[e] = ok[e] ? pack_src(p, k, ci[e], co[e]) : 0.f;
    return;
  }
  if (MODE == PACK_SEP_FOLD) {
    // s_j[ci] * P[ci][co],  s_j[ci] = sum_k fc[j][k] alpha[k][ci]
#pragma unroll
    for (int e = 0; e < N; ++e) {
      float sj = 0.f;
      for (int kk = 0; kk < p.K; ++kk) sj += p.fc.c[j[e]][kk] * p.alpha[(int64_t)kk * p.cin + ci[e]];
      v[e] = ok[e] ? sj * pack_src(p, 0, ci[e], co[e]) : 0.f;
    }
    return;
  }
  // KB values of k per batch: their loads are issued together, the additions follow in ascending k
  constexpr int KB = N == 1 ? 8 : 2;
  int kk = 0;
  for (; kk + KB <= p.K; kk += KB) {
    float w[KB][N];
#pragma unroll
    for (int q = 0; q < KB; ++q)
#pragma unroll
      for (int e = 0; e < N; ++e) w[q][e] = pack_src(p, kk + q, ci[e], co[e]);
#pragma unroll
    for (int q = 0; q < KB; ++q)
#pragma unroll
      for (int e = 0; e < N; ++e) v[e] += p.fc.c[j[e]][kk + q] * w[q][e];
  }
  for (; kk < p.K; ++kk)
#pragma unroll
    for (int e = 0; e < N; ++e) v[e] += p.fc.c[j[e]][kk] * pack_src(p, kk, ci[e], co[e]);
#pragma unroll
  for (int e = 0; e < N; ++e) v[e] = ok[e] ? v[e] : 0.f;
}

// one thread per element of the image: the image is small (128 KB at K = 16, 64 x 64), so the kernel lives on its
// launch and on how many threads share the strided reads (and, in the folded forms, the K loads of an element)
template <int MODE>
__global__ void __launch_bounds__(256) k_pack_elem(PackP p, int64_t n_elem) {
  const int64_t te = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (te >= n_elem) return;
  const int EPG = p.dst_bf16 ? 8 : 4;
  const int e = (int)(te % EPG);
  const int64_t t = te / EPG;
  const int lane = (int)(t & 63);
  int64_t q = t >> 6;
  const int g = (int)(q % PM_GC); q /= PM_GC;
  const int nbi = (int)(q % PM_NBS); q /= PM_NBS;
  const int64_t stage = q;
  const int k = (int)(stage % p.Kp);
  const int ch = (int)((stage / p.Kp) % p.NCH);
  const int nbg = (int)(stage / ((int64_t)p.Kp * p.NCH));
  const int n = (nbg * PM_NBS + nbi) * 32 + (lane & 31);
  const int hh = lane >> 5;
  const int c0 = ((ch * PM_GC + g) * 2 + hh) * EPG + e;
  float v[1];
  pack_values<MODE, 1>(p, k, c0, n, v);
  if (p.dst_bf16) ((uint16_t*)p.out)[te] = (uint16_t)f32_to_bf16_bits(v[0]);
  else ((float*)p.out)[te] = v[0];
}

pm_status pm_launch_pack(PackMode mode, pm_dtype dt, int K, int cin, int cout, const void* W, const FoldCoef* fc,
                         void* apack, hipStream_t st, const float* alpha) {
  PackP p;
  p.mode = mode; p.src_bf16 = (dt == PM_BF16); p.dst_bf16 = (dt == PM_BF16);
  p.K = K; p.cin = cin; p.cout = cout;
  switch (mode) {
    case PACK_PLAIN: p.Kp = K; p.Cc = cin; p.Cn = cout; break;
    case PACK_PLAIN_TWICE: p.Kp = 1; p.Cc = 128; p.Cn = cout; break;
    case PACK_TRANS: p.Kp = K; p.Cc = cout; p.Cn = cin; break;
    case PACK_FOLD: case PACK_SEP_FOLD: p.Kp = 1; p.Cc = 3 * cin; p.Cn = cout; break;
    case PACK_FOLD_TRANS: p.Kp = 1; p.Cc = cout; p.Cn = 3 * cin; break;
    default: p.Kp = 1; p.Cc = 3 * cout; p.Cn = cin; break;
  }
  PackGeom g = pm_pack_geom(p.Kp, p.Cc, p.Cn, dt);
  p.NCH = g.NCH; p.NBG = g.NBG;
  p.W = W; p.alpha = alpha; p.out = (uint4*)apack;
  if (fc) p.fc = *fc; else for (int j = 0; j < 3; ++j) for (int k = 0; k < PM_MAX_K; ++k) p.fc.c[j][k] = 0.f;
  // one thread per element of the image
  const int64_t n_elem = g.stages * STAGE_U4 * (p.dst_bf16 ? 8 : 4);
  { ProfScope ps__(st, "k_pack");
    const dim3 ge((unsigned)((n_elem + 255) / 256));
    switch (mode) {
      case PACK_PLAIN: hipLaunchKernelGGL(k_pack_elem<PACK_PLAIN>, ge, dim3(256), 0, st, p, n_elem); break;
      case PACK_PLAIN_TWICE: hipLaunchKernelGGL(k_pack_elem<PACK_PLAIN_TWICE>, ge, dim3(256), 0, st, p, n_elem); break;
      case PACK_TRANS: hipLaunchKernelGGL(k_pack_elem<PACK_TRANS>, ge, dim3(256), 0, st, p, n_elem); break;
      case PACK_FOLD: hipLaunchKernelGGL(k_pack_elem<PACK_FOLD>, ge, dim3(256), 0, st, p, n_elem); break;
      case PACK_FOLD_TRANS: hipLaunchKernelGGL(k_pack_elem<PACK_FOLD_TRANS>, ge, dim3(256), 0, st, p, n_elem); break;
      case PACK_FOLD_BWD: hipLaunchKernelGGL(k_pack_elem<PACK_FOLD_BWD>, ge, dim3(256), 0, st, p, n_elem); break;
      default: hipLaunchKernelGGL(k_pack_elem<PACK_SEP_FOLD>, ge, dim3(256), 0, st, p, n_elem); break;
    } }
  PM_CHECK_LAUNCH("k_pack");
  return PM_OK;
}

// ------------------------------------------------------------------------------------------------
// conv_rows dispatch (kernels live in pm_conv_kernel.h, instantiated by pm_conv_i*.hip)
// ------------------------------------------------------------------------------------------------
PM_CONV_DECLARE(0, B_NORMAL, X_DIRECT)
PM_CONV_DECLARE(0, B_NORMAL, X_GATHER_SUM)
PM_CONV_DECLARE(0, B_DIRS, X_DIRECT)
PM_CONV_DECLARE(0, B_DIRS, X_GATHER1)
PM_CONV_DECLARE(0, B_ONE, X_DIRECT)
PM_CONV_DECLARE(0, B_ONE, X_GATHER_CAT)
PM_CONV_DECLARE(1, B_NORMAL, X_DIRECT)
PM_CONV_DECLARE(1, B_NORMAL, X_GATHER_SUM)
PM_CONV_DECLARE(1, B_DIRS, X_DIRECT)
PM_CONV_DECLARE(1, B_DIRS, X_GATHER1)
PM_CONV_DECLARE(1, B_ONE, X_DIRECT)
PM_CONV_DECLARE(1, B_ONE, X_GATHER_CAT)

// LDS a workgroup may use on the current device (bytes)
static size_t pm_lds_max_bytes() {
  static int cached = -1;
  if (cached < 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
      v = 64 * 1024;
    cached = v;
  }
  return (size_t)cached;
}
// Largest weight image kept resident in LDS: 128 KiB, or less when the device offers less per workgroup.
static size_t lds_resident_max() {
  const size_t cap = pm_lds_max_bytes();
  return cap < 128 * 1024 ? cap : 128 * 1024;
}

#define PM_CONV_CASE(DT, BM, XM) \
  if (dt == DT && bm == BM && xm == XM) return pm_conv_dispatch_##DT##_##BM##_##XM(p, L, g.stages, st);

pm_status pm_launch_conv_rows(pm_dtype mt, BMode bm, XMode xm, int64_t R, int K, int Cc, int Cn, const BasisSrc& bs,
                              const RowSrc& xs, const void* apack, void* out, int out_is_bf16, hipStream_t st) {
  if (R == 0) return PM_OK;
  PackGeom g = pm_pack_geom(K, Cc, Cn, mt);
  ConvP p;
  p.R = R; p.Cc = Cc; p.Cn = Cn; p.NCH = g.NCH; p.NBG = g.NBG;
  p.resident = pm_pack_bytes(g) <= lds_resident_max();
  p.bs = bs; p.xs = xs; p.apack = (const uint4*)apack; p.out = out; p.out_bf16 = out_is_bf16;
  p.store_fast = (Cn % (PM_NBS * 32) == 0) && pm_aligned16(out);
  const int L = (bm == B_ONE) ? 0 : bs.sh.L;
  const int dt = (mt == PM_BF16) ? 1 : 0;
  PM_CONV_CASE(0, B_NORMAL, X_DIRECT)
  PM_CONV_CASE(0, B_NORMAL, X_GATHER_SUM)
  PM_CONV_CASE(0, B_DIRS, X_DIRECT)
  PM_CONV_CASE(0, B_DIRS, X_GATHER1)
  PM_CONV_CASE(0, B_ONE, X_DIRECT)
  PM_CONV_CASE(0, B_ONE, X_GATHER_CAT)
  PM_CONV_CASE(1, B_NORMAL, X_DIRECT)
  PM_CONV_CASE(1, B_NORMAL, X_GATHER_SUM)
  PM_CONV_CASE(1, B_DIRS, X_DIRECT)
  PM_CONV_CASE(1, B_DIRS, X_GATHER1)
  PM_CONV_CASE(1, B_ONE, X_DIRECT)
  PM_CONV_CASE(1, B_ONE, X_GATHER_CAT)
  return pm_fail(PM_ERR_UNSUPPORTED, "conv_rows mode (%d,%d)", (int)bm, (int)xm);
}

// ------------------------------------------------------------------------------------------------
// segmented reduction (facet -> vertex mean of Eq. 5; corner -> vertex sum of Eq. 6's backward;
// texture point -> facet mean of Eq. 7).  One lane group per segment, lanes span channels, entries
// are added in ascending order: no atomics, bitwise reproducible.
// ------------------------------------------------------------------------------------------------
struct SegP {
  int64_t n_seg;
  int C, div, mean, out_bf16, lpg;  // lpg = lanes per segment (power of two, <= 64)
  const void* src;                  // fp32 or bf16 rows
  const int32_t* row_ptr;
  const int32_t* col;
  void* out;
};

// SRC_BF16: the rows being reduced are bf16 (8 channels = 16 bytes per lane) instead of fp32 (4 channels).
// DIV: compile-time divisor of the column entries (1, 3) or 0 for the run-time value.
// The entries of a segment are taken NB at a time: first the column entries (one cooperative load of the segment's
// lane group where it has at least NB lanes), then the rows they name (all in flight together), then the additions,
// strictly in ascending entry order.
template <bool SRC_BF16, int DIV, int NB>
__global__ void __launch_bounds__(256) k_segreduce(SegP p) {
  constexpr int CPL = SRC_BF16 ? 8 : 4;
  const int gpb = 256 / p.lpg;  // segments per block
  const int sub = threadIdx.x % p.lpg;
  for (int64_t seg = (int64_t)blockIdx.x * gpb + threadIdx.x / p.lpg; seg < p.n_seg; seg += (int64_t)gridDim.x * gpb) {
  const int32_t b = p.row_ptr[seg], e = p.row_ptr[seg + 1];
  const float scale = (p.mean && e > b) ? 1.0f / (float)(e - b) : 1.0f;
  const bool vec = (p.C % CPL) == 0 && pm_aligned16_dev(p.src);
  // enough lanes per segment to fetch a batch of column entries in one load, and every lane of the group takes the
  // same trips through the channel loop (a lane that has left the loop cannot hand its entry on)
  const bool coop = p.lpg >= NB && (p.C % (p.lpg * CPL)) == 0;
  auto row_of = [&](int32_t i) -> int64_t {
    if (!p.col) return (int64_t)i;
    const int32_t c = p.col[i];
    if constexpr (DIV == 1) return (int64_t)c;
    else if constexpr (DIV == 3) return (int64_t)(((uint64_t)(uint32_t)c * 0xAAAAAAABull) >> 33);
    else return (int64_t)(c / p.div);
  };
  for (int c0 = sub * CPL; c0 < p.C; c0 += p.lpg * CPL) {
    float a[CPL];
#pragma unroll
    for (int i = 0; i < CPL; ++i) a[i] = 0.f;
    if (vec) {
      for (int32_t i0 = b; i0 < e; i0 += NB) {
        int64_t r[NB];
        if (coop) {
          // the lanes of the group fetch the batch's column entries together (one coalesced load), then hand them
          // round: every row address of the batch is known after ONE memory latency
          const int64_t mine = row_of(min(i0 + min(sub, NB - 1), e - 1));
#pragma unroll
          for (int j = 0; j < NB; ++j) r[j] = __shfl((int)mine, (threadIdx.x & 63 & ~(p.lpg - 1)) + j, 64);
        } else {
#pragma unroll
          for (int j = 0; j < NB; ++j) r[j] = row_of(min(i0 + j, e - 1));   // clamped: loads are unconditional
        }
        uint4 u[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const int64_t o = r[j] * p.C + c0;
          if constexpr (SRC_BF16) u[j] = *(const uint4*)((const uint16_t*)p.src + o);
          else u[j] = *(const uint4*)((const float*)p.src + o);
        }
        __builtin_amdgcn_sched_barrier(0);   // every load of the batch is out before the first addition waits
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          if (i0 + j >= e) u[j] = make_uint4(0, 0, 0, 0);   // a select: adding +0 leaves the sum as it is
          if constexpr (SRC_BF16) {
            a[0] += bf16lo_to_f32(u[j].x); a[1] += bf16hi_to_f32(u[j].x); a[2] += bf16lo_to_f32(u[j].y);
            a[3] += bf16hi_to_f32(u[j].y); a[4] += bf16lo_to_f32(u[j].z); a[5] += bf16hi_to_f32(u[j].z);
            a[6] += bf16lo_to_f32(u[j].w); a[7] += bf16hi_to_f32(u[j].w);
          } else {
            a[0] += __uint_as_float(u[j].x); a[1] += __uint_as_float(u[j].y);
            a[2] += __uint_as_float(u[j].z); a[3] += __uint_as_float(u[j].w);
          }
        }
      }
    } else {
      for (int32_t i = b; i < e; ++i) {
        const int64_t o = row_of(i) * p.C + c0;
#pragma unroll
        for (int q = 0; q < CPL; ++q)
          if (c0 + q < p.C)
            a[q] += SRC_BF16 ? bf16_to_f32(((const uint16_t*)p.src)[o + q]) : ((const float*)p.src)[o + q];
      }
    }
#pragma unroll
    for (int i = 0; i < CPL; ++i) a[i] *= scale;
    const int64_t o = seg * p.C + c0;
    if (vec && (p.C % 4) == 0 && pm_aligned16_dev(p.out)) {
      if (p.out_bf16) {
#pragma unroll
        for (int q = 0; q < CPL / 4; ++q) {
          uint2 w;
          w.x = pack_bf16x2(a[4 * q], a[4 * q + 1]); w.y = pack_bf16x2(a[4 * q + 2], a[4 * q + 3]);
          *(uint2*)((uint16_t*)p.out + o + 4 * q) = w;
        }
      } else {
#pragma unroll
        for (int q = 0; q < CPL / 4; ++q)
          *(float4*)((float*)p.out + o + 4 * q) = make_float4(a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < CPL; ++i)
        if (c0 + i < p.C) {
          if (p.out_bf16) ((uint16_t*)p.out)[o + i] = (uint16_t)f32_to_bf16_bits(a[i]);
          else ((float*)p.out)[o + i] = a[i];
        }
    }
  }
  }
}

template <bool SRC_BF16>
static void launch_segreduce_div(const SegP& p, dim3 grid, hipStream_t st) {
  // six entries per batch -- the mean valence of a triangle mesh, so most segments take one batch: one latency for the
  // column entries (fetched by the lanes of the group in one load), one for the rows, all in flight together.
  // Measured on MI355X at config 3: two entries per batch, each lane fetching its own, 0.118 ms; four per batch with
  // the cooperative fetch 0.107; six 0.089; eight (two wasted row requests per segment) 0.109
  if (p.div == 1) hipLaunchKernelGGL((k_segreduce<SRC_BF16, 1, 6>), grid, dim3(256), 0, st, p);
  else if (p.div == 3) hipLaunchKernelGGL((k_segreduce<SRC_BF16, 3, 6>), grid, dim3(256), 0, st, p);
  else hipLaunchKernelGGL((k_segreduce<SRC_BF16, 0, 6>), grid, dim3(256), 0, st, p);
}

pm_status pm_launch_segreduce(int64_t n_seg, int C, const void* src, int src_is_bf16, const int32_t* row_ptr,
                              const int32_t* col, int div, int mean, void* out, int out_is_bf16, hipStream_t st) {
  if (n_seg == 0) return PM_OK;
  if (div < 1) return pm_fail(PM_ERR_INVALID_ARG, "segreduce divisor %d", div);
  SegP p;
  p.n_seg = n_seg; p.C = C; p.div = div; p.mean = mean; p.out_bf16 = out_is_bf16;
  p.src = src; p.row_ptr = row_ptr; p.col = col; p.out = out;
  const int cpl = src_is_bf16 ? 8 : 4;
  int need = (C + cpl - 1) / cpl, lpg = 1;
  while (lpg < need && lpg < 64) lpg <<= 1;
  p.lpg = lpg;
  int gpb = 256 / lpg;
  int64_t nblk = (n_seg + gpb - 1) / gpb;
  if (nblk > 0x7fffffff) nblk = 0x7fffffff;   // the kernel strides over the segments
  const dim3 grid((unsigned)nblk);
  { ProfScope ps__(st, "k_segreduce");
    if (src_is_bf16) launch_segreduce_div<true>(p, grid, st);
    else launch_segreduce_div<false>(p, grid, st); }
  PM_CHECK_LAUNCH("k_segreduce");
  return PM_OK;
}

// Corner-slot sums at the vertices (backward of Eq. 6 before the matrix): one lane group per vertex, lanes
// span channels; an adjacency entry 3f+j adds row f to slot j.  Entries are taken two at a time (both rows
// in flight), added in ascending order; the slot is chosen by selects, so the code has no divergent branch.
template <bool SRC_BF16>
__global__ void __launch_bounds__(256) k_segsum_slots(SegP p) {
  constexpr int CPL = SRC_BF16 ? 8 : 4;
  constexpr int NB = 2;   // entries per batch (their rows in flight together; four measured slower here)
  const int gpb = 256 / p.lpg;
  const int sub = threadIdx.x % p.lpg;
  const bool vec = (p.C % CPL) == 0 && pm_aligned16_dev(p.src) && pm_aligned16_dev(p.out);
  for (int64_t seg = (int64_t)blockIdx.x * gpb + threadIdx.x / p.lpg; seg < p.n_seg; seg += (int64_t)gridDim.x * gpb) {
    const int32_t b = p.row_ptr[seg], e = p.row_ptr[seg + 1];
    for (int c0 = sub * CPL; c0 < p.C; c0 += p.lpg * CPL) {
      float a[3][CPL];
#pragma unroll
      for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int i = 0; i < CPL; ++i) a[j][i] = 0.f;
      for (int32_t i0 = b; i0 < e; i0 += NB) {
        int32_t cidx[NB];
        float x[NB][CPL];
        if (p.lpg >= NB && (p.C % (p.lpg * CPL)) == 0) {   // the group's lanes (all in this loop) fetch the batch's entries in one load
          const int32_t mine = p.col[min(i0 + (sub & (NB - 1)), e - 1)];
#pragma unroll
          for (int q = 0; q < NB; ++q) cidx[q] = __shfl(mine, (threadIdx.x & 63 & ~(p.lpg - 1)) + q, 64);
        } else {
#pragma unroll
          for (int q = 0; q < NB; ++q) cidx[q] = p.col[min(i0 + q, e - 1)];
        }
#pragma unroll
        for (int q = 0; q < NB; ++q) {
          const int64_t r = (int64_t)(((uint64_t)(uint32_t)cidx[q] * 0xAAAAAAABull) >> 33);   // / 3
          const int64_t o = r * p.C + c0;
          if (vec) {
            const uint4 u = SRC_BF16 ? *(const uint4*)((const uint16_t*)p.src + o) : *(const uint4*)((const float*)p.src + o);
            if constexpr (SRC_BF16) {
              x[q][0] = bf16lo_to_f32(u.x); x[q][1] = bf16hi_to_f32(u.x); x[q][2] = bf16lo_to_f32(u.y); x[q][3] = bf16hi_to_f32(u.y);
              x[q][4] = bf16lo_to_f32(u.z); x[q][5] = bf16hi_to_f32(u.z); x[q][6] = bf16lo_to_f32(u.w); x[q][7] = bf16hi_to_f32(u.w);
            } else {
              x[q][0] = __uint_as_float(u.x); x[q][1] = __uint_as_float(u.y); x[q][2] = __uint_as_float(u.z); x[q][3] = __uint_as_float(u.w);
            }
          } else {
#pragma unroll
            for (int i = 0; i < CPL; ++i) {
              float t = 0.f;
              if (c0 + i < p.C) t = SRC_BF16 ? bf16_to_f32(((const uint16_t*)p.src)[o + i]) : ((const float*)p.src)[o + i];
              x[q][i] = t;
            }
          }
        }
#pragma unroll
        for (int q = 0; q < NB; ++q) {
          const int slot = (i0 + q < e) ? cidx[q] - 3 * (int32_t)(((uint64_t)(uint32_t)cidx[q] * 0xAAAAAAABull) >> 33) : 3;
          // one 0/1 weight per slot and a multiply-add per element (a + 1 x and a + 0 x are exact: the sums are the
          // plain ascending-order sums of each slot); cheaper than a select and an add per element
#pragma unroll
          for (int j = 0; j < 3; ++j) {
            const float m = (slot == j) ? 1.f : 0.f;
#pragma unroll
            for (int i = 0; i < CPL; ++i) a[j][i] = fmaf(m, x[q][i], a[j][i]);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const int64_t o = (seg * 3 + j) * p.C + c0;
        if (vec) {
          if (p.out_bf16) {
#pragma unroll
            for (int q = 0; q < CPL / 4; ++q) {
              uint2 w;
              w.x = pack_bf16x2(a[j][4 * q], a[j][4 * q + 1]); w.y = pack_bf16x2(a[j][4 * q + 2], a[j][4 * q + 3]);
              *(uint2*)((uint16_t*)p.out + o + 4 * q) = w;
            }
          } else {
#pragma unroll
            for (int q = 0; q < CPL / 4; ++q)
              *(float4*)((float*)p.out + o + 4 * q) = make_float4(a[j][4 * q], a[j][4 * q + 1], a[j][4 * q + 2], a[j][4 * q + 3]);
          }
        } else {
#pragma unroll
          for (int i = 0; i < CPL; ++i)
            if (c0 + i < p.C) {
              if (p.out_bf16) ((uint16_t*)p.out)[o + i] = (uint16_t)f32_to_bf16_bits(a[j][i]);
              else ((float*)p.out)[o + i] = a[j][i];
            }
        }
      }
    }
  }
}

pm_status pm_launch_segsum_slots(int64_t n_seg, int C, const void* src, int src_is_bf16, const int32_t* row_ptr,
                                 const int32_t* col, void* out, int out_is_bf16, hipStream_t st) {
  if (n_seg == 0) return PM_OK;
  SegP p;
  p.n_seg = n_seg; p.C = C; p.div = 3; p.mean = 0; p.out_bf16 = out_is_bf16;
  p.src = src; p.row_ptr = row_ptr; p.col = col; p.out = out;
  const int cpl = src_is_bf16 ? 8 : 4;
  int need = (C + cpl - 1) / cpl, lpg = 1;
  while (lpg < need && lpg < 64) lpg <<= 1;
  p.lpg = lpg;
  const int gpb = 256 / lpg;
  int64_t nblk = (n_seg + gpb - 1) / gpb;
  if (nblk > 0x7fffffff) nblk = 0x7fffffff;
  { ProfScope ps__(st, "k_segsum_slots");
    if (src_is_bf16) hipLaunchKernelGGL(k_segsum_slots<true>, dim3((unsigned)nblk), dim3(256), 0, st, p);
    else hipLaunchKernelGGL(k_segsum_slots<false>, dim3((unsigned)nblk), dim3(256), 0, st, p); }
  PM_CHECK_LAUNCH("k_segsum_slots");
  return PM_OK;
}

// owner[p] = f for the points of facet f
__global__ void k_owner(int64_t F, const int32_t* __restrict__ off, int32_t* __restrict__ owner) {
  int64_t f = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (f >= F) return;
  for (int32_t q = off[f]; q < off[f + 1]; ++q) owner[q] = (int32_t)f;
}

pm_status pm_launch_owner(int64_t n_facet, const int32_t* tex_off, int32_t* owner, hipStream_t st) {
  if (n_facet == 0) return PM_OK;
  { ProfScope ps__(st, "k_owner");
    hipLaunchKernelGGL(k_owner, dim3((unsigned)((n_facet + 255) / 256)), dim3(256), 0, st, n_facet, tex_off, owner); }
  PM_CHECK_LAUNCH("k_owner");
  return PM_OK;
}
