// facet2facet (Eq. 7) for few input channels -- the paper's own shape: the texture points carry 3 colour channels.
//
// Eq. 7's sums commute:  g_f = (1/R_f sum_p B_p (x) h_p) . W  -- the mean of the Khatri-Rao rows over the points of a
// facet first, one contraction per FACET afterwards.  With K cin <= 64 that mean is one 64-channel row per facet,
// so the matrix work drops from 2 K 64 cout per POINT (three channels padded to a 64-channel chunk) to 2 . 64 . cout
// per facet, and the per-point work is K cin multiply-adds on the vector ALU:
//   forward   S_f[k cin + ci] = 1/R_f sum_p B_k(d_p) h_p[ci]          (k_f2f_gather, one thread per facet; bf16: stored as
//             a bf16 head and a bf16 remainder, 128 channels, contracted against the coefficients laid out twice)
//             g_f = S_f . W viewed as [K cin][cout]                   (conv_rows without a basis)
//   backward  dW viewed as [K cin][cout] = sum_f S_f (x) dg_f         (weight gradient without a basis, rows = facets)
//             T_f = W dg_f  ([K cin], fp32),  dh_p[ci] = 1/R_f sum_k B_k(d_p) T_f[k cin + ci]   (k_f2f_scatter, per point)
#include "pm_host.h"
#include "pm_device.h"

#define FS_ROW 64   /* channels of a staged row S_f (K cin values, then zeros) */

// S[f][0 .. K cin) = mean over the points of facet f of B_k(d_p) h_p[ci];  S[f][K cin .. 64) = 0.   A facet
// without points gets a zero row.  fp32 rows have 64 channels, bf16 rows 128 (head | remainder).
template <bool BF16, int LT, int CIN>
__global__ void __launch_bounds__(256) k_f2f_gather(int64_t F, const int32_t* __restrict__ tex_off,
                                                    const float* __restrict__ bary, ShTable sh,
                                                    const void* __restrict__ h, void* __restrict__ S) {
  constexpr int K = (LT + 1) * (LT + 1);
  static_assert(K * CIN <= FS_ROW, "one staged row per facet");
  const int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (f >= F) return;
  const int32_t p0 = tex_off[f], p1 = tex_off[f + 1];
  float acc[FS_ROW];
#pragma unroll
  for (int i = 0; i < FS_ROW; ++i) acc[i] = 0.f;
  // the next point's coordinates and channels are on their way while this point's basis is evaluated
  auto fetch = [&](int32_t p, float (&d)[3], float (&hv)[CIN]) {
    d[0] = bary[3 * (int64_t)p]; d[1] = bary[3 * (int64_t)p + 1]; d[2] = bary[3 * (int64_t)p + 2];
#pragma unroll
    for (int ci = 0; ci < CIN; ++ci)
      hv[ci] = BF16 ? bf16_to_f32(((const uint16_t*)h)[(int64_t)p * CIN + ci]) : ((const float*)h)[(int64_t)p * CIN + ci];
  };
  float d[3] = {0.f, 0.f, 1.f}, hv[CIN];
#pragma unroll
  for (int ci = 0; ci < CIN; ++ci) hv[ci] = 0.f;
  if (p1 > p0) fetch(p0, d, hv);
  for (int32_t p = p0; p < p1; ++p) {
    float dn[3], hn[CIN];
    fetch(min(p + 1, p1 - 1), dn, hn);
    float x = d[0], y = d[1], z = d[2];
    normalize_dir(x, y, z);
    sh_eval<LT>(x, y, z, sh, [&](int k, float v) {
#pragma unroll
      for (int ci = 0; ci < CIN; ++ci) acc[k * CIN + ci] = fmaf(v, hv[ci], acc[k * CIN + ci]);
    });
#pragma unroll
    for (int q = 0; q < 3; ++q) d[q] = dn[q];
#pragma unroll
    for (int ci = 0; ci < CIN; ++ci) hv[ci] = hn[ci];
  }
  const float w = p1 > p0 ? 1.0f / (float)(p1 - p0) : 0.f;
  if constexpr (BF16) {
    // a bf16 head in channels 0..63 and the bf16 remainder in channels 64..127: the matrix core sums both against
    // the same coefficients, so the staged mean enters the contraction with 16 significant bits, not 8
    uint4* dst = (uint4*)((uint16_t*)S + f * (2 * FS_ROW));
#pragma unroll
    for (int q = 0; q < FS_ROW / 8; ++q) {
      float hi[8], lo[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float v = acc[8 * q + i] * w;
        hi[i] = bf16_to_f32((uint16_t)f32_to_bf16_bits(v));
        lo[i] = v - hi[i];
      }
      uint4 o, r;
      o.x = pack_bf16x2(hi[0], hi[1]); o.y = pack_bf16x2(hi[2], hi[3]); o.z = pack_bf16x2(hi[4], hi[5]); o.w = pack_bf16x2(hi[6], hi[7]);
      r.x = pack_bf16x2(lo[0], lo[1]); r.y = pack_bf16x2(lo[2], lo[3]); r.z = pack_bf16x2(lo[4], lo[5]); r.w = pack_bf16x2(lo[6], lo[7]);
      dst[q] = o;
      dst[FS_ROW / 8 + q] = r;
    }
  } else {
    float4* dst = (float4*)((float*)S + f * FS_ROW);
#pragma unroll
    for (int q = 0; q < FS_ROW / 4; ++q)
      dst[q] = make_float4(acc[4 * q] * w, acc[4 * q + 1] * w, acc[4 * q + 2] * w, acc[4 * q + 3] * w);
  }
}

// dh[p][ci] = 1/R_f sum_k B_k(d_p) T[f][k cin + ci],  f = owner[p]
template <bool BF16, int LT, int CIN>
__global__ void __launch_bounds__(256) k_f2f_scatter(int64_t P, const int32_t* __restrict__ owner,
                                                     const int32_t* __restrict__ tex_off, const float* __restrict__ bary,
                                                     ShTable sh, const float* __restrict__ T, void* __restrict__ dh) {
  constexpr int K = (LT + 1) * (LT + 1);
  const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (p >= P) return;
  const int64_t f = owner[p];
  const float w = 1.0f / (float)(tex_off[f + 1] - tex_off[f]);      // >= 1 point: p itself
  float x = bary[3 * p], y = bary[3 * p + 1], z = bary[3 * p + 2];
  normalize_dir(x, y, z);
  const float* t = T + f * (int64_t)(K * CIN);
  float acc[CIN];
#pragma unroll
  for (int ci = 0; ci < CIN; ++ci) acc[ci] = 0.f;
  sh_eval<LT>(x, y, z, sh, [&](int k, float v) {
#pragma unroll
    for (int ci = 0; ci < CIN; ++ci) acc[ci] = fmaf(v, t[k * CIN + ci], acc[ci]);
  });
#pragma unroll
  for (int ci = 0; ci < CIN; ++ci) {
    if (BF16) ((uint16_t*)dh)[p * CIN + ci] = (uint16_t)f32_to_bf16_bits(acc[ci] * w);
    else ((float*)dh)[p * CIN + ci] = acc[ci] * w;
  }
}

bool pm_f2f_small_applies(int L, int cin) { return L >= 0 && L <= 3 && cin >= 1 && cin <= 4; }   // K cin <= 64

template <bool BF16, int LT, int CIN>
static void f2f_small_launch(bool gather, int64_t n, const int32_t* owner, const int32_t* tex_off, const float* bary,
                             const ShTable& sh, const void* in, void* out, hipStream_t st) {
  const dim3 grid((unsigned)((n + 255) / 256));
  if (gather) hipLaunchKernelGGL((k_f2f_gather<BF16, LT, CIN>), grid, dim3(256), 0, st, n, tex_off, bary, sh, in, out);
  else hipLaunchKernelGGL((k_f2f_scatter<BF16, LT, CIN>), grid, dim3(256), 0, st, n, owner, tex_off, bary, sh, (const float*)in, out);
}

template <bool BF16, int LT>
static void f2f_small_cin(int cin, bool gather, int64_t n, const int32_t* owner, const int32_t* tex_off, const float* bary,
                          const ShTable& sh, const void* in, void* out, hipStream_t st) {
  switch (cin) {
    case 1: f2f_small_launch<BF16, LT, 1>(gather, n, owner, tex_off, bary, sh, in, out, st); break;
    case 2: f2f_small_launch<BF16, LT, 2>(gather, n, owner, tex_off, bary, sh, in, out, st); break;
    case 3: f2f_small_launch<BF16, LT, 3>(gather, n, owner, tex_off, bary, sh, in, out, st); break;
    default: f2f_small_launch<BF16, LT, 4>(gather, n, owner, tex_off, bary, sh, in, out, st); break;
  }
}

template <bool BF16>
static void f2f_small_L(int L, int cin, bool gather, int64_t n, const int32_t* owner, const int32_t* tex_off,
                        const float* bary, const ShTable& sh, const void* in, void* out, hipStream_t st) {
  switch (L) {
    case 0: f2f_small_cin<BF16, 0>(cin, gather, n, owner, tex_off, bary, sh, in, out, st); break;
    case 1: f2f_small_cin<BF16, 1>(cin, gather, n, owner, tex_off, bary, sh, in, out, st); break;
    case 2: f2f_small_cin<BF16, 2>(cin, gather, n, owner, tex_off, bary, sh, in, out, st); break;
    default: f2f_small_cin<BF16, 3>(cin, gather, n, owner, tex_off, bary, sh, in, out, st); break;
  }
}

pm_status pm_launch_f2f_gather(int64_t n_facet, const int32_t* tex_off, const float* bary, const ShTable& sh, int cin,
                               int is_bf16, const void* h, void* S, hipStream_t st) {
  if (n_facet == 0) return PM_OK;
  if (!pm_f2f_small_applies(sh.L, cin)) return pm_fail(PM_ERR_UNSUPPORTED, "facet2facet row staging: L=%d cin=%d", sh.L, cin);
  { ProfScope ps__(st, "k_f2f_gather");
    if (is_bf16) f2f_small_L<true>(sh.L, cin, true, n_facet, nullptr, tex_off, bary, sh, h, S, st);
    else f2f_small_L<false>(sh.L, cin, true, n_facet, nullptr, tex_off, bary, sh, h, S, st); }
  PM_CHECK_LAUNCH("k_f2f_gather");
  return PM_OK;
}

pm_status pm_launch_f2f_scatter(int64_t n_tex, const int32_t* owner, const int32_t* tex_off, const float* bary,
                                const ShTable& sh, int cin, int is_bf16, const float* T, void* dh, hipStream_t st) {
  if (n_tex == 0) return PM_OK;
  if (!pm_f2f_small_applies(sh.L, cin)) return pm_fail(PM_ERR_UNSUPPORTED, "facet2facet row staging: L=%d cin=%d", sh.L, cin);
  { ProfScope ps__(st, "k_f2f_scatter");
    if (is_bf16) f2f_small_L<true>(sh.L, cin, false, n_tex, owner, tex_off, bary, sh, T, dh, st);
    else f2f_small_L<false>(sh.L, cin, false, n_tex, owner, tex_off, bary, sh, T, dh, st); }
  PM_CHECK_LAUNCH("k_f2f_scatter");
  return PM_OK;
}
