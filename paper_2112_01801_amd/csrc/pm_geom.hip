// Input preparation on the device: the facet geometric features (Section "Geometric Features", Eq. 9) and the
// texture resolution of a facet with its barycentric interpolation points (Eq. 8).  Small HBM-bound kernels,
// one thread per facet.
//
// Eq. 9: l1 = |x2-x1|, l2 = |x3-x2|, l3 = |x1-x3| (the pairing its denominators fix), the three normalised inner
// products of the edges meeting at a corner (cosines of the inner angles), the unit normal (x2-x1) x (x3-x1),
// optionally the heights z1 z2 z3.  Row layout [l1 l2 l3, theta1 theta2 theta3, nx ny nz, (z1 z2 z3)].
// A zero product of edge lengths gives theta = 0; the normal of a degenerate facet is (0, 0, 1).
//
// Eq. 8: gamma = floor(alpha (A - Amin)/(Amax - Amin)) + beta, extremes per mesh of the batch.  The floor of a
// floating-point value decides an integer: the arithmetic is fp32, one IEEE operation at a time (no contraction
// into fused multiply-adds) in the order written in facet_area() and k_tex_gamma below, so the result does not
// depend on the compiler; the ratio (A - Amin)/(Amax - Amin) is formed before the multiplication by alpha, which
// makes the two extreme facets of a mesh exact (0 and alpha).  A facet whose exact ratio times alpha lies within
// fp32 rounding of an integer may get either neighbouring value.
#include "pm_host.h"
#include "pm_device.h"

template <bool OUT_BF16>
__global__ void __launch_bounds__(256) k_facet_geometry(int64_t F, const float* __restrict__ vert,
                                                        const int32_t* __restrict__ facet, int with_heights,
                                                        void* __restrict__ out) {
  const int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (f >= F) return;
  const int32_t i1 = facet[3 * f], i2 = facet[3 * f + 1], i3 = facet[3 * f + 2];
  const float* p1 = vert + 3 * (int64_t)i1;
  const float* p2 = vert + 3 * (int64_t)i2;
  const float* p3 = vert + 3 * (int64_t)i3;
  const float x1[3] = {p1[0], p1[1], p1[2]}, x2[3] = {p2[0], p2[1], p2[2]}, x3[3] = {p3[0], p3[1], p3[2]};
  float a[3], b[3], c[3];   // a = x2-x1, b = x3-x2, c = x1-x3
#pragma unroll
  for (int i = 0; i < 3; ++i) { a[i] = x2[i] - x1[i]; b[i] = x3[i] - x2[i]; c[i] = x1[i] - x3[i]; }
  const float l1 = sqrtf(a[0] * a[0] + a[1] * a[1] + a[2] * a[2]);
  const float l2 = sqrtf(b[0] * b[0] + b[1] * b[1] + b[2] * b[2]);
  const float l3 = sqrtf(c[0] * c[0] + c[1] * c[1] + c[2] * c[2]);
  // corner 1: <x2-x1, x3-x1> = -<a, c>;  corner 2: <x1-x2, x3-x2> = -<a, b>;  corner 3: <x1-x3, x2-x3> = -<c, b>
  const float d1 = -(a[0] * c[0] + a[1] * c[1] + a[2] * c[2]);
  const float d2 = -(a[0] * b[0] + a[1] * b[1] + a[2] * b[2]);
  const float d3 = -(c[0] * b[0] + c[1] * b[1] + c[2] * b[2]);
  const float q1 = l1 * l3, q2 = l1 * l2, q3 = l2 * l3;
  float v[12];
  v[0] = l1; v[1] = l2; v[2] = l3;
  v[3] = q1 > 0.f ? d1 / q1 : 0.f;
  v[4] = q2 > 0.f ? d2 / q2 : 0.f;
  v[5] = q3 > 0.f ? d3 / q3 : 0.f;
  facet_normal(vert, i1, i2, i3, v[6], v[7], v[8]);
  v[9] = x1[2]; v[10] = x2[2]; v[11] = x3[2];
  const int n = with_heights ? 12 : 9;
  for (int i = 0; i < n; ++i) {
    if (OUT_BF16) ((uint16_t*)out)[f * n + i] = (uint16_t)f32_to_bf16_bits(v[i]);
    else ((float*)out)[f * n + i] = v[i];
  }
}

pm_status pm_launch_facet_geometry(const pm_mesh* mesh, int with_heights, int out_bf16, void* feat, hipStream_t st) {
  const int64_t F = mesh->n_facet;
  if (F == 0) return PM_OK;
  const dim3 grid((unsigned)((F + 255) / 256));
  { ProfScope ps__(st, "k_facet_geometry");
    if (out_bf16) hipLaunchKernelGGL(k_facet_geometry<true>, grid, dim3(256), 0, st, F, mesh->vert, mesh->facet, with_heights, feat);
    else hipLaunchKernelGGL(k_facet_geometry<false>, grid, dim3(256), 0, st, F, mesh->vert, mesh->facet, with_heights, feat); }
  PM_CHECK_LAUNCH("k_facet_geometry");
  return PM_OK;
}

// ---- Eq. 8 -----------------------------------------------------------------------------------------------
// fp32, one rounding per operation: e1 = x2-x1, e2 = x3-x1, c = e1 x e2, A = 0.5 sqrt((cx cx + cy cy) + cz cz)
__device__ __forceinline__ float facet_area(const float* __restrict__ vert, const int32_t* __restrict__ facet, int64_t f) {
#pragma clang fp contract(off)
  const float* p1 = vert + 3 * (int64_t)facet[3 * f];
  const float* p2 = vert + 3 * (int64_t)facet[3 * f + 1];
  const float* p3 = vert + 3 * (int64_t)facet[3 * f + 2];
  const float ux = p2[0] - p1[0], uy = p2[1] - p1[1], uz = p2[2] - p1[2];
  const float wx = p3[0] - p1[0], wy = p3[1] - p1[1], wz = p3[2] - p1[2];
  const float m1 = uy * wz, m2 = uz * wy, m3 = uz * wx, m4 = ux * wz, m5 = ux * wy, m6 = uy * wx;
  const float cx = m1 - m2, cy = m3 - m4, cz = m5 - m6;
  const float sx = cx * cx, sy = cy * cy, sz = cz * cz;
  const float s = (sx + sy) + sz;
  return 0.5f * __fsqrt_rn(s);
}

// mesh of facet f: the last m with facet_off[m] <= f
__device__ __forceinline__ int mesh_of_facet(const int32_t* __restrict__ facet_off, int n_mesh, int64_t f) {
  if (n_mesh <= 1 || !facet_off) return 0;
  int lo = 0, hi = n_mesh - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if ((int64_t)facet_off[mid] <= f) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// areas (non-negative, so their bit patterns order like the values) and the per-mesh extremes through integer
// atomics on the bit patterns: exact and order-independent.  A block walks a contiguous chunk of facets in
// tiles of 256; tiles inside one mesh accumulate in registers and reach memory once per block and mesh (waves
// reduce by shuffles, then LDS, then one pair of global atomics); a tile that straddles meshes goes direct.
__global__ void __launch_bounds__(256) k_tex_area(int64_t F, int64_t chunk, int n_mesh, const float* __restrict__ vert,
                                                  const int32_t* __restrict__ facet, const int32_t* __restrict__ facet_off,
                                                  float* __restrict__ area, uint32_t* __restrict__ minmax) {
  __shared__ uint32_t smin, smax;
  const int64_t f_begin = (int64_t)blockIdx.x * chunk, f_end = min(F, f_begin + chunk);
  uint32_t lo = 0x7f800000u, hi = 0u;
  int m_cur = -1;
  auto flush = [&]() {                      // the same for the whole block
    if (m_cur >= 0) {
      if (threadIdx.x == 0) { smin = 0x7f800000u; smax = 0u; }
      __syncthreads();
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        lo = min(lo, (uint32_t)__shfl_xor((int)lo, o, 64));
        hi = max(hi, (uint32_t)__shfl_xor((int)hi, o, 64));
      }
      if ((threadIdx.x & 63) == 0) { atomicMin(&smin, lo); atomicMax(&smax, hi); }
      __syncthreads();
      if (threadIdx.x == 0) { atomicMin(&minmax[2 * m_cur], smin); atomicMax(&minmax[2 * m_cur + 1], smax); }
      __syncthreads();
    }
    lo = 0x7f800000u; hi = 0u;
  };
  for (int64_t t0 = f_begin; t0 < f_end; t0 += 256) {
    const int64_t f = t0 + threadIdx.x;
    const int m0 = mesh_of_facet(facet_off, n_mesh, t0), m1 = mesh_of_facet(facet_off, n_mesh, min(t0 + 255, f_end - 1));
    if (m0 == m1 && m0 != m_cur) { flush(); m_cur = m0; }
    if (f < f_end) {
      const float a = facet_area(vert, facet, f);
      area[f] = a;
      const uint32_t u = __float_as_uint(a);
      if (m0 == m1) { lo = min(lo, u); hi = max(hi, u); }
      else {
        const int m = mesh_of_facet(facet_off, n_mesh, f);
        atomicMin(&minmax[2 * m], u);
        atomicMax(&minmax[2 * m + 1], u);
      }
    }
  }
  flush();
}

__global__ void __launch_bounds__(256) k_tex_gamma(int64_t F, int n_mesh, const int32_t* __restrict__ facet_off,
                                                   const float* __restrict__ area, const uint32_t* __restrict__ minmax,
                                                   int alpha, int beta, int32_t* __restrict__ gamma,
                                                   int32_t* __restrict__ cnt) {
#pragma clang fp contract(off)
  const int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (f >= F) return;
  const int m = mesh_of_facet(facet_off, n_mesh, f);
  const float lo = __uint_as_float(minmax[2 * m]), hi = __uint_as_float(minmax[2 * m + 1]);
  int32_t g = beta;
  if (hi > lo) {
    // the ratio first: it is exactly 1 for the largest facet, so that facet gets alpha + beta whatever the rounding
    const float ratio = __fdiv_rn(area[f] - lo, hi - lo);
    g = (int32_t)floorf((float)alpha * ratio) + beta;
  }
  gamma[f] = g;
  cnt[f] = (g + 1) * (g + 2) / 2;
}

// interpolation points of facet f: (i, j, gamma-i-j)/gamma, i descending then j descending; centroid for gamma = 0
__global__ void __launch_bounds__(256) k_tex_bary(int64_t F, const int32_t* __restrict__ gamma,
                                                  const int32_t* __restrict__ tex_off, int64_t n_tex,
                                                  float* __restrict__ bary) {
  const int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (f >= F) return;
  const int32_t g = gamma[f];
  int64_t p = tex_off[f];
  if (g <= 0) {
    if (p >= 0 && p < n_tex) { bary[3 * p] = 1.0f / 3.0f; bary[3 * p + 1] = 1.0f / 3.0f; bary[3 * p + 2] = 1.0f / 3.0f; }
    return;
  }
  const float gf = (float)g;
  for (int i = g; i >= 0; --i)
    for (int j = g - i; j >= 0; --j, ++p) {
      if (p < 0 || p >= n_tex) continue;
      bary[3 * p] = __fdiv_rn((float)i, gf);
      bary[3 * p + 1] = __fdiv_rn((float)j, gf);
      bary[3 * p + 2] = __fdiv_rn((float)(g - i - j), gf);
    }
}

// workspace: area [F] fp32, counts [F] int32, extremes [n_mesh][2], scan tiles
size_t pm_texture_ws_bytes_host(int64_t n_facet, int n_mesh) {
  return 2 * pm_round_up((size_t)(n_facet + 1) * 4, 256) + pm_round_up((size_t)(n_mesh > 0 ? n_mesh : 1) * 8, 256) +
         pm_scan_ws_bytes(n_facet);
}

__global__ void k_tex_init_minmax(int n_mesh, uint32_t* __restrict__ minmax) {
  const int m = blockIdx.x * blockDim.x + threadIdx.x;
  if (m < n_mesh) { minmax[2 * m] = 0x7f800000u; minmax[2 * m + 1] = 0u; }
}

pm_status pm_launch_texture_layout(const pm_mesh* mesh, int alpha, int beta, int32_t* gamma, int32_t* tex_off, void* ws,
                                   hipStream_t st) {
  const int64_t F = mesh->n_facet;
  const int n_mesh = mesh->n_mesh > 0 ? mesh->n_mesh : 1;
  char* p = (char*)ws;
  float* area = (float*)p;        p += pm_round_up((size_t)(F + 1) * 4, 256);
  int32_t* cnt = (int32_t*)p;     p += pm_round_up((size_t)(F + 1) * 4, 256);
  uint32_t* minmax = (uint32_t*)p; p += pm_round_up((size_t)n_mesh * 8, 256);
  void* tiles = p;
  if (F > 0) {
    const dim3 grid((unsigned)((F + 255) / 256));
    { ProfScope ps__(st, "k_tex_init_minmax");
      hipLaunchKernelGGL(k_tex_init_minmax, dim3((unsigned)((n_mesh + 255) / 256)), dim3(256), 0, st, n_mesh, minmax); }
    int64_t nblk = (F + 255) / 256;
    if (nblk > 1024) nblk = 1024;
    const int64_t chunk = ((F + nblk - 1) / nblk + 255) / 256 * 256;
    { ProfScope ps__(st, "k_tex_area");
      hipLaunchKernelGGL(k_tex_area, dim3((unsigned)((F + chunk - 1) / chunk)), dim3(256), 0, st, F, chunk, n_mesh, mesh->vert,
                         mesh->facet, mesh->facet_off, area, minmax); }
    { ProfScope ps__(st, "k_tex_gamma");
      hipLaunchKernelGGL(k_tex_gamma, grid, dim3(256), 0, st, F, n_mesh, mesh->facet_off, area, minmax, alpha, beta, gamma, cnt); }
    PM_CHECK_LAUNCH("texture layout");
  }
  return pm_launch_exclusive_scan(cnt, F, tex_off, tiles, st);
}

pm_status pm_launch_texture_bary(int64_t n_facet, const int32_t* gamma, const int32_t* tex_off, int64_t n_tex, float* bary,
                                 hipStream_t st) {
  if (n_facet == 0 || n_tex == 0) return PM_OK;
  { ProfScope ps__(st, "k_tex_bary");
    hipLaunchKernelGGL(k_tex_bary, dim3((unsigned)((n_facet + 255) / 256)), dim3(256), 0, st, n_facet, gamma, tex_off, n_tex, bary); }
  PM_CHECK_LAUNCH("k_tex_bary");
  return PM_OK;
}
