// Real truncated SH basis of Eq. 3-4: standalone kernels (facet normals, arbitrary directions, gradient)
// and the host-side constant tables.
#include <math.h>

#include "pm_host.h"

void pm_make_sh_table(int L, pm_sh_norm norm, ShTable* T) {
  const double PI = 3.141592653589793238462643383279502884;
  T->L = L;
  for (int i = 0; i < PM_NLM; ++i) T->N[i] = 0.f;
  for (int l = 0; l <= L; ++l)
    for (int m = 0; m <= l; ++m) {
      double r = 1.0;  // (l-m)!/(l+m)!
      for (int i = l - m + 1; i <= l + m; ++i) r /= (double)i;
      double n = sqrt((2.0 * l + 1.0) / (4.0 * PI) * r);
      if (m > 0 && norm == PM_SH_ORTHONORMAL) n *= sqrt(2.0);
      T->N[l * (l + 1) / 2 + m] = (float)n;
    }
}

// Double-precision evaluation of the same Cartesian form, used only for the three constant corner
// directions of Eq. 6 (barycentric unit vectors = angles (pi/2,0), (pi/2,pi/2), (0,0)).
void pm_corner_basis(int L, pm_sh_norm norm, double Bc[3][PM_MAX_K]) {
  const double PI = 3.141592653589793238462643383279502884;
  const double dir[3][3] = {{1, 0, 0}, {0, 1, 0}, {0, 0, 1}};
  for (int j = 0; j < 3; ++j) {
    double x = dir[j][0], y = dir[j][1], z = dir[j][2];
    double cm = 1, sm = 0, qmm = 1;
    for (int m = 0; m <= L; ++m) {
      if (m > 0) {
        double c2 = cm * x - sm * y;
        sm = cm * y + sm * x;
        cm = c2;
        qmm *= (2.0 * m - 1.0);
      }
      double q0 = qmm, q1 = 0;
      for (int l = m; l <= L; ++l) {
        double q;
        if (l == m) q = q0;
        else if (l == m + 1) { q1 = (2.0 * m + 1.0) * z * q0; q = q1; }
        else { q = ((2.0 * l - 1.0) * z * q1 - (l + m - 1.0) * q0) / (double)(l - m); q0 = q1; q1 = q; }
        double r = 1.0;
        for (int i = l - m + 1; i <= l + m; ++i) r /= (double)i;
        double n = sqrt((2.0 * l + 1.0) / (4.0 * PI) * r);
        if (m > 0 && norm == PM_SH_ORTHONORMAL) n *= sqrt(2.0);
        Bc[j][l * (l + 1) + m] = n * q * cm;
        if (m > 0) Bc[j][l * (l + 1) - m] = n * q * sm;
      }
    }
  }
}

template <int LT>
__global__ void __launch_bounds__(256) k_basis_mesh(int64_t F, const float* __restrict__ vert,
                                                    const int32_t* __restrict__ facet, ShTable T,
                                                    float* __restrict__ basis) {
  int64_t f = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (f >= F) return;
  constexpr int K = (LT + 1) * (LT + 1);
  float nx, ny, nz;
  facet_normal(vert, facet[3 * f], facet[3 * f + 1], facet[3 * f + 2], nx, ny, nz);
  float B[K];
  sh_eval<LT>(nx, ny, nz, T, [&](int k, float v) { B[k] = v; });
  float* out = basis + f * K;
  if constexpr (K % 4 == 0) {   // a row is a whole number of 16-byte pieces: vector stores
#pragma unroll
    for (int q = 0; q < K / 4; ++q) ((float4*)out)[q] = make_float4(B[4 * q], B[4 * q + 1], B[4 * q + 2], B[4 * q + 3]);
  } else {
#pragma unroll
    for (int k = 0; k < K; ++k) out[k] = B[k];
  }
}

__global__ void __launch_bounds__(256) k_basis_dirs(int64_t n, const float* __restrict__ dirs, ShTable T,
                                                    float* __restrict__ basis) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int K = (T.L + 1) * (T.L + 1);
  float x = dirs[3 * i], y = dirs[3 * i + 1], z = dirs[3 * i + 2];
  normalize_dir(x, y, z);
  float* out = basis + i * K;
  sh_eval_any(x, y, z, T, [&](int k, float v) { out[k] = v; });
}

// Gradient of sum_k db[k] B_k(d/|d|) with respect to d.  With u = d/|d|, the Cartesian form
// B = N Q_l^m(z) {C_m, S_m}(x,y) is differentiated as a polynomial in (x,y,z):
//   dC_m/dx = m C_{m-1}, dC_m/dy = -m S_{m-1}, dS_m/dx = m S_{m-1}, dS_m/dy = m C_{m-1}, dQ_l^m/dz = Q_l^{m+1},
// and the result is projected on the tangent plane and divided by |d| (Jacobian of d -> d/|d|).
__global__ void __launch_bounds__(256) k_basis_bwd(int64_t n, const float* __restrict__ dirs, ShTable T,
                                                   const float* __restrict__ dbasis, float* __restrict__ ddirs) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int L = T.L;
  const int K = (L + 1) * (L + 1);
  float x = dirs[3 * i], y = dirs[3 * i + 1], z = dirs[3 * i + 2];
  float len = sqrtf(x * x + y * y + z * z);
  float rl = 1.0f / len;
  x *= rl; y *= rl; z *= rl;
  const float* db = dbasis + i * K;
  float gx = 0.f, gy = 0.f, gz = 0.f;
  float cm = 1.f, sm = 0.f, cp = 0.f, sp = 0.f;  // (x+iy)^m and (x+iy)^(m-1)
  float qmm = 1.f;
  for (int m = 0; m <= L; ++m) {
    if (m > 0) {
      cp = cm; sp = sm;
      float c2 = cm * x - sm * y;
      sm = cm * y + sm * x;
      cm = c2;
      qmm *= (float)(2 * m - 1);
    }
    // order-m recurrence (a*) and order-(m+1) recurrence (b*) side by side
    float a0 = qmm, a1 = 0.f;
    float bmm = qmm * (float)(2 * m + 1);  // Q_{m+1}^{m+1}
    float b0 = bmm, b1 = 0.f;
    for (int l = m; l <= L; ++l) {
      float qa, qb;
      if (l == m) qa = a0;
      else if (l == m + 1) { a1 = (float)(2 * m + 1) * z * a0; qa = a1; }
      else { qa = ((float)(2 * l - 1) * z * a1 - (float)(l + m - 1) * a0) / (float)(l - m); a0 = a1; a1 = qa; }
      if (l == m) qb = 0.f;
      else if (l == m + 1) qb = b0;
      else if (l == m + 2) { b1 = (float)(2 * m + 3) * z * b0; qb = b1; }
      else { qb = ((float)(2 * l - 1) * z * b1 - (float)(l + m) * b0) / (float)(l - m - 1); b0 = b1; b1 = qb; }
      float N = T.N[l * (l + 1) / 2 + m];
      float dc = db[l * (l + 1) + m];
      float ds = (m > 0) ? db[l * (l + 1) - m] : 0.f;
      float fm = (float)m;
      // cos part: N qa C_m ; sin part: N qa S_m
      gx += N * qa * fm * (dc * cp + ds * sp);
      gy += N * qa * fm * (-dc * sp + ds * cp);
      gz += N * qb * (dc * cm + ds * sm);
    }
  }
  float dot = gx * x + gy * y + gz * z;
  ddirs[3 * i] = (gx - x * dot) * rl;
  ddirs[3 * i + 1] = (gy - y * dot) * rl;
  ddirs[3 * i + 2] = (gz - z * dot) * rl;
}

static inline unsigned nblocks(int64_t n, int b) { return (unsigned)((n + b - 1) / b); }

pm_status pm_launch_basis_mesh(const pm_mesh* mesh, const ShTable& T, float* basis, hipStream_t st) {
  if (mesh->n_facet == 0) return PM_OK;
  { ProfScope ps__(st, "k_basis_mesh");
    const dim3 grid(nblocks(mesh->n_facet, 256)), block(256);
    switch (T.L) {
      case 0: hipLaunchKernelGGL(k_basis_mesh<0>, grid, block, 0, st, mesh->n_facet, mesh->vert, mesh->facet, T, basis); break;
      case 1: hipLaunchKernelGGL(k_basis_mesh<1>, grid, block, 0, st, mesh->n_facet, mesh->vert, mesh->facet, T, basis); break;
      case 2: hipLaunchKernelGGL(k_basis_mesh<2>, grid, block, 0, st, mesh->n_facet, mesh->vert, mesh->facet, T, basis); break;
      case 3: hipLaunchKernelGGL(k_basis_mesh<3>, grid, block, 0, st, mesh->n_facet, mesh->vert, mesh->facet, T, basis); break;
      case 4: hipLaunchKernelGGL(k_basis_mesh<4>, grid, block, 0, st, mesh->n_facet, mesh->vert, mesh->facet, T, basis); break;
      default: hipLaunchKernelGGL(k_basis_mesh<5>, grid, block, 0, st, mesh->n_facet, mesh->vert, mesh->facet, T, basis); break;
    } }
  PM_CHECK_LAUNCH("k_basis_mesh");
  return PM_OK;
}
pm_status pm_launch_basis_dirs(int64_t n, const float* dirs, const ShTable& T, float* basis, hipStream_t st) {
  if (n == 0) return PM_OK;
  { ProfScope ps__(st, "k_basis_dirs");
    hipLaunchKernelGGL(k_basis_dirs, dim3(nblocks(n, 256)), dim3(256), 0, st, n, dirs, T, basis); }
  PM_CHECK_LAUNCH("k_basis_dirs");
  return PM_OK;
}
pm_status pm_launch_basis_bwd(int64_t n, const float* dirs, const ShTable& T, const float* dbasis, float* ddirs,
                              hipStream_t st) {
  if (n == 0) return PM_OK;
  { ProfScope ps__(st, "k_basis_bwd");
    hipLaunchKernelGGL(k_basis_bwd, dim3(nblocks(n, 256)), dim3(256), 0, st, n, dirs, T, dbasis, ddirs); }
  PM_CHECK_LAUNCH("k_basis_bwd");
  return PM_OK;
}
