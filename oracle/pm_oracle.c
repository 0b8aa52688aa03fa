/*
 * CPU oracle for the spherical-harmonic mesh convolutions (facet2vertex, vertex2facet,
 * facet2facet) of "Mesh Convolution with Continuous Filters for 3D Surface Parsing".
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64 evaluation of the
 * definitions in the paper, written to be checked against the paper by eye.  It shares no code
 * with the HIP library, and only tests, the smoke check and the benchmark's CPU-baseline leg
 * may call it.
 *
 * Conventions (the paper leaves these open; the GPU library documents the same choices):
 *   - basis index  k = l*(l+1) + m,  m in [-l, l];  m > 0 is the cos(m phi) function (coefficient
 *     a_lm of Eq. 4),  m < 0 the sin(|m| phi) function (coefficient b_l|m|),  m = 0 is a_l0.
 *   - norm = 0: the functions exactly as printed in Eq. 4 (no sqrt(2) on m != 0);
 *     norm = 1: m != 0 functions multiplied by sqrt(2) (orthonormal on the sphere).
 *   - dense filter coefficients W[k][ci][co] (Eq. 1 inner product with Eq. 4 coefficient vectors).
 *   - facet normal = (x2-x1) x (x3-x1), normalised; if its squared length < 1e-30 use (0,0,1).
 *   - a vertex without adjacent facets gets a zero output row.
 *
 * The depth-wise separable forms (orc_*_sep*) are pinned against the dense functions on the expanded
 * coefficients alpha[k][ci]*P[ci][co], by finite differences and by adjoint identities.
 *
 * Parity status: every function below is pinned by tests (quadrature Gram matrix, closed forms,
 * a library SH routine, tetrahedron / icosahedron closed forms, brute-force adjacency scans,
 * finite differences, adjoint identities) EXCEPT agreement with the authors' released code,
 * which is "parity unpinned" (that code is not available here; index order and the sqrt(2)
 * convention may differ from it by a fixed relabelling / rescaling of coefficients).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_MAX_L 8
#define ORC_MAX_K ((ORC_MAX_L + 1) * (ORC_MAX_L + 1))

static double factorial(int n) {
  double r = 1.0;
  for (int i = 2; i <= n; ++i) r *= (double)i;
  return r;
}

/* Eq. 3-4: K = (L+1)^2 real basis values at a direction d (any non-zero length). */
static void sh_basis_one(const double d[3], int L, int norm, double* B) {
  const double PI = 3.14159265358979323846;
  double len = sqrt(d[0] * d[0] + d[1] * d[1] + d[2] * d[2]);
  double x = d[0] / len, y = d[1] / len, z = d[2] / len;
  if (z > 1.0) z = 1.0;
  if (z < -1.0) z = -1.0;
  double theta = acos(z);          /* polar angle in [0, pi]   */
  double phi = atan2(y, x);        /* azimuth; atan2(0,0) = 0  */
  double t = cos(theta), s = sin(theta);
  /* associated Legendre functions WITHOUT the Condon-Shortley phase */
  double P[ORC_MAX_L + 1][ORC_MAX_L + 1];
  for (int m = 0; m <= L; ++m) {
    double pmm = 1.0;                                   /* (2m-1)!! * s^m */
    for (int i = 1; i <= m; ++i) pmm *= (double)(2 * i - 1) * s;
    P[m][m] = pmm;
    if (m + 1 <= L) P[m + 1][m] = (double)(2 * m + 1) * t * pmm;
    for (int l = m + 2; l <= L; ++l)
      P[l][m] = ((double)(2 * l - 1) * t * P[l - 1][m] - (double)(l + m - 1) * P[l - 2][m]) / (double)(l - m);
  }
  for (int l = 0; l <= L; ++l) {
    for (int m = 0; m <= l; ++m) {
      double N = sqrt((double)(2 * l + 1) / (4.0 * PI) * factorial(l - m) / factorial(l + m));
      double Ylm0 = N * P[l][m];                         /* Y_l^m(theta, 0) */
      if (m == 0) {
        B[l * (l + 1)] = Ylm0;
      } else {
        double sc = norm ? sqrt(2.0) : 1.0;
        B[l * (l + 1) + m] = sc * Ylm0 * cos((double)m * phi);
        B[l * (l + 1) - m] = sc * Ylm0 * sin((double)m * phi);
      }
    }
  }
}

void orc_sh_basis(int64_t n, const double* dirs, int L, int norm, double* B) {
  int K = (L + 1) * (L + 1);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) sh_basis_one(dirs + 3 * i, L, norm, B + i * K);
}

static void facet_normal_one(const float* vert, const int32_t* fc, double n[3]) {
  double a[3], b[3], c[3];
  for (int q = 0; q < 3; ++q) {
    a[q] = (double)vert[3 * (int64_t)fc[0] + q];
    b[q] = (double)vert[3 * (int64_t)fc[1] + q];
    c[q] = (double)vert[3 * (int64_t)fc[2] + q];
  }
  double u[3] = {b[0] - a[0], b[1] - a[1], b[2] - a[2]};
  double w[3] = {c[0] - a[0], c[1] - a[1], c[2] - a[2]};
  double cx = u[1] * w[2] - u[2] * w[1];
  double cy = u[2] * w[0] - u[0] * w[2];
  double cz = u[0] * w[1] - u[1] * w[0];
  double l2 = cx * cx + cy * cy + cz * cz;
  if (l2 < 1e-30) { n[0] = 0.0; n[1] = 0.0; n[2] = 1.0; return; }
  double l = sqrt(l2);
  n[0] = cx / l; n[1] = cy / l; n[2] = cz / l;
}

void orc_facet_normals(int64_t F, const float* vert, const int32_t* facet, double* nrm) {
#pragma omp parallel for schedule(static)
  for (int64_t f = 0; f < F; ++f) facet_normal_one(vert, facet + 3 * f, nrm + 3 * f);
}

/* N(v): the corner slots 3*f+j that reference vertex v, ascending. */
void orc_vf_adjacency(int64_t V, int64_t F, const int32_t* facet, int32_t* row_ptr, int32_t* col) {
  int64_t* cnt = (int64_t*)calloc((size_t)V + 1, sizeof(int64_t));
  for (int64_t e = 0; e < 3 * F; ++e) cnt[facet[e] + 1]++;
  for (int64_t v = 0; v < V; ++v) cnt[v + 1] += cnt[v];
  for (int64_t v = 0; v <= V; ++v) row_ptr[v] = (int32_t)cnt[v];
  for (int64_t e = 0; e < 3 * F; ++e) col[cnt[facet[e]]++] = (int32_t)e;   /* e ascending => rows ascending */
  free(cnt);
}

/* summand of Eq. 5 for one facet: y[co] = sum_k sum_ci B_k(n_f) h_f[ci] W[k][ci][co] */
static void filter_apply(const double* B, int K, int cin, int cout, const double* h, const double* W, double* y) {
  for (int co = 0; co < cout; ++co) y[co] = 0.0;
  for (int k = 0; k < K; ++k)
    for (int ci = 0; ci < cin; ++ci) {
      double bh = B[k] * h[ci];
      const double* w = W + ((int64_t)k * cin + ci) * cout;
      for (int co = 0; co < cout; ++co) y[co] += bh * w[co];
    }
}

/*
 * facet2vertex, Eq. 5:  g_v = 1/|N(v)| sum_{f in N(v)} F(theta_f, phi_f) h_f,  angles from the facet normal.
 * Computes the rows listed in `rows` (n_rows of them; rows == NULL means all V rows in order).
 * out is [n_rows, cout].
 */
void orc_f2v(int64_t V, int64_t F, const float* vert, const int32_t* facet, int L, int norm, int cin, int cout,
             const double* h, const double* W, int64_t n_rows, const int64_t* rows, double* out) {
  int K = (L + 1) * (L + 1);
  int32_t* rp = (int32_t*)malloc(((size_t)V + 1) * sizeof(int32_t));
  int32_t* col = (int32_t*)malloc((size_t)(3 * F + 1) * sizeof(int32_t));
  orc_vf_adjacency(V, F, facet, rp, col);
#pragma omp parallel
  {
    double* y = (double*)malloc((size_t)cout * sizeof(double));
#pragma omp for schedule(dynamic, 64)
    for (int64_t r = 0; r < n_rows; ++r) {
      int64_t v = rows ? rows[r] : r;
      double* g = out + r * cout;
      for (int co = 0; co < cout; ++co) g[co] = 0.0;
      int deg = rp[v + 1] - rp[v];
      for (int e = rp[v]; e < rp[v + 1]; ++e) {
        int64_t f = col[e] / 3;
        double n[3], B[ORC_MAX_K];
        facet_normal_one(vert, facet + 3 * f, n);
        sh_basis_one(n, L, norm, B);
        filter_apply(B, K, cin, cout, h + f * cin, W, y);
        for (int co = 0; co < cout; ++co) g[co] += y[co];
      }
      if (deg > 0)
        for (int co = 0; co < cout; ++co) g[co] /= (double)deg;
    }
    free(y);
  }
  free(rp); free(col);
}

/*
 * facet2vertex backward (transposed sums of Eq. 5):
 *   dy_f = sum_{j} dg[v_j(f)] / |N(v_j(f))|
 *   dh_f[ci]      = sum_k sum_co B_k(n_f) W[k][ci][co] dy_f[co]        (rows listed in `rows`, or all)
 *   dW[k][ci][co] = sum_f B_k(n_f) h_f[ci] dy_f[co]                    (always over ALL facets; skipped if NULL)
 */
void orc_f2v_bwd(int64_t V, int64_t F, const float* vert, const int32_t* facet, int L, int norm, int cin, int cout,
                 const double* h, const double* W, const double* dg, int64_t n_rows, const int64_t* rows,
                 double* dh, double* dW) {
  int K = (L + 1) * (L + 1);
  int64_t* deg = (int64_t*)calloc((size_t)V, sizeof(int64_t));
  for (int64_t e = 0; e < 3 * F; ++e) deg[facet[e]]++;
  if (dh) {
#pragma omp parallel
    {
      double* dy = (double*)malloc((size_t)cout * sizeof(double));
#pragma omp for schedule(static)
      for (int64_t r = 0; r < n_rows; ++r) {
        int64_t f = rows ? rows[r] : r;
        double n[3], B[ORC_MAX_K];
        facet_normal_one(vert, facet + 3 * f, n);
        sh_basis_one(n, L, norm, B);
        for (int co = 0; co < cout; ++co) dy[co] = 0.0;
        for (int j = 0; j < 3; ++j) {
          int64_t v = facet[3 * f + j];
          for (int co = 0; co < cout; ++co) dy[co] += dg[v * cout + co] / (double)deg[v];
        }
        for (int ci = 0; ci < cin; ++ci) {
          double acc = 0.0;
          for (int k = 0; k < K; ++k) {
            const double* w = W + ((int64_t)k * cin + ci) * cout;
            double t = 0.0;
            for (int co = 0; co < cout; ++co) t += w[co] * dy[co];
            acc += B[k] * t;
          }
          dh[r * cin + ci] = acc;
        }
      }
      free(dy);
    }
  }
  if (dW) {
    int64_t nW = (int64_t)K * cin * cout;
    for (int64_t i = 0; i < nW; ++i) dW[i] = 0.0;
    /* parallel over (k, ci) output rows; every thread walks all facets in ascending order */
    double* Ball = (double*)malloc((size_t)F * K * sizeof(double));
    double* dyall = (double*)malloc((size_t)F * cout * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int64_t f = 0; f < F; ++f) {
      double n[3];
      facet_normal_one(vert, facet + 3 * f, n);
      sh_basis_one(n, L, norm, Ball + f * K);
      double* dy = dyall + f * cout;
      for (int co = 0; co < cout; ++co) dy[co] = 0.0;
      for (int j = 0; j < 3; ++j) {
        int64_t v = facet[3 * f + j];
        for (int co = 0; co < cout; ++co) dy[co] += dg[v * cout + co] / (double)deg[v];
      }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t kc = 0; kc < (int64_t)K * cin; ++kc) {
      int k = (int)(kc / cin), ci = (int)(kc % cin);
      double* d = dW + kc * cout;
      for (int64_t f = 0; f < F; ++f) {
        double bh = Ball[f * K + k] * h[f * cin + ci];
        const double* dy = dyall + f * cout;
        for (int co = 0; co < cout; ++co) d[co] += bh * dy[co];
      }
    }
    free(Ball); free(dyall);
  }
  free(deg);
}

/* the three corner directions of Eq. 6: (pi/2,0), (pi/2,pi/2), (0,0)  <=>  barycentric unit vectors */
static void corner_basis(int L, int norm, double Bc[3][ORC_MAX_K]) {
  const double e[3][3] = {{1, 0, 0}, {0, 1, 0}, {0, 0, 1}};
  for (int j = 0; j < 3; ++j) sh_basis_one(e[j], L, norm, Bc[j]);
}

/* vertex2facet, Eq. 6:  g_f = F(pi/2,0) h_{v1} + F(pi/2,pi/2) h_{v2} + F(0,0) h_{v3}  (rows listed, or all F) */
void orc_v2f(int64_t V, int64_t F, const int32_t* facet, int L, int norm, int cin, int cout,
             const double* h, const double* W, int64_t n_rows, const int64_t* rows, double* out) {
  (void)V; (void)F;
  int K = (L + 1) * (L + 1);
  double Bc[3][ORC_MAX_K];
  corner_basis(L, norm, Bc);
#pragma omp parallel
  {
    double* y = (double*)malloc((size_t)cout * sizeof(double));
#pragma omp for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
      int64_t f = rows ? rows[r] : r;
      double* g = out + r * cout;
      for (int co = 0; co < cout; ++co) g[co] = 0.0;
      for (int j = 0; j < 3; ++j) {
        int64_t v = facet[3 * f + j];
        filter_apply(Bc[j], K, cin, cout, h + v * cin, W, y);
        for (int co = 0; co < cout; ++co) g[co] += y[co];
      }
    }
    free(y);
  }
}

/*
 * vertex2facet backward:
 *   dh_v[ci]      = sum_{(f,j): v_j(f)=v} sum_k sum_co B_k(e_j) W[k][ci][co] dg_f[co]   (rows listed, or all V)
 *   dW[k][ci][co] = sum_f sum_j B_k(e_j) h_{v_j(f)}[ci] dg_f[co]
 */
void orc_v2f_bwd(int64_t V, int64_t F, const int32_t* facet, int L, int norm, int cin, int cout,
                 const double* h, const double* W, const double* dg, int64_t n_rows, const int64_t* rows,
                 double* dh, double* dW) {
  int K = (L + 1) * (L + 1);
  double Bc[3][ORC_MAX_K];
  corner_basis(L, norm, Bc);
  if (dh) {
    int32_t* rp = (int32_t*)malloc(((size_t)V + 1) * sizeof(int32_t));
    int32_t* col = (int32_t*)malloc((size_t)(3 * F + 1) * sizeof(int32_t));
    orc_vf_adjacency(V, F, facet, rp, col);
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t r = 0; r < n_rows; ++r) {
      int64_t v = rows ? rows[r] : r;
      for (int ci = 0; ci < cin; ++ci) {
        double acc = 0.0;
        for (int e = rp[v]; e < rp[v + 1]; ++e) {
          int64_t f = col[e] / 3;
          int j = col[e] % 3;
          for (int k = 0; k < K; ++k) {
            const double* w = W + ((int64_t)k * cin + ci) * cout;
            double t = 0.0;
            for (int co = 0; co < cout; ++co) t += w[co] * dg[f * cout + co];
            acc += Bc[j][k] * t;
          }
        }
        dh[r * cin + ci] = acc;
      }
    }
    free(rp); free(col);
  }
  if (dW) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t kc = 0; kc < (int64_t)K * cin; ++kc) {
      int k = (int)(kc / cin), ci = (int)(kc % cin);
      double* d = dW + kc * cout;
      for (int co = 0; co < cout; ++co) d[co] = 0.0;
      for (int64_t f = 0; f < F; ++f)
        for (int j = 0; j < 3; ++j) {
          int64_t v = facet[3 * f + j];
          double bh = Bc[j][k] * h[v * cin + ci];
          for (int co = 0; co < cout; ++co) d[co] += bh * dg[f * cout + co];
        }
    }
  }
}

/*
 * facet2facet, Eq. 7:  g_f = 1/R_f sum_{p in f} <F(theta_p, phi_p), h_p>,  direction of point p = xi_p / |xi_p|
 * (barycentric coordinates projected radially onto the unit sphere).  tex_off is the facet -> point CSR.
 * A facet without points gets a zero row.
 */
void orc_f2f(int64_t F, const int32_t* tex_off, const float* bary, int L, int norm, int cin, int cout,
             const double* h, const double* W, int64_t n_rows, const int64_t* rows, double* out) {
  (void)F;
  int K = (L + 1) * (L + 1);
#pragma omp parallel
  {
    double* y = (double*)malloc((size_t)cout * sizeof(double));
#pragma omp for schedule(dynamic, 64)
    for (int64_t r = 0; r < n_rows; ++r) {
      int64_t f = rows ? rows[r] : r;
      double* g = out + r * cout;
      for (int co = 0; co < cout; ++co) g[co] = 0.0;
      int64_t p0 = tex_off[f], p1 = tex_off[f + 1];
      for (int64_t p = p0; p < p1; ++p) {
        double d[3] = {(double)bary[3 * p], (double)bary[3 * p + 1], (double)bary[3 * p + 2]};
        double B[ORC_MAX_K];
        sh_basis_one(d, L, norm, B);
        filter_apply(B, K, cin, cout, h + p * cin, W, y);
        for (int co = 0; co < cout; ++co) g[co] += y[co];
      }
      if (p1 > p0)
        for (int co = 0; co < cout; ++co) g[co] /= (double)(p1 - p0);
    }
    free(y);
  }
}

/*
 * facet2facet backward:
 *   dh_p[ci]      = 1/R_f sum_k sum_co B_k(d_p) W[k][ci][co] dg_f[co],  f = facet of point p  (rows = points listed, or all)
 *   dW[k][ci][co] = sum_f 1/R_f sum_{p in f} B_k(d_p) h_p[ci] dg_f[co]
 */
void orc_f2f_bwd(int64_t F, const int32_t* tex_off, const float* bary, int L, int norm, int cin, int cout,
                 const double* h, const double* W, const double* dg, int64_t n_rows, const int64_t* rows,
                 double* dh, double* dW) {
  int K = (L + 1) * (L + 1);
  int64_t P = tex_off[F];
  int32_t* owner = (int32_t*)malloc((size_t)(P + 1) * sizeof(int32_t));
  for (int64_t f = 0; f < F; ++f)
    for (int64_t p = tex_off[f]; p < tex_off[f + 1]; ++p) owner[p] = (int32_t)f;
  if (dh) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
      int64_t p = rows ? rows[r] : r;
      int64_t f = owner[p];
      double R = (double)(tex_off[f + 1] - tex_off[f]);
      double d[3] = {(double)bary[3 * p], (double)bary[3 * p + 1], (double)bary[3 * p + 2]};
      double B[ORC_MAX_K];
      sh_basis_one(d, L, norm, B);
      for (int ci = 0; ci < cin; ++ci) {
        double acc = 0.0;
        for (int k = 0; k < K; ++k) {
          const double* w = W + ((int64_t)k * cin + ci) * cout;
          double t = 0.0;
          for (int co = 0; co < cout; ++co) t += w[co] * dg[f * cout + co];
          acc += B[k] * t;
        }
        dh[r * cin + ci] = acc / R;
      }
    }
  }
  if (dW) {
    double* Ball = (double*)malloc((size_t)(P + 1) * K * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < P; ++p) {
      double d[3] = {(double)bary[3 * p], (double)bary[3 * p + 1], (double)bary[3 * p + 2]};
      sh_basis_one(d, L, norm, Ball + p * K);
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t kc = 0; kc < (int64_t)K * cin; ++kc) {
      int k = (int)(kc / cin), ci = (int)(kc % cin);
      double* dd = dW + kc * cout;
      for (int co = 0; co < cout; ++co) dd[co] = 0.0;
      for (int64_t p = 0; p < P; ++p) {
        int64_t f = owner[p];
        double R = (double)(tex_off[f + 1] - tex_off[f]);
        double bh = Ball[p * K + k] * h[p * cin + ci] / R;
        for (int co = 0; co < cout; ++co) dd[co] += bh * dg[f * cout + co];
      }
    }
    free(Ball);
  }
  free(owner);
}


/* ------------------------------------------------------------------------------------------------
 * Depth-wise separable form of facet2vertex / vertex2facet (Section "Mesh convolutions": Eq. 5 and
 * Eq. 6 with one scalar coefficient set {a_l0, a_lm, b_lm} per channel, followed by a point-wise
 * channel mixing).  alpha[k][ci] are the per-channel SH coefficients, P[ci][co] the point-wise matrix.
 * It equals the dense form with W[k][ci][co] = alpha[k][ci] * P[ci][co]; the loops below follow the
 * staged definition (depth-wise, aggregate, point-wise), not that expansion.
 * ------------------------------------------------------------------------------------------------ */

/* s[ci] = sum_k alpha[k][ci] B[k]: the filter value of channel ci at the direction whose basis is B */
static void dw_filter(const double* B, int K, int cin, const double* alpha, double* s) {
  for (int ci = 0; ci < cin; ++ci) {
    double t = 0.0;
    for (int k = 0; k < K; ++k) t += alpha[(int64_t)k * cin + ci] * B[k];
    s[ci] = t;
  }
}

/* z_v[ci] = 1/|N(v)| sum_{f in N(v)} F_ci(n_f) h_f[ci]   (depth-wise Eq. 5) for one vertex */
static void sep_vertex_mean(int64_t v, const int32_t* rp, const int32_t* col, const float* vert, const int32_t* facet,
                            int L, int norm, int cin, const double* h, const double* alpha, double* s, double* z) {
  int K = (L + 1) * (L + 1);
  for (int ci = 0; ci < cin; ++ci) z[ci] = 0.0;
  int deg = rp[v + 1] - rp[v];
  for (int e = rp[v]; e < rp[v + 1]; ++e) {
    int64_t f = col[e] / 3;
    double n[3], B[ORC_MAX_K];
    facet_normal_one(vert, facet + 3 * f, n);
    sh_basis_one(n, L, norm, B);
    dw_filter(B, K, cin, alpha, s);
    for (int ci = 0; ci < cin; ++ci) z[ci] += s[ci] * h[f * cin + ci];
  }
  if (deg > 0)
    for (int ci = 0; ci < cin; ++ci) z[ci] /= (double)deg;
}

/* separable facet2vertex: g_v = z_v P.  Rows listed in `rows` (or all V). out [n_rows, cout]. */
void orc_f2v_sep(int64_t V, int64_t F, const float* vert, const int32_t* facet, int L, int norm, int cin, int cout,
                 const double* h, const double* alpha, const double* P, int64_t n_rows, const int64_t* rows,
                 double* out) {
  int32_t* rp = (int32_t*)malloc(((size_t)V + 1) * sizeof(int32_t));
  int32_t* col = (int32_t*)malloc((size_t)(3 * F + 1) * sizeof(int32_t));
  orc_vf_adjacency(V, F, facet, rp, col);
#pragma omp parallel
  {
    double* s = (double*)malloc((size_t)cin * sizeof(double));
    double* z = (double*)malloc((size_t)cin * sizeof(double));
#pragma omp for schedule(dynamic, 64)
    for (int64_t r = 0; r < n_rows; ++r) {
      int64_t v = rows ? rows[r] : r;
      sep_vertex_mean(v, rp, col, vert, facet, L, norm, cin, h, alpha, s, z);
      for (int co = 0; co < cout; ++co) {
        double t = 0.0;
        for (int ci = 0; ci < cin; ++ci) t += z[ci] * P[(int64_t)ci * cout + co];
        out[r * cout + co] = t;
      }
    }
    free(s); free(z);
  }
  free(rp); free(col);
}

/*
 * separable facet2vertex backward (transposed sums):
 *   dz_v[ci]       = sum_co P[ci][co] dg_v[co]
 *   dy_f[ci]       = sum_j dz_{v_j(f)}[ci] / |N(v_j(f))|
 *   dh_f[ci]       = F_ci(n_f) dy_f[ci]                                  (rows = facets listed, or all)
 *   dalpha[k][ci]  = sum_f B_k(n_f) h_f[ci] dy_f[ci]                      (all facets; skipped if NULL)
 *   dP[ci][co]     = sum_v z_v[ci] dg_v[co]                               (all vertices; skipped if NULL)
 */
void orc_f2v_sep_bwd(int64_t V, int64_t F, const float* vert, const int32_t* facet, int L, int norm, int cin,
                     int cout, const double* h, const double* alpha, const double* P, const double* dg,
                     int64_t n_rows, const int64_t* rows, double* dh, double* dalpha, double* dP) {
  int K = (L + 1) * (L + 1);
  int64_t* deg = (int64_t*)calloc((size_t)V, sizeof(int64_t));
  for (int64_t e = 0; e < 3 * F; ++e) deg[facet[e]]++;
  double* dz = (double*)malloc((size_t)(V > 0 ? V : 1) * cin * sizeof(double));
#pragma omp parallel for schedule(static)
  for (int64_t v = 0; v < V; ++v)
    for (int ci = 0; ci < cin; ++ci) {
      double t = 0.0;
      for (int co = 0; co < cout; ++co) t += P[(int64_t)ci * cout + co] * dg[v * cout + co];
      dz[v * cin + ci] = t;
    }
  if (dh) {
#pragma omp parallel
    {
      double* s = (double*)malloc((size_t)cin * sizeof(double));
#pragma omp for schedule(static)
      for (int64_t r = 0; r < n_rows; ++r) {
        int64_t f = rows ? rows[r] : r;
        double n[3], B[ORC_MAX_K];
        facet_normal_one(vert, facet + 3 * f, n);
        sh_basis_one(n, L, norm, B);
        dw_filter(B, K, cin, alpha, s);
        for (int ci = 0; ci < cin; ++ci) {
          double dy = 0.0;
          for (int j = 0; j < 3; ++j) {
            int64_t v = facet[3 * f + j];
            dy += dz[v * cin + ci] / (double)deg[v];
          }
          dh[r * cin + ci] = s[ci] * dy;
        }
      }
      free(s);
    }
  }
  if (dalpha) {
    for (int64_t i = 0; i < (int64_t)K * cin; ++i) dalpha[i] = 0.0;
    for (int64_t f = 0; f < F; ++f) {   /* ascending facet order */
      double n[3], B[ORC_MAX_K];
      facet_normal_one(vert, facet + 3 * f, n);
      sh_basis_one(n, L, norm, B);
      for (int ci = 0; ci < cin; ++ci) {
        double dy = 0.0;
        for (int j = 0; j < 3; ++j) {
          int64_t v = facet[3 * f + j];
          dy += dz[v * cin + ci] / (double)deg[v];
        }
        double hd = h[f * cin + ci] * dy;
        for (int k = 0; k < K; ++k) dalpha[(int64_t)k * cin + ci] += B[k] * hd;
      }
    }
  }
  if (dP) {
    int32_t* rp = (int32_t*)malloc(((size_t)V + 1) * sizeof(int32_t));
    int32_t* col = (int32_t*)malloc((size_t)(3 * F + 1) * sizeof(int32_t));
    orc_vf_adjacency(V, F, facet, rp, col);
    double* s = (double*)malloc((size_t)cin * sizeof(double));
    double* z = (double*)malloc((size_t)cin * sizeof(double));
    for (int64_t i = 0; i < (int64_t)cin * cout; ++i) dP[i] = 0.0;
    for (int64_t v = 0; v < V; ++v) {
      sep_vertex_mean(v, rp, col, vert, facet, L, norm, cin, h, alpha, s, z);
      for (int ci = 0; ci < cin; ++ci)
        for (int co = 0; co < cout; ++co) dP[(int64_t)ci * cout + co] += z[ci] * dg[v * cout + co];
    }
    free(s); free(z); free(rp); free(col);
  }
  free(dz); free(deg);
}

/* separable vertex2facet: u_f[ci] = sum_j F_ci(e_j) h_{v_j(f)}[ci] (depth-wise Eq. 6),  g_f = u_f P */
void orc_v2f_sep(int64_t V, int64_t F, const int32_t* facet, int L, int norm, int cin, int cout, const double* h,
                 const double* alpha, const double* P, int64_t n_rows, const int64_t* rows, double* out) {
  int K = (L + 1) * (L + 1);
  double Bc[3][ORC_MAX_K];
  corner_basis(L, norm, Bc);
  double* sc = (double*)malloc((size_t)3 * cin * sizeof(double));
  for (int j = 0; j < 3; ++j) dw_filter(Bc[j], K, cin, alpha, sc + (int64_t)j * cin);
  (void)V; (void)F;
#pragma omp parallel
  {
    double* u = (double*)malloc((size_t)cin * sizeof(double));
#pragma omp for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
      int64_t f = rows ? rows[r] : r;
      for (int ci = 0; ci < cin; ++ci) {
        double t = 0.0;
        for (int j = 0; j < 3; ++j) t += sc[(int64_t)j * cin + ci] * h[(int64_t)facet[3 * f + j] * cin + ci];
        u[ci] = t;
      }
      for (int co = 0; co < cout; ++co) {
        double t = 0.0;
        for (int ci = 0; ci < cin; ++ci) t += u[ci] * P[(int64_t)ci * cout + co];
        out[r * cout + co] = t;
      }
    }
    free(u);
  }
  free(sc);
}

/*
 * separable vertex2facet backward:
 *   du_f[ci]      = sum_co P[ci][co] dg_f[co]
 *   dh_v[ci]      = sum_{(f,j): v_j(f)=v} F_ci(e_j) du_f[ci]              (rows = vertices listed, or all)
 *   dalpha[k][ci] = sum_f sum_j B_k(e_j) h_{v_j(f)}[ci] du_f[ci]
 *   dP[ci][co]    = sum_f u_f[ci] dg_f[co]
 */
void orc_v2f_sep_bwd(int64_t V, int64_t F, const int32_t* facet, int L, int norm, int cin, int cout, const double* h,
                     const double* alpha, const double* P, const double* dg, int64_t n_rows, const int64_t* rows,
                     double* dh, double* dalpha, double* dP) {
  int K = (L + 1) * (L + 1);
  double Bc[3][ORC_MAX_K];
  corner_basis(L, norm, Bc);
  double* sc = (double*)malloc((size_t)3 * cin * sizeof(double));
  for (int j = 0; j < 3; ++j) dw_filter(Bc[j], K, cin, alpha, sc + (int64_t)j * cin);
  double* du = (double*)malloc((size_t)(F > 0 ? F : 1) * cin * sizeof(double));
#pragma omp parallel for schedule(static)
  for (int64_t f = 0; f < F; ++f)
    for (int ci = 0; ci < cin; ++ci) {
      double t = 0.0;
      for (int co = 0; co < cout; ++co) t += P[(int64_t)ci * cout + co] * dg[f * cout + co];
      du[f * cin + ci] = t;
    }
  if (dh) {
    int32_t* rp = (int32_t*)malloc(((size_t)V + 1) * sizeof(int32_t));
    int32_t* col = (int32_t*)malloc((size_t)(3 * F + 1) * sizeof(int32_t));
    orc_vf_adjacency(V, F, facet, rp, col);
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t r = 0; r < n_rows; ++r) {
      int64_t v = rows ? rows[r] : r;
      for (int ci = 0; ci < cin; ++ci) dh[r * cin + ci] = 0.0;
      for (int e = rp[v]; e < rp[v + 1]; ++e) {
        int64_t f = col[e] / 3;
        int j = col[e] % 3;
        for (int ci = 0; ci < cin; ++ci) dh[r * cin + ci] += sc[(int64_t)j * cin + ci] * du[f * cin + ci];
      }
    }
    free(rp); free(col);
  }
  if (dalpha) {
    for (int64_t i = 0; i < (int64_t)K * cin; ++i) dalpha[i] = 0.0;
    for (int64_t f = 0; f < F; ++f)
      for (int j = 0; j < 3; ++j) {
        int64_t v = facet[3 * f + j];
        for (int ci = 0; ci < cin; ++ci) {
          double hd = h[v * cin + ci] * du[f * cin + ci];
          for (int k = 0; k < K; ++k) dalpha[(int64_t)k * cin + ci] += Bc[j][k] * hd;
        }
      }
  }
  if (dP) {
    for (int64_t i = 0; i < (int64_t)cin * cout; ++i) dP[i] = 0.0;
    for (int64_t f = 0; f < F; ++f)
      for (int ci = 0; ci < cin; ++ci) {
        double u = 0.0;
        for (int j = 0; j < 3; ++j) u += sc[(int64_t)j * cin + ci] * h[(int64_t)facet[3 * f + j] * cin + ci];
        for (int co = 0; co < cout; ++co) dP[(int64_t)ci * cout + co] += u * dg[f * cout + co];
      }
  }
  free(sc); free(du);
}

/* ------------------------------------------------------------------------------------------------
 * Selected rows of the coefficient gradients.  dW is a sum over every facet (point), so at sizes where
 * the whole tensor takes the oracle too long it evaluates the rows dW[k][ci][0..cout) named by
 * wrows[i] = k*cin + ci, each by the same ascending sum over all facets as the full functions above
 * (same definitions, transposed sums of Eq. 5 / 6 / 7; the results agree bit for bit with those rows).
 * out is [n_wrows, cout].
 * ------------------------------------------------------------------------------------------------ */
void orc_f2v_dW_rows(int64_t V, int64_t F, const float* vert, const int32_t* facet, int L, int norm, int cin, int cout,
                     const double* h, const double* dg, int64_t n_wrows, const int64_t* wrows, double* out) {
  int K = (L + 1) * (L + 1);
  int64_t* deg = (int64_t*)calloc((size_t)V, sizeof(int64_t));
  for (int64_t e = 0; e < 3 * F; ++e) deg[facet[e]]++;
  double* Ball = (double*)malloc((size_t)(F + 1) * K * sizeof(double));
#pragma omp parallel for schedule(static)
  for (int64_t f = 0; f < F; ++f) {
    double n[3];
    facet_normal_one(vert, facet + 3 * f, n);
    sh_basis_one(n, L, norm, Ball + f * K);
  }
#pragma omp parallel
  {
    double* dy = (double*)malloc((size_t)cout * sizeof(double));
#pragma omp for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_wrows; ++i) {
      int k = (int)(wrows[i] / cin), ci = (int)(wrows[i] % cin);
      double* d = out + i * cout;
      for (int co = 0; co < cout; ++co) d[co] = 0.0;
      for (int64_t f = 0; f < F; ++f) {
        for (int co = 0; co < cout; ++co) dy[co] = 0.0;
        for (int j = 0; j < 3; ++j) {
          int64_t v = facet[3 * f + j];
          for (int co = 0; co < cout; ++co) dy[co] += dg[v * cout + co] / (double)deg[v];
        }
        double bh = Ball[f * K + k] * h[f * cin + ci];
        for (int co = 0; co < cout; ++co) d[co] += bh * dy[co];
      }
    }
    free(dy);
  }
  free(Ball); free(deg);
}

void orc_v2f_dW_rows(int64_t V, int64_t F, const int32_t* facet, int L, int norm, int cin, int cout, const double* h,
                     const double* dg, int64_t n_wrows, const int64_t* wrows, double* out) {
  (void)V;
  double Bc[3][ORC_MAX_K];
  corner_basis(L, norm, Bc);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < n_wrows; ++i) {
    int k = (int)(wrows[i] / cin), ci = (int)(wrows[i] % cin);
    double* d = out + i * cout;
    for (int co = 0; co < cout; ++co) d[co] = 0.0;
    for (int64_t f = 0; f < F; ++f)
      for (int j = 0; j < 3; ++j) {
        int64_t v = facet[3 * f + j];
        double bh = Bc[j][k] * h[v * cin + ci];
        for (int co = 0; co < cout; ++co) d[co] += bh * dg[f * cout + co];
      }
  }
}

void orc_f2f_dW_rows(int64_t F, const int32_t* tex_off, const float* bary, int L, int norm, int cin, int cout,
                     const double* h, const double* dg, int64_t n_wrows, const int64_t* wrows, double* out) {
  int K = (L + 1) * (L + 1);
  int64_t P = tex_off[F];
  int32_t* owner = (int32_t*)malloc((size_t)(P + 1) * sizeof(int32_t));
  for (int64_t f = 0; f < F; ++f)
    for (int64_t p = tex_off[f]; p < tex_off[f + 1]; ++p) owner[p] = (int32_t)f;
  double* Ball = (double*)malloc((size_t)(P + 1) * K * sizeof(double));
#pragma omp parallel for schedule(static)
  for (int64_t p = 0; p < P; ++p) {
    double d[3] = {(double)bary[3 * p], (double)bary[3 * p + 1], (double)bary[3 * p + 2]};
    sh_basis_one(d, L, norm, Ball + p * K);
  }
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < n_wrows; ++i) {
    int k = (int)(wrows[i] / cin), ci = (int)(wrows[i] % cin);
    double* dd = out + i * cout;
    for (int co = 0; co < cout; ++co) dd[co] = 0.0;
    for (int64_t p = 0; p < P; ++p) {
      int64_t f = owner[p];
      double R = (double)(tex_off[f + 1] - tex_off[f]);
      double bh = Ball[p * K + k] * h[p * cin + ci] / R;
      for (int co = 0; co < cout; ++co) dd[co] += bh * dg[f * cout + co];
    }
  }
  free(Ball); free(owner);
}

int orc_max_l(void) { return ORC_MAX_L; }
