// Host-side declarations shared by the picassomesh translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pm_device.h"

// ---- error plumbing -------------------------------------------------------------------------
pm_status pm_fail(pm_status s, const char* fmt, ...);
#define PM_CHECK_HIP(expr)                                                                        \
  do {                                                                                            \
    hipError_t e__ = (expr);                                                                      \
    if (e__ != hipSuccess) return pm_fail(PM_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e__));   \
  } while (0)
#define PM_CHECK_LAUNCH(name)                                                                     \
  do {                                                                                            \
    hipError_t e__ = hipGetLastError();                                                           \
    if (e__ != hipSuccess) return pm_fail(PM_ERR_HIP, "launch %s: %s", name, hipGetErrorString(e__)); \
  } while (0)

#define PM_TRY(expr)                 \
  do {                               \
    pm_status s__ = (expr);          \
    if (s__ != PM_OK) return s__;    \
  } while (0)

// ---- optional per-kernel event timing (see pm_profile_* in the public header) -----------------
void pm_prof_begin(hipStream_t st, const char* kernel);
void pm_prof_end(hipStream_t st);
void pm_prof_set_op(const char* op);
struct ProfScope {
  hipStream_t st;
  ProfScope(hipStream_t s, const char* kernel) : st(s) { pm_prof_begin(st, kernel); }
  ~ProfScope() { pm_prof_end(st); }
};

// Raises a kernel's dynamic-LDS limit; the runtime call is made once per (kernel, device) and size, later calls
// are a table lookup.
pm_status pm_set_dyn_lds(const void* kernel, size_t bytes);

static inline bool pm_aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }
static inline size_t pm_round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Eq. 3 normalisation constants in double precision (times sqrt(2) for m > 0 when orthonormal).
void pm_make_sh_table(int L, pm_sh_norm norm, ShTable* T);
// Basis values (double) at the three corner directions of Eq. 6: Bc[j][k].
void pm_corner_basis(int L, pm_sh_norm norm, double Bc[3][PM_MAX_K]);

// ---- tiling constants of the MFMA kernels -----------------------------------------------------
// A "granule" is the 16 bytes one lane feeds to the matrix core for one c-group:
//   bf16: 8 contraction channels (one 32x32x16 MFMA covers a group of 16 = 2 half-waves x 8)
//   fp32: 4 contraction channels (four 32x32x2 MFMAs cover a group of 8 = 2 half-waves x 4)
#define PM_GC 4   /* c-groups per chunk held in registers            */
#define PM_NBS 2  /* 32-wide output-channel blocks per weight stage  */
static inline int pm_group_c(pm_dtype dt) { return dt == PM_BF16 ? 16 : 8; }
static inline int pm_chunk_c(pm_dtype dt) { return PM_GC * pm_group_c(dt); }
#define PM_STAGE_BYTES (PM_NBS * PM_GC * 64 * 16)

struct PackGeom {
  int K, Cc, Cn;   // logical sizes of Wp[k][c][n]
  int NCH;         // c-chunks
  int NBG;         // groups of PM_NBS output blocks
  int64_t stages;  // NBG * NCH * K
};
static inline PackGeom pm_pack_geom(int K, int Cc, int Cn, pm_dtype dt) {
  PackGeom g;
  g.K = K; g.Cc = Cc; g.Cn = Cn;
  g.NCH = (Cc + pm_chunk_c(dt) - 1) / pm_chunk_c(dt);
  g.NBG = (Cn + 32 * PM_NBS - 1) / (32 * PM_NBS);
  g.stages = (int64_t)g.NBG * g.NCH * K;
  return g;
}
static inline size_t pm_pack_bytes(const PackGeom& g) { return (size_t)g.stages * PM_STAGE_BYTES; }

// ---- kernel launchers (each enqueues on `st`, returns PM_OK or PM_ERR_HIP) ----------------------
enum PackMode { PACK_PLAIN = 0, PACK_TRANS = 1, PACK_FOLD = 2, PACK_FOLD_TRANS = 3, PACK_FOLD_BWD = 4,
                PACK_SEP_FOLD = 5, PACK_PLAIN_TWICE = 6 };
struct FoldCoef { float c[3][PM_MAX_K]; };
// Builds the MFMA operand image of Wp[k][c][n] from W[K][cin][cout] (src dtype = dt):
//   PLAIN: Wp[k][ci][co] = W[k][ci][co]          TRANS: Wp[k][co][ci] = W[k][ci][co]
//   FOLD:  Wp[0][j*cin+ci][co] = sum_k fc[j][k] W[k][ci][co]    FOLD_TRANS: Wp[0][co][j*cin+ci] = same
//   FOLD_BWD: Wp[0][j*cout+co][ci] = same   (backward-data of the folded form, contraction over (corner, co))
//   PLAIN_TWICE: K = 1, Wp[0][c][co] = W[0][c mod 64][co] for c < 128 (zero where c mod 64 >= cin): the operand rows carry
//   a bf16 head in channels 0..63 and the bf16 remainder in channels 64..127
//   SEP_FOLD (separable vertex2facet): like FOLD with the folded matrices
//   W_j[ci][co] = s_j[ci] P[ci][co],  s_j[ci] = sum_k fc[j][k] alpha[k][ci];  W is P [cin][cout], alpha [K][cin] fp32
pm_status pm_launch_pack(PackMode mode, pm_dtype dt, int K, int cin, int cout, const void* W, const FoldCoef* fc,
                         void* apack, hipStream_t st, const float* alpha = nullptr);

enum BMode { B_ONE = 0, B_NORMAL = 1, B_DIRS = 2 };
enum XMode { X_DIRECT = 0, X_GATHER_SUM = 1, X_GATHER_CAT = 2, X_GATHER1 = 3 };

// Source of one operand row set for the row-wise kernels.
struct RowSrc {
  const void* p;            // matrix [*, C] of the source dtype
  int is_bf16;              // 1: bf16 storage, 0: fp32
  int C;                    // channels per source row
  const int32_t* facet;     // [R,3]  X_GATHER_SUM / X_GATHER_CAT: rows gathered through the corner ids
  const int32_t* row_ptr;   // X_GATHER_SUM: each gathered row is divided by deg(v) = row_ptr[v+1]-row_ptr[v]
  const int32_t* owner;     // X_GATHER1: source row = owner[r]
  const int32_t* seg_off;   // X_GATHER1: scale = 1 / (seg_off[o+1] - seg_off[o])
};

struct BasisSrc {
  const float* vert;        // B_NORMAL
  const int32_t* facet;     // B_NORMAL: [R,3]
  const float* dirs;        // B_DIRS: [R,3]
  const float* bvals;       // precomputed basis rows [R,K] (weight-gradient kernel)
  const int32_t* owner;     // optional (B_DIRS): basis scaled by 1/(seg_off[o+1]-seg_off[o]) -- unused when NULL
  const int32_t* seg_off;
  ShTable sh;
};

// out[r][n] = sum_k B_r[k] sum_c X_r[c] Wp[k][c][n]      (B_ONE: K = 1, B = 1)
pm_status pm_launch_conv_rows(pm_dtype mt, BMode bm, XMode xm, int64_t R, int K, int Cc, int Cn, const BasisSrc& bs,
                              const RowSrc& xs, const void* apack, void* out, int out_is_bf16, hipStream_t st);

// out[v][c] = scale_v * sum_{e in [row_ptr[v], row_ptr[v+1])} src[(col ? col[e] : e) / div][c]
// scale_v = 1/deg (mean != 0) or 1.  src is fp32 or bf16; the sum is always accumulated in fp32.
pm_status pm_launch_segreduce(int64_t n_seg, int C, const void* src, int src_is_bf16, const int32_t* row_ptr,
                              const int32_t* col, int div, int mean, void* out, int out_is_bf16, hipStream_t st);

// dWp[k][c][n] = sum_r B_r[k] X_r[c] Y_r[n], fp32, deterministic (per-workgroup partials + fixed-order sum).
// X_GATHER_CAT here means: k indexes the corner, X^{(k)}_r = xs.p[facet[r][k]] (K must be 3, B_ONE).
// bs.bvals must hold the basis rows [R][K] (fp32) unless B_ONE or pm_wgrad_fuses_basis() says that the kernel
// chosen for these arguments evaluates the basis itself from bs.vert / bs.facet / bs.dirs.  Only that kernel
// accepts y_out != NULL: it then also writes the Y operand rows (after gathering), bf16 [R][Cn].
size_t pm_wgrad_ws_bytes(int64_t R, int K, int Cc, int Cn);
bool pm_wgrad_fuses_basis(pm_dtype mt, BMode bm, XMode xm, XMode ym, int K, int Cc, int Cn, const RowSrc& xs,
                          const RowSrc& ys);
pm_status pm_launch_wgrad(pm_dtype mt, BMode bm, XMode xm, XMode ym, int64_t R, int K, int Cc, int Cn,
                          const BasisSrc& bs, const RowSrc& xs, const RowSrc& ys, float* dWp, void* ws, size_t ws_bytes,
                          void* y_out, hipStream_t st);
// The same without a basis for bf16 rows of 32 / 64 channels (K = 3 gathered corner rows, or K = 1 direct rows):
// row-major LDS tiles and transposing LDS reads (pm_wgrad_stage.hip); pm_launch_wgrad takes it where it applies
bool pm_wgrad_stage_applies(pm_dtype mt, BMode bm, XMode xm, XMode ym, int K, int Cc, int Cn, const RowSrc& xs,
                            const RowSrc& ys);
pm_status pm_launch_wgrad_stage(XMode xm, int64_t R, int K, int Cc, int Cn, const RowSrc& xs, const RowSrc& ys, float* dWp,
                                void* ws, size_t ws_bytes, hipStream_t st);
// dW[k][ci][co] = sum_j fc[j][k] M[j][ci][co]
pm_status pm_launch_unfold(int K, int cin, int cout, const float* M, const FoldCoef* fc, float* dW, hipStream_t st);
// out[v][j][c] = sum over the entries e of segment v with col[e] % 3 == j of src[col[e] / 3][c]   (j = 0..2):
// the facet rows adjacent to a vertex, summed separately per corner slot, ascending entry order, fp32 sums.
pm_status pm_launch_segsum_slots(int64_t n_seg, int C, const void* src, int src_is_bf16, const int32_t* row_ptr,
                                 const int32_t* col, void* out, int out_is_bf16, hipStream_t st);
// out[i] = sum over n_slice slices of partial[slice][i], added in a fixed order (bitwise reproducible)
pm_status pm_launch_sum_slices(const float* partial, int64_t n, int n_slice, float* out, hipStream_t st);
pm_status pm_launch_sum_slices_strided(const float* partial, int64_t n, int64_t stride, int n_slice, float* out,
                                       hipStream_t st);

// Depth-wise stage of the separable facet2vertex form: y_f[c] = h_f[c] * sum_k alpha[k][c] B_k(n_f), and its backward
// (dh_f[c] = dy_f[c] * filter, dy_f = gathered mean of dz;  dalpha[k][c] = sum_f B_k(n_f) h_f[c] dy_f[c]);
// optionally dh leaves as dh * mask_scale * [h > 0] (the epilogue that produced h).  dz_prescaled: the rows of dz
// already carry their 1/deg(v).
size_t pm_sep_dalpha_ws_bytes(int64_t F, int K, int C, int is_bf16);
pm_status pm_launch_dw_f2v(int64_t F, int K, int C, int is_bf16, const BasisSrc& bs, const void* h, const float* alpha,
                           void* y, hipStream_t st);
pm_status pm_launch_dw_f2v_bwd(int64_t F, int K, int C, int is_bf16, const BasisSrc& bs, const void* h,
                               const float* alpha, const float* dz, const int32_t* row_ptr, void* dh, float* dalpha,
                               float* partial, const float* mask_scale, int mask_relu, int dz_prescaled, hipStream_t st);
// separable vertex2facet backward: out[v][c] = sum over entries (f, j) of v of s_j[c] T[f][c]
pm_status pm_launch_slot_scale_sum(int64_t V, int K, int C, int is_bf16, const void* T, const int32_t* row_ptr,
                                   const int32_t* col, const float* alpha, const FoldCoef* fc, float* sc, void* out,
                                   hipStream_t st);
// separable vertex2facet: dP, dalpha from the three corner matrices M [3][cin][cout]
pm_status pm_launch_sep_unfold(int K, int cin, int cout, int p_bf16, const float* M, const float* alpha, const void* P,
                               const FoldCoef* fc, float* dalpha, float* dP, hipStream_t st);
// facet2facet with few input channels (K cin <= 64): S[f][0..K cin) = mean over the points of f of B_k(d_p) h_p[ci], zero
// up to 64 channels (feature dtype), and dh[p][ci] = 1/R_f sum_k B_k(d_p) T[owner p][k cin + ci] with T fp32 [F][K cin]
bool pm_f2f_small_applies(int L, int cin);
pm_status pm_launch_f2f_gather(int64_t n_facet, const int32_t* tex_off, const float* bary, const ShTable& sh, int cin,
                               int is_bf16, const void* h, void* S, hipStream_t st);
pm_status pm_launch_f2f_scatter(int64_t n_tex, const int32_t* owner, const int32_t* tex_off, const float* bary,
                                const ShTable& sh, int cin, int is_bf16, const float* T, void* dh, hipStream_t st);
// owner[p] = f for p in [tex_off[f], tex_off[f+1])
pm_status pm_launch_owner(int64_t n_facet, const int32_t* tex_off, int32_t* owner, hipStream_t st);

pm_status pm_launch_basis_mesh(const pm_mesh* mesh, const ShTable& T, float* basis, hipStream_t st);
pm_status pm_launch_basis_dirs(int64_t n, const float* dirs, const ShTable& T, float* basis, hipStream_t st);
pm_status pm_launch_basis_bwd(int64_t n, const float* dirs, const ShTable& T, const float* dbasis, float* ddirs,
                              hipStream_t st);

size_t pm_adj_ws_bytes(int64_t n_vert, int64_t n_facet);
size_t pm_csr_ws_bytes(int64_t n_rows, int64_t n_entries);
pm_status pm_launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t st);
size_t pm_scan_ws_bytes(int64_t n);
pm_status pm_launch_exclusive_scan(const int32_t* cnt, int64_t n, int32_t* out, void* tile_ws, hipStream_t st);
// point-cloud convolution with the radial term (depth-wise stage and its transposed sums)
size_t pm_pc_coef_ws_bytes(int64_t M, int K, int C);
pm_status pm_launch_pc_dw(int64_t M, int64_t N, int K, int C, int is_bf16, float rho, const ShTable& sh, const float* xq,
                          const float* xs, const int32_t* nbr_ptr, const int32_t* nbr_idx, const void* h,
                          const float* alpha, const float* c0, void* y, hipStream_t st);
pm_status pm_launch_pc_dw_coef(int64_t M, int64_t N, int K, int C, int is_bf16, float rho, const ShTable& sh,
                               const float* xq, const float* xs, const int32_t* nbr_ptr, const int32_t* nbr_idx,
                               const void* h, const float* alpha, const float* c0, const float* dy, void* y,
                               float* dalpha, float* dc0, float* partial, hipStream_t st);
pm_status pm_launch_pc_dw_dh(int64_t M, int64_t N, int K, int C, int is_bf16, float rho, const ShTable& sh,
                             const float* xq, const float* xs, const int32_t* nbr_ptr, const int32_t* rev_ptr,
                             const int32_t* rev_col, const int32_t* owner, const float* alpha, const float* c0,
                             const float* dy, void* dh, hipStream_t st);
pm_status pm_launch_validate_nbr(int64_t M, int64_t N, int64_t nnz, const int32_t* ptr, const int32_t* idx,
                                 int32_t* flag, hipStream_t st);
// input preparation: facet geometric features (Eq. 9), texture resolution and interpolation lattice (Eq. 8)
pm_status pm_launch_facet_geometry(const pm_mesh* mesh, int with_heights, int out_bf16, void* feat, hipStream_t st);
size_t pm_texture_ws_bytes_host(int64_t n_facet, int n_mesh);
pm_status pm_launch_texture_layout(const pm_mesh* mesh, int alpha, int beta, int32_t* gamma, int32_t* tex_off, void* ws,
                                   hipStream_t st);
pm_status pm_launch_texture_bary(int64_t n_facet, const int32_t* gamma, const int32_t* tex_off, int64_t n_tex, float* bary,
                                 hipStream_t st);
pm_status pm_launch_csr(int64_t n_rows, int64_t n_entries, const int32_t* keys, int32_t* row_ptr, int32_t* col, void* ws,
                        hipStream_t st);
// vertex2facet forward with LDS-staged facet tiles (bf16, Cin = 32 or 64)
bool pm_v2f_stage_applies(pm_dtype dt, int cin, int cout, const void* h, const void* out);
pm_status pm_launch_v2f_stage(int64_t F, int cin, int cout, const int32_t* facet, const void* h, const void* apack,
                              void* out, hipStream_t st);
// the same kernel with the fused stages of the separable vertex2vertex block (see pm_v2f_stage.hip)
pm_status pm_launch_v2v_stage(int64_t R, int cin, int cout, const int32_t* facet, const void* h, const void* apack,
                              const float* ep_scale, const float* ep_shift, int relu, void* save, const float* alpha2,
                              int K2, const float* vert, const ShTable* sh, void* out, hipStream_t st);
bool pm_point_stage_wide_applies(pm_dtype dt, int cin, int cout, const void* rows, const void* out);
pm_status pm_launch_point_stage_wide(int64_t R, int cin, int cout, const void* rows, const void* apack, void* out,
                                     hipStream_t st);
pm_status pm_launch_point_stage_f32(int64_t R, int cin, int cout, const void* rows, const void* apack, float* out,
                                    const int32_t* row_ptr, hipStream_t st);
// x <- act(scale x + shift) in place, and its backward out = dy scale [y_saved > 0]   (scale / shift may be NULL)
pm_status pm_launch_affine_act(int64_t n_rows, int C, int is_bf16, void* x, const float* scale, const float* shift,
                               int relu, hipStream_t st);
pm_status pm_launch_affine_act_bwd(int64_t n_rows, int C, int is_bf16, const void* dy, const void* y_saved,
                                   const float* scale, int relu, void* out, hipStream_t st);
// pooling over vertex clusters
pm_status pm_launch_cluster_target(int64_t n_in, int64_t n_out, const int32_t* vcluster, const int32_t* iomap,
                                   int32_t* target, int32_t* bad, hipStream_t st);
pm_status pm_launch_segmax(int64_t n_out, int C, int is_bf16, const void* h_in, const int32_t* row_ptr,
                           const int32_t* col, void* h_out, int32_t* argmax, hipStream_t st);
pm_status pm_launch_cluster_gather(int mode, int64_t n_in, int C, int is_bf16, const int32_t* target,
                                   const int32_t* row_ptr, const int32_t* argmax, const void* src, void* out,
                                   hipStream_t st);
pm_status pm_launch_adjacency(const pm_mesh* mesh, int32_t* row_ptr, int32_t* col, void* ws, hipStream_t st);
pm_status pm_launch_validate(const pm_mesh* mesh, int32_t* flag, hipStream_t st);
