/*
 * picassomesh -- spherical-harmonic continuous-filter mesh convolutions on MI355X (gfx950).
 *
 * C ABI of the hot path of "Mesh Convolution with Continuous Filters for 3D Surface Parsing":
 * facet2vertex (Eq. 5), vertex2facet (Eq. 6), facet2facet (Eq. 7), their backward passes, the
 * real truncated SH basis (Eq. 3-4) and the vertex->facet adjacency the reductions run over.
 *
 * General rules for every entry point
 *   - Plain C linkage.  Every pointer is a DEVICE pointer unless the comment says HOST; all are
 *     borrowed (never freed or retained).  `stream` is a hipStream_t passed as void* (NULL = the
 *     default stream).  All work is enqueued on that stream; no entry point allocates device memory
 *     and only the pm_validate_* calls synchronise with the host.
 *   - Arrays are row-major and contiguous.  Base pointers of feature, weight, output and workspace
 *     arrays must be 16-byte aligned (checked -> PM_ERR_INVALID_ARG).
 *   - Meshes come as one packed heterogeneous batch ("Heterogeneous Batching" subsection): vertex
 *     arrays of all meshes concatenated, facet index arrays concatenated with the running vertex count
 *     already added, 0-indexed.  The convolutions themselves never need the per-mesh offsets.
 *   - n_vert, n_facet, n_tex and 3*n_facet must be < 2^31 (ids are int32); element offsets are
 *     computed in 64 bits.  Out-of-range ids are undefined behaviour in the convolutions; call
 *     pm_validate_mesh first when the input is untrusted.
 *   - Outputs are overwritten, never accumulated (dW included).  Results are bitwise reproducible
 *     from call to call: no floating-point atomics are used anywhere.
 *   - Filter coefficients are dense:  W[k][ci][co],  k = l*(l+1)+m,  m in [-l,l];  m > 0 multiplies
 *     the cos(m phi) function (a_lm of Eq. 4), m < 0 the sin(|m| phi) function (b_l|m|), m = 0 is a_l0.
 *     K = (L+1)^2 (the paper's kernel size T).  0 <= L <= PM_MAX_L.
 *   - dtype selects the storage type of features AND coefficients AND feature outputs (PM_F32 or
 *     PM_BF16).  Geometry, basis values, accumulation and dW are always fp32.
 *   - Return value: PM_OK or a negative pm_status; pm_last_error() gives a thread-local message.
 *     Argument errors are detected before anything is enqueued.
 */
#ifndef PICASSOMESH_H
#define PICASSOMESH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PM_MAX_L 5

typedef int32_t pm_status;
enum {
  PM_OK = 0,
  PM_ERR_INVALID_ARG = -1, /* NULL / misaligned pointer, negative size, size over the int32 limits   */
  PM_ERR_UNSUPPORTED = -2, /* L > PM_MAX_L, unknown dtype / norm / op                                */
  PM_ERR_WORKSPACE = -3,   /* workspace smaller than pm_workspace_bytes reports                      */
  PM_ERR_HIP = -4,         /* a HIP runtime call or kernel launch failed                             */
  PM_ERR_BAD_MESH = -5     /* pm_validate_mesh found an out-of-range id or inconsistent offsets      */
};

typedef enum { PM_F32 = 0, PM_BF16 = 1 } pm_dtype;

/* PM_SH_PAPER: the functions exactly as printed in Eq. 4 (squared L2 norm 1 for m = 0, 1/2 for m != 0).
 * PM_SH_ORTHONORMAL: m != 0 functions multiplied by sqrt(2), the orthonormal family the abstract names. */
typedef enum { PM_SH_PAPER = 0, PM_SH_ORTHONORMAL = 1 } pm_sh_norm;

typedef enum {
  PM_OP_ADJACENCY = 0, PM_OP_F2V = 1, PM_OP_F2V_BWD = 2, PM_OP_V2F = 3, PM_OP_V2F_BWD = 4,
  PM_OP_F2F = 5, PM_OP_F2F_BWD = 6,
  PM_OP_F2V_SEP = 7, PM_OP_F2V_SEP_BWD = 8, PM_OP_V2F_SEP = 9, PM_OP_V2F_SEP_BWD = 10
} pm_op;

/* Packed batch of triangle meshes (device arrays). */
typedef struct pm_mesh {
  int32_t n_mesh;
  int64_t n_vert, n_facet;
  const float* vert;        /* [n_vert,3]   xyz                                                       */
  const int32_t* facet;     /* [n_facet,3]  global vertex ids; corner order is significant (it fixes
                               the normal by the right-hand rule and the roles of Eq. 6's three terms) */
  const int32_t* vert_off;  /* [n_mesh+1]   may be NULL when n_mesh == 1; used by validation only      */
  const int32_t* facet_off; /* [n_mesh+1]   may be NULL when n_mesh == 1                              */
} pm_mesh;

/* Vertex -> facet adjacency N(v) of Eq. 5 as CSR over corner slots: entries of vertex v are
 * col[row_ptr[v] .. row_ptr[v+1]), each equal to 3*f+j (facet f, corner j), ascending. */
typedef struct pm_vf_adj {
  const int32_t* row_ptr; /* [n_vert+1] */
  const int32_t* col;     /* [3*n_facet] */
} pm_vf_adj;

const char* pm_status_string(pm_status s);
const char* pm_last_error(void);

/* Bytes of workspace an op needs for these sizes (HOST computation, no GPU call).  n_tex is the number
 * of texture points (facet2facet only, else 0).  Returns 0 on invalid arguments. */
size_t pm_workspace_bytes(pm_op op, int64_t n_vert, int64_t n_facet, int64_t n_tex, int L, int cin, int cout,
                          pm_dtype dtype);

/* Range-checks facet ids against each mesh's vertex range and the offset arrays.  Synchronises.
 * ws: >= 16 bytes of device memory. */
pm_status pm_validate_mesh(const pm_mesh* mesh, void* ws, size_t ws_bytes, void* stream);

/* Builds N(v) (the receptive field of Eq. 5) for the whole batch.  row_ptr [n_vert+1] and col [3*n_facet]
 * are outputs.  Deterministic: col is sorted ascending within each vertex. */
pm_status pm_build_vf_adjacency(const pm_mesh* mesh, int32_t* row_ptr, int32_t* col, void* ws, size_t ws_bytes,
                                void* stream);

/* Eq. 3-4 at the facet normals (x2-x1)x(x3-x1) of the mesh (facet2vertex's angular arguments):
 * basis [n_facet, K] fp32.  A facet whose cross product has squared length < 1e-30 uses (0,0,1). */
pm_status pm_sh_basis(const pm_mesh* mesh, int L, pm_sh_norm norm, float* basis, void* stream);
/* Eq. 3-4 at arbitrary directions dirs [n,3] (normalised inside; need not be unit): basis [n,K]. */
pm_status pm_sh_basis_dirs(int64_t n, const float* dirs, int L, pm_sh_norm norm, float* basis, void* stream);
/* Gradient of <dbasis, basis(dirs)> with respect to dirs: ddirs [n,3]. */
pm_status pm_sh_basis_bwd(int64_t n, const float* dirs, int L, pm_sh_norm norm, const float* dbasis, float* ddirs,
                          void* stream);

/* facet2vertex, Eq. 5:  g_v = 1/|N(v)| sum_{f in N(v)} sum_k sum_ci B_k(n_f) h_f[ci] W[k][ci][co].
 * h_facet [F,cin], W [K,cin,cout], g_vert [V,cout] (dtype).  Vertices with empty N(v) get zeros. */
pm_status pm_f2v(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype,
                 const void* h_facet, const void* W, void* g_vert, void* ws, size_t ws_bytes, void* stream);
/* Backward of Eq. 5.  dg_vert [V,cout] (dtype) -> dh_facet [F,cin] (dtype, may be NULL),
 * dW [K,cin,cout] fp32 (may be NULL). */
pm_status pm_f2v_bwd(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cout,
                     pm_dtype dtype, const void* h_facet, const void* W, const void* dg_vert, void* dh_facet,
                     float* dW, void* ws, size_t ws_bytes, void* stream);

/* vertex2facet, Eq. 6:  g_f = F(pi/2,0) h_{v1} + F(pi/2,pi/2) h_{v2} + F(0,0) h_{v3}  (no 1/3).
 * h_vert [V,cin], g_facet [F,cout].  Geometry is not read (mesh->vert may be NULL). */
pm_status pm_v2f(const pm_mesh* mesh, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype, const void* h_vert,
                 const void* W, void* g_facet, void* ws, size_t ws_bytes, void* stream);
/* For callers that cannot allocate or pass a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same operation and same result, bit for bit, as pm_v2f; the folded coefficient
 * image (the only scratch memory of the forward pass) is kept in a static device array of
 * PM_V2F_NOALLOC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends.  The call
 * allocates nothing and frees nothing.  Shapes whose image does not fit (roughly 3*cin*cout*sizeof(dtype), rounded
 * up to 8 KiB blocks) are refused with PM_ERR_WORKSPACE.  All calls on one GPU share the array: calls that
 * overlap on different streams of the same GPU race on it; calls on one stream are ordered and safe.  The first
 * call on a device looks up the array's address (no stream work); make one call outside a capture first. */
#define PM_V2F_NOALLOC_SCRATCH_BYTES (4u << 20)
pm_status pm_v2f_noalloc(const pm_mesh* mesh, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype,
                         const void* h_vert, const void* W, void* g_facet, void* stream);

/* Backward of Eq. 6.  dg_facet [F,cout] -> dh_vert [V,cin] (may be NULL; needs adj), dW fp32 (may be NULL). */
pm_status pm_v2f_bwd(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cout,
                     pm_dtype dtype, const void* h_vert, const void* W, const void* dg_facet, void* dh_vert, float* dW,
                     void* ws, size_t ws_bytes, void* stream);

/* facet2facet, Eq. 7:  g_f = 1/R_f sum_{p in f} sum_k sum_ci B_k(xi_p/|xi_p|) h_p[ci] W[k][ci][co].
 * tex_off [n_facet+1] is the facet -> texture-point CSR (points of a facet contiguous, R_f may be 0 ->
 * zero row); bary [n_tex,3] barycentric coordinates; h_tex [n_tex,cin]; g_facet [n_facet,cout].
 * With cin <= 4 and L <= 3 (the paper's shape: three colour channels) the sums are taken in the order
 * (mean over the points of a facet of B (x) h) . W, one contraction per facet; same result up to rounding. */
pm_status pm_f2f(int64_t n_facet, int64_t n_tex, const int32_t* tex_off, const float* bary, int L, pm_sh_norm norm,
                 int cin, int cout, pm_dtype dtype, const void* h_tex, const void* W, void* g_facet, void* ws,
                 size_t ws_bytes, void* stream);
/* Backward of Eq. 7.  dg_facet [n_facet,cout] -> dh_tex [n_tex,cin] (may be NULL), dW fp32 (may be NULL). */
pm_status pm_f2f_bwd(int64_t n_facet, int64_t n_tex, const int32_t* tex_off, const float* bary, int L,
                     pm_sh_norm norm, int cin, int cout, pm_dtype dtype, const void* h_tex, const void* W,
                     const void* dg_facet, void* dh_tex, float* dW, void* ws, size_t ws_bytes, void* stream);

/* Depth-wise separable form of facet2vertex and vertex2facet (Section "Mesh convolutions": Eq. 5 and Eq. 6
 * with one scalar SH coefficient set per channel, followed by a point-wise channel mixing):
 *   facet2vertex:  g_v = ( 1/|N(v)| sum_{f in N(v)} h_f (.) s(n_f) ) P,   s(d)[ci] = sum_k alpha[k][ci] B_k(d)
 *   vertex2facet:  g_f = ( sum_j h_{v_j(f)} (.) s(e_j) ) P
 * which is the dense form with W[k][ci][co] = alpha[k][ci] * P[ci][co].  alpha [K,cin] is always fp32; P [cin,cout]
 * has the feature dtype; dalpha [K,cin] and dP [cin,cout] are fp32.  Any of the three gradient outputs may be NULL
 * (dalpha and dP only together).  Same conventions as the dense entry points otherwise.
 * z_vert (facet2vertex forward, may be NULL) receives the vertex means before the point-wise matrix,
 * [n_vert,cin] of the feature dtype; handed back as z_saved (may be NULL) the backward pass takes dP from it
 * instead of recomputing it (two bandwidth-bound passes fewer; the results are the same bit for bit). */
pm_status pm_f2v_sep(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cout,
                     pm_dtype dtype, const void* h_facet, const float* alpha, const void* P, void* g_vert, void* z_vert,
                     void* ws, size_t ws_bytes, void* stream);
pm_status pm_f2v_sep_bwd(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cout,
                         pm_dtype dtype, const void* h_facet, const float* alpha, const void* P, const void* dg_vert,
                         const void* z_saved, void* dh_facet, float* dalpha, float* dP, void* ws, size_t ws_bytes,
                         void* stream);
pm_status pm_v2f_sep(const pm_mesh* mesh, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype,
                     const void* h_vert, const float* alpha, const void* P, void* g_facet, void* ws, size_t ws_bytes,
                     void* stream);
pm_status pm_v2f_sep_bwd(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cout,
                         pm_dtype dtype, const void* h_vert, const float* alpha, const void* P, const void* dg_facet,
                         void* dh_vert, float* dalpha, float* dP, void* ws, size_t ws_bytes, void* stream);

/* Separable vertex2vertex block (subsection "Angular Arguments in Different Convolutions", end of the vertex2facet
 * paragraph, and the figure of the four mesh convolutions: a vertex2facet convolution followed by a facet2vertex
 * convolution, normalisation on the facet and on the vertex features, ReLU as the activation):
 *   u_f = ( sum_j h_{v_j(f)} (.) s1(e_j) ) P1,                 g_f = act1(a1 (.) u_f + b1)          [n_facet,cmid]
 *   z_v = 1/|N(v)| sum_{f in N(v)} g_f (.) s2(n_f),            o_v = act2(a2 (.) (z_v P2) + b2)      [n_vert,cout]
 * with s1, s2 the per-channel SH filters of alpha1 [K,cin], alpha2 [K,cmid] (fp32) as in the separable entry
 * points above, P1 [cin,cmid], P2 [cmid,cout] of the feature dtype.  An epilogue is a per-channel affine map with
 * fixed coefficients (normalisation with frozen statistics; device fp32 vectors, either may be NULL = 1 / 0)
 * and an optional ReLU; a NULL pm_epilogue pointer means none.  For bf16 rows with cin in {32, 64} and cmid a
 * multiple of 32 up to 128 one kernel per facet tile gathers, contracts, applies the epilogue and the second
 * filter: the facet features g are not written (unless g_facet asks for them), only the filtered rows g (.) s2
 * pass through the workspace on their way to the vertex mean; other shapes run the same arithmetic through the
 * separable entry points' kernels.
 * g_facet [n_facet,cmid] and z_vert [n_vert,cmid] (both optional, feature dtype) receive the activated facet
 * features and the vertex means: the backward pass needs both (g_saved, z_saved) and, when act2 is a ReLU, the
 * output rows (out_saved).  It returns dh_vert [n_vert,cin] (feature dtype), dalpha1 [K,cin], dP1 [cin,cmid],
 * dalpha2 [K,cmid], dP2 [cmid,cout] (fp32) for fixed affine coefficients; any may be NULL (dalpha_i and dP_i only
 * together).  Workspace from pm_v2v_sep_ws_bytes (0 on invalid arguments). */
typedef struct pm_epilogue {
  const float* scale;   /* [C] or NULL */
  const float* shift;   /* [C] or NULL */
  int relu;             /* 0 / 1 */
} pm_epilogue;
size_t pm_v2v_sep_ws_bytes(int backward, int64_t n_vert, int64_t n_facet, int L, int cin, int cmid, int cout,
                           pm_dtype dtype);
pm_status pm_v2v_sep(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cmid, int cout,
                     pm_dtype dtype, const void* h_vert, const float* alpha1, const void* P1, const pm_epilogue* ep1,
                     const float* alpha2, const void* P2, const pm_epilogue* ep2, void* out_vert, void* g_facet,
                     void* z_vert, void* ws, size_t ws_bytes, void* stream);
pm_status pm_v2v_sep_bwd(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cmid,
                         int cout, pm_dtype dtype, const void* h_vert, const float* alpha1, const void* P1,
                         const pm_epilogue* ep1, const float* alpha2, const void* P2, const pm_epilogue* ep2,
                         const void* g_saved, const void* z_saved, const void* out_saved, const void* d_out,
                         void* dh_vert, float* dalpha1, float* dP1, float* dalpha2, float* dP2, void* ws,
                         size_t ws_bytes, void* stream);

/* ---- Mesh pooling / unpooling (Section "Mesh decimation", paragraph "(Un)poolings") --------------------
 * A decimation hands over two int32 vectors of the INPUT mesh's vertex count n_in: VCluster and IOmap.
 * Encoding taken here (the paper gives none): vcluster[v] = input-mesh index of the representative vertex of
 * v's cluster; iomap[u] = output-mesh index (0 <= . < n_out) of input vertex u when it is a representative,
 * else -1.  The output vertex of v is target[v] = iomap[vcluster[v]]; -1 = v reaches no output vertex.
 * Features are rows [n_in][C] (input mesh) and [n_out][C] (output mesh) of `dtype`, C >= 1.
 *
 * pm_build_cluster_map fills the three arrays every pooling call reads: target [n_in], row_ptr [n_out+1] and
 * col [n_in] (the members of each output vertex, ascending; the first row_ptr[n_out] entries are used).
 * An id outside its range is treated as -1, never dereferenced.  ws: pm_cluster_ws_bytes(n_in, n_out).
 * pm_validate_clusters counts such ids and returns PM_ERR_BAD_MESH if there are any (synchronises;
 * ws >= pm_cluster_ws_bytes(n_in, n_out)).  A pm_cluster_map not made by pm_build_cluster_map is undefined
 * behaviour in the calls below. */
typedef struct pm_cluster_map {
  int64_t n_in, n_out;
  const int32_t* target;  /* [n_in]    */
  const int32_t* row_ptr; /* [n_out+1] */
  const int32_t* col;     /* [n_in]    */
} pm_cluster_map;
typedef enum { PM_POOL_MAX = 0, PM_POOL_AVG = 1 } pm_pool_mode;

size_t pm_cluster_ws_bytes(int64_t n_in, int64_t n_out); /* HOST computation; 0 on invalid sizes */
pm_status pm_validate_clusters(int64_t n_in, int64_t n_out, const int32_t* vcluster, const int32_t* iomap, void* ws,
                               size_t ws_bytes, void* stream);
pm_status pm_build_cluster_map(int64_t n_in, int64_t n_out, const int32_t* vcluster, const int32_t* iomap,
                               int32_t* target, int32_t* row_ptr, int32_t* col, void* ws, size_t ws_bytes,
                               void* stream);

/* h_out[o] = max / average of h_in[v] over the members v of o; an output vertex without members gets 0.
 * PM_POOL_MAX: argmax (int32 [n_out][C], may be NULL) receives the input vertex each maximum came from
 * (ties: the lowest index; -1 for no members); NaN features are not supported.  Averages accumulate in fp32
 * in ascending member order. */
pm_status pm_pool(const pm_cluster_map* cm, pm_pool_mode mode, int C, pm_dtype dtype, const void* h_in, void* h_out,
                  int32_t* argmax, void* stream);
/* dh_in [n_in][C]: average: dg_out[target[v]] / |cluster|; maximum: dg_out[t][c] where argmax[t][c] == v, else 0
 * (argmax from pm_pool, required for PM_POOL_MAX, ignored for PM_POOL_AVG).  Rows with no output vertex are 0. */
pm_status pm_pool_bwd(const pm_cluster_map* cm, pm_pool_mode mode, int C, pm_dtype dtype, const void* dg_out,
                      const int32_t* argmax, void* dh_in, void* stream);
/* h_fine[v] = h_coarse[target[v]] (0 where there is none): every member replicates its output vertex. */
pm_status pm_unpool(const pm_cluster_map* cm, int C, pm_dtype dtype, const void* h_coarse, void* h_fine, void* stream);
/* dh_coarse[o] = sum of dg_fine[v] over the members of o, ascending, fp32 accumulation. */
pm_status pm_unpool_bwd(const pm_cluster_map* cm, int C, pm_dtype dtype, const void* dg_fine, void* dh_coarse,
                        void* stream);

/* ---- Point-cloud convolution with the radial term (subsection "Extension to Point Cloud Convolution") ----
 * F(theta, phi, r) = F(theta, phi) Z(r) + c0 (1 - Z(r)), Z(r) = r / rho, depth-wise separable.  For query point i
 * with the neighbours q_e (lists supplied by the caller; the range search is not part of this library):
 *   delta_e = xs[q_e] - xq[i], r_e = |delta_e|, Z_e = min(r_e / rho, 1), direction delta_e / r_e,
 *   s_e[c] = Z_e sum_k alpha[k][c] B_k(direction_e) + c0[c] (1 - Z_e),
 *   y_i[c] = 1/|N(i)| sum_e s_e[c] h[q_e][c]   (0 for an empty list),        g_i = y_i P.
 * xq [n_query][3], xs [n_source][3] fp32 (they may be the same array); ptr [n_query+1] and idx [nnz] int32 with
 * ptr[0] = 0, ptr non-decreasing, ptr[n_query] = nnz, 0 <= idx < n_source; rho > 0.  alpha [K][cin] and c0 [cin]
 * are fp32 (K + 1 numbers per channel), P [cin][cout] has the feature dtype; h [n_source][cin],
 * g [n_query][cout].  An id outside its range is clamped, never followed; pm_validate_neighbors reports bad
 * lists (synchronises; ws >= 16 bytes).  ws: pm_pcloud_ws_bytes(backward?, ...).
 * The backward pass sums over the reverse lists (the pairs of every source point, sorted).  It builds them in
 * its workspace on every call unless the caller built them once with pm_build_reverse_neighbors and set
 * rev_ptr [n_source+1], rev_col [nnz] (pair ids) and owner [nnz] (query of every pair): all three or none.
 * y_query (forward, may be NULL) receives the depth-wise output y [n_query,cin] of the feature dtype; handed
 * back as y_saved (may be NULL) the backward pass takes dP from it instead of recomputing it.
 * Arithmetic: basis and filter values in fp32, sums over a list in fp32 in list order.  With bf16 features and
 * L <= 4 the filter sum_k runs on the bf16 matrix cores with both operands split into a bf16 head and remainder
 * (three products, fp32 accumulation: relative error below 2^-15 per product, i.e. fp32 to within the stated
 * bar); the coefficient gradients dalpha, dc0 then sum bf16-rounded products h (.) dy in fp32. */
typedef struct pm_nbr {
  int64_t n_query, n_source, nnz;
  const float* xq;
  const float* xs;
  const int32_t* ptr;
  const int32_t* idx;
  float rho;
  const int32_t* rev_ptr; /* optional, see above */
  const int32_t* rev_col;
  const int32_t* owner;
} pm_nbr;
size_t pm_reverse_ws_bytes(int64_t n_source, int64_t nnz); /* HOST computation; 0 on invalid sizes */
pm_status pm_build_reverse_neighbors(const pm_nbr* nb, int32_t* rev_ptr, int32_t* rev_col, int32_t* owner, void* ws,
                                     size_t ws_bytes, void* stream);
size_t pm_pcloud_ws_bytes(int backward, int64_t n_query, int64_t n_source, int64_t nnz, int L, int cin, int cout,
                          pm_dtype dtype); /* HOST computation; 0 on invalid arguments */
pm_status pm_validate_neighbors(const pm_nbr* nb, void* ws, size_t ws_bytes, void* stream);
pm_status pm_pcloud_conv(const pm_nbr* nb, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype, const void* h,
                         const float* alpha, const float* c0, const void* P, void* g, void* y_query, void* ws,
                         size_t ws_bytes, void* stream);
/* dh [n_source][cin] (feature dtype; may be NULL); dalpha [K][cin], dc0 [cin], dP [cin][cout] fp32 (all three
 * or none).  Sums run in a fixed order over the caller's lists and over the reverse lists built here (sorted),
 * no float atomics. */
pm_status pm_pcloud_conv_bwd(const pm_nbr* nb, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype,
                             const void* h, const float* alpha, const float* c0, const void* P, const void* dg,
                             const void* y_saved, void* dh, float* dalpha, float* dc0, float* dP, void* ws,
                             size_t ws_bytes, void* stream);

/* ---- Input preparation ------------------------------------------------------------------------------
 * Facet geometric features (Section "Geometric Features", Eq. 9): feat [n_facet][9 or 12] of `dtype`, row
 * layout [l1 l2 l3, theta1 theta2 theta3, nx ny nz, (z1 z2 z3)] with l1 = |x2-x1|, l2 = |x3-x2|, l3 = |x1-x3|,
 * theta_i the normalised inner product of the two edges at corner i (the cosine of the inner angle; 0 when an
 * edge has zero length), n the unit normal of the stored corner order ((0,0,1) for a degenerate facet) and,
 * when with_heights != 0, the z coordinates of the three corners. */
pm_status pm_facet_geometry(const pm_mesh* mesh, int with_heights, pm_dtype dtype, void* feat, void* stream);

/* Texture resolution of every facet (Eq. 8): gamma[f] = floor(alpha (A_f - Amin)/(Amax - Amin)) + beta with the
 * extreme areas of the facet's own mesh (mesh->facet_off is required when n_mesh > 1; equal extremes give
 * beta), evaluated in fp32 one IEEE operation at a time in a fixed order, and tex_off [n_facet+1] = running
 * sum of the point counts (gamma+1)(gamma+2)/2.  0 <= alpha, beta, alpha + beta <= 255 and
 * n_facet (alpha+beta+1)(alpha+beta+2)/2 < 2^31 (the bound on the total, checked).  ws: pm_texture_ws_bytes(n_facet, n_mesh).  The caller reads tex_off[n_facet]
 * back to size the point arrays. */
size_t pm_texture_ws_bytes(int64_t n_facet, int32_t n_mesh); /* HOST computation; 0 on invalid sizes */
pm_status pm_texture_layout(const pm_mesh* mesh, int alpha, int beta, int32_t* gamma, int32_t* tex_off, void* ws,
                            size_t ws_bytes, void* stream);
/* Barycentric interpolation points of every facet, bary [n_tex][3] fp32 (the layout pm_f2f reads): the lattice
 * (i, j, gamma-i-j)/gamma, i descending then j descending, the centroid for gamma = 0.  Points at or past
 * n_tex are not written. */
pm_status pm_texture_bary(int64_t n_facet, const int32_t* gamma, const int32_t* tex_off, int64_t n_tex, float* bary,
                          void* stream);

/* Measurement aid (not part of the method): per-kernel timing with HIP events.
 * After pm_profile_enable(1) every kernel this thread's calls launch is bracketed by a pair of events
 * recorded on the call's stream (events are created on demand and reused; nothing else changes).
 * pm_profile_count() is the number of records since the last reset; pm_profile_read(i, ...) waits for
 * record i's stop event and returns its label ("<entry point>/<kernel>", truncated to name_cap-1
 * characters) and its duration in milliseconds.  pm_profile_reset() drops the records (keeps the events).
 * pm_profile_filter(part) limits the records to kernels whose label contains `part` (NULL or "" = all): a pair
 * of events costs the stream a few microseconds, so a timed loop brackets only the kernel it asks about. */
pm_status pm_profile_enable(int on);
pm_status pm_profile_filter(const char* label_part);
int32_t pm_profile_count(void);
pm_status pm_profile_read(int32_t i, char* name, size_t name_cap, float* ms);
pm_status pm_profile_reset(void);

/* Measurement aid (not part of the method): rates this device sustains in short issue loops, to quote beside
 * the published peaks.  The bf16 matrix loop exists with all-ones operands and with random signs and
 * mantissas: the shader clock is power-managed, so the rate depends on the data.  `ws` is device memory
 * the probe may overwrite (16-byte aligned, >= 1 MiB; the copy probe moves half of it to the other half,
 * so give it a few hundred MiB to measure HBM rather than the caches).  *value receives TFLOP/s (matrix
 * probes) or GB/s read+written (copy); *clock_mhz (may be NULL) the shader clock observed inside the probe
 * kernel.  The call synchronises `stream`; it allocates no device memory. */
typedef enum {
  PM_PEAK_MFMA_BF16_ONES = 0,
  PM_PEAK_MFMA_BF16_RANDOM = 1,
  PM_PEAK_MFMA_F32 = 2,
  PM_PEAK_HBM_COPY = 3
} pm_peak_kind;
pm_status pm_peak_probe(pm_peak_kind kind, void* ws, size_t ws_bytes, double* value, double* clock_mhz, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PICASSOMESH_H */
