// C ABI of picassomesh: argument checks, workspace carving, kernel sequencing.  See include/picassomesh.h.
#include <stdarg.h>
#include <stdio.h>

#include <string.h>

#include <map>
#include <mutex>
#include <utility>
#include <vector>

#include <algorithm>

#include "pm_host.h"

static thread_local char g_err[512] = "";

pm_status pm_fail(pm_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return s;
}

extern "C" const char* pm_last_error(void) { return g_err; }

// The dynamic-LDS limit of a kernel is a property of the loaded code object on a device: set it when a
// (kernel, device) pair is first launched with a given size, remember that, and skip the runtime call afterwards.
pm_status pm_set_dyn_lds(const void* kernel, size_t bytes) {
  static std::mutex mu;
  static std::map<std::pair<const void*, int>, size_t> done;
  int dev = 0;
  PM_CHECK_HIP(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(mu);
  auto it = done.find({kernel, dev});
  if (it != done.end() && it->second == bytes) return PM_OK;
  PM_CHECK_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  done[{kernel, dev}] = bytes;
  return PM_OK;
}

// ---- per-kernel event timing ------------------------------------------------------------------
struct ProfRec {
  char name[64];
  hipEvent_t start, stop;
};
static thread_local bool g_prof_on = false;
static thread_local const char* g_prof_op = "";
static thread_local std::vector<ProfRec> g_prof_recs;
static thread_local std::vector<hipEvent_t> g_prof_pool;
static thread_local bool g_prof_open = false;
static thread_local char g_prof_filter[64] = "";

static hipEvent_t prof_event() {
  if (!g_prof_pool.empty()) {
    hipEvent_t e = g_prof_pool.back();
    g_prof_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

void pm_prof_set_op(const char* op) { g_prof_op = op; }

void pm_prof_begin(hipStream_t st, const char* kernel) {
  g_prof_open = false;
  if (!g_prof_on) return;
  ProfRec r;
  snprintf(r.name, sizeof(r.name), "%s/%s", g_prof_op, kernel);
  if (g_prof_filter[0] && !strstr(r.name, g_prof_filter)) return;
  r.start = prof_event();
  r.stop = prof_event();
  if (!r.start || !r.stop) return;
  if (hipEventRecord(r.start, st) != hipSuccess) return;
  g_prof_recs.push_back(r);
  g_prof_open = true;
}

void pm_prof_end(hipStream_t st) {
  if (!g_prof_open) return;
  (void)hipEventRecord(g_prof_recs.back().stop, st);
  g_prof_open = false;
}

extern "C" pm_status pm_profile_enable(int on) {
  g_prof_on = on != 0;
  return PM_OK;
}
extern "C" pm_status pm_profile_filter(const char* label_part) {
  if (!label_part) label_part = "";
  strncpy(g_prof_filter, label_part, sizeof(g_prof_filter) - 1);
  g_prof_filter[sizeof(g_prof_filter) - 1] = 0;
  return PM_OK;
}
extern "C" int32_t pm_profile_count(void) { return (int32_t)g_prof_recs.size(); }
extern "C" pm_status pm_profile_read(int32_t i, char* name, size_t name_cap, float* ms) {
  if (i < 0 || i >= (int32_t)g_prof_recs.size() || !ms) return pm_fail(PM_ERR_INVALID_ARG, "profile record %d", i);
  ProfRec& r = g_prof_recs[i];
  PM_CHECK_HIP(hipEventSynchronize(r.stop));
  PM_CHECK_HIP(hipEventElapsedTime(ms, r.start, r.stop));
  if (name && name_cap) {
    strncpy(name, r.name, name_cap - 1);
    name[name_cap - 1] = 0;
  }
  return PM_OK;
}
extern "C" pm_status pm_profile_reset(void) {
  for (auto& r : g_prof_recs) {
    g_prof_pool.push_back(r.start);
    g_prof_pool.push_back(r.stop);
  }
  g_prof_recs.clear();
  return PM_OK;
}

extern "C" const char* pm_status_string(pm_status s) {
  switch (s) {
    case PM_OK: return "PM_OK";
    case PM_ERR_INVALID_ARG: return "PM_ERR_INVALID_ARG";
    case PM_ERR_UNSUPPORTED: return "PM_ERR_UNSUPPORTED";
    case PM_ERR_WORKSPACE: return "PM_ERR_WORKSPACE";
    case PM_ERR_HIP: return "PM_ERR_HIP";
    case PM_ERR_BAD_MESH: return "PM_ERR_BAD_MESH";
    default: return "PM_ERR_UNKNOWN";
  }
}

static const int64_t kMaxIds = 2147483647LL;

static pm_status check_conv_common(int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype) {
  if (L < 0 || L > PM_MAX_L) return pm_fail(PM_ERR_UNSUPPORTED, "SH degree L=%d outside [0,%d]", L, PM_MAX_L);
  if (norm != PM_SH_PAPER && norm != PM_SH_ORTHONORMAL) return pm_fail(PM_ERR_UNSUPPORTED, "unknown pm_sh_norm %d", (int)norm);
  if (dtype != PM_F32 && dtype != PM_BF16) return pm_fail(PM_ERR_UNSUPPORTED, "unknown pm_dtype %d", (int)dtype);
  if (cin < 1 || cout < 1 || cin > 65536 || cout > 65536) return pm_fail(PM_ERR_INVALID_ARG, "cin=%d cout=%d", cin, cout);
  return PM_OK;
}

static pm_status check_mesh(const pm_mesh* m, bool need_vert) {
  if (!m) return pm_fail(PM_ERR_INVALID_ARG, "mesh is NULL");
  if (m->n_vert < 0 || m->n_facet < 0 || m->n_mesh < 0) return pm_fail(PM_ERR_INVALID_ARG, "negative mesh size");
  if (m->n_vert >= kMaxIds || 3 * m->n_facet >= kMaxIds) return pm_fail(PM_ERR_INVALID_ARG, "mesh exceeds int32 ids");
  if (m->n_facet > 0 && !m->facet) return pm_fail(PM_ERR_INVALID_ARG, "mesh->facet is NULL");
  if (need_vert && m->n_vert > 0 && !m->vert) return pm_fail(PM_ERR_INVALID_ARG, "mesh->vert is NULL");
  return PM_OK;
}

static pm_status check_ptr(const void* p, const char* name, bool required) {
  if (!p) return required ? pm_fail(PM_ERR_INVALID_ARG, "%s is NULL", name) : (pm_status)PM_OK;
  if (!pm_aligned16(p)) return pm_fail(PM_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
  return PM_OK;
}

static size_t esize(pm_dtype d) { return d == PM_BF16 ? 2 : 4; }

// workspace layouts ------------------------------------------------------------------------------
struct WsPlan {
  size_t apack, inter, owner, small, wgrad, total;
};

static WsPlan plan_ws(pm_op op, int64_t V, int64_t F, int64_t P, int L, int cin, int cout, pm_dtype dt) {
  (void)V;
  const int K = (L + 1) * (L + 1);
  WsPlan w = {0, 0, 0, 0, 0, 0};
  switch (op) {
    case PM_OP_ADJACENCY: w.small = pm_adj_ws_bytes(V, F); break;
    case PM_OP_F2V:
      w.apack = pm_pack_bytes(pm_pack_geom(K, cin, cout, dt));
      w.inter = pm_round_up((size_t)F * cout * esize(dt), 256);   // per-facet summands, feature dtype
      break;
    case PM_OP_F2V_BWD:
      w.apack = pm_pack_bytes(pm_pack_geom(K, cout, cin, dt));
      // basis rows for the general weight-gradient kernel, or the gathered gradient rows dy (bf16) that the
      // producer/consumer kernel hands to the backward-data pass
      w.inter = pm_round_up(std::max((size_t)F * K * 4, (size_t)F * cout * 2), 256);
      w.wgrad = pm_wgrad_ws_bytes(F, K, cin, cout);
      break;
    case PM_OP_V2F:
      w.apack = pm_pack_bytes(pm_pack_geom(1, 3 * cin, cout, dt));
      break;
    case PM_OP_V2F_BWD:
      w.apack = pm_pack_bytes(pm_pack_geom(1, 3 * cout, cin, dt));
      w.inter = pm_round_up((size_t)V * 3 * cout * esize(dt), 256);   // per-vertex corner-slot sums of dg
      w.small = pm_round_up((size_t)3 * cin * cout * 4, 256);
      w.wgrad = pm_wgrad_ws_bytes(F, 3, cin, cout);
      break;
    case PM_OP_F2V_SEP:
      w.apack = pm_pack_bytes(pm_pack_geom(1, cin, cout, dt));
      w.inter = pm_round_up((size_t)F * cin * esize(dt), 256);     // depth-wise facet rows y
      w.owner = pm_round_up((size_t)V * cin * esize(dt), 256);     // their vertex means z
      break;
    case PM_OP_F2V_SEP_BWD:
      w.apack = pm_pack_bytes(pm_pack_geom(1, cout, cin, dt));
      w.inter = pm_round_up((size_t)F * cin * esize(dt), 256);     // y (for dP)
      w.owner = pm_round_up((size_t)V * cin * esize(dt), 256);     // z (for dP), then reused never: dz has its own
      w.small = pm_round_up((size_t)V * cin * 4, 256);             // dz = dg P^T, kept in fp32
      w.wgrad = std::max(pm_wgrad_ws_bytes(V, 1, cin, cout), pm_sep_dalpha_ws_bytes(F, K, cin, dt == PM_BF16));
      break;
    case PM_OP_V2F_SEP:
      w.apack = pm_pack_bytes(pm_pack_geom(1, 3 * cin, cout, dt));
      break;
    case PM_OP_V2F_SEP_BWD:
      w.apack = pm_pack_bytes(pm_pack_geom(1, cout, cin, dt));
      w.inter = pm_round_up((size_t)F * cin * esize(dt), 256);        // T_f = dg_f P^T
      w.small = pm_round_up((size_t)3 * cin * cout * 4, 256) + pm_round_up((size_t)3 * cin * 4, 256);   // M, corner scales
      w.wgrad = pm_wgrad_ws_bytes(F, 3, cin, cout);
      break;
    case PM_OP_F2F:
      if (pm_f2f_small_applies(L, cin)) {   // few input channels: one staged 64-channel row per facet
        w.apack = pm_pack_bytes(pm_pack_geom(1, dt == PM_BF16 ? 128 : K * cin, cout, dt));
        w.inter = pm_round_up((size_t)F * 256, 256);   // 64 fp32 channels, or a bf16 head and remainder of 64 each
        break;
      }
      w.apack = pm_pack_bytes(pm_pack_geom(K, cin, cout, dt));
      w.inter = pm_round_up((size_t)P * cout * esize(dt), 256);   // per-point summands, feature dtype
      break;
    case PM_OP_F2F_BWD:
      if (pm_f2f_small_applies(L, cin)) {
        w.apack = pm_pack_bytes(pm_pack_geom(1, cout, K * cin, dt));
        w.owner = pm_round_up((size_t)(P + 1) * 4, 256);
        w.inter = pm_round_up((size_t)F * 256, 256);                  // staged rows S_f
        w.small = pm_round_up((size_t)F * K * cin * 4, 256);           // T_f = W dg_f, fp32
        w.wgrad = pm_wgrad_ws_bytes(F, 1, K * cin, cout);
        break;
      }
      w.apack = pm_pack_bytes(pm_pack_geom(K, cout, cin, dt));
      w.owner = pm_round_up((size_t)(P + 1) * 4, 256);
      w.inter = pm_round_up((size_t)P * K * 4, 256);   // basis rows for the weight gradient
      w.wgrad = pm_wgrad_ws_bytes(P, K, cin, cout);
      break;
  }
  w.total = w.apack + w.inter + w.owner + w.small + w.wgrad;
  if (w.total == 0) w.total = 256;
  return w;
}

extern "C" size_t pm_workspace_bytes(pm_op op, int64_t n_vert, int64_t n_facet, int64_t n_tex, int L, int cin, int cout,
                                     pm_dtype dtype) {
  if (op < PM_OP_ADJACENCY || op > PM_OP_V2F_SEP_BWD) return 0;
  if (n_vert < 0 || n_facet < 0 || n_tex < 0) return 0;
  if (op != PM_OP_ADJACENCY && check_conv_common(L, PM_SH_PAPER, cin, cout, dtype) != PM_OK) return 0;
  if (op == PM_OP_ADJACENCY) { L = 0; cin = cout = 1; dtype = PM_F32; }
  return plan_ws(op, n_vert, n_facet, n_tex, L, cin, cout, dtype).total;
}

static pm_status check_ws(const WsPlan& w, void* ws, size_t ws_bytes) {
  PM_TRY(check_ptr(ws, "ws", true));
  if (ws_bytes < w.total) return pm_fail(PM_ERR_WORKSPACE, "workspace %zu < required %zu bytes", ws_bytes, w.total);
  return PM_OK;
}

// ---- mesh utilities ----------------------------------------------------------------------------
extern "C" pm_status pm_validate_mesh(const pm_mesh* mesh, void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("validate");
  PM_TRY(check_mesh(mesh, false));
  PM_TRY(check_ptr(ws, "ws", true));
  if (ws_bytes < 16) return pm_fail(PM_ERR_WORKSPACE, "validate needs 16 bytes of workspace");
  if (mesh->n_mesh > 1 && (!mesh->vert_off || !mesh->facet_off))
    return pm_fail(PM_ERR_INVALID_ARG, "n_mesh > 1 needs vert_off and facet_off");
  hipStream_t st = (hipStream_t)stream;
  PM_TRY(pm_launch_validate(mesh, (int32_t*)ws, st));
  int32_t flag = 0;
  PM_CHECK_HIP(hipMemcpyAsync(&flag, ws, sizeof(flag), hipMemcpyDeviceToHost, st));
  PM_CHECK_HIP(hipStreamSynchronize(st));
  if (flag & 2) return pm_fail(PM_ERR_BAD_MESH, "offset arrays are not monotone or do not span the batch");
  if (flag & 1) return pm_fail(PM_ERR_BAD_MESH, "a facet references a vertex outside its mesh");
  return PM_OK;
}

extern "C" pm_status pm_build_vf_adjacency(const pm_mesh* mesh, int32_t* row_ptr, int32_t* col, void* ws,
                                           size_t ws_bytes, void* stream) {
  pm_prof_set_op("adjacency");
  PM_TRY(check_mesh(mesh, false));
  if (!row_ptr || (mesh->n_facet > 0 && !col)) return pm_fail(PM_ERR_INVALID_ARG, "row_ptr / col is NULL");
  WsPlan w = plan_ws(PM_OP_ADJACENCY, mesh->n_vert, mesh->n_facet, 0, 0, 1, 1, PM_F32);
  PM_TRY(check_ws(w, ws, ws_bytes));
  return pm_launch_adjacency(mesh, row_ptr, col, ws, (hipStream_t)stream);
}

// ---- basis -------------------------------------------------------------------------------------
extern "C" pm_status pm_sh_basis(const pm_mesh* mesh, int L, pm_sh_norm norm, float* basis, void* stream) {
  pm_prof_set_op("sh_basis");
  PM_TRY(check_conv_common(L, norm, 1, 1, PM_F32));
  PM_TRY(check_mesh(mesh, true));
  if (mesh->n_facet > 0 && !basis) return pm_fail(PM_ERR_INVALID_ARG, "basis is NULL");
  ShTable T;
  pm_make_sh_table(L, norm, &T);
  return pm_launch_basis_mesh(mesh, T, basis, (hipStream_t)stream);
}

extern "C" pm_status pm_sh_basis_dirs(int64_t n, const float* dirs, int L, pm_sh_norm norm, float* basis, void* stream) {
  pm_prof_set_op("sh_basis_dirs");
  PM_TRY(check_conv_common(L, norm, 1, 1, PM_F32));
  if (n < 0 || n >= kMaxIds) return pm_fail(PM_ERR_INVALID_ARG, "n=%lld", (long long)n);
  if (n > 0 && (!dirs || !basis)) return pm_fail(PM_ERR_INVALID_ARG, "dirs / basis is NULL");
  ShTable T;
  pm_make_sh_table(L, norm, &T);
  return pm_launch_basis_dirs(n, dirs, T, basis, (hipStream_t)stream);
}

extern "C" pm_status pm_sh_basis_bwd(int64_t n, const float* dirs, int L, pm_sh_norm norm, const float* dbasis,
                                     float* ddirs, void* stream) {
  pm_prof_set_op("sh_basis_bwd");
  PM_TRY(check_conv_common(L, norm, 1, 1, PM_F32));
  if (n < 0 || n >= kMaxIds) return pm_fail(PM_ERR_INVALID_ARG, "n=%lld", (long long)n);
  if (n > 0 && (!dirs || !dbasis || !ddirs)) return pm_fail(PM_ERR_INVALID_ARG, "dirs / dbasis / ddirs is NULL");
  ShTable T;
  pm_make_sh_table(L, norm, &T);
  return pm_launch_basis_bwd(n, dirs, T, dbasis, ddirs, (hipStream_t)stream);
}

// ---- helpers to describe operand rows ------------------------------------------------------------
static RowSrc row_src(const void* p, pm_dtype dt, int C) {
  RowSrc s;
  s.p = p; s.is_bf16 = (dt == PM_BF16); s.C = C;
  s.facet = nullptr; s.row_ptr = nullptr; s.owner = nullptr; s.seg_off = nullptr;
  return s;
}
static BasisSrc basis_none() {
  BasisSrc b;
  b.vert = nullptr; b.facet = nullptr; b.dirs = nullptr; b.bvals = nullptr; b.owner = nullptr; b.seg_off = nullptr;
  pm_make_sh_table(0, PM_SH_PAPER, &b.sh);
  return b;
}
static void fold_coef(int L, pm_sh_norm norm, FoldCoef* fc) {
  double Bc[3][PM_MAX_K];
  pm_corner_basis(L, norm, Bc);
  const int K = (L + 1) * (L + 1);
  for (int j = 0; j < 3; ++j)
    for (int k = 0; k < PM_MAX_K; ++k) fc->c[j][k] = (k < K) ? (float)Bc[j][k] : 0.f;
}

// ---- facet2vertex (Eq. 5) ------------------------------------------------------------------------
extern "C" pm_status pm_f2v(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cout,
                            pm_dtype dtype, const void* h_facet, const void* W, void* g_vert, void* ws, size_t ws_bytes,
                            void* stream) {
  pm_prof_set_op("f2v");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_mesh(mesh, true));
  if (!adj || !adj->row_ptr || (mesh->n_facet > 0 && !adj->col)) return pm_fail(PM_ERR_INVALID_ARG, "adjacency is NULL");
  PM_TRY(check_ptr(W, "W", true));
  PM_TRY(check_ptr(h_facet, "h_facet", mesh->n_facet > 0));
  PM_TRY(check_ptr(g_vert, "g_vert", mesh->n_vert > 0));
  const int K = (L + 1) * (L + 1);
  const int64_t V = mesh->n_vert, F = mesh->n_facet;
  WsPlan w = plan_ws(PM_OP_F2V, V, F, 0, L, cin, cout, dtype);
  PM_TRY(check_ws(w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  void* y = apack + w.apack;   // per-facet summands of Eq. 5 in the feature dtype (summed in fp32 below)

  PM_TRY(pm_launch_pack(PACK_PLAIN, dtype, K, cin, cout, W, nullptr, apack, st));
  BasisSrc bs = basis_none();
  bs.vert = mesh->vert; bs.facet = mesh->facet;
  pm_make_sh_table(L, norm, &bs.sh);
  RowSrc xs = row_src(h_facet, dtype, cin);
  const int yb = dtype == PM_BF16;
  PM_TRY(pm_launch_conv_rows(dtype, B_NORMAL, X_DIRECT, F, K, cin, cout, bs, xs, apack, y, yb, st));
  return pm_launch_segreduce(V, cout, y, yb, adj->row_ptr, adj->col, 3, 1, g_vert, dtype == PM_BF16, st);
}

extern "C" pm_status pm_f2v_bwd(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cout,
                                pm_dtype dtype, const void* h_facet, const void* W, const void* dg_vert, void* dh_facet,
                                float* dW, void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("f2v_bwd");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_mesh(mesh, true));
  if (!adj || !adj->row_ptr) return pm_fail(PM_ERR_INVALID_ARG, "adjacency is NULL");
  PM_TRY(check_ptr(W, "W", true));
  PM_TRY(check_ptr(h_facet, "h_facet", mesh->n_facet > 0));
  PM_TRY(check_ptr(dg_vert, "dg_vert", mesh->n_vert > 0));
  PM_TRY(check_ptr(dh_facet, "dh_facet", false));
  PM_TRY(check_ptr(dW, "dW", false));
  const int K = (L + 1) * (L + 1);
  const int64_t V = mesh->n_vert, F = mesh->n_facet;
  WsPlan w = plan_ws(PM_OP_F2V_BWD, V, F, 0, L, cin, cout, dtype);
  PM_TRY(check_ws(w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  float* bvals = (float*)(apack + w.apack);
  void* wg = (char*)bvals + w.inter;

  BasisSrc bs = basis_none();
  bs.vert = mesh->vert; bs.facet = mesh->facet;
  pm_make_sh_table(L, norm, &bs.sh);
  RowSrc dys = row_src(dg_vert, dtype, cout);   // dy_f = sum_j dg[v_j] / deg(v_j)
  dys.facet = mesh->facet; dys.row_ptr = adj->row_ptr;
  RowSrc xs = row_src(h_facet, dtype, cin);
  // With both gradients wanted and the producer/consumer weight-gradient kernel applicable, that kernel runs
  // first and leaves the gathered rows dy (bf16: the very operand precision of the backward-data pass)
  // in the workspace, so the backward-data pass reads plain rows.
  const bool pc = dW && pm_wgrad_fuses_basis(dtype, B_NORMAL, X_DIRECT, X_GATHER_SUM, K, cin, cout, xs, dys);
  void* dy = (pc && dh_facet) ? (void*)bvals : nullptr;
  if (dW) {
    if (!pc) {
      PM_TRY(pm_launch_basis_mesh(mesh, bs.sh, bvals, st));
      bs.bvals = bvals;
    }
    PM_TRY(pm_launch_wgrad(dtype, B_NORMAL, X_DIRECT, X_GATHER_SUM, F, K, cin, cout, bs, xs, dys, dW, wg, w.wgrad, dy, st));
  }
  if (dh_facet) {
    PM_TRY(pm_launch_pack(PACK_TRANS, dtype, K, cin, cout, W, nullptr, apack, st));
    if (dy) {
      RowSrc dyr = row_src(dy, PM_BF16, cout);
      PM_TRY(pm_launch_conv_rows(dtype, B_NORMAL, X_DIRECT, F, K, cout, cin, bs, dyr, apack, dh_facet, dtype == PM_BF16, st));
    } else {
      PM_TRY(pm_launch_conv_rows(dtype, B_NORMAL, X_GATHER_SUM, F, K, cout, cin, bs, dys, apack, dh_facet,
                                 dtype == PM_BF16, st));
    }
  }
  return PM_OK;
}

// ---- vertex2facet (Eq. 6) ------------------------------------------------------------------------
extern "C" pm_status pm_v2f(const pm_mesh* mesh, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype,
                            const void* h_vert, const void* W, void* g_facet, void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("v2f");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_mesh(mesh, false));
  PM_TRY(check_ptr(W, "W", true));
  PM_TRY(check_ptr(h_vert, "h_vert", mesh->n_vert > 0));
  PM_TRY(check_ptr(g_facet, "g_facet", mesh->n_facet > 0));
  const int K = (L + 1) * (L + 1);
  const int64_t V = mesh->n_vert, F = mesh->n_facet;
  WsPlan w = plan_ws(PM_OP_V2F, V, F, 0, L, cin, cout, dtype);
  PM_TRY(check_ws(w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  FoldCoef fc;
  fold_coef(L, norm, &fc);
  // the three corner directions are constants => three folded cin x cout matrices W_j = sum_k B_k(e_j) W[k]
  PM_TRY(pm_launch_pack(PACK_FOLD, dtype, K, cin, cout, W, &fc, ws, st));
  if (pm_v2f_stage_applies(dtype, cin, cout, h_vert, g_facet))       // the memory-bound shape: LDS-staged facet tiles
    return pm_launch_v2f_stage(F, cin, cout, mesh->facet, h_vert, ws, g_facet, st);
  RowSrc xs = row_src(h_vert, dtype, cin);
  xs.facet = mesh->facet;
  return pm_launch_conv_rows(dtype, B_ONE, X_GATHER_CAT, F, 1, 3 * cin, cout, basis_none(), xs, ws, g_facet,
                             dtype == PM_BF16, st);
}

// ---- vertex2facet forward without any allocation by caller or library ---------------------------------
// The folded coefficient image that pm_v2f keeps in the caller's workspace lives here in a file-scope device array.
// In host code the array's name is only a handle for hipGetSymbolAddress: the device address is looked up once per
// device (every GPU holds its own copy of the array at its own address) and that pointer is what kernels get.
static __device__ __align__(256) unsigned char scratch[PM_V2F_NOALLOC_SCRATCH_BYTES];

static pm_status noalloc_scratch(void** out) {
  static std::mutex mu;
  static std::map<int, void*> addr;   // device -> address of its copy of `scratch`
  int dev = 0;
  PM_CHECK_HIP(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(mu);
  auto it = addr.find(dev);
  if (it == addr.end()) {
    void* p = nullptr;
    PM_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || !pm_aligned16(p)) return pm_fail(PM_ERR_HIP, "no device address for the static scratch array");
    it = addr.emplace(dev, p).first;
  }
  *out = it->second;
  return PM_OK;
}

extern "C" pm_status pm_v2f_noalloc(const pm_mesh* mesh, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype,
                                    const void* h_vert, const void* W, void* g_facet, void* stream) {
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_mesh(mesh, false));
  const size_t need = plan_ws(PM_OP_V2F, mesh->n_vert, mesh->n_facet, 0, L, cin, cout, dtype).total;
  if (need > (size_t)PM_V2F_NOALLOC_SCRATCH_BYTES)
    return pm_fail(PM_ERR_WORKSPACE, "pm_v2f_noalloc: cin=%d cout=%d need %zu bytes of scratch, the static array has %zu; "
                   "use pm_v2f with a workspace", cin, cout, need, (size_t)PM_V2F_NOALLOC_SCRATCH_BYTES);
  void* ptr = nullptr;
  PM_TRY(noalloc_scratch(&ptr));
  // the image is rebuilt from W by every call before it is read (stream order), nothing has to start at zero
  return pm_v2f(mesh, L, norm, cin, cout, dtype, h_vert, W, g_facet, ptr, PM_V2F_NOALLOC_SCRATCH_BYTES, stream);
}

extern "C" pm_status pm_v2f_bwd(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cout,
                                pm_dtype dtype, const void* h_vert, const void* W, const void* dg_facet, void* dh_vert,
                                float* dW, void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("v2f_bwd");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_mesh(mesh, false));
  PM_TRY(check_ptr(W, "W", true));
  PM_TRY(check_ptr(h_vert, "h_vert", mesh->n_vert > 0));
  PM_TRY(check_ptr(dg_facet, "dg_facet", mesh->n_facet > 0));
  PM_TRY(check_ptr(dh_vert, "dh_vert", false));
  PM_TRY(check_ptr(dW, "dW", false));
  if (dh_vert && (!adj || !adj->row_ptr || (mesh->n_facet > 0 && !adj->col)))
    return pm_fail(PM_ERR_INVALID_ARG, "dh_vert needs the adjacency");
  const int K = (L + 1) * (L + 1);
  const int64_t V = mesh->n_vert, F = mesh->n_facet;
  WsPlan w = plan_ws(PM_OP_V2F_BWD, V, F, 0, L, cin, cout, dtype);
  PM_TRY(check_ws(w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  void* sv = apack + w.apack;                          // [V][3][cout] corner-slot sums of dg (feature dtype)
  float* M = (float*)((char*)sv + w.inter);            // [3][cin][cout]
  void* wg = (char*)M + w.small;
  FoldCoef fc;
  fold_coef(L, norm, &fc);
  if (dh_vert) {
    // dh_v = sum_j W_j (sum over the facets that have v at corner j of dg_f),  W_j = sum_k B_k(e_j) W[k]:
    // first the corner-slot sums at the vertices (an adjacency entry 3f+j names facet and slot), then one
    // matrix pass over the vertex rows.  No per-facet intermediate is formed.
    const int fb = dtype == PM_BF16;
    PM_TRY(pm_launch_segsum_slots(V, cout, dg_facet, fb, adj->row_ptr, adj->col, sv, fb, st));
    PM_TRY(pm_launch_pack(PACK_FOLD_BWD, dtype, K, cin, cout, W, &fc, apack, st));
    if (pm_point_stage_wide_applies(dtype, 3 * cout, cin, sv, dh_vert)) {
      PM_TRY(pm_launch_point_stage_wide(V, 3 * cout, cin, sv, apack, dh_vert, st));
    } else {
      RowSrc xs = row_src(sv, dtype, 3 * cout);
      PM_TRY(pm_launch_conv_rows(dtype, B_ONE, X_DIRECT, V, 1, 3 * cout, cin, basis_none(), xs, apack, dh_vert, fb, st));
    }
  }
  if (dW) {
    RowSrc xs = row_src(h_vert, dtype, cin);
    xs.facet = mesh->facet;
    RowSrc ys = row_src(dg_facet, dtype, cout);
    PM_TRY(pm_launch_wgrad(dtype, B_ONE, X_GATHER_CAT, X_DIRECT, F, 3, cin, cout, basis_none(), xs, ys, M, wg, w.wgrad,
                           nullptr, st));
    PM_TRY(pm_launch_unfold(K, cin, cout, M, &fc, dW, st));
  }
  return PM_OK;
}

// ---- depth-wise separable facet2vertex / vertex2facet ---------------------------------------------
static pm_status check_sep(const float* alpha, const void* P) {
  if (!alpha || !pm_aligned16(alpha)) return pm_fail(PM_ERR_INVALID_ARG, "alpha is NULL or not 16-byte aligned");
  return check_ptr(P, "P", true);
}

// out = rows P on directly addressed rows (apack: the plain or transposed image of P): the staged-tile kernel for
// the bf16 shapes it covers, else the general row kernel
static pm_status pointwise_rows(pm_dtype dtype, int64_t R, int cin, int cout, const void* rows, const void* apack,
                                void* out, int out_bf16, hipStream_t st, const int32_t* mean_row_ptr = nullptr,
                                int* prescaled = nullptr) {
  if (prescaled) *prescaled = 0;
  if (pm_v2f_stage_applies(dtype, cin, cout, rows, out)) {
    if (!out_bf16) {
      // fp32 rows; on request each leaves divided by the length of its segment (told back through `prescaled`)
      if (prescaled && mean_row_ptr) *prescaled = 1;
      return pm_launch_point_stage_f32(R, cin, cout, rows, apack, (float*)out, prescaled ? mean_row_ptr : nullptr, st);
    }
    return pm_launch_v2v_stage(R, cin, cout, nullptr, rows, apack, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr,
                               nullptr, out, st);
  }
  RowSrc xs = row_src(rows, dtype, cin);
  return pm_launch_conv_rows(dtype, B_ONE, X_DIRECT, R, 1, cin, cout, basis_none(), xs, apack, out, out_bf16, st);
}

extern "C" pm_status pm_f2v_sep(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cout,
                                pm_dtype dtype, const void* h_facet, const float* alpha, const void* P, void* g_vert,
                                void* z_vert, void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("f2v_sep");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_mesh(mesh, true));
  if (!adj || !adj->row_ptr || (mesh->n_facet > 0 && !adj->col)) return pm_fail(PM_ERR_INVALID_ARG, "adjacency is NULL");
  PM_TRY(check_sep(alpha, P));
  PM_TRY(check_ptr(h_facet, "h_facet", mesh->n_facet > 0));
  PM_TRY(check_ptr(g_vert, "g_vert", mesh->n_vert > 0));
  PM_TRY(check_ptr(z_vert, "z_vert", false));
  const int K = (L + 1) * (L + 1);
  const int64_t V = mesh->n_vert, F = mesh->n_facet;
  WsPlan w = plan_ws(PM_OP_F2V_SEP, V, F, 0, L, cin, cout, dtype);
  PM_TRY(check_ws(w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  void* y = apack + w.apack;
  void* z = z_vert ? z_vert : (void*)((char*)y + w.inter);
  const int fb = dtype == PM_BF16;
  BasisSrc bs = basis_none();
  bs.vert = mesh->vert; bs.facet = mesh->facet;
  pm_make_sh_table(L, norm, &bs.sh);
  // depth-wise stage per facet, mean over the adjacent facets, then the point-wise matrix on the vertex rows
  // (the mean and the matrix commute, and there are half as many vertices as facets)
  PM_TRY(pm_launch_dw_f2v(F, K, cin, fb, bs, h_facet, alpha, y, st));
  PM_TRY(pm_launch_segreduce(V, cin, y, fb, adj->row_ptr, adj->col, 3, 1, z, fb, st));
  PM_TRY(pm_launch_pack(PACK_PLAIN, dtype, 1, cin, cout, P, nullptr, apack, st));
  return pointwise_rows(dtype, V, cin, cout, z, apack, g_vert, fb, st);
}

// mask_scale / mask_relu: dh_facet leaves through the epilogue that produced h_facet (vertex2vertex block)
static pm_status f2v_sep_bwd_impl(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin,
                                  int cout, pm_dtype dtype, const void* h_facet, const float* alpha, const void* P,
                                  const void* dg_vert, const void* z_saved, void* dh_facet, float* dalpha, float* dP,
                                  void* ws, size_t ws_bytes, void* stream, const float* mask_scale, int mask_relu) {
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_mesh(mesh, true));
  if (!adj || !adj->row_ptr || (mesh->n_facet > 0 && !adj->col)) return pm_fail(PM_ERR_INVALID_ARG, "adjacency is NULL");
  PM_TRY(check_sep(alpha, P));
  PM_TRY(check_ptr(h_facet, "h_facet", mesh->n_facet > 0));
  PM_TRY(check_ptr(dg_vert, "dg_vert", mesh->n_vert > 0));
  PM_TRY(check_ptr(z_saved, "z_saved", false));
  PM_TRY(check_ptr(dh_facet, "dh_facet", false));
  PM_TRY(check_ptr(dalpha, "dalpha", false));
  PM_TRY(check_ptr(dP, "dP", false));
  if ((dalpha == nullptr) != (dP == nullptr)) return pm_fail(PM_ERR_INVALID_ARG, "dalpha and dP come together");
  const int K = (L + 1) * (L + 1);
  const int64_t V = mesh->n_vert, F = mesh->n_facet;
  WsPlan w = plan_ws(PM_OP_F2V_SEP_BWD, V, F, 0, L, cin, cout, dtype);
  PM_TRY(check_ws(w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  void* y = apack + w.apack;
  void* z = (char*)y + w.inter;
  void* dz = (char*)z + w.owner;
  void* wg = (char*)dz + w.small;
  const int fb = dtype == PM_BF16;
  BasisSrc bs = basis_none();
  bs.vert = mesh->vert; bs.facet = mesh->facet;
  pm_make_sh_table(L, norm, &bs.sh);
  PM_TRY(pm_launch_pack(PACK_TRANS, dtype, 1, cin, cout, P, nullptr, apack, st));
  RowSrc gs = row_src(dg_vert, dtype, cout);
  // dz = dg P^T on the vertex rows; where the staged kernel runs, each row leaves divided by its vertex degree, so
  // the depth-wise backward gathers plain sums
  int dz_prescaled = 0;
  PM_TRY(pointwise_rows(dtype, V, cout, cin, dg_vert, apack, dz, 0, st, adj->row_ptr, &dz_prescaled));
  if (dP) {
    // dP = z^T dg with the vertex means z the forward call handed out, or recomputed here (depth-wise stage +
    // vertex mean: two bandwidth-bound passes)
    if (!z_saved) {
      PM_TRY(pm_launch_dw_f2v(F, K, cin, fb, bs, h_facet, alpha, y, st));
      PM_TRY(pm_launch_segreduce(V, cin, y, fb, adj->row_ptr, adj->col, 3, 1, z, fb, st));
    }
    RowSrc zs = row_src(z_saved ? z_saved : z, dtype, cin);
    PM_TRY(pm_launch_wgrad(dtype, B_ONE, X_DIRECT, X_DIRECT, V, 1, cin, cout, basis_none(), zs, gs, dP, wg, w.wgrad,
                           nullptr, st));
  }
  if (dh_facet || dalpha)
    PM_TRY(pm_launch_dw_f2v_bwd(F, K, cin, fb, bs, h_facet, alpha, (const float*)dz, adj->row_ptr, dh_facet, dalpha,
                                (float*)wg, mask_scale, mask_relu, dz_prescaled, st));
  return PM_OK;
}

extern "C" pm_status pm_f2v_sep_bwd(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin,
                                    int cout, pm_dtype dtype, const void* h_facet, const float* alpha, const void* P,
                                    const void* dg_vert, const void* z_saved, void* dh_facet, float* dalpha, float* dP,
                                    void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("f2v_sep_bwd");
  return f2v_sep_bwd_impl(mesh, adj, L, norm, cin, cout, dtype, h_facet, alpha, P, dg_vert, z_saved, dh_facet, dalpha, dP, ws,
                          ws_bytes, stream, nullptr, 0);
}

extern "C" pm_status pm_v2f_sep(const pm_mesh* mesh, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype,
                                const void* h_vert, const float* alpha, const void* P, void* g_facet, void* ws,
                                size_t ws_bytes, void* stream) {
  pm_prof_set_op("v2f_sep");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_mesh(mesh, false));
  PM_TRY(check_sep(alpha, P));
  PM_TRY(check_ptr(h_vert, "h_vert", mesh->n_vert > 0));
  PM_TRY(check_ptr(g_facet, "g_facet", mesh->n_facet > 0));
  const int K = (L + 1) * (L + 1);
  WsPlan w = plan_ws(PM_OP_V2F_SEP, mesh->n_vert, mesh->n_facet, 0, L, cin, cout, dtype);
  PM_TRY(check_ws(w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  // the three corner directions are constants: W_j = diag(s(e_j)) P, then the folded dense path
  FoldCoef fc;
  fold_coef(L, norm, &fc);
  PM_TRY(pm_launch_pack(PACK_SEP_FOLD, dtype, K, cin, cout, P, &fc, apack, st, alpha));
  if (pm_v2f_stage_applies(dtype, cin, cout, h_vert, g_facet))
    return pm_launch_v2f_stage(mesh->n_facet, cin, cout, mesh->facet, h_vert, apack, g_facet, st);
  RowSrc xs = row_src(h_vert, dtype, cin);
  xs.facet = mesh->facet;
  return pm_launch_conv_rows(dtype, B_ONE, X_GATHER_CAT, mesh->n_facet, 1, 3 * cin, cout, basis_none(), xs, apack,
                             g_facet, dtype == PM_BF16, st);
}

extern "C" pm_status pm_v2f_sep_bwd(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin,
                                    int cout, pm_dtype dtype, const void* h_vert, const float* alpha, const void* P,
                                    const void* dg_facet, void* dh_vert, float* dalpha, float* dP, void* ws,
                                    size_t ws_bytes, void* stream) {
  pm_prof_set_op("v2f_sep_bwd");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_mesh(mesh, false));
  PM_TRY(check_sep(alpha, P));
  PM_TRY(check_ptr(h_vert, "h_vert", mesh->n_vert > 0));
  PM_TRY(check_ptr(dg_facet, "dg_facet", mesh->n_facet > 0));
  PM_TRY(check_ptr(dh_vert, "dh_vert", false));
  PM_TRY(check_ptr(dalpha, "dalpha", false));
  PM_TRY(check_ptr(dP, "dP", false));
  if ((dalpha == nullptr) != (dP == nullptr)) return pm_fail(PM_ERR_INVALID_ARG, "dalpha and dP come together");
  if (dh_vert && (!adj || !adj->row_ptr || (mesh->n_facet > 0 && !adj->col)))
    return pm_fail(PM_ERR_INVALID_ARG, "dh_vert needs the adjacency");
  const int K = (L + 1) * (L + 1);
  const int64_t V = mesh->n_vert, F = mesh->n_facet;
  WsPlan w = plan_ws(PM_OP_V2F_SEP_BWD, V, F, 0, L, cin, cout, dtype);
  PM_TRY(check_ws(w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  void* sv = apack + w.apack;
  float* M = (float*)((char*)sv + w.inter);
  void* wg = (char*)M + w.small;
  const int fb = dtype == PM_BF16;
  FoldCoef fc;
  fold_coef(L, norm, &fc);
  if (dh_vert) {
    // one GEMM row per facet with P alone (the three corner matrices differ only by a channel scale), then the
    // per-vertex sum applies the scale of each entry's corner
    PM_TRY(pm_launch_pack(PACK_TRANS, dtype, 1, cin, cout, P, nullptr, apack, st));
    PM_TRY(pointwise_rows(dtype, F, cout, cin, dg_facet, apack, sv, fb, st));
    PM_TRY(pm_launch_slot_scale_sum(V, K, cin, fb, sv, adj->row_ptr, adj->col, alpha, &fc,
                                    (float*)((char*)M + pm_round_up((size_t)3 * cin * cout * 4, 256)), dh_vert, st));
  }
  if (dP) {
    RowSrc xs = row_src(h_vert, dtype, cin);
    xs.facet = mesh->facet;
    RowSrc ys = row_src(dg_facet, dtype, cout);
    PM_TRY(pm_launch_wgrad(dtype, B_ONE, X_GATHER_CAT, X_DIRECT, F, 3, cin, cout, basis_none(), xs, ys, M, wg, w.wgrad,
                           nullptr, st));
    PM_TRY(pm_launch_sep_unfold(K, cin, cout, fb, M, alpha, P, &fc, dalpha, dP, st));
  }
  return PM_OK;
}

// ---- separable vertex2vertex block ---------------------------------------------------------------------
struct V2vWs { size_t ap1, ap2, gbuf, dq, sub, total; };

static V2vWs plan_v2v(int bwd, int64_t V, int64_t F, int L, int cin, int cmid, int cout, pm_dtype dt) {
  V2vWs w = {0, 0, 0, 0, 0, 0};
  if (!bwd) {
    w.ap1 = pm_pack_bytes(pm_pack_geom(1, 3 * cin, cmid, dt));
    w.ap2 = pm_pack_bytes(pm_pack_geom(1, cmid, cout, dt));
    w.gbuf = pm_round_up((size_t)F * cmid * esize(dt), 256);      // facet rows: g (general path) or g (.) s2 (fused)
    w.sub = std::max(plan_ws(PM_OP_V2F_SEP, V, F, 0, L, cin, cmid, dt).total,
                     plan_ws(PM_OP_F2V_SEP, V, F, 0, L, cmid, cout, dt).total);
  } else {
    w.dq = pm_round_up((size_t)V * cout * esize(dt), 256);        // gradient at z P2
    w.gbuf = pm_round_up((size_t)F * cmid * esize(dt), 256);      // gradient at g, then at u
    w.sub = std::max(plan_ws(PM_OP_V2F_SEP_BWD, V, F, 0, L, cin, cmid, dt).total,
                     plan_ws(PM_OP_F2V_SEP_BWD, V, F, 0, L, cmid, cout, dt).total);
  }
  w.total = w.ap1 + w.ap2 + w.gbuf + w.dq + w.sub;
  return w;
}

static pm_status check_v2v(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cmid, int cout,
                           pm_dtype dtype, const float* alpha1, const void* P1, const float* alpha2, const void* P2) {
  PM_TRY(check_conv_common(L, norm, cin, cmid, dtype));
  PM_TRY(check_conv_common(L, norm, cmid, cout, dtype));
  PM_TRY(check_mesh(mesh, true));
  if (!adj || !adj->row_ptr || (mesh->n_facet > 0 && !adj->col)) return pm_fail(PM_ERR_INVALID_ARG, "adjacency is NULL");
  PM_TRY(check_sep(alpha1, P1));
  return check_sep(alpha2, P2);
}

extern "C" size_t pm_v2v_sep_ws_bytes(int backward, int64_t n_vert, int64_t n_facet, int L, int cin, int cmid, int cout,
                                      pm_dtype dtype) {
  if (n_vert < 0 || n_facet < 0) return 0;
  if (check_conv_common(L, PM_SH_PAPER, cin, cmid, dtype) != PM_OK) return 0;
  if (check_conv_common(L, PM_SH_PAPER, cmid, cout, dtype) != PM_OK) return 0;
  return plan_v2v(backward != 0, n_vert, n_facet, L, cin, cmid, cout, dtype).total;
}

extern "C" pm_status pm_v2v_sep(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cmid,
                                int cout, pm_dtype dtype, const void* h_vert, const float* alpha1, const void* P1,
                                const pm_epilogue* ep1, const float* alpha2, const void* P2, const pm_epilogue* ep2,
                                void* out_vert, void* g_facet, void* z_vert, void* ws, size_t ws_bytes, void* stream) {
  PM_TRY(check_v2v(mesh, adj, L, norm, cin, cmid, cout, dtype, alpha1, P1, alpha2, P2));
  PM_TRY(check_ptr(h_vert, "h_vert", mesh->n_vert > 0));
  PM_TRY(check_ptr(out_vert, "out_vert", mesh->n_vert > 0));
  PM_TRY(check_ptr(g_facet, "g_facet", false));
  PM_TRY(check_ptr(z_vert, "z_vert", false));
  const int K = (L + 1) * (L + 1);
  const int64_t V = mesh->n_vert, F = mesh->n_facet;
  V2vWs w = plan_v2v(0, V, F, L, cin, cmid, cout, dtype);
  PM_TRY(check_ptr(ws, "ws", true));
  if (ws_bytes < w.total) return pm_fail(PM_ERR_WORKSPACE, "workspace %zu < required %zu bytes", ws_bytes, w.total);
  hipStream_t st = (hipStream_t)stream;
  char* ap1 = (char*)ws;
  char* ap2 = ap1 + w.ap1;
  void* gbuf = ap2 + w.ap2;
  char* sub = (char*)gbuf + w.gbuf;
  const int fb = dtype == PM_BF16;
  const pm_epilogue none = {nullptr, nullptr, 0};
  const pm_epilogue e1 = ep1 ? *ep1 : none, e2 = ep2 ? *ep2 : none;
  if (F > 0 && pm_v2f_stage_applies(dtype, cin, cmid, h_vert, gbuf) && (!g_facet || pm_aligned16(g_facet))) {
    // fused: gather, fold, epilogue and depth-wise filter per facet tile; vertex means; point-wise matrix + epilogue
    pm_prof_set_op("v2v_sep");
    FoldCoef fc;
    fold_coef(L, norm, &fc);
    ShTable sh;
    pm_make_sh_table(L, norm, &sh);
    PM_TRY(pm_launch_pack(PACK_SEP_FOLD, dtype, K, cin, cmid, P1, &fc, ap1, st, alpha1));
    PM_TRY(pm_launch_v2v_stage(F, cin, cmid, mesh->facet, h_vert, ap1, e1.scale, e1.shift, e1.relu, g_facet, alpha2, K,
                               mesh->vert, &sh, gbuf, st));
    void* z = z_vert ? z_vert : (void*)sub;
    PM_TRY(pm_launch_segreduce(V, cmid, gbuf, fb, adj->row_ptr, adj->col, 3, 1, z, fb, st));
    PM_TRY(pm_launch_pack(PACK_PLAIN, dtype, 1, cmid, cout, P2, nullptr, ap2, st));
    if (pm_v2f_stage_applies(dtype, cmid, cout, z, out_vert))
      return pm_launch_v2v_stage(V, cmid, cout, nullptr, z, ap2, e2.scale, e2.shift, e2.relu, nullptr, nullptr, 0, nullptr,
                                 nullptr, out_vert, st);
    RowSrc xs = row_src(z, dtype, cmid);
    PM_TRY(pm_launch_conv_rows(dtype, B_ONE, X_DIRECT, V, 1, cmid, cout, basis_none(), xs, ap2, out_vert, fb, st));
    return pm_launch_affine_act(V, cout, fb, out_vert, e2.scale, e2.shift, e2.relu, st);
  }
  // general shapes: the separable entry points with the element-wise epilogues in between
  void* g = g_facet ? g_facet : gbuf;
  PM_TRY(pm_v2f_sep(mesh, L, norm, cin, cmid, dtype, h_vert, alpha1, P1, g, sub, w.sub, stream));
  pm_prof_set_op("v2v_sep");
  PM_TRY(pm_launch_affine_act(F, cmid, fb, g, e1.scale, e1.shift, e1.relu, st));
  PM_TRY(pm_f2v_sep(mesh, adj, L, norm, cmid, cout, dtype, g, alpha2, P2, out_vert, z_vert, sub, w.sub, stream));
  pm_prof_set_op("v2v_sep");
  return pm_launch_affine_act(V, cout, fb, out_vert, e2.scale, e2.shift, e2.relu, st);
}

extern "C" pm_status pm_v2v_sep_bwd(const pm_mesh* mesh, const pm_vf_adj* adj, int L, pm_sh_norm norm, int cin, int cmid,
                                    int cout, pm_dtype dtype, const void* h_vert, const float* alpha1, const void* P1,
                                    const pm_epilogue* ep1, const float* alpha2, const void* P2, const pm_epilogue* ep2,
                                    const void* g_saved, const void* z_saved, const void* out_saved, const void* d_out,
                                    void* dh_vert, float* dalpha1, float* dP1, float* dalpha2, float* dP2, void* ws,
                                    size_t ws_bytes, void* stream) {
  PM_TRY(check_v2v(mesh, adj, L, norm, cin, cmid, cout, dtype, alpha1, P1, alpha2, P2));
  const int64_t V = mesh->n_vert, F = mesh->n_facet;
  const pm_epilogue none = {nullptr, nullptr, 0};
  const pm_epilogue e1 = ep1 ? *ep1 : none, e2 = ep2 ? *ep2 : none;
  PM_TRY(check_ptr(h_vert, "h_vert", V > 0));
  PM_TRY(check_ptr(g_saved, "g_saved", F > 0));
  PM_TRY(check_ptr(z_saved, "z_saved", V > 0));
  PM_TRY(check_ptr(out_saved, "out_saved", V > 0 && e2.relu));
  PM_TRY(check_ptr(d_out, "d_out", V > 0));
  PM_TRY(check_ptr(dh_vert, "dh_vert", false));
  if ((dalpha1 == nullptr) != (dP1 == nullptr) || (dalpha2 == nullptr) != (dP2 == nullptr))
    return pm_fail(PM_ERR_INVALID_ARG, "dalpha and dP come together");
  V2vWs w = plan_v2v(1, V, F, L, cin, cmid, cout, dtype);
  PM_TRY(check_ptr(ws, "ws", true));
  if (ws_bytes < w.total) return pm_fail(PM_ERR_WORKSPACE, "workspace %zu < required %zu bytes", ws_bytes, w.total);
  hipStream_t st = (hipStream_t)stream;
  void* dg = ws;                                  // gradient at the facet features, then at u
  void* dq = (char*)dg + w.gbuf;
  char* sub = (char*)dq + w.dq;
  const int fb = dtype == PM_BF16;
  // gradient at z P2 (the epilogue of the vertex stage), then the facet2vertex stage
  pm_prof_set_op("v2v_sep_bwd");
  const void* dq_in = d_out;
  if (e2.scale || e2.relu) {
    PM_TRY(pm_launch_affine_act_bwd(V, cout, fb, d_out, out_saved, e2.scale, e2.relu, dq, st));
    dq_in = dq;
  }
  // the depth-wise backward kernel holds g in registers: it hands the gradient on through the facet epilogue,
  // du = dg a1 [g > 0]
  const bool need_dg = dh_vert || dP1;
  PM_TRY(f2v_sep_bwd_impl(mesh, adj, L, norm, cmid, cout, dtype, g_saved, alpha2, P2, dq_in, z_saved, need_dg ? dg : nullptr,
                          dalpha2, dP2, sub, w.sub, stream, e1.scale, e1.relu));
  if (!need_dg) return PM_OK;
  pm_status rc = pm_v2f_sep_bwd(mesh, adj, L, norm, cin, cmid, dtype, h_vert, alpha1, P1, dg, dh_vert, dalpha1, dP1, sub,
                                w.sub, stream);
  pm_prof_set_op("v2v_sep_bwd");
  return rc;
}

// ---- pooling / unpooling over vertex clusters ------------------------------------------------------
static pm_status check_cluster_sizes(int64_t n_in, int64_t n_out) {
  if (n_in < 0 || n_out < 0 || n_in >= kMaxIds || n_out >= kMaxIds)
    return pm_fail(PM_ERR_INVALID_ARG, "n_in=%lld n_out=%lld", (long long)n_in, (long long)n_out);
  return PM_OK;
}

extern "C" size_t pm_cluster_ws_bytes(int64_t n_in, int64_t n_out) {
  if (check_cluster_sizes(n_in, n_out) != PM_OK) return 0;
  return 256 + pm_round_up((size_t)(n_in + 1) * 4, 256) + pm_csr_ws_bytes(n_out, n_in);
}

static pm_status check_cluster_args(int64_t n_in, int64_t n_out, const int32_t* vcluster, const int32_t* iomap,
                                    void* ws, size_t ws_bytes) {
  PM_TRY(check_cluster_sizes(n_in, n_out));
  if (n_in > 0 && (!vcluster || !iomap)) return pm_fail(PM_ERR_INVALID_ARG, "vcluster / iomap is NULL");
  PM_TRY(check_ptr(ws, "ws", true));
  if (ws_bytes < pm_cluster_ws_bytes(n_in, n_out))
    return pm_fail(PM_ERR_WORKSPACE, "workspace %zu < required %zu bytes", ws_bytes, pm_cluster_ws_bytes(n_in, n_out));
  return PM_OK;
}

extern "C" pm_status pm_validate_clusters(int64_t n_in, int64_t n_out, const int32_t* vcluster, const int32_t* iomap,
                                          void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("validate_clusters");
  PM_TRY(check_cluster_args(n_in, n_out, vcluster, iomap, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  int32_t* bad = (int32_t*)ws;
  int32_t* target = (int32_t*)((char*)ws + 256);
  PM_TRY(pm_launch_fill_i32(bad, 1, 0, st));
  PM_TRY(pm_launch_cluster_target(n_in, n_out, vcluster, iomap, target, bad, st));
  int32_t n_bad = 0;
  PM_CHECK_HIP(hipMemcpyAsync(&n_bad, bad, sizeof(n_bad), hipMemcpyDeviceToHost, st));
  PM_CHECK_HIP(hipStreamSynchronize(st));
  if (n_bad) return pm_fail(PM_ERR_BAD_MESH, "%d cluster / map ids are out of range", (int)n_bad);
  return PM_OK;
}

extern "C" pm_status pm_build_cluster_map(int64_t n_in, int64_t n_out, const int32_t* vcluster, const int32_t* iomap,
                                          int32_t* target, int32_t* row_ptr, int32_t* col, void* ws, size_t ws_bytes,
                                          void* stream) {
  pm_prof_set_op("cluster_map");
  PM_TRY(check_cluster_args(n_in, n_out, vcluster, iomap, ws, ws_bytes));
  if (!row_ptr || (n_in > 0 && (!target || !col))) return pm_fail(PM_ERR_INVALID_ARG, "target / row_ptr / col is NULL");
  hipStream_t st = (hipStream_t)stream;
  PM_TRY(pm_launch_cluster_target(n_in, n_out, vcluster, iomap, target, nullptr, st));
  return pm_launch_csr(n_out, n_in, target, row_ptr, col, (char*)ws + 256 + pm_round_up((size_t)(n_in + 1) * 4, 256), st);
}

static pm_status check_pool(const pm_cluster_map* cm, int C, pm_dtype dtype, bool need_csr) {
  if (!cm) return pm_fail(PM_ERR_INVALID_ARG, "cluster map is NULL");
  PM_TRY(check_cluster_sizes(cm->n_in, cm->n_out));
  if (dtype != PM_F32 && dtype != PM_BF16) return pm_fail(PM_ERR_UNSUPPORTED, "unknown pm_dtype %d", (int)dtype);
  if (C < 1 || C > 65536) return pm_fail(PM_ERR_INVALID_ARG, "C=%d", C);
  if (cm->n_in > 0 && !cm->target) return pm_fail(PM_ERR_INVALID_ARG, "cluster map target is NULL");
  if (need_csr && (!cm->row_ptr || (cm->n_in > 0 && !cm->col))) return pm_fail(PM_ERR_INVALID_ARG, "cluster map CSR is NULL");
  return PM_OK;
}

extern "C" pm_status pm_pool(const pm_cluster_map* cm, pm_pool_mode mode, int C, pm_dtype dtype, const void* h_in,
                             void* h_out, int32_t* argmax, void* stream) {
  pm_prof_set_op("pool");
  PM_TRY(check_pool(cm, C, dtype, true));
  if (mode != PM_POOL_MAX && mode != PM_POOL_AVG) return pm_fail(PM_ERR_UNSUPPORTED, "unknown pm_pool_mode %d", (int)mode);
  PM_TRY(check_ptr(h_in, "h_in", cm->n_in > 0));
  PM_TRY(check_ptr(h_out, "h_out", cm->n_out > 0));
  const int fb = dtype == PM_BF16;
  hipStream_t st = (hipStream_t)stream;
  if (mode == PM_POOL_AVG)
    return pm_launch_segreduce(cm->n_out, C, h_in, fb, cm->row_ptr, cm->col, 1, 1, h_out, fb, st);
  return pm_launch_segmax(cm->n_out, C, fb, h_in, cm->row_ptr, cm->col, h_out, argmax, st);
}

extern "C" pm_status pm_pool_bwd(const pm_cluster_map* cm, pm_pool_mode mode, int C, pm_dtype dtype,
                                 const void* dg_out, const int32_t* argmax, void* dh_in, void* stream) {
  pm_prof_set_op("pool_bwd");
  PM_TRY(check_pool(cm, C, dtype, mode == PM_POOL_AVG));
  if (mode != PM_POOL_MAX && mode != PM_POOL_AVG) return pm_fail(PM_ERR_UNSUPPORTED, "unknown pm_pool_mode %d", (int)mode);
  PM_TRY(check_ptr(dg_out, "dg_out", cm->n_out > 0));
  PM_TRY(check_ptr(dh_in, "dh_in", cm->n_in > 0));
  if (mode == PM_POOL_MAX && cm->n_out > 0 && !argmax) return pm_fail(PM_ERR_INVALID_ARG, "max pooling backward needs argmax");
  return pm_launch_cluster_gather(mode == PM_POOL_AVG ? 1 : 2, cm->n_in, C, dtype == PM_BF16, cm->target, cm->row_ptr,
                                  argmax, dg_out, dh_in, (hipStream_t)stream);
}

extern "C" pm_status pm_unpool(const pm_cluster_map* cm, int C, pm_dtype dtype, const void* h_coarse, void* h_fine,
                               void* stream) {
  pm_prof_set_op("unpool");
  PM_TRY(check_pool(cm, C, dtype, false));
  PM_TRY(check_ptr(h_coarse, "h_coarse", cm->n_out > 0));
  PM_TRY(check_ptr(h_fine, "h_fine", cm->n_in > 0));
  return pm_launch_cluster_gather(0, cm->n_in, C, dtype == PM_BF16, cm->target, nullptr, nullptr, h_coarse, h_fine,
                                  (hipStream_t)stream);
}

extern "C" pm_status pm_unpool_bwd(const pm_cluster_map* cm, int C, pm_dtype dtype, const void* dg_fine,
                                   void* dh_coarse, void* stream) {
  pm_prof_set_op("unpool_bwd");
  PM_TRY(check_pool(cm, C, dtype, true));
  PM_TRY(check_ptr(dg_fine, "dg_fine", cm->n_in > 0));
  PM_TRY(check_ptr(dh_coarse, "dh_coarse", cm->n_out > 0));
  const int fb = dtype == PM_BF16;
  return pm_launch_segreduce(cm->n_out, C, dg_fine, fb, cm->row_ptr, cm->col, 1, 0, dh_coarse, fb, (hipStream_t)stream);
}

// ---- point-cloud convolution with the radial term ------------------------------------------------------
struct PcWs { size_t apack, dy, y, owner, rev_ptr, rev_col, csr, tail, total; };

static PcWs plan_pc(int bwd, int64_t M, int64_t N, int64_t nnz, int L, int cin, int cout, pm_dtype dt) {
  const int K = (L + 1) * (L + 1);
  PcWs w = {0, 0, 0, 0, 0, 0, 0, 0, 0};
  w.y = pm_round_up((size_t)M * cin * esize(dt), 256);
  if (!bwd) {
    w.apack = pm_pack_bytes(pm_pack_geom(1, cin, cout, dt));
  } else {
    w.apack = pm_pack_bytes(pm_pack_geom(1, cout, cin, dt));
    w.dy = pm_round_up((size_t)M * cin * 4, 256);
    w.owner = pm_round_up((size_t)(nnz + 1) * 4, 256);
    w.rev_ptr = pm_round_up((size_t)(N + 1) * 4, 256);
    w.rev_col = pm_round_up((size_t)(nnz + 1) * 4, 256);
    w.csr = pm_csr_ws_bytes(N, nnz);
    w.tail = std::max(pm_pc_coef_ws_bytes(M, K, cin), pm_wgrad_ws_bytes(M, 1, cin, cout));
  }
  w.total = w.apack + w.dy + w.y + w.owner + w.rev_ptr + w.rev_col + w.csr + w.tail;
  return w;
}

static pm_status check_nbr(const pm_nbr* nb) {
  if (!nb) return pm_fail(PM_ERR_INVALID_ARG, "neighbour lists are NULL");
  if (nb->n_query < 0 || nb->n_source < 0 || nb->nnz < 0 || nb->n_query >= kMaxIds || nb->n_source >= kMaxIds ||
      nb->nnz >= kMaxIds)
    return pm_fail(PM_ERR_INVALID_ARG, "n_query=%lld n_source=%lld nnz=%lld", (long long)nb->n_query,
                   (long long)nb->n_source, (long long)nb->nnz);
  if (!nb->ptr) return pm_fail(PM_ERR_INVALID_ARG, "ptr is NULL");
  if (nb->nnz > 0 && (!nb->idx || nb->n_source == 0)) return pm_fail(PM_ERR_INVALID_ARG, "idx is NULL or there are no sources");
  if ((nb->n_query > 0 && !nb->xq) || (nb->n_source > 0 && !nb->xs)) return pm_fail(PM_ERR_INVALID_ARG, "xq / xs is NULL");
  if (!(nb->rho > 0.f)) return pm_fail(PM_ERR_INVALID_ARG, "rho must be positive");
  if ((nb->rev_ptr || nb->rev_col || nb->owner) && (!nb->rev_ptr || (nb->nnz > 0 && (!nb->rev_col || !nb->owner))))
    return pm_fail(PM_ERR_INVALID_ARG, "rev_ptr, rev_col and owner come together");
  return PM_OK;
}

extern "C" size_t pm_pcloud_ws_bytes(int backward, int64_t n_query, int64_t n_source, int64_t nnz, int L, int cin,
                                     int cout, pm_dtype dtype) {
  if (n_query < 0 || n_source < 0 || nnz < 0 || n_query >= kMaxIds || n_source >= kMaxIds || nnz >= kMaxIds) return 0;
  if (check_conv_common(L, PM_SH_PAPER, cin, cout, dtype) != PM_OK) return 0;
  return plan_pc(backward != 0, n_query, n_source, nnz, L, cin, cout, dtype).total;
}

extern "C" size_t pm_reverse_ws_bytes(int64_t n_source, int64_t nnz) {
  if (n_source < 0 || nnz < 0 || n_source >= kMaxIds || nnz >= kMaxIds) return 0;
  return pm_csr_ws_bytes(n_source, nnz);
}

extern "C" pm_status pm_build_reverse_neighbors(const pm_nbr* nb, int32_t* rev_ptr, int32_t* rev_col, int32_t* owner,
                                                void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("reverse_neighbors");
  PM_TRY(check_nbr(nb));
  if (!rev_ptr || (nb->nnz > 0 && (!rev_col || !owner))) return pm_fail(PM_ERR_INVALID_ARG, "rev_ptr / rev_col / owner is NULL");
  PM_TRY(check_ptr(ws, "ws", true));
  const size_t need = pm_csr_ws_bytes(nb->n_source, nb->nnz);
  if (ws_bytes < need) return pm_fail(PM_ERR_WORKSPACE, "workspace %zu < required %zu bytes", ws_bytes, need);
  hipStream_t st = (hipStream_t)stream;
  PM_TRY(pm_launch_owner(nb->n_query, nb->ptr, owner, st));
  return pm_launch_csr(nb->n_source, nb->nnz, nb->idx, rev_ptr, rev_col, ws, st);
}

extern "C" pm_status pm_validate_neighbors(const pm_nbr* nb, void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("validate_neighbors");
  PM_TRY(check_nbr(nb));
  PM_TRY(check_ptr(ws, "ws", true));
  if (ws_bytes < 16) return pm_fail(PM_ERR_WORKSPACE, "validate needs 16 bytes of workspace");
  hipStream_t st = (hipStream_t)stream;
  PM_TRY(pm_launch_validate_nbr(nb->n_query, nb->n_source, nb->nnz, nb->ptr, nb->idx, (int32_t*)ws, st));
  int32_t flag = 0;
  PM_CHECK_HIP(hipMemcpyAsync(&flag, ws, sizeof(flag), hipMemcpyDeviceToHost, st));
  PM_CHECK_HIP(hipStreamSynchronize(st));
  if (flag & 1) return pm_fail(PM_ERR_BAD_MESH, "neighbour offsets are not monotone or do not span the list");
  if (flag & 2) return pm_fail(PM_ERR_BAD_MESH, "a neighbour id is outside the source set");
  return PM_OK;
}

extern "C" pm_status pm_pcloud_conv(const pm_nbr* nb, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype,
                                    const void* h, const float* alpha, const float* c0, const void* P, void* g,
                                    void* y_query, void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("pcloud_conv");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_nbr(nb));
  PM_TRY(check_sep(alpha, P));
  if (!c0 || !pm_aligned16(c0)) return pm_fail(PM_ERR_INVALID_ARG, "c0 is NULL or not 16-byte aligned");
  PM_TRY(check_ptr(h, "h", nb->n_source > 0));
  PM_TRY(check_ptr(g, "g", nb->n_query > 0));
  PM_TRY(check_ptr(y_query, "y_query", false));
  const int K = (L + 1) * (L + 1);
  const int64_t M = nb->n_query, N = nb->n_source;
  PcWs w = plan_pc(0, M, N, nb->nnz, L, cin, cout, dtype);
  PM_TRY(check_ptr(ws, "ws", true));
  if (ws_bytes < w.total) return pm_fail(PM_ERR_WORKSPACE, "workspace %zu < required %zu bytes", ws_bytes, w.total);
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  void* y = y_query ? y_query : (void*)(apack + w.apack);
  const int fb = dtype == PM_BF16;
  ShTable sh;
  pm_make_sh_table(L, norm, &sh);
  PM_TRY(pm_launch_pc_dw(M, N, K, cin, fb, nb->rho, sh, nb->xq, nb->xs, nb->ptr, nb->idx, h, alpha, c0, y, st));
  PM_TRY(pm_launch_pack(PACK_PLAIN, dtype, 1, cin, cout, P, nullptr, apack, st));
  RowSrc ys = row_src(y, dtype, cin);
  return pm_launch_conv_rows(dtype, B_ONE, X_DIRECT, M, 1, cin, cout, basis_none(), ys, apack, g, fb, st);
}

extern "C" pm_status pm_pcloud_conv_bwd(const pm_nbr* nb, int L, pm_sh_norm norm, int cin, int cout, pm_dtype dtype,
                                        const void* h, const float* alpha, const float* c0, const void* P,
                                        const void* dg, const void* y_saved, void* dh, float* dalpha, float* dc0,
                                        float* dP, void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("pcloud_conv_bwd");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_nbr(nb));
  PM_TRY(check_sep(alpha, P));
  if (!c0 || !pm_aligned16(c0)) return pm_fail(PM_ERR_INVALID_ARG, "c0 is NULL or not 16-byte aligned");
  PM_TRY(check_ptr(h, "h", nb->n_source > 0));
  PM_TRY(check_ptr(dg, "dg", nb->n_query > 0));
  PM_TRY(check_ptr(y_saved, "y_saved", false));
  PM_TRY(check_ptr(dh, "dh", false));
  PM_TRY(check_ptr(dalpha, "dalpha", false));
  PM_TRY(check_ptr(dc0, "dc0", false));
  PM_TRY(check_ptr(dP, "dP", false));
  if ((dalpha == nullptr) != (dP == nullptr) || (dalpha == nullptr) != (dc0 == nullptr))
    return pm_fail(PM_ERR_INVALID_ARG, "dalpha, dc0 and dP come together");
  const int K = (L + 1) * (L + 1);
  const int64_t M = nb->n_query, N = nb->n_source, nnz = nb->nnz;
  PcWs w = plan_pc(1, M, N, nnz, L, cin, cout, dtype);
  PM_TRY(check_ptr(ws, "ws", true));
  if (ws_bytes < w.total) return pm_fail(PM_ERR_WORKSPACE, "workspace %zu < required %zu bytes", ws_bytes, w.total);
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  float* dy = (float*)(apack + w.apack);
  void* y = (char*)dy + w.dy;
  int32_t* owner = (int32_t*)((char*)y + w.y);
  int32_t* rev_ptr = (int32_t*)((char*)owner + w.owner);
  int32_t* rev_col = (int32_t*)((char*)rev_ptr + w.rev_ptr);
  void* csr_ws = (char*)rev_col + w.rev_col;
  void* tail = (char*)csr_ws + w.csr;
  const int fb = dtype == PM_BF16;
  ShTable sh;
  pm_make_sh_table(L, norm, &sh);
  // dy = dg P^T on the query rows, kept in fp32
  PM_TRY(pm_launch_pack(PACK_TRANS, dtype, 1, cin, cout, P, nullptr, apack, st));
  RowSrc gs = row_src(dg, dtype, cout);
  PM_TRY(pm_launch_conv_rows(dtype, B_ONE, X_DIRECT, M, 1, cout, cin, basis_none(), gs, apack, dy, 0, st));
  if (dalpha) {
    // one walk over the lists gives the coefficient gradients and, unless the forward call handed it out,
    // recomputes the depth-wise output y for dP
    PM_TRY(pm_launch_pc_dw_coef(M, N, K, cin, fb, nb->rho, sh, nb->xq, nb->xs, nb->ptr, nb->idx, h, alpha, c0, dy,
                                y_saved ? nullptr : y, dalpha, dc0, (float*)tail, st));
    RowSrc ys = row_src(y_saved ? y_saved : y, dtype, cin);
    PM_TRY(pm_launch_wgrad(dtype, B_ONE, X_DIRECT, X_DIRECT, M, 1, cin, cout, basis_none(), ys, gs, dP, tail, w.tail,
                           nullptr, st));
  }
  if (dh) {
    const int32_t *rp = nb->rev_ptr, *rc = nb->rev_col, *ow = nb->owner;
    if (!rp) {                                  // reverse lists: the caller's, or built here
      PM_TRY(pm_launch_owner(M, nb->ptr, owner, st));
      PM_TRY(pm_launch_csr(N, nnz, nb->idx, rev_ptr, rev_col, csr_ws, st));
      rp = rev_ptr; rc = rev_col; ow = owner;
    }
    PM_TRY(pm_launch_pc_dw_dh(M, N, K, cin, fb, nb->rho, sh, nb->xq, nb->xs, nb->ptr, rp, rc, ow, alpha, c0, dy, dh, st));
  }
  return PM_OK;
}

// ---- input preparation (Eq. 8, Eq. 9) --------------------------------------------------------------
extern "C" pm_status pm_facet_geometry(const pm_mesh* mesh, int with_heights, pm_dtype dtype, void* feat, void* stream) {
  pm_prof_set_op("facet_geometry");
  PM_TRY(check_mesh(mesh, true));
  if (dtype != PM_F32 && dtype != PM_BF16) return pm_fail(PM_ERR_UNSUPPORTED, "unknown pm_dtype %d", (int)dtype);
  PM_TRY(check_ptr(feat, "feat", mesh->n_facet > 0));
  return pm_launch_facet_geometry(mesh, with_heights != 0, dtype == PM_BF16, feat, (hipStream_t)stream);
}

extern "C" size_t pm_texture_ws_bytes(int64_t n_facet, int32_t n_mesh) {
  if (n_facet < 0 || n_facet >= kMaxIds || n_mesh < 0) return 0;
  return pm_texture_ws_bytes_host(n_facet, n_mesh);
}

extern "C" pm_status pm_texture_layout(const pm_mesh* mesh, int alpha, int beta, int32_t* gamma, int32_t* tex_off,
                                       void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("texture_layout");
  PM_TRY(check_mesh(mesh, true));
  if (alpha < 0 || beta < 0 || alpha + beta > 255) return pm_fail(PM_ERR_INVALID_ARG, "alpha=%d beta=%d", alpha, beta);
  if (mesh->n_mesh > 1 && !mesh->facet_off) return pm_fail(PM_ERR_INVALID_ARG, "n_mesh > 1 needs facet_off");
  {
    // every facet may reach gamma = alpha + beta: the running point count must fit the int32 offsets
    const int64_t gmax = alpha + beta, kmax = (gmax + 1) * (gmax + 2) / 2;
    if (mesh->n_facet * kmax >= kMaxIds)
      return pm_fail(PM_ERR_INVALID_ARG, "%lld facets with up to %lld points each exceed the int32 offsets",
                     (long long)mesh->n_facet, (long long)kmax);
  }
  if (!tex_off || (mesh->n_facet > 0 && !gamma)) return pm_fail(PM_ERR_INVALID_ARG, "gamma / tex_off is NULL");
  PM_TRY(check_ptr(ws, "ws", true));
  const size_t need = pm_texture_ws_bytes_host(mesh->n_facet, mesh->n_mesh);
  if (ws_bytes < need) return pm_fail(PM_ERR_WORKSPACE, "workspace %zu < required %zu bytes", ws_bytes, need);
  return pm_launch_texture_layout(mesh, alpha, beta, gamma, tex_off, ws, (hipStream_t)stream);
}

extern "C" pm_status pm_texture_bary(int64_t n_facet, const int32_t* gamma, const int32_t* tex_off, int64_t n_tex,
                                     float* bary, void* stream) {
  pm_prof_set_op("texture_bary");
  if (n_facet < 0 || n_tex < 0 || n_facet >= kMaxIds || n_tex >= kMaxIds)
    return pm_fail(PM_ERR_INVALID_ARG, "n_facet=%lld n_tex=%lld", (long long)n_facet, (long long)n_tex);
  if (n_facet > 0 && (!gamma || !tex_off)) return pm_fail(PM_ERR_INVALID_ARG, "gamma / tex_off is NULL");
  if (n_tex > 0 && !bary) return pm_fail(PM_ERR_INVALID_ARG, "bary is NULL");
  return pm_launch_texture_bary(n_facet, gamma, tex_off, n_tex, bary, (hipStream_t)stream);
}

// ---- facet2facet (Eq. 7) -------------------------------------------------------------------------
static pm_status check_f2f(int64_t n_facet, int64_t n_tex, const int32_t* tex_off, const float* bary) {
  if (n_facet < 0 || n_tex < 0 || n_facet >= kMaxIds || n_tex >= kMaxIds)
    return pm_fail(PM_ERR_INVALID_ARG, "n_facet=%lld n_tex=%lld", (long long)n_facet, (long long)n_tex);
  if (!tex_off) return pm_fail(PM_ERR_INVALID_ARG, "tex_off is NULL");
  if (n_tex > 0 && !bary) return pm_fail(PM_ERR_INVALID_ARG, "bary is NULL");
  return PM_OK;
}

extern "C" pm_status pm_f2f(int64_t n_facet, int64_t n_tex, const int32_t* tex_off, const float* bary, int L,
                            pm_sh_norm norm, int cin, int cout, pm_dtype dtype, const void* h_tex, const void* W,
                            void* g_facet, void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("f2f");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_f2f(n_facet, n_tex, tex_off, bary));
  PM_TRY(check_ptr(W, "W", true));
  PM_TRY(check_ptr(h_tex, "h_tex", n_tex > 0));
  PM_TRY(check_ptr(g_facet, "g_facet", n_facet > 0));
  const int K = (L + 1) * (L + 1);
  WsPlan w = plan_ws(PM_OP_F2F, 0, n_facet, n_tex, L, cin, cout, dtype);
  PM_TRY(check_ws(w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  void* yp = apack + w.apack;   // per-point summands of Eq. 7, in the feature dtype (summed in fp32)
  const int yb = dtype == PM_BF16;
  BasisSrc bs = basis_none();
  bs.dirs = bary;
  pm_make_sh_table(L, norm, &bs.sh);
  if (pm_f2f_small_applies(L, cin)) {
    // few input channels (the paper's shape: 3 colours): mean of the Khatri-Rao rows B_p (x) h_p over the points of a
    // facet first (K cin <= 64 values), then one contraction per facet with W viewed as [K cin][cout]
    PM_TRY(pm_launch_f2f_gather(n_facet, tex_off, bary, bs.sh, cin, yb, h_tex, yp, st));
    PM_TRY(pm_launch_pack(yb ? PACK_PLAIN_TWICE : PACK_PLAIN, dtype, 1, K * cin, cout, W, nullptr, apack, st));
    const int sc = yb ? 128 : 64;      // bf16 rows: head and remainder
    RowSrc ss = row_src(yp, dtype, sc);
    return pm_launch_conv_rows(dtype, B_ONE, X_DIRECT, n_facet, 1, sc, cout, basis_none(), ss, apack, g_facet, yb, st);
  }
  PM_TRY(pm_launch_pack(PACK_PLAIN, dtype, K, cin, cout, W, nullptr, apack, st));
  RowSrc xs = row_src(h_tex, dtype, cin);
  PM_TRY(pm_launch_conv_rows(dtype, B_DIRS, X_DIRECT, n_tex, K, cin, cout, bs, xs, apack, yp, yb, st));
  return pm_launch_segreduce(n_facet, cout, yp, yb, tex_off, nullptr, 1, 1, g_facet, dtype == PM_BF16, st);
}

extern "C" pm_status pm_f2f_bwd(int64_t n_facet, int64_t n_tex, const int32_t* tex_off, const float* bary, int L,
                                pm_sh_norm norm, int cin, int cout, pm_dtype dtype, const void* h_tex, const void* W,
                                const void* dg_facet, void* dh_tex, float* dW, void* ws, size_t ws_bytes, void* stream) {
  pm_prof_set_op("f2f_bwd");
  PM_TRY(check_conv_common(L, norm, cin, cout, dtype));
  PM_TRY(check_f2f(n_facet, n_tex, tex_off, bary));
  PM_TRY(check_ptr(W, "W", true));
  PM_TRY(check_ptr(h_tex, "h_tex", n_tex > 0));
  PM_TRY(check_ptr(dg_facet, "dg_facet", n_facet > 0));
  PM_TRY(check_ptr(dh_tex, "dh_tex", false));
  PM_TRY(check_ptr(dW, "dW", false));
  const int K = (L + 1) * (L + 1);
  WsPlan w = plan_ws(PM_OP_F2F_BWD, 0, n_facet, n_tex, L, cin, cout, dtype);
  PM_TRY(check_ws(w, ws, ws_bytes));
  hipStream_t st = (hipStream_t)stream;
  char* apack = (char*)ws;
  int32_t* owner = (int32_t*)(apack + w.apack);
  float* bvals = (float*)((char*)owner + w.owner);
  void* wg = (char*)bvals + w.inter;
  PM_TRY(pm_launch_owner(n_facet, tex_off, owner, st));
  BasisSrc bs = basis_none();
  bs.dirs = bary;
  pm_make_sh_table(L, norm, &bs.sh);
  if (pm_f2f_small_applies(L, cin)) {
    // few input channels: everything per facet except the basis weighting of the points (see pm_f2f)
    const int fb = dtype == PM_BF16, kc = K * cin;
    void* S = bvals;
    float* T = (float*)((char*)S + w.inter);
    void* wgs = (char*)T + w.small;
    RowSrc dgr = row_src(dg_facet, dtype, cout);
    if (dh_tex) {
      PM_TRY(pm_launch_pack(PACK_TRANS, dtype, 1, kc, cout, W, nullptr, apack, st));
      PM_TRY(pm_launch_conv_rows(dtype, B_ONE, X_DIRECT, n_facet, 1, cout, kc, basis_none(), dgr, apack, T, 0, st));
      PM_TRY(pm_launch_f2f_scatter(n_tex, owner, tex_off, bary, bs.sh, cin, fb, T, dh_tex, st));
    }
    if (dW) {
      PM_TRY(pm_launch_f2f_gather(n_facet, tex_off, bary, bs.sh, cin, fb, h_tex, S, st));
      RowSrc sr = row_src(S, dtype, fb ? 128 : 64);     // bf16: the head alone (first 64 channels of the 128)
      PM_TRY(pm_launch_wgrad(dtype, B_ONE, X_DIRECT, X_DIRECT, n_facet, 1, kc, cout, basis_none(), sr, dgr, dW, wgs, w.wgrad,
                             nullptr, st));
    }
    return PM_OK;
  }
  RowSrc dys = row_src(dg_facet, dtype, cout);   // gradient reaching point p: dg[owner(p)] / R_owner
  dys.owner = owner; dys.seg_off = tex_off;
  if (dh_tex) {
    PM_TRY(pm_launch_pack(PACK_TRANS, dtype, K, cin, cout, W, nullptr, apack, st));
    PM_TRY(pm_launch_conv_rows(dtype, B_DIRS, X_GATHER1, n_tex, K, cout, cin, bs, dys, apack, dh_tex, dtype == PM_BF16,
                               st));
  }
  if (dW) {
    RowSrc xs = row_src(h_tex, dtype, cin);
    if (!pm_wgrad_fuses_basis(dtype, B_DIRS, X_DIRECT, X_GATHER1, K, cin, cout, xs, dys)) {
      PM_TRY(pm_launch_basis_dirs(n_tex, bary, bs.sh, bvals, st));
      bs.bvals = bvals;
    }
    PM_TRY(pm_launch_wgrad(dtype, B_DIRS, X_DIRECT, X_GATHER1, n_tex, K, cin, cout, bs, xs, dys, dW, wg, w.wgrad, nullptr, st));
  }
  return PM_OK;
}
