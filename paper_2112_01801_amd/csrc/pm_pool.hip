// Mesh pooling / unpooling over the vertex clusters of a decimation (Section "Mesh decimation", paragraph
// "(Un)poolings"): pooling takes the maximum or the average of the features of a cluster, unpooling copies
// the feature of the output vertex onto every member.
//
// Everything runs on the cluster map: target[v] = IOmap[VCluster[v]] (the output vertex of input vertex v,
// -1 for none) and the CSR of the members of every output vertex, ascending.  All kernels are bound by HBM:
// a lane owns a run of channels, a group of lanes a row.  Sums walk the members in ascending order (no float
// atomics); the average pooling and the unpooling gradient are the segmented reduction of the convolutions.
#include "pm_host.h"
#include "pm_chan.h"

// target[v] = iomap[vcluster[v]]; any id outside its range gives -1 and is counted in *bad
__global__ void __launch_bounds__(256) k_cluster_target(int64_t n_in, int64_t n_out, const int32_t* __restrict__ vcluster,
                                                        const int32_t* __restrict__ iomap, int32_t* __restrict__ target,
                                                        int32_t* __restrict__ bad) {
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= n_in) return;
  const int32_t c = vcluster[v];
  int32_t t = -1;
  bool wrong = c < 0 || c >= n_in;
  if (!wrong) {
    t = iomap[c];
    if (t < -1 || t >= n_out) { wrong = true; t = -1; }
  }
  target[v] = t;
  if (wrong && bad) atomicAdd(bad, 1);
}

struct PoolP {
  int64_t n_in, n_out;
  int C, lpg;
  const int32_t* target;    // [n_in]
  const int32_t* row_ptr;   // [n_out+1]
  const int32_t* col;       // members, ascending
  const void* src;
  void* out;
  int32_t* argmax;          // max pooling: [n_out][C] written (may be NULL) / read by its backward
};

// h_out[o][c] = max over the members v of o of h_in[v][c]; the first member that reaches the maximum is
// recorded (ties go to the lowest input index); an output vertex without members gets 0 and -1.
// Entries are taken two at a time (clamped to the last one: a repeated entry never replaces an equal value).
template <bool BF16, bool VEC>
__global__ void __launch_bounds__(256) k_segmax(PoolP p) {
  constexpr int CPL = BF16 ? 8 : 4;
  const int gpb = 256 / p.lpg;
  const int sub = threadIdx.x % p.lpg;
  for (int64_t seg = (int64_t)blockIdx.x * gpb + threadIdx.x / p.lpg; seg < p.n_out; seg += (int64_t)gridDim.x * gpb) {
    const int32_t b = p.row_ptr[seg], e = p.row_ptr[seg + 1];
    for (int c0 = sub * CPL; c0 < p.C; c0 += p.lpg * CPL) {
      float best[CPL];
      int32_t arg[CPL];
#pragma unroll
      for (int i = 0; i < CPL; ++i) { best[i] = -__builtin_inff(); arg[i] = -1; }
      for (int32_t i0 = b; i0 < e; i0 += 2) {
        int32_t id[2];
        float x[2][CPL];
#pragma unroll
        for (int q = 0; q < 2; ++q) id[q] = p.col[min(i0 + q, e - 1)];
#pragma unroll
        for (int q = 0; q < 2; ++q) chan_load<BF16, CPL, VEC>(p.src, (int64_t)id[q] * p.C, p.C, c0, x[q]);
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
          for (int i = 0; i < CPL; ++i) {
            const bool up = x[q][i] > best[i];
            best[i] = up ? x[q][i] : best[i];
            arg[i] = up ? id[q] : arg[i];
          }
      }
#pragma unroll
      for (int i = 0; i < CPL; ++i) best[i] = arg[i] < 0 ? 0.f : best[i];
      chan_store<BF16, CPL, VEC>(p.out, seg * p.C, p.C, c0, best);
      if (p.argmax) {
#pragma unroll
        for (int i = 0; i < CPL; ++i)
          if (c0 + i < p.C) p.argmax[seg * p.C + c0 + i] = arg[i];
      }
    }
  }
}

// One pass over the input-mesh rows, each reading the row of its output vertex:
//   MODE 0  unpooling:                 out[v] = src[t]
//   MODE 1  average pooling backward:  out[v] = src[t] / |cluster t|
//   MODE 2  maximum pooling backward:  out[v][c] = src[t][c] if argmax[t][c] == v else 0
// (t = target[v]; rows with t = -1 are zero.)
template <bool BF16, bool VEC, int MODE>
__global__ void __launch_bounds__(256) k_cluster_gather(PoolP p) {
  constexpr int CPL = BF16 ? 8 : 4;
  const int gpb = 256 / p.lpg;
  const int sub = threadIdx.x % p.lpg;
  for (int64_t v = (int64_t)blockIdx.x * gpb + threadIdx.x / p.lpg; v < p.n_in; v += (int64_t)gridDim.x * gpb) {
    const int32_t t = p.target[v];
    float scale = 1.f;
    if (MODE == 1 && t >= 0) scale = 1.0f / (float)(p.row_ptr[t + 1] - p.row_ptr[t]);
    for (int c0 = sub * CPL; c0 < p.C; c0 += p.lpg * CPL) {
      float x[CPL];
#pragma unroll
      for (int i = 0; i < CPL; ++i) x[i] = 0.f;
      if (t >= 0) {
        chan_load<BF16, CPL, VEC>(p.src, (int64_t)t * p.C, p.C, c0, x);
        if (MODE == 1) {
#pragma unroll
          for (int i = 0; i < CPL; ++i) x[i] *= scale;
        }
        if (MODE == 2) {
#pragma unroll
          for (int i = 0; i < CPL; ++i) {
            const int32_t a = (c0 + i < p.C) ? p.argmax[(int64_t)t * p.C + c0 + i] : -1;
            x[i] = (a == (int32_t)v) ? x[i] : 0.f;
          }
        }
      }
      chan_store<BF16, CPL, VEC>(p.out, v * p.C, p.C, c0, x);
    }
  }
}

static void pool_geom(int C, int is_bf16, int64_t rows, int* lpg, unsigned* grid) {
  const int cpl = is_bf16 ? 8 : 4;
  int need = (C + cpl - 1) / cpl, l = 1;
  while (l < need && l < 64) l <<= 1;
  *lpg = l;
  const int gpb = 256 / l;
  int64_t nblk = (rows + gpb - 1) / gpb;
  if (nblk > (1 << 20)) nblk = 1 << 20;      // the kernels stride over the rows
  *grid = (unsigned)(nblk < 1 ? 1 : nblk);
}

pm_status pm_launch_cluster_target(int64_t n_in, int64_t n_out, const int32_t* vcluster, const int32_t* iomap,
                                   int32_t* target, int32_t* bad, hipStream_t st) {
  if (n_in == 0) return PM_OK;
  { ProfScope ps__(st, "k_cluster_target");
    hipLaunchKernelGGL(k_cluster_target, dim3((unsigned)((n_in + 255) / 256)), dim3(256), 0, st, n_in, n_out, vcluster,
                       iomap, target, bad); }
  PM_CHECK_LAUNCH("k_cluster_target");
  return PM_OK;
}

pm_status pm_launch_segmax(int64_t n_out, int C, int is_bf16, const void* h_in, const int32_t* row_ptr,
                           const int32_t* col, void* h_out, int32_t* argmax, hipStream_t st) {
  if (n_out == 0) return PM_OK;
  PoolP p;
  p.n_in = 0; p.n_out = n_out; p.C = C; p.target = nullptr; p.row_ptr = row_ptr; p.col = col; p.src = h_in;
  p.out = h_out; p.argmax = argmax;
  unsigned grid;
  pool_geom(C, is_bf16, n_out, &p.lpg, &grid);
  const bool vec = chan_vec_ok(C, is_bf16, h_in, h_out, nullptr);
  auto kern = is_bf16 ? (vec ? k_segmax<true, true> : k_segmax<true, false>)
                      : (vec ? k_segmax<false, true> : k_segmax<false, false>);
  { ProfScope ps__(st, "k_segmax");
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, st, p); }
  PM_CHECK_LAUNCH("k_segmax");
  return PM_OK;
}

template <int MODE>
static void launch_gather_mode(const PoolP& p, int is_bf16, bool vec, unsigned grid, hipStream_t st) {
  auto kern = is_bf16 ? (vec ? k_cluster_gather<true, true, MODE> : k_cluster_gather<true, false, MODE>)
                      : (vec ? k_cluster_gather<false, true, MODE> : k_cluster_gather<false, false, MODE>);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, st, p);
}

// mode: 0 unpooling, 1 average pooling backward (needs row_ptr), 2 maximum pooling backward (needs argmax)
pm_status pm_launch_cluster_gather(int mode, int64_t n_in, int C, int is_bf16, const int32_t* target,
                                   const int32_t* row_ptr, const int32_t* argmax, const void* src, void* out,
                                   hipStream_t st) {
  if (n_in == 0) return PM_OK;
  PoolP p;
  p.n_in = n_in; p.n_out = 0; p.C = C; p.target = target; p.row_ptr = row_ptr; p.col = nullptr; p.src = src;
  p.out = out; p.argmax = const_cast<int32_t*>(argmax);
  unsigned grid;
  pool_geom(C, is_bf16, n_in, &p.lpg, &grid);
  const bool vec = chan_vec_ok(C, is_bf16, src, out, nullptr);
  { ProfScope ps__(st, "k_cluster_gather");
    if (mode == 0) launch_gather_mode<0>(p, is_bf16, vec, grid, st);
    else if (mode == 1) launch_gather_mode<1>(p, is_bf16, vec, grid, st);
    else launch_gather_mode<2>(p, is_bf16, vec, grid, st); }
  PM_CHECK_LAUNCH("k_cluster_gather");
  return PM_OK;
}
