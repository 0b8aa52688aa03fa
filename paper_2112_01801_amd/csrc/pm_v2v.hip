// Element-wise stages of the separable vertex2vertex block (vertex2facet, Eq. 6, followed by facet2vertex, Eq. 5,
// each with a per-channel affine map -- normalisation with fixed statistics -- and ReLU):
//     forward, in place:   x[r][c] <- act(scale[c] x[r][c] + shift[c])
//     backward:            out[r][c] = dy[r][c] scale[c] [y[r][c] > 0]         (y = the activated forward rows)
// Used where the fused kernels do not apply (any dtype and channel count) and by the backward pass.  Bound by
// HBM: one row read (two in the backward), one written.
#include "pm_host.h"
#include "pm_chan.h"

struct ActP {
  int64_t n_rows;
  int C;
  void* x;                 // forward: in/out
  const void* dy;          // backward
  const void* y;           // backward: activated forward rows (NULL without ReLU)
  void* out;               // backward
  const float* scale;      // [C] or NULL
  const float* shift;      // [C] or NULL
  int relu;
};

template <bool BF16, bool BWD, bool VEC>
__global__ void __launch_bounds__(256) k_affine_act(ActP p) {
  constexpr int CPL = BF16 ? 8 : 4;
  const int rpc = (p.C + CPL - 1) / CPL;                     // channel runs per row
  const int64_t n = p.n_rows * rpc;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / rpc;
    const int c0 = (int)(i - row * rpc) * CPL;
    float sc[CPL], sh[CPL], v[CPL];
#pragma unroll
    for (int q = 0; q < CPL; ++q) {
      const int c = min(c0 + q, p.C - 1);
      sc[q] = p.scale ? p.scale[c] : 1.f;
      sh[q] = (!BWD && p.shift) ? p.shift[c] : 0.f;
    }
    if constexpr (!BWD) {
      chan_load<BF16, CPL, VEC>(p.x, row * p.C, p.C, c0, v);
#pragma unroll
      for (int q = 0; q < CPL; ++q) {
        const float t = v[q] * sc[q] + sh[q];
        v[q] = p.relu ? fmaxf(t, 0.f) : t;
      }
      chan_store<BF16, CPL, VEC>(p.x, row * p.C, p.C, c0, v);
    } else {
      float y[CPL];
      chan_load<BF16, CPL, VEC>(p.dy, row * p.C, p.C, c0, v);
#pragma unroll
      for (int q = 0; q < CPL; ++q) y[q] = 1.f;
      if (p.relu) chan_load<BF16, CPL, VEC>(p.y, row * p.C, p.C, c0, y);
#pragma unroll
      for (int q = 0; q < CPL; ++q) v[q] = (y[q] > 0.f) ? v[q] * sc[q] : 0.f;
      chan_store<BF16, CPL, VEC>(p.out, row * p.C, p.C, c0, v);
    }
  }
}

template <bool BWD>
static pm_status act_launch(const ActP& p, int is_bf16, bool vec, hipStream_t st, const char* label) {
  if (p.n_rows == 0) return PM_OK;
  const int cpl = is_bf16 ? 8 : 4;
  const int64_t n = p.n_rows * ((p.C + cpl - 1) / cpl);
  const unsigned grid = (unsigned)std::min<int64_t>((n + 255) / 256, 8192);
  { ProfScope ps__(st, label);
    if (is_bf16) {
      if (vec) hipLaunchKernelGGL((k_affine_act<true, BWD, true>), dim3(grid), dim3(256), 0, st, p);
      else hipLaunchKernelGGL((k_affine_act<true, BWD, false>), dim3(grid), dim3(256), 0, st, p);
    } else {
      if (vec) hipLaunchKernelGGL((k_affine_act<false, BWD, true>), dim3(grid), dim3(256), 0, st, p);
      else hipLaunchKernelGGL((k_affine_act<false, BWD, false>), dim3(grid), dim3(256), 0, st, p);
    } }
  PM_CHECK_LAUNCH(label);
  return PM_OK;
}

pm_status pm_launch_affine_act(int64_t n_rows, int C, int is_bf16, void* x, const float* scale, const float* shift,
                               int relu, hipStream_t st) {
  if (!scale && !shift && !relu) return PM_OK;
  ActP p = {};
  p.n_rows = n_rows; p.C = C; p.x = x; p.scale = scale; p.shift = shift; p.relu = relu;
  return act_launch<false>(p, is_bf16, chan_vec_ok(C, is_bf16, x, x, x), st, "k_affine_act");
}

pm_status pm_launch_affine_act_bwd(int64_t n_rows, int C, int is_bf16, const void* dy, const void* y_saved,
                                   const float* scale, int relu, void* out, hipStream_t st) {
  ActP p = {};
  p.n_rows = n_rows; p.C = C; p.dy = dy; p.y = relu ? y_saved : nullptr; p.out = out; p.scale = scale; p.relu = relu;
  return act_launch<true>(p, is_bf16, chan_vec_ok(C, is_bf16, dy, relu ? y_saved : dy, out), st, "k_affine_act_bwd");
}
