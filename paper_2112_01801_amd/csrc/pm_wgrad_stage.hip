// Weight gradient without a basis, for the memory-bound shapes (bf16, Cin = 32 or 64, Cout = 32 .. 128):
//     M_j[ci][co] = sum_r X_j[r][ci] Y[r][co]
// NJ = 3: X_j[r] = h[facet[r][j]], the three corner matrices of vertex2facet (Eq. 6: dense backward, and dalpha / dP
// of the separable form); NJ = 1: X[r] = row r itself (dP of the point-wise stages).
// The contraction runs over the rows, so the matrix core wants, per lane, eight consecutive rows of one channel,
// while memory holds the channels of a row side by side.  Instead of transposing while staging (eight 2-byte LDS
// writes per 16 bytes loaded), the tiles sit in LDS as they sit in memory -- whole-row loads one tile ahead, ids
// two tiles ahead, as in the staged vertex2facet kernel -- and the operands are fetched with the LDS transposing
// read of gfx950 (ds_read_b64_tr_b16): within 16 lanes that address a block of 4 rows x 16 channels (lane l:
// row l / 4, channels 4 (l % 4) .. + 3), lane i receives the four rows of channel i.  Two such reads give a lane
// its eight rows; the four 16-lane groups of a wave cover the two channel halves and the two row halves of a
// 32 x 16 operand.
// Every workgroup walks a fixed set of tiles and writes its sums as one slice; the slices are added in a fixed
// order afterwards (bitwise reproducible, no atomics).
#include "pm_host.h"
#include "pm_device.h"

#define WS_ROWS 128                 /* rows per tile */
#define WS_TRY(expr) do { pm_status s__ = (expr); if (s__ != PM_OK) return s__; } while (0)

struct WsP {
  int64_t R;
  int cout;
  const int32_t* facet;     // NJ = 3: [R][3]
  const uint16_t* x;        // [.][CIN] bf16
  const uint16_t* y;        // [R][cout] bf16
  float* partial;           // [grid][NJ][CIN][cout]
};

typedef short ws_i16x4 __attribute__((ext_vector_type(4)));

// 32 channels x 16 rows of a row-major bf16 tile as a matrix-core operand: lane (c = lane % 32, half = lane / 32)
// gets rows row0 + 8 half .. + 7 of channel ch0 + c
__device__ __forceinline__ bf16x8 ws_frag(const char* tile, int pitch, int row0, int ch0, int lane) {
  const int g16 = lane >> 4, l16 = lane & 15;
  const char* a = tile + (row0 + 8 * (g16 >> 1) + (l16 >> 2)) * pitch + (ch0 + 16 * (g16 & 1) + 4 * (l16 & 3)) * 2;
  typedef ws_i16x4 __attribute__((address_space(3))) * lds_ptr;
  const ws_i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)a);
  const ws_i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(a + 4 * pitch));
  typedef short ws_i16x8 __attribute__((ext_vector_type(8)));
  const ws_i16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// CIN: 32 or 64.  NB: 32-wide blocks of Y channels (cout = 32 NB, 1..4).  NJ: 3 gathered corner rows or 1 direct row.
template <int CIN, int NB, int NJ>
__global__ void __launch_bounds__(256) k_wgrad_stage(WsP p) {
  extern __shared__ uint4 ws_lds[];
  constexpr int PPR = CIN / 8;                      // 16-byte pieces per source row
  constexpr int IPR = NJ * PPR;                     // X pieces per tile row
  constexpr int XPITCH = NJ * CIN * 2 + 16;
  constexpr int YPITCH = 64 * NB + 16;
  constexpr int XITEMS = WS_ROWS * IPR, YITEMS = WS_ROWS * 4 * NB;
  constexpr int XT = XITEMS / 256, YT = YITEMS / 256;
  constexpr int CB = CIN / 32;                      // 32-wide blocks of X channels
  constexpr int NBLK = CB * NB;                     // (ci block, co block) pairs, dealt to the four waves
  constexpr int T = (NBLK + 3) / 4;
  static_assert(XITEMS % 256 == 0 && YITEMS % 256 == 0, "whole passes of the workgroup");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  char* xt = (char*)ws_lds;                         // [WS_ROWS][XPITCH]
  char* yt = xt + WS_ROWS * XPITCH;                 // [WS_ROWS][YPITCH]
  const int64_t n_tiles = (p.R + WS_ROWS - 1) / WS_ROWS;

  auto load_ids = [&](int64_t tile, int32_t (&vid)[XT]) {
#pragma unroll
    for (int i = 0; i < XT; ++i) {
      const int item = tid + 256 * i;
      const int64_t r = tile * WS_ROWS + item / IPR;
      const int j = (item % IPR) / PPR;
      vid[i] = -1;
      if (tile < n_tiles && r < p.R) vid[i] = (NJ == 3) ? p.facet[3 * r + j] : (int32_t)r;
    }
  };
  auto load_rows = [&](int64_t tile, const int32_t (&vid)[XT], uint4 (&x)[XT], uint4 (&y)[YT]) {
#pragma unroll
    for (int i = 0; i < XT; ++i) {
      const int piece = (tid + 256 * i) % PPR;
      x[i] = make_uint4(0, 0, 0, 0);
      if (vid[i] >= 0) x[i] = *(const uint4*)(p.x + (int64_t)vid[i] * CIN + piece * 8);
    }
#pragma unroll
    for (int i = 0; i < YT; ++i) {
      const int item = tid + 256 * i;
      const int64_t r = tile * WS_ROWS + item / (4 * NB);
      y[i] = make_uint4(0, 0, 0, 0);
      if (tile < n_tiles && r < p.R) y[i] = *(const uint4*)(p.y + r * (32 * NB) + (item % (4 * NB)) * 8);
    }
  };
  auto stage = [&](const uint4 (&x)[XT], const uint4 (&y)[YT]) {
#pragma unroll
    for (int i = 0; i < XT; ++i) {
      const int item = tid + 256 * i;
      *(uint4*)(xt + (item / IPR) * XPITCH + (item % IPR) * 16) = x[i];
    }
#pragma unroll
    for (int i = 0; i < YT; ++i) {
      const int item = tid + 256 * i;
      *(uint4*)(yt + (item / (4 * NB)) * YPITCH + (item % (4 * NB)) * 16) = y[i];
    }
  };

  floatx16 acc[T][NJ];
#pragma unroll
  for (int t = 0; t < T; ++t)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[t][j][i] = 0.f;

  int32_t vid[XT];
  uint4 x[XT], y[YT];
  int64_t tile = blockIdx.x;
  load_ids(tile, vid);
  load_rows(tile, vid, x, y);
  load_ids(tile + gridDim.x, vid);
  stage(x, y);
  __syncthreads();
  for (; tile < n_tiles; tile += gridDim.x) {
    // next tile's rows and the ids of the one after: in flight during this tile's arithmetic
    load_rows(tile + gridDim.x, vid, x, y);
    load_ids(tile + 2 * (int64_t)gridDim.x, vid);
#pragma unroll
    for (int t = 0; t < T; ++t) {
      const int blk = wave + 4 * t;
      if (blk < NBLK) {                             // uniform per wave
        const int cb = blk / NB, nb = blk % NB;
#pragma unroll
        for (int s = 0; s < WS_ROWS / 16; ++s) {
          const bf16x8 yb = ws_frag(yt, YPITCH, 16 * s, nb * 32, lane);
#pragma unroll
          for (int j = 0; j < NJ; ++j) {
            const bf16x8 xa = ws_frag(xt, XPITCH, 16 * s, j * CIN + cb * 32, lane);
            acc[t][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, yb, acc[t][j], 0, 0, 0);
          }
        }
      }
    }
    __syncthreads();                            // every wave is done with this tile
    stage(x, y);
    __syncthreads();
  }

  // slice of this workgroup: lane (n = lane % 32, half) holds, per block, rows m = 8 q + 4 half + i of column n
  float* dst = p.partial + (int64_t)blockIdx.x * NJ * CIN * (32 * NB);
#pragma unroll
  for (int t = 0; t < T; ++t) {
    const int blk = wave + 4 * t;
    if (blk < NBLK) {
      const int cb = blk / NB, nb = blk % NB;
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          dst[((int64_t)(j * CIN + cb * 32 + m)) * (32 * NB) + nb * 32 + (lane & 31)] = acc[t][j][v];
        }
    }
  }
}

bool pm_wgrad_stage_applies(pm_dtype mt, BMode bm, XMode xm, XMode ym, int K, int Cc, int Cn, const RowSrc& xs,
                            const RowSrc& ys) {
  if (mt != PM_BF16 || bm != B_ONE || ym != X_DIRECT) return false;
  if (!((xm == X_GATHER_CAT && K == 3) || (xm == X_DIRECT && K == 1))) return false;
  if (!(Cc == 32 || Cc == 64) || Cn % 32 != 0 || Cn < 32 || Cn > 128) return false;
  return xs.is_bf16 && ys.is_bf16 && xs.C == Cc && ys.C == Cn && pm_aligned16(xs.p) && pm_aligned16(ys.p);
}

template <int CIN, int NB, int NJ>
static pm_status wgrad_stage_launch(const WsP& p, int grid, hipStream_t st) {
  const size_t lds = (size_t)WS_ROWS * (NJ * CIN * 2 + 16) + (size_t)WS_ROWS * (64 * NB + 16);
  auto kern = k_wgrad_stage<CIN, NB, NJ>;
  PM_TRY(pm_set_dyn_lds((const void*)kern, lds));
  { ProfScope ps__(st, "k_wgrad_stage");
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p); }
  PM_CHECK_LAUNCH("k_wgrad_stage");
  return PM_OK;
}

template <int NJ>
static pm_status wgrad_stage_dispatch(int cin, const WsP& p, int grid, hipStream_t st) {
  const int nb = p.cout / 32;
  if (cin == 32) {
    switch (nb) {
      case 1: return wgrad_stage_launch<32, 1, NJ>(p, grid, st);
      case 2: return wgrad_stage_launch<32, 2, NJ>(p, grid, st);
      case 3: return wgrad_stage_launch<32, 3, NJ>(p, grid, st);
      default: return wgrad_stage_launch<32, 4, NJ>(p, grid, st);
    }
  }
  switch (nb) {
    case 1: return wgrad_stage_launch<64, 1, NJ>(p, grid, st);
    case 2: return wgrad_stage_launch<64, 2, NJ>(p, grid, st);
    case 3: return wgrad_stage_launch<64, 3, NJ>(p, grid, st);
    default: return wgrad_stage_launch<64, 4, NJ>(p, grid, st);
  }
}

// dWp [K][Cc][Cn] fp32 (K = 3 corner matrices, or 1); ws holds the slices (at least one of K Cc Cn floats)
pm_status pm_launch_wgrad_stage(XMode xm, int64_t R, int K, int Cc, int Cn, const RowSrc& xs, const RowSrc& ys, float* dWp,
                                void* ws, size_t ws_bytes, hipStream_t st) {
  const int64_t n = (int64_t)K * Cc * Cn;
  int64_t grid = (R + WS_ROWS - 1) / WS_ROWS;
  if (grid > 512) grid = 512;
  if (grid > (int64_t)(ws_bytes / (n * sizeof(float)))) grid = (int64_t)(ws_bytes / (n * sizeof(float)));
  if (R > 0 && grid < 1) return pm_fail(PM_ERR_WORKSPACE, "wgrad workspace too small");
  if (R > 0) {
    WsP p;
    p.R = R; p.cout = Cn; p.facet = xs.facet; p.x = (const uint16_t*)xs.p; p.y = (const uint16_t*)ys.p;
    p.partial = (float*)ws;
    WS_TRY(xm == X_GATHER_CAT ? wgrad_stage_dispatch<3>(Cc, p, (int)grid, st) : wgrad_stage_dispatch<1>(Cc, p, (int)grid, st));
  } else {
    grid = 0;
  }
  return pm_launch_sum_slices((const float*)ws, n, (int)grid, dWp, st);
}
