// vertex2facet forward (Eq. 6) with LDS-staged facet tiles, for the memory-bound shape bf16, Cin = 64:
//     g_f = sum_j W_j^T h_{v_j(f)},   W_j = sum_k B_k(e_j) W[k]   (the three folded matrices of the packed image)
// The work per facet is three gathered 128-byte vertex rows, a 192 x Cout contraction and one output row, so the
// kernel lives on its memory system.  A workgroup of 4 waves walks tiles of 128 facets: the 384 vertex rows of a
// tile are fetched with fully coalesced accesses (8 lanes x 16 bytes per row) into a padded LDS tile, one tile
// ahead of the arithmetic (ids two tiles ahead), the matrix core takes its operand granules from LDS, and the
// output tile goes back through LDS so that it leaves in whole 128-byte rows.  The folded weights (24 or 48 KB)
// stay in LDS.
#include "pm_host.h"
#include "pm_device.h"

#define VT_ROWS 128                 /* facets per tile */
#define VT_PITCH 144                /* bytes per staged vertex row: 128 + 16 of padding (bank spread) */
#define VT_ITEMS (VT_ROWS * 3 * 8)  /* 16-byte pieces per tile */
#define VT_PER_THREAD (VT_ITEMS / 256)
#define VT_STAGE_U4 (PM_STAGE_BYTES / 16)

struct VtP {
  int64_t F;
  int NBG;                  // groups of 64 output channels (1 or 2)
  const int32_t* facet;     // [F][3]
  const uint16_t* h;        // [V][64] bf16
  const uint4* apack;       // folded image: stage (nbg * 3 + j)
  uint16_t* out;            // [F][64 NBG] bf16
};

template <int NB>
__global__ void __launch_bounds__(256) k_v2f_stage(VtP p) {
  extern __shared__ uint4 vt_lds[];
  constexpr int NBG = NB / 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hh = lane >> 5;
  uint4* Wl = vt_lds;                                              // [NBG * 3][VT_STAGE_U4]
  char* tiles = (char*)(vt_lds + NBG * 3 * VT_STAGE_U4);           // [2][VT_ROWS * 3][VT_PITCH]
  constexpr int TILE_BYTES = VT_ROWS * 3 * VT_PITCH;
  const int64_t n_tiles = (p.F + VT_ROWS - 1) / VT_ROWS;

  for (int i = tid; i < NBG * 3 * VT_STAGE_U4; i += 256) Wl[i] = p.apack[i];

  // piece i of this thread: item = tid + 256 i -> (facet of the tile, corner, 16-byte piece of the row)
  auto load_ids = [&](int64_t tile, int32_t (&vid)[VT_PER_THREAD]) {
#pragma unroll
    for (int i = 0; i < VT_PER_THREAD; ++i) {
      const int item = tid + 256 * i;
      const int64_t f = tile * VT_ROWS + item / 24;
      const int j = (item % 24) >> 3;
      vid[i] = (tile < n_tiles && f < p.F) ? p.facet[3 * f + j] : -1;
    }
  };
  auto load_rows = [&](const int32_t (&vid)[VT_PER_THREAD], uint4 (&x)[VT_PER_THREAD]) {
#pragma unroll
    for (int i = 0; i < VT_PER_THREAD; ++i) {
      const int piece = (tid + 256 * i) & 7;
      x[i] = make_uint4(0, 0, 0, 0);
      if (vid[i] >= 0) x[i] = *(const uint4*)(p.h + (int64_t)vid[i] * 64 + piece * 8);
    }
  };
  auto stage_rows = [&](int buf, const uint4 (&x)[VT_PER_THREAD]) {
#pragma unroll
    for (int i = 0; i < VT_PER_THREAD; ++i) {
      const int item = tid + 256 * i;
      *(uint4*)(tiles + buf * TILE_BYTES + (item >> 3) * VT_PITCH + (item & 7) * 16) = x[i];
    }
  };

  int32_t vid[VT_PER_THREAD];
  uint4 x[VT_PER_THREAD];
  int64_t tile = blockIdx.x;
  load_ids(tile, vid);
  load_rows(vid, x);
  load_ids(tile + gridDim.x, vid);
  stage_rows(0, x);
  __syncthreads();
  int buf = 0;
  for (; tile < n_tiles; tile += gridDim.x) {
    // next tile's rows and the ids of the one after: in flight during this tile's arithmetic
    load_rows(vid, x);
    load_ids(tile + 2 * (int64_t)gridDim.x, vid);

    // ---- this wave's 32 facets: operand granules from the staged tile, folded weights from LDS
    floatx16 y[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) y[nb][i] = 0.f;
    const char* trow = tiles + buf * TILE_BYTES + (wave * 32 + r) * 3 * VT_PITCH;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
#pragma unroll
      for (int g = 0; g < PM_GC; ++g) {
        const uint4 X = *(const uint4*)(trow + j * VT_PITCH + 32 * g + 16 * hh);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const uint4 a = Wl[((nb >> 1) * 3 + j) * VT_STAGE_U4 + (nb & 1) * PM_GC * 64 + g * 64 + lane];
          y[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, X),
                                                          y[nb], 0, 0, 0);
        }
      }
    }
    __syncthreads();                            // every wave is done with the staged rows of this tile
    // ---- output tile through the same LDS buffer: lane (r, hh) holds, per 32-wide block, channels
    //      q4 * 8 + hh * 4 + i of its facet; rows of 128 NBG bytes, then whole rows leave in 16-byte pieces
    {
      char* ot = tiles + buf * TILE_BYTES;
      constexpr int OP = 128 * NBG + 16;        // padded output row pitch
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          uint2 w;
          w.x = pack_bf16x2(y[nb][q4 * 4], y[nb][q4 * 4 + 1]);
          w.y = pack_bf16x2(y[nb][q4 * 4 + 2], y[nb][q4 * 4 + 3]);
          *(uint2*)(ot + (wave * 32 + r) * OP + (nb * 32 + q4 * 8 + hh * 4) * 2) = w;
        }
      __syncthreads();
      const int64_t f0 = tile * VT_ROWS;
      constexpr int PPR = 8 * NBG;              // 16-byte pieces per output row
#pragma unroll
      for (int i = 0; i < (VT_ROWS * PPR) / 256; ++i) {
        const int item = tid + 256 * i;
        const int row = item / PPR, piece = item % PPR;
        if (f0 + row < p.F)
          *(uint4*)(p.out + (f0 + row) * (64 * NBG) + piece * 8) = *(const uint4*)(ot + row * OP + piece * 16);
      }
    }
    __syncthreads();                            // the buffer is free again
    stage_rows(buf, x);                         // (the next tile goes into the buffer just vacated ...
    __syncthreads();                            //  ... and is visible to every wave)
  }
}

bool pm_v2f_stage_applies(pm_dtype dt, int cin, int cout, const void* h, const void* out) {
  return dt == PM_BF16 && cin == 64 && (cout == 64 || cout == 128) && pm_aligned16(h) && pm_aligned16(out);
}

// apack: the folded packed image (pm_launch_pack with PACK_FOLD or PACK_SEP_FOLD), already enqueued on `st`
pm_status pm_launch_v2f_stage(int64_t F, int cout, const int32_t* facet, const void* h, const void* apack, void* out,
                              hipStream_t st) {
  if (F == 0) return PM_OK;
  VtP p;
  p.F = F; p.NBG = cout / 64; p.facet = facet; p.h = (const uint16_t*)h; p.apack = (const uint4*)apack;
  p.out = (uint16_t*)out;
  const size_t lds = (size_t)p.NBG * 3 * PM_STAGE_BYTES + (size_t)VT_ROWS * 3 * VT_PITCH;
  int64_t grid = (F + VT_ROWS - 1) / VT_ROWS;
  if (grid > 512) grid = 512;
  auto kern = p.NBG == 1 ? k_v2f_stage<2> : k_v2f_stage<4>;
  PM_CHECK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  { ProfScope ps__(st, "k_v2f_stage");
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p); }
  PM_CHECK_LAUNCH("k_v2f_stage");
  return PM_OK;
}
