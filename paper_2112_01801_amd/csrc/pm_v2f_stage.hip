// vertex2facet forward (Eq. 6) with LDS-staged facet tiles, for the memory-bound shapes bf16, Cin = 32 or 64:
//     g_f = sum_j W_j^T h_{v_j(f)},   W_j = sum_k B_k(e_j) W[k]   (the three folded matrices of the packed image)
// The work per facet is three gathered vertex rows (64 or 128 bytes), a 3 Cin x Cout contraction and one output row, so the
// kernel lives on its memory system.  A workgroup of 4 waves walks tiles of 128 facets: the 384 vertex rows of a
// tile are fetched with whole-row accesses (16 bytes a lane) into a padded LDS tile (the three rows of a facet side
// by side, as the concatenated operand row of the folded form), one tile
// ahead of the arithmetic (ids two tiles ahead), the matrix core takes its operand granules from LDS, and the
// output tile goes back through LDS so that it leaves in whole rows.  The folded weights (up to 48 KB) stay in LDS.
#include "pm_host.h"
#include "pm_device.h"

#define VT_ROWS 128                 /* facets per tile */
#define VT_STAGE_U4 (PM_STAGE_BYTES / 16)

struct VtP {
  int64_t F;
  int cout;
  const int32_t* facet;     // [F][3]
  const uint16_t* h;        // [V][CIN] bf16
  const uint4* apack;       // folded image: stage (nbg * NCH + ch)
  uint16_t* out;            // [F][cout] bf16
};

// CIN: 32 or 64.  NB: 32-wide output blocks (cout = 32 NB, 1..4).
template <int CIN, int NB>
__global__ void __launch_bounds__(256) k_v2f_stage(VtP p) {
  extern __shared__ uint4 vt_lds[];
  constexpr int NBG = (NB + 1) / 2;                 // weight stages hold two 32-wide blocks
  constexpr int NCH = (3 * CIN + 63) / 64;          // 64-channel chunks of the concatenated operand row
  constexpr int PPR = CIN / 8;                      // 16-byte pieces per vertex row
  constexpr int ROWB = NCH * 128;                   // operand row bytes (zero beyond 3 CIN channels)
  constexpr int PITCH = ROWB + 16;                  // + 16 of padding (bank spread)
  constexpr int ITEMS = VT_ROWS * 3 * PPR;          // 16-byte pieces per tile
  constexpr int PT = (ITEMS + 255) / 256;
  constexpr int TILE_BYTES = VT_ROWS * PITCH;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hh = lane >> 5;
  uint4* Wl = vt_lds;                                              // [NBG * NCH][VT_STAGE_U4]
  char* tile_lds = (char*)(vt_lds + NBG * NCH * VT_STAGE_U4);      // [VT_ROWS][PITCH]
  const int64_t n_tiles = (p.F + VT_ROWS - 1) / VT_ROWS;

  for (int i = tid; i < NBG * NCH * VT_STAGE_U4; i += 256) Wl[i] = p.apack[i];
  for (int i = tid; i < TILE_BYTES / 16; i += 256) ((uint4*)tile_lds)[i] = make_uint4(0, 0, 0, 0);   // the pad stays zero
  __syncthreads();

  // piece i of this thread: item = tid + 256 i -> (facet of the tile, corner, 16-byte piece of the vertex row)
  auto load_ids = [&](int64_t tile, int32_t (&vid)[PT]) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int item = tid + 256 * i;
      const int64_t f = tile * VT_ROWS + item / (3 * PPR);
      const int j = (item % (3 * PPR)) / PPR;
      vid[i] = (item < ITEMS && tile < n_tiles && f < p.F) ? p.facet[3 * f + j] : -1;
    }
  };
  auto load_rows = [&](const int32_t (&vid)[PT], uint4 (&x)[PT]) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int piece = (tid + 256 * i) % PPR;
      x[i] = make_uint4(0, 0, 0, 0);
      if (vid[i] >= 0) x[i] = *(const uint4*)(p.h + (int64_t)vid[i] * CIN + piece * 8);
    }
  };
  auto stage_rows = [&](const uint4 (&x)[PT]) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int item = tid + 256 * i;
      if (item < ITEMS) *(uint4*)(tile_lds + (item / (3 * PPR)) * PITCH + (item % (3 * PPR)) * 16) = x[i];
    }
  };

  int32_t vid[PT];
  uint4 x[PT];
  int64_t tile = blockIdx.x;
  load_ids(tile, vid);
  load_rows(vid, x);
  load_ids(tile + gridDim.x, vid);
  stage_rows(x);
  __syncthreads();
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
    const char* trow = tile_lds + (wave * 32 + r) * PITCH;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
#pragma unroll
      for (int g = 0; g < PM_GC; ++g) {
        const uint4 X = *(const uint4*)(trow + (ch * PM_GC + g) * 32 + 16 * hh);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const uint4 a = Wl[((nb >> 1) * NCH + ch) * VT_STAGE_U4 + (nb & 1) * PM_GC * 64 + g * 64 + lane];
          y[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, X),
                                                          y[nb], 0, 0, 0);
        }
      }
    }
    __syncthreads();                            // every wave is done with the staged rows of this tile
    // ---- output tile through the same LDS buffer: lane (r, hh) holds, per 32-wide block, channels
    //      q4 * 8 + hh * 4 + i of its facet; then whole rows leave in 16-byte pieces
    {
      constexpr int OP = 64 * NB + 16;          // padded output row pitch (bytes)
      static_assert(VT_ROWS * OP <= TILE_BYTES, "the output tile fits the staging buffer");
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          uint2 w;
          w.x = pack_bf16x2(y[nb][q4 * 4], y[nb][q4 * 4 + 1]);
          w.y = pack_bf16x2(y[nb][q4 * 4 + 2], y[nb][q4 * 4 + 3]);
          *(uint2*)(tile_lds + (wave * 32 + r) * OP + (nb * 32 + q4 * 8 + hh * 4) * 2) = w;
        }
      __syncthreads();
      const int64_t f0 = tile * VT_ROWS;
      constexpr int OPR = 4 * NB;               // 16-byte pieces per output row
#pragma unroll
      for (int i = 0; i < (VT_ROWS * OPR) / 256; ++i) {
        const int item = tid + 256 * i;
        const int row = item / OPR, piece = item % OPR;
        if (f0 + row < p.F)
          *(uint4*)(p.out + (f0 + row) * (32 * NB) + piece * 8) = *(const uint4*)(tile_lds + row * OP + piece * 16);
      }
      __syncthreads();
      // the output overwrote the zero pad of the rows it touched: restore it where the staged rows do not reach
      if (3 * CIN * 2 < ROWB) {
        constexpr int PADP = (ROWB - 3 * CIN * 2) / 16;   // 16-byte pieces of pad per row
        for (int i = tid; i < VT_ROWS * PADP; i += 256)
          *(uint4*)(tile_lds + (i / PADP) * PITCH + 3 * CIN * 2 + (i % PADP) * 16) = make_uint4(0, 0, 0, 0);
      }
    }
    stage_rows(x);                              // the next tile goes into the vacated buffer ...
    __syncthreads();                            // ... and is visible to every wave
  }
}

bool pm_v2f_stage_applies(pm_dtype dt, int cin, int cout, const void* h, const void* out) {
  return dt == PM_BF16 && (cin == 32 || cin == 64) && cout % 32 == 0 && cout >= 32 && cout <= 128 && pm_aligned16(h) &&
         pm_aligned16(out);
}

template <int CIN, int NB>
static pm_status v2f_stage_launch(const VtP& p, hipStream_t st) {
  constexpr int NBG = (NB + 1) / 2, NCH = (3 * CIN + 63) / 64;
  const size_t lds = (size_t)NBG * NCH * PM_STAGE_BYTES + (size_t)VT_ROWS * (NCH * 128 + 16);
  int64_t grid = (p.F + VT_ROWS - 1) / VT_ROWS;
  if (grid > 512) grid = 512;
  auto kern = k_v2f_stage<CIN, NB>;
  PM_CHECK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  { ProfScope ps__(st, "k_v2f_stage");
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p); }
  PM_CHECK_LAUNCH("k_v2f_stage");
  return PM_OK;
}

// apack: the folded packed image (pm_launch_pack with PACK_FOLD or PACK_SEP_FOLD), already enqueued on `st`
pm_status pm_launch_v2f_stage(int64_t F, int cin, int cout, const int32_t* facet, const void* h, const void* apack,
                              void* out, hipStream_t st) {
  if (F == 0) return PM_OK;
  VtP p;
  p.F = F; p.cout = cout; p.facet = facet; p.h = (const uint16_t*)h; p.apack = (const uint4*)apack; p.out = (uint16_t*)out;
  const int nb = cout / 32;
  if (cin == 32) {
    switch (nb) {
      case 1: return v2f_stage_launch<32, 1>(p, st);
      case 2: return v2f_stage_launch<32, 2>(p, st);
      case 3: return v2f_stage_launch<32, 3>(p, st);
      default: return v2f_stage_launch<32, 4>(p, st);
    }
  }
  switch (nb) {
    case 1: return v2f_stage_launch<64, 1>(p, st);
    case 2: return v2f_stage_launch<64, 2>(p, st);
    case 3: return v2f_stage_launch<64, 3>(p, st);
    default: return v2f_stage_launch<64, 4>(p, st);
  }
}
