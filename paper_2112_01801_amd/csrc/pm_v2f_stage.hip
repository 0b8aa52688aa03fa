// vertex2facet forward (Eq. 6) with LDS-staged facet tiles, for the memory-bound shapes bf16, Cin = 32 or 64:
//     g_f = sum_j W_j^T h_{v_j(f)},   W_j = sum_k B_k(e_j) W[k]   (the three folded matrices of the packed image)
// The work per facet is three gathered vertex rows (64 or 128 bytes), a 3 Cin x Cout contraction and one output
// row, so the kernel lives on its memory system.  A workgroup of 4 waves walks tiles of 128 facets, 32 per wave: the
// 96 vertex rows of a wave's facets are fetched with whole-row accesses (16 bytes a lane) into the wave's own padded
// LDS region (the three rows of a facet side by side, as the concatenated operand row of the folded form), one tile
// ahead of the arithmetic (ids two tiles ahead), the matrix core takes its operand granules from LDS, and the
// wave's output rows go back through the same region so that they leave in whole rows.  The folded weights (up to
// 48 KB) stay in LDS, shared and read-only; apart from their load there is no workgroup barrier: each wave runs its
// fetch / contract / store phases on its own, and the phases of the eight waves of a CU overlap.
//
// The same kernel serves, by template arguments,
//   * a point-wise matrix on directly addressed rows (NJ = 1: the tile is 128 consecutive rows), and
//   * the fused stages of the separable vertex2vertex block (FUSE): a per-channel affine map and ReLU on the
//     accumulators, an optional copy of these activated rows, and the depth-wise facet2vertex filter
//     s_f[c] = sum_k alpha2[k][c] B_k(n_f) (Eq. 5) multiplied in before the store.  The filter values come from the
//     matrix core in the accumulators' own layout, D[c][row] = sum_k alpha2[k][c] B_k(n_row), 16 basis functions
//     per 32x32x16 tile.  Both operands are split into a bf16 head and a bf16 remainder (x = hi + lo, |lo| <=
//     2^-9 |x|) and the three leading products hi hi + hi lo + lo hi are accumulated in fp32: the dropped lo lo
//     term is below 2^-16 of a product, so the filter keeps fp32 accuracy at a fifth of the fp32 tiles' cost.
#include "pm_host.h"
#include "pm_device.h"
#include "pm_rows.h"

#define VT_ROWS 128                 /* rows per tile */
#define VT_STAGE_U4 (PM_STAGE_BYTES / 16)

struct VtP {
  int64_t F;                // rows: facets (NJ = 3) or directly addressed rows (NJ = 1)
  int cout;
  const int32_t* facet;     // NJ = 3: [F][3]
  const uint16_t* h;        // [.][CIN] bf16
  const uint4* apack;       // packed image with one basis slot: stage (nbg * NCH + ch)
  uint16_t* out;            // [F][cout] bf16
  int tile_bytes;           // LDS bytes of the tile buffer
  const int32_t* row_ptr;   // optional (direct rows): output row r is divided by row_ptr[r + 1] - row_ptr[r]
  // FUSE only
  const float* ep_scale;    // [cout] or NULL (1)
  const float* ep_shift;    // [cout] or NULL (0)
  int relu;
  uint16_t* save;           // [F][cout] activated rows, or NULL
  const float* alpha2;      // [K2][cout] depth-wise coefficients, or NULL (no depth-wise stage)
  int K2;
  const float* vert;        // vertex positions (facet normals)
  ShTable sh;
};

__host__ __device__ constexpr int vt_nch(int cin, int nj) { return (nj * cin + 63) / 64; }
__host__ __device__ constexpr int vt_pitch(int cin, int nj) { return vt_nch(cin, nj) * 128 + 16; }
__host__ __device__ constexpr int vt_out_pitch(int nb, bool f32 = false) { return (f32 ? 128 : 64) * nb + 16; }

// CIN: 32 or 64 (direct rows also 96, 192).  NB: 32-wide output blocks (cout = 32 NB, 1..4).  NJ: 3 gathered corner
// rows or 1 direct row.
// Gathered rows: two workgroups share a CU (two waves per SIMD, 256 registers each) unless weights and tile leave
// LDS for one only.  Direct rows need fewer registers and are left to the compiler's own choice.
// OF32: the output rows are fp32 instead of bf16 (direct rows only).
template <int CIN, int NB, int NJ, bool FUSE, bool OF32 = false>
__global__ void __launch_bounds__(256, (NJ == 1 || (CIN == 64 && NB >= 3)) ? 1 : 2) k_v2f_stage(VtP p) {
  extern __shared__ uint4 vt_lds[];
  constexpr int NBG = (NB + 1) / 2;                 // weight stages hold two 32-wide blocks
  constexpr int NCH = vt_nch(CIN, NJ);              // 64-channel chunks of the concatenated operand row
  constexpr int PPR = CIN / 8;                      // 16-byte pieces per source row
  constexpr int IPR = NJ * PPR;                     // pieces per tile row
  constexpr int ROWB = NCH * 128;                   // operand row bytes (zero beyond NJ CIN channels)
  constexpr int PITCH = vt_pitch(CIN, NJ);          // + 16 of padding (bank spread)
  constexpr int ITEMS = VT_ROWS * IPR;              // 16-byte pieces per tile
  constexpr int PT = ITEMS / 256;
  constexpr int CO = 32 * NB;
  constexpr int OP = vt_out_pitch(NB, OF32);        // padded output row pitch (bytes)
  static_assert(ITEMS % 256 == 0, "whole passes of the workgroup");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hh = lane >> 5;
  const int NKC = FUSE ? (p.K2 + 15) >> 4 : 0;      // chunks of 16 basis functions
  const int KP = p.K2 | 1;                          // odd pitch of a basis row: conflict-free reads
  uint4* Wl = vt_lds;                                              // [NBG * NCH][VT_STAGE_U4]
  uint4* Aw = vt_lds + NBG * NCH * VT_STAGE_U4;                    // FUSE: [NKC][NB][hi, lo][64] coefficient operands
  float* Ep = (float*)(Aw + NKC * NB * 2 * 64);                    // FUSE: [2][CO] affine
  char* tile_lds = (char*)(Ep + (FUSE ? 2 * CO : 0));             // four wave regions of tile_bytes / 4
  // Every wave owns 32 rows of a tile and an LDS region of its own: the staged rows [32][PITCH], reused for the
  // wave's output rows [32][OP] and (FUSE) its basis rows behind them.  No wave touches another's region, so the
  // tile loop has no workgroup barrier: the waves of a CU drift apart and each other's memory latencies overlap.
  char* wl = tile_lds + wave * (p.tile_bytes / 4);
  float* Bw = (float*)(wl + 32 * OP);                              // FUSE: this wave's basis rows [32][KP]
  auto wave_sync = [] {    // LDS writes of the wave's lanes are visible to its other lanes
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  };
  const int64_t n_tiles = (p.F + VT_ROWS - 1) / VT_ROWS;

  for (int i = tid; i < NBG * NCH * VT_STAGE_U4; i += 256) Wl[i] = p.apack[i];
  if constexpr (FUSE) {
    // operand of lane (c = lane % 32, half = lane / 32) for chunk kc, block nb: alpha2[16 kc + 8 half + i][32 nb + c]
    for (int idx = tid; idx < NKC * NB * 2 * 64; idx += 256) {
      const int ln = idx & 63, part = (idx >> 6) & 1, nb = (idx >> 7) % NB, kc = (idx >> 7) / NB;
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int k = kc * 16 + 8 * (ln >> 5) + i;
        const float a = (k < p.K2) ? p.alpha2[k * CO + nb * 32 + (ln & 31)] : 0.f;
        v[i] = part ? a - bf16_to_f32((uint16_t)f32_to_bf16_bits(a)) : a;
      }
      Aw[idx] = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
    }
    for (int i = tid; i < CO; i += 256) {
      Ep[i] = p.ep_scale ? p.ep_scale[i] : 1.f;
      Ep[CO + i] = p.ep_shift ? p.ep_shift[i] : 0.f;
    }
  }
  for (int i = tid; i < p.tile_bytes / 16; i += 256) ((uint4*)tile_lds)[i] = make_uint4(0, 0, 0, 0);   // the pad stays zero
  __syncthreads();

  // piece i of this lane: item = lane + 64 i -> (row of the wave's 32, corner, 16-byte piece of the source row)
  auto load_ids = [&](int64_t tile, int32_t (&vid)[PT]) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int item = lane + 64 * i;
      const int64_t f = tile * VT_ROWS + wave * 32 + item / IPR;
      const int j = (item % IPR) / PPR;
      vid[i] = -1;
      if (tile < n_tiles && f < p.F) vid[i] = (NJ == 3) ? p.facet[3 * f + j] : (int32_t)f;
    }
  };
  auto load_rows = [&](const int32_t (&vid)[PT], uint4 (&x)[PT]) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int piece = (lane + 64 * i) % PPR;
      x[i] = make_uint4(0, 0, 0, 0);
      if (vid[i] >= 0) x[i] = *(const uint4*)(p.h + (int64_t)vid[i] * CIN + piece * 8);
    }
  };
  auto stage_rows = [&](const uint4 (&x)[PT]) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int item = lane + 64 * i;
      *(uint4*)(wl + (item / IPR) * PITCH + (item % IPR) * 16) = x[i];
    }
  };
  // FUSE with the depth-wise stage: corner ids of the lane's own facet (one tile ahead), then its corner positions
  const bool dw = FUSE && p.alpha2 != nullptr;
  int32_t fid[3] = {0, 0, 0};
  auto load_fid = [&](int64_t tile) {
    const int64_t f = min(tile * VT_ROWS + wave * 32 + r, p.F - 1);
#pragma unroll
    for (int j = 0; j < 3; ++j) fid[j] = p.facet[3 * f + j];
  };

  int32_t vid[PT];
  uint4 x[PT];
  int64_t tile = blockIdx.x;
  load_ids(tile, vid);
  if (dw) load_fid(tile);
  load_rows(vid, x);
  load_ids(tile + gridDim.x, vid);
  stage_rows(x);
  wave_sync();
  for (; tile < n_tiles; tile += gridDim.x) {
    DirRaw dr;
    if (dw) {
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const float* q = p.vert + 3 * (int64_t)fid[j];
        dr.v[3 * j] = q[0]; dr.v[3 * j + 1] = q[1]; dr.v[3 * j + 2] = q[2];
      }
    }
    // next tile's rows and the ids of the one after: in flight during this tile's arithmetic
    load_rows(vid, x);
    load_ids(tile + 2 * (int64_t)gridDim.x, vid);
    if (dw) load_fid(tile + gridDim.x);

    // ---- this wave's 32 rows: operand granules from the staged tile, weights from LDS
    floatx16 y[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) y[nb][i] = 0.f;
    const char* trow = wl + r * PITCH;
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
    wave_sync();                                // the wave is done with its staged rows of this tile

    // the tile of accumulators leaves through the LDS buffer: lane (r, hh) holds, per 32-wide block, channels
    // q4 * 8 + hh * 4 + i of its row; whole rows then go out in 16-byte pieces
    const int64_t f0 = tile * VT_ROWS + wave * 32;   // the wave's first row
    auto store_tile = [&](uint16_t* dst) {
      constexpr int ESZ = OF32 ? 4 : 2;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          char* q = wl + r * OP + (nb * 32 + q4 * 8 + hh * 4) * ESZ;
          if constexpr (OF32) {
            *(float4*)q = make_float4(y[nb][q4 * 4], y[nb][q4 * 4 + 1], y[nb][q4 * 4 + 2], y[nb][q4 * 4 + 3]);
          } else {
            uint2 w;
            w.x = pack_bf16x2(y[nb][q4 * 4], y[nb][q4 * 4 + 1]);
            w.y = pack_bf16x2(y[nb][q4 * 4 + 2], y[nb][q4 * 4 + 3]);
            *(uint2*)q = w;
          }
        }
      wave_sync();
      constexpr int OPR = 4 * NB * (ESZ / 2);   // 16-byte pieces per output row
#pragma unroll
      for (int i = 0; i < (32 * OPR) / 64; ++i) {
        const int item = lane + 64 * i;
        const int row = item / OPR, piece = item % OPR;
        if (f0 + row < p.F)
          *(uint4*)((char*)dst + ((f0 + row) * CO * ESZ + piece * 16)) = *(const uint4*)(wl + row * OP + piece * 16);
      }
      wave_sync();
    };

    if constexpr (FUSE) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int co = nb * 32 + q4 * 8 + hh * 4;
          const float4 sc = *(const float4*)(Ep + co), sh = *(const float4*)(Ep + CO + co);
          const float scv[4] = {sc.x, sc.y, sc.z, sc.w}, shv[4] = {sh.x, sh.y, sh.z, sh.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float v = y[nb][q4 * 4 + i] * scv[i] + shv[i];
            y[nb][q4 * 4 + i] = p.relu ? fmaxf(v, 0.f) : v;
          }
        }
      if (p.save) store_tile(p.save);
      if (dw) {
        float nx, ny, nz;
        dir_finish<B_NORMAL>(dr, nx, ny, nz);
        constexpr bool L3REG = !(CIN == 32 && NB == 4);   // that instance has no registers to spare
        if (L3REG && p.sh.L == 3 && p.K2 == 16) {
          // L = 3: the 16 basis values of the lane's facet stay in registers (unrolled recurrence); the lane's operand
          // -- functions 8 hh .. 8 hh + 7 of its row -- is selected from them and split into head and remainder: no
          // LDS round trip, one chunk of 16 functions
          float b0[8], b1[8];        // two arrays: a select between elements of one would become a run-time index
          sh_eval<3>(nx, ny, nz, p.sh, [&](int k, float v) {
            if (k < 8) b0[k] = v;
            else b1[k - 8] = v;
          });
          float v[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) v[i] = hh ? b1[i] : b0[i];
          const uint4 bh = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                                      pack_bf16x2(v[6], v[7]));
          const uint32_t hw[4] = {bh.x, bh.y, bh.z, bh.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            v[2 * i] -= bf16lo_to_f32(hw[i]);
            v[2 * i + 1] -= bf16hi_to_f32(hw[i]);
          }
          const uint4 bl = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                                      pack_bf16x2(v[6], v[7]));
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            floatx16 S;
#pragma unroll
            for (int i = 0; i < 16; ++i) S[i] = 0.f;
            const bf16x8 ah = __builtin_bit_cast(bf16x8, Aw[(nb * 2 + 0) * 64 + lane]);
            const bf16x8 al = __builtin_bit_cast(bf16x8, Aw[(nb * 2 + 1) * 64 + lane]);
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, __builtin_bit_cast(bf16x8, bh), S, 0, 0, 0);
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, __builtin_bit_cast(bf16x8, bl), S, 0, 0, 0);
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, __builtin_bit_cast(bf16x8, bh), S, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 16; ++i) y[nb][i] *= S[i];
          }
        } else {
          // basis of the wave's 32 facets into its own LDS rows (both half-waves hold the same rows), then the
          // filter values of every accumulator element from the fp32 matrix core
          sh_eval_any(nx, ny, nz, p.sh, [&](int k, float v) {
            if (hh == 0) Bw[r * KP + k] = v;
          });
          __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
          __builtin_amdgcn_wave_barrier();
          // per 32-wide block and chunk of 16 basis functions: the lane's basis operand (functions 16 kc + 8 hh + i
          // of its row) split into head and remainder, then the three leading products
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            floatx16 S;
#pragma unroll
            for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll 1
            for (int kc = 0; kc < NKC; ++kc) {
              float v[8];
#pragma unroll
              for (int i = 0; i < 8; ++i) {
                const int k = kc * 16 + 8 * hh + i;
                v[i] = (k < p.K2) ? Bw[r * KP + k] : 0.f;
              }
              const uint4 bh = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                                          pack_bf16x2(v[6], v[7]));
              const uint32_t hw[4] = {bh.x, bh.y, bh.z, bh.w};
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                v[2 * i] -= bf16lo_to_f32(hw[i]);
                v[2 * i + 1] -= bf16hi_to_f32(hw[i]);
              }
              const uint4 bl = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                                          pack_bf16x2(v[6], v[7]));
              const bf16x8 ah = __builtin_bit_cast(bf16x8, Aw[((kc * NB + nb) * 2 + 0) * 64 + lane]);
              const bf16x8 al = __builtin_bit_cast(bf16x8, Aw[((kc * NB + nb) * 2 + 1) * 64 + lane]);
              S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, __builtin_bit_cast(bf16x8, bh), S, 0, 0, 0);
              S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, __builtin_bit_cast(bf16x8, bl), S, 0, 0, 0);
              S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, __builtin_bit_cast(bf16x8, bh), S, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) y[nb][i] *= S[i];
          }
          __builtin_amdgcn_wave_barrier();        // the basis rows have been read
        }
      }
    }
    if constexpr (NJ == 1 && !FUSE) {
      if (p.row_ptr) {                          // the mean's weight of the row, applied once here for its consumers
        const int64_t row = min(f0 + r, p.F - 1);
        const int32_t deg = p.row_ptr[row + 1] - p.row_ptr[row];
        const float w = deg > 0 ? 1.0f / (float)deg : 0.f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int i = 0; i < 16; ++i) y[nb][i] *= w;
      }
    }
    store_tile(p.out);
    // the output and the basis rows overwrote the zero pad of the rows they touched: restore it where the staged
    // rows do not reach
    if constexpr (NJ * CIN * 2 < ROWB) {
      constexpr int PADP = (ROWB - NJ * CIN * 2) / 16;   // 16-byte pieces of pad per row
      for (int i = lane; i < 32 * PADP; i += 64)
        *(uint4*)(wl + (i / PADP) * PITCH + NJ * CIN * 2 + (i % PADP) * 16) = make_uint4(0, 0, 0, 0);
    }
    stage_rows(x);                              // the wave's rows of the next tile go into the vacated region ...
    wave_sync();                                // ... and are visible to all its lanes
  }
}

bool pm_v2f_stage_applies(pm_dtype dt, int cin, int cout, const void* h, const void* out) {
  return dt == PM_BF16 && (cin == 32 || cin == 64) && cout % 32 == 0 && cout >= 32 && cout <= 128 && pm_aligned16(h) &&
         pm_aligned16(out);
}

template <int CIN, int NB, int NJ, bool FUSE, bool OF32 = false>
static pm_status v2f_stage_launch(VtP& p, hipStream_t st, const char* label) {
  constexpr int NBG = (NB + 1) / 2, NCH = vt_nch(CIN, NJ);
  const int nkc = FUSE ? (p.K2 + 15) / 16 : 0;
  const int bw = (FUSE && p.alpha2) ? 4 * 32 * (p.K2 | 1) * 4 : 0;
  // four wave regions: 32 staged rows, or 32 output rows and the wave's basis rows behind them
  p.tile_bytes = 4 * (int)pm_round_up((size_t)std::max(32 * vt_pitch(CIN, NJ), 32 * vt_out_pitch(NB, OF32) + bw / 4), 16);
  const size_t lds = (size_t)NBG * NCH * PM_STAGE_BYTES + (FUSE ? (size_t)nkc * NB * 2 * 1024 + 2 * 32 * NB * 4 : 0) + p.tile_bytes;
  if (lds > 160 * 1024) return pm_fail(PM_ERR_UNSUPPORTED, "staged tiles: %zu bytes of LDS", lds);
  int64_t grid = (p.F + VT_ROWS - 1) / VT_ROWS;
  if (grid > 512) grid = 512;
  auto kern = k_v2f_stage<CIN, NB, NJ, FUSE, OF32>;
  PM_TRY(pm_set_dyn_lds((const void*)kern, lds));
  { ProfScope ps__(st, label);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p); }
  PM_CHECK_LAUNCH(label);
  return PM_OK;
}

template <int NJ, bool FUSE, bool OF32 = false>
static pm_status v2f_stage_dispatch(int cin, VtP& p, hipStream_t st, const char* label) {
  const int nb = p.cout / 32;
  if (cin == 32) {
    switch (nb) {
      case 1: return v2f_stage_launch<32, 1, NJ, FUSE, OF32>(p, st, label);
      case 2: return v2f_stage_launch<32, 2, NJ, FUSE, OF32>(p, st, label);
      case 3: return v2f_stage_launch<32, 3, NJ, FUSE, OF32>(p, st, label);
      default: return v2f_stage_launch<32, 4, NJ, FUSE, OF32>(p, st, label);
    }
  }
  switch (nb) {
    case 1: return v2f_stage_launch<64, 1, NJ, FUSE, OF32>(p, st, label);
    case 2: return v2f_stage_launch<64, 2, NJ, FUSE, OF32>(p, st, label);
    case 3: return v2f_stage_launch<64, 3, NJ, FUSE, OF32>(p, st, label);
    default: return v2f_stage_launch<64, 4, NJ, FUSE, OF32>(p, st, label);
  }
}

// apack: the folded packed image (pm_launch_pack with PACK_FOLD or PACK_SEP_FOLD), already enqueued on `st`
pm_status pm_launch_v2f_stage(int64_t F, int cin, int cout, const int32_t* facet, const void* h, const void* apack,
                              void* out, hipStream_t st) {
  if (F == 0) return PM_OK;
  VtP p = {};
  p.F = F; p.cout = cout; p.facet = facet; p.h = (const uint16_t*)h; p.apack = (const uint4*)apack; p.out = (uint16_t*)out;
  return v2f_stage_dispatch<3, false>(cin, p, st, "k_v2f_stage");
}

// Fused stages of the separable vertex2vertex block.  facet != NULL: gathered corner rows (apack = folded image of
// 3 cin x cout), optional depth-wise facet2vertex filter (alpha2, K2 = (L+1)^2 of sh, vert).  facet == NULL: a
// point-wise matrix on R consecutive rows (apack = plain image of cin x cout).  Either way the accumulators pass
// through scale/shift (NULL: 1 / 0) and ReLU (relu != 0) first, and `save` (optional) receives them at that point.
pm_status pm_launch_v2v_stage(int64_t R, int cin, int cout, const int32_t* facet, const void* h, const void* apack,
                              const float* ep_scale, const float* ep_shift, int relu, void* save, const float* alpha2,
                              int K2, const float* vert, const ShTable* sh, void* out, hipStream_t st) {
  if (R == 0) return PM_OK;
  VtP p = {};
  p.F = R; p.cout = cout; p.facet = facet; p.h = (const uint16_t*)h; p.apack = (const uint4*)apack; p.out = (uint16_t*)out;
  p.ep_scale = ep_scale; p.ep_shift = ep_shift; p.relu = relu; p.save = (uint16_t*)save;
  p.alpha2 = facet ? alpha2 : nullptr; p.K2 = p.alpha2 ? K2 : 0; p.vert = vert;
  if (sh) p.sh = *sh;
  if (facet) return v2f_stage_dispatch<3, true>(cin, p, st, "k_v2v_facet");
  return v2f_stage_dispatch<1, true>(cin, p, st, "k_v2v_point");
}

// Point-wise matrix on R consecutive bf16 rows with fp32 output rows (apack: plain or transposed image of cin x cout);
// row_ptr (optional): row r leaves divided by row_ptr[r + 1] - row_ptr[r] (0 for an empty segment)
pm_status pm_launch_point_stage_f32(int64_t R, int cin, int cout, const void* rows, const void* apack, float* out,
                                    const int32_t* row_ptr, hipStream_t st) {
  if (R == 0) return PM_OK;
  VtP p = {};
  p.F = R; p.cout = cout; p.h = (const uint16_t*)rows; p.apack = (const uint4*)apack; p.out = (uint16_t*)out;
  p.row_ptr = row_ptr;
  return v2f_stage_dispatch<1, false, true>(cin, p, st, "k_point_stage");
}

// Point-wise matrix on R consecutive bf16 rows of 96 or 192 channels (the three corner-slot sums of a vertex side
// by side: dense vertex2facet backward), bf16 output rows of cout = 32 .. 128 channels
bool pm_point_stage_wide_applies(pm_dtype dt, int cin, int cout, const void* rows, const void* out) {
  return dt == PM_BF16 && (cin == 96 || cin == 192) && cout % 32 == 0 && cout >= 32 && cout <= 128 && pm_aligned16(rows) &&
         pm_aligned16(out);
}

pm_status pm_launch_point_stage_wide(int64_t R, int cin, int cout, const void* rows, const void* apack, void* out,
                                     hipStream_t st) {
  if (R == 0) return PM_OK;
  VtP p = {};
  p.F = R; p.cout = cout; p.h = (const uint16_t*)rows; p.apack = (const uint4*)apack; p.out = (uint16_t*)out;
  const char* label = "k_point_stage";
  const int nb = cout / 32;
  if (cin == 96) {
    switch (nb) {
      case 1: return v2f_stage_launch<96, 1, 1, false>(p, st, label);
      case 2: return v2f_stage_launch<96, 2, 1, false>(p, st, label);
      case 3: return v2f_stage_launch<96, 3, 1, false>(p, st, label);
      default: return v2f_stage_launch<96, 4, 1, false>(p, st, label);
    }
  }
  switch (nb) {
    case 1: return v2f_stage_launch<192, 1, 1, false>(p, st, label);
    case 2: return v2f_stage_launch<192, 2, 1, false>(p, st, label);
    case 3: return v2f_stage_launch<192, 3, 1, false>(p, st, label);
    default: return v2f_stage_launch<192, 4, 1, false>(p, st, label);
  }
}
