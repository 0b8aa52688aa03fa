// conv_rows kernel template and its per-degree launcher (included by the pm_conv_i*.hip instance files).
#pragma once
#include "pm_rows.h"

#define STAGE_U4 (PM_STAGE_BYTES / 16) /* 512 uint4 per stage */

// ------------------------------------------------------------------------------------------------
// conv_rows
// ------------------------------------------------------------------------------------------------
struct ConvP {
  int64_t R;
  int Cc, Cn, NCH, NBG;
  int resident;          // all stages fit in LDS
  BasisSrc bs;
  RowSrc xs;
  const uint4* apack;
  void* out;
  int out_bf16;
  int store_fast;        // Cn % 64 == 0 and the output rows are 16-byte aligned: unguarded vector stores
};

template <int DT>
__device__ __forceinline__ uint4 pack_granule(const float* v) {
  uint4 o;
  if constexpr (DT == 1) {
    o.x = pack_bf16x2(v[0], v[1]); o.y = pack_bf16x2(v[2], v[3]);
    o.z = pack_bf16x2(v[4], v[5]); o.w = pack_bf16x2(v[6], v[7]);
  } else {
    o.x = __float_as_uint(v[0]); o.y = __float_as_uint(v[1]);
    o.z = __float_as_uint(v[2]); o.w = __float_as_uint(v[3]);
  }
  return o;
}

// one c-group of the contraction: 16 channels (bf16) or 8 channels (fp32, four k=2 steps)
template <int DT>
__device__ __forceinline__ floatx16 mma_group(uint4 a, uint4 x, floatx16 c) {
  if constexpr (DT == 1) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, x), c, 0,
                                                   0, 0);
  } else {
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(x.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(x.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(x.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(x.w), c, 0, 0, 0);
    return c;
  }
}

// Fast path of the operand fetch (conditions checked on the host: storage dtype == MFMA dtype, rows
// 16-byte aligned, every granule inside its row).  Straight-line code in two halves -- loads only, then
// arithmetic -- so that the loads of a whole tile can be in flight while the previous tile is multiplied.
// `rowc` is a row index clamped into range; rows past the end are masked at the store.
template <int XM> struct NRaw { static constexpr int n = (XM == X_GATHER_SUM) ? 3 : 1; };

template <int XM, int DT>
__device__ __forceinline__ void granule_load(const RowSrc& s, int64_t rowc, const RowMeta& m, int c0,
                                             uint4 (&raw)[NRaw<XM>::n]) {
  constexpr int ESZ = (DT == 1) ? 2 : 4;
  const char* base = (const char*)s.p;
  if constexpr (XM == X_DIRECT) {
    raw[0] = *(const uint4*)(base + (rowc * (int64_t)s.C + c0) * ESZ);
  } else if constexpr (XM == X_GATHER_CAT) {
    const int j = c0 / s.C, cc = c0 - j * s.C;
    const int32_t id = (j == 0) ? m.id[0] : (j == 1 ? m.id[1] : m.id[2]);
    raw[0] = *(const uint4*)(base + ((int64_t)id * s.C + cc) * ESZ);
  } else {
#pragma unroll
    for (int j = 0; j < NRaw<XM>::n; ++j) raw[j] = *(const uint4*)(base + ((int64_t)m.id[j] * s.C + c0) * ESZ);
  }
}

template <int XM, int DT>
__device__ __forceinline__ uint4 granule_finish(const uint4 (&raw)[NRaw<XM>::n], const RowMeta& m) {
  if constexpr (XM == X_DIRECT || XM == X_GATHER_CAT) {
    return raw[0];   // storage format == operand format
  } else {
    constexpr int EPG = (DT == 1) ? 8 : 4;
    float acc[EPG];
#pragma unroll
    for (int j = 0; j < NRaw<XM>::n; ++j) {
      float t[EPG];
      if constexpr (DT == 1) {
        t[0] = bf16lo_to_f32(raw[j].x); t[1] = bf16hi_to_f32(raw[j].x); t[2] = bf16lo_to_f32(raw[j].y);
        t[3] = bf16hi_to_f32(raw[j].y); t[4] = bf16lo_to_f32(raw[j].z); t[5] = bf16hi_to_f32(raw[j].z);
        t[6] = bf16lo_to_f32(raw[j].w); t[7] = bf16hi_to_f32(raw[j].w);
      } else {
        t[0] = __uint_as_float(raw[j].x); t[1] = __uint_as_float(raw[j].y);
        t[2] = __uint_as_float(raw[j].z); t[3] = __uint_as_float(raw[j].w);
      }
#pragma unroll
      for (int i = 0; i < EPG; ++i) acc[i] = (j == 0) ? t[i] * m.w[0] : acc[i] + t[i] * m.w[j];
    }
    return pack_granule<DT>(acc);
  }
}

template <int XM, int DT>
__device__ __forceinline__ uint4 fetch_granule_fast(const RowSrc& s, int64_t rowc, const RowMeta& m, int c0) {
  uint4 raw[NRaw<XM>::n];
  granule_load<XM, DT>(s, rowc, m, c0, raw);
  return granule_finish<XM, DT>(raw, m);
}

// FM: 0 = general operand fetch, 1 = branch-free fetch (whole chunks of channels), 2 = the same with a last chunk that is
// only partly inside the row (granules at or beyond Cc are zero instead of loaded)
template <int DT, int BM, int XM, int LT, int NW, bool RES, int FM>
__global__ void __launch_bounds__(NW * 64) k_conv_rows(ConvP p) {
  constexpr bool FAST = FM != 0;
  extern __shared__ uint4 lds[];
  constexpr int K = (BM == B_ONE) ? 1 : (LT + 1) * (LT + 1);
  constexpr int NT = NW * 64;
  constexpr int EPG = (DT == 1) ? 8 : 4;       // channels per 16-byte granule
  constexpr int PER_T = STAGE_U4 / NT;         // uint4 per thread per stage copy
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int NCH = p.NCH, NBG = p.NBG;
  const int64_t S = (int64_t)NBG * NCH * K;
  const int64_t n_tiles = (p.R + NT - 1) / NT;
  // XCD-aware order: workgroup b runs on XCD b%8; give every XCD one contiguous band of tiles so rows
  // gathered by neighbouring tiles meet in the same L2.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, wg_per_xcd = gridDim.x >> 3;
  const int64_t tpx = (n_tiles + 7) / 8;

  if constexpr (RES) {
    for (int64_t i = tid; i < S * STAGE_U4; i += NT) lds[i] = p.apack[i];
    __syncthreads();
  }

  // Fast path: a two-deep software pipeline over the tiles of this workgroup.  While tile t is multiplied,
  // the row data of tile t+1 (operand rows, corner positions, CSR bounds) is already in flight, and the
  // ids those loads needed were fetched one tile earlier still.  Arithmetic on the loaded values is
  // deferred to the top of the tile that uses them, so nothing waits on memory inside the MFMA loop.
  // With 4 waves (512 registers each) the operand rows are prefetched a tile ahead as well and the A
  // fragments a chain ahead; with 8 waves (256 registers, two waves per SIMD that cover for each other)
  // only the geometry is, and the operand rows are fetched at the top of their tile, ahead of the SH
  // arithmetic that hides most of their latency.
  constexpr bool XPRE = (NW <= 4);
  struct TileRaw {
    int32_t gid[2][3];
    RowMeta meta[2];
    DirRaw dr[2];
    uint4 xr[XPRE ? 2 : 1][PM_GC][NRaw<XM>::n];
  };
  auto rows_of = [&](int64_t ti_, int fb) {
    const int64_t t_ = (int64_t)xcd * tpx + ti_;
    return min(t_ * NT + wave * 64 + fb * 32 + l32, p.R - 1);   // clamped: loads are unconditional
  };
  auto gload = [&](int64_t rc, const RowMeta& m, int c0, uint4 (&raw)[NRaw<XM>::n]) {
    if constexpr (FM == 2) {
      if (c0 >= p.Cc) {
#pragma unroll
        for (int j = 0; j < NRaw<XM>::n; ++j) raw[j] = make_uint4(0, 0, 0, 0);
        return;
      }
    }
    granule_load<XM, DT>(p.xs, rc, m, c0, raw);
  };
  auto issue_ids = [&](int64_t ti_, TileRaw& t) {
#pragma unroll
    for (int fb = 0; fb < 2; ++fb) {
      const int64_t rc = rows_of(ti_, fb);
      dir_ids<BM>(p.bs, rc, t.gid[fb]);
      load_meta_ids<XM>(p.xs, rc, true, t.meta[fb]);
    }
  };
  auto issue_loads = [&](int64_t ti_, TileRaw& t) {
#pragma unroll
    for (int fb = 0; fb < 2; ++fb) {
      const int64_t rc = rows_of(ti_, fb);
      if constexpr (BM != B_ONE) dir_load<BM>(p.bs, rc, t.gid[fb], t.dr[fb]);
      load_meta_w<XM>(p.xs, true, t.meta[fb]);
      if constexpr (XPRE) {
#pragma unroll
        for (int g = 0; g < PM_GC; ++g) gload(rc, t.meta[fb], (g * 2 + hh) * EPG, t.xr[fb][g]);
      }
    }
  };
  TileRaw cur, nxt;
  if constexpr (FAST) {
    issue_ids(slot, cur);
    issue_loads(slot, cur);
    issue_ids(slot + wg_per_xcd, nxt);
  }

  for (int64_t ti = slot; ti < tpx; ti += wg_per_xcd) {
    const int64_t tile = (int64_t)xcd * tpx + ti;
    const bool tile_ok = tile < n_tiles;
    const int64_t r0 = tile * NT + wave * 64;
    int64_t row[2], rowc[2];
    bool ok[2];
    RowMeta meta[2];
    float B[2][K];
    uint4 X0[2][PM_GC];  // fast path: first chunk of the operand rows
#pragma unroll
    for (int fb = 0; fb < 2; ++fb) {
      row[fb] = r0 + fb * 32 + l32;
      ok[fb] = tile_ok && row[fb] < p.R;
      rowc[fb] = FAST ? min(row[fb], p.R - 1) : row[fb];
    }
    if constexpr (FAST) {
      uint4 xnow[2][PM_GC][NRaw<XM>::n];
      if constexpr (!XPRE) {   // operand rows of this tile: out first, used after the SH arithmetic
#pragma unroll
        for (int fb = 0; fb < 2; ++fb)
#pragma unroll
          for (int g = 0; g < PM_GC; ++g)
            gload(rowc[fb], cur.meta[fb], (g * 2 + hh) * EPG, xnow[fb][g]);
      }
      // arithmetic on this tile's data (loaded during the previous tile)
#pragma unroll
      for (int fb = 0; fb < 2; ++fb) {
        meta[fb] = cur.meta[fb];
        meta_finish<XM>(meta[fb]);
        if constexpr (BM != B_ONE) {
          float x, y, z;
          dir_finish<BM>(cur.dr[fb], x, y, z);
          sh_eval<LT>(x, y, z, p.bs.sh, [&](int k, float v) { B[fb][k] = v; });
        } else {
          B[fb][0] = 1.f;
        }
#pragma unroll
        for (int g = 0; g < PM_GC; ++g) {
          if constexpr (XPRE) X0[fb][g] = granule_finish<XM, DT>(cur.xr[fb][g], meta[fb]);
          else X0[fb][g] = granule_finish<XM, DT>(xnow[fb][g], meta[fb]);
        }
      }
      // next tile: its ids are here, send out everything that depends on them; then the ids after that
      __builtin_amdgcn_sched_barrier(0);
      issue_loads(ti + wg_per_xcd, nxt);
      cur = nxt;
      issue_ids(ti + 2 * wg_per_xcd, nxt);
      __builtin_amdgcn_sched_barrier(0);
    } else {
#pragma unroll
      for (int fb = 0; fb < 2; ++fb) {
        load_meta<XM>(p.xs, rowc[fb], ok[fb], meta[fb]);
        if constexpr (BM != B_ONE) {
          float x = 0.f, y = 0.f, z = 1.f;
          if (ok[fb]) row_direction<BM>(p.bs, rowc[fb], x, y, z);
          sh_eval<LT>(x, y, z, p.bs.sh, [&](int k, float v) { B[fb][k] = v; });
        } else {
          B[fb][0] = 1.f;
        }
      }
    }

    // ---- helpers shared by the two loop orders -----------------------------------------------------
    auto fetch_chunk = [&](int ch, uint4 (&X)[2][PM_GC]) {
#pragma unroll
      for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int g = 0; g < PM_GC; ++g) {
          const int c0 = ((ch * PM_GC + g) * 2 + hh) * EPG;
          if constexpr (FAST) {
            if (ch == 0) X[fb][g] = X0[fb][g];
            else {
              uint4 raw[NRaw<XM>::n];
              gload(rowc[fb], meta[fb], c0, raw);
              X[fb][g] = granule_finish<XM, DT>(raw, meta[fb]);
            }
          } else {
            float v[EPG];
            fetch_vals<XM, EPG>(p.xs, row[fb], ok[fb], meta[fb], c0, v);
            X[fb][g] = pack_granule<DT>(v);
          }
        }
    };
    // one 32-wide block nb of output channels of row block fb
    auto store_block = [&](int nb, int fb, const floatx16& yv) {
      if (!ok[fb]) return;
      if (p.store_fast) {   // Cn % 64 == 0, aligned rows: unguarded 16-byte (fp32) / 8-byte (bf16) pieces
        const int64_t o = row[fb] * (int64_t)p.Cn + nb * 32 + hh * 4;
        if (p.out_bf16) {
          uint16_t* dst = (uint16_t*)p.out + o;
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            uint2 w;
            w.x = pack_bf16x2(yv[q4 * 4], yv[q4 * 4 + 1]);
            w.y = pack_bf16x2(yv[q4 * 4 + 2], yv[q4 * 4 + 3]);
            *(uint2*)(dst + q4 * 8) = w;
          }
        } else {
          float* dst = (float*)p.out + o;
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4)
            *(float4*)(dst + q4 * 8) = make_float4(yv[q4 * 4], yv[q4 * 4 + 1], yv[q4 * 4 + 2], yv[q4 * 4 + 3]);
        }
        return;
      }
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int n0 = nb * 32 + q4 * 8 + hh * 4;
        if (n0 >= p.Cn) continue;
        const float vv[4] = {yv[q4 * 4], yv[q4 * 4 + 1], yv[q4 * 4 + 2], yv[q4 * 4 + 3]};
        const int64_t o = row[fb] * (int64_t)p.Cn + n0;
        if (n0 + 4 <= p.Cn && (p.Cn & 3) == 0) {
          if (p.out_bf16) {
            uint2 w;
            w.x = pack_bf16x2(vv[0], vv[1]); w.y = pack_bf16x2(vv[2], vv[3]);
            *(uint2*)((uint16_t*)p.out + o) = w;
          } else {
            *(float4*)((float*)p.out + o) = make_float4(vv[0], vv[1], vv[2], vv[3]);
          }
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (n0 + i < p.Cn) {
              if (p.out_bf16) ((uint16_t*)p.out)[o + i] = (uint16_t)f32_to_bf16_bits(vv[i]);
              else ((float*)p.out)[o + i] = vv[i];
            }
        }
      }
    };
    // One chain = the 2*GC MFMA groups of one (k, n-block) for both row blocks, software-pipelined with
    // the FMA epilogue of the previous chain: a wave issues in order, so the matrix pipe only stays busy
    // during the SH weighting if every MFMA is followed, in program order, by a few of the pending FMAs
    // (sched_barrier pins that order).
    auto chain = [&](const uint4 (&ac)[PM_GC], const uint4 (&X)[2][PM_GC], bool have_pending, floatx16& y0,
                     floatx16& y1, floatx16& pu0, floatx16& pu1, float pb0, float pb1) {
      floatx16 u0, u1;
#pragma unroll
      for (int i = 0; i < 16; ++i) { u0[i] = 0.f; u1[i] = 0.f; }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < PM_GC; ++g) {
        u0 = mma_group<DT>(ac[g], X[0][g], u0);
        if (have_pending) {
          // four pending FMAs, pinned right here (an empty asm that "modifies" them): without the pin
          // the optimiser gathers all FMAs of a chain at its end and the MFMAs run back to back alone
          float t0 = y0[4 * g] + pb0 * pu0[4 * g], t1 = y0[4 * g + 1] + pb0 * pu0[4 * g + 1];
          float t2 = y0[4 * g + 2] + pb0 * pu0[4 * g + 2], t3 = y0[4 * g + 3] + pb0 * pu0[4 * g + 3];
          asm volatile("" : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3));
          y0[4 * g] = t0; y0[4 * g + 1] = t1; y0[4 * g + 2] = t2; y0[4 * g + 3] = t3;
        }
        __builtin_amdgcn_sched_barrier(0);
        u1 = mma_group<DT>(ac[g], X[1][g], u1);
        if (have_pending) {
          float t0 = y1[4 * g] + pb1 * pu1[4 * g], t1 = y1[4 * g + 1] + pb1 * pu1[4 * g + 1];
          float t2 = y1[4 * g + 2] + pb1 * pu1[4 * g + 2], t3 = y1[4 * g + 3] + pb1 * pu1[4 * g + 3];
          asm volatile("" : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3));
          y1[4 * g] = t0; y1[4 * g + 1] = t1; y1[4 * g + 2] = t2; y1[4 * g + 3] = t3;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      pu0 = u0; pu1 = u1;
    };

    if constexpr (RES && BM == B_ONE) {
      // No basis (K = 1): little matrix work per row, so the kernel lives on its row fetches.  Up to four
      // 32-wide output blocks accumulate at once (loop order  n-block group -> c-chunk -> n-block), every
      // chunk of the operand rows is fetched once per group, and the next chunk's loads are issued before
      // the current chunk is multiplied.
      const int NB = NBG * PM_NBS;
      for (int nb0 = 0; nb0 * 32 < p.Cn; nb0 += 4) {
        floatx16 y[4][2];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int fb = 0; fb < 2; ++fb)
#pragma unroll
            for (int i = 0; i < 16; ++i) y[q][fb][i] = 0.f;
        uint4 X[2][PM_GC];
        fetch_chunk(0, X);
        for (int ch = 0; ch < NCH; ++ch) {
          uint4 Xn[2][PM_GC];
          if (ch + 1 < NCH) fetch_chunk(ch + 1, Xn);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int nb = nb0 + q;
            if (nb < NB && nb * 32 < p.Cn) {
              const uint4* base = lds + ((int64_t)((nb / PM_NBS) * NCH + ch)) * STAGE_U4 + (nb % PM_NBS) * PM_GC * 64 + lane;
#pragma unroll
              for (int g = 0; g < PM_GC; ++g) {
                const uint4 a = base[g * 64];
                y[q][0] = mma_group<DT>(a, X[0][g], y[q][0]);
                y[q][1] = mma_group<DT>(a, X[1][g], y[q][1]);
              }
            }
          }
          if (ch + 1 < NCH) {
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
#pragma unroll
              for (int g = 0; g < PM_GC; ++g) X[fb][g] = Xn[fb][g];
          }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int nb = nb0 + q;
          if (nb < NB && nb * 32 < p.Cn) {
            store_block(nb, 0, y[q][0]);
            store_block(nb, 1, y[q][1]);
          }
        }
      }
    } else if constexpr (RES) {
      // Weights resident in LDS: one 32-wide block of output channels at a time (32 accumulator
      // registers), loop order  n-block -> c-chunk -> k.
      for (int nb = 0; nb < NBG * PM_NBS; ++nb) {
        if (nb * 32 >= p.Cn) break;
        const int nbg = nb / PM_NBS, nbi = nb % PM_NBS;
        floatx16 y0, y1;
#pragma unroll
        for (int i = 0; i < 16; ++i) { y0[i] = 0.f; y1[i] = 0.f; }
        for (int ch = 0; ch < NCH; ++ch) {
          uint4 X[2][PM_GC];
          fetch_chunk(ch, X);
          const uint4* base = lds + ((int64_t)(nbg * NCH + ch) * K) * STAGE_U4 + nbi * PM_GC * 64 + lane;
          if constexpr (BM == B_ONE) {
#pragma unroll
            for (int g = 0; g < PM_GC; ++g) {
              const uint4 a = base[g * 64];
              y0 = mma_group<DT>(a, X[0][g], y0);
              y1 = mma_group<DT>(a, X[1][g], y1);
            }
          } else {
            floatx16 pu0, pu1;
            float pb0 = 0.f, pb1 = 0.f;
            uint4 afr[PM_GC];
            if constexpr (XPRE) {
#pragma unroll
              for (int g = 0; g < PM_GC; ++g) afr[g] = base[g * 64];
            }
#pragma unroll
            for (int k = 0; k < K; ++k) {
              asm volatile("" ::: "memory");  // keep LDS reads of later k from being hoisted up here
              uint4 ac[PM_GC];
              if constexpr (XPRE) {
#pragma unroll
                for (int g = 0; g < PM_GC; ++g) ac[g] = afr[g];
                if (k + 1 < K) {   // fragments of the next chain, read while this one computes
#pragma unroll
                  for (int g = 0; g < PM_GC; ++g) afr[g] = base[(k + 1) * STAGE_U4 + g * 64];
                }
              } else {
#pragma unroll
                for (int g = 0; g < PM_GC; ++g) ac[g] = base[k * STAGE_U4 + g * 64];
              }
              chain(ac, X, k > 0, y0, y1, pu0, pu1, pb0, pb1);
              pb0 = B[0][k]; pb1 = B[1][k];
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {   // drain the pipeline
              y0[i] = fmaf(pb0, pu0[i], y0[i]);
              y1[i] = fmaf(pb1, pu1[i], y1[i]);
            }
            asm volatile("" : "+v"(y0), "+v"(y1));
          }
        }
        store_block(nb, 0, y0);
        store_block(nb, 1, y1);
      }
    } else {
      // Weights streamed through a two-slot LDS ring, one barrier per stage: loop order
      // n-block pair -> c-chunk -> k -> n-block, so that every stage is fetched once per tile.
      // blockIdx.y splits the groups of output blocks (few row tiles, many output channels: more workgroups than
      // tiles, each streaming its share of the weights)
      const int nbg_lo = (int)((int64_t)blockIdx.y * NBG / gridDim.y), nbg_hi = (int)((int64_t)(blockIdx.y + 1) * NBG / gridDim.y);
      const int64_t S_hi = (int64_t)nbg_hi * NCH * K;
      int64_t q = (int64_t)nbg_lo * NCH * K;  // stage sequence number
      __syncthreads();                        // the ring is free (previous tile)
#pragma unroll
      for (int i = 0; i < PER_T; ++i) lds[(q & 1) * STAGE_U4 + i * NT + tid] = p.apack[q * STAGE_U4 + i * NT + tid];
      __syncthreads();
      for (int nbg = nbg_lo; nbg < nbg_hi; ++nbg) {
        floatx16 y[PM_NBS][2];
#pragma unroll
        for (int a = 0; a < PM_NBS; ++a)
#pragma unroll
          for (int fb = 0; fb < 2; ++fb)
#pragma unroll
            for (int i = 0; i < 16; ++i) y[a][fb][i] = 0.f;
        for (int ch = 0; ch < NCH; ++ch) {
          uint4 X[2][PM_GC];
          fetch_chunk(ch, X);
          floatx16 pu0, pu1;
          float pb0 = 0.f, pb1 = 0.f;
#pragma unroll
          for (int k = 0; k < K; ++k, ++q) {
            asm volatile("" ::: "memory");
            const uint4* stage = lds + (q & 1) * STAGE_U4;
            uint4 pre[PER_T];
            if (q + 1 < S_hi) {
#pragma unroll
              for (int i = 0; i < PER_T; ++i) pre[i] = p.apack[(q + 1) * STAGE_U4 + i * NT + tid];
            }
#pragma unroll
            for (int nbi = 0; nbi < PM_NBS; ++nbi) {
              uint4 ac[PM_GC];
#pragma unroll
              for (int g = 0; g < PM_GC; ++g) ac[g] = stage[(nbi * PM_GC + g) * 64 + lane];
              if constexpr (BM == B_ONE) {
#pragma unroll
                for (int g = 0; g < PM_GC; ++g) {
                  y[nbi][0] = mma_group<DT>(ac[g], X[0][g], y[nbi][0]);
                  y[nbi][1] = mma_group<DT>(ac[g], X[1][g], y[nbi][1]);
                }
              } else {
                constexpr int LASTB = PM_NBS - 1;
                const int pn = (nbi == 0) ? LASTB : nbi - 1;
                chain(ac, X, (k > 0 || nbi > 0), y[pn][0], y[pn][1], pu0, pu1, pb0, pb1);
                pb0 = B[0][k]; pb1 = B[1][k];
              }
            }
            if (q + 1 < S_hi) {
#pragma unroll
              for (int i = 0; i < PER_T; ++i) lds[((q + 1) & 1) * STAGE_U4 + i * NT + tid] = pre[i];
            }
            __syncthreads();
          }
          if constexpr (BM != B_ONE) {  // drain the pipeline
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              y[PM_NBS - 1][0][i] = fmaf(pb0, pu0[i], y[PM_NBS - 1][0][i]);
              y[PM_NBS - 1][1][i] = fmaf(pb1, pu1[i], y[PM_NBS - 1][1][i]);
            }
            asm volatile("" : "+v"(y[PM_NBS - 1][0]), "+v"(y[PM_NBS - 1][1]));
          }
        }
#pragma unroll
        for (int nbi = 0; nbi < PM_NBS; ++nbi) {
          store_block(nbg * PM_NBS + nbi, 0, y[nbi][0]);
          store_block(nbg * PM_NBS + nbi, 1, y[nbi][1]);
        }
      }
    }
  }
}

template <int DT, int BM, int XM, int LT, int NW, bool RES, int FM>
static pm_status launch_conv_fast(const ConvP& p, int64_t S, hipStream_t st) {
  auto kern = k_conv_rows<DT, BM, XM, LT, NW, RES, FM>;
  size_t lds = RES ? (size_t)S * PM_STAGE_BYTES : 2 * (size_t)PM_STAGE_BYTES;
  PM_TRY(pm_set_dyn_lds((const void*)kern, lds));
  const int NT = NW * 64;
  int64_t n_tiles = (p.R + NT - 1) / NT;
  int64_t grid = n_tiles < 256 ? (n_tiles + 7) / 8 * 8 : 256;
  // streamed weights on a mesh with fewer row tiles than compute units: split the output-block groups over
  // workgroups as well (each streams its share of the weights; the rows are fetched once per share)
  int split = 1;
  if (!RES) {
    while (split * 2 <= p.NBG && grid * split * 2 <= 256) split *= 2;
    if (split > p.NBG) split = p.NBG;
  }
  { ProfScope ps__(st, "k_conv_rows");
    hipLaunchKernelGGL(kern, dim3((unsigned)grid, (unsigned)split), dim3(NT), lds, st, p); }
  PM_CHECK_LAUNCH("k_conv_rows");
  return PM_OK;
}

// The branch-free fetch needs: storage dtype == MFMA dtype, 16-byte aligned rows, whole chunks of channels.
template <int DT, int BM, int XM, int LT, int NW, bool RES>
static pm_status launch_conv_res(const ConvP& p, int64_t S, hipStream_t st) {
  const int esz = (DT == 1) ? 2 : 4;
  const int chunk = PM_GC * ((DT == 1) ? 16 : 8);
  const int pair = chunk / PM_GC;   // channels of one granule pair (the two half-waves): 16 bf16, 8 fp32
  const bool fast = (p.xs.is_bf16 == (DT == 1)) && pm_aligned16(p.xs.p) && ((p.xs.C * esz) % 16 == 0);
  if (fast && p.Cc % chunk == 0) return launch_conv_fast<DT, BM, XM, LT, NW, RES, 1>(p, S, st);
  // a partly filled last chunk (32 channels of bf16, say): whole granule pairs inside the operand row
  if (fast && p.Cc % pair == 0 && (XM == X_DIRECT || XM == X_GATHER_SUM || XM == X_GATHER1))
    return launch_conv_fast<DT, BM, XM, LT, NW, RES, 2>(p, S, st);
  return launch_conv_fast<DT, BM, XM, LT, NW, RES, 0>(p, S, st);
}

template <int DT, int BM, int XM, int LT, int NW>
static pm_status launch_conv_inst(const ConvP& p, int64_t S, hipStream_t st) {
  if (p.resident) return launch_conv_res<DT, BM, XM, LT, NW, true>(p, S, st);
  return launch_conv_res<DT, BM, XM, LT, NW, false>(p, S, st);
}

template <int DT, int BM, int XM>
static pm_status launch_conv_L(const ConvP& p, int L, int64_t S, hipStream_t st) {
  if constexpr (BM == B_ONE) {
    return launch_conv_inst<DT, BM, XM, 0, 4>(p, S, st);
  } else {
    switch (L) {
      case 0: return launch_conv_inst<DT, BM, XM, 0, 4>(p, S, st);
      case 1: return launch_conv_inst<DT, BM, XM, 1, 4>(p, S, st);
      case 2: return launch_conv_inst<DT, BM, XM, 2, 4>(p, S, st);
      // two waves per SIMD when the row loader is light enough to fit 256 registers
      case 3: return launch_conv_inst<DT, BM, XM, 3, (XM == X_GATHER_SUM || XM == X_GATHER1) ? 4 : 8>(p, S, st);
      case 4: return launch_conv_inst<DT, BM, XM, 4, 4>(p, S, st);
      case 5: return launch_conv_inst<DT, BM, XM, 5, 4>(p, S, st);
      default: return pm_fail(PM_ERR_UNSUPPORTED, "SH degree %d", L);
    }
  }
}


// One instance file defines one of these (both residency variants, all degrees).
#define PM_CONV_INSTANCE(DT, BM, XM)                                                                   \
  pm_status pm_conv_dispatch_##DT##_##BM##_##XM(const ConvP& p, int L, int64_t S, hipStream_t st) {    \
    return launch_conv_L<DT, BM, XM>(p, L, S, st);                                                     \
  }
#define PM_CONV_DECLARE(DT, BM, XM) \
  pm_status pm_conv_dispatch_##DT##_##BM##_##XM(const ConvP& p, int L, int64_t S, hipStream_t st);
