// Gradient with respect to the dense filter coefficients, producer/consumer form:
//     dWp[k][c][n] = sum_r B_r[k] * X_r[c] * Y_r[n]
// for bf16 rows X read directly and Y gathered (transposed sums of Eq. 5 and Eq. 7), with the basis B
// evaluated inside the kernel from the row's direction (Eq. 3-4).
//
// A workgroup has 12 waves.  Waves 8..11 are producers: lane = row of a 64-row block; they fetch the
// row's channels, its gathered gradient rows and its corner positions a tile ahead, combine them
// and write the block TRANSPOSED into LDS (channel-major, so an MFMA operand fragment -- 8 consecutive
// rows of one channel -- is one 16-byte read).  Waves 0..7 are consumers: each owns two k's of a
// 64x64 (c,n) slab (8 accumulator blocks of 32x32); per 16 rows it scales the Y fragment by the basis
// values (kept compactly, two registers per k, and broadcast inside lane quads by the multiply's own
// lane-select modifier) and issues the matrix instructions.  A tile is two 64-row blocks; one barrier
// per tile separates the two LDS buffers; producers and consumers work on different tiles at the same
// time, so global-memory latency, the gather arithmetic and the matrix pipe overlap across the waves
// of a SIMD (the longer the stretch between barriers, the better the waves of a SIMD fall into
// alternating LDS-read and matrix phases).
//
// Each workgroup covers a fixed contiguous range of rows and writes its partial sums to its own
// slice; the slices are added in a fixed order afterwards (bitwise reproducible, no float atomics).
// On request the producers also write the gathered Y rows (bf16) to global memory, so that the
// backward-data pass of the same call can read them as plain rows instead of gathering them again.
#include "pm_wgrad.h"

#define PC_CONS 8
#define PC_PROD 4
#define PC_THREADS ((PC_CONS + PC_PROD) * 64)
#define PC_XPB (XP_BF16 * 2)                          /* bytes per channel row of the X tile */
#define PC_XT_BYTES (64 * PC_XPB)
#define PC_YT_BYTES (64 * XP_F32 * 4)
#define PC_BS_BYTES (WG_KG * 64 * 4)
#define PC_HALF_BYTES (PC_XT_BYTES + PC_YT_BYTES + PC_BS_BYTES)   /* one staged block of 64 rows */
#define PC_HPT 2                                                    /* 64-row blocks per tile (per barrier) */
#define PC_BUF_BYTES (PC_HPT * PC_HALF_BYTES)

// value of lane (4*(lane/4) + J) of the same quad
template <int J>
__device__ __forceinline__ float quad_bcast(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), J * 0x55, 0xf, 0xf, true));
}

// position of a tile row inside its group of 8 in the basis tile: (r0,r4,r1,r5,r2,r6,r3,r7), so that
// quad lane q reads (B[q], B[4+q]) of a group with one 8-byte access
__device__ __forceinline__ int basis_pos(int row) { return (row & ~7) + 2 * (row & 3) + ((row >> 2) & 1); }

struct PcIds {
  int32_t y[3];  // gather ids of the Y rows
  int32_t g[3];  // corner ids for the facet normal
};

template <int NYS, int NY, int NX>
struct PcSet {
  uint4 x[NX > 0 ? NX : 1];
  uint4 y[NY > 0 ? NY : 1][NYS];
  int32_t lo[3], hi[3];
  DirRaw d;
};

// One producer wave.  It moves NX channel octets of X starting at octet X0, NY octets of Y starting at
// Y0 and (HASB) the basis values of each 64-row block.  Block b of the workgroup's row range lives in
// register set b&1 and in LDS buffer (b/2)&1, slot b&1; its loads are issued one tile before it is
// written to LDS, its ids one tile before that.
template <int BM, int YM, int LT, int CBN, int NBN, bool HASB, int NY, int Y0, int NX, int X0>
__device__ __forceinline__ void pc_producer(const WgradP& p, char* lds, const int lane, const int64_t rbeg,
                                            const int64_t rend, const int n_tiles, const int cbase, const int nbase,
                                            const int kbase) {
  const bool emit_y = p.y_out != nullptr && cbase == 0 && kbase == 0;   // one slab per n-range writes the rows
  constexpr int NYS = (YM == X_GATHER_SUM) ? 3 : 1;
  using Set = PcSet<NYS, NY, NX>;
  // rows past the end are clamped to the last row (every load unconditional and in bounds); their basis
  // values are written as zero, which removes them from every sum
  auto rowc = [&](int b) { return min(rbeg + (int64_t)b * WG_RT + lane, rend - 1); };

  auto load_ids = [&](int b, PcIds& d) {
    const int64_t r = rowc(b);
    d.y[0] = d.y[1] = d.y[2] = 0;
    if constexpr (NY > 0) {
      if constexpr (YM == X_GATHER_SUM) {
#pragma unroll
        for (int j = 0; j < 3; ++j) d.y[j] = p.ys.facet[3 * r + j];
      } else if constexpr (YM == X_GATHER1) {
        d.y[0] = p.ys.owner[r];
      }
    }
    if constexpr (HASB) dir_ids<BM>(p.bs, r, d.g);
  };

  // a slab narrower than 64 channels (Cc or Cn = 32, CBN or NBN = 1): the octets beyond it are neither loaded nor
  // written back; their LDS rows are zero
  auto x_in = [&](int i) { return (X0 + i) * 8 < 32 * CBN; };     // compile-time after unrolling
  auto y_in = [&](int i) { return (Y0 + i) * 8 < 32 * NBN; };
  auto issue = [&](int b, const PcIds& d, Set& s) {
    const int64_t r = rowc(b);
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      s.x[i] = make_uint4(0, 0, 0, 0);
      if (x_in(i)) s.x[i] = *(const uint4*)((const uint16_t*)p.xs.p + r * (int64_t)p.xs.C + cbase + (X0 + i) * 8);
    }
    if constexpr (NY > 0) {
#pragma unroll
      for (int j = 0; j < NYS; ++j) {
        const int64_t src = (YM == X_DIRECT) ? r : (int64_t)d.y[j];
#pragma unroll
        for (int i = 0; i < NY; ++i) {
          s.y[i][j] = make_uint4(0, 0, 0, 0);
          if (y_in(i)) s.y[i][j] = *(const uint4*)((const uint16_t*)p.ys.p + src * (int64_t)p.ys.C + nbase + (Y0 + i) * 8);
        }
      }
      if constexpr (YM == X_GATHER_SUM) {
#pragma unroll
        for (int j = 0; j < 3; ++j) {
          s.lo[j] = p.ys.row_ptr[d.y[j]];
          s.hi[j] = p.ys.row_ptr[d.y[j] + 1];
        }
      } else if constexpr (YM == X_GATHER1) {
        s.lo[0] = p.ys.seg_off[d.y[0]];
        s.hi[0] = p.ys.seg_off[d.y[0] + 1];
      }
    }
    if constexpr (HASB) dir_load<BM>(p.bs, r, d.g, s.d);
  };

  auto store = [&](int b, Set& s) {
    const bool ok = rbeg + (int64_t)b * WG_RT + lane < rend;
    char* XT = lds + ((b >> 1) & 1) * PC_BUF_BYTES + (b & 1) * PC_HALF_BYTES;
    float* YT = (float*)(XT + PC_XT_BYTES);
    float* Bs = YT + 64 * XP_F32;
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const uint32_t w[4] = {s.x[i].x, s.x[i].y, s.x[i].z, s.x[i].w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        uint16_t* dst = (uint16_t*)(XT + ((X0 + i) * 8 + e) * PC_XPB);
        dst[lane] = (uint16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu));
      }
    }
    if constexpr (NY > 0) {
      float wt[3] = {1.f, 1.f, 1.f};
      if constexpr (YM == X_GATHER_SUM) {
#pragma unroll
        for (int j = 0; j < 3; ++j) wt[j] = __builtin_amdgcn_rcpf((float)(s.hi[j] - s.lo[j]));   // 1 ulp
      } else if constexpr (YM == X_GATHER1) {
        wt[0] = __builtin_amdgcn_rcpf((float)(s.hi[0] - s.lo[0]));
      }
#pragma unroll
      for (int i = 0; i < NY; ++i) {
        float v[8];
#pragma unroll
        for (int j = 0; j < NYS; ++j) {
          const uint32_t w[4] = {s.y[i][j].x, s.y[i][j].y, s.y[i][j].z, s.y[i][j].w};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float f = (e & 1) ? bf16hi_to_f32(w[e >> 1]) : bf16lo_to_f32(w[e >> 1]);
            // explicit fused multiply-adds: left to the compiler's contraction, the copies of this code before and inside
            // the tile loop rounded differently (a row's dy then depended on where a workgroup's range starts)
            if (j == 0) v[e] = (YM == X_DIRECT) ? f : f * wt[0];
            else v[e] = fmaf(f, wt[j], v[e]);
          }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) YT[((Y0 + i) * 8 + e) * XP_F32 + lane] = v[e];
        if (emit_y && ok && y_in(i)) {
          uint4 w;
          w.x = pack_bf16x2(v[0], v[1]); w.y = pack_bf16x2(v[2], v[3]);
          w.z = pack_bf16x2(v[4], v[5]); w.w = pack_bf16x2(v[6], v[7]);
          const int64_t r = rbeg + (int64_t)b * WG_RT + lane;
          *(uint4*)((uint16_t*)p.y_out + r * (int64_t)p.Cn + nbase + (Y0 + i) * 8) = w;
        }
      }
    }
    if constexpr (HASB) {
      float x, y, z;
      dir_finish<BM>(s.d, x, y, z);
      const int pos = basis_pos(lane);
      sh_eval<LT>(x, y, z, p.bs.sh, [&](int k, float v) {
        if constexpr (LT >= 0 && (LT + 1) * (LT + 1) <= WG_KG) {   // one k group: kbase is 0
          Bs[k * 64 + pos] = ok ? v : 0.f;
        } else {
          const int kl = k - kbase;
          if (kl >= 0 && kl < WG_KG) Bs[kl * 64 + pos] = ok ? v : 0.f;
        }
      });
    }
  };

  if (n_tiles <= 0) return;
  PcIds i0, i1;
  Set s0, s1;
  load_ids(0, i0);
  load_ids(1, i1);
  issue(0, i0, s0);
  issue(1, i1, s1);
  load_ids(2, i0);
  load_ids(3, i1);
  store(0, s0);
  issue(2, i0, s0);
  load_ids(4, i0);
  store(1, s1);
  issue(3, i1, s1);
  load_ids(5, i1);
  // barrier t: tile t (blocks 2t, 2t+1) is complete in buffer t&1 and the consumers are done with the other
  // buffer, which now receives tile t+1; the loads of tile t+2 go out as soon as their registers are free
  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();
    store(2 * t + 2, s0);
    issue(2 * t + 4, i0, s0);
    load_ids(2 * t + 6, i0);
    store(2 * t + 3, s1);
    issue(2 * t + 5, i1, s1);
    load_ids(2 * t + 7, i1);
  }
}

// CBN, NBN: 32-wide blocks of X and of Y channels in a slab (2 = the full 64, 1 = a 32-channel operand)
template <int BM, int YM, int LT, int CBN, int NBN>
__global__ void __launch_bounds__(PC_THREADS) k_wgrad_pc(WgradP p) {
  extern __shared__ uint4 lds_raw[];
  char* lds = (char*)lds_raw;

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps the role and k tests scalar
  const int slab = blockIdx.y;
  const int kg = slab % p.KGn, cbp = (slab / p.KGn) % p.CBP, nbp = slab / (p.KGn * p.CBP);
  const int kbase = kg * WG_KG;
  const int kcount = min(WG_KG, p.K - kbase);
  const int cbase = cbp * 64, nbase = nbp * 64;
  const int64_t rbeg = (int64_t)blockIdx.x * p.rows_per_part;
  const int64_t rend = min(p.R, rbeg + p.rows_per_part);
  const int n_tiles = rbeg < rend ? (int)((rend - rbeg + PC_HPT * WG_RT - 1) / (PC_HPT * WG_RT)) : 0;

  if (wave >= PC_CONS) {
    // octets of Y cost ~50 vector instructions per row, the basis ~100, octets of X almost nothing
    switch (wave - PC_CONS) {
      case 0: pc_producer<BM, YM, LT, CBN, NBN, true, 1, 0, 4, 0>(p, lds, lane, rbeg, rend, n_tiles, cbase, nbase, kbase); break;
      case 1: pc_producer<BM, YM, LT, CBN, NBN, false, 3, 1, 0, 0>(p, lds, lane, rbeg, rend, n_tiles, cbase, nbase, kbase); break;
      case 2: pc_producer<BM, YM, LT, CBN, NBN, false, 2, 4, 2, 4>(p, lds, lane, rbeg, rend, n_tiles, cbase, nbase, kbase); break;
      default: pc_producer<BM, YM, LT, CBN, NBN, false, 2, 6, 2, 6>(p, lds, lane, rbeg, rend, n_tiles, cbase, nbase, kbase); break;
    }
    return;
  }

  const int kp = wave % p.NKPW, rs = wave / p.NKPW;
  const bool active = (rs < p.RS) && (2 * kp < kcount);
  const bool kv[2] = {active, active && (2 * kp + 1 < kcount)};

  floatx16 acc[2][CBN][NBN];  // [kk][cb][nb]
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < CBN; ++b)
#pragma unroll
      for (int c = 0; c < NBN; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][b][c][i] = 0.f;

  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();
    if (!active) continue;
    for (int ss = rs; ss < PC_HPT * WG_RT / 16; ss += p.RS) {
      const char* XT = lds + (t & 1) * PC_BUF_BYTES + (ss >> 2) * PC_HALF_BYTES;
      const float* YT = (const float*)(XT + PC_XT_BYTES);
      const float* Bs = YT + 64 * XP_F32;
      const int roff = (ss & 3) * 16 + hh * 8;
      uint4 xf[CBN];
#pragma unroll
      for (int cb = 0; cb < CBN; ++cb) xf[cb] = *(const uint4*)(XT + (cb * 32 + l32) * PC_XPB + roff * 2);
      float2 bq[2];
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) bq[kk] = *(const float2*)(Bs + (2 * kp + kk) * 64 + roff + 2 * (lane & 3));
#pragma unroll
      for (int nb = 0; nb < NBN; ++nb) {
        const float4* s = (const float4*)(YT + (nb * 32 + l32) * XP_F32 + roff);
        const float4 ya = s[0], yb = s[1];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          if (!kv[kk]) continue;
          uint4 yf;
          yf.x = pack_bf16x2(quad_bcast<0>(bq[kk].x) * ya.x, quad_bcast<1>(bq[kk].x) * ya.y);
          yf.y = pack_bf16x2(quad_bcast<2>(bq[kk].x) * ya.z, quad_bcast<3>(bq[kk].x) * ya.w);
          yf.z = pack_bf16x2(quad_bcast<0>(bq[kk].y) * yb.x, quad_bcast<1>(bq[kk].y) * yb.y);
          yf.w = pack_bf16x2(quad_bcast<2>(bq[kk].y) * yb.z, quad_bcast<3>(bq[kk].y) * yb.w);
#pragma unroll
          for (int cb = 0; cb < CBN; ++cb)
            acc[kk][cb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, xf[cb]), __builtin_bit_cast(bf16x8, yf), acc[kk][cb][nb], 0, 0, 0);
        }
      }
    }
  }

  // ---- write this wave's partial sums ----
  if (rs < p.RS) {
    const int64_t slice = (int64_t)blockIdx.x * p.RS + rs;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      if (!kv[kk]) continue;
      const int k = kbase + 2 * kp + kk;
      float* dst = p.partial + (slice * p.K + k) * (int64_t)p.Cc * p.Cn;
#pragma unroll
      for (int cb = 0; cb < CBN; ++cb)
#pragma unroll
        for (int nb = 0; nb < NBN; ++nb) {
          const int n = nbase + nb * 32 + l32;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int c = cbase + cb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
            dst[(int64_t)c * p.Cn + n] = acc[kk][cb][nb][i];
          }
        }
    }
  }
}

bool pm_wgrad_fuses_basis(pm_dtype mt, BMode bm, XMode xm, XMode ym, int K, int Cc, int Cn, const RowSrc& xs,
                          const RowSrc& ys) {
  if (mt != PM_BF16 || xm != X_DIRECT || K < 1) return false;
  if (!((bm == B_NORMAL && ym == X_GATHER_SUM) || (bm == B_DIRS && ym == X_GATHER1))) return false;
  if (!xs.is_bf16 || !ys.is_bf16) return false;
  if ((Cc % 64 != 0 && Cc != 32) || (Cn % 64 != 0 && Cn != 32) || Cc > xs.C || Cn > ys.C) return false;
  if (xs.C % 8 != 0 || ys.C % 8 != 0) return false;  // every row starts on a 16-byte boundary
  return pm_aligned16(xs.p) && pm_aligned16(ys.p);
}

template <int BM, int YM, int LT, int CBN, int NBN>
static pm_status launch_pc_blocks(const WgradP& p, int n_part, int slabs, hipStream_t st) {
  auto kern = k_wgrad_pc<BM, YM, LT, CBN, NBN>;
  const size_t lds = 2 * (size_t)PC_BUF_BYTES;
  PM_TRY(pm_set_dyn_lds((const void*)kern, lds));
  { ProfScope ps__(st, "k_wgrad");
    hipLaunchKernelGGL(kern, dim3((unsigned)n_part, (unsigned)slabs), dim3(PC_THREADS), lds, st, p); }
  PM_CHECK_LAUNCH("k_wgrad_pc");
  return PM_OK;
}

template <int BM, int YM, int LT>
static pm_status launch_pc(const WgradP& p, int n_part, int slabs, hipStream_t st) {
  const bool c32 = p.Cc == 32, n32 = p.Cn == 32;
  if (c32 && n32) return launch_pc_blocks<BM, YM, LT, 1, 1>(p, n_part, slabs, st);
  if (c32) return launch_pc_blocks<BM, YM, LT, 1, 2>(p, n_part, slabs, st);
  if (n32) return launch_pc_blocks<BM, YM, LT, 2, 1>(p, n_part, slabs, st);
  return launch_pc_blocks<BM, YM, LT, 2, 2>(p, n_part, slabs, st);
}

pm_status pm_launch_wgrad_pc(BMode bm, XMode ym, const WgradP& p, int n_part, int slabs, hipStream_t st) {
  const bool l3 = p.bs.sh.L == 3;
  if (bm == B_NORMAL && ym == X_GATHER_SUM)
    return l3 ? launch_pc<B_NORMAL, X_GATHER_SUM, 3>(p, n_part, slabs, st)
              : launch_pc<B_NORMAL, X_GATHER_SUM, -1>(p, n_part, slabs, st);
  if (bm == B_DIRS && ym == X_GATHER1)
    return l3 ? launch_pc<B_DIRS, X_GATHER1, 3>(p, n_part, slabs, st)
              : launch_pc<B_DIRS, X_GATHER1, -1>(p, n_part, slabs, st);
  return pm_fail(PM_ERR_UNSUPPORTED, "wgrad producer/consumer mode (%d,%d)", (int)bm, (int)ym);
}
