// Gradient with respect to the dense filter coefficients:
//     dWp[k][c][n] = sum_r B_r[k] * X_r[c] * Y_r[n]
// (F2V: r = facet, X = h_f, Y = dy_f gathered from the vertex gradients; V2F: k = corner, X = h of that
// corner's vertex, Y = dg_f; F2F: r = texture point, X = h_p, Y = dg of the owning facet / R_f.)
//
// This is a GEMM whose contraction runs over rows r.  Row tiles of 64 are staged in LDS TRANSPOSED
// (channel-major, rows contiguous) so that an MFMA operand fragment -- 8 consecutive rows of one
// channel -- is a single 16-byte LDS read.  The basis weighting multiplies the Y fragment in fp32
// before it is packed (the one place where a per-row product has to be formed explicitly).
//
// A workgroup (8 waves) owns a 64x64 (c,n) slab for up to 16 values of k: each wave accumulates two k's
// (8 accumulator blocks of 32x32); when there are fewer than 8 k-pairs the spare waves split the rows
// of every tile instead.  Each workgroup covers a fixed contiguous range of rows and writes its partial
// sums to its own slice of a workspace; a second kernel adds the slices in a fixed order, so the result
// is bitwise reproducible and uses no floating-point atomics.
#include "pm_wgrad.h"

// Eight consecutive channels of one source row as they sit in memory (no arithmetic yet, so that the
// loads can stay in flight while the previous tile is being multiplied).
struct Raw8 {
  uint4 a, b;   // bf16 source: a holds the 8 values; fp32 source (or the slow path): a, b hold 8 floats
  int f32;
};

__device__ __forceinline__ Raw8 raw_load8(const void* __restrict__ base, int is_bf16, int64_t row, int C, int c0,
                                          bool valid) {
  Raw8 r;
  r.a = make_uint4(0, 0, 0, 0);
  r.b = make_uint4(0, 0, 0, 0);
  r.f32 = !is_bf16;
  if (!valid) return r;
  const int64_t off = row * (int64_t)C + c0;
  if (c0 + 8 <= C) {
    if (is_bf16) {
      const uint16_t* p = (const uint16_t*)base + off;
      if ((((uintptr_t)p) & 15) == 0) {
        r.a = *(const uint4*)p;
        return r;
      }
    } else {
      const float* p = (const float*)base + off;
      if ((((uintptr_t)p) & 15) == 0) {
        r.a = ((const uint4*)p)[0];
        r.b = ((const uint4*)p)[1];
        return r;
      }
    }
  }
  float v[8];
  load_vals<8>(base, is_bf16, row, C, c0, v);   // guarded element path
  r.a = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
  r.b = make_uint4(__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7]));
  r.f32 = 1;
  return r;
}

// Fast path (host-checked): source dtype == DT, 16-byte aligned rows, octet inside the row.  No branches,
// so the loads of a whole tile can be in flight together.
template <int DT>
__device__ __forceinline__ Raw8 raw_load8_fast(const void* __restrict__ base, int64_t row, int C, int c0) {
  Raw8 r;
  const int64_t off = row * (int64_t)C + c0;
  if constexpr (DT == 1) {
    r.a = *(const uint4*)((const uint16_t*)base + off);
    r.b = make_uint4(0, 0, 0, 0);
    r.f32 = 0;
  } else {
    const uint4* p = (const uint4*)((const float*)base + off);
    r.a = p[0];
    r.b = p[1];
    r.f32 = 1;
  }
  return r;
}

__device__ __forceinline__ void raw_to_f32(const Raw8& r, float (&v)[8]) {
  if (r.f32) {
    v[0] = __uint_as_float(r.a.x); v[1] = __uint_as_float(r.a.y); v[2] = __uint_as_float(r.a.z); v[3] = __uint_as_float(r.a.w);
    v[4] = __uint_as_float(r.b.x); v[5] = __uint_as_float(r.b.y); v[6] = __uint_as_float(r.b.z); v[7] = __uint_as_float(r.b.w);
  } else {
    v[0] = bf16lo_to_f32(r.a.x); v[1] = bf16hi_to_f32(r.a.x); v[2] = bf16lo_to_f32(r.a.y); v[3] = bf16hi_to_f32(r.a.y);
    v[4] = bf16lo_to_f32(r.a.z); v[5] = bf16hi_to_f32(r.a.z); v[6] = bf16lo_to_f32(r.a.w); v[7] = bf16hi_to_f32(r.a.w);
  }
}

// number of source rows a mode reads per operand row
template <int M> struct NSrc { static constexpr int n = (M == X_GATHER_SUM || M == X_GATHER_CAT) ? 3 : 1; };

template <int M, int DT, bool FAST>
__device__ __forceinline__ void raw_fetch(const RowSrc& s, int64_t r, bool ok, const RowMeta& m, int c0,
                                          Raw8 (&raw)[NSrc<M>::n]) {
  if constexpr (FAST) {
    if constexpr (M == X_DIRECT) {
      raw[0] = raw_load8_fast<DT>(s.p, r, s.C, c0);
    } else if constexpr (M == X_GATHER1) {
      raw[0] = raw_load8_fast<DT>(s.p, m.id[0], s.C, c0);
    } else {
#pragma unroll
      for (int j = 0; j < 3; ++j) raw[j] = raw_load8_fast<DT>(s.p, m.id[j], s.C, c0);
    }
    return;
  }
  if constexpr (M == X_DIRECT) {
    raw[0] = raw_load8(s.p, s.is_bf16, r, s.C, c0, ok);
  } else if constexpr (M == X_GATHER1) {
    raw[0] = raw_load8(s.p, s.is_bf16, m.id[0], s.C, c0, ok);
  } else {
#pragma unroll
    for (int j = 0; j < 3; ++j) raw[j] = raw_load8(s.p, s.is_bf16, m.id[j], s.C, c0, ok);
  }
}

// the operand values of Eq. 5's / Eq. 7's transposed sums from the raw rows
template <int M>
__device__ __forceinline__ void raw_combine(const Raw8 (&raw)[NSrc<M>::n], const RowMeta& m, float (&v)[8]) {
  raw_to_f32(raw[0], v);
  if constexpr (M == X_GATHER1) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= m.w[0];
  } else if constexpr (M == X_GATHER_SUM) {
    float t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= m.w[0];
    raw_to_f32(raw[1], t);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = fmaf(t[i], m.w[1], v[i]);
    raw_to_f32(raw[2], t);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = fmaf(t[i], m.w[2], v[i]);
  }
}

template <int DT, int BM, int XM, int YM, bool FAST>
__global__ void __launch_bounds__(512) k_wgrad(WgradP p) {
  extern __shared__ uint4 lds_raw[];
  constexpr int NSUBX = (XM == X_GATHER_CAT) ? 3 : 1;        // one X tile per corner
  constexpr int XPB = (DT == 1) ? XP_BF16 * 2 : XP_F32 * 4;  // bytes per channel row of XT
  constexpr int XT_BYTES = NSUBX * 64 * XPB;
  constexpr int YT_BYTES = 64 * XP_F32 * 4;
  constexpr int BS_BYTES = WG_KG * XP_F32 * 4;
  constexpr int BUF_BYTES = XT_BYTES + YT_BYTES + BS_BYTES;
  char* lds = (char*)lds_raw;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int slab = blockIdx.y;
  const int kg = slab % p.KGn, cbp = (slab / p.KGn) % p.CBP, nbp = slab / (p.KGn * p.CBP);
  const int kbase = kg * WG_KG;
  const int kcount = min(WG_KG, p.K - kbase);
  const int kp = wave % p.NKPW, rs = wave / p.NKPW;
  const bool active = (rs < p.RS) && (2 * kp < kcount);
  const bool kv[2] = {active, active && (2 * kp + 1 < kcount)};
  const int cbase = cbp * 64, nbase = nbp * 64;

  floatx16 acc[2][2][2];  // [kk][cb][nb]
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][b][c][i] = 0.f;

  const int64_t rbeg = (int64_t)blockIdx.x * p.rows_per_part;
  const int64_t rend = min(p.R, rbeg + p.rows_per_part);

  // Staging role: wave w moves channel octet w (8 channels of X and of Y) of all 64 rows of a tile,
  // lane = row.  The transposed LDS writes of a wave are then 64 consecutive elements of one channel
  // row: conflict-free.  Waves 0..3 also move 4 basis values per row.
  struct Pref {
    Raw8 x[NSUBX][(XM == X_GATHER_CAT) ? 1 : NSrc<XM>::n];
    Raw8 y[NSrc<YM>::n];
    float4 bv;
  };
  struct Ids {
    RowMeta mx, my;
    bool ok;
  };
  // On the fast path rows past the end are clamped to the last row (so every load is unconditional and
  // in bounds) and zeroed when they are written to LDS.
  auto row_of = [&](int64_t t0) { return FAST ? min(t0 + lane, rend - 1) : t0 + lane; };
  auto load_ids = [&](int64_t t0, Ids& d) {
    const int64_t r = row_of(t0);
    d.ok = t0 + lane < rend;
    const bool go = FAST ? true : d.ok;
    load_meta_ids<XM>(p.xs, r, go, d.mx);
    load_meta_ids<YM>(p.ys, r, go, d.my);
  };
  auto load_w = [&](Ids& d) {   // loads that depend on the ids: issued one pipeline step after them
    const bool go = FAST ? true : d.ok;
    load_meta_w<XM>(p.xs, go, d.mx);
    load_meta_w<YM>(p.ys, go, d.my);
  };
  auto load_data = [&](int64_t t0, const Ids& d, Pref& f) {
    const int64_t r = row_of(t0);
    if constexpr (XM == X_GATHER_CAT) {
#pragma unroll
      for (int sub = 0; sub < 3; ++sub) {
        if constexpr (FAST) f.x[sub][0] = raw_load8_fast<DT>(p.xs.p, d.mx.id[sub], p.xs.C, cbase + wave * 8);
        else f.x[sub][0] = raw_load8(p.xs.p, p.xs.is_bf16, d.mx.id[sub], p.xs.C, cbase + wave * 8, d.ok);
      }
    } else {
      raw_fetch<XM, DT, FAST>(p.xs, r, d.ok, d.mx, cbase + wave * 8, f.x[0]);
    }
    raw_fetch<YM, DT, FAST>(p.ys, r, d.ok, d.my, nbase + wave * 8, f.y);
    f.bv = make_float4(0.f, 0.f, 0.f, 0.f);
    if constexpr (BM != B_ONE) {
      if constexpr (FAST) {
        // host guarantees K % 4 == 0: one aligned 16-byte load, unconditional (waves without a k range
        // read a clamped address and drop the value when the tile is written to LDS)
        const int k0 = min(kbase + (wave & 3) * 4, p.K - 4);
        f.bv = *(const float4*)(p.bs.bvals + r * (int64_t)p.K + k0);
      } else if (wave < WG_KG / 4 && d.ok) {
        const int k0 = kbase + wave * 4;
        const float* src = p.bs.bvals + r * (int64_t)p.K + k0;
        if (k0 + 4 <= p.K && (((uintptr_t)src) & 15) == 0) {
          f.bv = *(const float4*)src;
        } else {
          if (k0 + 0 < p.K) f.bv.x = src[0];
          if (k0 + 1 < p.K) f.bv.y = src[1];
          if (k0 + 2 < p.K) f.bv.z = src[2];
          if (k0 + 3 < p.K) f.bv.w = src[3];
        }
      }
    }
  };
  auto store_lds = [&](int buf, Ids& d, const Pref& f) {
    meta_finish<XM>(d.mx);
    meta_finish<YM>(d.my);
    char* XT = lds + buf * BUF_BYTES;
    float* YT = (float*)(XT + XT_BYTES);
    float* Bs = YT + 64 * XP_F32;
#pragma unroll
    for (int sub = 0; sub < NSUBX; ++sub) {
      float v[8];
      if constexpr (XM == X_GATHER_CAT) raw_to_f32(f.x[sub][0], v);
      else raw_combine<XM>(f.x[0], d.mx, v);
      if constexpr (FAST) {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = d.ok ? v[i] : 0.f;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        char* dst = XT + (sub * 64 + wave * 8 + i) * XPB;
        if constexpr (DT == 1) ((uint16_t*)dst)[lane] = (uint16_t)f32_to_bf16_bits(v[i]);
        else ((float*)dst)[lane] = v[i];
      }
    }
    {
      float v[8];
      raw_combine<YM>(f.y, d.my, v);
      if constexpr (FAST) {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = d.ok ? v[i] : 0.f;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) YT[(wave * 8 + i) * XP_F32 + lane] = v[i];
    }
    if constexpr (BM != B_ONE) {
      if (wave < WG_KG / 4) {
        float4 bv = f.bv;
        if constexpr (FAST) {
          if (!d.ok || kbase + wave * 4 >= p.K) bv = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        Bs[(wave * 4 + 0) * XP_F32 + lane] = bv.x;
        Bs[(wave * 4 + 1) * XP_F32 + lane] = bv.y;
        Bs[(wave * 4 + 2) * XP_F32 + lane] = bv.z;
        Bs[(wave * 4 + 3) * XP_F32 + lane] = bv.w;
      }
    }
  };

  Ids ids_cur, ids_nxt;
  Pref pref;
  if (rbeg < rend) {
    load_ids(rbeg, ids_cur);
    load_w(ids_cur);
    load_data(rbeg, ids_cur, pref);
    load_ids(rbeg + WG_RT, ids_nxt);
    store_lds(0, ids_cur, pref);
  }
  __syncthreads();

  int buf = 0;
  for (int64_t t0 = rbeg; t0 < rend; t0 += WG_RT, buf ^= 1) {
    const bool have_next = t0 + WG_RT < rend;
    // global loads of the next tile go out now and land while this tile is multiplied;
    // the gather ids of the tile after that are fetched one step earlier still
    if (have_next) {
      load_w(ids_nxt);
      load_data(t0 + WG_RT, ids_nxt, pref);
    }
    Ids ids_nn;
    load_ids(t0 + 2 * WG_RT, ids_nn);
    __builtin_amdgcn_sched_barrier(0);  // everything above is loads only: nothing may wait on them yet

    const char* XT = lds + buf * BUF_BYTES;
    const float* YT = (const float*)(XT + XT_BYTES);
    const float* Bs = YT + 64 * XP_F32;
    if (active) {
      if constexpr (DT == 1) {
        for (int ss = rs; ss < WG_RT / 16; ss += p.RS) {
          const int roff = ss * 16 + hh * 8;
          float yv[2][8];
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) {
            const float4* s = (const float4*)(YT + (nb * 32 + l32) * XP_F32 + roff);
            float4 a = s[0], b = s[1];
            yv[nb][0] = a.x; yv[nb][1] = a.y; yv[nb][2] = a.z; yv[nb][3] = a.w;
            yv[nb][4] = b.x; yv[nb][5] = b.y; yv[nb][6] = b.z; yv[nb][7] = b.w;
          }
          uint4 xf[2][2];  // [kk or 0][cb]
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) {
            const int sub = (XM == X_GATHER_CAT) ? min(kbase + 2 * kp + kk, 2) : 0;
            if (kk == 0 || XM == X_GATHER_CAT) {
#pragma unroll
              for (int cb = 0; cb < 2; ++cb)
                xf[kk][cb] = *(const uint4*)(XT + (sub * 64 + cb * 32 + l32) * XPB + roff * 2);
            } else {
              xf[kk][0] = xf[0][0]; xf[kk][1] = xf[0][1];
            }
          }
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) {
            if (!kv[kk]) continue;
            float bv[8];
            if constexpr (BM == B_ONE) {
#pragma unroll
              for (int i = 0; i < 8; ++i) bv[i] = 1.f;
            } else {
              const float4* s = (const float4*)(Bs + (2 * kp + kk) * XP_F32 + roff);
              float4 a = s[0], b = s[1];
              bv[0] = a.x; bv[1] = a.y; bv[2] = a.z; bv[3] = a.w;
              bv[4] = b.x; bv[5] = b.y; bv[6] = b.z; bv[7] = b.w;
            }
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
              uint4 yf;
              yf.x = pack_bf16x2(bv[0] * yv[nb][0], bv[1] * yv[nb][1]);
              yf.y = pack_bf16x2(bv[2] * yv[nb][2], bv[3] * yv[nb][3]);
              yf.z = pack_bf16x2(bv[4] * yv[nb][4], bv[5] * yv[nb][5]);
              yf.w = pack_bf16x2(bv[6] * yv[nb][6], bv[7] * yv[nb][7]);
#pragma unroll
              for (int cb = 0; cb < 2; ++cb)
                acc[kk][cb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, xf[kk][cb]), __builtin_bit_cast(bf16x8, yf), acc[kk][cb][nb], 0, 0, 0);
            }
          }
        }
      } else {
        for (int ss = rs; ss < WG_RT / 8; ss += p.RS) {
          const int roff = ss * 8 + hh * 4;
          float4 yv[2];
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) yv[nb] = *(const float4*)(YT + (nb * 32 + l32) * XP_F32 + roff);
          float4 xf[2][2];
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) {
            const int sub = (XM == X_GATHER_CAT) ? min(kbase + 2 * kp + kk, 2) : 0;
            if (kk == 0 || XM == X_GATHER_CAT) {
#pragma unroll
              for (int cb = 0; cb < 2; ++cb)
                xf[kk][cb] = *(const float4*)(XT + (sub * 64 + cb * 32 + l32) * XPB + roff * 4);
            } else {
              xf[kk][0] = xf[0][0]; xf[kk][1] = xf[0][1];
            }
          }
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) {
            if (!kv[kk]) continue;
            float4 bv = make_float4(1.f, 1.f, 1.f, 1.f);
            if constexpr (BM != B_ONE) bv = *(const float4*)(Bs + (2 * kp + kk) * XP_F32 + roff);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
              const float y0 = bv.x * yv[nb].x, y1 = bv.y * yv[nb].y, y2 = bv.z * yv[nb].z, y3 = bv.w * yv[nb].w;
#pragma unroll
              for (int cb = 0; cb < 2; ++cb) {
                floatx16 a = acc[kk][cb][nb];
                a = __builtin_amdgcn_mfma_f32_32x32x2f32(xf[kk][cb].x, y0, a, 0, 0, 0);
                a = __builtin_amdgcn_mfma_f32_32x32x2f32(xf[kk][cb].y, y1, a, 0, 0, 0);
                a = __builtin_amdgcn_mfma_f32_32x32x2f32(xf[kk][cb].z, y2, a, 0, 0, 0);
                a = __builtin_amdgcn_mfma_f32_32x32x2f32(xf[kk][cb].w, y3, a, 0, 0, 0);
                acc[kk][cb][nb] = a;
              }
            }
          }
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    // the other buffer was last read one iteration ago (a barrier has passed since): refill it
    if (have_next) store_lds(buf ^ 1, ids_nxt, pref);
    __syncthreads();
    ids_nxt = ids_nn;
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
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          const int n = nbase + nb * 32 + l32;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int c = cbase + cb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
            if (c < p.Cc && n < p.Cn) dst[(int64_t)c * p.Cn + n] = acc[kk][cb][nb][i];
          }
        }
    }
  }
}

// out[i] = sum over the slices in a fixed order (bitwise reproducible): the slices are cut into eight
// consecutive groups, each group is added sequentially by one thread (eight loads in flight), and the
// eight group sums are then added in group order.
__global__ void __launch_bounds__(256) k_sum_partials(const float* __restrict__ partial, int64_t n, int64_t stride,
                                                      int n_slice, float* __restrict__ out) {
  __shared__ float part[8][32];
  const int il = threadIdx.x & 31, g = threadIdx.x >> 5;
  const int64_t i = (int64_t)blockIdx.x * 32 + il;
  const int per = (n_slice + 7) / 8;
  const int q0 = g * per, q1 = min(n_slice, q0 + per);
  float s = 0.f;
  if (i < n) {
    int q = q0;
    for (; q + 8 <= q1; q += 8) {
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = partial[(int64_t)(q + j) * stride + i];
#pragma unroll
      for (int j = 0; j < 8; ++j) s += v[j];
    }
    for (; q < q1; ++q) s += partial[(int64_t)q * stride + i];
  }
  part[g][il] = s;
  __syncthreads();
  if (g == 0 && i < n) {
    float t = part[0][il];
#pragma unroll
    for (int j = 1; j < 8; ++j) t += part[j][il];
    out[i] = t;
  }
}

pm_status pm_launch_sum_slices(const float* partial, int64_t n, int n_slice, float* out, hipStream_t st) {
  return pm_launch_sum_slices_strided(partial, n, n, n_slice, out, st);
}

// the slices start `stride` floats apart (stride >= n): sums a window of n floats of every slice
pm_status pm_launch_sum_slices_strided(const float* partial, int64_t n, int64_t stride, int n_slice, float* out,
                                       hipStream_t st) {
  if (n <= 0) return PM_OK;
  { ProfScope ps__(st, "k_sum_partials");
    hipLaunchKernelGGL(k_sum_partials, dim3((unsigned)((n + 31) / 32)), dim3(256), 0, st, partial, n, stride, n_slice, out); }
  PM_CHECK_LAUNCH("k_sum_partials");
  return PM_OK;
}

struct WgradGeom {
  int KGn, CBP, NBP, slabs, NKPW, RS, n_part;
  int64_t rows_per_part;
};

static WgradGeom wgrad_geom(int64_t R, int K, int Cc, int Cn) {
  WgradGeom g;
  g.KGn = (K + WG_KG - 1) / WG_KG;
  g.CBP = (Cc + 63) / 64;
  g.NBP = (Cn + 63) / 64;
  g.slabs = g.KGn * g.CBP * g.NBP;
  int kmax = K < WG_KG ? K : WG_KG;
  g.NKPW = (kmax + 1) / 2;
  g.RS = 8 / g.NKPW;
  if (g.RS > 4) g.RS = 4;  // a 64-row tile has 4 bf16 sub-steps (8 for fp32); 4 serves both
  int64_t tiles = (R + WG_RT - 1) / WG_RT;
  int want = 256 / g.slabs;
  if (want < 16) want = 16;
  int64_t np = tiles < want ? tiles : want;
  if (np < 1) np = 1;
  int64_t tpp = (tiles + np - 1) / np;
  if (tpp < 1) tpp = 1;
  g.rows_per_part = tpp * WG_RT;
  g.n_part = (int)((tiles + tpp - 1) / tpp);
  if (g.n_part < 1) g.n_part = 1;
  return g;
}

size_t pm_wgrad_ws_bytes(int64_t R, int K, int Cc, int Cn) {
  WgradGeom g = wgrad_geom(R, K, Cc, Cn);
  return pm_round_up((size_t)g.n_part * g.RS * K * Cc * Cn * sizeof(float), 256);
}

template <int DT, int BM, int XM, int YM, bool FAST>
static pm_status launch_wgrad_fast(const WgradP& p, const WgradGeom& g, hipStream_t st) {
  auto kern = k_wgrad<DT, BM, XM, YM, FAST>;
  const int nsub = (XM == X_GATHER_CAT) ? 3 : 1;
  const int xpb = (DT == 1) ? XP_BF16 * 2 : XP_F32 * 4;
  size_t lds = 2 * ((size_t)nsub * 64 * xpb + (size_t)64 * XP_F32 * 4 + (size_t)WG_KG * XP_F32 * 4);
  PM_TRY(pm_set_dyn_lds((const void*)kern, lds));
  { ProfScope ps__(st, "k_wgrad");
    hipLaunchKernelGGL(kern, dim3((unsigned)g.n_part, (unsigned)g.slabs), dim3(512), lds, st, p); }
  PM_CHECK_LAUNCH("k_wgrad");
  return PM_OK;
}

// The branch-free loaders need: storage dtype == MFMA dtype, 16-byte aligned rows, every 64-channel slab
// inside the row, and (with a basis) K a multiple of 4.
template <int DT, int BM, int XM, int YM>
static pm_status launch_wgrad_inst(const WgradP& p, const WgradGeom& g, hipStream_t st) {
  const int esz = (DT == 1) ? 2 : 4;
  bool fast = (p.xs.is_bf16 == (DT == 1)) && (p.ys.is_bf16 == (DT == 1));
  fast = fast && (p.Cc % 64 == 0) && (p.Cn % 64 == 0) && (p.xs.C % 8 == 0) && (p.ys.C % 8 == 0);
  fast = fast && ((p.xs.C * esz) % 16 == 0) && ((p.ys.C * esz) % 16 == 0);
  fast = fast && pm_aligned16(p.xs.p) && pm_aligned16(p.ys.p);
  if (BM != B_ONE) fast = fast && (p.K % 4 == 0) && pm_aligned16(p.bs.bvals);
  if (fast) return launch_wgrad_fast<DT, BM, XM, YM, true>(p, g, st);
  return launch_wgrad_fast<DT, BM, XM, YM, false>(p, g, st);
}

template <int DT>
static pm_status launch_wgrad_mode(BMode bm, XMode xm, XMode ym, const WgradP& p, const WgradGeom& g, hipStream_t st) {
  if (bm == B_NORMAL && xm == X_DIRECT && ym == X_GATHER_SUM)
    return launch_wgrad_inst<DT, B_NORMAL, X_DIRECT, X_GATHER_SUM>(p, g, st);
  if (bm == B_ONE && xm == X_GATHER_CAT && ym == X_DIRECT)
    return launch_wgrad_inst<DT, B_ONE, X_GATHER_CAT, X_DIRECT>(p, g, st);
  if (bm == B_DIRS && xm == X_DIRECT && ym == X_GATHER1)
    return launch_wgrad_inst<DT, B_DIRS, X_DIRECT, X_GATHER1>(p, g, st);
  if (bm == B_ONE && xm == X_DIRECT && ym == X_DIRECT)
    return launch_wgrad_inst<DT, B_ONE, X_DIRECT, X_DIRECT>(p, g, st);
  return pm_fail(PM_ERR_UNSUPPORTED, "wgrad mode (%d,%d,%d)", (int)bm, (int)xm, (int)ym);
}

pm_status pm_launch_wgrad(pm_dtype mt, BMode bm, XMode xm, XMode ym, int64_t R, int K, int Cc, int Cn,
                          const BasisSrc& bs, const RowSrc& xs, const RowSrc& ys, float* dWp, void* ws, size_t ws_bytes,
                          void* y_out, hipStream_t st) {
  WgradGeom g = wgrad_geom(R, K, Cc, Cn);
  if (ws_bytes < pm_wgrad_ws_bytes(R, K, Cc, Cn)) return pm_fail(PM_ERR_WORKSPACE, "wgrad workspace too small");
  if (!y_out && pm_wgrad_stage_applies(mt, bm, xm, ym, K, Cc, Cn, xs, ys))
    return pm_launch_wgrad_stage(xm, R, K, Cc, Cn, xs, ys, dWp, ws, ws_bytes, st);
  WgradP p;
  p.R = R; p.rows_per_part = g.rows_per_part;
  p.K = K; p.Cc = Cc; p.Cn = Cn;
  p.KGn = g.KGn; p.CBP = g.CBP; p.NBP = g.NBP; p.NKPW = g.NKPW; p.RS = g.RS;
  p.bs = bs; p.xs = xs; p.ys = ys; p.partial = (float*)ws;
  p.y_out = y_out;
  pm_status s;
  if (pm_wgrad_fuses_basis(mt, bm, xm, ym, K, Cc, Cn, xs, ys))
    s = pm_launch_wgrad_pc(bm, ym, p, g.n_part, g.slabs, st);
  else if (y_out)
    return pm_fail(PM_ERR_UNSUPPORTED, "the general weight-gradient kernel does not write the Y rows");
  else
    s = (mt == PM_BF16) ? launch_wgrad_mode<1>(bm, xm, ym, p, g, st) : launch_wgrad_mode<0>(bm, xm, ym, p, g, st);
  if (s != PM_OK) return s;
  return pm_launch_sum_slices((const float*)ws, (int64_t)K * Cc * Cn, g.n_part * g.RS, dWp, st);
}

// dW[k][ci][co] = sum_j fc[j][k] * M[j][ci][co]   (vertex2facet: the three corner directions are constants)
__global__ void __launch_bounds__(256) k_unfold(int K, int64_t cc, const float* __restrict__ M, FoldCoef fc,
                                                float* __restrict__ dW) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)K * cc) return;
  int k = (int)(i / cc);
  int64_t e = i - (int64_t)k * cc;
  dW[i] = fc.c[0][k] * M[e] + fc.c[1][k] * M[cc + e] + fc.c[2][k] * M[2 * cc + e];
}

pm_status pm_launch_unfold(int K, int cin, int cout, const float* M, const FoldCoef* fc, float* dW, hipStream_t st) {
  int64_t cc = (int64_t)cin * cout;
  { ProfScope ps__(st, "k_unfold");
    hipLaunchKernelGGL(k_unfold, dim3((unsigned)((K * cc + 255) / 256)), dim3(256), 0, st, K, cc, M, *fc, dW); }
  PM_CHECK_LAUNCH("k_unfold");
  return PM_OK;
}
