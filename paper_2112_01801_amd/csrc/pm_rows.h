// Row loaders shared by the row-wise MFMA kernels: how one operand row (a facet, a texture point) gets
// its channels, its basis vector and its gather metadata.
#pragma once
#include "pm_host.h"

// elements [c0, c0+N) of row `row` of a [*, C] matrix (bf16 or fp32 storage) as floats; zero beyond C
template <int N>
__device__ __forceinline__ void load_vals(const void* __restrict__ base, int is_bf16, int64_t row, int C, int c0,
                                          float (&v)[N]) {
  const int64_t off = row * (int64_t)C + c0;
  if (c0 + N <= C) {
    if (is_bf16) {
      const uint16_t* p = (const uint16_t*)base + off;
      if ((((uintptr_t)p) & (2 * N - 1)) == 0) {
        if constexpr (N == 8) {
          uint4 u = *(const uint4*)p;
          v[0] = bf16lo_to_f32(u.x); v[1] = bf16hi_to_f32(u.x);
          v[2] = bf16lo_to_f32(u.y); v[3] = bf16hi_to_f32(u.y);
          v[4] = bf16lo_to_f32(u.z); v[5] = bf16hi_to_f32(u.z);
          v[6] = bf16lo_to_f32(u.w); v[7] = bf16hi_to_f32(u.w);
        } else {
          uint2 u = *(const uint2*)p;
          v[0] = bf16lo_to_f32(u.x); v[1] = bf16hi_to_f32(u.x);
          v[2] = bf16lo_to_f32(u.y); v[3] = bf16hi_to_f32(u.y);
        }
      } else {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = bf16_to_f32(p[i]);
      }
    } else {
      const float* p = (const float*)base + off;
      if ((((uintptr_t)p) & 15) == 0) {
#pragma unroll
        for (int q = 0; q < N / 4; ++q) {
          float4 f = ((const float4*)p)[q];
          v[4 * q] = f.x; v[4 * q + 1] = f.y; v[4 * q + 2] = f.z; v[4 * q + 3] = f.w;
        }
      } else {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = p[i];
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      float x = 0.f;
      if (c0 + i < C) x = is_bf16 ? bf16_to_f32(((const uint16_t*)base)[off + i]) : ((const float*)base)[off + i];
      v[i] = x;
    }
  }
}

// Gather metadata of one row, loaded once per tile.
struct RowMeta {
  int32_t id[3];  // X_GATHER_SUM / X_GATHER_CAT: corner vertex ids;  X_GATHER1: id[0] = owner
  float w[3];     // X_GATHER_SUM: 1/deg(v_j);  X_GATHER1: w[0] = 1/segment length
  int32_t lo[3], hi[3];  // raw CSR bounds the weights come from (set by load_meta_w, used by meta_finish)
};

// Two phases, so that a software pipeline can issue them in different iterations: the ids (one load,
// no dependency) and the weights (loads that depend on the ids).
template <int XM>
__device__ __forceinline__ void load_meta_ids(const RowSrc& s, int64_t r, bool valid, RowMeta& m) {
  m.id[0] = m.id[1] = m.id[2] = 0;
  m.w[0] = m.w[1] = m.w[2] = 0.f;
  if (!valid) return;
  if constexpr (XM == X_GATHER_SUM || XM == X_GATHER_CAT) {
#pragma unroll
    for (int j = 0; j < 3; ++j) m.id[j] = s.facet[3 * r + j];
  } else if constexpr (XM == X_GATHER1) {
    m.id[0] = s.owner[r];
  }
}

// loads only (no arithmetic on the loaded values, so nothing forces an early wait)
template <int XM>
__device__ __forceinline__ void load_meta_w(const RowSrc& s, bool valid, RowMeta& m) {
#pragma unroll
  for (int j = 0; j < 3; ++j) { m.lo[j] = 0; m.hi[j] = 1; }
  if (!valid) return;
  if constexpr (XM == X_GATHER_SUM) {
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      m.lo[j] = s.row_ptr[m.id[j]];
      m.hi[j] = s.row_ptr[m.id[j] + 1];
    }
  } else if constexpr (XM == X_GATHER1) {
    m.lo[0] = s.seg_off[m.id[0]];
    m.hi[0] = s.seg_off[m.id[0] + 1];
  }
}

// weights from the CSR bounds: 1/deg(v_j) (>= 1: the vertex is referenced by this very facet), 1/R_f
template <int XM>
__device__ __forceinline__ void meta_finish(RowMeta& m) {
  if constexpr (XM == X_GATHER_SUM) {
#pragma unroll
    for (int j = 0; j < 3; ++j) m.w[j] = 1.0f / (float)(m.hi[j] - m.lo[j]);
  } else if constexpr (XM == X_GATHER1) {
    m.w[0] = 1.0f / (float)(m.hi[0] - m.lo[0]);
  }
}

template <int XM>
__device__ __forceinline__ void load_meta(const RowSrc& s, int64_t r, bool valid, RowMeta& m) {
  load_meta_ids<XM>(s, r, valid, m);
  load_meta_w<XM>(s, valid, m);
  meta_finish<XM>(m);
}

// N consecutive channels [c0, c0+N) of the (virtual) operand row r, as floats.
//   X_DIRECT:      src[r][c]
//   X_GATHER_SUM:  sum_j src[v_j(r)][c] / deg(v_j(r))            (transposed facet->vertex mean)
//   X_GATHER_CAT:  concatenation over the three corners, channel c = j*C + cc -> src[v_j(r)][cc]
//   X_GATHER1:     src[owner(r)][c] / segment length             (transposed segment mean)
template <int XM, int N>
__device__ __forceinline__ void fetch_vals(const RowSrc& s, int64_t r, bool valid, const RowMeta& m, int c0,
                                           float (&v)[N]) {
  if (!valid) {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = 0.f;
    return;
  }
  if constexpr (XM == X_DIRECT) {
    load_vals<N>(s.p, s.is_bf16, r, s.C, c0, v);
  } else if constexpr (XM == X_GATHER_SUM) {
    float t[N];
    load_vals<N>(s.p, s.is_bf16, m.id[0], s.C, c0, t);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = t[i] * m.w[0];
    load_vals<N>(s.p, s.is_bf16, m.id[1], s.C, c0, t);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = fmaf(t[i], m.w[1], v[i]);   // explicit: every copy of this code rounds alike
    load_vals<N>(s.p, s.is_bf16, m.id[2], s.C, c0, t);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = fmaf(t[i], m.w[2], v[i]);
  } else if constexpr (XM == X_GATHER_CAT) {
    const int C = s.C;
    int j = c0 / C, cc = c0 - j * C;
    if (j < 3 && cc + N <= C) {
      int32_t id = (j == 0) ? m.id[0] : (j == 1 ? m.id[1] : m.id[2]);
      load_vals<N>(s.p, s.is_bf16, id, C, cc, v);
    } else {
#pragma unroll
      for (int i = 0; i < N; ++i) {
        int c = c0 + i;
        int jj = c / C, ci = c - jj * C;
        float x = 0.f;
        if (jj < 3) {
          int32_t id = (jj == 0) ? m.id[0] : (jj == 1 ? m.id[1] : m.id[2]);
          int64_t o = (int64_t)id * C + ci;
          x = s.is_bf16 ? bf16_to_f32(((const uint16_t*)s.p)[o]) : ((const float*)s.p)[o];
        }
        v[i] = x;
      }
    }
  } else {  // X_GATHER1
    load_vals<N>(s.p, s.is_bf16, m.id[0], s.C, c0, v);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] *= m.w[0];
  }
}

// Unit direction whose SH basis weights row r: the facet normal (Eq. 5) or a given direction (Eq. 7's
// barycentric point projected radially onto the sphere).
template <int BM>
__device__ __forceinline__ void row_direction(const BasisSrc& b, int64_t r, float& x, float& y, float& z) {
  if constexpr (BM == B_NORMAL) {
    facet_normal(b.vert, b.facet[3 * r], b.facet[3 * r + 1], b.facet[3 * r + 2], x, y, z);
  } else {
    x = b.dirs[3 * r]; y = b.dirs[3 * r + 1]; z = b.dirs[3 * r + 2];
    normalize_dir(x, y, z);
  }
}

// ---- the same, split into pipeline phases for the branch-free fast path ----------------------------
// phase 0: ids (no dependency)   phase 1: loads that need the ids   phase 2: arithmetic
struct DirRaw {
  float v[9];  // B_NORMAL: the three corner positions; B_DIRS: v[0..2] = the direction
};

template <int BM>
__device__ __forceinline__ void dir_ids(const BasisSrc& b, int64_t rowc, int32_t (&gid)[3]) {
  gid[0] = gid[1] = gid[2] = 0;
  if constexpr (BM == B_NORMAL) {
#pragma unroll
    for (int j = 0; j < 3; ++j) gid[j] = b.facet[3 * rowc + j];
  }
}

template <int BM>
__device__ __forceinline__ void dir_load(const BasisSrc& b, int64_t rowc, const int32_t (&gid)[3], DirRaw& d) {
  if constexpr (BM == B_NORMAL) {
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const float* q = b.vert + 3 * (int64_t)gid[j];
      d.v[3 * j] = q[0]; d.v[3 * j + 1] = q[1]; d.v[3 * j + 2] = q[2];
    }
  } else if constexpr (BM == B_DIRS) {
    d.v[0] = b.dirs[3 * rowc]; d.v[1] = b.dirs[3 * rowc + 1]; d.v[2] = b.dirs[3 * rowc + 2];
  }
}

// unit direction: facet normal by the right-hand rule ((0,0,1) when degenerate), or the normalised direction
template <int BM>
__device__ __forceinline__ void dir_finish(const DirRaw& d, float& x, float& y, float& z) {
  if constexpr (BM == B_NORMAL) {
    const float ux = d.v[3] - d.v[0], uy = d.v[4] - d.v[1], uz = d.v[5] - d.v[2];
    const float wx = d.v[6] - d.v[0], wy = d.v[7] - d.v[1], wz = d.v[8] - d.v[2];
    float cx, cy, cz;
    cross_fixed(ux, uy, uz, wx, wy, wz, cx, cy, cz);
    const float l2 = norm2_fixed(cx, cy, cz);
    const bool deg = l2 < 1e-30f;
    const float r = 1.0f / sqrtf(deg ? 1.0f : l2);
    x = deg ? 0.f : cx * r;
    y = deg ? 0.f : cy * r;
    z = deg ? 1.f : cz * r;
  } else {
    x = d.v[0]; y = d.v[1]; z = d.v[2];
    normalize_dir(x, y, z);
  }
}
