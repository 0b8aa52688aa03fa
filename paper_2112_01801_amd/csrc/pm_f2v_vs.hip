// facet2vertex forward (Eq. 5) in the vertex-side order:
//     g_v = sum_k W_k^T S_v[k],     S_v[k][ci] = 1/|N(v)| sum_{f in N(v)} B_k(n_f) h_f[ci]
// The sums of Eq. 5 commute, so the mean over the adjacent facets can be taken before the contraction: the
// matrix work runs over V rows (half as many as facets), and the per-facet summands never reach memory (no
// intermediate, no separate vertex mean).  The price is the outer products B (x) h per adjacency entry on the
// vector ALU; they are taken two entries at a time with the packed bf16 dot product (one instruction gives
// S += B_e1 h_e1 + B_e2 h_e2 in fp32), which needs the basis values in bf16.
//
// bf16 features and weights, Cin = 64, Cout in {64, 128}, K <= 16.  A workgroup of 8 waves owns 256 vertices, a
// wave 32 of them in the lane layout of the 32x32x16 MFMA operand: lane (r = lane % 32, hh = lane / 32) owns
// vertex r and the channels 16 g + 8 hh .. + 7 of the four c-groups g.  It keeps the rows of up to six adjacent
// facets in registers (96 dwords, entries interleaved in pairs), builds S_v[k] for one k at a time and feeds it
// to the matrix core against W_k, which the workgroup streams through a double-buffered 8 KB LDS stage (the
// packed operand image of the facet-side kernel).  Vertices with more than six facets take further passes over
// k that accumulate into the same matrix-core tiles (the contraction is linear in S).  Entries are taken in
// ascending order; nothing is atomic.
#include "pm_rows.h"

#define VS_E 6         /* adjacency entries per pass */
#define VS_STAGE_U4 (PM_STAGE_BYTES / 16)

struct VsP {
  int64_t V;
  int K, NBG;               // SH functions; groups of 64 output channels
  ShTable sh;
  const float* vert;
  const int32_t* facet;
  const int32_t* row_ptr;
  const int32_t* col;       // entries 3 f + j, ascending
  const uint16_t* h;        // [F][64] bf16
  const uint4* apack;       // packed image, stage (nbg * K + k)
  uint16_t* out;            // [V][64 NBG] bf16
};

typedef __bf16 vs_bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float vs_dot2(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(vs_bf16x2, a), __builtin_bit_cast(vs_bf16x2, b), c, false);
}

template <int NB>    // 32-wide output blocks: 2 NBG
__global__ void __launch_bounds__(512) k_f2v_vs(VsP p) {
  extern __shared__ uint4 vs_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, hh = lane >> 5;
  const int K = p.K;
  constexpr int NBG = NB / 2;
  uint4* Wbuf = vs_lds;                                             // [2][NBG][VS_STAGE_U4]
  uint32_t* Bp = (uint32_t*)(vs_lds + 2 * NBG * VS_STAGE_U4) + wave * (32 * 3 * 16);   // this wave's [32][3][16] bf16 pairs
  __shared__ int32_t wmax[8];
  const int64_t n_tiles = (p.V + 255) >> 8;

  for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int64_t v0 = tile * 256 + wave * 32;
    const int64_t v = v0 + r;
    const bool vok = v < p.V;
    int32_t b = 0, e = 0;
    if (vok) { b = p.row_ptr[v]; e = p.row_ptr[v + 1]; }
    int m = e - b;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = max(m, __shfl_xor(m, o, 64));
    __syncthreads();                          // the previous tile's readers of wmax and Wbuf are done
    if (lane == 0) wmax[wave] = m;
    __syncthreads();
    int maxdeg = 0;
#pragma unroll
    for (int w = 0; w < 8; ++w) maxdeg = max(maxdeg, wmax[w]);
    const int passes = max(1, (maxdeg + VS_E - 1) / VS_E);

    floatx16 y[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) y[nb][i] = 0.f;

    for (int pass = 0; pass < passes; ++pass) {
      const int32_t e0 = b + VS_E * pass;
      // ---- rows of this pass's entries: issued first, in flight while the basis is evaluated
      uint4 xr[3][PM_GC], zr[3][PM_GC];
#pragma unroll
      for (int pr = 0; pr < 3; ++pr) {
        const int32_t i1 = e0 + 2 * pr, i2 = i1 + 1;
        const bool l1 = i1 < e, l2 = i2 < e;
        const int32_t c1 = p.col[l1 ? i1 : 0], c2 = p.col[l2 ? i2 : 0];     // col[0] exists whenever a tile has entries
        const int64_t f1 = (int64_t)(((uint64_t)(uint32_t)c1 * 0xAAAAAAABull) >> 33);
        const int64_t f2 = (int64_t)(((uint64_t)(uint32_t)c2 * 0xAAAAAAABull) >> 33);
#pragma unroll
        for (int g = 0; g < PM_GC; ++g) {
          xr[pr][g] = *(const uint4*)(p.h + f1 * 64 + 16 * g + 8 * hh);
          zr[pr][g] = *(const uint4*)(p.h + f2 * 64 + 16 * g + 8 * hh);
          if (!l1) xr[pr][g] = make_uint4(0, 0, 0, 0);
          if (!l2) zr[pr][g] = make_uint4(0, 0, 0, 0);
        }
      }
      // ---- basis of this pass's entries: 32 vertices x 6 entries, one lane each (three rounds with their loads
      //      batched), scaled by 1/|N(v)|, stored as bf16 halves of the pair dwords
      __builtin_amdgcn_wave_barrier();
      {
        int32_t bb[3], ee[3], fid[3];
        bool lv[3];
        float px[3][9];
#pragma unroll
        for (int rd = 0; rd < 3; ++rd) {
          const int it = lane + 64 * rd;
          const int64_t vv = v0 + (it & 31);
          const int64_t vc = min(vv, p.V - 1);
          bb[rd] = p.row_ptr[vc]; ee[rd] = p.row_ptr[vc + 1];
          if (vv >= p.V) ee[rd] = bb[rd];
        }
#pragma unroll
        for (int rd = 0; rd < 3; ++rd) {
          const int en = (lane + 64 * rd) >> 5;
          const int32_t idx = bb[rd] + VS_E * pass + en;
          lv[rd] = idx < ee[rd];
          const int32_t c = p.col[lv[rd] ? idx : 0];
          fid[rd] = (int32_t)(((uint64_t)(uint32_t)c * 0xAAAAAAABull) >> 33);
        }
        int32_t vid[3][3];
#pragma unroll
        for (int rd = 0; rd < 3; ++rd)
#pragma unroll
          for (int j = 0; j < 3; ++j) vid[rd][j] = p.facet[3 * (int64_t)fid[rd] + j];
#pragma unroll
        for (int rd = 0; rd < 3; ++rd)
#pragma unroll
          for (int j = 0; j < 3; ++j) {
            const float* q = p.vert + 3 * (int64_t)vid[rd][j];
            px[rd][3 * j] = q[0]; px[rd][3 * j + 1] = q[1]; px[rd][3 * j + 2] = q[2];
          }
#pragma unroll
        for (int rd = 0; rd < 3; ++rd) {
          const int it = lane + 64 * rd;
          const int rv = it & 31, en = it >> 5;
          uint16_t* dst = (uint16_t*)(Bp + (rv * 3 + (en >> 1)) * 16) + (en & 1);
          const float ux = px[rd][3] - px[rd][0], uy = px[rd][4] - px[rd][1], uz = px[rd][5] - px[rd][2];
          const float wx = px[rd][6] - px[rd][0], wy = px[rd][7] - px[rd][1], wz = px[rd][8] - px[rd][2];
          const float cx = uy * wz - uz * wy, cy = uz * wx - ux * wz, cz = ux * wy - uy * wx;
          const float l2 = cx * cx + cy * cy + cz * cz;
          float nx = 0.f, ny = 0.f, nz = 1.f;
          if (l2 >= 1e-30f) { const float ir = 1.0f / sqrtf(l2); nx = cx * ir; ny = cy * ir; nz = cz * ir; }
          const float w = lv[rd] ? 1.0f / (float)(ee[rd] - bb[rd]) : 0.f;     // an absent entry gets zeros
          sh_eval<-1>(nx, ny, nz, p.sh, [&](int k, float val) { dst[2 * k] = (uint16_t)f32_to_bf16_bits(val * w); });
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();

      // ---- interleave the rows in pairs: H[pr][g][c] = (h_e1[ch], h_e2[ch]), ch = 16 g + 8 hh + c
      uint32_t H[3][PM_GC][8];
#pragma unroll
      for (int pr = 0; pr < 3; ++pr)
#pragma unroll
        for (int g = 0; g < PM_GC; ++g) {
          const uint32_t xs[4] = {xr[pr][g].x, xr[pr][g].y, xr[pr][g].z, xr[pr][g].w};
          const uint32_t zs[4] = {zr[pr][g].x, zr[pr][g].y, zr[pr][g].z, zr[pr][g].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            H[pr][g][2 * j] = __builtin_amdgcn_perm(zs[j], xs[j], 0x05040100u);       // (x.lo, z.lo)
            H[pr][g][2 * j + 1] = __builtin_amdgcn_perm(zs[j], xs[j], 0x07060302u);   // (x.hi, z.hi)
          }
        }

      // ---- k loop: W_k streams through the double buffer, S_v[k] is built and multiplied
      __syncthreads();                        // every wave is done with the stage buffers of the previous pass
      for (int i = tid; i < NBG * VS_STAGE_U4; i += 512) {
        const int nbg = i / VS_STAGE_U4, o = i - nbg * VS_STAGE_U4;
        Wbuf[i] = p.apack[(int64_t)(nbg * K) * VS_STAGE_U4 + o];
      }
      __syncthreads();
      for (int k = 0; k < K; ++k) {
        uint4 wn[NBG];
        if (k + 1 < K) {
#pragma unroll
          for (int nbg = 0; nbg < NBG; ++nbg) wn[nbg] = p.apack[(int64_t)(nbg * K + k + 1) * VS_STAGE_U4 + tid];
        }
        const uint32_t bp0 = Bp[(r * 3 + 0) * 16 + k], bp1 = Bp[(r * 3 + 1) * 16 + k], bp2 = Bp[(r * 3 + 2) * 16 + k];
        const uint4* wk = Wbuf + (k & 1) * NBG * VS_STAGE_U4;
#pragma unroll
        for (int g = 0; g < PM_GC; ++g) {
          float s[8];
#pragma unroll
          for (int c = 0; c < 8; ++c) {
            float t = vs_dot2(H[0][g][c], bp0, 0.f);
            t = vs_dot2(H[1][g][c], bp1, t);
            s[c] = vs_dot2(H[2][g][c], bp2, t);
          }
          uint4 X;
          X.x = pack_bf16x2(s[0], s[1]); X.y = pack_bf16x2(s[2], s[3]);
          X.z = pack_bf16x2(s[4], s[5]); X.w = pack_bf16x2(s[6], s[7]);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const uint4 a = wk[(nb >> 1) * VS_STAGE_U4 + (nb & 1) * PM_GC * 64 + g * 64 + lane];
            y[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, X),
                                                            y[nb], 0, 0, 0);
          }
        }
        if (k + 1 < K) {
          uint4* wd = Wbuf + ((k + 1) & 1) * NBG * VS_STAGE_U4;
#pragma unroll
          for (int nbg = 0; nbg < NBG; ++nbg) wd[nbg * VS_STAGE_U4 + tid] = wn[nbg];
        }
        __syncthreads();
      }
    }

    // ---- store: lane (r, hh) holds, per 32-wide block, the channels q4 * 8 + hh * 4 + i of its vertex
    if (vok) {
      const int Cn = 64 * NBG;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        uint16_t* dst = p.out + v * Cn + nb * 32 + hh * 4;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          uint2 w;
          w.x = pack_bf16x2(y[nb][q4 * 4], y[nb][q4 * 4 + 1]);
          w.y = pack_bf16x2(y[nb][q4 * 4 + 2], y[nb][q4 * 4 + 3]);
          *(uint2*)(dst + q4 * 8) = w;
        }
      }
    }
  }
}

bool pm_f2v_vs_applies(pm_dtype dt, int K, int cin, int cout, const void* h, const void* out) {
  return dt == PM_BF16 && K <= 16 && cin == 64 && (cout == 64 || cout == 128) && pm_aligned16(h) && pm_aligned16(out);
}

// apack: the PLAIN packed image of W (pm_launch_pack), already enqueued on `st`
pm_status pm_launch_f2v_vs(const pm_mesh* mesh, const int32_t* row_ptr, const int32_t* col, int K, int cout,
                           const ShTable& sh, const void* h, const void* apack, void* out, hipStream_t st) {
  const int64_t V = mesh->n_vert;
  if (V == 0) return PM_OK;
  VsP p;
  p.V = V; p.K = K; p.NBG = cout / 64; p.sh = sh; p.vert = mesh->vert; p.facet = mesh->facet; p.row_ptr = row_ptr;
  p.col = col; p.h = (const uint16_t*)h; p.apack = (const uint4*)apack; p.out = (uint16_t*)out;
  const size_t lds = (size_t)2 * p.NBG * PM_STAGE_BYTES + (size_t)8 * 32 * 3 * 16 * 4;
  int64_t grid = (V + 255) / 256;
  if (grid > 256) grid = 256;
  auto kern = p.NBG == 1 ? k_f2v_vs<2> : k_f2v_vs<4>;
  PM_CHECK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  { ProfScope ps__(st, "k_f2v_vs");
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), lds, st, p); }
  PM_CHECK_LAUNCH("k_f2v_vs");
  return PM_OK;
}
