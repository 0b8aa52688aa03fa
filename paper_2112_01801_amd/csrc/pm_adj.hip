// Vertex -> facet adjacency N(v) (receptive field of Eq. 5) as a CSR over corner slots, and mesh validation.
//
// Build: histogram of corner references (integer atomics: the counts are order-independent), exclusive
// scan, scatter of slot ids 3f+j through per-vertex cursors (order inside a row is arbitrary at this
// point), then every row is sorted ascending so that the result is unique and the reductions that
// walk it are reproducible.  Short rows are rank-sorted by one thread, long rows by one workgroup.
#include "pm_host.h"

#define SCAN_ITEMS 8
#define SCAN_BLOCK 256
#define SCAN_TILE (SCAN_ITEMS * SCAN_BLOCK)
#define SHORT_ROW 16
#define MID_ROW 256

__global__ void k_fill_i32(int32_t* p, int64_t n, int32_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// entries with a negative key belong to no row
__global__ void k_count(int64_t n3, const int32_t* __restrict__ facet, int32_t* __restrict__ cnt) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n3 && facet[e] >= 0) atomicAdd(&cnt[facet[e]], 1);
}

// block-wide exclusive scan of SCAN_TILE items; returns the tile total through *total (thread 0)
__device__ int32_t block_scan_tile(const int32_t* __restrict__ in, int32_t* __restrict__ out, int64_t base, int64_t n,
                                   int32_t offset, int32_t* sh) {
  const int t = threadIdx.x;
  int32_t v[SCAN_ITEMS];
  int32_t s = 0;
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    int64_t idx = base + (int64_t)t * SCAN_ITEMS + i;
    v[i] = (idx < n) ? in[idx] : 0;
    s += v[i];
  }
  sh[t] = s;
  __syncthreads();
  // Hillis-Steele inclusive scan over the 256 per-thread sums
  for (int d = 1; d < SCAN_BLOCK; d <<= 1) {
    int32_t add = (t >= d) ? sh[t - d] : 0;
    __syncthreads();
    sh[t] += add;
    __syncthreads();
  }
  int32_t excl = sh[t] - s + offset;
  int32_t total = sh[SCAN_BLOCK - 1];
  if (out) {
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
      int64_t idx = base + (int64_t)t * SCAN_ITEMS + i;
      if (idx < n) out[idx] = excl;
      excl += v[i];
    }
  }
  __syncthreads();
  return total;
}

__global__ void __launch_bounds__(SCAN_BLOCK) k_scan_tile_sums(const int32_t* __restrict__ in, int64_t n,
                                                               int32_t* __restrict__ tile_sum) {
  __shared__ int32_t sh[SCAN_BLOCK];
  int32_t tot = block_scan_tile(in, nullptr, (int64_t)blockIdx.x * SCAN_TILE, n, 0, sh);
  if (threadIdx.x == 0) tile_sum[blockIdx.x] = tot;
}

// single workgroup: exclusive scan of the tile sums, in place
__global__ void __launch_bounds__(SCAN_BLOCK) k_scan_sums(int32_t* __restrict__ tile_sum, int64_t n_tiles) {
  __shared__ int32_t sh[SCAN_BLOCK];
  int32_t carry = 0;
  for (int64_t base = 0; base < n_tiles; base += SCAN_TILE) {
    int32_t tot = block_scan_tile(tile_sum, tile_sum, base, n_tiles, carry, sh);
    carry += tot;
  }
}

// row_ptr[i] = exclusive prefix of cnt; also writes row_ptr[n] = total when the last tile finishes
__global__ void __launch_bounds__(SCAN_BLOCK) k_scan_apply(const int32_t* __restrict__ cnt, int64_t n,
                                                           const int32_t* __restrict__ tile_off,
                                                           int32_t* __restrict__ row_ptr, int32_t* __restrict__ cursor) {
  __shared__ int32_t sh[SCAN_BLOCK];
  int64_t base = (int64_t)blockIdx.x * SCAN_TILE;
  int32_t off = tile_off[blockIdx.x];
  int32_t tot = block_scan_tile(cnt, row_ptr, base, n, off, sh);
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) row_ptr[n] = off + tot;
  // cursors start at the row starts
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    int64_t idx = base + (int64_t)threadIdx.x * SCAN_ITEMS + i;
    if (cursor && idx < n) cursor[idx] = row_ptr[idx];
  }
}

__global__ void k_scatter(int64_t n3, const int32_t* __restrict__ facet, int32_t* __restrict__ cursor,
                          int32_t* __restrict__ tmp) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n3 && facet[e] >= 0) {
    int32_t pos = atomicAdd(&cursor[facet[e]], 1);
    tmp[pos] = (int32_t)e;
  }
}

// rank sort of short rows (entries are distinct); longer rows are queued: medium ones from the front of
// `long_rows` (count n_long[1]) for k_sort_mid, long ones from its back (count n_long[0]) for k_sort_long
__global__ void k_sort_short(int64_t V, const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ tmp,
                             int32_t* __restrict__ col, int32_t* __restrict__ long_rows, int32_t* __restrict__ n_long) {
  int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= V) return;
  int32_t b = row_ptr[v], e = row_ptr[v + 1];
  int32_t d = e - b;
  if (d > MID_ROW) {
    int32_t slot = atomicAdd(&n_long[0], 1);
    long_rows[V - 1 - slot] = (int32_t)v;
    return;
  }
  if (d > SHORT_ROW) {
    int32_t slot = atomicAdd(&n_long[1], 1);
    long_rows[slot] = (int32_t)v;
    return;
  }
  for (int32_t i = b; i < e; ++i) {
    int32_t x = tmp[i];
    int32_t rank = 0;
    for (int32_t j = b; j < e; ++j) rank += (tmp[j] < x) ? 1 : 0;
    col[b + rank] = x;
  }
}

// rows of SHORT_ROW+1 .. MID_ROW entries: one wave per queued row, the row in the wave's own LDS tile, every lane
// ranks its entries against the whole row
__global__ void __launch_bounds__(256) k_sort_mid(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ tmp,
                                                  int32_t* __restrict__ col, const int32_t* __restrict__ long_rows,
                                                  const int32_t* __restrict__ n_long) {
  __shared__ int32_t tiles[4][MID_ROW];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int32_t* tile = tiles[wave];
  const int32_t nl = n_long[1];
  for (int32_t q = blockIdx.x * 4 + wave; q < nl; q += gridDim.x * 4) {
    const int32_t v = long_rows[q];
    const int32_t b = row_ptr[v], d = row_ptr[v + 1] - b;
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < d; i += 64) tile[i] = tmp[b + i];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < d; i += 64) {
      const int32_t x = tile[i];
      int32_t rank = 0;
      for (int j = 0; j < d; ++j) rank += (tile[j] < x) ? 1 : 0;
      col[b + rank] = x;
    }
  }
}

__global__ void __launch_bounds__(256) k_sort_long(int64_t V, const int32_t* __restrict__ row_ptr,
                                                   const int32_t* __restrict__ tmp, int32_t* __restrict__ col,
                                                   const int32_t* __restrict__ long_rows,
                                                   const int32_t* __restrict__ n_long) {
  __shared__ int32_t tile[1024];
  const int32_t nl = n_long[0];
  for (int32_t q = blockIdx.x; q < nl; q += gridDim.x) {
    int32_t v = long_rows[V - 1 - q];
    int32_t b = row_ptr[v], e = row_ptr[v + 1];
    // every thread owns entries i = b + t, b + t + 256, ...; ranks accumulate over LDS tiles of the row
    for (int32_t i0 = b; i0 < e; i0 += 256) {
      int32_t i = i0 + threadIdx.x;
      int32_t x = (i < e) ? tmp[i] : 0;
      int32_t rank = 0;
      for (int32_t j0 = b; j0 < e; j0 += 1024) {
        __syncthreads();
        for (int32_t j = threadIdx.x; j < 1024; j += 256) tile[j] = (j0 + j < e) ? tmp[j0 + j] : 0x7fffffff;
        __syncthreads();
        int32_t lim = min(1024, e - j0);
        for (int32_t j = 0; j < lim; ++j) rank += (tile[j] < x) ? 1 : 0;
      }
      if (i < e) col[b + rank] = x;
    }
    __syncthreads();
  }
}

size_t pm_adj_ws_bytes(int64_t n_vert, int64_t n_facet) { return pm_csr_ws_bytes(n_vert, 3 * n_facet); }

// workspace of pm_launch_csr: n_vert rows, n3 entries
size_t pm_csr_ws_bytes(int64_t n_vert, int64_t n3) {
  int64_t n_tiles = (n_vert + SCAN_TILE - 1) / SCAN_TILE + 1;
  size_t b = 0;
  b += pm_round_up((size_t)(n_vert + 1) * 4, 256);  // cnt
  b += pm_round_up((size_t)(n_vert + 1) * 4, 256);  // cursor
  b += pm_round_up((size_t)n_tiles * 4, 256);       // tile sums
  b += pm_round_up((size_t)(n3 + 1) * 4, 256);      // tmp
  b += pm_round_up((size_t)(n_vert + 1) * 4, 256);  // long rows
  b += 256;                                         // n_long
  return b;
}

static inline unsigned nblk(int64_t n, int b) { return (unsigned)((n + b - 1) / b); }

pm_status pm_launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t st) {
  if (n <= 0) return PM_OK;
  { ProfScope ps__(st, "k_fill_i32");
    hipLaunchKernelGGL(k_fill_i32, dim3(nblk(n, 256)), dim3(256), 0, st, p, n, v); }
  PM_CHECK_LAUNCH("k_fill_i32");
  return PM_OK;
}

// out[i] = sum of cnt[0..i) for i = 0..n (n + 1 outputs); tile_ws holds pm_scan_ws_bytes(n)
size_t pm_scan_ws_bytes(int64_t n) { return pm_round_up((size_t)((n + SCAN_TILE - 1) / SCAN_TILE + 2) * 4, 256); }

pm_status pm_launch_exclusive_scan(const int32_t* cnt, int64_t n, int32_t* out, void* tile_ws, hipStream_t st) {
  if (n == 0) return pm_launch_fill_i32(out, 1, 0, st);
  const int64_t n_tiles = (n + SCAN_TILE - 1) / SCAN_TILE;
  int32_t* tsum = (int32_t*)tile_ws;
  { ProfScope ps__(st, "k_scan_tile_sums");
    hipLaunchKernelGGL(k_scan_tile_sums, dim3((unsigned)n_tiles), dim3(SCAN_BLOCK), 0, st, cnt, n, tsum); }
  { ProfScope ps__(st, "k_scan_sums");
    hipLaunchKernelGGL(k_scan_sums, dim3(1), dim3(SCAN_BLOCK), 0, st, tsum, n_tiles); }
  { ProfScope ps__(st, "k_scan_apply");
    hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)n_tiles), dim3(SCAN_BLOCK), 0, st, cnt, n, tsum, out, (int32_t*)nullptr); }
  PM_CHECK_LAUNCH("exclusive scan");
  return PM_OK;
}

pm_status pm_launch_adjacency(const pm_mesh* mesh, int32_t* row_ptr, int32_t* col, void* ws, hipStream_t st) {
  return pm_launch_csr(mesh->n_vert, 3 * mesh->n_facet, mesh->facet, row_ptr, col, ws, st);
}

// CSR of the entries e = 0..n3-1 grouped by key[e] in [0, V) (negative keys are skipped), ascending inside a row
pm_status pm_launch_csr(int64_t V, int64_t n3, const int32_t* keys, int32_t* row_ptr, int32_t* col, void* ws,
                        hipStream_t st) {
  const int64_t n_tiles = (V + SCAN_TILE - 1) / SCAN_TILE;
  char* p = (char*)ws;
  int32_t* cnt = (int32_t*)p;      p += pm_round_up((size_t)(V + 1) * 4, 256);
  int32_t* cursor = (int32_t*)p;   p += pm_round_up((size_t)(V + 1) * 4, 256);
  int32_t* tsum = (int32_t*)p;     p += pm_round_up((size_t)(n_tiles + 1) * 4, 256);
  int32_t* tmp = (int32_t*)p;      p += pm_round_up((size_t)(n3 + 1) * 4, 256);
  int32_t* long_rows = (int32_t*)p; p += pm_round_up((size_t)(V + 1) * 4, 256);
  int32_t* n_long = (int32_t*)p;

  { ProfScope ps__(st, "k_fill_i32");
    hipLaunchKernelGGL(k_fill_i32, dim3(nblk(V + 1, 256)), dim3(256), 0, st, cnt, V + 1, 0); }
  { ProfScope ps__(st, "k_fill_i32");
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, st, n_long, (int64_t)2, 0); }
  if (V == 0) {
    { ProfScope ps__(st, "k_fill_i32");
      hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, st, row_ptr, (int64_t)1, 0); }
    PM_CHECK_LAUNCH("adjacency(empty)");
    return PM_OK;
  }
  if (n3 > 0) hipLaunchKernelGGL(k_count, dim3(nblk(n3, 256)), dim3(256), 0, st, n3, keys, cnt);
  { ProfScope ps__(st, "k_scan_tile_sums");
    hipLaunchKernelGGL(k_scan_tile_sums, dim3((unsigned)n_tiles), dim3(SCAN_BLOCK), 0, st, cnt, V, tsum); }
  { ProfScope ps__(st, "k_scan_sums");
    hipLaunchKernelGGL(k_scan_sums, dim3(1), dim3(SCAN_BLOCK), 0, st, tsum, n_tiles); }
  { ProfScope ps__(st, "k_scan_apply");
    hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)n_tiles), dim3(SCAN_BLOCK), 0, st, cnt, V, tsum, row_ptr, cursor); }
  if (n3 > 0) {
    { ProfScope ps__(st, "k_scatter");
      hipLaunchKernelGGL(k_scatter, dim3(nblk(n3, 256)), dim3(256), 0, st, n3, keys, cursor, tmp); }
    { ProfScope ps__(st, "k_sort_short");
      hipLaunchKernelGGL(k_sort_short, dim3(nblk(V, 256)), dim3(256), 0, st, V, row_ptr, tmp, col, long_rows, n_long); }
    { ProfScope ps__(st, "k_sort_mid");
      hipLaunchKernelGGL(k_sort_mid, dim3(2048), dim3(256), 0, st, row_ptr, tmp, col, long_rows, n_long); }
    { ProfScope ps__(st, "k_sort_long");
      hipLaunchKernelGGL(k_sort_long, dim3(256), dim3(256), 0, st, V, row_ptr, tmp, col, long_rows, n_long); }
  }
  PM_CHECK_LAUNCH("adjacency");
  return PM_OK;
}

// flag bit 0: facet id outside its mesh's vertex range; bit 1: offsets not monotone / not spanning
__global__ void k_validate(int n_mesh, int64_t V, int64_t F, const int32_t* __restrict__ facet,
                           const int32_t* __restrict__ vert_off, const int32_t* __restrict__ facet_off,
                           int32_t* __restrict__ flag) {
  int64_t f = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (f == 0 && vert_off && facet_off) {
    int bad = (vert_off[0] != 0) || (facet_off[0] != 0) || (vert_off[n_mesh] != V) || (facet_off[n_mesh] != F);
    for (int m = 0; m < n_mesh; ++m) bad |= (vert_off[m + 1] < vert_off[m]) || (facet_off[m + 1] < facet_off[m]);
    if (bad) atomicOr(flag, 2);
  }
  if (f >= F) return;
  int64_t lo = 0, hi = V;
  if (vert_off && facet_off) {
    int a = 0, b = n_mesh;  // find m with facet_off[m] <= f < facet_off[m+1]
    while (b - a > 1) {
      int mid = (a + b) >> 1;
      if (facet_off[mid] <= f) a = mid; else b = mid;
    }
    lo = vert_off[a];
    hi = vert_off[a + 1];
  }
  for (int j = 0; j < 3; ++j) {
    int32_t v = facet[3 * f + j];
    if (v < lo || v >= hi) atomicOr(flag, 1);
  }
}

pm_status pm_launch_validate(const pm_mesh* mesh, int32_t* flag, hipStream_t st) {
  { ProfScope ps__(st, "k_fill_i32");
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, st, flag, (int64_t)1, 0); }
  int64_t n = mesh->n_facet > 0 ? mesh->n_facet : 1;
  { ProfScope ps__(st, "k_validate");
    hipLaunchKernelGGL(k_validate, dim3(nblk(n, 256)), dim3(256), 0, st, mesh->n_mesh, mesh->n_vert, mesh->n_facet,
                     mesh->facet, mesh->vert_off, mesh->facet_off, flag); }
  PM_CHECK_LAUNCH("k_validate");
  return PM_OK;
}
