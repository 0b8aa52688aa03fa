// Declarations shared by the two weight-gradient kernels (general and producer/consumer).
#pragma once
#include "pm_rows.h"

#define WG_RT 64          /* rows per staged tile */
#define WG_KG 16          /* k values per workgroup */
#define XP_BF16 72        /* LDS pitch of a channel row, bf16 elements (144 B) */
#define XP_F32 68         /* LDS pitch, fp32 elements (272 B) */

struct WgradP {
  int64_t R, rows_per_part;
  int K, Cc, Cn;
  int KGn, CBP, NBP;   // slab decomposition
  int NKPW, RS;        // k-pairs per workgroup, row splits
  BasisSrc bs;         // bs.bvals: precomputed basis rows [R][K] (unused for B_ONE)
  RowSrc xs, ys;
  float* partial;      // [n_part * RS][K][Cc][Cn]
  void* y_out;         // optional (producer/consumer kernel): the Y operand rows [R][Cn] are also written here, bf16
};

// Producer/consumer variant (see pm_wgrad_fuses_basis for when it applies).
pm_status pm_launch_wgrad_pc(BMode bm, XMode ym, const WgradP& p, int n_part, int slabs, hipStream_t st);
