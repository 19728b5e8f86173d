// Host-callable launchers of the HIP kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>

#include "muon_tables.h"

namespace muon {

// One-time per-process kernel attribute setup (large dynamic LDS).  Returns a hipError_t.
hipError_t gemm_setup();
// Blocks of a persistent coarse GEMM launch = compute units of the device gemm_setup ran on (0 before it).
int gemm_coarse_blocks();

// a1-a3: momentum, sum of squares, cast + orient.  both_layouts != 0: U goes to X and Xt[0] (one holds U, the other
// U^T); 0: only X (the orientation with rows <= cols) is written.  One block per EwTile.
hipError_t launch_momentum_norm_cast(const MatDesc* mats, const MatPtrs* ptrs, const EwTile* tiles, int n_tiles,
                                     float mu, int nesterov, int both_layouts, int ns_dtype, hipStream_t s);

// a2 second stage: fixed-order sum of the partials of each matrix, s = 1/(sqrt(sum)+eps).
hipError_t launch_norm_finalize(const MatDesc* mats, int first_mat, int n_mats, double eps, hipStream_t s);

// a4-a6: grouped NT GEMM with fused epilogue.  alpha_idx: -1 none, 0 -> scal[0], 1 -> scal[1].  diag_add: constant
// added to the diagonal of the outputs of problems that ask for it (GemmProblem::diag_add), bf16 kernel only.
// coarse: 0 = every tile of the table is 128 x 128 (two blocks per compute unit); 1 = the table mixes 256 x 256 and,
// with kGemmStrips in `flags`, 512 x 128 tiles (one block per compute unit; the flag selects the larger LDS
// allocation).  kGemmPersistent: one block per compute unit works through the table with stride gridDim (for launches
// whose tiles run K loops of nearly the same length, which the planner balances statically; with a wide spread of K
// the hardware's dynamic block dispatch does better).
// l_kmajor: every problem of the launch stores its L operand K-major (element (i, k) at L[k * ldl + i]).
// planes: 1 = plain bf16; 2 or 3 = every matrix is a sum of that many bf16 planes (GemmProblem::*_plane strides).
constexpr int kGemmStrips = 1, kGemmPersistent = 2;
hipError_t launch_gemm_bf16(int coarse, int flags, const GemmProblem* probs, const GemmTile* tiles, int n_tiles,
                            float beta_acc, float beta_e, int alpha_idx, float diag_add, int l_kmajor, int planes,
                            hipStream_t s);
hipError_t launch_gemm_f32(const GemmProblem* probs, const GemmTile* tiles, int n_tiles,
                           float beta_acc, float beta_e, int alpha_idx, hipStream_t s);

// a8: W <- W - lr*(scale*O + wd*W); also leaves per-tile sums of O^2 in the partials.
// o_sel: where O sits in W's orientation: bit 0 picks Xt[0] / Xt[1] for matrices iterated on their transpose, bit 1
// picks X (0) or Xt[0] (1) for the others; use_s: multiply O by scal[0] (only when no Newton-Schulz iteration ran).
// scale_mode: 0 factor = rms_scale*sqrt(max(A,B)); 1 factor = rms_scale*sqrt_hidden; 2 factor = rms_scale*scal[2]
// (scal[2] = 1/RMS of the stored O, left there by launch_update_rms(..., to_scal = 1)).
hipError_t launch_apply_update(const MatDesc* mats, const MatPtrs* ptrs, const EwTile* tiles, int n_tiles,
                               float lr, float wd, float rms_scale, int scale_mode, float sqrt_hidden, int o_sel,
                               int use_s, int ns_dtype, hipStream_t s);

// Per-tile sums of O^2 into the partials, without touching W (first pass of the "Update Norm" variant).
hipError_t launch_update_sumsq(const MatDesc* mats, const EwTile* tiles, int n_tiles, int o_sel, int ns_dtype, hipStream_t s);

// From the per-tile sums of O^2: to_scal = 0 writes sqrt(mean(O^2)) per matrix to out; to_scal = 1 writes
// 1/sqrt(mean(stored O^2)) (0 when O = 0) to scal[2].
hipError_t launch_update_rms(const MatDesc* mats, int first_mat, int n_mats, int use_s, int to_scal, float* out, hipStream_t s);

// Test hook: O of one matrix -> dst (rows x cols contiguous).
hipError_t launch_read_update(const MatDesc* mats, int mat, int o_sel, int use_s, int ns_dtype, void* dst,
                              int dst_dtype, hipStream_t s);

// AdamW (non-matrix parameters): up to kAdamwSlots tensors per launch, passed by value in the kernel arguments.
constexpr int kAdamwSlots = 24;
struct AdamwBatch {
  void* p[kAdamwSlots];
  const void* g[kAdamwSlots];
  float* m[kAdamwSlots];
  float* v[kAdamwSlots];
  long long numel[kAdamwSlots];
  int block_start[kAdamwSlots + 1];   // first block of each tensor; [n] = total blocks
  int p_dtype[kAdamwSlots], g_dtype[kAdamwSlots];
  int n;
};
long long adamw_blocks_for(long long numel);
hipError_t launch_adamw(const AdamwBatch& batch, int n_blocks, float lr, float wd, float beta1, float beta2, float eps,
                        float inv_bc1, float inv_bc2, hipStream_t s);

}  // namespace muon
