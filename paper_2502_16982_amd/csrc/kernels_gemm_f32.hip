// fp32 Newton-Schulz products for gfx950 (Eq. 2 of the paper), used when the caller asks for fp32 iteration
// arithmetic: grouped "NT" GEMM  C[i][j] = sum_k L[i][k] * R[j][k]  with the same problem/tile tables and
// fused epilogue  val = alpha * (beta_acc * acc + beta_e * E[i][j])  as the bf16 MFMA kernel.
#include <hip/hip_runtime.h>

#include "muon_launch.h"

namespace muon {
namespace {

// ------------------------------------------------------------------------------------------------------
// fp32 Newton-Schulz product: 64x64 block tile, 16-wide K slab, each thread a 4x4 micro-tile, plain FMA.
// Same problem/tile tables and epilogue as the bf16 kernel.
// ------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ns_gemm_f32_kernel(const GemmProblem* __restrict__ probs,
                                                           const GemmTile* __restrict__ tiles, float beta_acc,
                                                           float beta_e, int alpha_idx) {
  constexpr int T = kF32Tile, KS = 16;
  __shared__ float sL[KS][T + 4];
  __shared__ float sR[KS][T + 4];
  const GemmTile tile = tiles[blockIdx.x];
  const GemmProblem p = probs[tile.prob];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int row0 = tile.r0 * kTileUnit, col0 = tile.c0 * kTileUnit;
  const int ld_row = tid >> 2, ld_k4 = (tid & 3) * 4;
  const float* lptr = static_cast<const float*>(p.L) + (size_t)(row0 + ld_row) * p.ldl + ld_k4;
  const float* rptr = static_cast<const float*>(p.R) + (size_t)(col0 + ld_row) * p.ldr + ld_k4;

  // Two-level accumulation: `acc` takes at most kFlush slabs (1024 terms) before it is added to `total`, so the
  // rounding error of a dot product grows with K / 1024 + 1024 terms instead of K (a single fp32 accumulator over
  // 2^20 squares drifts by 4e-4 relative).
  constexpr int kFlush = 64;
  float acc[4][4], total[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = total[i][j] = 0.f;
  int since = 0;

  for (int k0 = 0; k0 < p.K; k0 += KS) {
    const float4 lv = *reinterpret_cast<const float4*>(lptr + k0);
    const float4 rv = *reinterpret_cast<const float4*>(rptr + k0);
    __syncthreads();
    sL[ld_k4 + 0][ld_row] = lv.x; sL[ld_k4 + 1][ld_row] = lv.y; sL[ld_k4 + 2][ld_row] = lv.z; sL[ld_k4 + 3][ld_row] = lv.w;
    sR[ld_k4 + 0][ld_row] = rv.x; sR[ld_k4 + 1][ld_row] = rv.y; sR[ld_k4 + 2][ld_row] = rv.z; sR[ld_k4 + 3][ld_row] = rv.w;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      const float4 a = *reinterpret_cast<const float4*>(&sL[k][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&sR[k][tx * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w};
      const float bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    if (++since == kFlush) {
      since = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          total[i][j] += acc[i][j];
          acc[i][j] = 0.f;
        }
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) total[i][j] += acc[i][j];

  const float alpha = alpha_idx >= 0 ? p.scal[alpha_idx] : 1.f;
  const float* E = static_cast<const float*>(p.E);
  float* C = static_cast<float*>(p.C);
  float* Ct = static_cast<float*>(p.Ct);
  int ldct = p.ldct;
  if (p.symmetric) {
    Ct = (tile.flags & kTileDiagonal) ? nullptr : C;
    ldct = p.ldc;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = row0 + ty * 4 + i;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = col0 + tx * 4 + j;
      float x = beta_acc * total[i][j];
      if (E) x = fmaf(beta_e, E[(size_t)r * p.lde + c], x);
      x *= alpha;
      if (C) C[(size_t)r * p.ldc + c] = x;
      if (Ct) Ct[(size_t)c * ldct + r] = x;
    }
  }
}

}  // namespace

hipError_t launch_gemm_f32(const GemmProblem* probs, const GemmTile* tiles, int n_tiles, float beta_acc, float beta_e,
                           int alpha_idx, hipStream_t s) {
  if (n_tiles <= 0) return hipSuccess;
  ns_gemm_f32_kernel<<<n_tiles, 256, 0, s>>>(probs, tiles, beta_acc, beta_e, alpha_idx);
  return hipGetLastError();
}

}  // namespace muon
