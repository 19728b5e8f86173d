// Newton-Schulz products for gfx950 (Eq. 2 of the paper): grouped "NT" GEMMs
//     C[i][j] = sum_k L[i][k] * R[j][k]
// with a fused epilogue  val = alpha * (beta_acc * acc + beta_e * E[i][j]).  All three products of one
// iteration have this form once the iterate is kept in both layouts (X and X^T):
//     Gram      A  = X X^T            L = R = X        (symmetric output)
//     polynomial B = b A + c A A      L = R = A        (A symmetric, so A A = A A^T; symmetric output)
//     apply     X' = a X + B X        L = B, R = X^T   (stores X' and/or X'^T)
// Operands are zero-padded to whole tiles by the producer, so the kernels have no edge handling.
//
// bf16 kernel: v_mfma_f32_32x32x16_bf16, fp32 accumulation, 4 waves per block arranged 2x2, K staged through
// LDS in 64-wide slabs, double buffered, global loads for slab k+1 in flight while slab k is multiplied.
#include <hip/hip_runtime.h>

#include "muon_launch.h"

namespace muon {
namespace {

typedef unsigned short u16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 64;            // K slab (bf16 elements)
constexpr int PITCH = BK + 8;     // LDS row pitch in elements: 144 B, keeps 16-lane b128 reads on distinct banks

__device__ __forceinline__ float bf16_to_f32(u16 h) { return __uint_as_float(((unsigned)h) << 16); }
__device__ __forceinline__ u16 f32_to_bf16(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u16)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (u16)(u >> 16);
}

template <int BM, int BN>
__global__ __launch_bounds__(256, 1) void ns_gemm_bf16_kernel(const GemmProblem* __restrict__ probs,
                                                               const GemmTile* __restrict__ tiles, float beta_acc,
                                                               float beta_e, int alpha_idx) {
  constexpr int WTM = BM / 2, WTN = BN / 2;   // wave tile
  constexpr int FM = WTM / 32, FN = WTN / 32; // 32x32 MFMA tiles per wave
  constexpr int LCH = BM * 8 / 256, RCH = BN * 8 / 256;  // 16-byte chunks per thread per slab
  constexpr int STAGE = (BM + BN) * PITCH;    // elements per LDS stage

  extern __shared__ __align__(16) unsigned char smem_raw[];
  u16* smem = reinterpret_cast<u16*>(smem_raw);

  const GemmTile tile = tiles[blockIdx.x];
  const GemmProblem p = probs[tile.prob];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int row0 = tile.ti * BM, col0 = tile.tj * BN;

  // global -> register staging: chunk c = tid + 256*i covers row (tid>>3) + 32*i, k-chunk tid&7
  const int ld_row = tid >> 3, ld_kc = tid & 7;
  const u16* lptr = static_cast<const u16*>(p.L) + (size_t)(row0 + ld_row) * p.ldl + ld_kc * 8;
  const u16* rptr = static_cast<const u16*>(p.R) + (size_t)(col0 + ld_row) * p.ldr + ld_kc * 8;
  const size_t lstep = (size_t)32 * p.ldl, rstep = (size_t)32 * p.ldr;
  u32x4 lreg[LCH], rreg[RCH];

  auto gload = [&](int kt) {
#pragma unroll
    for (int i = 0; i < LCH; ++i) lreg[i] = *reinterpret_cast<const u32x4*>(lptr + i * lstep + (size_t)kt * BK);
#pragma unroll
    for (int i = 0; i < RCH; ++i) rreg[i] = *reinterpret_cast<const u32x4*>(rptr + i * rstep + (size_t)kt * BK);
  };
  auto sstore = [&](int stage) {
    u16* sl = smem + stage * STAGE + ld_row * PITCH + ld_kc * 8;
    u16* sr = sl + BM * PITCH;
#pragma unroll
    for (int i = 0; i < LCH; ++i) *reinterpret_cast<u32x4*>(sl + i * 32 * PITCH) = lreg[i];
#pragma unroll
    for (int i = 0; i < RCH; ++i) *reinterpret_cast<u32x4*>(sr + i * 32 * PITCH) = rreg[i];
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int KT = p.K / BK;
  // fragment read offsets inside a stage (elements)
  const int a_off = (wm * WTM + (lane & 31)) * PITCH + (lane >> 5) * 8;
  const int b_off = BM * PITCH + (wn * WTN + (lane & 31)) * PITCH + (lane >> 5) * 8;

  gload(0);
  sstore(0);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) gload(kt + 1);
    const u16* sa = smem + cur * STAGE + a_off;
    const u16* sb = smem + cur * STAGE + b_off;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[FM], bfr[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(sa + i * 32 * PITCH + kk * 16);
#pragma unroll
      for (int j = 0; j < FN; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(sb + j * 32 * PITCH + kk * 16);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) sstore(cur ^ 1);
    __syncthreads();
  }

  // ---- epilogue: val = alpha * (beta_acc*acc + beta_e*E), stored to C and/or transposed to Ct ----
  const float alpha = alpha_idx >= 0 ? p.scal[alpha_idx] : 1.f;
  const u16* E = static_cast<const u16*>(p.E);
  u16* C = static_cast<u16*>(p.C);
  u16* Ct = static_cast<u16*>(p.Ct);
  int ldct = p.ldct;
  if (p.symmetric) {
    Ct = (tile.ti != tile.tj) ? C : nullptr;
    ldct = p.ldc;
  }
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int c = col0 + wn * WTN + j * 32 + (lane & 31);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int rbase = row0 + wm * WTM + i * 32 + 8 * q + 4 * (lane >> 5);
        u16 h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float x = beta_acc * acc[i][j][4 * q + e];
          if (E) x = fmaf(beta_e, bf16_to_f32(E[(size_t)(rbase + e) * p.lde + c]), x);
          h[e] = f32_to_bf16(alpha * x);
          if (C) C[(size_t)(rbase + e) * p.ldc + c] = h[e];
        }
        if (Ct) {
          u32x2 pk;
          pk.x = (unsigned)h[0] | ((unsigned)h[1] << 16);
          pk.y = (unsigned)h[2] | ((unsigned)h[3] << 16);
          *reinterpret_cast<u32x2*>(Ct + (size_t)c * ldct + rbase) = pk;
        }
      }
    }
  }
}

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
  const int row0 = tile.ti * T, col0 = tile.tj * T;
  const int ld_row = tid >> 2, ld_k4 = (tid & 3) * 4;
  const float* lptr = static_cast<const float*>(p.L) + (size_t)(row0 + ld_row) * p.ldl + ld_k4;
  const float* rptr = static_cast<const float*>(p.R) + (size_t)(col0 + ld_row) * p.ldr + ld_k4;

  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

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
  }

  const float alpha = alpha_idx >= 0 ? p.scal[alpha_idx] : 1.f;
  const float* E = static_cast<const float*>(p.E);
  float* C = static_cast<float*>(p.C);
  float* Ct = static_cast<float*>(p.Ct);
  int ldct = p.ldct;
  if (p.symmetric) {
    Ct = (tile.ti != tile.tj) ? C : nullptr;
    ldct = p.ldc;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = row0 + ty * 4 + i;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = col0 + tx * 4 + j;
      float x = beta_acc * acc[i][j];
      if (E) x = fmaf(beta_e, E[(size_t)r * p.lde + c], x);
      x *= alpha;
      if (C) C[(size_t)r * p.ldc + c] = x;
      if (Ct) Ct[(size_t)c * ldct + r] = x;
    }
  }
}

template <int BM, int BN>
constexpr size_t gemm_lds_bytes() { return (size_t)2 * (BM + BN) * PITCH * sizeof(u16); }

}  // namespace

hipError_t gemm_setup() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&ns_gemm_bf16_kernel<128, 128>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds_bytes<128, 128>());
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&ns_gemm_bf16_kernel<256, 256>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds_bytes<256, 256>());
}

hipError_t launch_gemm_bf16(int shape, const GemmProblem* probs, const GemmTile* tiles, int n_tiles, float beta_acc,
                            float beta_e, int alpha_idx, hipStream_t s) {
  if (n_tiles <= 0) return hipSuccess;
  if (shape == kShape128)
    ns_gemm_bf16_kernel<128, 128><<<n_tiles, 256, gemm_lds_bytes<128, 128>(), s>>>(probs, tiles, beta_acc, beta_e, alpha_idx);
  else if (shape == kShape256)
    ns_gemm_bf16_kernel<256, 256><<<n_tiles, 256, gemm_lds_bytes<256, 256>(), s>>>(probs, tiles, beta_acc, beta_e, alpha_idx);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_gemm_f32(const GemmProblem* probs, const GemmTile* tiles, int n_tiles, float beta_acc, float beta_e,
                           int alpha_idx, hipStream_t s) {
  if (n_tiles <= 0) return hipSuccess;
  ns_gemm_f32_kernel<<<n_tiles, 256, 0, s>>>(probs, tiles, beta_acc, beta_e, alpha_idx);
  return hipGetLastError();
}

}  // namespace muon
