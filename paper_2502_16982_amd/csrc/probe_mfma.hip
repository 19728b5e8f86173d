// Measurement aid: what the matrix cores of this chip sustain on bf16 operands that never leave registers.
// One 256-thread block per compute unit runs 4x4 register-blocked v_mfma_f32_32x32x16_bf16 (the Newton-Schulz
// kernels' instruction and blocking) with no memory traffic at all, so the result is the ceiling that any bf16
// GEMM on this chip lives under.  It depends on the operand VALUES: with random operands the chip lowers its
// clock to stay inside its power budget, with zeros it does not.  The optimizer path never calls this.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "../../include/muon.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kFrags = 16;        // 8 A-side + 8 B-side operand fragments per lane
constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads, 1) void mfma_rate_kernel(const u32x4* __restrict__ in, float* __restrict__ out,
                                                                long long* __restrict__ clk, int iters) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, in[i * kThreads + threadIdx.x]);
    b[i] = __builtin_bit_cast(bf16x8, in[(8 + i) * kThreads + threadIdx.x]);
  }
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[h * 4 + i], b[h * 4 + j], acc[i][j], 0, 0, 0);
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) s += acc[i][j][v];
  out[blockIdx.x * kThreads + threadIdx.x] = s;        // keeps the accumulators alive
  if (threadIdx.x == 0) {
    clk[blockIdx.x * 2] = c1 - c0;                     // core clocks
    clk[blockIdx.x * 2 + 1] = w1 - w0;                 // 100 MHz ticks
  }
}

unsigned short f32_to_bf16_host(float f) {
  unsigned u;
  __builtin_memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

}  // namespace

extern "C" int muon_probe_mfma_rate(int random_operands, int iters, double* tflops_out, double* clock_mhz_out) {
  if (iters <= 0 || iters > (1 << 20) || !tflops_out || !clock_mhz_out) return MUON_E_INVALID_ARG;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MUON_E_HIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return MUON_E_HIP;
  const size_t n = (size_t)kFrags * kThreads * 8;      // bf16 elements
  std::vector<unsigned short> host(n, 0);
  if (random_operands) {
    uint32_t state = 0x9e3779b9u;                      // xorshift32: values uniform in (-1, 1)
    for (auto& v : host) {
      state ^= state << 13; state ^= state >> 17; state ^= state << 5;
      v = f32_to_bf16_host((float)(state >> 8) * (2.0f / 16777216.0f) - 1.0f);
    }
  }
  unsigned short* d_in = nullptr;
  float* d_out = nullptr;
  long long* d_clk = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = MUON_E_HIP;
  do {
    if (hipMalloc(&d_in, n * 2) != hipSuccess) break;
    if (hipMalloc(&d_out, (size_t)cus * kThreads * sizeof(float)) != hipSuccess) break;
    if (hipMalloc(&d_clk, (size_t)cus * 2 * sizeof(long long)) != hipSuccess) break;
    if (hipMemcpy(d_in, host.data(), n * 2, hipMemcpyHostToDevice) != hipSuccess) break;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) break;
    float ms = 0.f;
    bool ok = true;
    for (int rep = 0; rep < 3 && ok; ++rep) {          // the last repetition is the one reported (clock settled)
      ok = hipEventRecord(e0, nullptr) == hipSuccess;
      mfma_rate_kernel<<<cus, kThreads, 0, nullptr>>>(reinterpret_cast<const u32x4*>(d_in), d_out, d_clk, iters);
      ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(e1, nullptr) == hipSuccess &&
           hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    }
    if (!ok || ms <= 0.f) break;
    long long hc[2] = {0, 0};
    if (hipMemcpy(hc, d_clk, sizeof(hc), hipMemcpyDeviceToHost) != hipSuccess) break;
    const double flops = (double)cus * 4 /*waves*/ * iters * 32 /*MFMAs*/ * 2.0 * 32 * 32 * 16;
    *tflops_out = flops / (ms * 1e-3) / 1e12;
    *clock_mhz_out = hc[1] > 0 ? (double)hc[0] / (double)hc[1] * 100.0 : 0.0;
    rc = MUON_OK;
  } while (false);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(d_in);
  (void)hipFree(d_out);
  (void)hipFree(d_clk);
  return rc;
}
