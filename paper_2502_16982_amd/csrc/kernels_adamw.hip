// AdamW for the parameters that stay off Muon (RMSNorm gains, LM head, embeddings; section 2.2 of the paper), sharing
// lr and weight decay with it.  HBM-bound elementwise kernel: one launch covers up to kAdamwSlots tensors, whose
// pointers and sizes travel in the kernel arguments (no device table, no workspace); each block owns one
// 4096-element span of one tensor.  fp32 math, moments in fp32, one rounding to the parameter's dtype.
#include <hip/hip_runtime.h>

#include "muon_launch.h"

namespace muon {
namespace {

typedef unsigned short u16;
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

constexpr int kSpan = 4096;   // elements per block (16 per thread)

__device__ __forceinline__ float ld1(const float* p) { return *p; }
__device__ __forceinline__ float ld1(const u16* p) { return __uint_as_float(((unsigned)*p) << 16); }
__device__ __forceinline__ void st1(float* p, float v) { *p = v; }
__device__ __forceinline__ void st1(u16* p, float v) {
  const f32x2_t t = {v, 0.f};
  *p = (u16)(__builtin_bit_cast(unsigned, __builtin_convertvector(t, bf16x2_t)) & 0xffffu);
}

struct AdamwScalars {
  float lr, wd, beta1, beta2, eps;
  float inv_bc1, inv_bc2;   // 1/(1 - beta1^t), 1/(1 - beta2^t)
};

__device__ __forceinline__ void adamw_elem(float& p, float g, float& m, float& v, const AdamwScalars& h) {
  m = fmaf(h.beta1, m, (1.f - h.beta1) * g);
  v = fmaf(h.beta2, v, (1.f - h.beta2) * g * g);
  const float mhat = m * h.inv_bc1, vhat = v * h.inv_bc2;
  const float upd = mhat / (sqrtf(vhat) + h.eps);
  p = fmaf(-h.lr, fmaf(h.wd, p, upd), p);
}

template <typename PT, typename GT>
__device__ __forceinline__ void adamw_span(PT* p, const GT* g, float* m, float* v, long long begin, long long numel,
                                           const AdamwScalars& h) {
  // thread t handles 4 groups of 4 consecutive elements, groups 1024 apart: every wave access is contiguous
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const long long i0 = begin + k * 1024 + threadIdx.x * 4;
    if (i0 + 4 <= numel && ((reinterpret_cast<uintptr_t>(m + i0) | reinterpret_cast<uintptr_t>(v + i0)) & 15u) == 0) {
      float4 mv = *reinterpret_cast<const float4*>(m + i0), vv = *reinterpret_cast<const float4*>(v + i0);
      float pv[4], gv[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) { pv[e] = ld1(p + i0 + e); gv[e] = ld1(g + i0 + e); }
      adamw_elem(pv[0], gv[0], mv.x, vv.x, h);
      adamw_elem(pv[1], gv[1], mv.y, vv.y, h);
      adamw_elem(pv[2], gv[2], mv.z, vv.z, h);
      adamw_elem(pv[3], gv[3], mv.w, vv.w, h);
      *reinterpret_cast<float4*>(m + i0) = mv;
      *reinterpret_cast<float4*>(v + i0) = vv;
#pragma unroll
      for (int e = 0; e < 4; ++e) st1(p + i0 + e, pv[e]);
    } else {
      for (int e = 0; e < 4; ++e) {
        const long long i = i0 + e;
        if (i < numel) {
          float pv = ld1(p + i), mv = m[i], vv = v[i];
          adamw_elem(pv, ld1(g + i), mv, vv, h);
          m[i] = mv; v[i] = vv; st1(p + i, pv);
        }
      }
    }
  }
}

__global__ __launch_bounds__(256) void adamw_kernel(AdamwBatch batch, AdamwScalars h) {
  // find the tensor that owns this block: block_start is a prefix sum over the tensors' block counts
  int t = 0;
#pragma unroll 1
  while (t + 1 < batch.n && (int)blockIdx.x >= batch.block_start[t + 1]) ++t;
  const long long begin = (long long)((int)blockIdx.x - batch.block_start[t]) * kSpan;
  const long long numel = batch.numel[t];
  float* m = batch.m[t];
  float* v = batch.v[t];
  const int pd = batch.p_dtype[t], gd = batch.g_dtype[t];
  if (pd == kDtypeBF16) {
    if (gd == kDtypeBF16) adamw_span(static_cast<u16*>(batch.p[t]), static_cast<const u16*>(batch.g[t]), m, v, begin, numel, h);
    else adamw_span(static_cast<u16*>(batch.p[t]), static_cast<const float*>(batch.g[t]), m, v, begin, numel, h);
  } else {
    if (gd == kDtypeBF16) adamw_span(static_cast<float*>(batch.p[t]), static_cast<const u16*>(batch.g[t]), m, v, begin, numel, h);
    else adamw_span(static_cast<float*>(batch.p[t]), static_cast<const float*>(batch.g[t]), m, v, begin, numel, h);
  }
}

}  // namespace

long long adamw_blocks_for(long long numel) { return (numel + kSpan - 1) / kSpan; }

hipError_t launch_adamw(const AdamwBatch& batch, int n_blocks, float lr, float wd, float beta1, float beta2, float eps,
                        float inv_bc1, float inv_bc2, hipStream_t s) {
  if (n_blocks <= 0) return hipSuccess;
  AdamwScalars h{lr, wd, beta1, beta2, eps, inv_bc1, inv_bc2};
  adamw_kernel<<<n_blocks, 256, 0, s>>>(batch, h);
  return hipGetLastError();
}

}  // namespace muon
