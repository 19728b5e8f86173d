// HBM-bound kernels of the Muon step for gfx950: momentum + Frobenius partials + cast/orient,
// norm finalisation, the scaled weight-decayed apply, update-RMS and a test read-back.
//
// All of them walk a table of 64x64 element tiles so that one launch covers every matrix of a chunk.
#include <hip/hip_runtime.h>

#include "muon_launch.h"

namespace muon {
namespace {

typedef unsigned short u16;

__device__ __forceinline__ float bf16_to_f32(u16 h) { return __uint_as_float(((unsigned)h) << 16); }

// round-to-nearest-even, NaN kept quiet
__device__ __forceinline__ u16 f32_to_bf16(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u16)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (u16)(u >> 16);
}

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// two floats -> packed bf16 pair, round-to-nearest-even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned pack2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}

// Deterministic block-wide sum (256 threads): butterfly inside each wave, then the 4 wave sums in order.
__device__ __forceinline__ float block_sum_256(float v, float* red /* >= 4 floats of LDS */) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

template <typename T>
__device__ __forceinline__ void load16(const T* p, float* out);
template <>
__device__ __forceinline__ void load16<float>(const float* p, float* out) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float4 v = reinterpret_cast<const float4*>(p)[i];
    out[4 * i + 0] = v.x; out[4 * i + 1] = v.y; out[4 * i + 2] = v.z; out[4 * i + 3] = v.w;
  }
}
template <>
__device__ __forceinline__ void load16<u16>(const u16* p, float* out) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const uint4 v = reinterpret_cast<const uint4*>(p)[i];
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      out[8 * i + 2 * j] = __uint_as_float(w[j] << 16);
      out[8 * i + 2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
    }
  }
}

template <typename T>
__device__ __forceinline__ void store16(T* p, const float* in);
template <>
__device__ __forceinline__ void store16<float>(float* p, const float* in) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
    reinterpret_cast<float4*>(p)[i] = make_float4(in[4 * i], in[4 * i + 1], in[4 * i + 2], in[4 * i + 3]);
}
template <>
__device__ __forceinline__ void store16<u16>(u16* p, const float* in) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
    reinterpret_cast<uint4*>(p)[i] = make_uint4(pack2(in[8 * i], in[8 * i + 1]), pack2(in[8 * i + 2], in[8 * i + 3]),
                                                pack2(in[8 * i + 4], in[8 * i + 5]), pack2(in[8 * i + 6], in[8 * i + 7]));
}

template <typename T>
__device__ __forceinline__ float load1(const T* p);
template <>
__device__ __forceinline__ float load1<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load1<u16>(const u16* p) { return bf16_to_f32(*p); }
template <typename T>
__device__ __forceinline__ void store1(T* p, float v);
template <>
__device__ __forceinline__ void store1<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store1<u16>(u16* p, float v) { *p = f32_to_bf16(v); }

__device__ __forceinline__ bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Newton-Schulz storage with PL planes (PL = 1: one array of XT; PL > 1, XT = bf16: the value is the sum of PL bf16
// arrays `plane` elements apart, array q holding what the arrays before it left of the fp32 value after rounding).
template <typename XT, int PL>
__device__ __forceinline__ void ns_store16(XT* p, size_t plane, const float* in) {
  if constexpr (PL == 1) {
    store16<XT>(p, in);
  } else {
    float rest[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) rest[i] = in[i];
#pragma unroll
    for (int q = 0; q < PL; ++q) {
      store16<XT>(p + q * plane, rest);
      if (q + 1 < PL) {
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const unsigned w = pack2(rest[i], rest[i + 1]);
          rest[i] -= __uint_as_float(w << 16);              // exact: the rounding error of an fp32 value is an fp32 value
          rest[i + 1] -= __uint_as_float(w & 0xffff0000u);
        }
      }
    }
  }
}
template <typename XT, int PL>
__device__ __forceinline__ void ns_load16(const XT* p, size_t plane, float* out) {
  load16<XT>(p + (PL - 1) * plane, out);
  if constexpr (PL > 1) {
#pragma unroll
    for (int q = PL - 2; q >= 0; --q) {        // smallest plane first
      float v[16];
      load16<XT>(p + q * plane, v);
#pragma unroll
      for (int i = 0; i < 16; ++i) out[i] += v[i];
    }
  }
}
template <typename XT, int PL>
__device__ __forceinline__ float ns_load1(const XT* p, size_t plane) {
  float v = load1<XT>(p + (PL - 1) * plane);
  if constexpr (PL > 1) {
#pragma unroll
    for (int q = PL - 2; q >= 0; --q) v += load1<XT>(p + q * plane);
  }
  return v;
}

// ------------------------------------------------------------------------------------------------------
// a1 + a2 (first stage) + a3.  Thread t of a block owns row t/4 and 16 consecutive columns of a 64x64 tile
// in U's orientation.  GT: gradient element type; XT: Newton-Schulz element type.
// Writes: M (guarded), the tile of U into the buffer of the same orientation, the transposed tile (through
// LDS) into the buffer of the other orientation, both zero-filled outside A x B, and one partial sum of U^2.
// ------------------------------------------------------------------------------------------------------
template <typename GT, typename XT, int PL>
__device__ __forceinline__ void momentum_tile(const MatDesc& d, const MatPtrs& pt, int tr, int tc, float mu, int nesterov,
                                              bool both, float (*lds)[kEwTile + 1], float* red) {
  const int tid = threadIdx.x;
  const int r = tr * kEwTile + (tid >> 2);
  const int c0 = tc * kEwTile + (tid & 3) * 16;
  const int A = d.rows, B = d.cols;
  const GT* g = static_cast<const GT*>(pt.g);
  float* m = pt.m;

  float u[16];
  float ss = 0.f;
  const bool row_ok = r < A;
  const size_t base = (size_t)r * (size_t)B + (size_t)c0;
  const bool fast = row_ok && (c0 + 16 <= B) && ((B & 7) == 0) && aligned16(m) && aligned16(g);
  if (fast) {
    float mv[16], gv[16];
    load16<float>(m + base, mv);
    load16<GT>(g + base, gv);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float mn = fmaf(mu, mv[i], gv[i]);
      mv[i] = mn;
      u[i] = nesterov ? fmaf(mu, mn, gv[i]) : mn;
      ss = fmaf(u[i], u[i], ss);
    }
    store16<float>(m + base, mv);
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float ui = 0.f;
      if (row_ok && c0 + i < B) {
        const float gi = load1<GT>(g + base + i);
        const float mn = fmaf(mu, m[base + i], gi);
        m[base + i] = mn;
        ui = nesterov ? fmaf(mu, mn, gi) : mn;
      }
      u[i] = ui;
      ss = fmaf(ui, ui, ss);
    }
  }

  // Orientation: the buffer whose rows run along U's rows, and the one holding U^T.
  // not transposed: X = U (pitch np), Xt = U^T (pitch mp).  transposed: Xt = U (pitch mp), X = U^T (pitch np).
  XT* same = static_cast<XT*>(d.transposed ? d.Xt[0] : d.X);
  XT* flip = static_cast<XT*>(d.transposed ? d.X : d.Xt[0]);
  const int pitch_same = d.transposed ? d.mp : d.np;
  const int pitch_flip = d.transposed ? d.np : d.mp;

  const bool write_same = both || !d.transposed, write_flip = both || d.transposed;
  if (write_same) ns_store16<XT, PL>(same + (size_t)r * pitch_same + c0, (size_t)d.x_plane, u);

  // the transposed tile goes through LDS; skipped (block-uniformly) where only the untransposed layout is wanted
  const int lr_ = tid >> 2, lc0 = (tid & 3) * 16;
  if (write_flip) {
#pragma unroll
    for (int i = 0; i < 16; ++i) lds[lc0 + i][lr_] = u[i];
  }
  const float total = block_sum_256(ss, red);   // contains the barrier that publishes the LDS tile
  if (write_flip) {
    float t[16];
    const int fc = tid >> 2, fr0 = (tid & 3) * 16;   // row of U^T (= column of U), 16 consecutive columns of U^T
#pragma unroll
    for (int i = 0; i < 16; ++i) t[i] = lds[fc][fr0 + i];
    ns_store16<XT, PL>(flip + (size_t)(tc * kEwTile + fc) * pitch_flip + tr * kEwTile + fr0, (size_t)d.x_plane, t);
  }

  if (tid == 0) d.partials[tr * d.ew_tiles_c + tc] = total;
}

template <typename XT, int PL>
__global__ __launch_bounds__(256) void momentum_norm_cast_kernel(const MatDesc* __restrict__ mats,
                                                                  const MatPtrs* __restrict__ ptrs,
                                                                  const EwTile* __restrict__ tiles, float mu,
                                                                  int nesterov, int both) {
  __shared__ float lds[kEwTile][kEwTile + 1];
  __shared__ float red[4];
  const EwTile t = tiles[blockIdx.x];
  const MatDesc d = mats[t.mat];
  const MatPtrs pt = ptrs[t.mat];
  for (int k = 0; k < t.count; ++k) {
    if (k) __syncthreads();     // the LDS tile and the reduction scratch are reused
    if (d.g_dtype == kDtypeBF16)
      momentum_tile<u16, XT, PL>(d, pt, t.tr, t.tc + k, mu, nesterov, both != 0, lds, red);
    else
      momentum_tile<float, XT, PL>(d, pt, t.tr, t.tc + k, mu, nesterov, both != 0, lds, red);
  }
}

// ------------------------------------------------------------------------------------------------------
// a2 second stage: one block per matrix sums its partials in a fixed order, in double.
// ------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void norm_finalize_kernel(const MatDesc* __restrict__ mats, int first_mat, double eps) {
  __shared__ double red[256];
  const MatDesc d = mats[first_mat + blockIdx.x];
  double acc = 0.0;
  for (int i = threadIdx.x; i < d.n_part; i += 256) acc += (double)d.partials[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double inv = 1.0 / (sqrt(red[0]) + eps);
    // an all-zero U with eps = 0 would give inf; X is all zero then, and 0 * inf must not appear
    const float s = (red[0] > 0.0 || eps > 0.0) ? (float)inv : 0.f;
    d.scal[0] = s;
    d.scal[1] = (red[0] > 0.0 || eps > 0.0) ? (float)(inv * inv) : 0.f;
  }
}

// ------------------------------------------------------------------------------------------------------
// a8: W <- W - lr * (rms_scale*sqrt(max(A,B)) * O + wd * W), fp32 math, one rounding to W's dtype.
// ------------------------------------------------------------------------------------------------------
// Where O (in W's orientation) lives after the Newton-Schulz phase.  o_sel bit 0: which of Xt[0..1] for matrices
// iterated on their transpose; bit 1: X (0) or Xt[0] used as the second m_pad x n_pad buffer (1) for the others.
// The record is read in place, never copied into a local: with a local copy the compiler turned the selections below
// into loads from a selected address of that copy, which put the whole 128-byte record into per-thread scratch memory
// - 8 bytes of scratch traffic per matrix element; the HBM-side write counter of the update kernel read twice the
// bytes of W because of it.
__device__ __forceinline__ const void* o_source(const MatDesc& d, int o_sel) {
  if (d.transposed) return (o_sel & 1) ? d.Xt[1] : d.Xt[0];
  return (o_sel & 2) ? d.Xt[0] : d.X;
}

// 8 consecutive elements: one 16-byte access for bf16, two for fp32
template <typename T>
__device__ __forceinline__ void load8(const T* p, float* out);
template <>
__device__ __forceinline__ void load8<float>(const float* p, float* out) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float4 v = reinterpret_cast<const float4*>(p)[i];
    out[4 * i + 0] = v.x; out[4 * i + 1] = v.y; out[4 * i + 2] = v.z; out[4 * i + 3] = v.w;
  }
}
template <>
__device__ __forceinline__ void load8<u16>(const u16* p, float* out) {
  // streaming hint: every element of the update is touched once; without it the L2 refetched a third of the lines
  // (measured: 1.20 GB fetched for 0.81 GB of W and O on the 4096-wide block, 0.89 GB with the hint)
  const u32x4_t vv = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  const uint4 v = make_uint4(vv.x, vv.y, vv.z, vv.w);
  const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    out[2 * j] = __uint_as_float(w[j] << 16);
    out[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
  }
}
template <typename T>
__device__ __forceinline__ void store8(T* p, const float* in);
template <>
__device__ __forceinline__ void store8<float>(float* p, const float* in) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
    reinterpret_cast<float4*>(p)[i] = make_float4(in[4 * i], in[4 * i + 1], in[4 * i + 2], in[4 * i + 3]);
}
template <>
__device__ __forceinline__ void store8<u16>(u16* p, const float* in) {
  const u32x4_t vv = {pack2(in[0], in[1]), pack2(in[2], in[3]), pack2(in[4], in[5]), pack2(in[6], in[7])};
  __builtin_nontemporal_store(vv, reinterpret_cast<u32x4_t*>(p));
}
template <typename XT, int PL>
__device__ __forceinline__ void ns_load8(const XT* p, size_t plane, float* out) {
  load8<XT>(p + (PL - 1) * plane, out);
  if constexpr (PL > 1) {
#pragma unroll
    for (int q = PL - 2; q >= 0; --q) {        // smallest plane first
      float v[8];
      load8<XT>(p + q * plane, v);
#pragma unroll
      for (int i = 0; i < 8; ++i) out[i] += v[i];
    }
  }
}

// One 64x64 tile of the update.  Thread t owns 8 consecutive columns, (t % 8) * 8 .., of rows t / 8 and t / 8 + 32:
// the 8 lanes that share a row cover one whole 128-byte line of a bf16 array with every load or store instruction
// (a thread that owned 16 consecutive elements wrote every line in two instructions of scattered 16-byte pieces).
template <typename WT, typename XT, int PL, bool UPDATE>
__device__ __forceinline__ void apply_tile(const MatDesc& d, const MatPtrs& pt, int tr, int tc, float lr, float wd,
                                           float scale, int o_sel, float* red) {
  const int tid = threadIdx.x;
  const int c0 = tc * kEwTile + (tid & 7) * 8;
  const int A = d.rows, B = d.cols;
  WT* w = static_cast<WT*>(pt.w);
  const XT* o = static_cast<const XT*>(o_source(d, o_sel));
  const int pitch = d.transposed ? d.mp : d.np;
  const size_t plane = (size_t)d.x_plane;
  const int r0 = tr * kEwTile + (tid >> 3), r1 = r0 + 32;
  float ss = 0.f;
  const bool wide = (c0 + 8 <= B) && ((B & 7) == 0) && (!UPDATE || aligned16(w));
  if (wide && r1 < A) {
    // both rows at once: all loads are issued before the first store
    float ov[2][8], wv[2][8];
    ns_load8<XT, PL>(o + (size_t)r0 * pitch + c0, plane, ov[0]);
    ns_load8<XT, PL>(o + (size_t)r1 * pitch + c0, plane, ov[1]);
    if (UPDATE) {
      load8<WT>(w + (size_t)r0 * (size_t)B + c0, wv[0]);
      load8<WT>(w + (size_t)r1 * (size_t)B + c0, wv[1]);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        ss = fmaf(ov[u][i], ov[u][i], ss);
        if (UPDATE) {
          const float t = fmaf(wd, wv[u][i], scale * ov[u][i]);
          wv[u][i] = fmaf(-lr, t, wv[u][i]);
        }
      }
    if (UPDATE) {
      store8<WT>(w + (size_t)r0 * (size_t)B + c0, wv[0]);
      store8<WT>(w + (size_t)r1 * (size_t)B + c0, wv[1]);
    }
  } else {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int r = u ? r1 : r0;
      if (r >= A || c0 >= B) continue;
      const size_t base = (size_t)r * (size_t)B + (size_t)c0;
      const XT* op = o + (size_t)r * pitch + c0;
      if (wide) {
        float ov[8], wv[8];
        ns_load8<XT, PL>(op, plane, ov);
        if (UPDATE) load8<WT>(w + base, wv);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          ss = fmaf(ov[i], ov[i], ss);
          if (UPDATE) {
            const float t = fmaf(wd, wv[i], scale * ov[i]);
            wv[i] = fmaf(-lr, t, wv[i]);
          }
        }
        if (UPDATE) store8<WT>(w + base, wv);
      } else {
        for (int i = 0; i < 8 && c0 + i < B; ++i) {
          const float ov = ns_load1<XT, PL>(op + i, plane);
          ss = fmaf(ov, ov, ss);
          if (UPDATE) {
            const float wv = load1<WT>(w + base + i);
            const float t = fmaf(wd, wv, scale * ov);
            store1<WT>(w + base + i, fmaf(-lr, t, wv));
          }
        }
      }
    }
  }
  const float total = block_sum_256(ss, red);
  if (tid == 0) d.partials[tr * d.ew_tiles_c + tc] = total;
}

template <typename XT, int PL>
__global__ __launch_bounds__(256) void apply_update_kernel(const MatDesc* __restrict__ mats, const MatPtrs* __restrict__ ptrs,
                                                            const EwTile* __restrict__ tiles, float lr, float wd,
                                                            float rms_scale, int scale_mode, float sqrt_hidden, int o_sel,
                                                            int use_s) {
  __shared__ float red[4];
  const EwTile t = tiles[blockIdx.x];
  const MatDesc& d = mats[t.mat];     // read in place (uniform address: scalar loads); see o_source
  const MatPtrs pt = ptrs[t.mat];
  // factor that multiplies the stored O: the three variants of section 3.1 (Eq. 5-7)
  float scale;
  if (scale_mode == 2) {
    scale = rms_scale * d.scal[2];              // 1/RMS of the stored O: any common factor of O cancels
  } else {
    scale = rms_scale * (scale_mode == 1 ? sqrt_hidden : d.sqrt_max);
    if (use_s) scale *= d.scal[0];
  }
  for (int k = 0; k < t.count; ++k) {
    if (k) __syncthreads();     // the reduction scratch is reused
    if (d.w_dtype == kDtypeBF16)
      apply_tile<u16, XT, PL, true>(d, pt, t.tr, t.tc + k, lr, wd, scale, o_sel, red);
    else
      apply_tile<float, XT, PL, true>(d, pt, t.tr, t.tc + k, lr, wd, scale, o_sel, red);
  }
}

// Per-tile sums of O^2 only (first pass of the "Update Norm" variant, Eq. 6).
template <typename XT, int PL>
__global__ __launch_bounds__(256) void update_sumsq_kernel(const MatDesc* __restrict__ mats, const EwTile* __restrict__ tiles,
                                                            int o_sel) {
  __shared__ float red[4];
  const EwTile t = tiles[blockIdx.x];
  const MatDesc& d = mats[t.mat];     // read in place (uniform address: scalar loads); see o_source
  const MatPtrs none{nullptr, nullptr, nullptr};
  for (int k = 0; k < t.count; ++k) {
    if (k) __syncthreads();
    apply_tile<float, XT, PL, false>(d, none, t.tr, t.tc + k, 0.f, 0.f, 0.f, o_sel, red);
  }
}

// sqrt(mean(O^2)) per matrix from the per-tile sums left by apply_update_kernel.
__global__ __launch_bounds__(256) void update_rms_kernel(const MatDesc* __restrict__ mats, int first_mat, int use_s,
                                                          int to_scal, float* __restrict__ out) {
  __shared__ double red[256];
  const MatDesc d = mats[first_mat + blockIdx.x];
  double acc = 0.0;
  for (int i = threadIdx.x; i < d.n_part; i += 256) acc += (double)d.partials[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    double rms = sqrt(red[0] / ((double)d.rows * (double)d.cols));
    if (to_scal) {
      d.scal[2] = rms > 0.0 ? (float)(1.0 / rms) : 0.f;
    } else {
      if (use_s) rms *= (double)d.scal[0];
      out[first_mat + blockIdx.x] = (float)rms;
    }
  }
}

template <typename XT, int PL, typename DT>
__global__ __launch_bounds__(256) void read_update_kernel(const MatDesc* __restrict__ mats, int mat, int o_sel, int use_s,
                                                           DT* __restrict__ dst) {
  const MatDesc& d = mats[mat];
  const XT* o = static_cast<const XT*>(o_source(d, o_sel));
  const int pitch = d.transposed ? d.mp : d.np;
  const float s = use_s ? d.scal[0] : 1.f;
  const size_t total = (size_t)d.rows * (size_t)d.cols;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t r = i / (size_t)d.cols, c = i % (size_t)d.cols;
    store1<DT>(dst + i, s * ns_load1<XT, PL>(o + r * pitch + c, (size_t)d.x_plane));
  }
}

}  // namespace

// ns_dtype -> (element type, planes): fp32; bf16; bf16 x 2 planes; bf16 x 3 planes
#define MUON_NS_DISPATCH(ns_dtype, CALL)                 \
  switch (ns_dtype) {                                    \
    case kDtypeF32: { CALL(float, 1); break; }           \
    case kDtypeBF16: { CALL(u16, 1); break; }            \
    case kDtypeBF16X2: { CALL(u16, 2); break; }          \
    case kDtypeBF16X3: { CALL(u16, 3); break; }          \
    default: return hipErrorInvalidValue;                \
  }

hipError_t launch_momentum_norm_cast(const MatDesc* mats, const MatPtrs* ptrs, const EwTile* tiles, int n_tiles, float mu,
                                     int nesterov, int both_layouts, int ns_dtype, hipStream_t s) {
  if (n_tiles <= 0) return hipSuccess;
#define MUON_CALL(XT, PL) momentum_norm_cast_kernel<XT, PL><<<n_tiles, 256, 0, s>>>(mats, ptrs, tiles, mu, nesterov, both_layouts)
  MUON_NS_DISPATCH(ns_dtype, MUON_CALL)
#undef MUON_CALL
  return hipGetLastError();
}

hipError_t launch_norm_finalize(const MatDesc* mats, int first_mat, int n_mats, double eps, hipStream_t s) {
  if (n_mats <= 0) return hipSuccess;
  norm_finalize_kernel<<<n_mats, 256, 0, s>>>(mats, first_mat, eps);
  return hipGetLastError();
}

hipError_t launch_apply_update(const MatDesc* mats, const MatPtrs* ptrs, const EwTile* tiles, int n_tiles, float lr, float wd,
                               float rms_scale, int scale_mode, float sqrt_hidden, int o_sel, int use_s, int ns_dtype,
                               hipStream_t s) {
  if (n_tiles <= 0) return hipSuccess;
#define MUON_CALL(XT, PL) \
  apply_update_kernel<XT, PL><<<n_tiles, 256, 0, s>>>(mats, ptrs, tiles, lr, wd, rms_scale, scale_mode, sqrt_hidden, o_sel, use_s)
  MUON_NS_DISPATCH(ns_dtype, MUON_CALL)
#undef MUON_CALL
  return hipGetLastError();
}

hipError_t launch_update_sumsq(const MatDesc* mats, const EwTile* tiles, int n_tiles, int o_sel, int ns_dtype, hipStream_t s) {
  if (n_tiles <= 0) return hipSuccess;
#define MUON_CALL(XT, PL) update_sumsq_kernel<XT, PL><<<n_tiles, 256, 0, s>>>(mats, tiles, o_sel)
  MUON_NS_DISPATCH(ns_dtype, MUON_CALL)
#undef MUON_CALL
  return hipGetLastError();
}

hipError_t launch_update_rms(const MatDesc* mats, int first_mat, int n_mats, int use_s, int to_scal, float* out, hipStream_t s) {
  if (n_mats <= 0) return hipSuccess;
  update_rms_kernel<<<n_mats, 256, 0, s>>>(mats, first_mat, use_s, to_scal, out);
  return hipGetLastError();
}

hipError_t launch_read_update(const MatDesc* mats, int mat, int o_sel, int use_s, int ns_dtype, void* dst, int dst_dtype,
                              hipStream_t s) {
  const int grid = 1024;
  if (dst_dtype == kDtypeBF16) {
#define MUON_CALL(XT, PL) read_update_kernel<XT, PL, u16><<<grid, 256, 0, s>>>(mats, mat, o_sel, use_s, static_cast<u16*>(dst))
    MUON_NS_DISPATCH(ns_dtype, MUON_CALL)
#undef MUON_CALL
  } else {
#define MUON_CALL(XT, PL) read_update_kernel<XT, PL, float><<<grid, 256, 0, s>>>(mats, mat, o_sel, use_s, static_cast<float*>(dst))
    MUON_NS_DISPATCH(ns_dtype, MUON_CALL)
#undef MUON_CALL
  }
  return hipGetLastError();
}

}  // namespace muon
