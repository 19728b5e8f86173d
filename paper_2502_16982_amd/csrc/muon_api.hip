// C ABI and host-side planner of the MI355X Muon step (see include/muon.h for the contract).
//
// muon_init turns a list of matrix shapes into: the orientation and padded extents of every matrix, the
// chunking of the list against the workspace, and device tables (matrix records, elementwise tiles, one
// grouped-GEMM problem table and tile table per Newton-Schulz product).  muon_step only enqueues kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/muon.h"
#include "muon_launch.h"
#include "muon_plan.h"

using namespace muon;

namespace {

thread_local int g_last_hip_error = 0;

inline int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return MUON_E_HIP;
}
#define MUON_HIP(expr)                          \
  do {                                          \
    hipError_t e__ = (expr);                    \
    if (e__ != hipSuccess) return hip_fail(e__); \
  } while (0)

// Every entry point runs its body through this: nothing may unwind through the C ABI.
template <typename F>
int guarded(F&& body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return MUON_E_NO_MEMORY;
  } catch (...) {
    return MUON_E_INVALID_ARG;
  }
}

// Scratch of muon_step_static, the entry point for callers that cannot allocate device memory: the tables and
// Newton-Schulz temporaries that muon_step keeps in the caller's workspace live in this array instead.  Every device
// the library runs on holds its own copy, at its own address, until the process ends.  In host code the name is only
// a handle for hipGetSymbolAddress; the device address it yields (StaticSlot::ptr) is what kernels and copies get.
constexpr size_t kStaticScratchBytes = MUON_STATIC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

}  // namespace

struct muon_ctx {
  int n = 0;
  int ns_dtype = MUON_BF16;
  int device = 0;
  Plan plan;             // orientation, padding, chunking, host image of the device tables
  unsigned char* ws = nullptr;
  size_t ws_bytes = 0;
  // device tables
  MatDesc* d_mats = nullptr;
  MatPtrs* d_ptrs = nullptr;
  // dynamic pointer upload
  MatPtrs* h_ptrs_pinned = nullptr;
  std::vector<MatPtrs> last_ptrs;
  bool ptrs_valid = false;
  hipEvent_t upload_done = nullptr;
  // host-only plan (muon_plan_only): no device tables exist
  bool plan_only = false;
  // state of the last step, for the debug read
  int last_o_sel = 0, last_use_s = 0, last_chunk = -1;
  // optional per-launch event timing
  bool profiling = false;
  std::vector<hipEvent_t> prof_events;   // pairs: start, stop
  std::vector<int> prof_pending;         // kernel class of each pending pair
  double prof_ms[MUON_PROF_COUNT] = {};
  int64_t prof_launches[MUON_PROF_COUNT] = {};
};

namespace {

constexpr size_t kProfPairs = 2048;

int prof_drain(muon_ctx* ctx) {
  for (size_t i = 0; i < ctx->prof_pending.size(); ++i) {
    float ms = 0.f;
    MUON_HIP(hipEventSynchronize(ctx->prof_events[2 * i + 1]));
    MUON_HIP(hipEventElapsedTime(&ms, ctx->prof_events[2 * i], ctx->prof_events[2 * i + 1]));
    ctx->prof_ms[ctx->prof_pending[i]] += (double)ms;
    ctx->prof_launches[ctx->prof_pending[i]] += 1;
  }
  ctx->prof_pending.clear();
  return MUON_OK;
}

// Brackets one launch with events when profiling is on.
template <typename F>
int timed(muon_ctx* ctx, int cls, hipStream_t s, F&& launch) {
  if (!ctx->profiling) {
    MUON_HIP(launch());
    return MUON_OK;
  }
  if (ctx->prof_pending.size() >= kProfPairs) {
    int st = prof_drain(ctx);
    if (st != MUON_OK) return st;
  }
  const size_t k = ctx->prof_pending.size();
  MUON_HIP(hipEventRecord(ctx->prof_events[2 * k], s));
  MUON_HIP(launch());
  MUON_HIP(hipEventRecord(ctx->prof_events[2 * k + 1], s));
  ctx->prof_pending.push_back(cls);
  return MUON_OK;
}
#define MUON_TIMED(cls, call)                                   \
  do {                                                          \
    int st__ = timed(ctx, cls, s, [&]() { return (call); });    \
    if (st__ != MUON_OK) return st__;                           \
  } while (0)

}  // namespace

extern "C" {

int muon_default_hparams(muon_hparams* hp) {
  if (!hp) return MUON_E_INVALID_ARG;
  hp->lr = 0.0;
  hp->weight_decay = 0.0;
  hp->momentum = 0.95;
  hp->a = 3.4445;
  hp->b = -4.7750;
  hp->c = 2.0315;
  hp->rms_scale = 0.2;
  hp->eps = 1e-7;
  hp->ns_steps = 5;
  hp->nesterov = 1;
  hp->scale_mode = MUON_SCALE_ADJUSTED_LR;
  hp->reserved = 0;
  hp->hidden_size = 0.0;
  hp->coeff_schedule = nullptr;
  return MUON_OK;
}

int muon_workspace_bytes(const muon_param* shapes, int32_t n, int32_t ns_dtype, size_t max_bytes, size_t* out) {
  return guarded([&]() { return plan_workspace_bytes(shapes, n, ns_dtype, max_bytes, out); });
}

}  // extern "C"

namespace {

// Validates the arguments of a step against the plan.  *changed: the pointer list differs from the uploaded one.
int check_step_args(const muon_ctx* ctx, const muon_param* params, int32_t n, const muon_hparams* hp, bool* changed) {
  if (!ctx || !params || !hp || ctx->plan_only) return MUON_E_INVALID_ARG;
  if (n != ctx->n) return MUON_E_SHAPE_MISMATCH;
  if (hp->ns_steps < 0 || !(hp->eps >= 0.0) || !std::isfinite(hp->lr) || !std::isfinite(hp->weight_decay) ||
      !std::isfinite(hp->momentum) || !std::isfinite(hp->a) || !std::isfinite(hp->b) || !std::isfinite(hp->c) ||
      !std::isfinite(hp->rms_scale) || hp->scale_mode < MUON_SCALE_ADJUSTED_LR || hp->scale_mode > MUON_SCALE_UPDATE_NORM ||
      hp->reserved != 0 || (hp->scale_mode == MUON_SCALE_BASELINE && !(hp->hidden_size > 0.0 && std::isfinite(hp->hidden_size))))
    return MUON_E_INVALID_ARG;
  if (hp->coeff_schedule)
    for (int i = 0; i < 3 * hp->ns_steps; ++i)
      if (!std::isfinite(hp->coeff_schedule[i])) return MUON_E_INVALID_ARG;
  *changed = !ctx->ptrs_valid;
  for (int i = 0; i < n; ++i) {
    const muon_param& p = params[i];
    const MatPlan& q = ctx->plan.mats[i];
    if (p.rows != q.rows || p.cols != q.cols || p.w_dtype != q.w_dtype || p.g_dtype != q.g_dtype) return MUON_E_SHAPE_MISMATCH;
    if (!p.w || !p.g || !p.m) return MUON_E_INVALID_ARG;
    const uintptr_t wa = p.w_dtype == MUON_BF16 ? 1u : 3u, ga = p.g_dtype == MUON_BF16 ? 1u : 3u;
    if ((reinterpret_cast<uintptr_t>(p.w) & wa) || (reinterpret_cast<uintptr_t>(p.g) & ga) || (reinterpret_cast<uintptr_t>(p.m) & 3u))
      return MUON_E_MISALIGNED;
    const MatPtrs& l = ctx->last_ptrs[i];
    if (l.w != p.w || l.g != p.g || l.m != p.m) *changed = true;
  }
  return MUON_OK;
}

// Enqueues every kernel of one step on stream s (the pointer table is already on its way on the same stream).
int enqueue_step(muon_ctx* ctx, const muon_hparams* hp, hipStream_t s, float* update_rms_out) {
  const int N = hp->ns_steps;
  const int use_s = N == 0;
  const bool mc = on_matrix_cores(ctx->ns_dtype);   // bf16 or split-bf16: the MFMA kernels and their one-layout plan
  const int planes = planes_of(ctx->ns_dtype);
  // where O ends up (see o_source in the elementwise kernels): fp32 path: X in place, its transpose in Xt[N & 1];
  // bf16 path: X ping-pong index N & 1 (bit 1), transposed matrices in Xt[1], or Xt[0] when no iteration ran (bit 0)
  const int o_sel = mc ? ((N & 1) << 1) | (N > 0 ? 1 : 0) : (N & 1);

  for (size_t ci = 0; ci < ctx->plan.chunks.size(); ++ci) {
    const Chunk& ch = ctx->plan.chunks[ci];
    const EwTile* ew = reinterpret_cast<const EwTile*>(ctx->ws + ch.ew_tiles_off);
    MUON_TIMED(MUON_PROF_MOMENTUM, launch_momentum_norm_cast(ctx->d_mats, ctx->d_ptrs, ew, ch.n_ew_tiles, (float)hp->momentum,
                                                             hp->nesterov != 0, (!mc || N == 0) ? 1 : 0, ctx->ns_dtype, s));
    MUON_TIMED(MUON_PROF_NORM, launch_norm_finalize(ctx->d_mats, ch.first, ch.count, hp->eps, s));
    for (int it = 0; it < N; ++it) {
      const int first = it == 0, last = it == N - 1, par = it & 1;
      const double* sch = hp->coeff_schedule ? hp->coeff_schedule + 3 * it : nullptr;
      const float a = (float)(sch ? sch[0] : hp->a), b = (float)(sch ? sch[1] : hp->b), c = (float)(sch ? sch[2] : hp->c);
      for (const Group& g : ch.groups) {
        auto P = [&](size_t o) { return reinterpret_cast<const GemmProblem*>(ctx->ws + o); };
        auto T = [&](size_t o) { return reinterpret_cast<const GemmTile*>(ctx->ws + o); };
        // one launch per product and level (the coarse tiles first, then what they leave)
        for (int level = 1; level >= 0; --level) {
          const TileSet& ts = level ? g.coarse : g.fine;
          if (ts.n_sym == 0) continue;
          if (mc)
            MUON_TIMED(MUON_PROF_GRAM, launch_gemm_bf16(level, (ts.strips ? kGemmStrips : 0) | (ts.persistent_n ? kGemmPersistent : 0), P(g.prob_gram[par]), T(ts.sym), ts.n_sym, 1.f, 0.f,
                                                        first ? 1 : -1, 0.f, 0, planes, s));
          else
            MUON_TIMED(MUON_PROF_GRAM, launch_gemm_f32(P(g.prob_gram[par]), T(ts.sym), ts.n_sym, 1.f, 0.f, first ? 1 : -1, s));
        }
        for (int level = 1; level >= 0; --level) {
          const TileSet& ts = level ? g.coarse : g.fine;
          if (ts.n_sym == 0) continue;
          if (mc)
            MUON_TIMED(MUON_PROF_POLY, launch_gemm_bf16(level, (ts.strips ? kGemmStrips : 0) | (ts.persistent_m ? kGemmPersistent : 0), P(g.prob_poly), T(ts.poly), ts.n_poly, c, b, -1, a, 0, planes, s));
          else
            MUON_TIMED(MUON_PROF_POLY, launch_gemm_f32(P(g.prob_poly), T(ts.poly), ts.n_poly, c, b, -1, s));
        }
        for (int level = 1; level >= 0; --level) {
          const TileSet& ts = level ? g.coarse : g.fine;
          const size_t t_app = last ? ts.apply_last : ts.apply;
          const int n_app = last ? ts.n_apply_last : ts.n_apply;
          if (n_app == 0) continue;
          if (mc)
            MUON_TIMED(MUON_PROF_APPLY_POLY, launch_gemm_bf16(level, (ts.strips ? kGemmStrips : 0) | (ts.persistent_m ? kGemmPersistent : 0), P(g.prob_apply[par * 2 + last]), T(t_app),
                                                              n_app, 1.f, a, first ? 0 : -1, 0.f, 1, planes, s));
          else
            MUON_TIMED(MUON_PROF_APPLY_POLY, launch_gemm_f32(P(g.prob_apply[par * 2 + last]), T(t_app), n_app, 1.f, a,
                                                             first ? 0 : -1, s));
        }
      }
    }
    if (hp->scale_mode == MUON_SCALE_UPDATE_NORM) {
      // Eq. 6 needs RMS(O) before the update: one extra pass over O
      MUON_TIMED(MUON_PROF_RMS, launch_update_sumsq(ctx->d_mats, ew, ch.n_ew_tiles, o_sel, ctx->ns_dtype, s));
      MUON_TIMED(MUON_PROF_RMS, launch_update_rms(ctx->d_mats, ch.first, ch.count, use_s, 1, nullptr, s));
    }
    MUON_TIMED(MUON_PROF_UPDATE, launch_apply_update(ctx->d_mats, ctx->d_ptrs, ew, ch.n_ew_tiles, (float)hp->lr,
                                                     (float)hp->weight_decay, (float)hp->rms_scale, hp->scale_mode,
                                                     (float)std::sqrt(hp->hidden_size > 0.0 ? hp->hidden_size : 0.0), o_sel, use_s,
                                                     ctx->ns_dtype, s));
    if (update_rms_out) MUON_TIMED(MUON_PROF_RMS, launch_update_rms(ctx->d_mats, ch.first, ch.count, use_s, 0, update_rms_out, s));
  }
  ctx->last_o_sel = o_sel;
  ctx->last_use_s = use_s;
  ctx->last_chunk = (int)ctx->plan.chunks.size() - 1;
  return MUON_OK;
}

int step_impl(muon_ctx* ctx, const muon_param* params, int32_t n, const muon_hparams* hp, void* hip_stream,
              float* update_rms_out) {
  bool changed = false;
  const int st = check_step_args(ctx, params, n, hp, &changed);
  if (st != MUON_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (changed) {
    // the previous upload may still be reading the pinned staging buffer
    if (ctx->ptrs_valid) MUON_HIP(hipEventSynchronize(ctx->upload_done));
    // until the new table is known to be on its way, the device table counts as unknown: a failure below must not
    // leave a later step believing that its (identical) pointers are already uploaded
    ctx->ptrs_valid = false;
    for (int i = 0; i < n; ++i) ctx->h_ptrs_pinned[i] = MatPtrs{params[i].w, params[i].g, params[i].m};
    MUON_HIP(hipMemcpyAsync(ctx->d_ptrs, ctx->h_ptrs_pinned, sizeof(MatPtrs) * (size_t)n, hipMemcpyHostToDevice, s));
    MUON_HIP(hipEventRecord(ctx->upload_done, s));
    for (int i = 0; i < n; ++i) ctx->last_ptrs[i] = ctx->h_ptrs_pinned[i];
    ctx->ptrs_valid = true;
  }
  return enqueue_step(ctx, hp, s, update_rms_out);
}

}  // namespace

namespace {

// Everything muon_init does: the plan (host only) and, with `upload`, the transfer of its table image to the
// workspace and the per-context HIP objects.
int build_context(muon_ctx** out, const muon_param* shapes, int32_t n, int32_t ns_dtype, void* workspace,
                  size_t workspace_bytes, bool upload) {
  if (!out) return MUON_E_INVALID_ARG;
  *out = nullptr;
  int st = validate_shapes(shapes, n, ns_dtype);
  if (st != MUON_OK) return st;
  if (!workspace) return MUON_E_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MUON_E_MISALIGNED;
  muon_ctx* ctx = new muon_ctx();
  struct Guard {     // releases the half-built context on every early return and on exceptions
    muon_ctx* c;
    ~Guard() { if (c) muon_destroy(c); }
  } guard{ctx};
  ctx->n = n;
  ctx->ns_dtype = ns_dtype;
  ctx->ws = static_cast<unsigned char*>(workspace);
  ctx->ws_bytes = workspace_bytes;
  {
    size_t least = 0;                // rejected before the device is touched
    st = plan_workspace_bytes(shapes, n, ns_dtype, 1, &least);
    if (st != MUON_OK) return st;
    if (workspace_bytes < least) return MUON_E_WORKSPACE_TOO_SMALL;
  }
  if (upload) {
    // before the plan: it evens out the persistent launches against the device's number of compute units
    hipError_t e = hipGetDevice(&ctx->device);
    if (e == hipSuccess) e = gemm_setup();
    if (e != hipSuccess) return hip_fail(e);
    ctx->plan.coarse_blocks = gemm_coarse_blocks();
  }
  st = plan_build(ctx->plan, shapes, n, ns_dtype, reinterpret_cast<uintptr_t>(workspace), workspace_bytes);
  if (st != MUON_OK) return st;
  ctx->d_mats = reinterpret_cast<MatDesc*>(ctx->ws + ctx->plan.off_mats);
  ctx->d_ptrs = reinterpret_cast<MatPtrs*>(ctx->ws + ctx->plan.off_ptrs);
  if (!upload) {
    ctx->plan_only = true;
  } else {
    hipError_t e = hipMemcpy(ctx->ws, ctx->plan.image.data(), ctx->plan.image.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&ctx->h_ptrs_pinned), sizeof(MatPtrs) * (size_t)n, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->upload_done, hipEventDisableTiming);
    if (e != hipSuccess) return hip_fail(e);
    ctx->last_ptrs.resize(n);
  }
  guard.c = nullptr;
  *out = ctx;
  return MUON_OK;
}

}  // namespace

extern "C" {

int muon_init(muon_ctx** out, const muon_param* shapes, int32_t n, int32_t ns_dtype, void* workspace,
              size_t workspace_bytes) {
  return guarded([&]() { return build_context(out, shapes, n, ns_dtype, workspace, workspace_bytes, true); });
}

int muon_plan_only(muon_ctx** out, const muon_param* shapes, int32_t n, int32_t ns_dtype, size_t workspace_bytes) {
  // table pointers are computed from the workspace address but never followed: any aligned non-null address will do
  return guarded([&]() {
    return build_context(out, shapes, n, ns_dtype, reinterpret_cast<void*>(uintptr_t{1} << 32), workspace_bytes, false);
  });
}

int muon_plan_tiles(const muon_ctx* ctx, int32_t chunk, int32_t product, int32_t level, int32_t* out, int32_t cap_records) {
  if (!ctx || !ctx->plan_only || chunk < 0 || chunk >= (int)ctx->plan.chunks.size() || product < 0 || product > 3 || level < 0 ||
      level > 1 || cap_records < 0 || (cap_records > 0 && !out))
    return MUON_E_INVALID_ARG;
  return guarded([&]() { return (int)std::min<int64_t>(plan_tiles(ctx->plan, chunk, product, level, out, cap_records), INT32_MAX); });
}

int muon_step(muon_ctx* ctx, const muon_param* params, int32_t n, const muon_hparams* hp, void* hip_stream,
              float* update_rms_out) {
  return guarded([&]() { return step_impl(ctx, params, n, hp, hip_stream, update_rms_out); });
}

}  // extern "C"

namespace {

constexpr int kStaticMaxDevices = 64;
struct PtrPack {                     // the per-step pointers of muon_step_static travel as a kernel argument
  MatPtrs p[MUON_STATIC_MAX_MATRICES];
};
struct StaticSlot {
  unsigned char* ptr = nullptr;      // device address of `scratch` on this device (hipGetSymbolAddress)
  muon_ctx* ctx = nullptr;           // plan and tables of the shape list of the last call on this device
  std::vector<muon_param> key;       // that shape list (rows, cols, dtypes)
};
StaticSlot g_static[kStaticMaxDevices];

__global__ void set_ptrs_kernel(PtrPack pack, MatPtrs* __restrict__ dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = pack.p[i];
}

int step_static_impl(const muon_param* params, int32_t n, int32_t ns_dtype, const muon_hparams* hp, void* hip_stream,
                     float* update_rms_out) {
  int st = validate_shapes(params, n, ns_dtype);
  if (st != MUON_OK) return st;
  if (!hp) return MUON_E_INVALID_ARG;
  if (n > MUON_STATIC_MAX_MATRICES) return MUON_E_STATIC_LIMIT;
  size_t need = 0;
  st = plan_workspace_bytes(params, n, ns_dtype, 0, &need);
  if (st != MUON_OK) return st;
  if (need > kStaticScratchBytes) return MUON_E_STATIC_LIMIT;

  int dev = 0;
  MUON_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kStaticMaxDevices) return MUON_E_INVALID_ARG;
  StaticSlot& slot = g_static[dev];
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (!slot.ptr) {                   // first call on this device: where does this device keep the array?
    void* p = nullptr;
    MUON_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return MUON_E_MISALIGNED;
    MUON_HIP(gemm_setup());
    slot.ptr = static_cast<unsigned char*>(p);
  }
  bool same = slot.ctx && slot.ctx->ns_dtype == ns_dtype && (int)slot.key.size() == n;
  for (int i = 0; same && i < n; ++i)
    same = slot.key[i].rows == params[i].rows && slot.key[i].cols == params[i].cols &&
           slot.key[i].w_dtype == params[i].w_dtype && slot.key[i].g_dtype == params[i].g_dtype;
  if (!same) {
    // Another shape list than the last call's: plan again (host memory only) and put the new tables at the head of
    // the scratch.  Earlier work on this stream may still be using the old tables, and the copy reads host memory
    // that must outlive it: wait on both sides of it.  The array keeps whatever the last call left; nothing in it has
    // to start at zero (every temporary is written in full before it is read), only the tables must be the new ones.
    MUON_HIP(hipStreamSynchronize(s));
    if (slot.ctx) {
      muon_destroy(slot.ctx);
      slot.ctx = nullptr;
    }
    muon_ctx* ctx = new muon_ctx();
    struct Guard {
      muon_ctx* c;
      ~Guard() { if (c) muon_destroy(c); }
    } guard{ctx};
    ctx->n = n;
    ctx->ns_dtype = ns_dtype;
    ctx->device = dev;
    ctx->ws = slot.ptr;
    ctx->ws_bytes = kStaticScratchBytes;
    ctx->plan.coarse_blocks = gemm_coarse_blocks();
    st = plan_build(ctx->plan, params, n, ns_dtype, reinterpret_cast<uintptr_t>(slot.ptr), kStaticScratchBytes);
    if (st != MUON_OK) return st;
    if (ctx->plan.chunks.size() != 1) return MUON_E_STATIC_LIMIT;
    ctx->d_mats = reinterpret_cast<MatDesc*>(ctx->ws + ctx->plan.off_mats);
    ctx->d_ptrs = reinterpret_cast<MatPtrs*>(ctx->ws + ctx->plan.off_ptrs);
    ctx->last_ptrs.resize(n);
    MUON_HIP(hipMemcpyAsync(slot.ptr, ctx->plan.image.data(), ctx->plan.image.size(), hipMemcpyHostToDevice, s));
    MUON_HIP(hipStreamSynchronize(s));
    slot.key.assign(params, params + n);
    slot.ctx = ctx;
    guard.c = nullptr;
  }
  muon_ctx* ctx = slot.ctx;
  ctx->ptrs_valid = true;            // check_step_args compares against last_ptrs only to report a change; unused here
  bool changed = false;
  st = check_step_args(ctx, params, n, hp, &changed);
  if (st != MUON_OK) return st;
  PtrPack pack{};
  for (int i = 0; i < n; ++i) pack.p[i] = MatPtrs{params[i].w, params[i].g, params[i].m};
  set_ptrs_kernel<<<1, MUON_STATIC_MAX_MATRICES, 0, s>>>(pack, ctx->d_ptrs, n);
  MUON_HIP(hipGetLastError());
  return enqueue_step(ctx, hp, s, update_rms_out);
}

}  // namespace

extern "C" {

int muon_step_static(const muon_param* params, int32_t n, int32_t ns_dtype, const muon_hparams* hp, void* hip_stream,
                     float* update_rms_out) {
  return guarded([&]() { return step_static_impl(params, n, ns_dtype, hp, hip_stream, update_rms_out); });
}

int muon_debug_read_update(muon_ctx* ctx, int32_t index, void* dst, int32_t dst_dtype, void* hip_stream) {
  if (!ctx || ctx->plan_only || !dst || index < 0 || index >= ctx->n) return MUON_E_INVALID_ARG;
  if (dst_dtype != MUON_F32 && dst_dtype != MUON_BF16) return MUON_E_UNSUPPORTED_DTYPE;
  if (ctx->last_chunk < 0 || ctx->plan.mats[index].chunk != ctx->last_chunk) return MUON_E_NOT_RESIDENT;
  MUON_HIP(launch_read_update(ctx->d_mats, index, ctx->last_o_sel, ctx->last_use_s, ctx->ns_dtype, dst, dst_dtype,
                              static_cast<hipStream_t>(hip_stream)));
  return MUON_OK;
}

int muon_plan_describe(const muon_ctx* ctx, int32_t index, int64_t* out, int32_t cap) {
  if (!ctx || !out || index < 0 || index >= ctx->n || cap < 0) return MUON_E_INVALID_ARG;
  const MatPlan& q = ctx->plan.mats[index];
  const int coarse = on_matrix_cores(ctx->ns_dtype) && q.mp >= kCoarse ? kCoarse : q.tile;
  const int64_t v[8] = {q.m, q.n, q.transposed, q.mp, q.np, q.chunk, coarse, q.tile};
  const int k = std::min<int>(cap, 8);
  for (int i = 0; i < k; ++i) out[i] = v[i];
  return k;
}

int muon_profile_enable(muon_ctx* ctx, int enable) {
  if (!ctx || ctx->plan_only) return MUON_E_INVALID_ARG;
  return guarded([&]() -> int {
  if (enable && ctx->prof_events.empty()) {
    ctx->prof_events.reserve(2 * kProfPairs);
    for (size_t i = 0; i < 2 * kProfPairs; ++i) {
      hipEvent_t ev = nullptr;
      MUON_HIP(hipEventCreate(&ev));
      ctx->prof_events.push_back(ev);
    }
  }
  if (!enable && ctx->profiling) {
    int st = prof_drain(ctx);
    if (st != MUON_OK) return st;
  }
  ctx->profiling = enable != 0;
  return MUON_OK;
  });
}

int muon_profile_read(muon_ctx* ctx, double* ms_out, int64_t* launches_out, int reset) {
  if (!ctx) return MUON_E_INVALID_ARG;
  int st = prof_drain(ctx);
  if (st != MUON_OK) return st;
  for (int i = 0; i < MUON_PROF_COUNT; ++i) {
    if (ms_out) ms_out[i] = ctx->prof_ms[i];
    if (launches_out) launches_out[i] = ctx->prof_launches[i];
    if (reset) {
      ctx->prof_ms[i] = 0.0;
      ctx->prof_launches[i] = 0;
    }
  }
  return MUON_OK;
}

int muon_adamw_step(const muon_adamw_param* params, int32_t n, const muon_adamw_hparams* hp, void* hip_stream) {
  if (!params || !hp || n <= 0) return MUON_E_INVALID_ARG;
  if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0) || !(hp->beta2 >= 0.0 && hp->beta2 < 1.0) || !(hp->eps >= 0.0) || hp->step < 1 ||
      !std::isfinite(hp->lr) || !std::isfinite(hp->weight_decay) || !std::isfinite(hp->eps))
    return MUON_E_INVALID_ARG;
  for (int i = 0; i < n; ++i) {
    const muon_adamw_param& q = params[i];
    if (!q.p || !q.g || !q.m || !q.v || q.numel < 1) return MUON_E_INVALID_ARG;
    if ((q.p_dtype != MUON_F32 && q.p_dtype != MUON_BF16) || (q.g_dtype != MUON_F32 && q.g_dtype != MUON_BF16))
      return MUON_E_UNSUPPORTED_DTYPE;
    const uintptr_t pa = q.p_dtype == MUON_BF16 ? 1u : 3u, ga = q.g_dtype == MUON_BF16 ? 1u : 3u;
    if ((reinterpret_cast<uintptr_t>(q.p) & pa) || (reinterpret_cast<uintptr_t>(q.g) & ga) ||
        (reinterpret_cast<uintptr_t>(q.m) & 3u) || (reinterpret_cast<uintptr_t>(q.v) & 3u))
      return MUON_E_MISALIGNED;
    if (adamw_blocks_for(q.numel) > (1ll << 30)) return MUON_E_INVALID_ARG;
  }
  // bias corrections in double, handed to the kernel as reciprocals
  const float inv_bc1 = (float)(1.0 / (1.0 - std::pow(hp->beta1, (double)hp->step)));
  const float inv_bc2 = (float)(1.0 / (1.0 - std::pow(hp->beta2, (double)hp->step)));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  for (int first = 0; first < n;) {
    AdamwBatch b{};
    long long blocks = 0;
    int k = 0;
    while (first + k < n && k < kAdamwSlots && blocks + adamw_blocks_for(params[first + k].numel) <= (1ll << 30)) {
      const muon_adamw_param& q = params[first + k];
      b.p[k] = q.p; b.g[k] = q.g; b.m[k] = q.m; b.v[k] = q.v;
      b.numel[k] = q.numel;
      b.p_dtype[k] = q.p_dtype; b.g_dtype[k] = q.g_dtype;
      b.block_start[k] = (int)blocks;
      blocks += adamw_blocks_for(q.numel);
      ++k;
    }
    b.block_start[k] = (int)blocks;
    b.n = k;
    MUON_HIP(launch_adamw(b, (int)blocks, (float)hp->lr, (float)hp->weight_decay, (float)hp->beta1, (float)hp->beta2,
                          (float)hp->eps, inv_bc1, inv_bc2, s));
    first += k;
  }
  return MUON_OK;
}

int muon_plan_chunks(const muon_ctx* ctx) { return ctx ? (int)ctx->plan.chunks.size() : MUON_E_INVALID_ARG; }

void muon_destroy(muon_ctx* ctx) {
  if (!ctx) return;
  if (ctx->upload_done) {
    (void)hipEventSynchronize(ctx->upload_done);
    (void)hipEventDestroy(ctx->upload_done);
  }
  if (ctx->h_ptrs_pinned) (void)hipHostFree(ctx->h_ptrs_pinned);
  for (hipEvent_t ev : ctx->prof_events) (void)hipEventDestroy(ev);
  delete ctx;
}

const char* muon_status_string(int status) {
  switch (status) {
    case MUON_OK: return "ok";
    case MUON_E_INVALID_ARG: return "invalid argument";
    case MUON_E_UNSUPPORTED_DTYPE: return "unsupported dtype";
    case MUON_E_SHAPE_MISMATCH: return "parameter list does not match the one given at init";
    case MUON_E_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MUON_E_HIP: return "HIP runtime error";
    case MUON_E_NOT_RESIDENT: return "matrix temporaries are not resident";
    case MUON_E_MISALIGNED: return "misaligned buffer";
    case MUON_E_NO_MEMORY: return "out of host memory";
    case MUON_E_STATIC_LIMIT: return "input exceeds the limits of muon_step_static";
    default: return "unknown status";
  }
}

int muon_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
