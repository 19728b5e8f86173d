/*
 * muon.h - C ABI of the MI355X (gfx950) scaled-Muon optimizer step.
 *
 * One call to muon_step() performs, for every 2-D matrix in a list, the update
 * rule of "Muon is Scalable for LLM Training" (arXiv 2502.16982):
 *
 *   M_t = mu * M_{t-1} + G                                  (section 2.1, the recurrence printed above Eq. 1)
 *   U   = M_t            or   mu * M_t + G  (Nesterov)      (section 2.1, footnote 1)
 *   X_0 = U / (||U||_F + eps), transposed so rows <= cols   (section 2.1, "Newton-Schulz Iterations")
 *   X_k = a X + b (X X^T) X + c (X X^T)^2 X,  k = 1..N      (Eq. 2)
 *   O   = X_N (transposed back)                             (Eq. 1, O_t = Newton-Schulz(M_t))
 *   W_t = W_{t-1} - lr * (rms_scale * sqrt(max(A,B)) * O + weight_decay * W_{t-1})   (Eq. 4, contains Eq. 3)
 *
 * All buffer pointers are DEVICE pointers owned by the caller.  The library
 * never allocates device memory: it works inside a caller-provided workspace.
 * Every function returns MUON_OK (0) or a negative muon_status; nothing here
 * throws (C++ exceptions inside the library, such as a failed host allocation, are caught at the boundary and
 * reported as a status), aborts or prints.  A context is not thread-safe; distinct contexts are
 * independent.  All work of muon_step() is enqueued on the caller's HIP stream
 * and the call returns without synchronising with the device.
 */
#ifndef MUON_H_
#define MUON_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MUON_F32 = 0,    /* IEEE binary32 */
  MUON_BF16 = 1,   /* bfloat16 (upper 16 bits of a binary32, round-to-nearest-even on store) */
  /* Newton-Schulz arithmetic only (ns_dtype), never a buffer dtype: every iterate and temporary is kept as the
   * sum of two / three bf16 arrays (value, rounding remainder, remainder of the remainder) and every product
   * of Eq. 2 runs on the bf16 matrix cores over the plane pairs (i, j) with i + j < planes: 3 / 6 times the
   * work of MUON_BF16 for about 2^-16 / 2^-23 relative accuracy per product instead of 2^-8. */
  MUON_BF16X2 = 2,
  MUON_BF16X3 = 3
} muon_dtype;

typedef enum {
  MUON_OK = 0,
  MUON_E_INVALID_ARG = -1,         /* null pointer, n <= 0, rows/cols < 1, bad hyper-parameter        */
  MUON_E_UNSUPPORTED_DTYPE = -2,   /* a buffer dtype is neither MUON_F32 nor MUON_BF16, or ns_dtype is unknown */
  MUON_E_SHAPE_MISMATCH = -3,      /* the list given to muon_step differs from the one given to init   */
  MUON_E_WORKSPACE_TOO_SMALL = -4, /* workspace cannot hold the tables plus the largest single matrix  */
  MUON_E_HIP = -5,                 /* a HIP runtime call failed (see muon_last_hip_error)              */
  MUON_E_NOT_RESIDENT = -6,        /* debug read of a matrix whose workspace has been reused           */
  MUON_E_MISALIGNED = -7,          /* a buffer pointer is not aligned to its element size              */
  MUON_E_NO_MEMORY = -8,           /* host memory for the plan or its tables could not be allocated    */
  MUON_E_STATIC_LIMIT = -9         /* muon_step_static: more matrices or more workspace than its limits */
} muon_status;

/* The three ways of controlling the update RMS compared in section 3.1; the update is
 * W_t = W_{t-1} - lr * (factor * O_t + weight_decay * W_{t-1}). */
typedef enum {
  MUON_SCALE_ADJUSTED_LR = 0,  /* factor = rms_scale * sqrt(max(A,B))   (Eq. 7 = Eq. 4, the paper's choice) */
  MUON_SCALE_BASELINE = 1,     /* factor = rms_scale * sqrt(hidden_size) (Eq. 5)                             */
  MUON_SCALE_UPDATE_NORM = 2   /* factor = rms_scale / RMS(O_t)          (Eq. 6; O_t = 0 gives factor 0)     */
} muon_scale_mode;

/* One 2-D parameter.  W, G and M are rows x cols, row-major, contiguous. */
typedef struct {
  void* w;              /* device; weight W_{t-1}, dtype w_dtype; overwritten with W_t                 */
  const void* g;        /* device; gradient of this step, dtype g_dtype; read only                     */
  float* m;             /* device; fp32 momentum M_{t-1}; overwritten with M_t; zero before step 1     */
  int64_t rows, cols;   /* A, B of section 2.2 (the matrix as the model defines it, un-sharded)        */
  int32_t w_dtype;      /* muon_dtype                                                                  */
  int32_t g_dtype;      /* muon_dtype                                                                  */
} muon_param;

/* Hyper-parameters of one step (all may change from step to step). */
typedef struct {
  double lr;            /* eta_t                                             */
  double weight_decay;  /* lambda of Eq. 3                                   */
  double momentum;      /* mu                                                */
  double a, b, c;       /* quintic coefficients of Eq. 2 (3.4445, -4.7750, 2.0315) */
  double rms_scale;     /* the 0.2 of Eq. 4                                  */
  double eps;           /* added to ||U||_F; 0 reproduces the paper's formula, >0 guards an all-zero U */
  int32_t ns_steps;     /* N >= 0 (the paper uses 5)                         */
  int32_t nesterov;     /* 0: U = M_t;  1: U = mu*M_t + G                    */
  int32_t scale_mode;   /* muon_scale_mode: which factor multiplies O in the update (section 3.1) */
  int32_t reserved;     /* must be 0                                         */
  double hidden_size;   /* H of the "Baseline" variant (Eq. 5); ignored by the other modes */
  const double* coeff_schedule; /* null (the paper: one triple for all iterations), or a HOST array of 3*ns_steps
                                   doubles, iteration k of Eq. 2 using (a,b,c) = [3k], [3k+1], [3k+2] instead of
                                   a, b, c above; read during the call, not kept                              */
} muon_hparams;

typedef struct muon_ctx muon_ctx;

/* Fills *hp with the paper's settings: mu 0.95, N 5, (a,b,c) above, rms_scale 0.2, nesterov 1,
 * eps 1e-7, lr 0, weight_decay 0, scale_mode MUON_SCALE_ADJUSTED_LR, hidden_size 0. */
int muon_default_hparams(muon_hparams* hp);

/*
 * Workspace size for a parameter list.  Only rows/cols/dtypes of `shapes` are read (pointers may be
 * null).  ns_dtype selects the Newton-Schulz arithmetic: MUON_BF16 (bf16 operands, fp32 accumulation;
 * section 2.3 notes bf16 suffices), MUON_F32 (vector ALUs; meant for small matrices), or the split
 * forms MUON_BF16X2 / MUON_BF16X3 (fp32-class accuracy on the matrix cores, the "more accurate"
 * direction of section 2.2 at model sizes).  The Newton-Schulz temporaries of all matrices are
 * kept resident when they fit in `max_bytes`; otherwise the list is processed in consecutive chunks
 * that reuse the workspace.  max_bytes == 0 means "no limit".  *out receives the number of bytes to
 * allocate (256-byte aligned device memory); it is never below the minimum that muon_init accepts.
 *
 * Accuracy of O = the Newton-Schulz result of Eq. 2, as relative Frobenius error against exact arithmetic:
 *   MUON_F32, MUON_BF16X2   <= 1e-4        MUON_BF16X3   <= 1e-5
 *   MUON_BF16               <= 2e-2 for ns_steps <= 5 on matrices whose rows are not all multiples of one row
 *                           and whose shorter side is not a mere handful (measured: 4 rows by 2^20 columns misses
 *                           it, every shape of a transformer from 64 x 64 up to 11008 x 4096 meets it with 1e-2).
 * Outside that range the bf16 arithmetic is not a defect of the kernels but of the format: the quintic is expansive
 * at its fixed point, so rounding noise grows with ns_steps (2.3e-2 at 10 iterations); with a handful of rows, or
 * with identical rows, every singular value carries the same rounding error and nothing averages (2.2-2.9e-2).
 * Use MUON_BF16X2 there.  A singular value of exactly zero has its rounding noise amplified `a`-fold per iteration
 * in every arithmetic: O is accurate on the row and column space of the input only.
 *
 * Range of the input: sum(U^2), 1/||U||_F and 1/||U||_F^2 are fp32 values inside the kernels, so ||U||_F has to lie
 * roughly within [1e-18, 1e18]; a U of all zeros is handled by eps > 0.
 */
int muon_workspace_bytes(const muon_param* shapes, int32_t n, int32_t ns_dtype, size_t max_bytes, size_t* out);

/*
 * Builds the launch plan (orientation, padded extents, tile tables, chunking) for a parameter list and
 * uploads its tables into `workspace` (device memory of `workspace_bytes` bytes, owned by the caller,
 * which must stay alive and untouched until muon_destroy).  Only rows/cols/dtypes are read from
 * `shapes`.  Uses the current HIP device; synchronises with the device once.  On success *out holds a
 * context to be released with muon_destroy.
 */
int muon_init(muon_ctx** out, const muon_param* shapes, int32_t n, int32_t ns_dtype,
              void* workspace, size_t workspace_bytes);

/*
 * One optimizer step over the whole list (same n, shapes and dtypes as at init; buffer pointers may
 * change between steps).  hip_stream is a hipStream_t (null = default stream).  update_rms_out is
 * null or a device array of n floats that receives sqrt(mean(O^2)) per matrix, the logging value
 * returned by Algorithm 1.  Asynchronous: returns after enqueueing.  W and M are updated in place,
 * G is not written.  The only host-side wait happens when the pointer list differs from the previous
 * step's (a small table is then re-uploaded through pinned memory).
 */
int muon_step(muon_ctx* ctx, const muon_param* params, int32_t n, const muon_hparams* hp,
              void* hip_stream, float* update_rms_out);

/*
 * muon_step for callers that cannot allocate device memory - code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc: one call does what muon_init + muon_step do, with the tables and Newton-Schulz
 * temporaries in a fixed device array inside the library instead of a caller-provided workspace.  It calls no
 * hipMalloc, hipFree, hipHostMalloc or event/stream creation.  Same arguments and results as muon_step (params carry
 * the buffer pointers AND the shapes; ns_dtype as for muon_init), on the current device.
 * Limits: n <= MUON_STATIC_MAX_MATRICES, and muon_workspace_bytes(params, n, ns_dtype, 0) <= MUON_STATIC_MAX_BYTES;
 * beyond them the call does nothing and returns MUON_E_STATIC_LIMIT.  Every device the library has run this call on
 * holds MUON_STATIC_MAX_BYTES of device memory until the process ends.
 * All calls on one device share that array: calls that overlap in time on one device (two host threads, or two
 * streams whose work is not ordered) race; calls on one stream, one after the other, are safe.  The array keeps the
 * previous call's contents; nothing in it needs clearing (every temporary is written in full before it is read).
 * When the shape list differs from the previous call's on this device the launch plan is rebuilt in host memory and
 * its tables are uploaded, waiting for hip_stream twice; repeated calls with one shape list only enqueue kernels.
 */
#define MUON_STATIC_MAX_BYTES (64u << 20)
#define MUON_STATIC_MAX_MATRICES 64
int muon_step_static(const muon_param* params, int32_t n, int32_t ns_dtype, const muon_hparams* hp, void* hip_stream,
                     float* update_rms_out);

/*
 * Test hook: copies O_t of matrix `index`, as left by the last muon_step, into dst (device, rows x cols,
 * row-major, dtype dst_dtype), in W's orientation.  Enqueued on hip_stream.  Fails with
 * MUON_E_NOT_RESIDENT when the list is processed in chunks and the matrix is not in the last one.
 */
int muon_debug_read_update(muon_ctx* ctx, int32_t index, void* dst, int32_t dst_dtype, void* hip_stream);

/*
 * Plan introspection (host only, no device work): writes up to `cap` int64 values describing matrix
 * `index`: {m, n, transposed, m_pad, n_pad, chunk, tile_m, tile_n}.  Returns the number written or
 * a negative status.
 */
int muon_plan_describe(const muon_ctx* ctx, int32_t index, int64_t* out, int32_t cap);

/* Number of chunks the list is processed in (1 = everything resident). */
int muon_plan_chunks(const muon_ctx* ctx);

/*
 * Host only: builds the launch plan that muon_init would build for a workspace of `workspace_bytes`, without
 * touching any device (no HIP call is made).  The context it returns can be given to muon_plan_describe,
 * muon_plan_chunks, muon_plan_tiles and muon_destroy only; muon_step and muon_debug_read_update reject it.
 * Same status codes as muon_init.
 */
int muon_plan_only(muon_ctx** out, const muon_param* shapes, int32_t n, int32_t ns_dtype, size_t workspace_bytes);

/*
 * Host only: the tile table of one grouped launch of a context made by muon_plan_only.  `product`: 0 Gram
 * (A = X X^T), 1 polynomial, 2 apply, 3 apply of the last iteration; `level`: 1 = the coarse launch of the
 * matrix-core paths (256 x 256 tiles, plus 512 x 128 tiles over the 128-wide column strip that an m_pad which is an
 * odd multiple of 128 leaves), 0 = the fine launch that takes the rest (128 x 128 tiles on the matrix-core paths,
 * 64 x 64 on the fp32 path, which has no coarse launch).  Writes up to `cap_records` records of six int32
 * {matrix index in the list, first row, first column, rows, columns (in elements), number of 32 x 32 blocks of the
 * tile that are computed}, in launch order, and returns the number of records of the table (which may exceed
 * cap_records) or a negative status.  The block count is rows * columns / 1024 except for the 256 x 256 tiles on the
 * diagonal of a symmetric product in plain bf16, which are computed from the 36 blocks of their upper triangle.  Gram and polynomial tables
 * hold tiles on and above the diagonal of the m_pad x m_pad output; apply tables hold the tiles of X'^T
 * (n_pad x m_pad) on the matrix-core paths and of X' (m_pad x n_pad) on the fp32 path.  The last 512 x 128 tile of
 * a strip is shifted to end at the matrix edge and may overlap its neighbour (both then write the same values).
 */
int muon_plan_tiles(const muon_ctx* ctx, int32_t chunk, int32_t product, int32_t level, int32_t* out,
                    int32_t cap_records);

/*
 * Per-kernel timing with HIP events on the step's own stream, for measurement (not part of the method).
 * While enabled, muon_step brackets every kernel launch with a pair of events; muon_profile_read waits for
 * the recorded work, adds the elapsed times per kernel class to running totals, copies the totals out
 * (milliseconds and launch counts, MUON_PROF_COUNT entries each, either may be null) and optionally resets
 * them.  Enabling costs two event records per launch; when more than 2048 launches are pending, muon_step
 * drains them with a host-side wait.
 */
enum {
  MUON_PROF_MOMENTUM = 0,   /* momentum + sum of squares + cast/orient        */
  MUON_PROF_NORM = 1,       /* norm finalisation                              */
  MUON_PROF_GRAM = 2,       /* A = X X^T                                      */
  MUON_PROF_POLY = 3,       /* B = b A + c A A                                */
  MUON_PROF_APPLY_POLY = 4, /* X = a X + B X                                  */
  MUON_PROF_UPDATE = 5,     /* weight update (Eq. 4)                          */
  MUON_PROF_RMS = 6,        /* update-RMS side output                         */
  MUON_PROF_COUNT = 7
};
int muon_profile_enable(muon_ctx* ctx, int enable);
int muon_profile_read(muon_ctx* ctx, double* ms_out, int64_t* launches_out, int reset);

/*
 * AdamW for the parameters that stay off Muon (RMSNorm gains, LM head, embeddings: section 2.2, "Matching update
 * RMS of AdamW"), sharing lr and weight decay with it:
 *   m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2;
 *   p = p - lr * ( m/(1-beta1^t) / (sqrt(v/(1-beta2^t)) + eps) + weight_decay * p ).
 * Tensors are flat arrays of `numel` elements (any shape); p and g may be fp32 or bf16, the moments m and v
 * are fp32 and updated in place.  Stateless: needs no context and no workspace (pointers travel in kernel
 * arguments, 24 tensors per launch).  Asynchronous on hip_stream.  `step` is t, counted from 1.
 */
typedef struct {
  void* p;            /* device; parameter, dtype p_dtype; updated in place   */
  const void* g;      /* device; gradient, dtype g_dtype; read only           */
  float* m;           /* device; first moment, fp32; updated in place         */
  float* v;           /* device; second moment, fp32; updated in place        */
  int64_t numel;      /* number of elements (>= 1)                            */
  int32_t p_dtype;    /* muon_dtype                                           */
  int32_t g_dtype;    /* muon_dtype                                           */
} muon_adamw_param;

typedef struct {
  double lr, weight_decay;   /* shared with Muon                               */
  double beta1, beta2, eps;  /* 0 <= beta < 1; eps >= 0                        */
  int64_t step;              /* t >= 1                                         */
} muon_adamw_hparams;

int muon_adamw_step(const muon_adamw_param* params, int32_t n, const muon_adamw_hparams* hp, void* hip_stream);

/*
 * Measurement aid (not part of the optimizer path; Section 2.1's Newton-Schulz products are what it prices):
 * runs the bf16 matrix-core instruction and register blocking of the Newton-Schulz GEMMs with operands that never
 * leave registers, one 256-thread block per compute unit, and reports the sustained rate.  That rate bounds every
 * bf16 GEMM on the device; it depends on the operand values (random_operands != 0: uniform in (-1, 1); 0: all
 * zeros) because the chip lowers its clock under switching load.
 *   iters          loop trips, 32 MFMAs per wave each (1 .. 2^20); 40000 runs about 20 ms
 *   tflops_out     host pointer, receives TFLOP/s          clock_mhz_out  host pointer, receives the mean core clock
 * Allocates and frees a few KB of device memory, launches on the default stream of the current device and waits.
 * Returns MUON_OK, MUON_E_INVALID_ARG or MUON_E_HIP.
 */
int muon_probe_mfma_rate(int random_operands, int iters, double* tflops_out, double* clock_mhz_out);

/* Releases host-side state.  The workspace is the caller's to free afterwards. */
void muon_destroy(muon_ctx* ctx);

/* Static, human-readable name of a status code. */
const char* muon_status_string(int status);

/* The hipError_t (as int) recorded by the last call on this thread that returned MUON_E_HIP. */
int muon_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MUON_H_ */
