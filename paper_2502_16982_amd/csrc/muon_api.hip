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

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int round_up_i(int64_t v, int a) { return (int)((v + a - 1) / a * a); }

constexpr int64_t kMaxDim = 1 << 20;   // tile indices are 16-bit in units of >= 64 elements

struct MatPlan {
  int64_t rows, cols;
  int m, n, mp, np, transposed;
  int w_dtype, g_dtype;
  int tile;         // fine GEMM block tile = padding granule, in elements
  int chunk;
  int ew_tr, ew_tc; // 64x64 tiles in U's orientation (padded)
  size_t ns_bytes;  // X + Xt[0] (+ Xt[1], see x_buffers) + Ag + Bp
  size_t part_off;  // first partial (floats)
};

// Tile tables of one block-tile size (byte offsets in the table region).
struct TileSet {
  size_t sym = 0, apply = 0, apply_last = 0;
  int n_sym = 0, n_apply = 0, n_apply_last = 0;
};

// Launch group: all matrices of one chunk.  Each product is one launch per block-tile size: the 256x256 kernel
// covers the part of every output that whole 256-tiles can cover, the fine kernel (128x128 bf16, 64x64 fp32)
// the remaining strips, so that nothing is padded beyond the fine tile.
struct Group {
  int n_prob;
  std::vector<int> members;                       // problem index -> matrix index in the caller's list
  size_t prob_gram[2], prob_poly, prob_apply[4];  // byte offsets of the problem tables ([parity], [parity * 2 + last])
  TileSet fine, coarse;
};

struct Chunk {
  int first, count;
  size_t ew_tiles_off;   // byte offset of the EwTile table
  int n_ew_tiles;
  std::vector<Group> groups;
};

constexpr int kCoarse = 256;   // block tile of the large bf16 kernel

// The bf16 kernel's cheap output is the transposed one: a last iteration that needs only X is posed swapped.
// bf16 path, m >= 64: the a*X term of Eq. 2 is folded into the polynomial, B' = b A + c A A + a I, so that the apply
// product X' = B' X needs no addend (a third of its epilogue's memory traffic).  B's diagonal is rounded to bf16
// once either way; for tiny matrices, where the diagonal carries most of the product, the explicit addend is kept.
bool folds_identity(const MatPlan& q, int ns_dtype) { return ns_dtype == MUON_BF16 && q.m >= 64; }
// The matrix-core paths: plain bf16 and the split forms (every temporary = sum of 2 or 3 bf16 planes, stored one after
// the other; all of them share the bf16 planner, tile tables and kernels).  The split forms keep the explicit a*X
// addend: folded into B's diagonal it would be rounded at the diagonal's magnitude (a = 3.44), not the iterate's.
bool on_matrix_cores(int ns_dtype) { return ns_dtype != MUON_F32; }
int planes_of(int ns_dtype) { return ns_dtype == MUON_BF16X2 ? 2 : ns_dtype == MUON_BF16X3 ? 3 : 1; }
// Iterate-sized buffers per matrix: X and Xt[0] always; Xt[1] on the fp32 path (transpose ping-pong) and, on the
// bf16 path, only for matrices iterated on their transpose (it receives O in W's orientation).
int x_buffers(const MatPlan& q, int ns_dtype) { return (!on_matrix_cores(ns_dtype) || q.transposed) ? 3 : 2; }

// Workgroups are handed to the 8 accelerator dies (XCDs, each with a private L2) round-robin by workgroup index:
// entry b of a tile table runs on XCD b % 8.  Tiles that share operand panels are therefore dealt to the same
// XCD: when a launch holds many problems, each goes whole to the least-loaded XCD; otherwise every problem is
// cut into 8 contiguous runs of its row-major tile list.  Problems arrive longest-first, so the tail of a launch
// is made of short tiles.
constexpr int kXcds = 8;

// Tiles of one problem in an order whose consecutive runs of 32 (one tile per compute unit of an XCD) form
// 4 x 8 blocks of the tile grid: the 32 tiles running together on an XCD then share 4 row panels and 8 column
// panels, which they sweep along k in step, instead of 1 + 32 panels for a row-major run.
// Tiles (i, j) with i < skip_m and j < skip_n are left out (they are covered by the coarser kernel).
// `cuts` receives the list positions at which a block ends.
void blocked_tiles(int32_t prob, int tm, int tn, bool upper_only, int skip_m, int skip_n, std::vector<GemmTile>& out,
                   std::vector<int>& cuts, int BH = 4, int BW = 8) {
  for (int bi = 0; bi < tm; bi += BH)
    for (int bj = 0; bj < tn; bj += BW) {
      for (int i = bi; i < std::min(bi + BH, tm); ++i)
        for (int j = bj; j < std::min(bj + BW, tn); ++j)
          if ((!upper_only || j >= i) && !(i < skip_m && j < skip_n)) out.push_back(GemmTile{prob, (int16_t)i, (int16_t)j});
      if (!out.empty() && (cuts.empty() || cuts.back() != (int)out.size())) cuts.push_back((int)out.size());
    }
}

size_t deal_tiles(const std::vector<std::vector<GemmTile>>& per_problem, const std::vector<std::vector<int>>& per_problem_cuts,
                  GemmTile* out) {
  std::vector<std::vector<GemmTile>> seq(kXcds);
  int rr = 0;
  const bool whole = per_problem.size() >= 4 * (size_t)kXcds;
  for (size_t pi = 0; pi < per_problem.size(); ++pi) {
    const std::vector<GemmTile>& tiles = per_problem[pi];
    const std::vector<int>& cuts = per_problem_cuts[pi];
    if (whole) {
      // least-loaded XCD, ties broken round-robin
      int best = rr;
      for (int x = 0; x < kXcds; ++x)
        if (seq[(rr + x) % kXcds].size() < seq[best].size()) best = (rr + x) % kXcds;
      seq[best].insert(seq[best].end(), tiles.begin(), tiles.end());
      rr = (rr + 1) % kXcds;
    } else {
      // 8 contiguous runs of equal length (so that entry b of the dealt table still lands on die b % 8).  A run
      // starts and ends inside blocks; its whole blocks go first, so that the tiles a die runs together come from
      // one block, and the two partial blocks at its ends follow.
      const size_t n = tiles.size();
      for (int x = 0; x < kXcds; ++x) {
        const size_t lo = n * x / kXcds, hi = n * (x + 1) / kXcds;
        size_t c0 = lo, c1 = lo;                   // first and last block boundary inside [lo, hi] (none: c0 = c1 = lo)
        bool found = false;
        for (int c : cuts)
          if ((size_t)c >= lo && (size_t)c <= hi) {
            if (!found) c0 = (size_t)c;
            c1 = (size_t)c;
            found = true;
          }
        seq[x].insert(seq[x].end(), tiles.begin() + c0, tiles.begin() + c1);
        seq[x].insert(seq[x].end(), tiles.begin() + lo, tiles.begin() + c0);
        seq[x].insert(seq[x].end(), tiles.begin() + c1, tiles.begin() + hi);
      }
    }
  }
  size_t o = 0;
  for (size_t s = 0;; ++s) {
    bool any = false;
    for (int x = 0; x < kXcds; ++x)
      if (s < seq[x].size()) {
        out[o++] = seq[x][s];
        any = true;
      }
    if (!any) break;
  }
  return o;
}

int validate_shapes(const muon_param* p, int32_t n, int32_t ns_dtype) {
  if (!p || n <= 0) return MUON_E_INVALID_ARG;
  if (ns_dtype != MUON_F32 && ns_dtype != MUON_BF16 && ns_dtype != MUON_BF16X2 && ns_dtype != MUON_BF16X3)
    return MUON_E_UNSUPPORTED_DTYPE;
  for (int i = 0; i < n; ++i) {
    if (p[i].rows < 1 || p[i].cols < 1 || p[i].rows > kMaxDim || p[i].cols > kMaxDim) return MUON_E_INVALID_ARG;
    if ((p[i].w_dtype != MUON_F32 && p[i].w_dtype != MUON_BF16) || (p[i].g_dtype != MUON_F32 && p[i].g_dtype != MUON_BF16))
      return MUON_E_UNSUPPORTED_DTYPE;
  }
  return MUON_OK;
}

void plan_matrices(const muon_param* p, int n, int ns_dtype, std::vector<MatPlan>& out, size_t& total_partials) {
  out.resize(n);
  total_partials = 0;
  const size_t es = on_matrix_cores(ns_dtype) ? 2 : 4;
  for (int i = 0; i < n; ++i) {
    MatPlan& q = out[i];
    q.rows = p[i].rows;
    q.cols = p[i].cols;
    q.transposed = q.rows > q.cols;
    q.m = (int)std::min(q.rows, q.cols);
    q.n = (int)std::max(q.rows, q.cols);
    q.w_dtype = p[i].w_dtype;
    q.g_dtype = p[i].g_dtype;
    q.tile = on_matrix_cores(ns_dtype) ? kShapeTile[kShape128] : kF32Tile;
    q.mp = round_up_i(q.m, q.tile);
    q.np = round_up_i(q.n, q.tile);
    const int ap = q.transposed ? q.np : q.mp, bp = q.transposed ? q.mp : q.np;
    q.ew_tr = ap / kEwTile;
    q.ew_tc = bp / kEwTile;
    q.ns_bytes = (align_up(es * (size_t)q.mp * q.np, 256) * x_buffers(q, ns_dtype) + align_up(es * (size_t)q.mp * q.mp, 256) * 2) *
                 (size_t)planes_of(ns_dtype);
    q.part_off = total_partials;
    total_partials += (size_t)q.ew_tr * q.ew_tc;
    q.chunk = 0;
  }
}

// Size of everything that is not Newton-Schulz temporaries, for a given chunking.
struct TableLayout {
  size_t mats, ptrs, scal, partials, ew_tiles, gemm, total;
};

size_t gemm_tables_bytes_for(const MatPlan& q) {
  const int tm = q.mp / q.tile, tn = q.np / q.tile;
  const size_t sym = (size_t)tm * (tm + 1) / 2, app = (size_t)tm * tn;
  return 6 * sizeof(GemmProblem) + (sym + 2 * app) * sizeof(GemmTile);
}

TableLayout table_layout(const std::vector<MatPlan>& mp, size_t total_partials) {
  TableLayout t{};
  const size_t n = mp.size();
  size_t gemm = 0;
  for (const MatPlan& q : mp) gemm += gemm_tables_bytes_for(q);
  // every table start is aligned to 256 B; chunks x groups x 8 tables bounds the slack
  t.mats = align_up(n * sizeof(MatDesc), 256);
  t.ptrs = align_up(n * sizeof(MatPtrs), 256);
  t.scal = align_up(n * 4 * sizeof(float), 256);
  t.partials = align_up(total_partials * sizeof(float), 256);
  t.ew_tiles = align_up(total_partials * sizeof(EwTile), 256) + 256 * n;  // per-chunk alignment slack
  t.gemm = align_up(gemm, 256) + (size_t)n * 16 * 256;                                     // alignment slack: <= 2 groups x 8 tables per chunk
  t.total = t.mats + t.ptrs + t.scal + t.partials + t.ew_tiles + t.gemm;
  return t;
}

}  // namespace

struct muon_ctx {
  int n = 0;
  int ns_dtype = MUON_BF16;
  int device = 0;
  std::vector<MatPlan> mats;
  std::vector<Chunk> chunks;
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
  // host-only plan (muon_plan_only): no device tables exist; the table image is kept for muon_plan_tiles
  bool plan_only = false;
  std::vector<unsigned char> host_image;
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
  if (!out) return MUON_E_INVALID_ARG;
  int st = validate_shapes(shapes, n, ns_dtype);
  if (st != MUON_OK) return st;
  std::vector<MatPlan> mp;
  size_t total_partials = 0;
  plan_matrices(shapes, n, ns_dtype, mp, total_partials);
  const TableLayout tl = table_layout(mp, total_partials);
  size_t all = 0, biggest = 0;
  for (const MatPlan& q : mp) {
    all += q.ns_bytes;
    biggest = std::max(biggest, q.ns_bytes);
  }
  size_t want = tl.total + all;
  const size_t least = tl.total + biggest;
  if (max_bytes != 0 && want > max_bytes) want = std::max(max_bytes, least);
  *out = align_up(want, 256);
  return MUON_OK;
}

}  // extern "C"

namespace {

// Everything muon_init does short of touching the device: the plan and the host image of the table region.  With
// `upload` the image goes to the workspace and the per-context HIP objects are created.
int build_context(muon_ctx** out, const muon_param* shapes, int32_t n, int32_t ns_dtype, void* workspace,
                  size_t workspace_bytes, bool upload) {
  if (!out) return MUON_E_INVALID_ARG;
  *out = nullptr;
  int st = validate_shapes(shapes, n, ns_dtype);
  if (st != MUON_OK) return st;
  if (!workspace) return MUON_E_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MUON_E_MISALIGNED;

  muon_ctx* ctx = new (std::nothrow) muon_ctx();
  if (!ctx) return MUON_E_INVALID_ARG;
  ctx->n = n;
  ctx->ns_dtype = ns_dtype;
  ctx->ws = static_cast<unsigned char*>(workspace);
  ctx->ws_bytes = workspace_bytes;
  size_t total_partials = 0;
  plan_matrices(shapes, n, ns_dtype, ctx->mats, total_partials);
  const TableLayout tl = table_layout(ctx->mats, total_partials);

  size_t biggest = 0;
  for (const MatPlan& q : ctx->mats) biggest = std::max(biggest, q.ns_bytes);
  if (workspace_bytes < tl.total + biggest) {
    delete ctx;
    return MUON_E_WORKSPACE_TOO_SMALL;
  }
  const size_t ns_budget = workspace_bytes - tl.total;

  // ---- chunking: consecutive matrices while their temporaries fit ----
  {
    size_t used = 0;
    Chunk cur{};
    cur.first = 0;
    for (int i = 0; i < n; ++i) {
      if (cur.count > 0 && used + ctx->mats[i].ns_bytes > ns_budget) {
        ctx->chunks.push_back(cur);
        cur = Chunk{};
        cur.first = i;
        used = 0;
      }
      ctx->mats[i].chunk = (int)ctx->chunks.size();
      used += ctx->mats[i].ns_bytes;
      cur.count++;
    }
    ctx->chunks.push_back(cur);
  }

  // ---- host image of the table region ----
  std::vector<unsigned char> img(tl.total, 0);
  size_t off = 0;
  const size_t off_mats = off; off += tl.mats;
  const size_t off_ptrs = off; off += tl.ptrs;
  const size_t off_scal = off; off += tl.scal;
  const size_t off_part = off; off += tl.partials;
  size_t cursor = off;   // ew tiles and gemm tables are appended from here
  unsigned char* ns_base = ctx->ws + tl.total;
  const size_t es = on_matrix_cores(ns_dtype) ? 2 : 4;
  const size_t planes = (size_t)planes_of(ns_dtype);

  MatDesc* h_mats = reinterpret_cast<MatDesc*>(img.data() + off_mats);
  auto dev = [&](size_t o) { return ctx->ws + o; };

  for (Chunk& ch : ctx->chunks) {
    size_t ns_off = 0;
    for (int i = ch.first; i < ch.first + ch.count; ++i) {
      const MatPlan& q = ctx->mats[i];
      MatDesc& d = h_mats[i];
      const size_t xb = align_up(es * (size_t)q.mp * q.np, 256), ab = align_up(es * (size_t)q.mp * q.mp, 256);
      d.X = ns_base + ns_off; ns_off += xb * planes;
      d.Xt[0] = ns_base + ns_off; ns_off += xb * planes;
      d.Xt[1] = nullptr;
      if (x_buffers(q, ns_dtype) == 3) { d.Xt[1] = ns_base + ns_off; ns_off += xb * planes; }
      d.Ag = ns_base + ns_off; ns_off += ab * planes;
      d.Bp = ns_base + ns_off; ns_off += ab * planes;
      d.x_plane = planes > 1 ? (int64_t)(xb / es) : 0;
      d.pad_ = 0;
      d.partials = reinterpret_cast<float*>(dev(off_part)) + q.part_off;
      d.scal = reinterpret_cast<float*>(dev(off_scal)) + 4 * (size_t)i;
      d.rows = (int)q.rows; d.cols = (int)q.cols;
      d.m = q.m; d.n = q.n; d.mp = q.mp; d.np = q.np;
      d.transposed = q.transposed;
      d.w_dtype = q.w_dtype; d.g_dtype = q.g_dtype;
      d.n_part = q.ew_tr * q.ew_tc;
      d.ew_tiles_c = q.ew_tc;
      d.sqrt_max = (float)std::sqrt((double)q.n);
    }

    // elementwise tiles of the chunk
    cursor = align_up(cursor, 256);
    ch.ew_tiles_off = cursor;
    ch.n_ew_tiles = 0;
    {
      EwTile* t = reinterpret_cast<EwTile*>(img.data() + cursor);
      for (int i = ch.first; i < ch.first + ch.count; ++i) {
        const MatPlan& q = ctx->mats[i];
        for (int r = 0; r < q.ew_tr; ++r)
          for (int c = 0; c < q.ew_tc; c += kEwRun) {
            t[ch.n_ew_tiles].mat = i;
            t[ch.n_ew_tiles].tr = (int16_t)r;
            t[ch.n_ew_tiles].tc = (int16_t)c;
            t[ch.n_ew_tiles].count = (int16_t)std::min(kEwRun, q.ew_tc - c);
            t[ch.n_ew_tiles].pad_ = 0;
            ch.n_ew_tiles++;
          }
      }
      cursor += (size_t)ch.n_ew_tiles * sizeof(EwTile);
    }

    // GEMM group of the chunk
    {
      std::vector<int> members;
      for (int i = ch.first; i < ch.first + ch.count; ++i) members.push_back(i);
      // longest work first, so that the tail of the launch is made of short tiles
      std::stable_sort(members.begin(), members.end(), [&](int x, int y) {
        const MatPlan &a = ctx->mats[x], &b = ctx->mats[y];
        return (int64_t)a.np + a.mp > (int64_t)b.np + b.mp;
      });
      Group g{};
      g.n_prob = (int)members.size();
      g.members = members;
      auto take = [&](size_t bytes) {
        cursor = align_up(cursor, 256);
        const size_t o = cursor;
        cursor += bytes;
        return o;
      };
      for (int v = 0; v < 2; ++v) g.prob_gram[v] = take(sizeof(GemmProblem) * members.size());
      g.prob_poly = take(sizeof(GemmProblem) * members.size());
      for (int v = 0; v < 4; ++v) g.prob_apply[v] = take(sizeof(GemmProblem) * members.size());
      for (size_t k = 0; k < members.size(); ++k) {
        const MatPlan& q = ctx->mats[members[k]];
        const MatDesc& d = h_mats[members[k]];
        GemmProblem gp{};
        gp.scal = d.scal;
        const bool mc = on_matrix_cores(ns_dtype);
        const size_t xb = align_up(es * (size_t)q.mp * q.np, 256), ab = align_up(es * (size_t)q.mp * q.mp, 256);
        const int64_t xpl = planes > 1 ? (int64_t)(xb / es) : 0, apl = planes > 1 ? (int64_t)(ab / es) : 0;
        // bf16 path: ONE layout of the iterate, ping-ponging between X and Xt[0] (both m_pad x n_pad); fp32 path: X
        // updated in place plus its transpose ping-ponging between Xt[0] and Xt[1].
        void* const xbuf[2] = {d.X, mc ? d.Xt[0] : d.X};
        // Gram: A = X X^T
        for (int par = 0; par < 2; ++par) {
          gp.L = xbuf[par]; gp.R = xbuf[par]; gp.E = nullptr; gp.Et = nullptr; gp.C = d.Ag; gp.Ct = nullptr;
          gp.K = q.np; gp.ldl = q.np; gp.ldr = q.np; gp.lde = 0; gp.ldet = 0; gp.ldc = q.mp; gp.ldct = q.mp; gp.symmetric = 1;
          gp.l_plane = xpl; gp.r_plane = xpl; gp.et_plane = 0; gp.c_plane = apl; gp.ct_plane = apl;
          reinterpret_cast<GemmProblem*>(img.data() + g.prob_gram[par])[k] = gp;
        }
        // polynomial: B = b A + c A A  (A is symmetric, so it is its own transposed addend)
        gp.L = d.Ag; gp.R = d.Ag; gp.E = d.Ag; gp.Et = d.Ag; gp.C = d.Bp; gp.Ct = nullptr;
        gp.K = q.mp; gp.ldl = q.mp; gp.ldr = q.mp; gp.lde = q.mp; gp.ldet = q.mp; gp.ldc = q.mp; gp.ldct = q.mp; gp.symmetric = 1;
        gp.l_plane = apl; gp.r_plane = apl; gp.et_plane = apl; gp.c_plane = apl; gp.ct_plane = apl;
        gp.diag_add = folds_identity(q, ns_dtype) ? 1 : 0;
        reinterpret_cast<GemmProblem*>(img.data() + g.prob_poly)[k] = gp;
        gp.diag_add = 0;
        for (int par = 0; par < 2; ++par)
          for (int last = 0; last < 2; ++last) {
            gp.symmetric = 0;
            if (mc) {
              // apply, bf16: the product is posed transposed, T = X'^T = X^T B, with its L operand X^T read K-major
              // straight from the row-major X; the kernel's cheap transposed store of T is then X' itself, row-major.
              // Only the last iteration of a matrix iterated on its transpose needs T as it is (O in W's
              // orientation), through the kernel's other output, into Xt[1].
              gp.L = xbuf[par]; gp.R = d.Bp; gp.K = q.mp; gp.ldl = q.np; gp.ldr = q.mp;
              gp.E = nullptr; gp.lde = 0;
              gp.Et = folds_identity(q, ns_dtype) ? nullptr : xbuf[par]; gp.ldet = q.np;
              gp.C = nullptr; gp.ldc = 0; gp.Ct = xbuf[par ^ 1]; gp.ldct = q.np;
              if (last && q.transposed) { gp.C = d.Xt[1]; gp.ldc = q.mp; gp.Ct = nullptr; gp.ldct = 0; }
              gp.l_plane = xpl; gp.r_plane = apl; gp.et_plane = xpl; gp.c_plane = xpl; gp.ct_plane = xpl;
            } else {
              // apply, fp32: X' = a X + B X, reading X^T from Xt[p], writing X in place and X'^T to Xt[p^1]; the last
              // iteration writes only the layout W needs.
              gp.L = d.Bp; gp.R = d.Xt[par]; gp.E = d.X; gp.Et = d.Xt[par]; gp.C = d.X; gp.Ct = d.Xt[par ^ 1];
              gp.K = q.mp; gp.ldl = q.mp; gp.ldr = q.mp; gp.lde = q.np; gp.ldet = q.mp; gp.ldc = q.np; gp.ldct = q.mp;
              if (last) {
                if (q.transposed) gp.C = nullptr;
                else gp.Ct = nullptr;
              }
            }
            reinterpret_cast<GemmProblem*>(img.data() + g.prob_apply[par * 2 + last])[k] = gp;
          }
      }
      // tile tables: level 1 = whole 256-tiles (bf16 only), level 0 = what they leave uncovered
      for (int level = 1; level >= 0; --level) {
        if (level == 1 && !on_matrix_cores(ns_dtype)) continue;
        std::vector<std::vector<GemmTile>> sym(members.size()), app(members.size()), app_last(members.size());
        std::vector<std::vector<int>> sym_cuts(members.size()), app_cuts(members.size());
        size_t n_sym = 0, n_app = 0, n_last = 0;
        for (size_t k = 0; k < members.size(); ++k) {
          const MatPlan& q = ctx->mats[members[k]];
          const int cm = on_matrix_cores(ns_dtype) ? q.mp / kCoarse : 0, cn = on_matrix_cores(ns_dtype) ? q.np / kCoarse : 0;
          if (level == 1) {
            blocked_tiles((int32_t)k, cm, cm, true, 0, 0, sym[k], sym_cuts[k]);
            // tiles of X'^T; 8 x 4 blocks measured 1 % faster than 4 x 8 here (the K-major panels are the strided ones)
            if (on_matrix_cores(ns_dtype)) blocked_tiles((int32_t)k, cn, cm, false, 0, 0, app[k], app_cuts[k], 8, 4);
            else blocked_tiles((int32_t)k, cm, cn, false, 0, 0, app[k], app_cuts[k]);
            app_last[k] = app[k];
          } else {
            const int tm = q.mp / q.tile, tn = q.np / q.tile, r = kCoarse / q.tile;
            blocked_tiles((int32_t)k, tm, tm, true, cm * r, cm * r, sym[k], sym_cuts[k]);
            if (on_matrix_cores(ns_dtype)) blocked_tiles((int32_t)k, tn, tm, false, cn * r, cm * r, app[k], app_cuts[k], 8, 4);
            else blocked_tiles((int32_t)k, tm, tn, false, cm * r, cn * r, app[k], app_cuts[k]);
            app_last[k] = app[k];
          }
          n_sym += sym[k].size();
          n_app += app[k].size();
          n_last += app_last[k].size();
        }
        TileSet& ts = level ? g.coarse : g.fine;
        ts.sym = take(n_sym * sizeof(GemmTile));
        ts.apply = take(n_app * sizeof(GemmTile));
        ts.apply_last = take(n_last * sizeof(GemmTile));
        ts.n_sym = (int)deal_tiles(sym, sym_cuts, reinterpret_cast<GemmTile*>(img.data() + ts.sym));
        ts.n_apply = (int)deal_tiles(app, app_cuts, reinterpret_cast<GemmTile*>(img.data() + ts.apply));
        ts.n_apply_last = (int)deal_tiles(app_last, app_cuts, reinterpret_cast<GemmTile*>(img.data() + ts.apply_last));
      }
      ch.groups.push_back(g);
    }
  }
  if (cursor > tl.total) {   // the layout bound is conservative; this cannot happen
    delete ctx;
    return MUON_E_WORKSPACE_TOO_SMALL;
  }

  ctx->d_mats = reinterpret_cast<MatDesc*>(dev(off_mats));
  ctx->d_ptrs = reinterpret_cast<MatPtrs*>(dev(off_ptrs));
  if (!upload) {
    ctx->plan_only = true;
    img.resize(cursor);
    ctx->host_image.swap(img);
    *out = ctx;
    return MUON_OK;
  }

  hipError_t e = hipGetDevice(&ctx->device);
  if (e == hipSuccess) e = gemm_setup();
  if (e == hipSuccess) e = hipMemcpy(ctx->ws, img.data(), cursor, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&ctx->h_ptrs_pinned), sizeof(MatPtrs) * (size_t)n, hipHostMallocDefault);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->upload_done, hipEventDisableTiming);
  if (e != hipSuccess) {
    muon_destroy(ctx);
    return hip_fail(e);
  }
  ctx->last_ptrs.resize(n);
  *out = ctx;
  return MUON_OK;
}

}  // namespace

extern "C" {

int muon_init(muon_ctx** out, const muon_param* shapes, int32_t n, int32_t ns_dtype, void* workspace,
              size_t workspace_bytes) {
  return build_context(out, shapes, n, ns_dtype, workspace, workspace_bytes, true);
}

int muon_plan_only(muon_ctx** out, const muon_param* shapes, int32_t n, int32_t ns_dtype, size_t workspace_bytes) {
  // table pointers are computed from the workspace address but never followed: any aligned non-null address will do
  return build_context(out, shapes, n, ns_dtype, reinterpret_cast<void*>(uintptr_t{1} << 32), workspace_bytes, false);
}

int muon_plan_tiles(const muon_ctx* ctx, int32_t chunk, int32_t product, int32_t level, int32_t* out, int32_t cap_records) {
  if (!ctx || !ctx->plan_only || chunk < 0 || chunk >= (int)ctx->chunks.size() || product < 0 || product > 3 || level < 0 ||
      level > 1 || cap_records < 0 || (cap_records > 0 && !out))
    return MUON_E_INVALID_ARG;
  int64_t total = 0;
  for (const Group& g : ctx->chunks[chunk].groups) {
    const TileSet& ts = level ? g.coarse : g.fine;
    const size_t off = product <= 1 ? ts.sym : product == 2 ? ts.apply : ts.apply_last;
    const int count = product <= 1 ? ts.n_sym : product == 2 ? ts.n_apply : ts.n_apply_last;
    const GemmTile* t = reinterpret_cast<const GemmTile*>(ctx->host_image.data() + off);
    for (int i = 0; i < count; ++i, ++total) {
      if (total >= cap_records) continue;
      const int mat = g.members[t[i].prob];
      const int size = level ? kCoarse : ctx->mats[mat].tile;
      int32_t* r = out + 4 * total;
      r[0] = mat; r[1] = t[i].ti; r[2] = t[i].tj; r[3] = size;
    }
  }
  return (int)std::min<int64_t>(total, INT32_MAX);
}

int muon_step(muon_ctx* ctx, const muon_param* params, int32_t n, const muon_hparams* hp, void* hip_stream,
              float* update_rms_out) {
  if (!ctx || !params || !hp || ctx->plan_only) return MUON_E_INVALID_ARG;
  if (n != ctx->n) return MUON_E_SHAPE_MISMATCH;
  if (hp->ns_steps < 0 || !(hp->eps >= 0.0) || !std::isfinite(hp->lr) || !std::isfinite(hp->weight_decay) ||
      !std::isfinite(hp->momentum) || !std::isfinite(hp->a) || !std::isfinite(hp->b) || !std::isfinite(hp->c) ||
      !std::isfinite(hp->rms_scale) || hp->scale_mode < MUON_SCALE_ADJUSTED_LR || hp->scale_mode > MUON_SCALE_UPDATE_NORM ||
      hp->reserved != 0 || (hp->scale_mode == MUON_SCALE_BASELINE && !(hp->hidden_size > 0.0 && std::isfinite(hp->hidden_size))))
    return MUON_E_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  bool changed = !ctx->ptrs_valid;
  for (int i = 0; i < n; ++i) {
    const muon_param& p = params[i];
    const MatPlan& q = ctx->mats[i];
    if (p.rows != q.rows || p.cols != q.cols || p.w_dtype != q.w_dtype || p.g_dtype != q.g_dtype) return MUON_E_SHAPE_MISMATCH;
    if (!p.w || !p.g || !p.m) return MUON_E_INVALID_ARG;
    const uintptr_t wa = p.w_dtype == MUON_BF16 ? 1u : 3u, ga = p.g_dtype == MUON_BF16 ? 1u : 3u;
    if ((reinterpret_cast<uintptr_t>(p.w) & wa) || (reinterpret_cast<uintptr_t>(p.g) & ga) || (reinterpret_cast<uintptr_t>(p.m) & 3u))
      return MUON_E_MISALIGNED;
    const MatPtrs& l = ctx->last_ptrs[i];
    if (l.w != p.w || l.g != p.g || l.m != p.m) changed = true;
  }
  if (changed) {
    // the previous upload may still be reading the pinned staging buffer
    if (ctx->ptrs_valid) MUON_HIP(hipEventSynchronize(ctx->upload_done));
    for (int i = 0; i < n; ++i) {
      ctx->last_ptrs[i] = MatPtrs{params[i].w, params[i].g, params[i].m};
      ctx->h_ptrs_pinned[i] = ctx->last_ptrs[i];
    }
    MUON_HIP(hipMemcpyAsync(ctx->d_ptrs, ctx->h_ptrs_pinned, sizeof(MatPtrs) * (size_t)n, hipMemcpyHostToDevice, s));
    MUON_HIP(hipEventRecord(ctx->upload_done, s));
    ctx->ptrs_valid = true;
  }

  const int N = hp->ns_steps;
  const int use_s = N == 0;
  const bool mc = on_matrix_cores(ctx->ns_dtype);   // bf16 or split-bf16: the MFMA kernels and their one-layout plan
  const int planes = planes_of(ctx->ns_dtype);
  // where O ends up (see o_source in the elementwise kernels): fp32 path: X in place, its transpose in Xt[N & 1];
  // bf16 path: X ping-pong index N & 1 (bit 1), transposed matrices in Xt[1], or Xt[0] when no iteration ran (bit 0)
  const int o_sel = mc ? ((N & 1) << 1) | (N > 0 ? 1 : 0) : (N & 1);
  if (hp->coeff_schedule)
    for (int i = 0; i < 3 * N; ++i)
      if (!std::isfinite(hp->coeff_schedule[i])) return MUON_E_INVALID_ARG;

  for (size_t ci = 0; ci < ctx->chunks.size(); ++ci) {
    const Chunk& ch = ctx->chunks[ci];
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
        // one launch per product and block-tile size (256-tiles first, then the strips they leave)
        for (int level = 1; level >= 0; --level) {
          const TileSet& ts = level ? g.coarse : g.fine;
          if (ts.n_sym == 0) continue;
          if (mc)
            MUON_TIMED(MUON_PROF_GRAM, launch_gemm_bf16(level ? kShape256 : kShape128, P(g.prob_gram[par]), T(ts.sym), ts.n_sym, 1.f, 0.f,
                                                        first ? 1 : -1, 0.f, 0, planes, s));
          else
            MUON_TIMED(MUON_PROF_GRAM, launch_gemm_f32(P(g.prob_gram[par]), T(ts.sym), ts.n_sym, 1.f, 0.f, first ? 1 : -1, s));
        }
        for (int level = 1; level >= 0; --level) {
          const TileSet& ts = level ? g.coarse : g.fine;
          if (ts.n_sym == 0) continue;
          if (mc)
            MUON_TIMED(MUON_PROF_POLY, launch_gemm_bf16(level ? kShape256 : kShape128, P(g.prob_poly), T(ts.sym), ts.n_sym, c, b, -1, a, 0, planes, s));
          else
            MUON_TIMED(MUON_PROF_POLY, launch_gemm_f32(P(g.prob_poly), T(ts.sym), ts.n_sym, c, b, -1, s));
        }
        for (int level = 1; level >= 0; --level) {
          const TileSet& ts = level ? g.coarse : g.fine;
          const size_t t_app = last ? ts.apply_last : ts.apply;
          const int n_app = last ? ts.n_apply_last : ts.n_apply;
          if (n_app == 0) continue;
          if (mc)
            MUON_TIMED(MUON_PROF_APPLY_POLY, launch_gemm_bf16(level ? kShape256 : kShape128, P(g.prob_apply[par * 2 + last]), T(t_app),
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
  ctx->last_chunk = (int)ctx->chunks.size() - 1;
  return MUON_OK;
}

int muon_debug_read_update(muon_ctx* ctx, int32_t index, void* dst, int32_t dst_dtype, void* hip_stream) {
  if (!ctx || ctx->plan_only || !dst || index < 0 || index >= ctx->n) return MUON_E_INVALID_ARG;
  if (dst_dtype != MUON_F32 && dst_dtype != MUON_BF16) return MUON_E_UNSUPPORTED_DTYPE;
  if (ctx->last_chunk < 0 || ctx->mats[index].chunk != ctx->last_chunk) return MUON_E_NOT_RESIDENT;
  MUON_HIP(launch_read_update(ctx->d_mats, index, ctx->last_o_sel, ctx->last_use_s, ctx->ns_dtype, dst, dst_dtype,
                              static_cast<hipStream_t>(hip_stream)));
  return MUON_OK;
}

int muon_plan_describe(const muon_ctx* ctx, int32_t index, int64_t* out, int32_t cap) {
  if (!ctx || !out || index < 0 || index >= ctx->n || cap < 0) return MUON_E_INVALID_ARG;
  const MatPlan& q = ctx->mats[index];
  const int coarse = on_matrix_cores(ctx->ns_dtype) && q.mp >= kCoarse ? kCoarse : q.tile;
  const int64_t v[8] = {q.m, q.n, q.transposed, q.mp, q.np, q.chunk, coarse, q.tile};
  const int k = std::min<int>(cap, 8);
  for (int i = 0; i < k; ++i) out[i] = v[i];
  return k;
}

int muon_profile_enable(muon_ctx* ctx, int enable) {
  if (!ctx || ctx->plan_only) return MUON_E_INVALID_ARG;
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

int muon_plan_chunks(const muon_ctx* ctx) { return ctx ? (int)ctx->chunks.size() : MUON_E_INVALID_ARG; }

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
    default: return "unknown status";
  }
}

int muon_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
