// Host-side launch planner of the Muon step (see muon_plan.h).  Plain C++: no HIP header, no device call.
#include "muon_plan.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>

namespace muon {

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int round_up_i(int64_t v, int a) { return (int)((v + a - 1) / a * a); }

// Iterate-sized buffers per matrix: X and Xt[0] always; Xt[1] on the fp32 path (transpose ping-pong) and, on the
// bf16 path, only for matrices iterated on their transpose (it receives O in W's orientation).
int x_buffers(const MatPlan& q, int ns_dtype) { return (!on_matrix_cores(ns_dtype) || q.transposed) ? 3 : 2; }

// Workgroups are handed to the 8 accelerator dies (XCDs, each with a private L2) round-robin by workgroup index:
// entry b of a tile table runs on XCD b % 8.  Tiles that share operand panels are therefore dealt to the same
// XCD: when a launch holds many problems, each goes whole to the least-loaded XCD; otherwise every problem is
// cut into 8 contiguous runs of its tile list.  Problems arrive longest-first, so the tail of a launch is made of
// short tiles.
constexpr int kXcds = 8;

GemmTile make_tile(int32_t prob, int row0, int col0, int shape, int flags) {
  GemmTile t{};
  t.prob = prob;
  t.r0 = (uint16_t)(row0 / kTileUnit);
  t.c0 = (uint16_t)(col0 / kTileUnit);
  t.shape = (uint8_t)shape;
  t.flags = (uint8_t)flags;
  t.pad_ = 0;
  return t;
}

// Square tiles of `size` elements over a tm x tn grid, in an order whose consecutive runs of 32 (one tile per compute
// unit of an XCD) form BH x BW blocks of the grid: the 32 tiles running together on an XCD then share BH row panels
// and BW column panels, which they sweep along k in step, instead of 1 + 32 panels for a row-major run.
// Tiles (i, j) with i < skip_m and j < skip_n are left out (a coarser shape covers them), as is column skip_col
// (covered by strip tiles; -1: none).  upper_only: tiles on or above the diagonal; those on it get kTileDiagonal and,
// when diag_shape >= 0, that shape.
// `cuts` receives the list positions at which a block ends.
void blocked_tiles(int32_t prob, int size, int shape, int tm, int tn, bool upper_only, int skip_m, int skip_n, int skip_col,
                   std::vector<GemmTile>& out, std::vector<int>& cuts, int BH = 4, int BW = 8, int diag_shape = -1) {
  for (int bi = 0; bi < tm; bi += BH)
    for (int bj = 0; bj < tn; bj += BW) {
      for (int i = bi; i < std::min(bi + BH, tm); ++i)
        for (int j = bj; j < std::min(bj + BW, tn); ++j)
          if ((!upper_only || j >= i) && !(i < skip_m && j < skip_n) && j != skip_col) {
            const bool diag = upper_only && i == j;
            out.push_back(make_tile(prob, i * size, j * size, diag && diag_shape >= 0 ? diag_shape : shape, diag ? kTileDiagonal : 0));
          }
      if (!out.empty() && (cuts.empty() || cuts.back() != (int)out.size())) cuts.push_back((int)out.size());
    }
}

// 512 x 128 tiles over the 128-wide column strip [0, rows) x [col0, col0 + 128) of an output (rows >= 512, a multiple
// of 128).  The last tile is shifted up to end at `rows`; where it overlaps its neighbour both compute the same
// values from the same operands in the same order.
void strip_tiles(int32_t prob, int rows, int col0, std::vector<GemmTile>& out, std::vector<int>& cuts) {
  const int H = kShapeRows[kShape512x128];
  for (int r0 = 0; r0 < rows; r0 += H) out.push_back(make_tile(prob, std::min(r0, rows - H), col0, kShape512x128, 0));
  cuts.push_back((int)out.size());
}

// A persistent launch (one block per compute unit striding through the table) gives every block the same number of
// tiles only if the table length is a multiple of the number of blocks; the r tiles beyond that cost the launch a whole
// extra round.  When r is small they are taken out of the coarse lists - plain 256 x 256 tiles from the end of the
// problems that come last in the launch order - and handed to the fine launch, four 128 x 128 tiles each, where they
// run side by side, one per compute unit.  `moved` receives them per problem; returns how many were moved.
constexpr int kMaxMovedTiles = 64;
size_t move_tail_to_fine(const std::vector<int>& order, std::vector<std::vector<GemmTile>>& lists,
                         std::vector<std::vector<int>>& cuts, int blocks, std::vector<std::vector<GemmTile>>& moved) {
  size_t total = 0;
  for (const auto& l : lists) total += l.size();
  if (blocks <= 0 || total <= (size_t)blocks) return 0;
  const size_t r = total % (size_t)blocks;
  if (r == 0 || r > (size_t)kMaxMovedTiles) return 0;
  size_t plain = 0;
  for (const auto& l : lists)
    for (const GemmTile& t : l) plain += (t.shape == kShape256 && !(t.flags & kTileDiagonal)) ? 1 : 0;
  if (plain < r) return 0;
  size_t left = r;
  for (size_t oi = order.size(); oi-- > 0 && left > 0;) {
    std::vector<GemmTile>& l = lists[order[oi]];
    for (size_t i = l.size(); i-- > 0 && left > 0;)
      if (l[i].shape == kShape256 && !(l[i].flags & kTileDiagonal)) {
        moved[order[oi]].push_back(l[i]);
        l.erase(l.begin() + (std::ptrdiff_t)i);
        --left;
      }
    // block boundaries are list positions: those past the shortened list go
    std::vector<int>& c = cuts[order[oi]];
    while (!c.empty() && c.back() > (int)l.size()) c.pop_back();
  }
  return r;
}

// `slots` > 0 (coarse tables; the compute units of a die): a persistent launch gives the block in slot c of a die the
// entries c, c + slots, c + 2 slots, ... of that die's sequence.  Tiles differ in cost (a diagonal tile issues 9/16
// of the MFMAs of a full one), so within every run of `slots` entries - the tiles the die runs at the same time,
// whose set stays as it is - the tiles are handed to the slots most expensive first, each to the slot that has
// accumulated least so far.
size_t deal_tiles(const std::vector<int>& order, const std::vector<std::vector<GemmTile>>& per_problem,
                  const std::vector<std::vector<int>>& per_problem_cuts, const std::vector<int64_t>& weight, GemmTile* out,
                  int slots = 0) {
  std::vector<std::vector<GemmTile>> seq(kXcds);
  std::vector<int64_t> load(kXcds, 0);
  int rr = 0;
  size_t nonempty = 0;
  for (const auto& t : per_problem) nonempty += t.empty() ? 0 : 1;
  const bool whole = nonempty >= 4 * (size_t)kXcds;
  for (int pi : order) {
    const std::vector<GemmTile>& tiles = per_problem[pi];
    const std::vector<int>& cuts = per_problem_cuts[pi];
    if (tiles.empty()) continue;
    if (whole) {
      // least-loaded XCD (tiles weighted by the length of their K loop), ties broken round-robin
      int best = rr;
      for (int x = 0; x < kXcds; ++x)
        if (load[(rr + x) % kXcds] < load[best]) best = (rr + x) % kXcds;
      seq[best].insert(seq[best].end(), tiles.begin(), tiles.end());
      load[best] += weight[pi] * (int64_t)tiles.size();
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
  if (slots > 0) {
    // cost in units of K: the MFMA work of the main loop plus a fixed part for the first slabs and the epilogue; a
    // 512 x 128 tile counts a quarter more than a 256 x 256 one (640 operand rows per K slab instead of 512; measured:
    // factors 1.15 to 1.3 do equally well, the fixed part hardly matters)
    auto cost = [&](const GemmTile& t) {
      int64_t blocks = t.shape == kShape256Diag ? 36 : (int64_t)kShapeRows[t.shape] * kShapeCols[t.shape] / 1024;
      if (t.shape == kShape512x128) blocks += blocks / 4;
      return (int64_t)512 + weight[t.prob] * blocks / 64;
    };
    for (auto& q : seq) {
      std::vector<int64_t> acc((size_t)slots, 0);
      for (size_t r0 = 0; r0 < q.size(); r0 += (size_t)slots) {
        const size_t cnt = std::min((size_t)slots, q.size() - r0);
        std::vector<GemmTile> round(q.begin() + (std::ptrdiff_t)r0, q.begin() + (std::ptrdiff_t)(r0 + cnt));
        std::stable_sort(round.begin(), round.end(), [&](const GemmTile& a, const GemmTile& b) { return cost(a) > cost(b); });
        std::vector<size_t> slot(cnt);
        std::iota(slot.begin(), slot.end(), (size_t)0);
        std::stable_sort(slot.begin(), slot.end(), [&](size_t a, size_t b) { return acc[a] < acc[b]; });
        for (size_t i = 0; i < cnt; ++i) {
          q[r0 + slot[i]] = round[i];
          acc[slot[i]] += cost(round[i]);
        }
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
    q.tile = on_matrix_cores(ns_dtype) ? kShapeRows[kShape128] : kF32Tile;
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

// Size of everything that is not Newton-Schulz temporaries.
struct TableLayout {
  size_t mats, ptrs, scal, partials, ew_tiles, gemm, total;
};

// No tile shape is smaller than the fine tile, so the fine-tile counts bound the table sizes.
size_t gemm_tables_bytes_for(const MatPlan& q) {
  const int tm = q.mp / q.tile, tn = q.np / q.tile;
  const size_t sym = (size_t)tm * (tm + 1) / 2 + 1, app = (size_t)tm * tn + 1;
  return 7 * sizeof(GemmProblem) + (2 * sym + 2 * app) * sizeof(GemmTile);
}

TableLayout table_layout(const std::vector<MatPlan>& mp, size_t total_partials) {
  TableLayout t{};
  const size_t n = mp.size();
  size_t gemm = 0;
  for (const MatPlan& q : mp) gemm += gemm_tables_bytes_for(q);
  // every table start is aligned to 256 B; chunks x groups x 13 tables bounds the slack
  t.mats = align_up(n * sizeof(MatDesc), 256);
  t.ptrs = align_up(n * sizeof(MatPtrs), 256);
  t.scal = align_up(n * 4 * sizeof(float), 256);
  t.partials = align_up(total_partials * sizeof(float), 256);
  t.ew_tiles = align_up(total_partials * sizeof(EwTile), 256) + 256 * n;  // per-chunk alignment slack
  t.gemm = align_up(gemm, 256) + (size_t)n * 16 * 256;
  t.total = t.mats + t.ptrs + t.scal + t.partials + t.ew_tiles + t.gemm;
  return t;
}

// Consecutive matrices per chunk, never more than `cap` bytes of temporaries in one (a single matrix always fits).
int count_chunks(const std::vector<MatPlan>& mats, size_t cap) {
  int chunks = 1;
  size_t used = 0;
  for (const MatPlan& q : mats) {
    if (used > 0 && used + q.ns_bytes > cap) {
      ++chunks;
      used = 0;
    }
    used += q.ns_bytes;
  }
  return chunks;
}

}  // namespace

bool on_matrix_cores(int ns_dtype) { return ns_dtype != MUON_F32; }
int planes_of(int ns_dtype) { return ns_dtype == MUON_BF16X2 ? 2 : ns_dtype == MUON_BF16X3 ? 3 : 1; }
// bf16 path, m >= 64: the a*X term of Eq. 2 is folded into the polynomial, B' = b A + c A A + a I, so that the apply
// product X' = B' X needs no addend (a third of its epilogue's memory traffic).  B's diagonal is rounded to bf16
// once either way; for tiny matrices, where the diagonal carries most of the product, the explicit addend is kept.
// The split forms keep the explicit addend: folded into B's diagonal it would be rounded at the diagonal's magnitude
// (a = 3.44), not the iterate's.
bool folds_identity(const MatPlan& q, int ns_dtype) { return ns_dtype == MUON_BF16 && q.m >= 64; }

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

int plan_workspace_bytes(const muon_param* shapes, int32_t n, int32_t ns_dtype, size_t max_bytes, size_t* out) {
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

int plan_build(Plan& plan, const muon_param* shapes, int32_t n, int32_t ns_dtype, uintptr_t ws_base, size_t workspace_bytes) {
  int st = validate_shapes(shapes, n, ns_dtype);
  if (st != MUON_OK) return st;
  plan = Plan{};
  plan.n = n;
  plan.ns_dtype = ns_dtype;
  size_t total_partials = 0;
  plan_matrices(shapes, n, ns_dtype, plan.mats, total_partials);
  const TableLayout tl = table_layout(plan.mats, total_partials);

  size_t biggest = 0;
  for (const MatPlan& q : plan.mats) biggest = std::max(biggest, q.ns_bytes);
  if (workspace_bytes < tl.total + biggest) return MUON_E_WORKSPACE_TOO_SMALL;
  const size_t ns_budget = workspace_bytes - tl.total;

  // ---- chunking: consecutive matrices while their temporaries fit.  The number of chunks is what the budget
  // forces; the cut positions then come from the smallest cap that still gives that number, so that the chunks carry
  // about equal work instead of leaving a short last one (every chunk's launches end in a tail). ----
  {
    const int want = count_chunks(plan.mats, ns_budget);
    size_t lo = biggest, hi = ns_budget;     // count_chunks(hi) == want; find the smallest cap with that property
    while (lo < hi) {
      const size_t mid = lo + (hi - lo) / 2;
      if (count_chunks(plan.mats, mid) <= want) hi = mid;
      else lo = mid + 1;
    }
    const size_t cap = hi;
    size_t used = 0;
    Chunk cur{};
    for (int i = 0; i < n; ++i) {
      if (cur.count > 0 && used + plan.mats[i].ns_bytes > cap) {
        plan.chunks.push_back(cur);
        cur = Chunk{};
        cur.first = i;
        used = 0;
      }
      plan.mats[i].chunk = (int)plan.chunks.size();
      used += plan.mats[i].ns_bytes;
      cur.count++;
    }
    plan.chunks.push_back(cur);
  }

  // ---- host image of the table region ----
  std::vector<unsigned char> img(tl.total, 0);
  size_t off = 0;
  const size_t off_mats = off; off += tl.mats;
  const size_t off_ptrs = off; off += tl.ptrs;
  const size_t off_scal = off; off += tl.scal;
  const size_t off_part = off; off += tl.partials;
  size_t cursor = off;   // ew tiles and gemm tables are appended from here
  unsigned char* const ws = reinterpret_cast<unsigned char*>(ws_base);   // address arithmetic only, never dereferenced
  unsigned char* ns_base = ws + tl.total;
  const bool mc = on_matrix_cores(ns_dtype);
  const size_t es = mc ? 2 : 4;
  const size_t planes = (size_t)planes_of(ns_dtype);

  MatDesc* h_mats = reinterpret_cast<MatDesc*>(img.data() + off_mats);
  auto dev = [&](size_t o) { return ws + o; };

  for (Chunk& ch : plan.chunks) {
    size_t ns_off = 0;
    for (int i = ch.first; i < ch.first + ch.count; ++i) {
      const MatPlan& q = plan.mats[i];
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
        const MatPlan& q = plan.mats[i];
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
      Group g{};
      g.n_prob = (int)members.size();
      g.members = members;
      const size_t np_ = members.size();
      auto take = [&](size_t bytes) {
        cursor = align_up(cursor, 256);
        const size_t o = cursor;
        cursor += bytes;
        return o;
      };
      for (int v = 0; v < 2; ++v) g.prob_gram[v] = take(sizeof(GemmProblem) * np_);
      g.prob_poly = take(sizeof(GemmProblem) * np_);
      for (int v = 0; v < 4; ++v) g.prob_apply[v] = take(sizeof(GemmProblem) * np_);
      for (size_t k = 0; k < np_; ++k) {
        const MatPlan& q = plan.mats[members[k]];
        const MatDesc& d = h_mats[members[k]];
        GemmProblem gp{};
        gp.scal = d.scal;
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
      // Launch order of the problems, longest K loop first (the tail of a launch is then made of short tiles):
      // the Gram product runs over n, the other two over m.
      std::vector<int> by_n(np_), by_m(np_);
      std::iota(by_n.begin(), by_n.end(), 0);
      std::iota(by_m.begin(), by_m.end(), 0);
      std::stable_sort(by_n.begin(), by_n.end(), [&](int x, int y) {
        const MatPlan &a = plan.mats[members[x]], &b = plan.mats[members[y]];
        return a.np != b.np ? a.np > b.np : a.mp > b.mp;
      });
      std::stable_sort(by_m.begin(), by_m.end(), [&](int x, int y) {
        const MatPlan &a = plan.mats[members[x]], &b = plan.mats[members[y]];
        return a.mp != b.mp ? a.mp > b.mp : a.np > b.np;
      });
      std::vector<int64_t> w_n(np_), w_m(np_);
      for (size_t k = 0; k < np_; ++k) {
        w_n[k] = plan.mats[members[k]].np;
        w_m[k] = plan.mats[members[k]].mp;
      }
      // tile tables: level 1 = 256 x 256 tiles and 512 x 128 strip tiles (matrix cores only), level 0 = what they
      // leave uncovered, in fine tiles
      // uniform: every tile of the Gram product (n) / of the other two products (m) runs the same K.  steady: the
      // longest K is at most 1.5 times the shortest - such launches run persistent blocks with the planner's static,
      // cost-balanced assignment (measured: 27-layer MoE list, K = 1408 and 2048 mixed, polynomial launches -7 %);
      // with a wider spread the hardware's dynamic dispatch of one block per tile does better (K = 4096 and 11008
      // mixed: persistent +7 %).
      bool uniform_n = true, uniform_m = true;
      int64_t lo_n = w_n[0], hi_n = w_n[0], lo_m = w_m[0], hi_m = w_m[0];
      for (size_t k = 0; k < np_; ++k) {
        if (w_n[k] != w_n[0]) uniform_n = false;
        if (w_m[k] != w_m[0]) uniform_m = false;
        lo_n = std::min(lo_n, w_n[k]); hi_n = std::max(hi_n, w_n[k]);
        lo_m = std::min(lo_m, w_m[k]); hi_m = std::max(hi_m, w_m[k]);
      }
      const bool steady_n = 2 * hi_n <= 3 * lo_n, steady_m = 2 * hi_m <= 3 * lo_m;
      std::vector<std::vector<GemmTile>> moved_sym(np_), moved_app(np_);   // coarse tiles handed to the fine level
      for (int level = 1; level >= 0; --level) {
        if (level == 1 && !mc) continue;
        std::vector<std::vector<GemmTile>> sym(np_), app(np_);
        std::vector<std::vector<int>> sym_cuts(np_), app_cuts(np_);
        size_t n_sym = 0, n_app = 0;
        bool strips = false;
        for (size_t k = 0; k < np_; ++k) {
          const MatPlan& q = plan.mats[members[k]];
          const int cm = mc ? q.mp / kCoarse : 0, cn = mc ? q.np / kCoarse : 0;
          const int tm = q.mp / q.tile, tn = q.np / q.tile, r = kCoarse / q.tile;
          const int strip_h = kShapeRows[kShape512x128];
          // the 128 columns an odd multiple of 128 leaves beside the 256-tiles go to 512 x 128 tiles where the
          // output is at least 512 rows high
          const bool odd_m = mc && (q.mp % kCoarse) != 0;
          const bool sym_strip = odd_m && q.mp >= strip_h, app_strip = odd_m && q.np >= strip_h;
          if (level == 1) {
            // plain bf16: a diagonal tile is computed from its upper triangle of 32 x 32 blocks (9/16 of the MFMAs)
            blocked_tiles((int32_t)k, kCoarse, kShape256, cm, cm, true, 0, 0, -1, sym[k], sym_cuts[k], 4, 8,
                          ns_dtype == MUON_BF16 ? (int)kShape256Diag : -1);
            if (sym_strip) strip_tiles((int32_t)k, q.mp, q.mp - q.tile, sym[k], sym_cuts[k]);
            // tiles of X'^T in 8 x 2 blocks: measured against 8 x 4, 4 x 8, 16 x 2 and whole-width blocks, 0.7 % (4096-wide
            // block) to 1.5 % (MoE shapes) faster than 8 x 4, the next best (the K-major panels are the strided ones)
            blocked_tiles((int32_t)k, kCoarse, kShape256, cn, cm, false, 0, 0, -1, app[k], app_cuts[k], 8, 2);
            if (app_strip) strip_tiles((int32_t)k, q.np, q.mp - q.tile, app[k], app_cuts[k]);
            strips = strips || sym_strip || app_strip;
          } else {
            const int fine_shape = mc ? (int)kShape128 : 0;
            blocked_tiles((int32_t)k, q.tile, fine_shape, tm, tm, true, cm * r, cm * r, sym_strip ? tm - 1 : -1, sym[k], sym_cuts[k]);
            if (mc) blocked_tiles((int32_t)k, q.tile, fine_shape, tn, tm, false, cn * r, cm * r, app_strip ? tm - 1 : -1, app[k], app_cuts[k], 8, 4);
            else blocked_tiles((int32_t)k, q.tile, fine_shape, tm, tn, false, 0, 0, -1, app[k], app_cuts[k]);
            // the coarse tiles moved here: four fine tiles each (never a diagonal tile, so none of the four is one)
            for (int which = 0; which < 2; ++which) {
              const std::vector<GemmTile>& mv = which ? moved_app[k] : moved_sym[k];
              std::vector<GemmTile>& dst = which ? app[k] : sym[k];
              std::vector<int>& dcuts = which ? app_cuts[k] : sym_cuts[k];
              for (const GemmTile& t : mv) {
                for (int dr = 0; dr < r; ++dr)
                  for (int dc = 0; dc < r; ++dc)
                    dst.push_back(make_tile((int32_t)k, t.r0 * kTileUnit + dr * q.tile, t.c0 * kTileUnit + dc * q.tile, fine_shape, 0));
                dcuts.push_back((int)dst.size());
              }
            }
          }
        }
        if (level == 1) {
          // launches whose tiles all run the same K are persistent: even out their last round
          if (uniform_n && uniform_m) move_tail_to_fine(by_n, sym, sym_cuts, plan.coarse_blocks, moved_sym);
          if (uniform_m) move_tail_to_fine(by_m, app, app_cuts, plan.coarse_blocks, moved_app);
        }
        for (size_t k = 0; k < np_; ++k) {
          n_sym += sym[k].size();
          n_app += app[k].size();
        }
        TileSet& ts = level ? g.coarse : g.fine;
        ts.strips = strips;
        ts.persistent_n = steady_n;
        ts.persistent_m = steady_m;
        ts.sym = take(n_sym * sizeof(GemmTile));
        ts.poly = take(n_sym * sizeof(GemmTile));
        ts.apply = take(n_app * sizeof(GemmTile));
        ts.apply_last = take(n_app * sizeof(GemmTile));
        // The two symmetric products run the same tiles but not the same K (n for the Gram product, m for the
        // polynomial), so each gets its own table: dealt longest K first and weighted by its own K, and with the costs
        // evened out over a die's blocks where its launch is persistent (where the hardware hands out the blocks the
        // plain order measured better).
        const int slots = level == 1 ? plan.coarse_blocks / kXcds : 0;
        ts.n_sym = (int)deal_tiles(by_n, sym, sym_cuts, w_n, reinterpret_cast<GemmTile*>(img.data() + ts.sym), steady_n ? slots : 0);
        ts.n_poly = (int)deal_tiles(by_m, sym, sym_cuts, w_m, reinterpret_cast<GemmTile*>(img.data() + ts.poly), steady_m ? slots : 0);
        ts.n_apply = (int)deal_tiles(by_m, app, app_cuts, w_m, reinterpret_cast<GemmTile*>(img.data() + ts.apply), steady_m ? slots : 0);
        ts.n_apply_last = (int)deal_tiles(by_m, app, app_cuts, w_m, reinterpret_cast<GemmTile*>(img.data() + ts.apply_last), steady_m ? slots : 0);
      }
      ch.groups.push_back(g);
    }
  }
  if (cursor > tl.total) return MUON_E_WORKSPACE_TOO_SMALL;   // the layout bound is conservative; this cannot happen
  img.resize(cursor);
  plan.image.swap(img);
  plan.off_mats = off_mats;
  plan.off_ptrs = off_ptrs;
  return MUON_OK;
}

int64_t plan_tiles(const Plan& plan, int chunk, int product, int level, int32_t* out, int32_t cap_records) {
  int64_t total = 0;
  const bool mc = on_matrix_cores(plan.ns_dtype);
  for (const Group& g : plan.chunks[chunk].groups) {
    const TileSet& ts = level ? g.coarse : g.fine;
    const size_t off = product == 0 ? ts.sym : product == 1 ? ts.poly : product == 2 ? ts.apply : ts.apply_last;
    const int count = product == 0 ? ts.n_sym : product == 1 ? ts.n_poly : product == 2 ? ts.n_apply : ts.n_apply_last;
    const GemmTile* t = reinterpret_cast<const GemmTile*>(plan.image.data() + off);
    for (int i = 0; i < count; ++i, ++total) {
      if (total >= cap_records) continue;
      int32_t* r = out + 6 * total;
      r[0] = g.members[t[i].prob];
      r[1] = t[i].r0 * kTileUnit;
      r[2] = t[i].c0 * kTileUnit;
      r[3] = mc ? kShapeRows[t[i].shape] : kF32Tile;
      r[4] = mc ? kShapeCols[t[i].shape] : kF32Tile;
      // 32 x 32 blocks of the tile that are computed: all of them, except for the diagonal shape (upper triangle)
      r[5] = mc && t[i].shape == kShape256Diag ? 36 : r[3] / 32 * (r[4] / 32);
    }
  }
  return total;
}

}  // namespace muon
