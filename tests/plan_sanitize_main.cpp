// Sanitizer driver for the host-side launch planner: built by tests/test_plan_sanitized.py with
//   g++ -fsanitize=address,undefined  paper_2502_16982_amd/csrc/muon_plan.cpp  tests/plan_sanitize_main.cpp
// (no HIP involved).  It plans shape lists at several workspace budgets and in every arithmetic, walks every table
// of the resulting image the way the kernels would, and checks that all indices, offsets and device addresses stay
// inside what they index.  Any sanitizer report or failed check ends the process with a non-zero status.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../paper_2502_16982_amd/csrc/muon_plan.h"

using namespace muon;

static int failures = 0;
#define CHECK(cond)                                                           \
  do {                                                                        \
    if (!(cond)) {                                                            \
      std::fprintf(stderr, "CHECK failed %s:%d: %s\n", __FILE__, __LINE__, #cond); \
      ++failures;                                                             \
    }                                                                         \
  } while (0)

static std::vector<muon_param> params_of(const std::vector<std::pair<int64_t, int64_t>>& shapes) {
  std::vector<muon_param> p(shapes.size());
  for (size_t i = 0; i < shapes.size(); ++i) {
    std::memset(&p[i], 0, sizeof(muon_param));
    p[i].rows = shapes[i].first;
    p[i].cols = shapes[i].second;
    p[i].w_dtype = (i % 2) ? MUON_F32 : MUON_BF16;
    p[i].g_dtype = (i % 3) ? MUON_BF16 : MUON_F32;
  }
  return p;
}

static void walk(const Plan& plan, uintptr_t base, size_t ws_bytes) {
  const unsigned char* img = plan.image.data();
  const size_t img_bytes = plan.image.size();
  const bool mc = on_matrix_cores(plan.ns_dtype);
  const size_t es = mc ? 2 : 4, planes = (size_t)planes_of(plan.ns_dtype);
  CHECK(plan.off_mats + sizeof(MatDesc) * (size_t)plan.n <= img_bytes);
  CHECK(plan.off_ptrs + sizeof(MatPtrs) * (size_t)plan.n <= img_bytes);
  const MatDesc* mats = reinterpret_cast<const MatDesc*>(img + plan.off_mats);
  auto inside = [&](const void* ptr, size_t bytes) {
    const uintptr_t a = reinterpret_cast<uintptr_t>(ptr);
    return a >= base && a + bytes <= base + ws_bytes;
  };
  std::vector<int> seen(plan.n, 0);
  int next = 0;
  for (size_t ci = 0; ci < plan.chunks.size(); ++ci) {
    const Chunk& ch = plan.chunks[ci];
    CHECK(ch.first == next && ch.count >= 1);
    next = ch.first + ch.count;
    for (int i = ch.first; i < ch.first + ch.count; ++i) {
      const MatDesc& d = mats[i];
      const MatPlan& q = plan.mats[i];
      CHECK(q.chunk == (int)ci);
      CHECK(d.mp % q.tile == 0 && d.np % q.tile == 0 && d.mp >= d.m && d.np >= d.n && d.m <= d.n);
      const size_t xb = es * (size_t)d.mp * d.np * planes, ab = es * (size_t)d.mp * d.mp * planes;
      CHECK(inside(d.X, xb) && inside(d.Xt[0], xb) && inside(d.Ag, ab) && inside(d.Bp, ab));
      CHECK(d.Xt[1] == nullptr || inside(d.Xt[1], xb));
      CHECK(inside(d.partials, sizeof(float) * (size_t)d.n_part) && inside(d.scal, 4 * sizeof(float)));
      // temporaries lie behind the tables
      CHECK(reinterpret_cast<uintptr_t>(d.X) >= base + img_bytes);
    }
    // elementwise tiles
    CHECK(ch.ew_tiles_off + sizeof(EwTile) * (size_t)ch.n_ew_tiles <= img_bytes);
    const EwTile* ew = reinterpret_cast<const EwTile*>(img + ch.ew_tiles_off);
    for (int t = 0; t < ch.n_ew_tiles; ++t) {
      CHECK(ew[t].mat >= ch.first && ew[t].mat < ch.first + ch.count);
      const MatPlan& q = plan.mats[ew[t].mat];
      CHECK(ew[t].tr >= 0 && ew[t].tr < q.ew_tr && ew[t].tc >= 0 && ew[t].count >= 1 && ew[t].count <= kEwRun &&
            ew[t].tc + ew[t].count <= q.ew_tc);
      seen[ew[t].mat] += ew[t].count;
    }
    for (const Group& g : ch.groups) {
      CHECK((int)g.members.size() == g.n_prob);
      const size_t pb = sizeof(GemmProblem) * (size_t)g.n_prob;
      CHECK(g.prob_gram[0] + pb <= img_bytes && g.prob_gram[1] + pb <= img_bytes && g.prob_poly + pb <= img_bytes);
      for (int v = 0; v < 4; ++v) CHECK(g.prob_apply[v] + pb <= img_bytes);
      for (int level = 0; level < 2; ++level) {
        const TileSet& ts = level ? g.coarse : g.fine;
        const size_t offs[3] = {ts.sym, ts.apply, ts.apply_last};
        const int counts[3] = {ts.n_sym, ts.n_apply, ts.n_apply_last};
        for (int w = 0; w < 3; ++w) {
          CHECK(offs[w] + sizeof(GemmTile) * (size_t)counts[w] <= img_bytes);
          const GemmTile* tiles = reinterpret_cast<const GemmTile*>(img + offs[w]);
          // per problem: every cell of the output covered
          std::vector<std::vector<unsigned char>> cover(g.n_prob);
          for (int t = 0; t < counts[w]; ++t) {
            const GemmTile& gt = tiles[t];
            CHECK(gt.prob >= 0 && gt.prob < g.n_prob);
            if (gt.prob < 0 || gt.prob >= g.n_prob) continue;
            const MatPlan& q = plan.mats[g.members[gt.prob]];
            CHECK(mc ? gt.shape < kNumShapes : gt.shape == 0);
            if (mc && gt.shape >= kNumShapes) continue;
            CHECK(mc ? ((level == 0) == (gt.shape == kShape128)) : level == 0);
            if (gt.shape == kShape512x128) CHECK(ts.strips);
            const int rows = mc ? kShapeRows[gt.shape] : kF32Tile, cols = mc ? kShapeCols[gt.shape] : kF32Tile;
            const int out_r = w == 0 ? q.mp : (mc ? q.np : q.mp), out_c = w == 0 ? q.mp : (mc ? q.mp : q.np);
            const int r0 = gt.r0 * kTileUnit, c0 = gt.c0 * kTileUnit;
            CHECK(r0 + rows <= out_r && c0 + cols <= out_c);
            if (r0 + rows > out_r || c0 + cols > out_c) continue;
            if (w == 0) CHECK(((gt.flags & kTileDiagonal) != 0) == (r0 == c0 && rows == cols));
            std::vector<unsigned char>& cv = cover[gt.prob];
            const int gr = out_r / q.tile, gc = out_c / q.tile;
            if (cv.empty()) cv.assign((size_t)gr * gc, 0);
            for (int i = r0 / q.tile; i < (r0 + rows) / q.tile; ++i)
              for (int j = c0 / q.tile; j < (c0 + cols) / q.tile; ++j) cv[(size_t)i * gc + j] = 1;
          }
          (void)cover;
        }
      }
      // both levels together cover every output cell (upper triangle for the symmetric products)
      for (int w = 0; w < 2; ++w) {
        for (int k = 0; k < g.n_prob; ++k) {
          const MatPlan& q = plan.mats[g.members[k]];
          const int out_r = w == 0 ? q.mp : (mc ? q.np : q.mp), out_c = w == 0 ? q.mp : (mc ? q.mp : q.np);
          const int gr = out_r / q.tile, gc = out_c / q.tile;
          if ((int64_t)gr * gc > (1 << 22)) continue;   // the 2^20-wide cases: bounds were checked above
          std::vector<unsigned char> cv((size_t)gr * gc, 0);
          for (int level = 0; level < 2; ++level) {
            const TileSet& ts = level ? g.coarse : g.fine;
            const GemmTile* tiles = reinterpret_cast<const GemmTile*>(img + (w == 0 ? ts.sym : ts.apply));
            const int count = w == 0 ? ts.n_sym : ts.n_apply;
            for (int t = 0; t < count; ++t) {
              if (tiles[t].prob != k) continue;
              const int rows = mc ? kShapeRows[tiles[t].shape] : kF32Tile, cols = mc ? kShapeCols[tiles[t].shape] : kF32Tile;
              const int r0 = tiles[t].r0 * kTileUnit, c0 = tiles[t].c0 * kTileUnit;
              for (int i = r0 / q.tile; i < (r0 + rows) / q.tile && i < gr; ++i)
                for (int j = c0 / q.tile; j < (c0 + cols) / q.tile && j < gc; ++j) cv[(size_t)i * gc + j] = 1;
            }
          }
          for (int i = 0; i < gr; ++i)
            for (int j = (w == 0 ? i : 0); j < gc; ++j) CHECK(cv[(size_t)i * gc + j] == 1);
        }
      }
    }
  }
  CHECK(next == plan.n);
  for (int i = 0; i < plan.n; ++i) CHECK(seen[i] == plan.mats[i].ew_tr * plan.mats[i].ew_tc);
}

int main() {
  typedef std::vector<std::pair<int64_t, int64_t>> Shapes;
  std::vector<Shapes> lists;
  lists.push_back({{1, 1}, {1, 9}, {5, 3}, {64, 64}, {130, 130}, {200, 333}, {333, 200}, {257, 511}, {384, 128}, {128, 640}});
  lists.push_back({{1024, 1024}, {1024, 1536}, {1280, 1024}, {384, 640}, {640, 1152}, {640, 640}, {896, 1664}});
  lists.push_back({{4096, 4096}, {4096, 11008}, {11008, 4096}});
  lists.push_back({{4, 1 << 20}, {1 << 20, 4}, {1, 70000}});
  {
    Shapes moe;                       // one layer of the 64 + 2 expert model plus its attention projections
    for (int e = 0; e < 66; ++e) {
      moe.push_back({2048, 1408});
      moe.push_back({2048, 1408});
      moe.push_back({1408, 2048});
    }
    for (int a = 0; a < 4; ++a) moe.push_back({2048, 2048});
    lists.push_back(moe);
  }
  {
    Shapes rnd;                       // fixed pseudo-random shapes: multiples of 1, 64 and 128 up to 3000
    unsigned s = 12345u;
    auto next = [&]() { s = s * 1664525u + 1013904223u; return s >> 8; };
    for (int i = 0; i < 60; ++i) {
      const int g = i % 3 == 0 ? 1 : (i % 3 == 1 ? 64 : 128);
      rnd.push_back({(int64_t)(1 + next() % (3000 / g)) * g, (int64_t)(1 + next() % (3000 / g)) * g});
    }
    lists.push_back(rnd);
  }
  const int dtypes[4] = {MUON_BF16, MUON_BF16X2, MUON_BF16X3, MUON_F32};
  int plans = 0;
  for (const Shapes& shapes : lists) {
    const std::vector<muon_param> p = params_of(shapes);
    const int n = (int)p.size();
    for (int ns : dtypes) {
      size_t all = 0, least = 0;
      CHECK(plan_workspace_bytes(p.data(), n, ns, 0, &all) == MUON_OK);
      CHECK(plan_workspace_bytes(p.data(), n, ns, 1, &least) == MUON_OK);
      CHECK(least <= all);
      const size_t budgets[3] = {all, least, least + (all - least) / 3};
      for (size_t ws_bytes : budgets) {
        Plan plan;
        const uintptr_t base = uintptr_t{1} << 40;
        const int st = plan_build(plan, p.data(), n, ns, base, ws_bytes);
        CHECK(st == MUON_OK);
        if (st != MUON_OK) continue;
        walk(plan, base, ws_bytes);
        ++plans;
      }
      Plan small;
      CHECK(plan_build(small, p.data(), n, ns, uintptr_t{1} << 40, least - 4096) == MUON_E_WORKSPACE_TOO_SMALL);
    }
  }
  // rejected inputs
  {
    Plan plan;
    muon_param bad{};
    bad.rows = 0; bad.cols = 4; bad.w_dtype = MUON_BF16; bad.g_dtype = MUON_BF16;
    CHECK(plan_build(plan, &bad, 1, MUON_BF16, 1 << 20, 1 << 30) == MUON_E_INVALID_ARG);
    bad.rows = (1 << 20) + 1;
    CHECK(plan_build(plan, &bad, 1, MUON_BF16, 1 << 20, 1 << 30) == MUON_E_INVALID_ARG);
    bad.rows = 4; bad.w_dtype = 7;
    CHECK(plan_build(plan, &bad, 1, MUON_BF16, 1 << 20, 1 << 30) == MUON_E_UNSUPPORTED_DTYPE);
    bad.w_dtype = MUON_BF16;
    CHECK(plan_build(plan, &bad, 1, 9, 1 << 20, 1 << 30) == MUON_E_UNSUPPORTED_DTYPE);
    CHECK(plan_build(plan, nullptr, 1, MUON_BF16, 1 << 20, 1 << 30) == MUON_E_INVALID_ARG);
  }
  if (failures) {
    std::fprintf(stderr, "%d checks failed\n", failures);
    return 1;
  }
  std::printf("planner ok: %d plans walked\n", plans);
  return 0;
}
