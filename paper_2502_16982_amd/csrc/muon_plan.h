// Host-side launch planner of the Muon step: plain C++, no HIP include, so that it also builds with the host
// compiler alone (the sanitizer build of the tests does that).
//
// A plan turns a list of matrix shapes into: the orientation and padded extents of every matrix, the chunking of
// the list against the workspace, and the host image of the device tables (matrix records, elementwise tiles, one
// grouped-GEMM problem table and tile table per Newton-Schulz product).  Pointers inside the image are computed from
// the workspace base address and never followed on the host.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/muon.h"
#include "muon_tables.h"

namespace muon {

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

// Tile tables of one launch level (byte offsets in the table region).
struct TileSet {
  size_t sym = 0, poly = 0, apply = 0, apply_last = 0;     // Gram, polynomial, apply, last apply
  int n_sym = 0, n_poly = 0, n_apply = 0, n_apply_last = 0;
  bool strips = false;    // the tables hold 512 x 128 tiles (the launch then needs the larger LDS allocation)
  // the K loops of the launch's tiles are of nearly the same length (Gram product: n_pad; the other two: m_pad), so
  // the launch runs persistent blocks that take the planner's static assignment of tiles
  bool persistent_n = false, persistent_m = false;
};

// Launch group: all matrices of one chunk.  Each product is one launch per level: the coarse launch (matrix-core
// paths only) runs 256 x 256 tiles over the part of every output that whole such tiles cover plus 512 x 128 tiles
// over the 128-wide column strip an odd multiple of 128 leaves; the fine launch (128 x 128 bf16, 64 x 64 fp32) takes
// what remains, so that nothing is padded beyond the fine tile.
struct Group {
  int n_prob = 0;
  std::vector<int> members;                       // problem index -> matrix index in the caller's list
  size_t prob_gram[2] = {0, 0}, prob_poly = 0, prob_apply[4] = {0, 0, 0, 0};  // byte offsets ([parity], [parity * 2 + last])
  TileSet fine, coarse;
};

struct Chunk {
  int first = 0, count = 0;
  size_t ew_tiles_off = 0;   // byte offset of the EwTile table
  int n_ew_tiles = 0;
  std::vector<Group> groups;
};

struct Plan {
  int n = 0;
  int ns_dtype = MUON_BF16;
  std::vector<MatPlan> mats;
  std::vector<Chunk> chunks;
  std::vector<unsigned char> image;   // host image of the table region (what muon_init uploads)
  size_t off_mats = 0, off_ptrs = 0;  // byte offsets of the matrix records and of the per-step pointer table
  int coarse_blocks = 256;            // blocks of a persistent coarse launch (compute units of the device); set before plan_build
};

constexpr int kCoarse = 256;          // block tile of the large bf16 kernel
constexpr int64_t kMaxDim = 1 << 20;  // tile offsets are 16-bit in units of 64 elements

bool on_matrix_cores(int ns_dtype);
int planes_of(int ns_dtype);
bool folds_identity(const MatPlan& q, int ns_dtype);

// MUON_OK or the status muon_init would return for this list.
int validate_shapes(const muon_param* p, int32_t n, int32_t ns_dtype);

// Bytes to allocate for a list (see muon_workspace_bytes).  May throw std::bad_alloc.
int plan_workspace_bytes(const muon_param* shapes, int32_t n, int32_t ns_dtype, size_t max_bytes, size_t* out);

// Builds the plan for a workspace at address `ws_base` of `ws_bytes` bytes.  Returns MUON_OK,
// MUON_E_WORKSPACE_TOO_SMALL or a validation status.  May throw std::bad_alloc.
int plan_build(Plan& out, const muon_param* shapes, int32_t n, int32_t ns_dtype, uintptr_t ws_base, size_t ws_bytes);

// Tile table of one grouped launch as records {matrix, first row, first column, rows, columns (in elements),
// computed 32 x 32 blocks}
// (see muon_plan_tiles).  Returns the number of records of the table.
int64_t plan_tiles(const Plan& plan, int chunk, int product, int level, int32_t* out, int32_t cap_records);

}  // namespace muon
