// Device-visible tables shared by the host planner and the HIP kernels of the Muon step.
// Plain-old-data only; every pointer is a device pointer into caller memory or the workspace.
#pragma once
#include <stdint.h>

namespace muon {

constexpr int kEwTile = 64;        // elementwise kernels work on 64x64 element tiles
constexpr int kDtypeF32 = 0;
constexpr int kDtypeBF16 = 1;
constexpr int kDtypeBF16X2 = 2;    // Newton-Schulz storage only: sum of two bf16 planes
constexpr int kDtypeBF16X3 = 3;    // Newton-Schulz storage only: sum of three bf16 planes

// Static per-matrix record (built once at init).
struct MatDesc {
  void* X;            // m_pad x n_pad, row-major, NS dtype: the iterate in "rows <= cols" orientation
  void* Xt[2];        // fp32 path: n_pad x m_pad, the iterate's transpose, ping-pong pair.  bf16 path (one layout of
                      // the iterate): Xt[0] is the second m_pad x n_pad buffer of the X ping-pong (and receives U in
                      // W's orientation when no iteration runs), Xt[1] receives O as n_pad x m_pad for matrices that
                      // are iterated on their transpose
  void* Ag;           // m_pad x m_pad: Gram matrix X X^T
  void* Bp;           // m_pad x m_pad: b*A + c*A*A
  float* partials;    // one partial sum of squares per 64x64 tile
  float* scal;        // [0] = 1/(||U||_F + eps), [1] = its square, [2] = sum(O^2) scratch, [3] spare
  int32_t rows, cols; // A, B
  int32_t m, n;       // min, max
  int32_t mp, np;     // padded to the GEMM tile
  int32_t transposed; // A > B: NS runs on U^T
  int32_t w_dtype, g_dtype;
  int32_t n_part;     // number of partials
  int32_t ew_tiles_c; // 64-wide tile columns in U's orientation (padded)
  float sqrt_max;     // sqrt(max(A, B))
  int32_t pad_;
  int64_t x_plane;    // split-bf16 path: elements from one bf16 plane of X / Xt[] to the next (0 otherwise)
};

// Per-step pointers (re-uploaded only when they change).
struct MatPtrs {
  void* w;
  const void* g;
  float* m;
};

// One work item of an elementwise pass: `count` consecutive 64x64 tiles of one tile row.
constexpr int kEwRun = 4;          // tiles per work item (amortises the table look-ups of a block)
struct EwTile {
  int32_t mat;        // absolute matrix index (into MatDesc / MatPtrs)
  int16_t tr, tc;     // tile row / first tile column in U's (= W's) orientation
  int16_t count;      // 1 .. kEwRun
  int16_t pad_;
};

// One product  C[i][j] = sum_k L[i][k] * R[j][k]  ("NT": both operands contiguous along k),
// followed by  val = alpha * (beta_acc * acc + beta_e * E[i][j]) (+ d on the matrix diagonal when diag_add is set;
// d is a launch argument)  and stores of C and/or its transpose.
// The bf16 kernel writes Ct straight from the accumulator layout and C through one extra MFMA transpose,
// so single-output problems are posed with Ct as the output.
struct GemmProblem {
  const void* L;      // M x K, leading dimension ldl (K-major launches: element (i, k) at L[k * ldl + i])
  const void* R;      // N x K, leading dimension ldr
  const void* E;      // M x N addend at the output position (may be null), leading dimension lde
  const void* Et;     // the same addend stored transposed, N x M, leading dimension ldet (bf16 kernel reads this one)
  void* C;            // M x N output (may be null), leading dimension ldc
  void* Ct;           // N x M transposed output, leading dimension ldct (the bf16 kernel requires it unless symmetric)
  const float* scal;  // per-matrix scalars (alpha source)
  int32_t K;
  int32_t ldl, ldr, lde, ldet, ldc, ldct;
  int32_t symmetric;  // output is symmetric: off-diagonal tiles are also stored mirrored into C
  int32_t diag_add;   // square output only: add the launch's diagonal constant to C[i][i] before rounding
  // split-bf16 launches (every matrix = sum of several bf16 planes): elements from one plane to the next
  int64_t l_plane, r_plane, et_plane, c_plane, ct_plane;
};

// One block's output tile.  Rows and columns are counted in units of kTileUnit elements, so that tiles of several
// block shapes (and tiles shifted to end at the matrix edge) share one table format.
constexpr int kTileUnit = 64;
// Block-tile shapes of the bf16 matrix-core kernel (the fp32 kernel has one 64 x 64 shape and ignores the field).
// kShape256Diag: a 256 x 256 tile on the diagonal of a symmetric product (plain bf16 only), computed from its upper
// triangle of 32 x 32 blocks.
enum GemmShape : int { kShape128 = 0, kShape256 = 1, kShape512x128 = 2, kShape256Diag = 3, kNumShapes = 4 };
constexpr int kShapeRows[kNumShapes] = {128, 256, 512, 256};
constexpr int kShapeCols[kNumShapes] = {128, 256, 128, 256};
constexpr int kF32Tile = 64;       // block tile of the fp32 Newton-Schulz GEMM
constexpr int kTileDiagonal = 1;   // GemmTile::flags: tile on the diagonal of a symmetric product: it is its own mirror
                                   // image, so only one of the two stores is made
struct GemmTile {
  int32_t prob;
  uint16_t r0, c0;    // first output row / column, in units of kTileUnit
  uint8_t shape;      // GemmShape
  uint8_t flags;      // kTileDiagonal
  uint16_t pad_;
};

}  // namespace muon
