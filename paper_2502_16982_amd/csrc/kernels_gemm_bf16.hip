// bf16 Newton-Schulz products for gfx950 (Eq. 2 of the paper): grouped GEMMs
//     T[i][j] = sum_k L[i][k] * R[j][k]          (bf16 operands, fp32 accumulation on the matrix cores)
// with a fused epilogue  val = alpha * (beta_acc * acc + beta_e * E[i][j]) (+ a constant on the diagonal), storing
// T^T (cheap: it is the accumulator layout) and/or T.  R is always contiguous along k; L either contiguous along k
// or K-major (element (i, k) at L[k * ldl + i]).  With ONE row-major copy of the iterate X (m x n):
//     Gram       A  = X X^T                L = R = X                   (symmetric output)
//     polynomial B' = b A + c A A + a I    L = R = A                   (A symmetric; the a X term of the apply
//                                                                       product travels in B's diagonal)
//     apply      T  = X'^T = X^T B'        L = X read K-major, R = B'  (stores T^T = X' row-major; T itself only
//                                                                       where O is wanted transposed)
// Operands are zero-padded to whole tiles by the producer, so the kernel has no edge handling.
// The same kernel also runs the split-bf16 forms (template parameter PL, see seg_count below): every matrix a sum of
// 2 or 3 bf16 planes, each product one K loop over the plane pairs that matter, the epilogue splitting the fp32
// result into planes again.
//
// Design for CDNA4:
//  * v_mfma_f32_32x32x16_bf16 (the 16x16x32 form runs at half the rate on this chip), wave tile = FM x FN
//    MFMA tiles, accumulators stay in registers for the whole K loop.
//  * K is consumed in 64-wide slabs, i.e. one 128-byte line per row: measured on this chip, the L1 hands a
//    compute unit ~57 B/clk when 8 lanes ask for a whole line and only ~26 B/clk for half lines.
//    Global memory -> LDS goes through the LDS-DMA path (global_load_lds_dwordx4): no staging registers, no
//    ds_write instructions.  A wave-level DMA instruction fills 1 KB of LDS contiguously (lane i -> byte 16*i),
//    i.e. 8 rows of 128 B; the 16-byte chunks of a row are XOR-swizzled by (row/2)%8 - each lane simply fetches
//    the global chunk that belongs in its slot - so that the 16 lanes served together by a ds_read_b128
//    fragment read hit 16 distinct bank groups (the bank-conflict counter reads zero).
//  * The LDS stages form a ring; a slab is requested one whole iteration (64 MFMAs per wave for the 256x256
//    tile) before it is needed.  One s_waitcnt + s_barrier per slab, placed in front of the last k-step so
//    that the next slab's first fragments are already being read while that k-step's MFMAs execute.
//  * Epilogue: the (transposed) addend tile is DMA-ed into LDS with coalesced 16-byte requests, each lane
//    combines it with its accumulators (fp32 math, one v_cvt_pk_bf16_f32 rounding), and results leave through
//    swizzled LDS images so that both the tile and its transpose are written with full 16-byte-per-lane
//    coalesced stores; the second orientation comes from a 2-MFMA transpose per 32x32 tile.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "muon_launch.h"

namespace muon {
namespace {

typedef unsigned short u16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef const __attribute__((address_space(1))) void* gptr;
typedef __attribute__((address_space(3))) void* lptr;
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16* lds_v4i16_ptr;
typedef __attribute__((address_space(1))) u32x4* gvec_ptr;   // 16-byte global store target (keeps the stores off the flat path)

constexpr int BK = 64;        // K slab in elements: one 128-byte line per row, the request size the L1 serves at full rate
constexpr int ROWB = 128;     // bytes per LDS row of a pipeline stage (BK bf16, unpadded, swizzled)

__device__ __forceinline__ float bf16_to_f32(u16 h) { return __uint_as_float(((unsigned)h) << 16); }
__device__ __forceinline__ u16 f32_to_bf16(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u16)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (u16)(u >> 16);
}

// s_waitcnt vmcnt(N), other counters untouched (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14])
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

template <int BM, int BN>
struct TileCfg {
  static constexpr size_t pipeline_bytes(int nstage) { return (size_t)nstage * (BM + BN) * ROWB; }
  static constexpr size_t image_bytes() { return (size_t)BM * BN * 2; }
  static constexpr size_t lds_main(int nstage) {
    return pipeline_bytes(nstage) > image_bytes() ? pipeline_bytes(nstage) : image_bytes();
  }
  static constexpr size_t lds_bytes(int nstage) { return lds_main(nstage); }
};

// f(integral_constant<int, I>) for I = FIRST .. LAST-1, unrolled at compile time
template <int FIRST, int LAST, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (FIRST < LAST) {
    f(std::integral_constant<int, FIRST>{});
    static_for<FIRST + 1, LAST>(f);
  }
}

// s_waitcnt lgkmcnt(0), vmcnt untouched: this wave's LDS reads have returned
__device__ __forceinline__ void wait_lgkm0() { __builtin_amdgcn_s_waitcnt(15 | (3 << 14) | (7 << 4) | (0 << 8)); }

// Hand-placed LDS waits whose covered registers are read-write operands of the wait itself (see the K-major path of
// the kernel): s_waitcnt lgkmcnt(CNT) "producing" the A-side fragment halves of one k-step, and empty statements that
// tie further registers to the same point.  An asm statement takes at most 30 operands, hence the split.
template <int CNT>
__device__ __forceinline__ void wait_lgkm_tie(u32x2 (&h)[4][2]) {
  asm volatile("s_waitcnt lgkmcnt(%8)"
               : "+v"(h[0][0]), "+v"(h[0][1]), "+v"(h[1][0]), "+v"(h[1][1]), "+v"(h[2][0]), "+v"(h[2][1]), "+v"(h[3][0]), "+v"(h[3][1])
               : "n"(CNT)
               : "memory");
}
template <int CNT>
__device__ __forceinline__ void wait_lgkm_tie(u32x2 (&h)[2][2]) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(h[0][0]), "+v"(h[0][1]), "+v"(h[1][0]), "+v"(h[1][1]) : "n"(CNT) : "memory");
}
__device__ __forceinline__ void tie_regs(u32x2 (&h)[4][2]) {
  asm volatile(""
               : "+v"(h[0][0]), "+v"(h[0][1]), "+v"(h[1][0]), "+v"(h[1][1]), "+v"(h[2][0]), "+v"(h[2][1]), "+v"(h[3][0]), "+v"(h[3][1])
               :
               : "memory");
}
__device__ __forceinline__ void tie_regs(u32x2 (&h)[2][2]) {
  asm volatile("" : "+v"(h[0][0]), "+v"(h[0][1]), "+v"(h[1][0]), "+v"(h[1][1]) : : "memory");
}
__device__ __forceinline__ void tie_regs(u32x4 (&b)[4]) {
  asm volatile("" : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]) : : "memory");
}
__device__ __forceinline__ void tie_regs(u32x4 (&b)[2]) { asm volatile("" : "+v"(b[0]), "+v"(b[1]) : : "memory"); }

// Split operands (PL > 1 planes): every matrix is the sum of PL bf16 arrays ("planes", plane q at element offset
// q * plane stride from the base pointer), each holding what the planes before it left of the fp32 value after
// rounding to bf16, i.e. about 2^-8 of its predecessor.  A product of two such sums is taken over the plane pairs
// (i, j) with i + j < PL - the pairs left out are below 2^(-8 PL) of the result - as ONE K loop over
// PL (PL + 1) / 2 segments that all accumulate into the same fp32 registers, smallest terms first.
constexpr int seg_count(int pl) { return pl * (pl + 1) / 2; }
// plane of the L (which = 0) or R (which = 1) operand in segment s: pairs by decreasing i + j, then decreasing i
constexpr int seg_plane(int pl, int s, int which) {
  int n = 0;
  for (int total = pl - 1; total >= 0; --total)
    for (int i = total; i >= 0; --i, ++n)
      if (n == s) return which == 0 ? i : total - i;
  return 0;
}

// LKM: the L operand is stored K-major (element (i, k) at L[k * ldl + i], i.e. the product is L^T-by-R^T of two
// row-major arrays); its MFMA fragments then come from LDS through the transposing read ds_read_b64_tr_b16.
// PL: number of bf16 planes per matrix (1: plain bf16).
__device__ __forceinline__ int thread_index(int wave_id) {
  unsigned zero = 0;
  asm volatile("" : "+v"(zero));                 // opaque, so that the lane count below is redone where it is used
  return (wave_id << 6) | (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, zero));
}

template <int BM, int BN, int WM_, int WN_, int NSTAGE, bool LKM, int PL>
__device__ __forceinline__ void gemm_tile_body(const GemmProblem& p, const GemmTile& tile, unsigned char* smem, float beta_acc,
                                               float beta_e, int alpha_idx, float diag_add, int wave_id) {
  constexpr int NW = WM_ * WN_, NT = NW * 64;
  constexpr int WTM = BM / WM_, WTN = BN / WN_;    // wave tile
  constexpr int FM = WTM / 32, FN = WTN / 32;      // 32x32 MFMA tiles per wave
  constexpr int LI = BM / 8 / NW, RI = BN / 8 / NW;     // DMA instructions per wave per slab (8 rows each)
  constexpr int NLOAD = LI + RI;
  constexpr int STAGE_B = (BM + BN) * ROWB;        // bytes per stage
  constexpr int KSTEPS = BK / 16;                  // MFMA k-steps per slab
  constexpr int NSEG = seg_count(PL);              // K-loop segments (plane pairs)
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0 && WTM % 32 == 0 && WTN % 32 == 0, "tile shape");
  static_assert(NW % 2 == 0 && NSTAGE == 2 && NLOAD < 32, "pipeline shape");
  static_assert(4 * FM == WTM / 8 && (WTM / 8 & (WTM / 8 - 1)) == 0 && BM / 8 >= 16, "slot addressing: 4i+q and wm*WTM/8 use disjoint bits");
  (void)NT;

  // The thread index is made opaque once per tile: everything below that derives from it (lane addresses, swizzle
  // keys) is then recomputed for every tile of a persistent block instead of being hoisted out of the tile loop, where
  // it would occupy registers for the whole kernel and push the epilogues into scratch.  It is put together from the
  // wave's number (a scalar the kernel keeps) and the lane's position, not taken from the register the hardware
  // delivers it in: that one does not survive a tile, and fetching a saved copy from scratch would mean waiting for
  // vector memory, i.e. for every store of the block's previous tile.
  int tid = thread_index(wave_id);
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN_, wn = wave % WN_;
  const int row0 = tile.r0 * kTileUnit, col0 = tile.c0 * kTileUnit;

  // ---- DMA addressing: a wave instruction fills 8 rows x 128 B; lane i -> slot (row i/8, chunk position i%8).
  // Position s of row R holds logical chunk s ^ ((R/2)%8); R = 8*(instruction index) + i/8 and the instruction
  // index has the parity of the wave number.
  const int dma_row = wave * 8 + (lane >> 3);
  const int dma_key = ((lane >> 4) & 3) + 4 * (wave & 1);
  const int dma_chunk = (lane & 7) ^ dma_key;
  // K-major L: a slab is 64 k-rows of BM elements; a wave instruction fills RPK whole k-rows; position s of k-row
  // R holds logical chunk s ^ 4*(R%4), which spreads the four k-rows a transposing read touches over the banks.
  constexpr int CPRK = BM / 8, RPK = 64 / CPRK;
  const int km_row = wave * RPK + lane / CPRK;
  const int km_chunk = (lane % CPRK) ^ (4 * (km_row & 3));
  const u16* lsrc = LKM ? static_cast<const u16*>(p.L) + (size_t)km_row * p.ldl + row0 + km_chunk * 8
                        : static_cast<const u16*>(p.L) + (size_t)(row0 + dma_row) * p.ldl + dma_chunk * 8;
  const u16* rsrc = static_cast<const u16*>(p.R) + (size_t)(col0 + dma_row) * p.ldr + dma_chunk * 8;
  const size_t lstep = (size_t)(LKM ? NW * RPK : 8 * NW) * p.ldl, rstep = (size_t)(8 * NW) * p.ldr;
  const size_t lslab = LKM ? (size_t)BK * p.ldl : (size_t)BK;      // elements from one K slab of L to the next
  const int KT1 = p.K / BK;                        // slabs per segment
  // requests DMA instructions [first, first + count) of slab kt (instructions 0..LI-1 fetch L rows, the rest R rows)
  auto request_part = [&](int kt, int stage, auto first_tag, auto count_tag) {
    constexpr int FIRST = decltype(first_tag)::value, COUNT = decltype(count_tag)::value;
    unsigned char* base = smem + stage * STAGE_B + wave * 1024;
    size_t loff, roff;                             // element offsets of slab kt in L and R (wave-uniform)
    if constexpr (PL == 1) {
      loff = (size_t)kt * lslab;
      roff = (size_t)kt * BK;
    } else {
      int seg = 0, kl = kt;
#pragma unroll
      for (int sgm = 1; sgm < NSEG; ++sgm)
        if (kt >= sgm * KT1) { seg = sgm; kl = kt - sgm * KT1; }
      int lpl = seg_plane(PL, 0, 0), rpl = seg_plane(PL, 0, 1);
#pragma unroll
      for (int sgm = 1; sgm < NSEG; ++sgm)
        if (seg == sgm) { lpl = seg_plane(PL, sgm, 0); rpl = seg_plane(PL, sgm, 1); }
      loff = (size_t)kl * lslab + (size_t)lpl * (size_t)p.l_plane;
      roff = (size_t)kl * BK + (size_t)rpl * (size_t)p.r_plane;
    }
#pragma unroll
    for (int n = FIRST; n < FIRST + COUNT; ++n) {
      if (n < LI)
        __builtin_amdgcn_global_load_lds((gptr)(lsrc + n * lstep + loff), (lptr)(base + n * NW * 1024), 16, 0, 0);
      else
        __builtin_amdgcn_global_load_lds((gptr)(rsrc + (n - LI) * rstep + roff),
                                         (lptr)(base + BM * ROWB + (n - LI) * NW * 1024), 16, 0, 0);
    }
  };
  using Zero = std::integral_constant<int, 0>;
  using AllN = std::integral_constant<int, NLOAD>;

  // ---- fragment addressing: lane (r = lane%32, h = lane/32) reads logical chunk 2*kk + h of its row ----
  const int fr = lane & 31, fh = lane >> 5;
  const int fkey = (fr >> 1) & 7;
  const int a_base = (wm * WTM + fr) * ROWB, b_base = BM * ROWB + (wn * WTN + fr) * ROWB;

  // The zero the accumulators start from is opaque to the compiler: a constant 16-register tuple would be hoisted
  // out of a persistent block's tile loop, find no register there and come back from scratch at every tile.
  float acc0 = 0.f;
  asm volatile("" : "+v"(acc0));
  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = acc0;

  // K-major L: the 16 lanes of a group (g = lane/16) each address 8 bytes of a 4 (k) x 16 (i) block - lane l: k-row
  // l/4, columns 4*(l%4)..+3 - and each receives one column's 4 consecutive k values; two such reads make the 8
  // k values (8h..8h+7, h = g/2) that lane r = lane%32 owes the MFMA for row i = 32*tile + r.
  int a_km[FM];
  {
    const int l16 = lane & 15, g = lane >> 4, r4 = l16 >> 2;
#pragma unroll
    for (int i = 0; i < FM; ++i)
      a_km[i] = (8 * (g >> 1) + r4) * (BM * 2) + ((((wm * (WTM / 8) + 4 * i) ^ (4 * r4)) + 2 * (g & 1) + ((l16 & 3) >> 1)) * 16) + (l16 & 1) * 8;
  }
  bf16x8 af[KSTEPS][FM], bfr[KSTEPS][FN];
  auto fread = [&](int stage, int kk) {
    const unsigned char* s = smem + stage * STAGE_B + (((2 * kk + fh) ^ fkey) * 16);
    {
#pragma unroll
      for (int i = 0; i < FM; ++i) af[kk][i] = *reinterpret_cast<const bf16x8*>(s + a_base + i * 32 * ROWB);
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) bfr[kk][j] = *reinterpret_cast<const bf16x8*>(s + b_base + j * 32 * ROWB);
  };
  auto mma = [&](int kk) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk][i], bfr[kk][j], acc[i][j], 0, 0, 0);
  };
  // K-major path: the assembly reads take no part in the compiler's instruction-group scheduling, so phases A and
  // B are written out instruction by instruction (read number r of k-step kk: the A-side tile rows first - two
  // transposing reads each - then the B-side tiles; MFMA number t of a k-step: tile (t / FN, t % FN)).
  constexpr int RPS = 2 * FM + FN;               // LDS read instructions per k-step on the K-major path
  // On this path ALL fragment reads are assembly and the waits for them are placed by hand (the compiler neither
  // sees the reads nor counts them; it puts a wait for ALL vector-memory traffic in front of the builtin form of the
  // transposing read, which drains the slab prefetch): one wait for the k-step-0 fragments before phase B's first MFMA,
  // one for everything at the end of phase B.  The LDS returns data in issue order.  Every wait is an asm statement
  // that takes the fragment registers it covers as read-write operands (land_kstep below): to the compiler the
  // wait produces those values, so every MFMA that consumes a fragment depends on the wait that covers it and
  // reads the registers the wait names - it cannot be moved ahead of the wait.  What the source cannot forbid is a
  // compiler-made copy or spill of a read's destination between the read and its wait; the generated code is
  // therefore checked at every build of the tests (tests/test_kmajor_asm_hazards.py walks the control-flow graph of
  // the compiled kernels and fails if any instruction touches the destination of an LDS read that no wait has
  // retired yet).
  u32x2 km_half[KSTEPS][FM][2];
  u32x4 km_b[KSTEPS][FN];
  auto read_one = [&](int stage, int kk, int r) {
    if (r < 2 * FM) {
      const int i = r >> 1, half = r & 1;
      const unsigned addr = (unsigned)(size_t)(lds_v4i16_ptr)(smem + stage * STAGE_B + (16 * kk) * (BM * 2) + a_km[i]);
      if (half == 0) asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(km_half[kk][i][0]) : "v"(addr) : "memory");
      else asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(km_half[kk][i][1]) : "v"(addr), "n"(4 * (BM * 2)) : "memory");
    } else {
      const int j = r - 2 * FM;
      const unsigned addr = (unsigned)(size_t)(lds_v4i16_ptr)(smem + stage * STAGE_B + (((2 * kk + fh) ^ fkey) * 16) + b_base + j * 32 * ROWB);
      asm volatile("ds_read_b128 %0, %1" : "=v"(km_b[kk][j]) : "v"(addr) : "memory");
    }
  };
  // "wait, then these registers hold the fragments of k-step kk"; only the first k-step of a group carries the
  // s_waitcnt, the others just tie their registers to the same point of the instruction stream.
  auto land_kstep = [&](int kk, auto cnt_tag, bool with_wait) {
    if (with_wait) wait_lgkm_tie<decltype(cnt_tag)::value>(km_half[kk]);
    else tie_regs(km_half[kk]);
    tie_regs(km_b[kk]);
  };
  auto mma_one = [&](int kk, int t) {
    const int i = t / FN, j = t % FN;
    bf16x8 a, b;
    if (LKM) {
      const u32x4 both = {km_half[kk][i][0].x, km_half[kk][i][0].y, km_half[kk][i][1].x, km_half[kk][i][1].y};
      a = __builtin_bit_cast(bf16x8, both);
      b = __builtin_bit_cast(bf16x8, km_b[kk][j]);
    } else {
      a = af[kk][i];
      b = bfr[kk][j];
    }
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i][j], 0, 0, 0);
  };
  // ---- pipeline: two LDS stages.  Measured on this chip: a wave instruction that requests 1 KB keeps the wave's
  // (in-order) issue port busy until the memory pipeline accepts it (~57 clocks each when 4 waves request 16 KB
  // apiece in a burst), and the 4 waves' fragment reads fill the LDS port completely when all of a slab's reads sit
  // in half an iteration.  So requests are never issued in a burst (one after every second MFMA of phase C), and the
  // fragment reads of a slab are spread over three phases: the k-step-0 fragments of the NEXT slab are read during
  // phase C (moving them there from phase A took 8-10 % off the main loop).  That needs slab kt+1 in LDS when phase
  // C of iteration kt starts, so one barrier per iteration does both jobs: "stage cur may be overwritten" and "slab
  // kt+1 is visible".  The loop is skewed by one k-step so that no MFMA waits for LDS latency.  Iteration kt (slab kt
  // sits in stage `cur`, slab kt+1 in `cur^1`; the k-step-0 fragments of slab kt are already in registers):
  //   A  MFMAs of k-step 3 of slab kt-1 | fragment reads of k-step 1
  //   B  MFMAs of k-step 0              | fragment reads of k-steps 2, 3
  //      wait: my reads of stage `cur` and my requests of slab kt+1 have completed; barrier
  //   C  MFMAs of k-steps 1, 2          | the requests of slab kt+2, into stage `cur`
  //                                     | fragment reads of k-step 0 of slab kt+1
  const int KT = NSEG * KT1;
  request_part(0, 0, Zero{}, AllN{});
  if (KT > 1) request_part(1, 1, Zero{}, AllN{});
  wait_vmcnt<0>();
  __syncthreads();
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int t = 0; t < 8; ++t) af[KSTEPS - 1][i][t] = (__bf16)0.0f;     // first pass of phase A multiplies zeros
#pragma unroll
  for (int i = 0; i < FM; ++i) km_half[KSTEPS - 1][i][0] = km_half[KSTEPS - 1][i][1] = u32x2{0u, 0u};
#pragma unroll
  for (int j = 0; j < FN; ++j) km_b[KSTEPS - 1][j] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
  for (int j = 0; j < FN; ++j)
#pragma unroll
    for (int t = 0; t < 8; ++t) bfr[KSTEPS - 1][j][t] = (__bf16)0.0f;
  // k-step 0 of slab 0 (on the K-major path the first iteration's waits cover these reads like any others)
  if (LKM) {
#pragma unroll
    for (int r = 0; r < RPS; ++r) read_one(0, 0, r);
  } else {
    fread(0, 0);
  }

  // Transposed addend tile -> LDS image [BN][BM]; wave-level DMA instruction idx fills image bytes [1024 idx, +1024).
  // The half of the image that lies in the stage the last iteration no longer needs is requested during that
  // iteration (`early`), the rest after the main loop.
  const u16* Et = static_cast<const u16*>(p.Et);
  constexpr int CPT = BM / 8;                    // 16-byte chunks per row of the transposed image
  constexpr int KEYMASK = (CPT < 32 ? CPT : 32) - 1;   // image row c keeps its chunks XOR-swizzled by c & KEYMASK
  constexpr int RPI_T = 64 / CPT > 0 ? 64 / CPT : 1;   // image rows per wave-level DMA instruction / per 64 lanes
  static_assert(CPT <= 64, "one wave instruction covers at least one row of the transposed image");
  constexpr int TI = BN / RPI_T / NW;            // DMA instructions (or 64-lane store groups) per wave
  constexpr int IPS = STAGE_B / 1024 / NW;       // image DMA instructions per wave that land in one pipeline stage
  constexpr int CNT0 = IPS < TI ? IPS : TI, CNT1 = TI - CNT0 < IPS ? TI - CNT0 : IPS;   // instructions per region
  // instruction i of the part of the image that overlays pipeline stage `region` (the last region may hold fewer
  // instructions than a stage has room for)
  auto et_request_one = [&](int region, int i, int plane = 0) {
    if (i >= (region == 0 ? CNT0 : CNT1)) return;
    const int idx0 = region * IPS * NW + wave;
    const int c = idx0 * RPI_T + lane / CPT + i * NW * RPI_T;
    const u16* src = Et + (size_t)(col0 + c) * p.ldet + row0;
    if constexpr (PL > 1) src += (size_t)plane * (size_t)p.et_plane;
    const int chunk = (lane % CPT) ^ (c & KEYMASK);
    __builtin_amdgcn_global_load_lds((gptr)(src + chunk * 8), (lptr)(smem + idx0 * 1024 + i * NW * 1024), 16, 0, 0);
  };
  auto et_request = [&](int region, int plane = 0) {
#pragma unroll
    for (int i = 0; i < CNT0; ++i) et_request_one(region, i, plane);
  };

  int cur = 0;
  int kt = 0;
  // one iteration; REFILL: slab kt+2 exists (requested here); SYNC: slab kt+1 exists (its k-step-0 fragments are
  // read here).  Every MFMA of phases A and C is followed by its share of the phase's other instructions and a
  // scheduling fence, so the instruction order is the one written here.
  constexpr int MT = FM * FN;                    // MFMAs per k-step
  constexpr int NR = LKM ? RPS : FM + FN;        // LDS read instructions per k-step
  auto read_frag = [&](int stage, int kk, int r) {
    if (LKM) {
      read_one(stage, kk, r);
    } else {
      const unsigned char* sp = smem + stage * STAGE_B + (((2 * kk + fh) ^ fkey) * 16);
      if (r < FM) af[kk][r] = *reinterpret_cast<const bf16x8*>(sp + a_base + r * 32 * ROWB);
      else bfr[kk][r - FM] = *reinterpret_cast<const bf16x8*>(sp + b_base + (r - FM) * 32 * ROWB);
    }
  };
  auto iteration = [&](auto refill_tag, auto sync_tag) {
    constexpr bool REFILL = decltype(refill_tag)::value, SYNC = decltype(sync_tag)::value;
    // A: reads of k-step 1 under the MFMAs of k-step 3 of the previous slab
    static_for<0, MT>([&](auto t_tag) {
      constexpr int t = decltype(t_tag)::value;
      mma_one(KSTEPS - 1, t);
#pragma unroll
      for (int r = t * NR / MT; r < (t + 1) * NR / MT; ++r) read_frag(cur, 1, r);
      __builtin_amdgcn_sched_barrier(0);
    });
    if (LKM) {
      constexpr int NG = FM + FN, RG = 2 * RPS / NG;
      constexpr int LEAD = MT >= NG + 2 ? 2 : 0; // MFMAs of k-step 0 issued ahead of phase B's reads
      static_assert(!LKM || (2 * RPS % NG == 0 && MT >= NG + LEAD), "K-major phase layout");
      // B: MFMAs of k-step 0 lead, then one per group of reads of k-steps 2, 3.  The k-step-0 fragments were read
      // during the previous phase C; the reads of k-step 1 (RPS of them) may still be in flight.
      land_kstep(0, std::integral_constant<int, (RPS < 15 ? RPS : 15)>{}, true);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int t = 0; t < LEAD; ++t) mma_one(0, t);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < NG; ++g) {
#pragma unroll
        for (int r = 0; r < RG; ++r) read_one(cur, 2 + (g * RG + r) / RPS, (g * RG + r) % RPS);
        mma_one(0, LEAD + g);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int t = LEAD + NG; t < MT; ++t) mma_one(0, t);
      __builtin_amdgcn_sched_barrier(0);
      land_kstep(1, Zero{}, true);               // k-steps 1..3 are in (and nobody of this wave reads the stage any more)
      land_kstep(2, Zero{}, false);
      land_kstep(3, Zero{}, false);
      __builtin_amdgcn_sched_barrier(0);
    } else {
      // B.  MFMAs go first: the LDS counter is only 4 bits wide, so a wait placed behind more than 15 younger reads
      // degenerates into "wait for everything".
      constexpr int DSG = 2;                     // LDS reads per scheduling group
      fread(cur, 2);
      fread(cur, 3);
      mma(0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
#pragma unroll
      for (int g = 0; g < FM + FN; ++g) {
        __builtin_amdgcn_sched_group_barrier(0x100, DSG, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, FM * FN, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (SYNC) {
      wait_lgkm0();                              // my fragment reads of stage `cur` have returned
      wait_vmcnt<0>();                           // my requests of slab kt+1 have landed
      __builtin_amdgcn_s_barrier();              // ... everybody's: stage `cur` is free and slab kt+1 is visible
    }
    // C: 2 MT MFMAs; among them, evenly, the NLOAD requests of slab kt+2, the NR reads of k-step 0 of slab kt+1 and, in
    // the last iteration, the part of the addend image that overlays the stage no longer in use
    constexpr int NC = (KSTEPS - 2) * MT;
    constexpr bool EARLY_ET = PL == 1 && !REFILL && !SYNC;
    const bool early_et = EARLY_ET && Et != nullptr;
    static_for<0, NC>([&](auto t_tag) {
      constexpr int t = decltype(t_tag)::value;
      mma_one(1 + t / MT, t % MT);
      if constexpr (REFILL) {
        static_for<t * NLOAD / NC, (t + 1) * NLOAD / NC>([&](auto n_tag) { request_part(kt + 2, cur, n_tag, std::integral_constant<int, 1>{}); });
      }
      if constexpr (SYNC) {
#pragma unroll
        for (int r = t * NR / NC; r < (t + 1) * NR / NC; ++r) read_frag(cur ^ 1, 0, r);
      }
      if constexpr (EARLY_ET) {
        if (early_et) {
#pragma unroll
          for (int i = t * CNT0 / NC; i < (t + 1) * CNT0 / NC; ++i) et_request_one(cur ^ 1, i);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    cur ^= 1;
    ++kt;
  };
  using T_ = std::true_type;
  using F_ = std::false_type;
  while (kt + 2 < KT) iteration(T_{}, T_{});
  if (kt + 1 < KT) iteration(F_{}, T_{});
  iteration(F_{}, F_{});
  if (LKM) {                                     // k-step 3 of the last slab
#pragma unroll
    for (int t = 0; t < FM * FN; ++t) mma_one(KSTEPS - 1, t);
  } else {
    mma(KSTEPS - 1);
  }

  // ======================================= epilogue =======================================
  // val = alpha * (beta_acc*acc + beta_e*E).  Each lane owns, per MFMA tile, one column c and rows 8q+4h+e
  // (e = 0..3 contiguous): exactly 8 contiguous bytes of the TRANSPOSED tile.  So the transposed addend tile is
  // DMA-ed into an LDS image [BN][BM] (16-byte chunks of row c XOR-swizzled by the low bits of c), each lane replaces its
  // 8-byte pieces in place with the results, and the image leaves with coalesced 16-byte stores: that is Ct.
  // For C the packed results are transposed on the matrix cores (P^T = P^T * I with a 0/1 selector operand,
  // exact in fp32), which hands each lane 8 contiguous bytes of a ROW of the tile; same image trick, [BM][BN].
  wait_vmcnt<0>();
  __syncthreads();                               // every wave is done with the pipeline stages
  const float alpha = alpha_idx >= 0 ? p.scal[alpha_idx] : 1.f;
  const float ab_acc = alpha * beta_acc, ab_e = alpha * beta_e;   // val = alpha*(beta_acc*acc + beta_e*E), alpha folded in
  u16* C = static_cast<u16*>(p.C);
  u16* Ct = static_cast<u16*>(p.Ct);
  int ldct = p.ldct;
  if (p.symmetric) {                             // mirror store below the diagonal; T itself only off the diagonal
    Ct = C;
    ldct = p.ldc;
    if (tile.flags & kTileDiagonal) C = nullptr;
  }
  if constexpr (PL == 1) {
  if (Et) {
    et_request(cur ^ 1);        // `cur` was flipped after the last iteration: cur^1 is the stage that iteration still read
    wait_vmcnt<0>();
    __syncthreads();
  }
  }

  // Each lane's slot for (MFMA tile i, j; quarter q): image row c = wn*WTN + 32j + r, logical chunk
  // wm*WTM/8 + 4i + q, half h.  The swizzle key c & KEYMASK equals r & KEYMASK (wave and MFMA tile origins are
  // multiples of 32), so the slot address is a per-lane base XOR a compile-time constant.  The addend pieces of tile t+1 are read while tile t is being combined.
  u32x2 pk[FM][FN][4];
  // diagonal constant: this wave's MFMA tile (i, j) starts at row row0 + wm*WTM + 32 i and column col0 + wn*WTN + 32 j
  // of the output; it holds elements C[r][r] when the two are equal, and then row 8q + 4h + e of the MFMA tile meets
  // column fr.  diag_shift = 32 (j - i) for the MFMA tiles that lie on the matrix diagonal (all starts are multiples
  // of 32); any other value: none of this wave's.
  const int diag_shift = p.diag_add != 0 ? (row0 + wm * WTM) - (col0 + wn * WTN) : 1;
  const unsigned slot_base = (unsigned)((wn * WTN + fr) * (BM * 2) + fh * 8) + ((unsigned)((wm * (WTM / 8)) ^ (fr & KEYMASK)) << 4);
  auto slot_of = [&](int i, int j, int q) -> unsigned char* {
    return smem + ((slot_base + (unsigned)(j * 32 * BM * 2)) ^ (unsigned)((4 * i + q) << 4));
  };
  auto combine = [&](auto has_e) {
    constexpr bool HAS_E = decltype(has_e)::value;
    u32x2 ev[2][4];
    if (HAS_E) {
#pragma unroll
      for (int q = 0; q < 4; ++q) ev[0][q] = *reinterpret_cast<const u32x2*>(slot_of(0, 0, q));
    }
#pragma unroll
    for (int t = 0; t < FM * FN; ++t) {
      const int i = t / FN, j = t % FN;
      if (HAS_E && t + 1 < FM * FN) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          ev[(t + 1) & 1][q] = *reinterpret_cast<const u32x2*>(slot_of((t + 1) / FN, (t + 1) % FN, q));
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = ab_acc * acc[i][j][4 * q + e];
        if (HAS_E) {
          const u32x2 e2 = ev[t & 1][q];
          x[0] = fmaf(ab_e, __uint_as_float(e2.x << 16), x[0]);
          x[1] = fmaf(ab_e, __uint_as_float(e2.x & 0xffff0000u), x[1]);
          x[2] = fmaf(ab_e, __uint_as_float(e2.y << 16), x[2]);
          x[3] = fmaf(ab_e, __uint_as_float(e2.y & 0xffff0000u), x[3]);
        }
        if (diag_shift == 32 * (j - i)) {        // wave-uniform
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] += (fr == 8 * q + 4 * fh + e) ? diag_add : 0.f;
        }
        const f32x2 lo = {x[0], x[1]}, hi = {x[2], x[3]};
        pk[i][j][q].x = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2));
        pk[i][j][q].y = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2));
        *reinterpret_cast<u32x2*>(slot_of(i, j, q)) = pk[i][j][q];   // this slot belongs to this lane alone
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  if constexpr (PL == 1) {
  if (Et) combine(std::true_type{}); else combine(std::false_type{});
  if (Ct) {
    __syncthreads();
    constexpr int SB = TI < 8 ? TI : 8;          // image chunks read per batch before they are stored
    // image row of step i: c = c_first + i * (NW * RPI_T); the swizzle key c % 16 only has period 16 / (NW * RPI_T)
    constexpr int CSTEP = NW * RPI_T, PERIOD = (KEYMASK + 1) / CSTEP > 0 ? (KEYMASK + 1) / CSTEP : 1;
    const int c_first = wave * RPI_T + lane / CPT;
    u16* dst[PERIOD];
#pragma unroll
    for (int k = 0; k < PERIOD; ++k) {
      const int c = c_first + k * CSTEP;
      dst[k] = Ct + (size_t)(col0 + c) * ldct + row0 + ((lane % CPT) ^ (c & KEYMASK)) * 8;
    }
    const size_t dstep = (size_t)(CSTEP * PERIOD) * ldct;
#pragma unroll
    for (int i0 = 0; i0 < TI; i0 += SB) {
      u32x4 v[SB];
#pragma unroll
      for (int u = 0; u < SB; ++u) v[u] = *reinterpret_cast<const u32x4*>(smem + ((i0 + u) * NW + wave) * 1024 + lane * 16);
#pragma unroll
      for (int u = 0; u < SB; ++u) {
        const int i = i0 + u;
        *(gvec_ptr)(dst[i % PERIOD] + (size_t)(i / PERIOD) * dstep) = v[u];
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  if (C) {
    // selector operand: k index (h, t) of k-step s stands for tile row 16s + 4h + t (t < 4) or 16s + 8 + 4h + t - 4
    bf16x8 sel[2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int row = 16 * s + 4 * fh + (t < 4 ? t : 4 + t);
        sel[s][t] = (__bf16)(fr == row ? 1.0f : 0.0f);
      }
    constexpr int CPR = BN / 8;                  // 16-byte chunks per row of the row-major image
    constexpr int RPI_C = 64 / CPR;
    constexpr int CI = BM / RPI_C / NW;
    __syncthreads();                             // the transposed image has been read out (or the addend consumed)
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        f32x16 d;
#pragma unroll
        for (int v = 0; v < 16; ++v) d[v] = 0.f;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          const u32x4 raw = {pk[i][j][2 * s].x, pk[i][j][2 * s].y, pk[i][j][2 * s + 1].x, pk[i][j][2 * s + 1].y};
          d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), sel[s], d, 0, 0, 0);
        }
        const int r = wm * WTM + i * 32 + fr;    // this lane now holds row r, columns 8q + 4h + e of the MFMA tile
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int lchunk = (wn * WTN + j * 32) / 8 + q;
          const f32x2 lo = {d[4 * q], d[4 * q + 1]}, hi = {d[4 * q + 2], d[4 * q + 3]};
          u32x2 w;
          w.x = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2));
          w.y = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2));
          *reinterpret_cast<u32x2*>(smem + r * (BN * 2) + ((lchunk ^ (r & (CPR - 1))) * 16) + fh * 8) = w;
        }
      }
    __syncthreads();
    constexpr int SB = CI < 8 ? CI : 8;
    constexpr int RSTEP = NW * RPI_C, PERIOD = CPR / RSTEP > 0 ? CPR / RSTEP : 1;
    const int r_first = wave * RPI_C + lane / CPR;
    u16* dst[PERIOD];
#pragma unroll
    for (int k = 0; k < PERIOD; ++k) {
      const int r = r_first + k * RSTEP;
      dst[k] = C + (size_t)(row0 + r) * p.ldc + col0 + ((lane % CPR) ^ (r & (CPR - 1))) * 8;
    }
    const size_t dstep = (size_t)(RSTEP * PERIOD) * p.ldc;
#pragma unroll
    for (int i0 = 0; i0 < CI; i0 += SB) {
      u32x4 v[SB];
#pragma unroll
      for (int u = 0; u < SB; ++u) v[u] = *reinterpret_cast<const u32x4*>(smem + ((i0 + u) * NW + wave) * 1024 + lane * 16);
#pragma unroll
      for (int u = 0; u < SB; ++u) {
        const int i = i0 + u;
        *(gvec_ptr)(dst[i % PERIOD] + (size_t)(i / PERIOD) * dstep) = v[u];
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  } else {
    // ---- split operands: val = alpha * (beta_acc * acc + beta_e * sum_q E_q) (+ diagonal constant) is formed in
    // the accumulator registers in fp32; plane q of the outputs is bf16(val_q) with val_0 = val and
    // val_{q+1} = val_q - bf16(val_q) (exact in fp32).  Every plane takes the same route through the LDS images
    // as the single plane of the plain path; nothing is overlapped here - three to six times the matrix-core work
    // stands against this epilogue.
    const size_t ctpl = (size_t)(p.symmetric ? p.c_plane : p.ct_plane), cpl = (size_t)p.c_plane;
    auto pack4 = [](float x0, float x1, float x2, float x3) -> u32x2 {
      const f32x2 lo = {x0, x1}, hi = {x2, x3};
      u32x2 w;
      w.x = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2));
      w.y = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2));
      return w;
    };
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] *= ab_acc;
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
        if (diag_shift == 32 * (j - i)) {        // wave-uniform
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[i][j][v] += (fr == 8 * (v >> 2) + 4 * fh + (v & 3)) ? diag_add : 0.f;
        }
    if (Et) {
#pragma unroll 1
      for (int q = 0; q < PL; ++q) {
        if (q) __syncthreads();                  // every lane has taken its pieces of the previous plane's image
        et_request(0, q);
        et_request(1, q);
        wait_vmcnt<0>();
        __syncthreads();
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
              const u32x2 e2 = *reinterpret_cast<const u32x2*>(slot_of(i, j, qq));
              acc[i][j][4 * qq + 0] = fmaf(ab_e, __uint_as_float(e2.x << 16), acc[i][j][4 * qq + 0]);
              acc[i][j][4 * qq + 1] = fmaf(ab_e, __uint_as_float(e2.x & 0xffff0000u), acc[i][j][4 * qq + 1]);
              acc[i][j][4 * qq + 2] = fmaf(ab_e, __uint_as_float(e2.y << 16), acc[i][j][4 * qq + 2]);
              acc[i][j][4 * qq + 3] = fmaf(ab_e, __uint_as_float(e2.y & 0xffff0000u), acc[i][j][4 * qq + 3]);
              if (qq == 3) __builtin_amdgcn_sched_barrier(0);   // one MFMA tile at a time: keeps the register count down
            }
      }
    }
    // store-out of the transposed image [BN][BM] and of the row-major image [BM][BN]: 16 bytes per lane, coalesced
    constexpr int SBT = TI < 8 ? TI : 8;
    constexpr int CSTEP = NW * RPI_T, PERIOD_T = (KEYMASK + 1) / CSTEP > 0 ? (KEYMASK + 1) / CSTEP : 1;
    auto store_ct = [&](u16* base) {
      const int c_first = wave * RPI_T + lane / CPT;
      u16* dst[PERIOD_T];
#pragma unroll
      for (int k = 0; k < PERIOD_T; ++k) {
        const int c = c_first + k * CSTEP;
        dst[k] = base + (size_t)(col0 + c) * ldct + row0 + ((lane % CPT) ^ (c & KEYMASK)) * 8;
      }
      const size_t dstep = (size_t)(CSTEP * PERIOD_T) * ldct;
#pragma unroll
      for (int i0 = 0; i0 < TI; i0 += SBT) {
        u32x4 v[SBT];
#pragma unroll
        for (int u = 0; u < SBT; ++u) v[u] = *reinterpret_cast<const u32x4*>(smem + ((i0 + u) * NW + wave) * 1024 + lane * 16);
#pragma unroll
        for (int u = 0; u < SBT; ++u) {
          const int i = i0 + u;
          *(gvec_ptr)(dst[i % PERIOD_T] + (size_t)(i / PERIOD_T) * dstep) = v[u];
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    constexpr int CPR = BN / 8, RPI_C = 64 / CPR, CI = BM / RPI_C / NW;
    constexpr int SBC = CI < 8 ? CI : 8;
    constexpr int RSTEP = NW * RPI_C, PERIOD_C = CPR / RSTEP > 0 ? CPR / RSTEP : 1;
    auto store_c = [&](u16* base) {
      const int r_first = wave * RPI_C + lane / CPR;
      u16* dst[PERIOD_C];
#pragma unroll
      for (int k = 0; k < PERIOD_C; ++k) {
        const int r = r_first + k * RSTEP;
        dst[k] = base + (size_t)(row0 + r) * p.ldc + col0 + ((lane % CPR) ^ (r & (CPR - 1))) * 8;
      }
      const size_t dstep = (size_t)(RSTEP * PERIOD_C) * p.ldc;
#pragma unroll
      for (int i0 = 0; i0 < CI; i0 += SBC) {
        u32x4 v[SBC];
#pragma unroll
        for (int u = 0; u < SBC; ++u) v[u] = *reinterpret_cast<const u32x4*>(smem + ((i0 + u) * NW + wave) * 1024 + lane * 16);
#pragma unroll
        for (int u = 0; u < SBC; ++u) {
          const int i = i0 + u;
          *(gvec_ptr)(dst[i % PERIOD_C] + (size_t)(i / PERIOD_C) * dstep) = v[u];
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    bf16x8 sel[2];                               // 0/1 selector of the MFMA transpose (see the plain path)
#pragma unroll
    for (int sx = 0; sx < 2; ++sx)
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int row = 16 * sx + 4 * fh + (t < 4 ? t : 4 + t);
        sel[sx][t] = (__bf16)(fr == row ? 1.0f : 0.0f);
      }
    // all planes at once, MFMA tile by MFMA tile: the fp32 values leave the accumulator registers for good
    u32x2 pkq[PL][FM][FN][4];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) {
          float x0 = acc[i][j][4 * qq], x1 = acc[i][j][4 * qq + 1], x2 = acc[i][j][4 * qq + 2], x3 = acc[i][j][4 * qq + 3];
#pragma unroll
          for (int q = 0; q < PL; ++q) {
            const u32x2 w = pack4(x0, x1, x2, x3);
            pkq[q][i][j][qq] = w;
            if (q + 1 < PL) {                    // what this plane left of the value
              x0 -= __uint_as_float(w.x << 16);
              x1 -= __uint_as_float(w.x & 0xffff0000u);
              x2 -= __uint_as_float(w.y << 16);
              x3 -= __uint_as_float(w.y & 0xffff0000u);
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
    for (int q = 0; q < PL; ++q) {
      if (Ct) {
        __syncthreads();                         // the image is free (addend consumed / previous plane stored)
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) *reinterpret_cast<u32x2*>(slot_of(i, j, qq)) = pkq[q][i][j][qq];
        __syncthreads();
        store_ct(Ct + (size_t)q * ctpl);
      }
      if (C) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j) {
            f32x16 d;
#pragma unroll
            for (int v = 0; v < 16; ++v) d[v] = 0.f;
#pragma unroll
            for (int sx = 0; sx < 2; ++sx) {
              const u32x4 raw = {pkq[q][i][j][2 * sx].x, pkq[q][i][j][2 * sx].y, pkq[q][i][j][2 * sx + 1].x, pkq[q][i][j][2 * sx + 1].y};
              d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), sel[sx], d, 0, 0, 0);
            }
            const int r = wm * WTM + i * 32 + fr;
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
              const int lchunk = (wn * WTN + j * 32) / 8 + qq;
              *reinterpret_cast<u32x2*>(smem + r * (BN * 2) + ((lchunk ^ (r & (CPR - 1))) * 16) + fh * 8) =
                  pack4(d[4 * qq], d[4 * qq + 1], d[4 * qq + 2], d[4 * qq + 3]);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        __syncthreads();
        store_c(C + (size_t)q * cpl);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// Diagonal 256 x 256 tiles of the symmetric products (L = R, plain bf16).  Such a tile is symmetric itself: of its
// 8 x 8 blocks of 32 x 32 only the 36 on or above the diagonal are computed, dealt 9 to a wave (against 16 a wave in
// an ordinary tile), and both the block and - for the 28 off the diagonal - its transpose are written into ONE image of
// the tile.  The tile needs one operand panel instead of two, so a pipeline stage is 32 KB and a slab takes 8 requests
// per wave.  Everything else (slab pipeline, swizzles, image store) is the ordinary tile's.
//
// A wave's share: the blocks (bi[t], bj[t]), bi <= bj, and the set fb[] of 32-row panel blocks their operands come from
// (fa[t] / fc[t]: positions of bi[t] / bj[t] in fb).
struct DiagWave0 {   // rows 0-2 x columns 3-5
  static constexpr int N = 9, NF = 6;
  static constexpr int bi[N] = {0, 0, 0, 1, 1, 1, 2, 2, 2}, bj[N] = {3, 4, 5, 3, 4, 5, 3, 4, 5};
  static constexpr int fb[NF] = {0, 1, 2, 3, 4, 5};
  static constexpr int fa[N] = {0, 0, 0, 1, 1, 1, 2, 2, 2}, fc[N] = {3, 4, 5, 3, 4, 5, 3, 4, 5};
};
struct DiagWave1 {   // triangle of rows 0-2, and rows 3-5 x column 6
  static constexpr int N = 9, NF = 7;
  static constexpr int bi[N] = {0, 0, 0, 1, 1, 2, 3, 4, 5}, bj[N] = {0, 1, 2, 1, 2, 2, 6, 6, 6};
  static constexpr int fb[NF] = {0, 1, 2, 3, 4, 5, 6};
  static constexpr int fa[N] = {0, 0, 0, 1, 1, 2, 3, 4, 5}, fc[N] = {0, 1, 2, 1, 2, 2, 6, 6, 6};
};
struct DiagWave2 {   // triangle of rows 3-5, and rows 3-5 x column 7
  static constexpr int N = 9, NF = 4;
  static constexpr int bi[N] = {3, 3, 3, 4, 4, 5, 3, 4, 5}, bj[N] = {3, 4, 5, 4, 5, 5, 7, 7, 7};
  static constexpr int fb[NF] = {3, 4, 5, 7};
  static constexpr int fa[N] = {0, 0, 0, 1, 1, 2, 0, 1, 2}, fc[N] = {0, 1, 2, 1, 2, 2, 3, 3, 3};
};
struct DiagWave3 {   // rows 0-2 x columns 6-7, and the triangle of rows 6-7
  static constexpr int N = 9, NF = 5;
  static constexpr int bi[N] = {0, 0, 1, 1, 2, 2, 6, 6, 7}, bj[N] = {6, 7, 6, 7, 6, 7, 6, 7, 7};
  static constexpr int fb[NF] = {0, 1, 2, 6, 7};
  static constexpr int fa[N] = {0, 0, 1, 1, 2, 2, 3, 3, 4}, fc[N] = {3, 4, 3, 4, 3, 4, 3, 4, 4};
};

template <typename W>
__device__ __forceinline__ void diag_wave_body(const GemmProblem& p, int row0, unsigned char* smem, float beta_acc, float beta_e,
                                               int alpha_idx, float diag_add, int tid) {
  constexpr int BM = 256, NW = 4, N = W::N, NF = W::NF;
  constexpr int LI = BM / 8 / NW;                  // DMA instructions per wave per slab
  constexpr int STAGE_B = BM * ROWB;               // one operand panel per stage
  constexpr int KSTEPS = BK / 16;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // requests: as in the ordinary tile (8 rows x 128 B per wave instruction, chunks XOR-swizzled by (row/2)%8)
  const int dma_row = wave * 8 + (lane >> 3);
  const int dma_chunk = (lane & 7) ^ (((lane >> 4) & 3) + 4 * (wave & 1));
  const u16* lsrc = static_cast<const u16*>(p.L) + (size_t)(row0 + dma_row) * p.ldl + dma_chunk * 8;
  const size_t lstep = (size_t)(8 * NW) * p.ldl;
  auto request_one = [&](int kt, int stage, int n) {
    __builtin_amdgcn_global_load_lds((gptr)(lsrc + n * lstep + (size_t)kt * BK),
                                     (lptr)(smem + stage * STAGE_B + wave * 1024 + n * NW * 1024), 16, 0, 0);
  };
  const int fr = lane & 31, fh = lane >> 5;
  const int fkey = (fr >> 1) & 7;
  float acc0 = 0.f;
  asm volatile("" : "+v"(acc0));                 // see gemm_tile_body
  f32x16 acc[N];
#pragma unroll
  for (int t = 0; t < N; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = acc0;
  bf16x8 fg[KSTEPS][NF];
  auto read_frag = [&](int stage, int kk, int f) {
    fg[kk][f] = *reinterpret_cast<const bf16x8*>(smem + stage * STAGE_B + (32 * W::fb[f] + fr) * ROWB + (((2 * kk + fh) ^ fkey) * 16));
  };
  auto mma_one = [&](int kk, int t) {
    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fg[kk][W::fa[t]], fg[kk][W::fc[t]], acc[t], 0, 0, 0);
  };

  // addend image [256][256] (transposed addend = the addend itself, the matrix being symmetric): instruction i of the
  // image half `half` (64 KB each; the upper half lies beyond both pipeline stages and can be requested at any time)
  const u16* Et = static_cast<const u16*>(p.Et);
  constexpr int CPT = BM / 8, KEYMASK = 31, RPI_T = 2, TI = BM / RPI_T / NW;   // 32 chunks per image row, 32 instr per wave
  auto et_request_one = [&](int half, int i) {
    const int idx0 = half * (TI / 2) * NW + wave;
    const int c = idx0 * RPI_T + lane / CPT + i * NW * RPI_T;
    const int chunk = (lane % CPT) ^ (c & KEYMASK);
    __builtin_amdgcn_global_load_lds((gptr)(Et + (size_t)(row0 + c) * p.ldet + row0 + chunk * 8),
                                     (lptr)(smem + idx0 * 1024 + i * NW * 1024), 16, 0, 0);
  };

  // ---- main loop: the ordinary tile's pipeline (see there) with 9 MFMAs per k-step ----
  const int KT = p.K / BK;
#pragma unroll
  for (int n = 0; n < LI; ++n) request_one(0, 0, n);
  if (KT > 1) {
#pragma unroll
    for (int n = 0; n < LI; ++n) request_one(1, 1, n);
  }
  wait_vmcnt<0>();
  __syncthreads();
#pragma unroll
  for (int f = 0; f < NF; ++f)
#pragma unroll
    for (int t = 0; t < 8; ++t) fg[KSTEPS - 1][f][t] = (__bf16)0.0f;     // first pass of phase A multiplies zeros
#pragma unroll
  for (int f = 0; f < NF; ++f) read_frag(0, 0, f);
  int cur = 0, kt = 0;
  auto iteration = [&](auto refill_tag, auto sync_tag) {
    constexpr bool REFILL = decltype(refill_tag)::value, SYNC = decltype(sync_tag)::value;
    // A: MFMAs of k-step 3 of the previous slab | reads of k-step 1
    static_for<0, N>([&](auto t_tag) {
      constexpr int t = decltype(t_tag)::value;
      mma_one(KSTEPS - 1, t);
#pragma unroll
      for (int f = t * NF / N; f < (t + 1) * NF / N; ++f) read_frag(cur, 1, f);
      __builtin_amdgcn_sched_barrier(0);
    });
    // B: MFMAs of k-step 0 | reads of k-steps 2, 3
    static_for<0, N>([&](auto t_tag) {
      constexpr int t = decltype(t_tag)::value;
      mma_one(0, t);
#pragma unroll
      for (int r = t * 2 * NF / N; r < (t + 1) * 2 * NF / N; ++r) read_frag(cur, 2 + r / NF, r % NF);
      __builtin_amdgcn_sched_barrier(0);
    });
    if (SYNC) {
      wait_lgkm0();                              // my fragment reads of stage `cur` have returned
      wait_vmcnt<0>();                           // my requests of slab kt+1 have landed
      __builtin_amdgcn_s_barrier();              // ... everybody's: stage `cur` is free and slab kt+1 is visible
    }
    // C: MFMAs of k-steps 1, 2 | requests of slab kt+2 | reads of k-step 0 of slab kt+1 | in the last iteration the
    // upper half of the addend image
    constexpr int NC = 2 * N;
    const bool early_et = !REFILL && !SYNC && Et != nullptr;
    static_for<0, NC>([&](auto t_tag) {
      constexpr int t = decltype(t_tag)::value;
      mma_one(1 + t / N, t % N);
      if constexpr (REFILL) {
#pragma unroll
        for (int n = t * LI / NC; n < (t + 1) * LI / NC; ++n) request_one(kt + 2, cur, n);
      }
      if constexpr (SYNC) {
#pragma unroll
        for (int f = t * NF / NC; f < (t + 1) * NF / NC; ++f) read_frag(cur ^ 1, 0, f);
      }
      if constexpr (!REFILL && !SYNC) {
        if (early_et) {
#pragma unroll
          for (int i = t * (TI / 2) / NC; i < (t + 1) * (TI / 2) / NC; ++i) et_request_one(1, i);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    cur ^= 1;
    ++kt;
  };
  using T_ = std::true_type;
  using F_ = std::false_type;
  while (kt + 2 < KT) iteration(T_{}, T_{});
  if (kt + 1 < KT) iteration(F_{}, T_{});
  iteration(F_{}, F_{});
#pragma unroll
  for (int t = 0; t < N; ++t) mma_one(KSTEPS - 1, t);

  // ---- epilogue: val = alpha * (beta_acc * acc + beta_e * E) (+ the diagonal constant), one rounding to bf16 ----
  wait_vmcnt<0>();
  __syncthreads();                               // every wave is done with the pipeline stages
  const float alpha = alpha_idx >= 0 ? p.scal[alpha_idx] : 1.f;
  const float ab_acc = alpha * beta_acc, ab_e = alpha * beta_e;
  if (Et) {
#pragma unroll
    for (int i = 0; i < TI / 2; ++i) et_request_one(0, i);
    wait_vmcnt<0>();
    __syncthreads();
  }
  // Block (bi, bj) as the accumulators hold it: lane (fr, fh) owns column fr of block column bj and rows 8q + 4fh + e
  // of block row bi, i.e. 8 contiguous bytes of image row 32 bj + fr (16-byte chunk 4 bi + q, half fh; the chunk position is
  // XOR-swizzled by the image row's low 5 bits = fr): the image then holds the block transposed, which by symmetry
  // is the tile's block (bj, bi).  For bi < bj the block itself is produced by a transpose on the matrix cores and
  // written to image rows 32 bi + fr, chunks 4 bj + q - slots of a block below the diagonal, which nobody computes.
  auto slot = [&](int brow, int bchunk, int q) -> unsigned char* {
    return smem + (32 * brow + fr) * (BM * 2) + ((((4 * bchunk + q) ^ fr) & (CPT - 1)) << 4) + fh * 8;
  };
  bf16x8 sel[2];                                 // 0/1 selector of the MFMA transpose (see the ordinary tile)
#pragma unroll
  for (int sx = 0; sx < 2; ++sx)
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int row = 16 * sx + 4 * fh + (t < 4 ? t : 4 + t);
      sel[sx][t] = (__bf16)(fr == row ? 1.0f : 0.0f);
    }
  const bool add_diag = p.diag_add != 0;
#pragma unroll
  for (int t = 0; t < N; ++t) {
    u32x2 pk[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float x[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = ab_acc * acc[t][4 * q + e];
      if (Et) {
        const u32x2 e2 = *reinterpret_cast<const u32x2*>(slot(W::bj[t], W::bi[t], q));
        x[0] = fmaf(ab_e, __uint_as_float(e2.x << 16), x[0]);
        x[1] = fmaf(ab_e, __uint_as_float(e2.x & 0xffff0000u), x[1]);
        x[2] = fmaf(ab_e, __uint_as_float(e2.y << 16), x[2]);
        x[3] = fmaf(ab_e, __uint_as_float(e2.y & 0xffff0000u), x[3]);
      }
      if (W::bi[t] == W::bj[t] && add_diag) {
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] += (fr == 8 * q + 4 * fh + e) ? diag_add : 0.f;
      }
      const f32x2 lo = {x[0], x[1]}, hi = {x[2], x[3]};
      pk[q].x = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2));
      pk[q].y = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2));
      *reinterpret_cast<u32x2*>(slot(W::bj[t], W::bi[t], q)) = pk[q];
    }
    if (W::bi[t] != W::bj[t]) {
      f32x16 d;
#pragma unroll
      for (int v = 0; v < 16; ++v) d[v] = 0.f;
#pragma unroll
      for (int sx = 0; sx < 2; ++sx) {
        const u32x4 raw = {pk[2 * sx].x, pk[2 * sx].y, pk[2 * sx + 1].x, pk[2 * sx + 1].y};
        d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), sel[sx], d, 0, 0, 0);
      }
      // this lane now holds row fr of the block, columns 8q + 4fh + e
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x2 lo = {d[4 * q], d[4 * q + 1]}, hi = {d[4 * q + 2], d[4 * q + 3]};
        u32x2 w;
        w.x = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2));
        w.y = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2));
        *reinterpret_cast<u32x2*>(slot(W::bi[t], W::bj[t], q)) = w;
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  __syncthreads();
  // the image leaves with coalesced 16-byte stores (image row c = output row row0 + c)
  {
    u16* C = static_cast<u16*>(p.C);
    constexpr int CSTEP = NW * RPI_T, PERIOD = (KEYMASK + 1) / CSTEP, SB = 8;
    const int c_first = wave * RPI_T + lane / CPT;
    u16* dst[PERIOD];
#pragma unroll
    for (int k = 0; k < PERIOD; ++k) {
      const int c = c_first + k * CSTEP;
      dst[k] = C + (size_t)(row0 + c) * p.ldc + row0 + ((lane % CPT) ^ (c & KEYMASK)) * 8;
    }
    const size_t dstep = (size_t)(CSTEP * PERIOD) * p.ldc;
#pragma unroll
    for (int i0 = 0; i0 < TI; i0 += SB) {
      u32x4 v[SB];
#pragma unroll
      for (int u = 0; u < SB; ++u) v[u] = *reinterpret_cast<const u32x4*>(smem + ((i0 + u) * NW + wave) * 1024 + lane * 16);
#pragma unroll
      for (int u = 0; u < SB; ++u) {
        const int i = i0 + u;
        *(gvec_ptr)(dst[i % PERIOD] + (size_t)(i / PERIOD) * dstep) = v[u];
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

__device__ __forceinline__ void diag_tile_body(const GemmProblem& p, const GemmTile& tile, unsigned char* smem, float beta_acc,
                                               float beta_e, int alpha_idx, float diag_add, int wave_id) {
  int tid = thread_index(wave_id);
  asm volatile("" : "+v"(tid));                  // see gemm_tile_body
  const int row0 = tile.r0 * kTileUnit;
  switch (__builtin_amdgcn_readfirstlane(tid >> 6)) {
    case 0: diag_wave_body<DiagWave0>(p, row0, smem, beta_acc, beta_e, alpha_idx, diag_add, tid); break;
    case 1: diag_wave_body<DiagWave1>(p, row0, smem, beta_acc, beta_e, alpha_idx, diag_add, tid); break;
    case 2: diag_wave_body<DiagWave2>(p, row0, smem, beta_acc, beta_e, alpha_idx, diag_add, tid); break;
    default: diag_wave_body<DiagWave3>(p, row0, smem, beta_acc, beta_e, alpha_idx, diag_add, tid); break;
  }
}

// ---- kernels.  Fine launch: 128 x 128 tiles, two blocks per compute unit.  Coarse launch: one block per compute
// unit, each block running the shape its table entry names - 256 x 256 (2 x 2 waves) or 512 x 128 (4 x 1 waves; the
// 128-wide strips that an odd multiple of 128 leaves beside the 256-tiles).  Both coarse shapes give every wave a
// 128 x 128 tile, so they share register budget, MFMA schedule and per-wave LDS traffic, and a launch mixes them freely:
// the strips fill compute units next to the 256-tiles of the same product instead of running as a launch of their own.
constexpr size_t kLds128 = TileCfg<128, 128>::lds_bytes(2);
constexpr size_t kLds256 = TileCfg<256, 256>::lds_bytes(2);
constexpr size_t kLds512 = TileCfg<512, 128>::lds_bytes(2);
constexpr int kMaxPlanes = 3;

// A table entry through whole-dword loads, so that they are scalar loads: the sub-dword fields would otherwise come
// through a vector load, and the wait for it is a wait for every store of the block's previous tile as well.
__device__ __forceinline__ GemmTile load_tile(const GemmTile* __restrict__ tiles, int t) {
  static_assert(sizeof(GemmTile) == 12, "three dwords");
  const uint32_t* w = reinterpret_cast<const uint32_t*>(tiles) + 3 * (size_t)t;
  const uint32_t w0 = w[0], w1 = w[1], w2 = w[2];
  GemmTile r;
  r.prob = (int32_t)w0;
  r.r0 = (uint16_t)(w1 & 0xffffu);
  r.c0 = (uint16_t)(w1 >> 16);
  r.shape = (uint8_t)(w2 & 0xffu);
  r.flags = (uint8_t)((w2 >> 8) & 0xffu);
  r.pad_ = 0;
  return r;
}

template <bool LKM, int PL>
__global__ __launch_bounds__(256, 2) void ns_gemm_bf16_fine_kernel(const GemmProblem* __restrict__ probs,
                                                                    const GemmTile* __restrict__ tiles, float beta_acc,
                                                                    float beta_e, int alpha_idx, float diag_add) {
  extern __shared__ __align__(16) unsigned char smem[];
  const GemmTile tile = load_tile(tiles, blockIdx.x);
  const GemmProblem p = probs[tile.prob];
  gemm_tile_body<128, 128, 2, 2, 2, LKM, PL>(p, tile, smem, beta_acc, beta_e, alpha_idx, diag_add,
                                             __builtin_amdgcn_readfirstlane(threadIdx.x >> 6));
}

// Block b works through table entries b, b + gridDim.x, ...  Launched with one block per tile, or persistent: one
// block per compute unit (a multiple of the 8 dies, so an entry still runs on die index % 8); a persistent block that
// goes on to its next tile neither waits for its stores to drain nor is re-dispatched, and its next tile's first
// operand requests overlap both (measured +2 % on the MoE bank; with tiles of mixed K the static dealing loses that
// again, so such launches stay one block per tile).
template <bool LKM, int PL>
__global__ __launch_bounds__(256, 1) void ns_gemm_bf16_kernel(const GemmProblem* __restrict__ probs,
                                                               const GemmTile* __restrict__ tiles, int n_tiles, float beta_acc,
                                                               float beta_e, int alpha_idx, float diag_add) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int wave_id = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  for (int t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const GemmTile tile = load_tile(tiles, t);
    const GemmProblem p = probs[tile.prob];
    const int shape = __builtin_amdgcn_readfirstlane(tile.shape);
    if (shape == kShape512x128) {
      gemm_tile_body<512, 128, 4, 1, 2, LKM, PL>(p, tile, smem, beta_acc, beta_e, alpha_idx, diag_add, wave_id);
    } else if (!LKM && PL == 1 && shape == kShape256Diag) {
      if constexpr (!LKM && PL == 1) diag_tile_body(p, tile, smem, beta_acc, beta_e, alpha_idx, diag_add, wave_id);
    } else {
      gemm_tile_body<256, 256, 2, 2, 2, LKM, PL>(p, tile, smem, beta_acc, beta_e, alpha_idx, diag_add, wave_id);
    }
    __syncthreads();        // every wave has read its part of the LDS images: the next tile may overwrite them
  }
}

int g_coarse_grid = 0;      // blocks of a coarse launch: one per compute unit (set by gemm_setup)

template <bool LKM, int PL>
hipError_t setup_pair() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&ns_gemm_bf16_fine_kernel<LKM, PL>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds128);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&ns_gemm_bf16_kernel<LKM, PL>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds512);
}

template <bool LKM, int PL>
void launch_one(int coarse, int flags, const GemmProblem* probs, const GemmTile* tiles, int n_tiles, float beta_acc,
                float beta_e, int alpha_idx, float diag_add, hipStream_t s) {
  if (!coarse)
    ns_gemm_bf16_fine_kernel<LKM, PL><<<n_tiles, 256, kLds128, s>>>(probs, tiles, beta_acc, beta_e, alpha_idx, diag_add);
  else
    ns_gemm_bf16_kernel<LKM, PL><<<(flags & kGemmPersistent) && n_tiles > g_coarse_grid ? g_coarse_grid : n_tiles, 256,
                                   (flags & kGemmStrips) ? kLds512 : kLds256, s>>>(
        probs, tiles, n_tiles, beta_acc, beta_e, alpha_idx, diag_add);
}

}  // namespace

int gemm_coarse_blocks() { return g_coarse_grid; }

hipError_t gemm_setup() {
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  g_coarse_grid = cus > 0 ? cus : 256;
  e = setup_pair<false, 1>();
  if (e == hipSuccess) e = setup_pair<true, 1>();
  if (e == hipSuccess) e = setup_pair<false, 2>();
  if (e == hipSuccess) e = setup_pair<true, 2>();
  if (e == hipSuccess) e = setup_pair<false, 3>();
  if (e == hipSuccess) e = setup_pair<true, 3>();
  return e;
}

hipError_t launch_gemm_bf16(int coarse, int flags, const GemmProblem* probs, const GemmTile* tiles, int n_tiles, float beta_acc,
                            float beta_e, int alpha_idx, float diag_add, int l_kmajor, int planes, hipStream_t s) {
  if (n_tiles <= 0) return hipSuccess;
  if (planes < 1 || planes > kMaxPlanes) return hipErrorInvalidValue;
#define MUON_GEMM_CASE(K, P)                                                                                     \
  if ((l_kmajor != 0) == K && planes == P) launch_one<K, P>(coarse, flags, probs, tiles, n_tiles, beta_acc, beta_e, alpha_idx, diag_add, s)
  MUON_GEMM_CASE(false, 1);
  MUON_GEMM_CASE(true, 1);
  MUON_GEMM_CASE(false, 2);
  MUON_GEMM_CASE(true, 2);
  MUON_GEMM_CASE(false, 3);
  MUON_GEMM_CASE(true, 3);
#undef MUON_GEMM_CASE
  return hipGetLastError();
}

}  // namespace muon
