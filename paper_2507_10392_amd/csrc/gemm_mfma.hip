// 16-bit (bf16 / fp16) MFMA GEMM: argument checks and the choice of workgroup tile.  The kernels live in
// gemm_mfma_impl.h, one translation unit per tile shape.
#include "kernels.h"

namespace zs {

hipError_t gemm_mfma_256x256(hipStream_t st, const Gemm& g);   // 8 wavefronts
hipError_t gemm_mfma_128x128(hipStream_t st, const Gemm& g);   // 4 wavefronts, two workgroups per CU
hipError_t gemm_mfma_256x256_f16(hipStream_t st, const Gemm& g);
hipError_t gemm_mfma_128x128_f16(hipStream_t st, const Gemm& g);

namespace {
bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
int g_force_tile = 0;   // 0 automatic; 1: 256x256, 2: 128x128 (set through gemm_mfma_force_tile)
}  // namespace

// The kernel needs 16-byte aligned rows for its vector loads: base pointers 16-byte aligned and
// every leading dimension, batch stride and segment size a multiple of 8 elements; the extent
// along each operand's contiguous axis must be a multiple of 8 as well.
bool gemm_mfma_supported(DType dt, const Gemm& g) {
  if (dt != BF16 && dt != F16) return false;
  if (g.M < 1 || g.N < 1 || g.K < 1 || g.batch < 1) return false;
  if (!aligned16(g.A) || !aligned16(g.B)) return false;
  if (g.lda % 8 || g.ldb % 8 || g.sA % 8 || g.sB % 8) return false;
  if (g.K % 8) return false;                       // k-contiguous operands are read 8 k at a time; tails are zero-filled
  if (g.transA && g.M % 8) return false;           // row-contiguous operands are read 8 rows at a time
  if (!g.transB && g.N % 8) return false;
  if (g.glu) {   // gated unit fused into the store
    if (g.glu != 1 && g.glu != 2) return false;
    if (g.transA || (g.glu == 1) == (g.transB != 0)) return false;   // 1: y = x [Wg | Wu]; 2: da = dy Wd^T
    if (g.c_f32_accum || g.batch != 1 || g.bias || g.resid || g.rope || g.kseg || g.nx) return false;
    if (!g.gu || !aligned16(g.gu) || g.gu_ld % 8 || g.gu_up % 8 || g.N % 8) return false;
    if (g.glu == 1 && g.sB <= 0) return false;
  }
  if (g.nx) {   // multi-part K range of an accumulating product
    if (g.nx < 0 || g.nx >= GEMM_MAX_PARTS) return false;
    // the K loop takes two slabs of 64 rows per step, and a step must lie inside one part
    if (!g.transA || g.transB || !g.c_f32_accum || g.kseg <= 0 || g.kseg % 128 || (int64_t)g.kseg * g.nx >= g.K) return false;
    for (int p = 0; p < g.nx; ++p)
      if (!g.Ax[p] || !g.Bx[p] || !aligned16(g.Ax[p]) || !aligned16(g.Bx[p])) return false;
  } else if (g.kseg) {
    if (!g.transB || g.kseg % 8 || g.segB % 8 || g.K % g.kseg) return false;
  }
  // the bf16 epilogue moves 8 consecutive columns per 16-byte access
  if (!g.c_f32_accum) {
    if (!aligned16(g.C) || g.ldc % 8 || g.sC % 8) return false;
    if (g.resid && (!aligned16(g.resid) || g.ldr % 8)) return false;
    if (g.bias && (!aligned16(g.bias) || g.sBias % 8)) return false;
    // the fused rotation works on whole 8-column vectors that do not straddle heads
    if (g.rope && (g.N % 8 || g.rope_d % 8 || g.rope_S < 1 || ((uintptr_t)g.rope & 15))) return false;
  } else {
    if (g.rope) return false;
    // the accumulating epilogue updates 4 consecutive floats per 16-byte access through 32-bit byte offsets
    if (!aligned16(g.C) || g.ldc % 4 || g.sC % 4 || g.N % 4) return false;
    if (g.bias || g.resid) return false;
    if (((int64_t)g.M + 256) * g.ldc * 4 >= (1ll << 31)) return false;
  }
  // byte offsets inside one operand are 32-bit in the kernel
  // every part of a multi-part range has a descriptor of its own; the last part may be the longest
  const int64_t rowsA = g.nx ? ((int64_t)g.K - (int64_t)g.nx * g.kseg > g.kseg ? (int64_t)g.K - (int64_t)g.nx * g.kseg : g.kseg) : g.K;
  const int64_t extA = (g.transA ? rowsA * g.lda : (int64_t)g.M * g.lda) * 2;
  const int64_t nseg = g.kseg ? g.K / g.kseg : 1;
  const int64_t nsegB = g.nx ? 1 : nseg;
  const int64_t extB = (g.transB ? (nsegB - 1) * g.segB + (int64_t)g.N * g.ldb : rowsA * g.ldb + (g.glu == 1 ? g.sB : 0)) * 2;
  if (extA >= (1ll << 30) || extB >= (1ll << 30)) return false;
  return true;
}

// Which tile: the MI355X has 256 CUs.  256x256 tiles (8 waves, one workgroup per CU) move the fewest LDS and
// L2 bytes per flop; 128x128 tiles (two workgroups per CU) run at about 0.8 of their rate (measured at
// K = 4096) but waste less of the last round of workgroups and give small problems enough workgroups to
// fill the chip.  The shape with the smaller estimated time wins.
namespace {
// Estimated time of a grid of `small` 128x128 tiles in units of one round of 256x256 tiles: full rounds hold
// 512 small tiles (two per CU, each at 0.8 of the big tile's rate); a remainder of at most 256 tiles runs
// one per CU.
double small_rounds(int64_t small) {
  const int64_t rem = small % 512;
  return ((double)(small / 512) * 2.0 + (rem == 0 ? 0.0 : rem <= 256 ? 1.0 : 2.0)) * 0.25 / 0.8;
}
// Tile columns of a grid of tiles `width` wide: a gate|up tile (glu = 1) covers width/2 columns of each matrix.
int64_t tile_cols(const Gemm& g, int width) { return cdiv(g.N, g.glu == 1 ? width / 2 : width); }
}  // namespace

int gemm_mfma_pick_tile(const Gemm& g) {
  if (g_force_tile) return g_force_tile;
  const int64_t big = cdiv(g.M, 256) * tile_cols(g, 256) * g.batch;
  const int64_t small = cdiv(g.M, 128) * tile_cols(g, 128) * g.batch;
  return small_rounds(small) < (double)cdiv(big, 256) ? 2 : 1;
}

void gemm_mfma_force_tile(int id) { g_force_tile = id; }

namespace {

hipError_t run_tile(hipStream_t st, DType dt, const Gemm& g, bool small) {
  if (dt == F16) return small ? gemm_mfma_128x128_f16(st, g) : gemm_mfma_256x256_f16(st, g);
  return small ? gemm_mfma_128x128(st, g) : gemm_mfma_256x256(st, g);
}

// A grid of 256x256 tiles that ends in a round with few tiles (1376 tiles = 5 rounds + 96 tiles on 256 CUs) pays a
// whole round for them.  When the leading tile columns make up whole rounds exactly, the product is cut along N:
// those columns run on big tiles, the remaining ones on 128x128 tiles, which fill the chip (two workgroups per CU)
// and take about 0.625 of a big round.  Returns false when the shape does not ask for it.
bool split_tail(DType dt, const Gemm& g, Gemm& head, Gemm& tail) {
  const int64_t tm = cdiv(g.M, 256), tn = tile_cols(g, 256);
  const int64_t tiles = tm * tn * g.batch, rem = tiles % 256;
  if (tiles < 256 || rem == 0 || rem > 128) return false;   // up to 128 big tiles make one round of small ones
  const int64_t col = tm * g.batch;                       // tiles per tile column
  if (rem % col) return false;
  const int64_t c1 = tn - rem / col;                      // leading columns: (tiles - rem) tiles, whole rounds
  if (c1 < 1) return false;
  const int64_t n1 = c1 * (g.glu == 1 ? 128 : 256);
  if (g.rope && n1 % g.rope_d) return false;
  head = g; tail = g;
  head.N = (int)n1;
  tail.N = g.N - (int)n1;
  const int64_t cb = g.c_f32_accum ? 4 : 2;
  tail.C = (char*)g.C + n1 * cb;
  if (g.bias) tail.bias = (const char*)g.bias + n1 * 2;
  if (g.resid) tail.resid = (const char*)g.resid + n1 * 2;
  if (g.gu) tail.gu = (char*)g.gu + n1 * 2;
  const int64_t boff = (g.transB ? n1 * g.ldb : n1) * 2;
  tail.B = (const char*)g.B + boff;
  for (int p = 0; p < g.nx; ++p) tail.Bx[p] = (const char*)g.Bx[p] + boff;
  return gemm_mfma_supported(dt, head) && gemm_mfma_supported(dt, tail);
}

}  // namespace

hipError_t gemm_mfma(hipStream_t st, DType dt, const Gemm& g) {
  const bool small = gemm_mfma_pick_tile(g) == 2;
  Gemm head, tail;
  if (!g_force_tile && split_tail(dt, g, head, tail)) {
    // whole rounds of big tiles + the rest on small ones, against the better of the two uniform grids
    const int64_t big = cdiv(g.M, 256) * tile_cols(g, 256) * g.batch;
    const double t_split = (double)(big / 256) + small_rounds(cdiv(tail.M, 128) * tile_cols(tail, 128) * tail.batch);
    const double t_uniform = small ? small_rounds(cdiv(g.M, 128) * tile_cols(g, 128) * g.batch) : (double)cdiv(big, 256);
    if (t_split < t_uniform) {
      const hipError_t e = run_tile(st, dt, head, false);
      return e != hipSuccess ? e : run_tile(st, dt, tail, true);
    }
  }
  return run_tile(st, dt, g, small);
}

}  // namespace zs
