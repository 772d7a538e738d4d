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

// ---- K range of the last round's tiles cut into chunks -------------------------------------------------------------
// A multi-part product whose 256x256 tiles do not fill whole rounds of 256 workgroups runs as two launches of the same
// kernel over ranges of its tile order (counted over all batches): the leading tiles, whole rounds, as they are, and the
// remaining `rem` tiles as rem x nchunks workgroups, each multiplying chunk_parts of the parts.  Chunk 0 adds to C; the
// other chunks leave partial tiles in scratch, which add_partials_kernel adds to C in the order of the chunks.
struct KCut {
  Gemm head, tail;
  int rem = 0;              // tiles of the cut-off range
  int64_t ws_need = 0;      // bytes of partial tiles
};

constexpr int64_t KCUT_MAX_WS = 256ll << 20;   // no plan wants more scratch than this

// Times of the cut-off tiles are estimated in units of one part on one tile, 2*256*256*kseg flops at the 5.3 TFLOP/s a
// CU sustains.  A round of workgroups costs its parts plus about 20 us for its first loads and its store pass; the second
// kernel reads the partial tiles and reads and writes C at about 4 TB/s.  Measured at 11008 x 4096 with 8 parts of 4096 rows:
// 2538 us uncut, 2458 us in 4 chunks of 2 parts (the estimate says 79 us less); with 4 parts a cut costs time, and is not made.
double kcut_part_seconds(int kseg) { return 2.0 * 256.0 * 256.0 * (double)kseg / 5.3e12; }
double kcut_round_fixed_parts(int kseg) { return 20e-6 / kcut_part_seconds(kseg); }
double kcut_fixup_parts(int rem, int nch, int kseg) {
  const double bytes = (double)(nch - 1 + 2) * rem * 256.0 * 256.0 * 4.0;
  return bytes / 4.0e12 / kcut_part_seconds(kseg);
}

bool plan_kcut(DType dt, const Gemm& g, KCut& k) {
  if (!g.nx || !g.c_f32_accum || !g.transA || g.transB || g.kseg < 1) return false;
  const int64_t tm = cdiv(g.M, 256), tn = cdiv(g.N, 256), tiles = tm * tn * g.batch, rem = tiles % 256;
  if (tiles < 256 || rem == 0 || tiles >= (1ll << 30)) return false;
  const int parts = g.nx + 1;
  const double fx = kcut_round_fixed_parts(g.kseg);
  double t_now = (double)parts + fx;                                  // a whole round
  Gemm h2, t2;
  if (split_tail(dt, g, h2, t2))                                      // today's other way: the rest on 128x128 tiles
    t_now = std::min(t_now, small_rounds(cdiv(t2.M, 128) * tile_cols(t2, 128) * t2.batch) * (parts + fx));
  double best = t_now * 0.97;                                         // a cut has to win at least 3 %
  int best_cp = 0;
  for (int cp = 1; cp < parts; ++cp) {
    const int nch = (int)cdiv(parts, cp);
    if ((int64_t)(nch - 1) * rem * 256 * 256 * 4 > KCUT_MAX_WS) continue;
    const double t = (double)cdiv(rem * nch, 256) * (cp + fx) + kcut_fixup_parts((int)rem, nch, g.kseg);
    if (t < best) { best = t; best_cp = cp; }
  }
  if (!best_cp) return false;
  k.rem = (int)rem;
  k.head = g; k.tail = g;
  k.head.ws = nullptr; k.head.ws_bytes = 0; k.head.chunk_parts = 0; k.head.nchunks = 1;
  k.head.tile_base = 0; k.head.tile_count = (int)(tiles - rem);
  k.tail.tile_base = (int)(tiles - rem); k.tail.tile_count = (int)rem;
  k.tail.chunk_parts = best_cp;
  k.tail.nchunks = (int)cdiv(parts, best_cp);
  k.ws_need = (int64_t)(k.tail.nchunks - 1) * rem * 256 * 256 * 4;
  return true;
}

// C tile += partial tile of chunk 1, then of chunk 2, ...: one workgroup per quarter tile (64 rows), 16 bytes per lane.
// Tile `idx` of the range is position tile_base + idx of the tile order.
__global__ __launch_bounds__(256) void add_partials_kernel(float* C, int64_t ldc, int64_t sC, int M, int N, int tiles_m, int tiles_n,
                                                           int tile_base, int tile_count, const float* __restrict__ partial, int nadd) {
  const int idx = blockIdx.x >> 2, quarter = blockIdx.x & 3;
  const int pos = tile_base + idx, ntiles = tiles_m * tiles_n;
  int tm, tn;
  gemm_tile_of(pos % ntiles, tiles_m, tiles_n, tm, tn);
  const int m0 = tm * 256 + quarter * 64, n0 = tn * 256;
  float* Cz = C + (int64_t)(pos / ntiles) * sC;
  const float* P0 = partial + (int64_t)idx * 65536 + quarter * 64 * 256;
  const int64_t chunk_stride = (int64_t)tile_count * 65536;
#pragma unroll 4
  for (int v = threadIdx.x; v < 64 * 64; v += 256) {
    const int r = v >> 6, c = (v & 63) * 4;
    if (m0 + r >= M || n0 + c >= N) continue;                         // N is a multiple of 4
    float* pc = Cz + (int64_t)(m0 + r) * ldc + n0 + c;
    f32x4 s = *reinterpret_cast<const f32x4*>(pc);
    for (int a = 0; a < nadd; ++a) s += *reinterpret_cast<const f32x4*>(P0 + a * chunk_stride + r * 256 + c);
    *reinterpret_cast<f32x4*>(pc) = s;
  }
}

}  // namespace

int64_t gemm_mfma_ws_bytes(const Gemm& g) {
  KCut k;
  return (!g_force_tile && plan_kcut(BF16, g, k)) ? k.ws_need : 0;
}

hipError_t gemm_mfma(hipStream_t st, DType dt, const Gemm& g) {
  const bool small = gemm_mfma_pick_tile(g) == 2;
  if (g.ws && !g_force_tile) {
    KCut k;
    if (plan_kcut(dt, g, k) && k.ws_need <= g.ws_bytes && ((uintptr_t)g.ws & 15) == 0 && gemm_mfma_supported(dt, g)) {
      hipError_t e = run_tile(st, dt, k.head, false);
      if (e != hipSuccess) return e;
      e = run_tile(st, dt, k.tail, false);
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(add_partials_kernel, dim3((unsigned)(k.rem * 4)), dim3(256), 0, st, (float*)g.C, g.ldc, g.sC, g.M, g.N,
                         (int)cdiv(g.M, 256), (int)cdiv(g.N, 256), k.tail.tile_base, k.tail.tile_count, (const float*)g.ws,
                         k.tail.nchunks - 1);
      return hipGetLastError();
    }
  }
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
