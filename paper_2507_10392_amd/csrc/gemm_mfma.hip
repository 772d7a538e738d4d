// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// One workgroup of 4 wavefronts computes a 256x256 tile of C; each wavefront owns a 128x128
// quadrant as 4x4 MFMA blocks of 32x32 (256 accumulator registers per lane).  The K loop walks
// 64-wide slabs.  A slab of each operand is fetched from HBM with 16-byte loads into registers
// one iteration ahead, stored into one of two LDS buffers in the layout the MFMA operands want
// ([row][k], k contiguous, rows padded to 72 elements so that the 16-byte operand reads of 16
// neighbouring lanes fall into distinct banks), and read back as one ds_read_b128 per operand
// fragment.  Operands whose contraction index is not contiguous in memory (B of y = x W with W
// stored [in,out]; both operands of dW = x^T dy) are transposed in registers, 8x8 blocks per
// lane, on their way into LDS, so the inner loop is identical for all four storage variants.
// Workgroup ids are remapped so that the 8 XCDs (ids are dealt round-robin to them) each work
// on a compact patch of C and re-use their own L2's A rows and B columns.
#include "kernels.h"

namespace zs {

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int LDS_LD = BK + 8;                    // padded row length in elements (144 bytes)
constexpr int TILE_ELEMS = BM * LDS_LD;           // one operand slab in LDS
constexpr int NTHREADS = 256;

struct Frag { bf16x8 v[8]; };                     // one thread's share of a 256x64 slab: 8 x 16 bytes

__device__ __forceinline__ bf16x8 zero8() {
  bf16x8 z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = (bf16)0.f;
  return z;
}

// Slab of an operand whose contraction index is contiguous: stored [rows, K], ld = row stride.
// Thread t reads vectors v = t + 256*i: row = v/8, k-vector = v%8 (= t%8 for every i).
__device__ __forceinline__ void load_kmajor(Frag& f, const bf16* __restrict__ base, int64_t ld, int row0, int nrows,
                                            int k0, int K, int tid) {
  const int kv = (tid & 7) * 8;
  const bool kok = k0 + kv < K;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = row0 + (tid >> 3) + 32 * i;
    f.v[i] = (kok && r < nrows) ? *reinterpret_cast<const bf16x8*>(base + (int64_t)r * ld + k0 + kv) : zero8();
  }
}
__device__ __forceinline__ void store_kmajor(const Frag& f, bf16* lds, int tid) {
  const int kv = (tid & 7) * 8;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = (tid >> 3) + 32 * i;
    *reinterpret_cast<bf16x8*>(lds + r * LDS_LD + kv) = f.v[i];
  }
}

// Slab of an operand stored [K, rows] (the tile's row index is contiguous in memory).  Thread t
// owns the 8x8 block  k in kb*8..+8, rows rb*8..+8  with rb = t%32, kb = t/32: 8 loads of 16 bytes.
__device__ __forceinline__ void load_rowmajor(Frag& f, const bf16* __restrict__ base, int64_t ld, int row0, int nrows,
                                              int k0, int K, int tid) {
  const int rb = (tid & 31) * 8, kb = (tid >> 5) * 8;
  const bool rok = row0 + rb < nrows;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int k = k0 + kb + j;
    f.v[j] = (rok && k < K) ? *reinterpret_cast<const bf16x8*>(base + (int64_t)k * ld + row0 + rb) : zero8();
  }
}
// 8x8 transpose in registers, then 8 stores of 16 bytes: LDS row rb+c gets k = kb..kb+7.
__device__ __forceinline__ void store_transposed(const Frag& f, bf16* lds, int tid) {
  const int rb = (tid & 31) * 8, kb = (tid >> 5) * 8;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    bf16x8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = f.v[j][c];
    *reinterpret_cast<bf16x8*>(lds + (rb + c) * LDS_LD + kb) = o;
  }
}

template <int TA, int TB, int SEG>
__global__ __launch_bounds__(NTHREADS) void gemm_mfma_kernel(Gemm g, int tiles_m, int tiles_n) {
  extern __shared__ __align__(16) char smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(smem_raw);        // [2 buffers][A slab | B slab]

  // ---- tile assignment: XCD-aware, then grouped along M
  int pid = blockIdx.x;
  const int ntiles = tiles_m * tiles_n;
  {
    const int per = ntiles / 8;                           // ids [0, 8*per) are remapped, the rest stay
    if (pid < per * 8) pid = (pid % 8) * per + pid / 8;
  }
  constexpr int GROUP = 8;
  const int width = GROUP * tiles_n;
  const int group_id = pid / width;
  const int first_m = group_id * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  const int tm = first_m + (pid % width) % gsz;
  const int tn = (pid % width) / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  const int z = blockIdx.y;
  const bf16* A = (const bf16*)g.A + (int64_t)z * g.sA;
  const bf16* B = (const bf16*)g.B + (int64_t)z * g.sB;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (g.K + BK - 1) / BK;
  Frag fa, fb;

  auto fetch = [&](int kt) {
    const int k0 = kt * BK;
    if (TA == 0) load_kmajor(fa, A, g.lda, m0, g.M, k0, g.K, tid);
    else load_rowmajor(fa, A, g.lda, m0, g.M, k0, g.K, tid);
    if (TB == 1) {
      if (SEG) {  // the thread's k offset inside the slab is fixed, so one segment lookup per slab
        const int k = k0 + (tid & 7) * 8;
        const int seg = k / g.kseg;
        const bf16* Bs = B + (int64_t)seg * g.segB - (int64_t)seg * g.kseg;   // so that Bs[n*ldb + k] is in segment seg
        load_kmajor(fb, Bs, g.ldb, n0, g.N, k0, g.K, tid);
      } else {
        load_kmajor(fb, B, g.ldb, n0, g.N, k0, g.K, tid);
      }
    } else {
      load_rowmajor(fb, B, g.ldb, n0, g.N, k0, g.K, tid);
    }
  };
  auto stash = [&](int buf) {
    bf16* As = smem + buf * 2 * TILE_ELEMS;
    bf16* Bs = As + TILE_ELEMS;
    if (TA == 0) store_kmajor(fa, As, tid); else store_transposed(fa, As, tid);
    if (TB == 1) store_kmajor(fb, Bs, tid); else store_transposed(fb, Bs, tid);
  };

  if (nk > 0) {
    fetch(0);
    stash(0);
  }
  __syncthreads();
  const int lrow = lane & 31, lk = (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) fetch(kt + 1);                      // global loads in flight during the MFMAs below
    const bf16* As = smem + buf * 2 * TILE_ELEMS + (wm + lrow) * LDS_LD + lk;
    const bf16* Bs = smem + buf * 2 * TILE_ELEMS + TILE_ELEMS + (wn + lrow) * LDS_LD + lk;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const bf16x8*>(As + i * 32 * LDS_LD + ks * 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = *reinterpret_cast<const bf16x8*>(Bs + j * 32 * LDS_LD + ks * 16);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) stash(buf ^ 1);                     // the other buffer was last read before the previous barrier
    __syncthreads();
  }

  // ---- epilogue.  acc[i][j][r] is C[row, col] with row = 8*(r/4) + 4*(lane/32) + r%4, col = lane%32 of the block.
  const bf16* bias = g.bias ? (const bf16*)g.bias + (int64_t)z * g.sBias : nullptr;
  const bf16* R = g.resid ? (const bf16*)g.resid + (int64_t)z * g.sC : nullptr;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int col = n0 + wn + j * 32 + (lane & 31);
    if (col >= g.N) continue;
    const float bv = bias ? (float)bias[col] : 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row >= g.M) continue;
        float v = acc[i][j][r] + bv;
        if (R) v += (float)R[(int64_t)row * g.ldr + col];
        if (g.c_f32_accum) {
          float* C = (float*)g.C + (int64_t)z * g.sC + (int64_t)row * g.ldc + col;
          *C += v;
        } else {
          bf16* C = (bf16*)g.C + (int64_t)z * g.sC + (int64_t)row * g.ldc + col;
          *C = (bf16)v;
        }
      }
    }
  }
}

constexpr size_t SMEM_BYTES = 2 * 2 * TILE_ELEMS * sizeof(bf16);   // 147456

template <int TA, int TB, int SEG> hipError_t launch(hipStream_t st, const Gemm& g) {
  static bool configured = false;
  auto kern = gemm_mfma_kernel<TA, TB, SEG>;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_m = (int)cdiv(g.M, BM), tiles_n = (int)cdiv(g.N, BN);
  dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)g.batch), blk(NTHREADS);
  hipLaunchKernelGGL(kern, grid, blk, SMEM_BYTES, st, g, tiles_m, tiles_n);
  return hipGetLastError();
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

// The kernel needs 16-byte aligned rows for its vector loads: base pointers 16-byte aligned and
// every leading dimension, batch stride and segment size a multiple of 8 elements; the extent
// along each operand's contiguous axis must be a multiple of 8 as well.
bool gemm_mfma_supported(DType dt, const Gemm& g) {
  if (dt != BF16) return false;
  if (g.M < 1 || g.N < 1 || g.K < 1 || g.batch < 1) return false;
  if (!aligned16(g.A) || !aligned16(g.B)) return false;
  if (g.lda % 8 || g.ldb % 8 || g.sA % 8 || g.sB % 8) return false;
  if (g.K % 8) return false;                       // k-contiguous operands are read 8 k at a time; tails are zero-filled
  if (g.transA && g.M % 8) return false;           // row-contiguous operands are read 8 rows at a time
  if (!g.transB && g.N % 8) return false;
  if (g.kseg) {
    if (!g.transB || g.kseg % 8 || g.segB % 8 || g.K % g.kseg) return false;
  }
  return true;
}

hipError_t gemm_mfma(hipStream_t st, const Gemm& g) {
  if (g.kseg) {
    return g.transA ? launch<1, 1, 1>(st, g) : launch<0, 1, 1>(st, g);
  }
  if (!g.transA && !g.transB) return launch<0, 0, 0>(st, g);
  if (!g.transA && g.transB) return launch<0, 1, 0>(st, g);
  if (g.transA && !g.transB) return launch<1, 0, 0>(st, g);
  return launch<1, 1, 0>(st, g);
}

}  // namespace zs
