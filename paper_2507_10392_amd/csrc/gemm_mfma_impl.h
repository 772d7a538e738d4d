// 16-bit (bf16 or IEEE half) GEMM on the CDNA4 matrix cores (v_mfma_f32_16x16x32_bf16 / _f16), fp32 accumulation: the tile kernel,
// templated on the workgroup tile BM x BN and the number of wavefronts.
//
// One workgroup of 4 (2 x 2) or 8 (2 x 4) wavefronts computes a BM x BN tile of C; each wavefront owns
// its part as MFMA blocks of 16x16 (4 accumulator registers per block and lane).
// The K loop walks 64-wide slabs.  A slab of each operand is fetched from HBM with 16-byte buffer
// loads into registers one iteration ahead and stored into one of two LDS buffers:
//   * contraction index contiguous in memory  -> LDS [row][k], 128-byte rows whose 16-byte pieces are
//     permuted by the row index (piece p of row r at position p ^ r%8); an MFMA operand fragment
//     (8 consecutive k of one row) is one ds_read_b128;
//   * row index contiguous in memory (B of y = x W with W stored [in,out]; both operands of
//     dW = x^T dy) -> LDS [k][row], k-lines padded by 32 elements, pairs of 16-row chunks swapped on
//     the odd eights of k; the fragment is two ds_read_b64_tr_b16, the LDS transpose read of gfx950,
//     each returning 4 consecutive k.
// Permutation and padding keep slab stores and fragment reads free of bank conflicts (measured per
// access pattern: the LDS does not serve a wave's 16-byte accesses in groups of 16 consecutive lanes).
// Workgroup ids are remapped so that the 8 XCDs (ids are dealt round-robin to them) each work
// on a compact patch of C and re-use their own L2's A rows and B columns.
// The 256x256 tile runs 8 wavefronts (128 accumulator registers each, two waves per SIMD); the 128x128 tile
// runs 4 and needs 64 accumulator registers and 74 KB of LDS, so two workgroups share a CU.  Either way a
// SIMD always has a second wave to issue MFMAs while the first waits for memory, LDS or a barrier.
#pragma once
#include "kernels.h"

namespace zs {
namespace gemm_impl {

constexpr int BK = 64;
constexpr int LDK = BK;                           // [row][k] layout: 128-byte rows, no padding; the 16-byte piece p of row r sits at
                                                  // position p ^ (r % 8), which keeps both the slab stores (8 rows x 8 pieces per wave)
                                                  // and the fragment reads (16 rows x 4 pieces per wave) free of bank conflicts
// [k][row] slabs: k-lines are padded by RPAD elements.  A transpose read serves 32 lanes per cycle, which
// touch 8 k-lines x 32 bytes; k-lines are 16 banks apart (mod 64) and the chunk swap of store_rmajor moves
// the second four lines by 8 banks, so those are 64 different banks.
constexpr int RPAD = 32;
constexpr int slab_elems(int R) { return R * LDK > BK * (R + RPAD) ? R * LDK : BK * (R + RPAD); }

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

template <int R, int NT> struct Frag { u32x4 v[R * 8 / NT]; };   // one thread's share of an R x 64 slab, 16 bytes each

// Operands are read through raw buffer descriptors: the per-lane offset is one VGPR, the per-load
// offset a scalar, and anything at or beyond num_records reads as zero, which handles the ragged edge
// along each operand's OUTER dimension for free.  Along the inner (contiguous) dimension the pieces past
// the edge get a per-lane offset that is out of range (DEAD, below).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
// A per-lane byte offset of DEAD lies beyond every num_records (operand extents are below 2^30 bytes), so a
// lane whose piece must read as zero is simply sent there: no masks or branches in the K loop.
constexpr int DEAD = 0x40000000;

// Operand stored [rows, K] (k contiguous), ld = row stride.  With NT threads, thread t carries vectors
// v = t + NT*i: row = v/8, k-vector = v%8 (= t%8 for every i).  voff = ((t/8)*ld + (t%8)*8)*2 bytes (+ segment shift).
// Rows past the operand's last row lie beyond num_records; k-vectors at or past K (ragged last slab, and
// slabs past the end) would run into the next row and are sent out of range.
template <int R, int NT>
__device__ __forceinline__ void load_kmajor(Frag<R, NT>& f, __amdgpu_buffer_rsrc_t rs, int voff, int ld, int row0, int k0,
                                            int K, int tid, int i0 = 0, int i1 = R * 8 / NT) {
  const int vo = k0 + (tid & 7) * 8 >= K ? DEAD : voff;
#pragma unroll
  for (int i = 0; i < R * 8 / NT; ++i)
    if (i >= i0 && i < i1) f.v[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, vo, ((row0 + (NT / 8) * i) * ld + k0) * 2, 0);
}
// (load_kmajor, like the other three, handles vectors [i0, i1) of the thread's share)
template <int R, int NT>
__device__ __forceinline__ void store_kmajor(const Frag<R, NT>& f, bf16* lds, int tid, int i0 = 0, int i1 = R * 8 / NT) {
  static_assert((NT / 8) % 8 == 0, "a thread's row keeps its value mod 8 over the passes");
  bf16* p = lds + (tid >> 3) * LDK + (((tid & 7) ^ ((tid >> 3) & 7)) * 8);
#pragma unroll
  for (int i = 0; i < R * 8 / NT; ++i)
    if (i >= i0 && i < i1) *reinterpret_cast<u32x4*>(p + (NT / 8) * i * LDK) = f.v[i];
}

// Operand stored [K, rows] (row index contiguous).  A k-line of the slab is R/8 vectors; thread t carries
// vectors v = t + NT*i: k = v/(R/8), row-vector = v%(R/8) (= t%(R/8) for every i).
// Row-vectors at or past the operand's last row (ragged edge tile) would read the next k-line: out of range.
template <int R> __device__ __forceinline__ int voff_rmajor(int ld, int tid, int row0, int nrows) {
  return row0 + (tid % (R / 8)) * 8 >= nrows ? DEAD : ((tid / (R / 8)) * ld + (tid % (R / 8)) * 8) * 2;
}
// The same for a tile whose first R/2 rows come from one matrix (rows row0 .. of `nrows`) and whose last R/2 rows
// are the same rows of a second matrix lying `second` elements behind the first: gate and up projections side by side.
template <int R> __device__ __forceinline__ int voff_rmajor_two(int ld, int tid, int row0, int nrows, int second) {
  constexpr int PER = R / 8, HALF = PER / 2;
  const int j = tid % PER, jj = j % HALF;
  return row0 + jj * 8 >= nrows ? DEAD : ((tid / PER) * ld + jj * 8 + (j >= HALF ? second : 0)) * 2;
}
template <int R, int NT>
__device__ __forceinline__ void load_rmajor(Frag<R, NT>& f, __amdgpu_buffer_rsrc_t rs, int voff, int ld, int row0, int k0,
                                            int i0 = 0, int i1 = R * 8 / NT) {
  constexpr int KSTEP = NT / (R / 8);             // k-lines covered by one pass of the NT threads
#pragma unroll
  for (int i = 0; i < R * 8 / NT; ++i)
    if (i >= i0 && i < i1) f.v[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, ((k0 + KSTEP * i) * ld + row0) * 2, 0);
}
template <int R, int NT>
__device__ __forceinline__ void store_rmajor(const Frag<R, NT>& f, bf16* lds, int tid, int i0 = 0, int i1 = R * 8 / NT) {
  constexpr int KSTEP = NT / (R / 8), LDR = R + RPAD;
  static_assert(KSTEP % 16 == 0, "bit 3 of a thread's k-line must not depend on the pass");
  const int kl = tid / (R / 8);                   // k-line of pass 0; passes add multiples of 16
  bf16* p = lds + kl * LDR + (((tid % (R / 8)) ^ (((kl >> 3) & 1) << 1)) * 8);   // 16-row chunks swap in pairs on odd eights of k
#pragma unroll
  for (int i = 0; i < R * 8 / NT; ++i)
    if (i >= i0 && i < i1) *reinterpret_cast<u32x4*>(p + KSTEP * i * LDR) = f.v[i];
}

// MFMA operand fragment for lane (row = lane%16, g = lane/16): the 8 values k = k32 + 8g .. +7 of that row
// (row0 is a multiple of 16, so the row's value mod 8 is the lane's).
__device__ __forceinline__ bf16x8 frag_kmajor(const bf16* tile, int row0, int k32, int lane) {
  return *reinterpret_cast<const bf16x8*>(tile + (row0 + (lane & 15)) * LDK + (((k32 >> 3) + (lane >> 4)) ^ (lane & 7)) * 8);
}
// Same fragment from a [k][row] tile.  One transpose read serves 16 lanes: lane r of the group points at
// 4 consecutive rows of k-line (r/4) and receives the 4 k-lines' values of ONE row; group g reads k-lines k32 + 8g ...
// The LDS serves two groups per cycle, here the SAME 16 rows of k-lines 8 apart, i.e. the same banks; so the slab is
// stored with each pair of 16-row chunks swapped on the odd eights of k (store_rmajor), and the read undoes it.
template <int R> __device__ __forceinline__ bf16x8 frag_rmajor(const bf16* tile, int row0, int k32, int lane) {
  constexpr int LDR = R + RPAD;
  const int r = lane & 15, gi = lane >> 4;
  const bf16* p = tile + (k32 + 8 * gi + (r >> 2)) * LDR + ((row0 + 4 * (r & 3)) ^ ((gi & 1) << 4));
  union { struct { s16x4 a, b; } s; bf16x8 v; } u;
  u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
  u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * LDR));
  return u.v;
}

// Workgroup id -> tile origin.  Ids are dealt round-robin to the 8 XCDs, so id%8 picks the XCD; each XCD
// is given a contiguous run of the tile order, and that order walks groups of 8 tile rows column by
// column, so the tiles an XCD works on at one time share A rows and B columns in its L2.
template <int BM, int BN>
__device__ __forceinline__ void tile_origin(int pid, int tiles_m, int tiles_n, int& m0, int& n0) {
  const int ntiles = tiles_m * tiles_n;
  const int per = ntiles / 8;                             // ids [0, 8*per) are remapped, the rest stay
  if (pid < per * 8) pid = (pid % 8) * per + pid / 8;
  int tm, tn;
  gemm_tile_of(pid, tiles_m, tiles_n, tm, tn);
  m0 = tm * BM;
  n0 = tn * BN;
}

// Both epilogues pass the tile through LDS (free after the K loop) as fp32, in two halves of BM/2 rows.
// The MFMAs were issued with the operands swapped, mfma(B fragment, A fragment), which yields the
// transposed block: acc[i][j][r] is C[row, col] of 16x16 block (i, j) with row = lane%16 and col = 4*(lane/16) + r,
// so a lane owns 4 consecutive columns per block and writes them as one float4.
template <int BN> struct Staging { static constexpr int LDW = BN + 4; };   // padded row (floats)

template <int BN, int MI, int NJ>
__device__ __forceinline__ void stage_quads(float* stage, f32x4 (&acc)[MI][NJ], int wn, int lane) {
  constexpr int LDW = Staging<BN>::LDW;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
      *reinterpret_cast<f32x4*>(stage + (i * 16 + (lane & 15)) * LDW + wn + j * 16 + 4 * (lane >> 4)) = acc[i][j];
}

// Epilogue for C (fp32) += product (no bias, no residual).  Ct points at the tile's first element, of which rows x cols
// exist.  After staging, ALL threads walk the half tile 4 columns at a time: the old values of C are loaded 16 bytes per
// lane (consecutive lanes, consecutive pieces of a row), all loads of a half in flight across the barrier, then sum and
// store.  Loads and stores go through a buffer descriptor over the tile: rows past the last one fall beyond num_records
// and columns past the last one are sent there, so the ragged edge needs no branches.  A tile belongs to one workgroup and
// launches are ordered by the stream, so the sum over microbatches is formed in a fixed order.  overwrite: the tile is
// stored as it is (a partial sum that another kernel adds to C).
template <int BM, int BN, int NT, int MI, int NJ>
__device__ __forceinline__ void epilogue_accum(float* Ct, int ldc, int rows, int cols, bool overwrite, f32x4 (&acc)[MI][NJ],
                                               int wave_m, int wn, int tid, float* stage) {
  constexpr int LDW = Staging<BN>::LDW;
  static_assert((BM / 2) * LDW * 4 <= 2 * (slab_elems(BM) + slab_elems(BN)) * 2, "staging tile must fit the K-loop buffers");
  constexpr int VPR = BN / 4;                              // float4 per row
  constexpr int NV = (BM / 2) * VPR / NT;                  // float4 per thread and half
  const __amdgpu_buffer_rsrc_t rsC = make_rsrc(Ct, (uint32_t)((int64_t)(rows - 1) * ldc + cols) * 4u);
  const int lr0 = tid / VPR, cv = tid % VPR;               // vector v = tid + NT*it: row lr0 + (NT/VPR)*it, same columns
  const bool col_ok = cv * 4 < cols;                       // cols is a multiple of 4
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    __syncthreads();
    if (wave_m == half) stage_quads<BN, MI, NJ>(stage, acc, wn, tid & 63);
    u32x4 old[NV];
    uint32_t off[NV];
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int row = half * (BM / 2) + lr0 + (NT / VPR) * it;
      off[it] = col_ok ? (uint32_t)(row * ldc + cv * 4) * 4u : 0x80000000u;
      old[it] = overwrite ? u32x4{0u, 0u, 0u, 0u} : __builtin_amdgcn_raw_buffer_load_b128(rsC, (int)off[it], 0, 0);
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const f32x4 x = *reinterpret_cast<const f32x4*>(stage + (lr0 + (NT / VPR) * it) * LDW + cv * 4);
      union { u32x4 u; f32x4 f; } o;
      o.u = old[it];
      o.f += x;
      __builtin_amdgcn_raw_buffer_store_b128(o.u, rsC, (int)off[it], 0, 0);
    }
  }
}

// The matrix-core instruction for the element type E; fragments travel as 16-bit containers (bf16x8).
// 16x16x32 rather than 32x32x16: the same flops per cycle, but per flop it moves a fifth fewer register bytes (A, B, C
// and D of one instruction), and the chip, which runs these kernels at its power limit, clocks higher for it: with random
// operands in registers and no memory traffic 2.08 PFLOP/s are sustained against 1.79-1.85.
template <typename E> __device__ __forceinline__ f32x4 mfma_16x16x32(bf16x8 a, bf16x8 b, f32x4 c);
template <> __device__ __forceinline__ f32x4 mfma_16x16x32<bf16>(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x4 mfma_16x16x32<f16>(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Epilogue for 16-bit output (E = bf16 or IEEE half): after staging, ALL threads read rows back 8 columns at a time, add bias and
// residual in fp32, round once to bf16 and store 16 bytes per lane, consecutive lanes covering
// consecutive 16-byte pieces of a row of C.  A thread keeps its 8 columns through all rows it visits, so the bias is
// loaded once, and what depends on the row (residual, rotary angles, or the gate and up values of GLU = 2) is loaded
// for a whole half before the staging barrier: the loads' latency runs under the staging instead of once per row.
template <typename E, int BM, int BN, int NT, int MI, int NJ, int GLU>
__device__ __forceinline__ void epilogue_store(const Gemm& g, int z, f32x4 (&acc)[MI][NJ], int m0, int n0, int wave_m,
                                               int wn, int tid, float* stage) {
  constexpr int LDW = Staging<BN>::LDW;
  static_assert((BM / 2) * LDW * 4 <= 2 * (slab_elems(BM) + slab_elems(BN)) * 2, "staging tile must fit the K-loop buffers");
  constexpr int VPR = BN / 8;                              // 16-byte output vectors per row
  constexpr int NV = (BM / 2) * VPR / NT;                  // vectors per thread and half
  constexpr int RSTEP = NT / VPR;                          // rows between a thread's consecutive vectors
  static_assert(NT % VPR == 0 && ((BM / 2) * VPR) % NT == 0, "a thread keeps its columns");
  typedef typename Vec<E>::type E8;
  const int lane = tid & 63;
  const E* bias = g.bias ? (const E*)g.bias + (int64_t)z * g.sBias : nullptr;
  const E* R = g.resid ? (const E*)g.resid + (int64_t)z * g.sC : nullptr;
  E* Cz = (E*)g.C + (int64_t)z * g.sC;
  const bool rope = g.rope && z < g.rope_batches;
  const int lr0 = tid / VPR, cv = (tid % VPR) * 8, col = n0 + cv;
  const bool full = col + 8 <= g.N;                        // all 8 columns exist: the vector path
  const bool pre_resid = GLU == 0 && R, pre_rope = GLU == 0 && rope && !R;
  E8 bb = {};
  if (GLU == 0 && bias && full) bb = *reinterpret_cast<const E8*>(bias + col);
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    __syncthreads();                                       // K-loop reads / previous half's reads are done
    const int row0 = m0 + half * (BM / 2) + lr0;
    u32x4 pre0[NV], pre1[NV];                              // one source address per slot, so each slot has one load
    const bool want0 = full && (GLU == 2 || pre_resid || pre_rope), want1 = full && (GLU == 2 || pre_rope);
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int row = row0 + RSTEP * it;
      const E* src0 = nullptr;
      const E* src1 = nullptr;
      if (GLU == 2) {
        src0 = (const E*)g.gu + (int64_t)row * g.gu_ld + col;
        src1 = src0 + g.gu_up;
      } else if (pre_resid) {
        src0 = R + (int64_t)row * g.ldr + col;
      } else if (pre_rope) {                               // (cos, sin) of pairs 0,1 and 2,3 at this row's position
        const float2* cs = g.rope + (int64_t)(row % g.rope_S) * (g.rope_d / 2) + (col % g.rope_d) / 2;
        src0 = reinterpret_cast<const E*>(cs);
        src1 = reinterpret_cast<const E*>(cs + 2);
      }
      pre0[it] = pre1[it] = u32x4{0, 0, 0, 0};
      if (want0 && row < g.M) pre0[it] = *reinterpret_cast<const u32x4*>(src0);
      if (want1 && row < g.M) pre1[it] = *reinterpret_cast<const u32x4*>(src1);
    }
    if (wave_m == half) stage_quads<BN, MI, NJ>(stage, acc, wn, lane);
    __syncthreads();
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int lr = lr0 + RSTEP * it, row = row0 + RSTEP * it;
      if (row >= g.M || col >= g.N) continue;
      const f32x4 x0 = *reinterpret_cast<const f32x4*>(stage + lr * LDW + cv);
      const f32x4 x1 = *reinterpret_cast<const f32x4*>(stage + lr * LDW + cv + 4);
      float x[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
      if (GLU == 2) {   // x is da: (gate, up) of these 8 columns become (dgate, dup) in place (N is a multiple of 8)
        E* pg = (E*)g.gu + (int64_t)row * g.gu_ld + col;
        const E8 gg = __builtin_bit_cast(E8, pre0[it]), uu = __builtin_bit_cast(E8, pre1[it]);
        E8 og, ou;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float dg, du;
          glu_df(x[e], (float)gg[e], (float)uu[e], dg, du);
          og[e] = (E)dg;
          ou[e] = (E)du;
        }
        *reinterpret_cast<E8*>(pg) = og;
        *reinterpret_cast<E8*>(pg + g.gu_up) = ou;
        continue;
      }
      if (full) {
        if (bias) {
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] += (float)bb[e];
        }
        if (R) {
          const E8 rr = __builtin_bit_cast(E8, pre0[it]);
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] += (float)rr[e];
        }
        if (rope) {   // rotate the 4 adjacent pairs by the angles of this row's position
          f32x4 t0, t1;
          if (pre_rope) {
            t0 = __builtin_bit_cast(f32x4, pre0[it]);
            t1 = __builtin_bit_cast(f32x4, pre1[it]);
          } else {
            const f32x4* cs = reinterpret_cast<const f32x4*>(g.rope + (int64_t)(row % g.rope_S) * (g.rope_d / 2) + (col % g.rope_d) / 2);
            t0 = cs[0];
            t1 = cs[1];
          }
          const float c4[4] = {t0[0], t0[2], t1[0], t1[2]}, s4[4] = {t0[1], t0[3], t1[1], t1[3]};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float u = x[2 * i], w = x[2 * i + 1];
            x[2 * i] = u * c4[i] - w * s4[i];
            x[2 * i + 1] = u * s4[i] + w * c4[i];
          }
        }
        E8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (E)x[e];
        *reinterpret_cast<E8*>(Cz + (int64_t)row * g.ldc + col) = o;
      } else {
        for (int e = 0; e < 8 && col + e < g.N; ++e) {
          float y = x[e];
          if (bias) y += (float)bias[col + e];
          if (R) y += (float)R[(int64_t)row * g.ldr + col + e];
          Cz[(int64_t)row * g.ldc + col + e] = (E)y;
        }
      }
    }
  }
}

// Epilogue of the gate|up projection (GLU = 1): the tile's first BN/2 columns are gate columns c0 .. and its last
// BN/2 the up columns of the same index.  Both are rounded and stored into gu, and silu(gate) * up of the rounded
// values goes to C: the three arrays the batched product followed by the activation kernel would leave.
template <typename E, int BM, int BN, int NT, int MI, int NJ>
__device__ __forceinline__ void epilogue_glu(const Gemm& g, f32x4 (&acc)[MI][NJ], int m0, int c0, int wave_m, int wn, int tid,
                                             float* stage) {
  constexpr int LDW = Staging<BN>::LDW;
  typedef typename Vec<E>::type E8;
  const int lane = tid & 63;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    __syncthreads();
    if (wave_m == half) stage_quads<BN, MI, NJ>(stage, acc, wn, lane);
    __syncthreads();
    constexpr int VPR = BN / 16;                           // 8-column pieces of each matrix per row
#pragma unroll
    for (int it = 0; it < (BM / 2) * VPR / NT; ++it) {
      const int v = tid + NT * it;
      const int lr = v / VPR, cv = (v % VPR) * 8, col = c0 + cv;
      const int row = m0 + half * (BM / 2) + lr;
      if (row >= g.M || col >= g.N) continue;              // N is a multiple of 8
      const float* sp = stage + lr * LDW + cv;
      const f32x4 g0 = *reinterpret_cast<const f32x4*>(sp), g1 = *reinterpret_cast<const f32x4*>(sp + 4);
      const f32x4 u0 = *reinterpret_cast<const f32x4*>(sp + BN / 2), u1 = *reinterpret_cast<const f32x4*>(sp + BN / 2 + 4);
      E8 og, ou, oa;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        og[e] = (E)(e < 4 ? g0[e & 3] : g1[e & 3]);
        ou[e] = (E)(e < 4 ? u0[e & 3] : u1[e & 3]);
        oa[e] = (E)glu_f((float)og[e], (float)ou[e]);
      }
      E* pg = (E*)g.gu + (int64_t)row * g.gu_ld + col;
      *reinterpret_cast<E8*>(pg) = og;
      *reinterpret_cast<E8*>(pg + g.gu_up) = ou;
      *reinterpret_cast<E8*>((E*)g.C + (int64_t)row * g.ldc + col) = oa;
    }
  }
}

// NW wavefronts: 4 as a 2 x 2 grid, or 8 as 2 (m) x 4 (n), in which case two waves share each SIMD and one
// wave's loads, LDS traffic and barrier waits overlap the other's MFMAs.
template <typename E, int BM, int BN, int NW, int TA, int TB, int SEG, int ACC, int GLU>
__global__ __launch_bounds__(64 * NW, (NW == 4 && BM * BN <= 128 * 128) ? 2 : 1) void gemm_mfma_kernel(Gemm g, int tiles_m,
                                                                                                        int tiles_n) {
  constexpr int NT = 64 * NW, WN = NW / 2;               // threads; waves along n (2 along m)
  constexpr int MI = BM / 32, NJ = BN / (16 * WN);       // 16x16 blocks per wave along m and n
  constexpr int SLAB_A = slab_elems(BM), SLAB_B = slab_elems(BN);   // LDS elements per operand slab, either layout
  extern __shared__ __align__(16) char smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(smem_raw);        // [2 buffers][A slab | B slab]

  // A launch of a cut product (multi-part K, fp32 accumulation) covers tile_count positions of the tile order from tile_base
  // on, counted over all batches; its ids are dealt to the XCDs like those of a whole grid.
  int m0, n0, z = blockIdx.y, sub = 0;                    // sub: position inside the launch's range
  if (SEG && TA == 1 && TB == 0 && ACC && g.tile_count > 0) {
    const int per = g.tile_count / 8;
    sub = blockIdx.x;
    if (sub < per * 8) sub = (sub % 8) * per + sub / 8;
    const int pos = g.tile_base + sub, ntiles = tiles_m * tiles_n;
    int tm, tn;
    gemm_tile_of(pos % ntiles, tiles_m, tiles_n, tm, tn);
    z = pos / ntiles;
    m0 = tm * BM;
    n0 = tn * BN;
  } else {
    tile_origin<BM, BN>(blockIdx.x, tiles_m, tiles_n, m0, n0);
  }
  const bf16* A = (const bf16*)g.A + (int64_t)z * g.sA;
  const bf16* B = (const bf16*)g.B + (int64_t)z * g.sB;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave / WN) * (BM / 2), wn = (wave % WN) * (BN / WN);
  static_assert(GLU == 0 || (GLU == 1 && !TA && !TB && !SEG && !ACC) || (GLU == 2 && !TA && TB && !SEG && !ACC), "fused gated unit");
  const int nb0 = GLU == 1 ? n0 / 2 : n0;                // first column of the tile inside B (GLU = 1: inside each of the two)

  f32x4 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

  const int nk = (g.K + BK - 1) / BK;
  // Two register stages.  While slab kt is multiplied out of one LDS buffer, slab kt+1 (loaded during the
  // previous iteration) is written into the other buffer BETWEEN the MFMA steps, and the loads of slab
  // kt+2 are in flight.  The LDS writes thereby overlap MFMAs instead of forming a phase of their own in
  // which every wave of the workgroup writes and the matrix cores idle.
  Frag<BM, NT> fa0, fa1;
  Frag<BN, NT> fb0, fb1;
  const int lda = (int)g.lda, ldb = (int)g.ldb;
  // PAIR: the K range is made of g.nx+1 parts of kseg rows, each with operands of its own (both row-contiguous)
  constexpr bool PAIR = SEG && TA == 1 && TB == 0;
  const int K1 = PAIR ? g.kseg : g.K;                    // rows of a part (or of the only one)
  const __amdgpu_buffer_rsrc_t rsA =
      make_rsrc(A, (uint32_t)(TA == 0 ? ((int64_t)(g.M - 1) * lda + g.K) : ((int64_t)(K1 - 1) * lda + g.M)) * 2u);
  const int nseg = (SEG && !PAIR) ? g.K / g.kseg : 1;
  const __amdgpu_buffer_rsrc_t rsB = make_rsrc(
      B, (uint32_t)(TB == 1 ? ((int64_t)(nseg - 1) * g.segB + (int64_t)(g.N - 1) * ldb + (SEG ? g.kseg : g.K))
                            : ((int64_t)(K1 - 1) * ldb + g.N + (GLU == 1 ? g.sB : 0))) * 2u);
  // Descriptors of part p >= 1 (the last part has the rows that remain); a part past the last one gets an empty
  // range, so a surplus slab reads zeros.
  // A launch may cut the K range into chunks of chunk_parts parts (grid.z chunks): this workgroup then multiplies the
  // parts p0..p1 only; chunk 0 adds its tile to C, the others store theirs as partial sums.
  const int chunk = (PAIR && ACC) ? (int)blockIdx.z : 0;
  const int cparts = (PAIR && ACC && g.chunk_parts > 0 && gridDim.z > 1) ? g.chunk_parts : g.nx + 1;
  const int p0 = chunk * cparts, p1 = min(g.nx, p0 + cparts - 1);
  auto part_a = [&](int p) {
    const int rows = p < g.nx ? K1 : g.K - g.nx * K1;
    return (p >= 1 && p <= p1) ? make_rsrc((const bf16*)g.Ax[p - 1] + (int64_t)z * g.sA, (uint32_t)((int64_t)(rows - 1) * lda + g.M) * 2u)
                               : make_rsrc(A, 0u);
  };
  auto part_b = [&](int p) {
    const int rows = p < g.nx ? K1 : g.K - g.nx * K1;
    return (p >= 1 && p <= p1) ? make_rsrc((const bf16*)g.Bx[p - 1] + (int64_t)z * g.sB, (uint32_t)((int64_t)(rows - 1) * ldb + g.N) * 2u)
                               : make_rsrc(B, 0u);
  };
  // PAIR: descriptors of the part whose slabs are being loaded
  __amdgpu_buffer_rsrc_t curA = p0 == 0 ? rsA : part_a(p0), curB = p0 == 0 ? rsB : part_b(p0);
  const int voffA = TA == 0 ? ((tid >> 3) * lda + (tid & 7) * 8) * 2 : voff_rmajor<BM>(lda, tid, m0, g.M);
  const int voffB = TB == 1     ? ((tid >> 3) * ldb + (tid & 7) * 8) * 2
                    : GLU == 1 ? voff_rmajor_two<BN>(ldb, tid, nb0, g.N, (int)g.sB)
                               : voff_rmajor<BN>(ldb, tid, n0, g.N);

  constexpr int VA = BM * 8 / NT, VB = BN * 8 / NT;        // 16-byte vectors per thread and slab
  static_assert(VA % 4 == 0 && VB % 4 == 0, "a quarter of the slab is stored per MFMA step");
  // Loads vectors [i0, i1) of the thread's share of slab kt, counted over the A vectors followed by the B vectors.
  auto fetch = [&](int kt, Frag<BM, NT>& fa0, Frag<BN, NT>& fb0, int i0 = 0, int i1 = 1 << 20) {
    const int k0 = kt * BK;
    if (TA == 0) load_kmajor<BM, NT>(fa0, rsA, voffA, lda, m0, k0, g.K, tid, i0, i1);
    else load_rmajor<BM, NT>(fa0, rsA, voffA, lda, m0, k0, i0, i1);
    if (TB == 1) {
      int vo = voffB;
      if (SEG && !PAIR) {  // the thread's k offset inside the slab is fixed, so one segment lookup per slab
        const int seg = (k0 + (tid & 7) * 8) / g.kseg;
        vo += seg * ((int)g.segB - g.kseg) * 2;          // element (n, k) of segment seg lies at seg*segB + n*ldb + k - seg*kseg
      }
      load_kmajor<BN, NT>(fb0, rsB, vo, ldb, n0, k0, g.K, tid, i0 - VA, i1 - VA);
    } else {
      load_rmajor<BN, NT>(fb0, rsB, voffB, ldb, nb0, k0, i0 - VA, i1 - VA);
    }
  };
  auto stash_a = [&](int buf, const Frag<BM, NT>& fa, int i0 = 0, int i1 = 64) {
    bf16* As = smem + buf * (SLAB_A + SLAB_B);
    if (TA == 0) store_kmajor<BM, NT>(fa, As, tid, i0, i1); else store_rmajor<BM, NT>(fa, As, tid, i0, i1);
  };
  auto stash_b = [&](int buf, const Frag<BN, NT>& fb, int i0 = 0, int i1 = 64) {
    bf16* Bs = smem + buf * (SLAB_A + SLAB_B) + SLAB_A;
    if (TB == 1) store_kmajor<BN, NT>(fb, Bs, tid, i0, i1); else store_rmajor<BN, NT>(fb, Bs, tid, i0, i1);
  };
  // multiplies the slab in LDS buffer `buf`; after each of the four MFMA steps it writes a quarter of the
  // next slab (held in fa, fb) into the other buffer, which nobody reads now.  The loads of the slab after that
  // are issued an eighth at a time, after every half MFMA step (`load(i0, i1)` loads vectors [i0, i1) of the thread's
  // share): the CU's load unit takes 16 cycles per 1 KB wave load, and a wave that issues its whole share at once
  // (64 loads per workgroup and slab, all waves at the same point of the loop) waits in that unit's queue for
  // hundreds of cycles in which it issues no MFMA.  The scheduling fences keep the compiler from gathering the loads
  // at the end of the loop body again.
  constexpr int VL = (VA + VB) / 8;                        // vectors per load group
  static_assert(MI == 8 || MI == 4, "a load group and a stash quarter go out after every MI/4 rows of MFMA blocks");
  // A slab is multiplied in 8 regions of MI/4 rows of blocks each.  The schedule is laid down by hand, with scheduling
  // fences between its parts: a region first issues the LDS reads of the NEXT region's fragments, then its own MFMAs,
  // then a quarter of one operand's share of the next slab's stores (A and B in turn), then its share of the global loads.
  auto multiply = [&](int buf, const Frag<BM, NT>& fa, const Frag<BN, NT>& fb, auto&& load) {
    const bf16* As = smem + buf * (SLAB_A + SLAB_B);
    const bf16* Bs = As + SLAB_A;
    constexpr int RI = MI / 4;                             // rows of blocks per region
    bf16x8 a[2][RI], b[2][NJ];
    auto read_a = [&](int e) {                             // fragments of region e = 4 ks + q
#pragma unroll
      for (int ii = 0; ii < RI; ++ii) {
        const int row = wm + ((e & 3) * RI + ii) * 16, k32 = (e >> 2) * 32;
        a[e & 1][ii] = TA == 0 ? frag_kmajor(As, row, k32, lane) : frag_rmajor<BM>(As, row, k32, lane);
      }
    };
    auto read_b = [&](int ks) {
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        b[ks][j] = TB == 1 ? frag_kmajor(Bs, wn + j * 16, ks * 32, lane) : frag_rmajor<BN>(Bs, wn + j * 16, ks * 32, lane);
    };
    read_b(0);
    read_a(0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (e == 2) read_b(1);
      if (e < 7) read_a(e + 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ii = 0; ii < RI; ++ii)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[(e & 3) * RI + ii][j] = mfma_16x16x32<E>(b[e >> 2][j], a[e & 1][ii], acc[(e & 3) * RI + ii][j]);
      if (e & 1) stash_b(buf ^ 1, fb, (e >> 1) * VB / 4, ((e >> 1) + 1) * VB / 4);
      else stash_a(buf ^ 1, fa, (e >> 1) * VA / 4, ((e >> 1) + 1) * VA / 4);
      __builtin_amdgcn_sched_barrier(0);
      load(e * VL, (e + 1) * VL);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Slabs past K read zeros (their loads are out of range), so the loop needs no conditions: it walks K in
  // pairs of slabs and a surplus slab contributes nothing.
  if (PAIR) {
    // The same pipeline over a K range made of parts: the loads run one pair of slabs ahead of the products, a
    // pair lies inside one part (kseg is a multiple of two slabs), and the descriptors change between the inner
    // loops, so the inner loop is that of the single-range kernel.  After the last part comes an empty one whose
    // single pair of loads returns zeros while the last real pair is multiplied.
    auto fetch_part = [&](int kin, Frag<BM, NT>& fa, Frag<BN, NT>& fb, int i0 = 0, int i1 = 1 << 20) {
      load_rmajor<BM, NT>(fa, curA, voffA, lda, m0, kin, i0, i1);
      load_rmajor<BN, NT>(fb, curB, voffB, ldb, n0, kin, i0 - VA, i1 - VA);
    };
    const int full = K1 / (2 * BK);                                    // slab pairs of a part of kseg rows
    const int tail = (g.K - g.nx * K1 + 2 * BK - 1) / (2 * BK);        // of the last part (rows past its end read as zero)
    fetch_part(0, fa0, fb0);
    stash_a(0, fa0);
    stash_b(0, fb0);
    fetch_part(BK, fa1, fb1);
    __syncthreads();
    for (int p = p0; p <= p1 + 1; ++p) {
      const int pairs = p > p1 ? 1 : p < g.nx ? full : tail;
      for (int j = p == p0 ? 1 : 0; j < pairs; ++j) {
        multiply(0, fa1, fb1, [&](int i0, int i1) { fetch_part(j * 2 * BK, fa0, fb0, i0, i1); });
        __syncthreads();
        multiply(1, fa0, fb0, [&](int i0, int i1) { fetch_part(j * 2 * BK + BK, fa1, fb1, i0, i1); });
        __syncthreads();
      }
      curA = part_a(p + 1);
      curB = part_b(p + 1);
    }
  } else {
    fetch(0, fa0, fb0);
    stash_a(0, fa0);
    stash_b(0, fb0);
    fetch(1, fa1, fb1);
    __syncthreads();
    for (int kt = 0; kt < nk; kt += 2) {
      multiply(0, fa1, fb1, [&](int i0, int i1) { fetch(kt + 2, fa0, fb0, i0, i1); });
      __syncthreads();
      multiply(1, fa0, fb0, [&](int i0, int i1) { fetch(kt + 3, fa1, fb1, i0, i1); });
      __syncthreads();
    }
  }

  if (ACC) {
    if (chunk == 0) {
      float* Ct = (float*)g.C + (int64_t)z * g.sC + (int64_t)m0 * g.ldc + n0;
      epilogue_accum<BM, BN, NT, MI, NJ>(Ct, (int)g.ldc, min(BM, g.M - m0), min(BN, g.N - n0), false, acc, wave / WN, wn, tid,
                                         reinterpret_cast<float*>(smem_raw));
    } else {   // partial tile number (chunk-1) * tile_count + position inside the launch's range
      const int64_t slot = (int64_t)(chunk - 1) * g.tile_count + sub;
      epilogue_accum<BM, BN, NT, MI, NJ>((float*)g.ws + slot * (BM * BN), BN, BM, BN, true, acc, wave / WN, wn, tid,
                                         reinterpret_cast<float*>(smem_raw));
    }
  }
  else if (GLU == 1) epilogue_glu<E, BM, BN, NT, MI, NJ>(g, acc, m0, nb0, wave / WN, wn, tid, reinterpret_cast<float*>(smem_raw));
  else epilogue_store<E, BM, BN, NT, MI, NJ, GLU>(g, z, acc, m0, n0, wave / WN, wn, tid, reinterpret_cast<float*>(smem_raw));
}

template <typename E, int BM, int BN, int NW, int TA, int TB, int SEG, int ACC, int GLU = 0>
hipError_t launch2(hipStream_t st, const Gemm& g) {
  constexpr size_t SMEM_BYTES = 2 * (slab_elems(BM) + slab_elems(BN)) * sizeof(bf16);
  static bool configured = false;
  auto kern = gemm_mfma_kernel<E, BM, BN, NW, TA, TB, SEG, ACC, GLU>;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_m = (int)cdiv(g.M, BM), tiles_n = (int)cdiv(g.N, GLU == 1 ? BN / 2 : BN);   // a gate|up tile holds BN/2 columns of each
  const bool range = SEG && TA == 1 && TB == 0 && ACC && g.tile_count > 0;   // part of a cut product
  const bool chunks = range && g.chunk_parts > 0 && g.nchunks > 1;
  dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)g.batch), blk(64 * NW);
  if (range) grid = dim3((unsigned)g.tile_count, 1u, chunks ? (unsigned)g.nchunks : 1u);
  hipLaunchKernelGGL(kern, grid, blk, SMEM_BYTES, st, g, tiles_m, tiles_n);
  return hipGetLastError();
}

template <typename E, int BM, int BN, int NW, int TA, int TB, int SEG> hipError_t launch(hipStream_t st, const Gemm& g) {
  return g.c_f32_accum ? launch2<E, BM, BN, NW, TA, TB, SEG, 1>(st, g) : launch2<E, BM, BN, NW, TA, TB, SEG, 0>(st, g);
}

template <typename E, int BM, int BN, int NW> hipError_t gemm_mfma_tile(hipStream_t st, const Gemm& g) {
  if (g.glu == 1) return launch2<E, BM, BN, NW, 0, 0, 0, 0, 1>(st, g);
  if (g.glu == 2) return launch2<E, BM, BN, NW, 0, 1, 0, 0, 2>(st, g);
  if (g.nx) return launch<E, BM, BN, NW, 1, 0, 1>(st, g);
  if (g.kseg) return g.transA ? launch<E, BM, BN, NW, 1, 1, 1>(st, g) : launch<E, BM, BN, NW, 0, 1, 1>(st, g);
  if (!g.transA && !g.transB) return launch<E, BM, BN, NW, 0, 0, 0>(st, g);
  if (!g.transA && g.transB) return launch<E, BM, BN, NW, 0, 1, 0>(st, g);
  if (g.transA && !g.transB) return launch<E, BM, BN, NW, 1, 0, 0>(st, g);
  return launch<E, BM, BN, NW, 1, 1, 0>(st, g);
}

}  // namespace gemm_impl
}  // namespace zs
