// Flash-style causal attention on the CDNA4 matrix cores, head dim 128, bf16 in, fp32 softmax.
//
// The S x S score matrix is never stored: K/V (forward, dQ) or Q/dO (dK/dV) tiles of 64 rows are
// staged in LDS and every wavefront keeps its own 32 rows' operands and accumulators in
// registers.  All products are computed TRANSPOSED (S^T = K Q^T, O^T = V^T P^T, ...): with
// v_mfma_f32_32x32x16_bf16 a lane then owns one query (or key) column, so the softmax row
// maximum and sum are reductions over the lane's own registers plus one exchange with lane^32,
// and the fp32 accumulator registers of one product are, converted to bf16, already laid out
// as the B operand of the next one.  The A operands that need the transposed tile (V^T, K^T,
// dO^T, Q^T) are read with ds_read_b64_tr_b16, which hands a lane 4 values that are consecutive
// along the tile's ROW index, so tiles sit in LDS exactly as they sit in memory.
//
// Backward is two kernels without atomics (fixed summation order): one owns 128 queries and
// produces dQ, one owns 128 keys and produces dK and dV; both recompute P from the saved
// log-sum-exp.  delta_i = dO_i . O_i is formed by the dQ kernel for its own rows and stored for the other.
#include "kernels.h"

// This file is compiled twice: as it stands for bf16, and through attention_mfma_f16.hip (which defines
// ZS_ATTN_F16 and includes it) for IEEE half.  e16 is the 16-bit element type of the build; the two builds
// differ in the conversions to and from float, the matrix-core instruction and the names they export.
#ifdef ZS_ATTN_F16
#define ZS_ATTN_MFMA __builtin_amdgcn_mfma_f32_32x32x16_f16
#define ZS_ATTN_NAME(x) x##_f16
namespace zs { typedef f16 e16; typedef f16x8 e16x8; typedef f16x4 e16x4; }
#else
#define ZS_ATTN_MFMA __builtin_amdgcn_mfma_f32_32x32x16_bf16
#define ZS_ATTN_NAME(x) x
namespace zs { typedef bf16 e16; typedef bf16x8 e16x8; typedef bf16x4 e16x4; }
#endif


namespace zs {

namespace {

constexpr int D = 128;             // head dim
constexpr int TR = 64;             // rows of a staged tile
// Padded LDS row length in elements: 304 bytes = 76 banks = 12 (mod 64).  The 16 rows that one cycle of a
// row-fragment read touches then start in 16 different 4-bank groups (no conflicts); the 4 rows x 64 bytes
// of a transposing read overlap in 4 of their 16 banks, the least any padding allows next to that.
constexpr int LDT = D + 24;
constexpr int TILE = TR * LDT;     // elements of one staged tile
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ e16x8 zero8() {
  e16x8 z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = (e16)0.f;
  return z;
}

// A-operand fragment of a row-major LDS tile: lane (row = lane%32, g = lane/32) gets 8 consecutive columns.
__device__ __forceinline__ e16x8 lds_frag(const e16* tile, int row0, int col0, int lane) {
  return *reinterpret_cast<const e16x8*>(tile + (row0 + (lane & 31)) * LDT + col0 + 8 * (lane >> 5));
}

// A-operand fragment of the TRANSPOSE of a row-major LDS tile M[k][n]: lane (i = lane%32, g = lane/32)
// gets M[k][n0+i] for the 8 contraction slots  k = k0 + 4g + {0,1,2,3, 8,9,10,11}.  This slot order is
// the order in which a lane's accumulator registers 8s..8s+7 of a 32-row MFMA block hold rows, so the
// matching B operand is just those registers.
__device__ __forceinline__ e16x8 lds_frag_tr(const e16* tile, int k0, int n0, int lane) {
  const int r = lane & 15, gi = lane >> 4;
  const e16* p = tile + (k0 + 4 * (gi >> 1) + (r >> 2)) * LDT + n0 + 16 * (gi & 1) + 4 * (r & 3);
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * LDT));
  union { struct { s16x4 a, b; } s; e16x8 v; } u;
  u.s.a = lo;
  u.s.b = hi;
  return u.v;
}

__device__ __forceinline__ e16x8 pack8(const f32x16& a, int s) {
  e16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (e16)a[8 * s + e];
  return o;
}

// A 64 x 128 tile moves HBM -> registers (fetch, issued before the MFMAs of the current tile so the
// latency hides behind them) -> LDS (put, after them).  Thread t carries 4 vectors of 16 bytes:
// vector v = t + 256 i is row v/16, columns 8*(v%16)...
template <int NT> struct TileRegs { e16x8 v[1024 / NT]; };   // NT threads share the 1024 vectors of a tile
// Rows of one (batch, head) are read through a raw buffer descriptor over [first row, last row's 128 columns]:
// the per-lane offset is one register, the tile's row offset a scalar, and rows at or past nrows fall
// beyond num_records and read as zero without a branch.  Offsets are 32-bit: nrows * ld * 2 < 2^31.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t head_rsrc(const e16* base, int64_t ld, int nrows) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<e16*>(base), 0, (int)((((int64_t)nrows - 1) * ld + D) * 2), 0x00020000);
}
template <int NT>
__device__ __forceinline__ void fetch_tile(TileRegs<NT>& x, __amdgpu_buffer_rsrc_t rs, int ld, int row0, int tid) {
  const int voff = ((tid >> 4) * ld + (tid & 15) * 8) * 2;
#pragma unroll
  for (int i = 0; i < 1024 / NT; ++i) {
    union { u32x4 u; e16x8 h; } c;
    c.u = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, (row0 + (NT / 16) * i) * ld * 2, 0);
    x.v[i] = c.h;
  }
}
template <int NT> __device__ __forceinline__ void put_tile(const TileRegs<NT>& x, e16* tile, int tid) {
#pragma unroll
  for (int i = 0; i < 1024 / NT; ++i) {
    const int v = tid + NT * i;
    *reinterpret_cast<e16x8*>(tile + (v >> 4) * LDT + (v & 15) * 8) = x.v[i];
  }
}

// Row fragments kept in registers for a whole kernel: lane (row = row0 + lane%32, g) holds, for each of the
// 8 contraction steps over d, 8 consecutive elements.  Rows >= nrows read as zero.
__device__ __forceinline__ void load_row_frags(e16x8 (&f)[8], const e16* __restrict__ src, int64_t ld, int row0,
                                               int nrows, int lane) {
  const int row = row0 + (lane & 31);
#pragma unroll
  for (int s = 0; s < 8; ++s)
    f[s] = row < nrows ? *reinterpret_cast<const e16x8*>(src + (int64_t)row * ld + 16 * s + 8 * (lane >> 5)) : zero8();
}

// Row index (inside a 32-row MFMA block) held by accumulator register r of this lane.
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// Causal blocks differ in work by up to the number of tiles, so the launch order matters: workgroups are
// dispatched in increasing linear id, and id -> (rank, head) with the rank (0 = most work) in the slow
// position puts the heavy blocks of ALL heads first and leaves light blocks for the tail.  Consecutive
// ids go to different XCDs round-robin; with nh*mb a multiple of 8 a head keeps its XCD, whose L2 then
// holds the K/V (or Q/dO) rows its blocks stream.
struct BlockId { int rank, h, b; };
__device__ __forceinline__ BlockId block_id(int nh, int mb) {
  const int nhb = nh * mb, id = blockIdx.x, hb = id % nhb;
  return BlockId{id / nhb, hb % nh, hb / nh};
}

// Inverse rotary rotation of 4 consecutive head-dim values (two adjacent pairs) of position pos, first
// value at head-dim index d0 (a multiple of 4): (u, w) -> (u c + w s, -u s + w c).
typedef float f32x4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void unrotate4(float (&x)[4], const float2* __restrict__ rope, int pos, int d0) {
  const f32x4v t = *reinterpret_cast<const f32x4v*>(rope + (int64_t)pos * (D / 2) + d0 / 2);   // (cos, sin) x 2
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float c = t[2 * i], sn = t[2 * i + 1], u = x[2 * i], w = x[2 * i + 1];
    x[2 * i] = u * c + w * sn;
    x[2 * i + 1] = w * c - u * sn;
  }
}

// ------------------------------------------------------------------------------------------ forward
// grid ceil(S/(32 NW))*nh*mb, NW waves; wave w owns queries q0 + 32w .. +31; heavy (late) blocks are launched first.
// NW = 4: two workgroups per CU.  NW = 8: one workgroup per CU whose staged K/V tiles serve 256 queries, so a wave
// issues half as many tile loads and LDS stores per key tile (used when that still gives every CU a workgroup).
template <int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attn_fwd_kernel(int S, const e16* __restrict__ q, const e16* __restrict__ k,
                                                       const e16* __restrict__ v, int64_t ld, e16* __restrict__ o,
                                                       int64_t ldo, float* __restrict__ lse, float scale_log2, int nh,
                                                       int mb) {
  extern __shared__ __align__(16) char smem_raw[];
  e16* smem = reinterpret_cast<e16*>(smem_raw);            // [2][K tile | V tile]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const BlockId bid = block_id(nh, mb);
  const int qb = (S + 32 * NW - 1) / (32 * NW) - 1 - bid.rank, h = bid.h, b = bid.b;
  const int64_t tok0 = (int64_t)b * S;
  const e16* qh = q + tok0 * ld + h * D;
  const e16* kh = k + tok0 * ld + h * D;
  const e16* vh = v + tok0 * ld + h * D;
  const __amdgpu_buffer_rsrc_t rsk = head_rsrc(kh, ld, S), rsv = head_rsrc(vh, ld, S);
  const int q0 = qb * 32 * NW, wq0 = q0 + wave * 32;
  const int my_q = wq0 + (lane & 31);

  e16x8 qf[8];
  load_row_frags(qf, qh, ld, wq0, S, lane);
  f32x16 oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int last_q = min(q0 + 32 * NW - 1, S - 1);
  const int ntiles = last_q / TR + 1;
  TileRegs<64 * NW> kr, vr;
  fetch_tile(kr, rsk, (int)ld, 0, tid);
  fetch_tile(vr, rsv, (int)ld, 0, tid);
  put_tile(kr, smem, tid);
  put_tile(vr, smem + TILE, tid);
  __syncthreads();
  for (int t = 0; t < ntiles; ++t) {
    const e16* Kt = smem + (t & 1) * 2 * TILE;
    const e16* Vt = Kt + TILE;
    if (t + 1 < ntiles) {
      fetch_tile(kr, rsk, (int)ld, (t + 1) * TR, tid);
      fetch_tile(vr, rsv, (int)ld, (t + 1) * TR, tid);
    }
    const int key0 = t * TR;
    if (key0 <= wq0 + 31) {   // otherwise every key of the tile is in this wave's future
      f32x16 sacc[2];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[jb][r] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s)
          sacc[jb] = ZS_ATTN_MFMA(lds_frag(Kt, jb * 32, 16 * s, lane), qf[s], sacc[jb], 0, 0, 0);
      }
      if (key0 + TR - 1 > wq0) {   // tile touches the diagonal: mask keys in the future of this lane's query
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (key0 + jb * 32 + acc_row(r, lane) > my_q) sacc[jb][r] = -INFINITY;
      }
      float mx = -INFINITY;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[jb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;   // scale > 0, so the maximum commutes with it
      // Lazy rescaling: the reference maximum m only moves when some row's maximum grew by more than 2^8;
      // until then P is formed against the old reference (values up to 2^8, harmless in e16/fp32) and the
      // 64 accumulator registers are left alone.  m, l and O always refer to the same reference, so
      // O/l and m + log2(l) are exact whatever the schedule of updates.
      if (__any(mx > m + 8.0f)) {
        const float mn = fmaxf(m, mx);          // finite: key 0 is visible to every query in the first tile
        const float alpha = __builtin_amdgcn_exp2f(m - mn);
        l *= alpha;
        m = mn;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
      }
      float rs = 0.f;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[jb][r], scale_log2, -m));
          sacc[jb][r] = p;
          rs += p;
        }
      rs += __shfl_xor(rs, 32, 64);
      l += rs;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const e16x8 pf = pack8(sacc[jb], s2);
#pragma unroll
          for (int db = 0; db < 4; ++db)
            oacc[db] = ZS_ATTN_MFMA(lds_frag_tr(Vt, jb * 32 + 16 * s2, db * 32, lane), pf,
                                                               oacc[db], 0, 0, 0);
        }
    }
    if (t + 1 < ntiles) {   // the other buffer was last read before the barrier that ended the previous iteration
      put_tile(kr, smem + ((t + 1) & 1) * 2 * TILE, tid);
      put_tile(vr, smem + ((t + 1) & 1) * 2 * TILE + TILE, tid);
    }
    __syncthreads();
  }
  if (my_q < S) {
    const float inv = 1.0f / l;
    e16* orow = o + (tok0 + my_q) * ldo + h * D;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        e16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (e16)(oacc[db][4 * c + e] * inv);
        *reinterpret_cast<e16x4*>(orow + db * 32 + 8 * c + 4 * (lane >> 5)) = w;
      }
    if (lane < 32) lse[((int64_t)b * nh + h) * S + my_q] = (m + log2f(l)) * LN2;
  }
}

// ------------------------------------------------------------------------------------------ dQ
// grid ceil(S/(32 NW))*nh*mb, NW waves (4 or 8 as in the forward kernel); wave w owns queries q0+32w..; loops over K/V
// tiles up to the diagonal.
// dQ^T[d][q] += K^T[d][key] dS^T[key][q],  dS^T = P^T o (dP^T - delta_q),  dP^T = V dO^T.
template <int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attn_bwd_dq_kernel(int S, const e16* __restrict__ q, const e16* __restrict__ k,
                                                          const e16* __restrict__ v, int64_t ld,
                                                          const e16* __restrict__ o, const e16* __restrict__ dout,
                                                          int64_t ldo, const float* __restrict__ lse,
                                                          float* __restrict__ delta,
                                                          e16* __restrict__ dq, int64_t ldd, float scale, int nh,
                                                          int mb, const float2* __restrict__ rope) {
  extern __shared__ __align__(16) char smem_raw[];
  e16* smem = reinterpret_cast<e16*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const BlockId bid = block_id(nh, mb);
  const int qb = (S + 32 * NW - 1) / (32 * NW) - 1 - bid.rank, h = bid.h, b = bid.b;
  const int64_t tok0 = (int64_t)b * S;
  const e16* qh = q + tok0 * ld + h * D;
  const e16* kh = k + tok0 * ld + h * D;
  const e16* vh = v + tok0 * ld + h * D;
  const e16* doh = dout + tok0 * ldo + h * D;
  const __amdgpu_buffer_rsrc_t rsk = head_rsrc(kh, ld, S), rsv = head_rsrc(vh, ld, S);
  const int q0 = qb * 32 * NW, wq0 = q0 + wave * 32;
  const int my_q = wq0 + (lane & 31);
  const float scale_log2 = scale * LOG2E;

  e16x8 qf[8], dof[8];
  load_row_frags(qf, qh, ld, wq0, S, lane);
  load_row_frags(dof, doh, ldo, wq0, S, lane);
  const int64_t stat = ((int64_t)b * nh + h) * S + min(my_q, S - 1);
  const float lse2 = lse[stat] * LOG2E;
  // delta_q = dO_q . O_q: each lane sums its 64 of the row's 128 products, lane^32 holds the others.
  // The value is also stored for the dK/dV kernel, which runs after this one.
  float dlt = 0.f;
  {
    e16x8 of[8];
    load_row_frags(of, o + tok0 * ldo + h * D, ldo, wq0, S, lane);
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) dlt = fmaf((float)dof[s][e], (float)of[s][e], dlt);
    dlt += __shfl_xor(dlt, 32, 64);
    if (lane < 32 && my_q < S) delta[stat] = dlt;
  }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  const int last_q = min(q0 + 32 * NW - 1, S - 1);
  const int ntiles = last_q / TR + 1;
  TileRegs<64 * NW> kr, vr;
  fetch_tile(kr, rsk, (int)ld, 0, tid);
  fetch_tile(vr, rsv, (int)ld, 0, tid);
  put_tile(kr, smem, tid);
  put_tile(vr, smem + TILE, tid);
  __syncthreads();
  for (int t = 0; t < ntiles; ++t) {
    const e16* Kt = smem + (t & 1) * 2 * TILE;
    const e16* Vt = Kt + TILE;
    if (t + 1 < ntiles) {
      fetch_tile(kr, rsk, (int)ld, (t + 1) * TR, tid);
      fetch_tile(vr, rsv, (int)ld, (t + 1) * TR, tid);
    }
    const int key0 = t * TR;
    if (key0 <= wq0 + 31) {
      const bool diag = key0 + TR - 1 > wq0;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
        f32x16 sacc, pacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = pacc[r] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          sacc = ZS_ATTN_MFMA(lds_frag(Kt, jb * 32, 16 * s, lane), qf[s], sacc, 0, 0, 0);
          pacc = ZS_ATTN_MFMA(lds_frag(Vt, jb * 32, 16 * s, lane), dof[s], pacc, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = __builtin_amdgcn_exp2f(fmaf(sacc[r], scale_log2, -lse2)) * (pacc[r] - dlt);
        if (diag) {   // keys in the future of this lane's query contribute nothing
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (key0 + jb * 32 + acc_row(r, lane) > my_q) sacc[r] = 0.f;
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const e16x8 dsf = pack8(sacc, s2);
#pragma unroll
          for (int db = 0; db < 4; ++db)
            acc[db] = ZS_ATTN_MFMA(lds_frag_tr(Kt, jb * 32 + 16 * s2, db * 32, lane), dsf,
                                                              acc[db], 0, 0, 0);
        }
      }
    }
    if (t + 1 < ntiles) {   // the other buffer was last read before the barrier that ended the previous iteration
      put_tile(kr, smem + ((t + 1) & 1) * 2 * TILE, tid);
      put_tile(vr, smem + ((t + 1) & 1) * 2 * TILE + TILE, tid);
    }
    __syncthreads();
  }
  if (my_q < S) {
    e16* row = dq + (tok0 + my_q) * ldd + h * D;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = acc[db][4 * c + e] * scale;
        if (rope) unrotate4(x, rope, my_q, db * 32 + 8 * c + 4 * (lane >> 5));
        e16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (e16)x[e];
        *reinterpret_cast<e16x4*>(row + db * 32 + 8 * c + 4 * (lane >> 5)) = w;
      }
  }
}

// ------------------------------------------------------------------------------------------ dK, dV
// grid ceil(S/(32 NW))*nh*mb, NW waves; wave w owns keys k0+32w..; loops over Q/dO tiles from the diagonal to the
// end.  With 8 waves the staged Q/dO tiles serve 256 keys and two waves share each SIMD, so one wave's
// softmax arithmetic overlaps the other's MFMAs.
// S[q][key] = Q K^T (lane = key, registers = queries), P = exp2(S c - lse_q), dP = dO V^T,
// dV^T[d][key] += dO^T[d][q] P[q][key],  dK^T[d][key] += Q^T[d][q] dS[q][key].
template <int NW>
__global__ __launch_bounds__(64 * NW) void attn_bwd_dkv_kernel(int S, const e16* __restrict__ q, const e16* __restrict__ k,
                                                           const e16* __restrict__ v, int64_t ld,
                                                           const e16* __restrict__ dout, int64_t ldo,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           e16* __restrict__ dk, e16* __restrict__ dv, int64_t ldd,
                                                           float scale, int nh, int mb, const float2* __restrict__ rope) {
  extern __shared__ __align__(16) char smem_raw[];
  e16* smem = reinterpret_cast<e16*>(smem_raw);                 // [2][Q tile | dO tile]
  float* stats = reinterpret_cast<float*>(smem + 4 * TILE);       // [2][lse2[64] | delta[64]]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const BlockId bid = block_id(nh, mb);
  const int kb = bid.rank, h = bid.h, b = bid.b;                   // early key blocks (most work) first
  const int64_t tok0 = (int64_t)b * S;
  const e16* qh = q + tok0 * ld + h * D;
  const e16* kh = k + tok0 * ld + h * D;
  const e16* vh = v + tok0 * ld + h * D;
  const e16* doh = dout + tok0 * ldo + h * D;
  const __amdgpu_buffer_rsrc_t rsq = head_rsrc(qh, ld, S), rsdo = head_rsrc(doh, ldo, S);
  const float* lse_h = lse + ((int64_t)b * nh + h) * S;
  const float* dlt_h = delta + ((int64_t)b * nh + h) * S;
  const int k0 = kb * 32 * NW, wk0 = k0 + wave * 32;
  const int my_k = wk0 + (lane & 31);
  const float scale_log2 = scale * LOG2E;

  // K fragments stay in registers; the wave's 32 rows of V go to a private LDS block instead and are
  // read back as B operands (same fragment pattern as the A operands), which keeps the kernel within
  // the register budget of two waves per SIMD.
  e16x8 kf[8];
  load_row_frags(kf, kh, ld, wk0, S, lane);
  e16* Vw = reinterpret_cast<e16*>(stats + 256) + wave * 32 * LDT;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int vv = lane + 64 * i, r = vv >> 4, c = (vv & 15) * 8;
    *reinterpret_cast<e16x8*>(Vw + r * LDT + c) =
        wk0 + r < S ? *reinterpret_cast<const e16x8*>(vh + (int64_t)(wk0 + r) * ld + c) : zero8();
  }
  f32x16 dkacc[4], dvacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dkacc[i][r] = dvacc[i][r] = 0.f;

  TileRegs<64 * NW> qr, dor;
  float statr = 0.f;
  auto fetch = [&](int t) {
    fetch_tile(qr, rsq, (int)ld, t * TR, tid);
    fetch_tile(dor, rsdo, (int)ldo, t * TR, tid);
    if (tid < 128) {
      const int r = t * TR + (tid & 63);
      statr = 0.f;
      if (r < S) statr = tid < 64 ? lse_h[r] * LOG2E : dlt_h[r];
    }
  };
  auto put = [&](int buf) {
    put_tile(qr, smem + buf * 2 * TILE, tid);
    put_tile(dor, smem + buf * 2 * TILE + TILE, tid);
    if (tid < 128) stats[buf * 128 + tid] = statr;
  };
  const int t_begin = k0 / TR, t_end = (S - 1) / TR + 1;
  fetch(t_begin);
  put(0);
  __syncthreads();
  for (int t = t_begin; t < t_end; ++t) {
    const int buf = (t - t_begin) & 1;
    const e16* Qt = smem + buf * 2 * TILE;
    const e16* dOt = Qt + TILE;
    const float* st = stats + buf * 128;
    if (t + 1 < t_end) fetch(t + 1);
    const int qrow0 = t * TR;
    if (qrow0 + TR - 1 >= wk0) {   // otherwise every query of the tile precedes this wave's keys
      const bool diag = qrow0 < wk0 + 31;
#pragma unroll
      for (int ib = 0; ib < 2; ++ib) {
        f32x16 sacc, pacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = pacc[r] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          sacc = ZS_ATTN_MFMA(lds_frag(Qt, ib * 32, 16 * s, lane), kf[s], sacc, 0, 0, 0);
          pacc = ZS_ATTN_MFMA(lds_frag(dOt, ib * 32, 16 * s, lane), lds_frag(Vw, 0, 16 * s, lane), pacc,
                                                         0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int qi = ib * 32 + acc_row(r, lane);
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[r], scale_log2, -st[qi]));
          sacc[r] = p;
          pacc[r] = p * (pacc[r] - st[64 + qi]);
        }
        if (diag || qrow0 + TR > S) {   // queries before this lane's key, and rows past the end, contribute nothing
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int qi = ib * 32 + acc_row(r, lane);
            if (qrow0 + qi < my_k || qrow0 + qi >= S) sacc[r] = pacc[r] = 0.f;
          }
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const e16x8 pf = pack8(sacc, s2), dsf = pack8(pacc, s2);
#pragma unroll
          for (int db = 0; db < 4; ++db) {
            dvacc[db] = ZS_ATTN_MFMA(lds_frag_tr(dOt, ib * 32 + 16 * s2, db * 32, lane), pf,
                                                                dvacc[db], 0, 0, 0);
            dkacc[db] = ZS_ATTN_MFMA(lds_frag_tr(Qt, ib * 32 + 16 * s2, db * 32, lane), dsf,
                                                                dkacc[db], 0, 0, 0);
          }
        }
      }
    }
    if (t + 1 < t_end) put(buf ^ 1);
    __syncthreads();
  }
  if (my_k < S) {
    e16* krow = dk + (tok0 + my_k) * ldd + h * D;
    e16* vrow = dv + (tok0 + my_k) * ldd + h * D;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = dkacc[db][4 * c + e] * scale;
        if (rope) unrotate4(x, rope, my_k, db * 32 + 8 * c + 4 * (lane >> 5));
        e16x4 wk, wv;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          wk[e] = (e16)x[e];
          wv[e] = (e16)dvacc[db][4 * c + e];
        }
        *reinterpret_cast<e16x4*>(krow + db * 32 + 8 * c + 4 * (lane >> 5)) = wk;
        *reinterpret_cast<e16x4*>(vrow + db * 32 + 8 * c + 4 * (lane >> 5)) = wv;
      }
  }
}

constexpr size_t SMEM_FWD = 4 * TILE * sizeof(e16);                    // 77824
constexpr size_t smem_dkv(int nw) { return 4 * TILE * sizeof(e16) + 256 * sizeof(float) + (size_t)nw * 32 * LDT * sizeof(e16); }

// Blocks of 256 rows (8 waves) instead of 128 (4 waves): for the key blocks of the dK/dV kernel whenever that still
// gives every CU a workgroup; for the query blocks of the forward and dQ kernels only from S = 4096 on (measured: 7 % and
// 3 % faster at S = 4096 with 32 heads, 7 % slower at S = 2048 with 80 head-sequences, where a block has half the tiles to
// amortise its idle waves on the diagonal).
inline bool wide_blocks(int S, int nh, int mb) { return cdiv(S, 256) * nh * mb >= 256; }
inline bool wide_query_blocks(int S, int nh, int mb) { return wide_blocks(S, nh, mb) && S >= 4096; }

template <typename K> hipError_t set_smem(K kern, size_t bytes, bool& done) {
  if (done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) done = true;
  return e;
}

}  // namespace

#ifndef ZS_ATTN_F16
bool attn_mfma_supported(DType dt, int S, int d) { return (dt == BF16 || dt == F16) && d == D && S >= 1; }
#endif

hipError_t ZS_ATTN_NAME(attn_fwd_mfma)(hipStream_t st, int mb, int S, int nh, int d, const void* q, const void* k, const void* v,
                         int64_t ld, void* o, int64_t ldo, float* lse) {
  if ((int64_t)S * ld * 2 >= (1ll << 31)) return hipErrorInvalidValue;      // 32-bit buffer offsets
  static bool cfg4 = false, cfg8 = false;
  hipError_t e = set_smem(attn_fwd_kernel<4>, SMEM_FWD, cfg4);
  if (e == hipSuccess) e = set_smem(attn_fwd_kernel<8>, SMEM_FWD, cfg8);
  if (e != hipSuccess) return e;
  // 256 queries per workgroup when that still gives every CU a workgroup, else 128
  if (wide_query_blocks(S, nh, mb))
    hipLaunchKernelGGL(attn_fwd_kernel<8>, dim3((unsigned)(cdiv(S, 256) * nh * mb)), dim3(512), SMEM_FWD, st, S, (const e16*)q,
                       (const e16*)k, (const e16*)v, ld, (e16*)o, ldo, lse, LOG2E / sqrtf((float)d), nh, mb);
  else
    hipLaunchKernelGGL(attn_fwd_kernel<4>, dim3((unsigned)(cdiv(S, 128) * nh * mb)), dim3(256), SMEM_FWD, st, S, (const e16*)q,
                       (const e16*)k, (const e16*)v, ld, (e16*)o, ldo, lse, LOG2E / sqrtf((float)d), nh, mb);
  return hipGetLastError();
}

hipError_t ZS_ATTN_NAME(attn_bwd_mfma)(hipStream_t st, int mb, int S, int nh, int d, const void* q, const void* k, const void* v,
                         int64_t ld, const void* o, const void* dout, int64_t ldo, const float* lse, float* delta,
                         void* dq, void* dk, void* dv, int64_t ldd, const float2* rope) {
  if ((int64_t)S * (ld > ldo ? ld : ldo) * 2 >= (1ll << 31)) return hipErrorInvalidValue;   // 32-bit buffer offsets
  static bool cfg1 = false, cfg1b = false, cfg2 = false, cfg3 = false;
  hipError_t e = set_smem(attn_bwd_dq_kernel<4>, SMEM_FWD, cfg1);
  if (e == hipSuccess) e = set_smem(attn_bwd_dq_kernel<8>, SMEM_FWD, cfg1b);
  if (e == hipSuccess) e = set_smem(attn_bwd_dkv_kernel<4>, smem_dkv(4), cfg2);
  if (e == hipSuccess) e = set_smem(attn_bwd_dkv_kernel<8>, smem_dkv(8), cfg3);
  if (e != hipSuccess) return e;
  const float scale = 1.0f / sqrtf((float)d);
  dim3 grid((unsigned)(cdiv(S, 128) * nh * mb)), blk(256);
  const bool wide = wide_blocks(S, nh, mb);
  if (wide_query_blocks(S, nh, mb))
    hipLaunchKernelGGL(attn_bwd_dq_kernel<8>, dim3((unsigned)(cdiv(S, 256) * nh * mb)), dim3(512), SMEM_FWD, st, S, (const e16*)q,
                       (const e16*)k, (const e16*)v, ld, (const e16*)o, (const e16*)dout, ldo, lse, delta, (e16*)dq, ldd, scale, nh,
                       mb, rope);
  else
    hipLaunchKernelGGL(attn_bwd_dq_kernel<4>, grid, blk, SMEM_FWD, st, S, (const e16*)q, (const e16*)k, (const e16*)v, ld,
                       (const e16*)o, (const e16*)dout, ldo, lse, delta, (e16*)dq, ldd, scale, nh, mb, rope);
  if (wide) {
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<8>, dim3((unsigned)(cdiv(S, 256) * nh * mb)), dim3(512), smem_dkv(8), st,
                       S, (const e16*)q, (const e16*)k, (const e16*)v, ld, (const e16*)dout, ldo, lse, delta, (e16*)dk,
                       (e16*)dv, ldd, scale, nh, mb, rope);
  } else {
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<4>, grid, blk, smem_dkv(4), st, S, (const e16*)q, (const e16*)k, (const e16*)v, ld,
                       (const e16*)dout, ldo, lse, delta, (e16*)dk, (e16*)dv, ldd, scale, nh, mb, rope);
  }
  return hipGetLastError();
}

}  // namespace zs
