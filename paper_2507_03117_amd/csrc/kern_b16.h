// Product kernel for 16 x 16 blocks (the smallest block size of BLaST's block-size sweeps, Sec. 5).
//
// A 16-wide block is half the contraction depth of v_mfma_f32_16x16x32_bf16, so the unit of work is a PAIR of
// stored blocks of one block row: consecutive blocks of a row are consecutive in the value array, and the 64
// lanes' 16-byte operand pieces (lane l: block l/32 of the pair, row l%16, columns 8*((l/16)%2) ...) are
// exactly the pair's 1 KiB, one fully coalesced load.  The activation operand of the same instruction is, per
// lane, 16 bytes of one token row at the block's column: both operands go from global memory straight into the
// registers the matrix instruction reads - no LDS, no barrier, nothing to synchronise but the wave's own loads.
// The weight rows are the M side of the instruction, so a lane ends up with four consecutive output rows of one
// token: one 16-byte (fp32) or 8-byte (bf16) store per 16-token tile.
//
// A wave owns (block row, NS tiles of 16 tokens); the four waves of a workgroup take neighbouring token tiles of
// the same block row, so the pair's weights are fetched from the L2 once per workgroup.  What bounds the kernel is
// the vector memory path: every matrix instruction needs a fresh 1 KiB activation fragment (16 bytes per lane =
// 16 flop per byte loaded), where a 64-wide block shares one staged tile between 64 rows.  In a token-major
// tensor that fragment is 32 segments of 32 bytes in 32 different cache lines, and the L2 sends a whole 128-byte
// line for each: with activations stored in column groups of 16 features ([K/16][T][16]: the 16 tokens x 16
// features of a fragment are 512 consecutive bytes) the same fragment is eight whole lines.  The kernel reads
// and writes either layout; the MLP regroups X once (k_group16) and keeps H grouped from the start.
#pragma once
#include "kern_common.h"

namespace blast_dev {

typedef float f32x4_b16 __attribute__((ext_vector_type(4)));

template <int NS>
struct B16Frag {
  bf16x8 w;
  bf16x8 x[NS];
};

// Block column of this lane's block of the pair (kp, kp + 1) of a row that ends at ke (lanes of the second half
// repeat block kp when the row has no block kp + 1); 0 beyond the row.
__device__ __forceinline__ int b16_col(const MatDev& m, int kp, int ke) {
  if (kp >= ke) return 0;
  const int blk = kp + ((threadIdx.x & 63) >> 5);
  return m.col_idx[blk < ke ? blk : kp];
}

// Operands of the pair of blocks (kp, kp + 1), block column c per lane from b16_col.  Lanes of the second half
// hold zeros as their weights when the row has no block kp + 1.
template <int NS>
__device__ __forceinline__ void b16_load(const TileArgs& a, const MatDev& m, int kp, int ke, int64_t c,
                                         const int64_t (&xrow)[NS], int64_t cstride, B16Frag<NS>& f) {
  const int lane = threadIdx.x & 63;
  const int blk = kp + (lane >> 5);
  const bool valid = blk < ke;
  const int src = valid ? blk : kp;
  const int piece = ((lane >> 4) & 1) * 8;
  const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  const bf16x8 w = *reinterpret_cast<const bf16x8*>(m.vals + (int64_t)src * 256 + (lane & 15) * 16 + piece);
  f.w = valid ? w : zero;
#pragma unroll
  for (int s = 0; s < NS; ++s) f.x[s] = *reinterpret_cast<const bf16x8*>(a.X + xrow[s] + c * cstride + piece);
}

// The stored blocks of block row r of matrix m, two per matrix instruction: pairs pair0, pair0 + pstride, ... of
// the row.  The next pair's operands are on their way while the current pair is multiplied, and the block
// columns are read one pair further ahead (an operand's address depends on them).
template <int NS>
__device__ __forceinline__ void b16_row(const TileArgs& a, const MatDev& m, int r, const int64_t (&xrow)[NS],
                                        int64_t cstride, f32x4_b16 (&acc)[NS], int pair0 = 0, int pstride = 1) {
  const int ke = m.row_ptr[r + 1], step = 2 * pstride;
  int kp = m.row_ptr[r] + 2 * pair0;
  if (kp >= ke) return;
  B16Frag<NS> cur, nxt;
  int c_nxt = b16_col(m, kp + step, ke);
  b16_load<NS>(a, m, kp, ke, b16_col(m, kp, ke), xrow, cstride, cur);
  for (; kp < ke; kp += step) {
    const bool more = kp + step < ke;
    const int c_far = b16_col(m, kp + 2 * step, ke);
    if (more) b16_load<NS>(a, m, kp + step, ke, c_nxt, xrow, cstride, nxt);
#pragma unroll
    for (int s = 0; s < NS; ++s) acc[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.w, cur.x[s], acc[s], 0, 0, 0);
    if (more) cur = nxt;
    c_nxt = c_far;
  }
}

// Adds the waves' partial sums; every wave calls it, wave 0 returns with the totals (added in wave order).
template <int NS, int NW>
__device__ __forceinline__ void b16_join(f32x4_b16 (&acc)[NS]) {
  __shared__ f32x4_b16 part[NW - 1][NS][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (wave != 0) {
#pragma unroll
    for (int s = 0; s < NS; ++s) part[wave - 1][s][lane] = acc[s];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int w = 0; w < NW - 1; ++w) acc[s] += part[w][s][lane];
  }
}

// One wave = one (block row, 16 * NS tokens).  DUAL: two matrices with the same block rows, the output is
// bf16-or-fp32 act(W0 x) * (W1 x); POST: one matrix, the activation on its output.
// y_vec: the four rows of a lane can be stored with one 16-byte (fp32) / 8-byte (bf16) store (always so for a
// grouped output).
// SPLIT (decode token counts): the whole workgroup owns one (block row, token tile), its NW waves (4 or 16) deal
// the row's pairs among themselves and the partial sums meet in LDS - there are too few rows to fill the chip
// with a wave each, and a row walked by one wave is a chain of dependent loads.
template <bool DUAL, bool POST, int NS, bool SPLIT = false, int NW = 4>
__global__ __launch_bounds__(NW * 64) void k_spmm_b16(const TileArgs a, const int y_vec) {
  static_assert(SPLIT || NW == 4, "without SPLIT a workgroup is four independent waves");
  static_assert(!(POST && DUAL), "an activation on the output belongs to the single-matrix product");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t item = SPLIT ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * 4 + wave;
  const int rank = (int)(item / a.ntt), tt = (int)(item % a.ntt);
  if (rank >= a.nbr) return;  // (whole waves leave; with SPLIT the whole workgroup does)
  const int r = a.row_order ? a.row_order[rank] : rank;
  const int t0 = tt * 16 * NS;

  // element offset of this lane's token row in each tile (rows past the end read the last token), and the
  // distance between block columns: [T][K] or [K/16][T][16]
  const int64_t tstride = a.x_grp16 ? 16 : a.sxt, cstride = a.x_grp16 ? (int64_t)a.T * 16 : 16;
  int64_t xrow[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const int t = t0 + s * 16 + (lane & 15);
    xrow[s] = (int64_t)(t < a.T ? t : a.T - 1) * tstride;
  }
  f32x4_b16 acc0[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) acc0[s] = f32x4_b16{0.f, 0.f, 0.f, 0.f};
  b16_row<NS>(a, a.m0, r, xrow, cstride, acc0, SPLIT ? wave : 0, SPLIT ? NW : 1);
  if (DUAL) {
    f32x4_b16 acc1[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) acc1[s] = f32x4_b16{0.f, 0.f, 0.f, 0.f};
    b16_row<NS>(a, a.m1, r, xrow, cstride, acc1, SPLIT ? wave : 0, SPLIT ? NW : 1);
    if (SPLIT) b16_join<NS, NW>(acc1);
    if (SPLIT) __syncthreads();  // the buffer is used again for the first matrix
    if (SPLIT) b16_join<NS, NW>(acc0);
    if (SPLIT && wave != 0) return;
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc0[s][j] = apply_act(a.act, acc0[s][j]) * acc1[s][j];
  } else if (SPLIT) {
    b16_join<NS, NW>(acc0);
    if (wave != 0) return;
  }
  if (POST) {
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc0[s][j] = apply_act(a.act, acc0[s][j]);
  }

  // Result layout of the 16x16 instruction: lane -> token lane % 16, register j -> row 4 * (lane / 16) + j.
  const int64_t row0 = (int64_t)r * 16 + (lane >> 4) * 4;
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const int t = t0 + s * 16 + (lane & 15);
    if (t >= a.T) continue;
    if (y_vec) {
      const int64_t off = a.y_grp16 ? ((int64_t)r * a.T + t) * 16 + (lane >> 4) * 4 : (int64_t)t * a.syt + row0;
      if (a.y_bf16) {
        uint2 v;
        v.x = (uint32_t)f32_to_bf16_rne(acc0[s][0]) | ((uint32_t)f32_to_bf16_rne(acc0[s][1]) << 16);
        v.y = (uint32_t)f32_to_bf16_rne(acc0[s][2]) | ((uint32_t)f32_to_bf16_rne(acc0[s][3]) << 16);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.Y) + off) = v;
      } else {
        *reinterpret_cast<f32x4_b16*>(reinterpret_cast<float*>(a.Y) + off) = acc0[s];
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int64_t off = (int64_t)t * a.syt + (row0 + j) * a.syi;
        if (a.y_bf16)
          reinterpret_cast<uint16_t*>(a.Y)[off] = f32_to_bf16_rne(acc0[s][j]);
        else
          reinterpret_cast<float*>(a.Y)[off] = acc0[s][j];
      }
    }
  }
}

// Token-major activations [T][K] (row pitch ld) into column groups of 16 features, [K/16][T][16].  A workgroup
// turns 16 tokens x 128 features; a half-wave writes the 512 consecutive bytes of one (column group, 16 tokens).
__global__ __launch_bounds__(256) void k_group16(const uint16_t* __restrict__ X, int64_t ld, int T, int nbc,
                                                 uint16_t* __restrict__ Xg) {
  const int i = threadIdx.x;
  const int half = i & 1, t = (int)blockIdx.x * 16 + ((i >> 1) & 15), c = (int)blockIdx.y * 8 + (i >> 5);
  if (t >= T || c >= nbc) return;
  *reinterpret_cast<uint4*>(Xg + ((int64_t)c * T + t) * 16 + half * 8) =
      *reinterpret_cast<const uint4*>(X + (int64_t)t * ld + c * 16 + half * 8);
}

}  // namespace blast_dev
