// Generic tile kernel: one workgroup per (block row, token tile), register-staged
// global -> LDS copies.  Handles every layout, alignment and block size; it is
// the fallback of the streaming kernel and the reference point for it.
#pragma once
#include "kern_common.h"

namespace blast_dev {

template <int B>
struct TileCfg {
  static constexpr int TOKW = (B == 128) ? 2 : 4;       // waves along tokens
  static constexpr int ROWW = 4 / TOKW;                 // waves along weight rows
  static constexpr int WT_ROW = (B >= 64) ? 64 : B;     // weight rows per wave
  static constexpr int NI = (WT_ROW + 31) / 32;         // 32-row MFMA tiles per wave
  static constexpr int MI = 2;                          // 32-token MFMA tiles per wave
  static constexpr int TT = TOKW * 64;                  // tokens per workgroup tile
  static constexpr int LD = B + 8;                      // LDS row pitch in bf16 (16-byte pad: conflict-free b128 reads)
  static constexpr int CPR = B / 8;                     // 16-byte chunks per row
  static constexpr int NCHW = B * CPR;                  // chunks in a weight block
  static constexpr int NCHX = TT * CPR;                 // chunks in an X tile
  static constexpr int WPT = (NCHW + 255) / 256;
  static constexpr int XPT = (NCHX + 255) / 256;
  static constexpr int KSTEPS = B / 16;
  static constexpr size_t LDS_BYTES = (size_t)(TT + B) * LD * 2;
};

template <int B>
struct Staged {
  uint4 w[TileCfg<B>::WPT];
  uint4 x[TileCfg<B>::XPT];
};

// Global -> registers for stored block k of a matrix (its values and the X slice it selects).
template <int B>
__device__ __forceinline__ void load_stage(const TileArgs& a, const MatDev& m, int k, int t0, Staged<B>& s) {
  using C = TileCfg<B>;
  const int tid = threadIdx.x;
  const uint16_t* wblk = m.vals + (int64_t)k * B * B;
  const int64_t c = m.col_idx[k];
#pragma unroll
  for (int j = 0; j < C::WPT; ++j) {
    const int idx = tid + 256 * j;
    if (C::NCHW % 256 == 0 || idx < C::NCHW) s.w[j] = *reinterpret_cast<const uint4*>(wblk + (int64_t)idx * 8);
  }
#pragma unroll
  for (int j = 0; j < C::XPT; ++j) {
    const int idx = tid + 256 * j;
    const int tok = idx / C::CPR, c8 = idx % C::CPR;
    const int t = t0 + tok;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (t < a.T) {
      if (a.x_vec) {
        v = *reinterpret_cast<const uint4*>(a.X + (int64_t)t * a.sxt + c * B + c8 * 8);
      } else {
        const uint16_t* p = a.X + (int64_t)t * a.sxt + (c * B + c8 * 8) * a.sxk;
        uint32_t e[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) e[q] = p[q * a.sxk];
        v = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
      }
    }
    s.x[j] = v;
  }
}

template <int B>
__device__ __forceinline__ void store_stage(uint16_t* Xs, uint16_t* Ws, const Staged<B>& s) {
  using C = TileCfg<B>;
  const int tid = threadIdx.x;
#pragma unroll
  for (int j = 0; j < C::WPT; ++j) {
    const int idx = tid + 256 * j;
    if (C::NCHW % 256 == 0 || idx < C::NCHW)
      *reinterpret_cast<uint4*>(Ws + (idx / C::CPR) * C::LD + (idx % C::CPR) * 8) = s.w[j];
  }
#pragma unroll
  for (int j = 0; j < C::XPT; ++j) {
    const int idx = tid + 256 * j;
    *reinterpret_cast<uint4*>(Xs + (idx / C::CPR) * C::LD + (idx % C::CPR) * 8) = s.x[j];
  }
}

// acc[mi][ni] += Xtile(wave's 64 tokens) * Wblock(wave's rows)^T from LDS.
template <int B>
__device__ __forceinline__ void mma_stage(const uint16_t* Xs, const uint16_t* Ws, int tw, int rw,
                                          f32x16 (&acc)[TileCfg<B>::MI][TileCfg<B>::NI]) {
  using C = TileCfg<B>;
  const int lane = threadIdx.x & 63, l32 = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int kk = 0; kk < C::KSTEPS; ++kk) {
    bf16x8 af[C::MI], bfg[C::NI];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
      af[mi] = *reinterpret_cast<const bf16x8*>(Xs + (tw * 64 + mi * 32 + l32) * C::LD + kk * 16 + lh * 8);
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      if (C::WT_ROW >= 32 || l32 < C::WT_ROW) {
        bfg[ni] = *reinterpret_cast<const bf16x8*>(Ws + (rw * C::WT_ROW + ni * 32 + l32) * C::LD + kk * 16 + lh * 8);
      } else {
        bfg[ni] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      }
    }
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfg[ni], acc[mi][ni], 0, 0, 0);
  }
}

// All stored blocks of block row r of matrix m, register-prefetched one block ahead.
template <int B>
__device__ __forceinline__ void run_row(const TileArgs& a, const MatDev& m, int r, int t0, uint16_t* Xs, uint16_t* Ws,
                                        int tw, int rw, f32x16 (&acc)[TileCfg<B>::MI][TileCfg<B>::NI]) {
  const int kb = m.row_ptr[r], ke = m.row_ptr[r + 1];
  Staged<B> st;
  if (kb < ke) load_stage<B>(a, m, kb, t0, st);
  for (int k = kb; k < ke; ++k) {
    __syncthreads();  // everyone is done reading the previous stage
    store_stage<B>(Xs, Ws, st);
    __syncthreads();
    if (k + 1 < ke) load_stage<B>(a, m, k + 1, t0, st);
    mma_stage<B>(Xs, Ws, tw, rw, acc);
  }
}

// One workgroup = one (block row, token tile).  DUAL: two matrices with the same
// shape share the tile; the epilogue writes bf16 act(acc0) * acc1.
template <int B, bool DUAL, bool POST = false>
__global__ __launch_bounds__(256) void k_spmm_tile(const TileArgs a) {
  static_assert(!(POST && DUAL), "an activation on the output belongs to the single-matrix product");
  using C = TileCfg<B>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Xs = reinterpret_cast<uint16_t*>(smem);
  uint16_t* Ws = Xs + C::TT * C::LD;

  const int wg = blockIdx.x;
  const int rank = wg / a.ntt, tt = wg % a.ntt;
  const int r = a.row_order ? a.row_order[rank] : rank;
  const int t0 = tt * C::TT;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l32 = lane & 31, lh = lane >> 5;
  const int tw = wave % C::TOKW, rw = wave / C::TOKW;

  f32x16 acc0[C::MI][C::NI];
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = 0.0f;
  run_row<B>(a, a.m0, r, t0, Xs, Ws, tw, rw, acc0);

  if (DUAL) {
    f32x16 acc1[C::MI][C::NI];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc1[mi][ni][j] = 0.0f;
    run_row<B>(a, a.m1, r, t0, Xs, Ws, tw, rw, acc1);
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = apply_act(a.act, acc0[mi][ni][j]) * acc1[mi][ni][j];
  }
  if (POST) {
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = apply_act(a.act, acc0[mi][ni][j]);
  }

  // Result layout of the 32x32 MFMA: lane -> column (weight row) l32, register j -> token 8*(j/4) + 4*lh + j%4.
  if (C::WT_ROW < 32 && l32 >= C::WT_ROW) return;
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      const int64_t row = (int64_t)r * B + rw * C::WT_ROW + ni * 32 + l32;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int tok = t0 + tw * 64 + mi * 32 + 8 * (j / 4) + 4 * lh + (j % 4);
        if (tok < a.T) {
          const float v = acc0[mi][ni][j];
          const int64_t off = (int64_t)tok * a.syt + row * a.syi;
          if (a.y_bf16)
            reinterpret_cast<uint16_t*>(a.Y)[off] = f32_to_bf16_rne(v);
          else
            reinterpret_cast<float*>(a.Y)[off] = v;
        }
      }
    }
}


}  // namespace blast_dev
