// Decode kernel: block-sparse product for a handful of tokens (T <= 128 or so).
//
// At these token counts the product is bound by streaming the stored blocks out
// of HBM once (the paper's abstract: data movement dominates), so the kernel is
// organised around getting every weight byte requested as early as possible:
//  - one workgroup per (block row, 16-row slice); its four waves deal the stored
//    blocks of the row among themselves, so even a row with a single block keeps
//    a wave busy and a row with many blocks is read by four waves at once;
//  - a wave requests the slices of up to BPR of its blocks back to back, straight
//    into registers in matrix-core operand layout (16 rows x 32 k per
//    instruction), before it touches any activation;
//  - activations (a few KiB, cache resident) are read as the second operand,
//    16 tokens per matrix instruction (v_mfma_f32_16x16x32_bf16);
//  - the four partial sums meet in LDS; wave 0 applies the epilogue.
// Same arithmetic as the tile kernels: bf16 products, fp32 accumulation,
// activation on the fp32 sums, one rounding to bf16 where the output is bf16.
#pragma once
#include "kern_common.h"

namespace blast_dev {

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct DecArgs {
  MatDev m0, m1;  // m1 only for the dual (gate/up) kernel
  const uint16_t* X;
  int64_t sxt;    // elements between tokens (token-major, 16-byte aligned rows)
  void* Y;
  int64_t syt, syi;
  int y_bf16;
  int T;
  int act;
};

template <int B, bool DUAL, int NTT>
__global__ __launch_bounds__(256) void k_decode(const DecArgs a) {
  constexpr int SLICES = B / 16;  // 16-row slices per block row
  constexpr int KST = B / 32;     // 32-wide k-steps per block
  constexpr int BPR = 4;          // blocks per wave and round
  constexpr int NM = DUAL ? 2 : 1;
  __shared__ float red[3][NM][NTT][4][64];

  // blockIdx.y selects a group of NTT * 16 tokens: more tokens mean more workgroups, each re-reading its
  // weight slice (the first read comes from HBM, the others from cache)
  const int t_base = blockIdx.y * (NTT * 16);
  const int unit = blockIdx.x;
  const int r = unit / SLICES, q = unit % SLICES;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l16 = lane & 15, g = lane >> 4;

  const int kb0 = ld_idx(a.m0.row_ptr, r), n0 = ld_idx(a.m0.row_ptr, r + 1) - kb0;
  int kb1 = 0, n1 = 0;
  if (DUAL) {
    kb1 = ld_idx(a.m1.row_ptr, r);
    n1 = ld_idx(a.m1.row_ptr, r + 1) - kb1;
  }
  const int n = n0 + n1;

  f32x4 acc[NM][NTT];
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int tt = 0; tt < NTT; ++tt) acc[m][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // per-lane offset of this lane's 16 bytes inside a block slice / an activation row
  const uint32_t woff = (uint32_t)((q * 16 + l16) * B + g * 8) * 2u;
  uint32_t xoff[NTT];
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt) {
    int t = t_base + tt * 16 + l16;
    t = t < a.T ? t : a.T - 1;
    xoff[tt] = ((uint32_t)t * (uint32_t)a.sxt + (uint32_t)g * 8u) * 2u;
  }

  for (int base = wave; base < n; base += 4 * BPR) {
    // 1. request the weight slices of this round's blocks
    bf16x8 wf[BPR][KST];
    int cols[BPR];
    bool second[BPR];
#pragma unroll
    for (int p = 0; p < BPR; ++p) {
      const int i = base + 4 * p;
      second[p] = DUAL && i >= n0;
      if (i < n) {
        const MatDev& m = second[p] ? a.m1 : a.m0;
        const int k = second[p] ? kb1 + (i - n0) : kb0 + i;
        const unsigned char* wblk = reinterpret_cast<const unsigned char*>(m.vals) + (int64_t)k * (B * B * 2);
#pragma unroll
        for (int s = 0; s < KST; ++s) wf[p][s] = *reinterpret_cast<const bf16x8*>(wblk + woff + s * 64);
        cols[p] = ld_idx(m.col_idx, k);
      }
    }
    // 2. activations and matrix instructions
#pragma unroll
    for (int p = 0; p < BPR; ++p) {
      const int i = base + 4 * p;
      if (i < n) {
        const unsigned char* xcol = reinterpret_cast<const unsigned char*>(a.X) + (int64_t)cols[p] * (B * 2);
#pragma unroll
        for (int tt = 0; tt < NTT; ++tt) {
          bf16x8 xf[KST];
#pragma unroll
          for (int s = 0; s < KST; ++s) xf[s] = *reinterpret_cast<const bf16x8*>(xcol + xoff[tt] + s * 64);
#pragma unroll
          for (int s = 0; s < KST; ++s) {
            if (DUAL && second[p])
              acc[NM - 1][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[s], wf[p][s], acc[NM - 1][tt], 0, 0, 0);
            else
              acc[0][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[s], wf[p][s], acc[0][tt], 0, 0, 0);
          }
        }
      }
    }
  }

  // 3. the four partial sums meet in LDS
  if (wave > 0) {
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[wave - 1][m][tt][j][lane] = acc[m][tt][j];
  }
  __syncthreads();
  if (wave > 0) return;
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[m][tt][j] += (red[0][m][tt][j][lane] + red[1][m][tt][j][lane]) + red[2][m][tt][j][lane];

  // 4. epilogue.  Result layout of the 16x16 tile: lane -> weight row l16, register j -> token 4*g + j.
  const int64_t row = (int64_t)r * B + q * 16 + l16;
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int tok = t_base + tt * 16 + 4 * g + j;
      if (tok < a.T) {
        float v = acc[0][tt][j];
        if (DUAL) v = apply_act(a.act, v) * acc[NM - 1][tt][j];
        const int64_t off = (int64_t)tok * a.syt + row * a.syi;
        if (a.y_bf16)
          reinterpret_cast<uint16_t*>(a.Y)[off] = f32_to_bf16_rne(v);
        else
          reinterpret_cast<float*>(a.Y)[off] = v;
      }
    }
}

}  // namespace blast_dev
