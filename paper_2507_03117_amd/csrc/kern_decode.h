// Decode kernel: block-sparse product for a handful of tokens (T <= 128 or so).
//
// At these token counts the product is bound by streaming the stored blocks out
// of HBM once (the paper's abstract: data movement dominates), so the kernel is
// organised around the memory pipeline:
//  - one workgroup per (block row, 16-row slice); its four waves deal the stored
//    blocks of the row among themselves, so even a row with a single block keeps
//    a wave busy and a row with many blocks is read by four waves at once;
//  - a 16-row slice of a block is contiguous in memory (16 B rows): a wave copies
//    it global -> LDS with wave-wide 1 KiB requests (whole 128-byte lines, the
//    request shape the L1 path handles best) and reads the matrix-core operand
//    fragments back from LDS; no other wave touches that LDS region, so no
//    barrier is involved, only the wave's own memory counter;
//  - rounds of BPR blocks are double buffered: the copies of the next round are
//    in flight while the current one is multiplied;
//  - activations (a few KiB, cache resident) are read as the second operand,
//    16 tokens per matrix instruction (v_mfma_f32_16x16x32_bf16);
//  - the four partial sums meet in LDS; wave 0 applies the epilogue.
// Same arithmetic as the tile kernels: bf16 products, fp32 accumulation,
// activation on the fp32 sums, one rounding to bf16 where the output is bf16.
#pragma once
#include <type_traits>

#include "kern_common.h"
#include "kern_stream.h"

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
struct DecCfg {
  static constexpr int SLICES = B / 16;       // 16-row slices per block row
  static constexpr int KST = B / 32;          // 32-wide k-steps per block
  static constexpr int SLB = 16 * B * 2;      // bytes of one 16-row slice of a block
  static constexpr int NI = SLB / 1024;       // wave-wide copy instructions per slice
  static constexpr int BPR = (B == 128) ? 2 : 4;  // blocks per wave and round
  static constexpr int NM = DUAL ? 2 : 1;
  static constexpr int PER_ROUND = BPR * (NI + KST * NTT);  // vector-memory operations a wave issues per round
  static constexpr int W_LDS = 4 * 2 * BPR * SLB;           // [wave][buffer][block of the round][slice]
  static constexpr int RED_LDS = 3 * NM * NTT * 4 * 64 * 4;
  static constexpr size_t LDS_BYTES = (size_t)W_LDS + RED_LDS;
  static_assert(SLB % 1024 == 0 && PER_ROUND < 64, "copy granularity / counter range");
};

template <int B, bool DUAL, int NTT>
__global__ __launch_bounds__(256) void k_decode(const DecArgs a) {
  using C = DecCfg<B, DUAL, NTT>;
  constexpr int KST = C::KST, BPR = C::BPR, NM = C::NM;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float (*red)[NM][NTT][4][64] = reinterpret_cast<float (*)[NM][NTT][4][64]>(smem + C::W_LDS);

  // blockIdx.y selects a group of NTT * 16 tokens: more tokens mean more workgroups, each re-reading its
  // weight slice (the first read comes from HBM, the others from cache)
  const int t_base = blockIdx.y * (NTT * 16);
  const int unit = blockIdx.x;
  const int r = unit / C::SLICES, q = unit % C::SLICES;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, l16 = lane & 15, g = lane >> 4;
  unsigned char* wlds = smem + wave * (2 * BPR * C::SLB);

  const int kb0 = ld_idx(a.m0.row_ptr, r), n0 = ld_idx(a.m0.row_ptr, r + 1) - kb0;
  int kb1 = 0, n1 = 0;
  if (DUAL) {
    kb1 = ld_idx(a.m1.row_ptr, r);
    n1 = ld_idx(a.m1.row_ptr, r + 1) - kb1;
  }
  const int n = n0 + n1;
  // this wave's blocks are i = wave + 4 j, j < cnt
  const int cnt = n > wave ? (n - wave + 3) >> 2 : 0;
  const int rounds = (cnt + BPR - 1) / BPR;

  f32x4 acc[NM][NTT];
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int tt = 0; tt < NTT; ++tt) acc[m][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // per-lane byte offsets: inside a slice for the copy (contiguous), inside an activation row, and of
  // this lane's operand fragment inside the LDS image of a slice (row l16, 16-byte chunk 4 s + g)
  const uint32_t cp_off = (uint32_t)(q * C::SLB + lane * 16);
  const uint32_t frag_off = (uint32_t)(l16 * B * 2 + g * 16);
  uint32_t xoff[NTT];
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt) {
    int t = t_base + tt * 16 + l16;
    t = t < a.T ? t : a.T - 1;
    xoff[tt] = ((uint32_t)t * (uint32_t)a.sxt + (uint32_t)g * 8u) * 2u;
  }

  bf16x8 xf[2][BPR][NTT][KST];
  // Requests of one round.  Every round issues the same number of operations (slots past the wave's
  // last block repeat it: a cache hit), so the counter value that means "the previous round has
  // landed" is a compile-time constant.
  auto issue = [&](int rd, auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
#pragma unroll
    for (int p = 0; p < BPR; ++p) {
      int j = rd * BPR + p;
      j = j < cnt ? j : cnt - 1;
      const int i = wave + 4 * j;
      const bool second = DUAL && i >= n0;
      const MatDev& m = second ? a.m1 : a.m0;
      const int k = second ? kb1 + (i - n0) : kb0 + i;
      const int col = ld_idx(m.col_idx, k);
      const unsigned char* xcol = reinterpret_cast<const unsigned char*>(a.X) + (int64_t)col * (B * 2);
#pragma unroll
      for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
        for (int s = 0; s < KST; ++s) xf[buf][p][tt][s] = *reinterpret_cast<const bf16x8*>(xcol + xoff[tt] + s * 64);
      const unsigned char* wblk = reinterpret_cast<const unsigned char*>(m.vals) + (int64_t)k * (B * B * 2);
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        BLAST_GLDS16(wblk + cp_off + ni * 1024, wlds + (buf * BPR + p) * C::SLB + ni * 1024);
    }
  };
  // Straight-line on purpose: a slot past the wave's last block, or a block of the other matrix,
  // multiplies a zeroed operand instead of branching around the matrix instruction (the arithmetic
  // is unchanged: adding 0 * x to an fp32 sum is exact; matrix instructions are not the bottleneck
  // at these token counts).
  auto compute = [&](int rd, auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int p = 0; p < BPR; ++p) {
      const int j = rd * BPR + p;
      const bool valid = j < cnt;
      const bool second = DUAL && (wave + 4 * j) >= n0;
#pragma unroll
      for (int s = 0; s < KST; ++s) {
        const bf16x8 wf = *reinterpret_cast<const bf16x8*>(wlds + (buf * BPR + p) * C::SLB + frag_off + s * 64);
        const bf16x8 w0 = (valid && !second) ? wf : zero;
#pragma unroll
        for (int tt = 0; tt < NTT; ++tt)
          acc[0][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[buf][p][tt][s], w0, acc[0][tt], 0, 0, 0);
        if (DUAL) {
          const bf16x8 w1 = (valid && second) ? wf : zero;
#pragma unroll
          for (int tt = 0; tt < NTT; ++tt)
            acc[NM - 1][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[buf][p][tt][s], w1, acc[NM - 1][tt], 0, 0, 0);
        }
      }
    }
  };
  using Buf0 = std::integral_constant<int, 0>;
  using Buf1 = std::integral_constant<int, 1>;
  // One pipeline stage: start the next round (if any) into the other buffer, wait for this one, multiply.
  auto stage = [&](int rd, auto cur, auto nxt) {
    if (rd + 1 < rounds) {
      issue(rd + 1, nxt);
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(C::PER_ROUND));
    } else {
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0));
    }
    asm volatile("" ::: "memory");
    compute(rd, cur);
    asm volatile("" ::: "memory");
  };
  if (rounds > 0) issue(0, Buf0{});
  for (int rd = 0; rd < rounds; rd += 2) {
    stage(rd, Buf0{}, Buf1{});
    if (rd + 1 < rounds) stage(rd + 1, Buf1{}, Buf0{});
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
