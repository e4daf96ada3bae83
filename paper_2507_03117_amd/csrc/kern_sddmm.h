// Gradient of the stored blocks: dvals[q] = dY[:, block row of q]^T-contracted-over-tokens with
// X[:, block column of q], i.e. the entries of dY X^T that fall on kept blocks (the backward pass keeps
// the sparsity pattern of the forward pass: BLaST Sec. 3.2).
//
// The contraction runs over tokens, and activations are token-major: both operands of the matrix
// instruction need, per lane, consecutive TOKENS of one feature, which is a column walk through a
// [token][feature] tile.  gfx950 has a transposing LDS read for exactly this (ds_read_b64_tr_b16): within
// a group of 16 lanes, lane p supplies the address of 4 consecutive features of token row p/4 starting
// at feature 4*(p%4), and lane j receives the 4 token rows of feature j.  So the tiles are copied
// global -> LDS as they are (LDS-DMA, whole 64/128-byte row segments) and turned on the way into the
// registers, two reads per 8-token operand fragment.
//
// Work decomposition: a wave owns a unit = (stored block, SB x SB sub-block, token chunk) and walks its
// tokens 16 at a time through a private ring of LDS stages - no barriers; the memory counter of the wave
// is the only synchronisation (same scheme as the decode kernel).  A 64 x 64 sub-block per wave gives each
// fragment two uses (2 x 2 register blocking).  When a matrix has too few blocks to fill the chip, the
// tokens are cut into chunks and the partial sums meet through fp32 atomics on a zeroed output.
#pragma once
#include "kern_common.h"
#include "kern_stream.h"

namespace blast_dev {

typedef short s16x4 __attribute__((ext_vector_type(4)));

struct SddmmArgs {
  const int* row_ptr;
  const int* col_idx;
  const uint16_t* dY;  // token-major [T][rows], row pitch ldy elements
  const uint16_t* X;   // token-major [T][cols], row pitch ldx elements
  int64_t ldy, ldx;
  float* dvals;        // [nnz][b][b]
  int T;
  int nbr;
  int nnz;
  int tsplit;          // token chunks per sub-block (> 1: atomic accumulation into zeroed dvals)
  int chunk_tokens;    // tokens per chunk, a multiple of 16
  int n_units;         // nnz * SUB * SUB * tsplit
};

template <int B>
struct SdCfg {
  static_assert(B == 32 || B == 64 || B == 128, "block sizes with at least one 32 x 32 matrix tile");
  static constexpr int SB = B < 64 ? B : 64;   // edge of the sub-block one wave accumulates
  static constexpr int NQ = SB / 32;           // 32-wide matrix tiles per side of it
  static constexpr int SUB = B / SB;           // sub-blocks per side of a block
  static constexpr int KT = 16;                // tokens per stage (one matrix instruction deep)
  static constexpr int ROWB = SB * 2;          // bytes of a tile row
  static constexpr int CPR = ROWB / 16;        // 16-byte chunks per tile row
  static constexpr int TILE = KT * ROWB;       // bytes of one operand tile
  static constexpr int NI = TILE / 1024;       // wave-wide copy instructions per tile
  static constexpr int OPS = 2 * NI;           // per stage (dY tile + X tile)
  static constexpr int STAGE = 2 * TILE;
  static constexpr int NSTAGE = 8;
  static constexpr int WAVE_LDS = NSTAGE * STAGE;
  static constexpr size_t LDS_BYTES = 4 * (size_t)WAVE_LDS;
  static_assert(TILE % 1024 == 0 && (NSTAGE - 1) * OPS < 64, "copy granularity / counter range");
  // Swizzle key of a tile row: the four token rows that one transposing read touches must land on
  // different banks.  Rows are ROWB bytes apart, so 128 / ROWB rows share a 128-byte bank line.
  __device__ static __forceinline__ int key(int row) { return (2 * ((row / (128 / ROWB)) % 4)) % CPR; }
};

__device__ __forceinline__ void sd_wait_vm(int later, int ops) {
  // copies retire in issue order: "at most later * ops outstanding" = the current stage has landed
  switch (later * ops) {
    case 0: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0)); break;
    case 2: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(2)); break;
    case 4: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(4)); break;
    case 6: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(6)); break;
    case 8: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(8)); break;
    case 10: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(10)); break;
    case 12: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(12)); break;
    case 14: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(14)); break;
    case 16: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(16)); break;
    case 20: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(20)); break;
    case 24: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(24)); break;
    case 28: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(28)); break;
    default: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0)); break;  // more than needed is always safe
  }
}

template <int B>
__global__ __launch_bounds__(256) void k_sddmm(const SddmmArgs a) {
  using C = SdCfg<B>;
  constexpr int NQ = C::NQ, NI = C::NI, NSTAGE = C::NSTAGE;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int unit = blockIdx.x * 4 + wave;
  if (unit >= a.n_units) return;  // whole wave; there is no barrier in this kernel
  unsigned char* ring = smem + wave * C::WAVE_LDS;

  // unit -> (stored block q, sub-block (si, sj), token chunk tc); token chunks of one sub-block are adjacent
  const int tc = unit % a.tsplit;
  const int rest = unit / a.tsplit;
  const int sj = rest % C::SUB, si = (rest / C::SUB) % C::SUB;
  const int q = rest / (C::SUB * C::SUB);
  // block row of q: the last r with row_ptr[r] <= q
  int lo = 0, hi = a.nbr - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (ld_idx(a.row_ptr, mid) <= q) lo = mid; else hi = mid - 1;
  }
  const int r = lo, c = ld_idx(a.col_idx, q);
  const int t_lo = tc * a.chunk_tokens;
  int t_hi = t_lo + a.chunk_tokens;
  if (t_hi > a.T) t_hi = a.T;
  const int n_stage = t_hi > t_lo ? (t_hi - t_lo + C::KT - 1) / C::KT : 0;

  // ---- per-lane constants -----------------------------------------------------------------------
  // Copy side: instruction ni of a tile writes LDS bytes [ni*1024 + lane*16, +16) = position p = ni*64 + lane
  // in 16-byte units = (tile row p / CPR, slot p % CPR); it fetches chunk slot ^ key(row) of that token row.
  int crow[NI], cchunk[NI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int p = ni * 64 + lane;
    crow[ni] = p / C::CPR;
    cchunk[ni] = (p % C::CPR) ^ C::key(p / C::CPR);
  }
  const unsigned char* ybase = reinterpret_cast<const unsigned char*>(a.dY) + ((int64_t)r * B + si * C::SB) * 2;
  const unsigned char* xbase = reinterpret_cast<const unsigned char*>(a.X) + ((int64_t)c * B + sj * C::SB) * 2;
  // Fragment side: 16-lane group g, lane p in it.  Read h (0, 1) of matrix tile nq fetches token rows
  // 8*(g/2) + 4*h + p/4 at features 32*nq + 16*(g%2) + 4*(p%4) .. +3 and returns token rows
  // 8*(g/2) + 4*h .. +3 of feature 32*nq + 16*(g%2) + p: lane l holds feature l % 32 of the tile and
  // the 8 tokens 8*(l/32) .. +7, the operand layout of the 32x32x16 matrix instruction.
  uint32_t foff[NQ][2];
  {
    const int g = lane >> 4, p = lane & 15;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int row = 8 * (g >> 1) + 4 * h + (p >> 2);
        const int col = 32 * nq + 16 * (g & 1) + 4 * (p & 3);
        foff[nq][h] = (uint32_t)(row * C::ROWB + (((col >> 3) ^ C::key(row)) << 4) + (col & 7) * 2);
      }
  }

  f32x16 acc[NQ][NQ];
#pragma unroll
  for (int mi = 0; mi < NQ; ++mi)
#pragma unroll
    for (int nj = 0; nj < NQ; ++nj)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][nj][v] = 0.0f;

  // token rows past the end are clamped to the last token for the copy and zeroed in the fragments
  auto issue = [&](int s) {
    unsigned char* slot = ring + (s % NSTAGE) * C::STAGE;
    const int t0 = t_lo + s * C::KT;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      int t = t0 + crow[ni];
      t = t < a.T ? t : a.T - 1;
      BLAST_GLDS16(ybase + ((int64_t)t * a.ldy + cchunk[ni] * 8) * 2, slot + ni * 1024);
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      int t = t0 + crow[ni];
      t = t < a.T ? t : a.T - 1;
      BLAST_GLDS16(xbase + ((int64_t)t * a.ldx + cchunk[ni] * 8) * 2, slot + C::TILE + ni * 1024);
    }
  };

#pragma unroll 1
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < n_stage) issue(s);

#pragma unroll 1
  for (int s = 0; s < n_stage; ++s) {
    // fragment reads of the previous stage have returned before its slot is handed back to the copier
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    asm volatile("" ::: "memory");
    if (s + NSTAGE - 1 < n_stage) issue(s + NSTAGE - 1);
    const int later = (n_stage - 1 - s) < (NSTAGE - 1) ? (n_stage - 1 - s) : (NSTAGE - 1);
    sd_wait_vm(later, C::OPS);
    asm volatile("" ::: "memory");
    const unsigned char* slot = ring + (s % NSTAGE) * C::STAGE;
    // tokens of this stage that exist: all 16 except in the last stage of the last chunk
    const int valid = a.T - (t_lo + s * C::KT);
    bf16x8 fy[NQ], fx[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      s16x4 y0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(slot + foff[nq][0]));
      s16x4 y1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(slot + foff[nq][1]));
      s16x4 x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(slot + C::TILE + foff[nq][0]));
      s16x4 x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(slot + C::TILE + foff[nq][1]));
      if (valid < C::KT) {
        const int k0 = 8 * (lane >> 5);  // first token of this lane's fragment inside the stage
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (k0 + e >= valid) { y0[e] = 0; x0[e] = 0; }
          if (k0 + 4 + e >= valid) { y1[e] = 0; x1[e] = 0; }
        }
      }
      const short __attribute__((ext_vector_type(8))) yy = __builtin_shufflevector(y0, y1, 0, 1, 2, 3, 4, 5, 6, 7);
      const short __attribute__((ext_vector_type(8))) xx = __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7);
      fy[nq] = __builtin_bit_cast(bf16x8, yy);
      fx[nq] = __builtin_bit_cast(bf16x8, xx);
    }
    // D[m][n] += sum_k A[m][k] B[k][n]: m = feature of dY (row of the block), n = feature of X (column)
#pragma unroll
    for (int mi = 0; mi < NQ; ++mi)
#pragma unroll
      for (int nj = 0; nj < NQ; ++nj)
        acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[mi], fx[nj], acc[mi][nj], 0, 0, 0);
    asm volatile("" ::: "memory");
  }

  // ---- store.  Result layout of the 32x32 tile: lane -> column n = lane % 32, register v -> row
  // m = 8*(v/4) + 4*(lane/32) + v%4: a store instruction writes two 128-byte row segments.
  float* out = a.dvals + (int64_t)q * (B * B) + (int64_t)(si * C::SB) * B + sj * C::SB;
  const int l32 = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int mi = 0; mi < NQ; ++mi)
#pragma unroll
    for (int nj = 0; nj < NQ; ++nj)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = 32 * mi + 8 * (v / 4) + 4 * lh + (v % 4);
        float* dst = out + m * B + 32 * nj + l32;
        if (a.tsplit > 1)
          atomicAdd(dst, acc[mi][nj][v]);
        else
          *dst = acc[mi][nj][v];
      }
}

// Any block size, any strides: one workgroup per stored block, plain fp32 multiply-adds from global memory.
// Serves b = 16, feature-major or unaligned operands (sizes at which a tuned kernel would not matter).
struct SddmmGenericArgs {
  const int* row_ptr;
  const int* col_idx;
  const uint16_t* dY;
  const uint16_t* X;
  int64_t syi, syt, sxk, sxt;  // element strides along features / tokens
  float* dvals;
  int T, nbr, b;
};

__global__ __launch_bounds__(256) void k_sddmm_generic(const SddmmGenericArgs a) {
  const int q = blockIdx.x;
  int lo = 0, hi = a.nbr - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (a.row_ptr[mid] <= q) lo = mid; else hi = mid - 1;
  }
  const int r = lo, c = a.col_idx[q];
  const int b = a.b;
  for (int idx = threadIdx.x; idx < b * b; idx += blockDim.x) {
    const int i = idx / b, j = idx % b;
    const uint16_t* py = a.dY + ((int64_t)r * b + i) * a.syi;
    const uint16_t* px = a.X + ((int64_t)c * b + j) * a.sxk;
    float s = 0.0f;
    for (int t = 0; t < a.T; ++t) {
      const float y = __builtin_bit_cast(float, (uint32_t)py[(int64_t)t * a.syt] << 16);
      const float x = __builtin_bit_cast(float, (uint32_t)px[(int64_t)t * a.sxt] << 16);
      s = __builtin_fmaf(y, x, s);
    }
    a.dvals[(int64_t)q * b * b + idx] = s;
  }
}

__global__ __launch_bounds__(256) void k_zero_f32(float* p, int64_t n) {
  const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i + 3 < n) {
    *reinterpret_cast<float4*>(p + i) = float4{0.f, 0.f, 0.f, 0.f};
  } else {
    for (int64_t k = i; k < n; ++k) p[k] = 0.f;
  }
}

}  // namespace blast_dev
