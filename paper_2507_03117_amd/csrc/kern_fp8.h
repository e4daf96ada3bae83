// Block-sparse product with both operands in E5M2 (8-bit floating point: the second data type the paper
// runs its kernel in, BLaST Sec. 5.2): Y = W~ X, fp32 accumulation.
//
// Same loop as the bf16 product (Sec. 3.4: every output tile walks the stored blocks of its block row),
// organised like the stored-block-gradient kernel: a wave accumulates a 64-token x 64-row tile (2 x 2
// register blocking of 32x32x64 matrix instructions of the f8f6f4 family, which run at twice the rate of the
// 16-bit ones) from a private ring of LDS stages filled by LDS-DMA copies; there is no barrier in the loop,
// the wave's memory counter is the only synchronisation.
//  - A stage is a 64-deep contraction slice: 64 weight rows x 64 bytes and 64 tokens x 64 bytes, 4 KiB each
//    (the L1 path is bound by cache lines requested, not bytes: 64-byte row segments are the widest a
//    64 x 64 block offers, and a block's weight tile is then 4 KiB of whole lines).
//  - A lane reads two 16-byte chunks per operand row (32 contraction indices), the operand of one 64-deep
//    matrix instruction; lanes 0-31 take chunks 0 and 2 of a row, lanes 32-63 chunks 1 and 3.  Both
//    operands use the same assignment, so every contraction index meets its partner exactly once.
//  - The four chunks of a row are XOR-swizzled in LDS by (row / 2) % 4 (on the global-address side of the
//    copy): the eight rows one read cycle touches then cover all banks.
// One byte per value halves every byte count of the bf16 kernels (HBM, L2 -> LDS, LDS -> registers) per
// multiply-add, which is what bounds them.
//  - KSPLIT = false (many tokens): a workgroup owns (block row, 64-row sub-block, 256 tokens), one 64-token
//    tile per wave; the four waves read the same weight tiles (L1 hits).
//  - KSPLIT = true (up to a few token tiles): a workgroup owns (block row, sub-block, 64 tokens) and its
//    four waves deal the stages among themselves; the partial sums are added in LDS in a fixed order.
//    With CHUNK the unit is a chunk of at most 16 stored blocks from the packer's chunk plan instead of a
//    whole block row; rows cut into several chunks add into a zeroed fp32 output atomically (a very long
//    row would otherwise be the critical path of the launch).
#pragma once
#include "kern_common.h"
#include "kern_stream.h"

namespace blast_dev {

struct Fp8Args {
  const int* row_ptr;
  const int* col_idx;
  const int* row_order;  // may be null
  const uint8_t* vals;   // [nnz][b][b] E5M2
  const uint8_t* X;      // token-major [T][cols] E5M2, row pitch ldx bytes (multiple of 16); or column groups, see x_cg
  int64_t ldx;
  int64_t x_cg;          // 0: token-major.  Else X is [cols/64][T][64]: bytes between two column groups (ldx = 64)
  void* Y;               // token-major [T][rows], row pitch ldy elements
  int64_t ldy;
  int y_bf16;
  int y_fast;            // 1: every byte offset inside a 64-token slab of Y fits 31 bits
  int T;
  int n_units;           // (block rows, or chunk slots with CHUNK) * SUB
  int groups;            // token groups per unit (256 tokens each without KSPLIT, 64 with)
  // chunk plan written by the packer (CHUNK instances only): hdr[0] = number of chunks
  const int* hdr;
  const int* chunk_row;  // block row of the chunk; bit 31 set when the row has several chunks
  const int* chunk_kb;   // first stored block of the chunk
  const int* chunk_ke;   // one past its last stored block
};

#ifndef BLAST_FP8_NSTAGE
#define BLAST_FP8_NSTAGE 2  // 16 KiB of ring per wave, 64 KiB per workgroup: two workgroups per CU (measured: three stages with one workgroup per CU are 20-30 % slower)
#endif

template <int B>
struct Fp8Cfg {
  static_assert(B == 64 || B == 128, "blocks of at least 64 x 64");
  static constexpr int SB = 64;               // weight rows (and tokens) of a wave's tile
  static constexpr int SUB = B / SB;          // sub-blocks of rows per block row
  static constexpr int KS = 64;               // contraction depth of a stage, = bytes of a tile row
  static constexpr int KSL = B / KS;          // stages per stored block
  static constexpr int CPR = KS / 16;         // 16-byte chunks per tile row
  static constexpr int TILE = SB * KS;        // 4 KiB
  static constexpr int NI = TILE / 1024;      // wave-wide copy instructions per tile
  static constexpr int OPS = 2 * NI;
  static constexpr int STAGE = 2 * TILE;
  static constexpr int NSTAGE = BLAST_FP8_NSTAGE;
  static constexpr int WAVE_LDS = NSTAGE * STAGE;
  static constexpr size_t LDS_BYTES = 4 * (size_t)WAVE_LDS;
  __device__ static __forceinline__ int key(int row) { return (row >> 1) & 3; }
};


__device__ __forceinline__ void fp8_wait_vm(int outstanding) {
  switch (outstanding) {
    case 0: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0)); break;
    case 8: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(8)); break;
    case 16: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(16)); break;
    case 24: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(24)); break;
    default: __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0)); break;  // more than needed is always safe
  }
}

typedef long i64x2 __attribute__((ext_vector_type(2)));

template <int B, bool KSPLIT, bool CHUNK = false>
__global__ __launch_bounds__(256) void k_spmm_fp8(const Fp8Args a) {
  static_assert(!CHUNK || KSPLIT, "the chunk plan serves the few-token form");
  using C = Fp8Cfg<B>;
  constexpr int NI = C::NI, NSTAGE = C::NSTAGE;
  static_assert(C::OPS == 8 && (NSTAGE - 1) * C::OPS <= 24, "fp8_wait_vm lists multiples of eight up to 24");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  // Workgroup ids are dealt round-robin to the 8 XCDs: the token groups of one unit are given ids 8 apart,
  // so they run on one XCD and the re-reads of the unit's weight tiles hit its L2.
  const int blk = blockIdx.x, span = 8 * a.groups;
  const int rem = blk % span;
  const int unit = (blk / span) * 8 + (rem & 7);
  if (unit >= a.n_units) return;  // whole workgroup, before any barrier
  const int tg = rem >> 3;
  const int rank = unit / C::SUB, si = unit % C::SUB;
  int r, kb, row_stages;
  bool shared_row = false;
  if (CHUNK) {
    if (rank >= ld_idx(a.hdr, 0)) return;  // the grid is sized by an upper bound of the number of chunks
    const int cr = ld_idx(a.chunk_row, rank);
    r = cr & 0x7FFFFFFF;
    shared_row = cr < 0;
    kb = ld_idx(a.chunk_kb, rank);
    row_stages = (ld_idx(a.chunk_ke, rank) - kb) * C::KSL;
  } else {
    r = a.row_order ? ld_idx(a.row_order, rank) : rank;
    kb = ld_idx(a.row_ptr, r);
    row_stages = (ld_idx(a.row_ptr, r + 1) - kb) * C::KSL;
  }
  // first token of this wave's tile; which stages of the row it walks
  const int t0 = KSPLIT ? tg * C::SB : (tg * 4 + wave) * C::SB;
  const int first = KSPLIT ? wave : 0, step = KSPLIT ? 4 : 1;
  int n_stage = row_stages > first ? (row_stages - first + step - 1) / step : 0;
  if (t0 >= a.T) {
    if (!KSPLIT) return;  // a wave without tokens (no barrier in this mode)
    n_stage = 0;
  }
  unsigned char* ring = smem + wave * C::WAVE_LDS;

  // ---- per-lane constants -----------------------------------------------------------------------
  // Copy side: instruction ni of a tile writes LDS bytes [ni*1024 + lane*16, +16) = position p = ni*64 + lane
  // in 16-byte units = (tile row p / 4, slot p % 4); it fetches chunk slot ^ key(row) of that row.
  uint32_t woff[NI], xoff[NI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int p = ni * 64 + lane, row = p / C::CPR, chunk = (p % C::CPR) ^ C::key(row);
    woff[ni] = (uint32_t)((si * C::SB + row) * B + chunk * 16);
    int t = t0 + row;
    t = t < a.T ? t : a.T - 1;  // rows past the last token re-read it; their results are never stored
    t = t < 0 ? 0 : t;
    xoff[ni] = (uint32_t)t * (uint32_t)a.ldx + (uint32_t)(chunk * 16);
  }
  // Fragment side: lane l reads the 16-byte chunks l / 32 and l / 32 + 2 of tile row 32 h + l % 32.
  uint32_t foff[2][2];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int row = 32 * h + (lane & 31);
      foff[h][c] = (uint32_t)(row * C::KS + ((((lane >> 5) + 2 * c) ^ C::key(row)) << 4));
    }

  f32x16 acc[2][2];  // [token half][row half]
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int nj = 0; nj < 2; ++nj)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][nj][v] = 0.0f;

  auto issue = [&](int s) {
    const int gs = first + step * s;          // stage of the row: stored block gs / KSL, slice gs % KSL
    const int q = kb + gs / C::KSL, ks = gs % C::KSL;
    const int col = ld_idx(a.col_idx, q);
    unsigned char* slot = ring + (s % NSTAGE) * C::STAGE;
    const unsigned char* wsrc = a.vals + (int64_t)q * (B * B) + ks * C::KS;
    // column groups of 64: one token's share of a stage is a whole row of the group, so the copy instructions
    // fetch whole 128-byte lines (two tokens each) instead of the 64-byte half of a line per token
    const unsigned char* xsrc = a.x_cg ? a.X + ((int64_t)col * C::KSL + ks) * a.x_cg : a.X + (int64_t)col * B + ks * C::KS;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) BLAST_GLDS16(wsrc + woff[ni], slot + ni * 1024);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) BLAST_GLDS16(xsrc + xoff[ni], slot + C::TILE + ni * 1024);
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
    // copies retire in issue order: "at most (stages issued after s) * OPS outstanding" = stage s has landed
    const int later = (n_stage - 1 - s) < (NSTAGE - 1) ? (n_stage - 1 - s) : (NSTAGE - 1);
    fp8_wait_vm(later * C::OPS);
    asm volatile("" ::: "memory");
    const unsigned char* slot = ring + (s % NSTAGE) * C::STAGE;
    i64x2 fw[2][2], fx[2][2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        fw[h][c] = *reinterpret_cast<const i64x2*>(slot + foff[h][c]);
        fx[h][c] = *reinterpret_cast<const i64x2*>(slot + C::TILE + foff[h][c]);
      }
    // D[m][n] += sum_k A[m][k] B[k][n]: m = token, n = weight row.  One 64-deep matrix instruction of the
    // f8f6f4 family per 32 x 32 tile and stage (twice the rate of the 16-deep E5M2 instruction): a lane hands
    // over its 32 bytes of the row - the same two chunks on both operands, so whatever contraction index the
    // hardware gives byte j of lane half h, it meets its partner.  Formats: E5M2 (code 1) on both sides; the
    // block scales the instruction takes are all 2^0 (E8M0 code 127 in every byte).
    typedef int v8i __attribute__((ext_vector_type(8)));
    struct Pair {
      i64x2 lo, hi;
    };
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj) {
        const v8i ax = __builtin_bit_cast(v8i, (Pair{fx[mi][0], fx[mi][1]}));
        const v8i bw = __builtin_bit_cast(v8i, (Pair{fw[nj][0], fw[nj][1]}));
        acc[mi][nj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ax, bw, acc[mi][nj], 1, 1, 0, 0x7F7F7F7F, 0,
                                                                       0x7F7F7F7F);
      }
    asm volatile("" ::: "memory");
  }

  // Result layout of a 32x32 tile: lane -> weight row n = lane % 32, register v -> token
  // m = 8*(v/4) + 4*(lane/32) + v%4: a store instruction writes 32 consecutive rows of two tokens.
  const int l32 = lane & 31, lh = lane >> 5;
  const int64_t row0 = (int64_t)r * B + si * C::SB;
  auto store = [&](int mi, int nj, int v, float val) {
    const int t = t0 + 32 * mi + 8 * (v >> 2) + 4 * lh + (v & 3);
    if (t < a.T) {
      const int64_t off = (int64_t)t * a.ldy + row0 + 32 * nj + l32;
      if (CHUNK && shared_row)
        atomicAdd(reinterpret_cast<float*>(a.Y) + off, val);  // fp32 output, zeroed before the launch
      else if (a.y_bf16)
        reinterpret_cast<uint16_t*>(a.Y)[off] = f32_to_bf16_rne(val);
      else
        reinterpret_cast<float*>(a.Y)[off] = val;
    }
  };
  if (!KSPLIT) {
    if (t0 + C::SB <= a.T && a.y_fast) {
      // Whole token tile: one 64-bit lane address, the token step as a uniform 32-bit product, no predication
      // (a stored value then costs a conversion, an add and the store).
      const uint32_t esz = a.y_bf16 ? 2u : 4u;
      uint32_t pitch = (uint32_t)a.ldy * esz;
      asm volatile("" : "+s"(pitch));  // keeps the multiples of the pitch out of long-lived registers
      unsigned char* p0 = reinterpret_cast<unsigned char*>(a.Y) + ((int64_t)(t0 + 4 * lh) * a.ldy + row0 + l32) * esz;
#pragma unroll
      for (int nj = 0; nj < 2; ++nj)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const uint32_t dt = 32 * mi + 8 * (v >> 2) + (v & 3);
            unsigned char* pj = p0 + 32 * nj * esz + __builtin_amdgcn_readfirstlane(dt * pitch);
            if (a.y_bf16)
              *reinterpret_cast<uint16_t*>(pj) = f32_to_bf16_rne(acc[mi][nj][v]);
            else
              *reinterpret_cast<float*>(pj) = acc[mi][nj][v];
          }
      return;
    }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj)
#pragma unroll
        for (int v = 0; v < 16; ++v) store(mi, nj, v, acc[mi][nj][v]);
  } else {
    // the four partial sums meet in LDS (the rings are free once every wave has left its loop); wave w then
    // owns accumulator tile w: adds the four copies in a fixed order and stores
    float (*red)[64][64] = reinterpret_cast<float (*)[64][64]>(smem);
    static_assert(sizeof(float) * 4 * 64 * 64 <= C::LDS_BYTES, "the reduction reuses the ring memory");
    __syncthreads();
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int nj = 0; nj < 2; ++nj)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][(mi * 2 + nj) * 16 + v][lane] = acc[mi][nj][v];
    __syncthreads();
    const int mi = wave >> 1, nj = wave & 1;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int id = wave * 16 + v;
      store(mi, nj, v, ((red[0][id][lane] + red[1][id][lane]) + red[2][id][lane]) + red[3][id][lane]);
    }
  }
}

// Exact widening of an E5M2 code: it is the upper byte of an IEEE half.
__device__ __forceinline__ float e5m2_to_f32(uint8_t c) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)((uint16_t)c << 8));
}

// Any block size, any strides: one workgroup per (block row, 64 tokens), plain fp32 multiply-adds from
// global memory.  Serves b = 16 / 32, feature-major or unaligned operands.
struct Fp8GenericArgs {
  const int* row_ptr;
  const int* col_idx;
  const uint8_t* vals;
  const uint8_t* X;
  int64_t sxk, sxt;  // byte strides of X along features / tokens
  void* Y;
  int64_t syt, syi;  // element strides of Y along tokens / rows
  int y_bf16;
  int T, b;
};

__global__ __launch_bounds__(256) void k_spmm_fp8_generic(const Fp8GenericArgs a) {
  const int r = blockIdx.x, t_base = blockIdx.y * 64;
  const int b = a.b;
  const int kb = a.row_ptr[r], ke = a.row_ptr[r + 1];
  for (int idx = threadIdx.x; idx < b * 64; idx += blockDim.x) {
    const int i = idx / 64, t = t_base + idx % 64;
    if (t >= a.T) continue;
    float s = 0.0f;
    for (int q = kb; q < ke; ++q) {
      const uint8_t* w = a.vals + ((int64_t)q * b + i) * b;
      const uint8_t* x = a.X + (int64_t)a.col_idx[q] * b * a.sxk + (int64_t)t * a.sxt;
      for (int j = 0; j < b; ++j) s = __builtin_fmaf(e5m2_to_f32(w[j]), e5m2_to_f32(x[(int64_t)j * a.sxk]), s);
    }
    const int64_t off = (int64_t)t * a.syt + ((int64_t)r * b + i) * a.syi;
    if (a.y_bf16)
      reinterpret_cast<uint16_t*>(a.Y)[off] = f32_to_bf16_rne(s);
    else
      reinterpret_cast<float*>(a.Y)[off] = s;
  }
}

// bf16 -> E5M2, round to nearest, ties to the even mantissa, overflow to infinity; integer arithmetic on
// the bit patterns (no dependence on a conversion instruction's rounding or saturation mode).
__device__ __forceinline__ uint8_t bf16_to_e5m2(uint16_t h) {
  const uint32_t sign = (h >> 8) & 0x80u;
  const int e8 = (h >> 7) & 0xFF;
  const uint32_t m7 = h & 0x7Fu;
  if (e8 == 0xFF) return (uint8_t)(sign | (m7 ? 0x7Eu : 0x7Cu));  // nan / inf
  if (e8 == 0) return (uint8_t)sign;                               // zero and bf16 subnormals (below 2^-126)
  const int E = e8 - 127;
  if (E >= -14) {
    // normal: keep 2 of the 7 mantissa bits
    uint32_t q = m7 >> 5;
    const uint32_t rem = m7 & 31u;
    if (rem > 16u || (rem == 16u && (q & 1u))) ++q;
    int biased = E + 15;
    if (q == 4u) {
      q = 0u;
      ++biased;
    }
    if (biased >= 31) return (uint8_t)(sign | 0x7Cu);
    return (uint8_t)(sign | ((uint32_t)biased << 2) | q);
  }
  // subnormal target: the value in units of 2^-16 is (128 + m7) * 2^(E + 9), with E + 9 <= -6
  const int sh = -(E + 9);
  if (sh > 9) return (uint8_t)sign;  // below a quarter of the smallest subnormal
  const uint32_t sig = 128u + m7;
  uint32_t n = sig >> sh;
  const uint32_t rem = sig & ((1u << sh) - 1u), half = 1u << (sh - 1);
  if (rem > half || (rem == half && (n & 1u))) ++n;
  return (uint8_t)(sign | n);  // n = 4 is the smallest normal: the carry is the right code
}

// One thread converts 8 consecutive values (a 16-byte read and an 8-byte write when both pointers allow it).
__global__ __launch_bounds__(256) void k_quantize_e5m2(const uint16_t* __restrict__ in, int64_t n,
                                                       uint8_t* __restrict__ out) {
  const int64_t i0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (i0 >= n) return;
  const bool wide = ((reinterpret_cast<uintptr_t>(in) & 15u) | (reinterpret_cast<uintptr_t>(out) & 7u)) == 0 && i0 + 8 <= n;
  if (wide) {
    const uint4 v = *reinterpret_cast<const uint4*>(in + i0);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    unsigned long long packed = 0ull;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      packed |= (unsigned long long)bf16_to_e5m2((uint16_t)(w[j] & 0xFFFFu)) << (16 * j);
      packed |= (unsigned long long)bf16_to_e5m2((uint16_t)(w[j] >> 16)) << (16 * j + 8);
    }
    *reinterpret_cast<unsigned long long*>(out + i0) = packed;
  } else {
    for (int64_t i = i0; i < n && i < i0 + 8; ++i) out[i] = bf16_to_e5m2(in[i]);
  }
}

// Token-major bf16 [T][K] (row pitch ld elements) -> E5M2 in column groups of 64: out[(k/64) T + t][k%64].
// One thread converts 8 consecutive features: a 16-byte read, an 8-byte write.
__global__ __launch_bounds__(256) void k_quantize_e5m2_groups(const uint16_t* __restrict__ in, int64_t ld, int64_t T,
                                                              int64_t K, uint8_t* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // over T * K / 8
  const int64_t per_row = K / 8;
  if (i >= T * per_row) return;
  const int64_t t = i / per_row, k = (i % per_row) * 8;
  const uint16_t* src = in + t * ld + k;
  unsigned long long packed = 0ull;
#pragma unroll
  for (int j = 0; j < 8; ++j) packed |= (unsigned long long)bf16_to_e5m2(src[j]) << (8 * j);
  *reinterpret_cast<unsigned long long*>(out + ((k / 64) * T + t) * 64 + (k % 64)) = packed;
}

}  // namespace blast_dev
