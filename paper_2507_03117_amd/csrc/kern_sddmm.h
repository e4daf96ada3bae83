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
// Work decomposition: a workgroup owns a unit = (stored block, SB x SB sub-block, token chunk); its four
// waves deal the 16-token stages of the chunk among themselves, each accumulating the whole sub-block
// (64 x 64: 2 x 2 register blocking, every fragment used twice) from a private ring of LDS stages - no
// barrier inside the loop, the wave's memory counter is the only synchronisation (the scheme of the
// decode kernel) - and the four partial sums are added in LDS at the end.  When a matrix has too few
// blocks to fill the chip even so, the tokens are cut into chunks across workgroups as well and those
// partial sums meet through fp32 atomics on a zeroed output.
#pragma once
#include "kern_common.h"
#include "kern_stream.h"

namespace blast_dev {

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// The transposing reads of one stage, written as ONE block of assembly that ends with the wait for their
// results.  Two reasons.  (1) The compiler makes every LDS read it knows about wait for ALL outstanding
// LDS-DMA copies (it cannot tell which stage a read touches), which would drain the ring at every stage;
// a read it does not know about waits for nothing, and the wait for the copies of this one stage is
// written out by hand before the block.  (2) Results of an LDS read land some time after the instruction
// was issued; the compiler takes the outputs of an assembly statement as valid at its end, so the wait
// has to sit inside the same statement - otherwise a register copy it chooses to place right after the
// reads would pick up stale values.
// a0 / a1: LDS byte addresses of this lane's half-0 dY fragment of matrix tile 0 / 1; H = distance of
// half 1 (four token rows), X = distance of the X tile.
template <int H, int X>
__device__ __forceinline__ void sd_read_stage2(uint32_t a0, uint32_t a1, u32x2 (&fr)[8]) {
  asm volatile(
      "ds_read_b64_tr_b16 %0, %8 offset:0\n\t"
      "ds_read_b64_tr_b16 %1, %8 offset:%10\n\t"
      "ds_read_b64_tr_b16 %2, %9 offset:0\n\t"
      "ds_read_b64_tr_b16 %3, %9 offset:%10\n\t"
      "ds_read_b64_tr_b16 %4, %8 offset:%11\n\t"
      "ds_read_b64_tr_b16 %5, %8 offset:%12\n\t"
      "ds_read_b64_tr_b16 %6, %9 offset:%11\n\t"
      "ds_read_b64_tr_b16 %7, %9 offset:%12\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(fr[0]), "=&v"(fr[1]), "=&v"(fr[2]), "=&v"(fr[3]), "=&v"(fr[4]), "=&v"(fr[5]), "=&v"(fr[6]), "=&v"(fr[7])
      : "v"(a0), "v"(a1), "n"(H), "n"(X), "n"(X + H)
      : "memory");
}
template <int H, int X>
__device__ __forceinline__ void sd_read_stage1(uint32_t a0, u32x2 (&fr)[4]) {
  asm volatile(
      "ds_read_b64_tr_b16 %0, %4 offset:0\n\t"
      "ds_read_b64_tr_b16 %1, %4 offset:%5\n\t"
      "ds_read_b64_tr_b16 %2, %4 offset:%6\n\t"
      "ds_read_b64_tr_b16 %3, %4 offset:%7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(fr[0]), "=&v"(fr[1]), "=&v"(fr[2]), "=&v"(fr[3])
      : "v"(a0), "n"(H), "n"(X), "n"(X + H)
      : "memory");
}

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
  int n_units;         // workgroups with work: nnz * SUB * SUB * tsplit
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
  static constexpr int NSTAGE = 4;             // 16 KiB of ring per wave at SB = 64: two workgroups per CU
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
  // Workgroup ids are dealt round-robin to the 8 XCDs: consecutive units (blocks of one block row, which
  // read the same columns of dY) are given ids 8 apart, so they run on one XCD and share its L2.
  const int per_xcd = (a.n_units + 7) >> 3;
  const int unit = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (unit >= a.n_units) return;  // whole workgroup, before any barrier
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
  // the four waves deal the 16-token stages of the chunk among themselves: wave w takes w, w + 4, ...
  const int chunk_stages = t_hi > t_lo ? (t_hi - t_lo + C::KT - 1) / C::KT : 0;
  const int n_stage = chunk_stages > wave ? (chunk_stages - wave + 3) >> 2 : 0;

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

  // Copy side, continued: byte offset of a lane's chunk from the first token row of a stage.  A stage that
  // runs past the last token (only the last stage of the last chunk can) clamps its rows to the last token
  // for the copy; the fragments zero those tokens.
  uint32_t yoff[NI], xoff[NI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    yoff[ni] = (uint32_t)crow[ni] * (uint32_t)a.ldy * 2u + (uint32_t)cchunk[ni] * 16u;
    xoff[ni] = (uint32_t)crow[ni] * (uint32_t)a.ldx * 2u + (uint32_t)cchunk[ni] * 16u;
  }
  auto issue = [&](int s) {
    unsigned char* slot = ring + (s % NSTAGE) * C::STAGE;
    const int t0 = t_lo + (wave + 4 * s) * C::KT;
    const unsigned char* ys = ybase + (int64_t)t0 * a.ldy * 2;
    const unsigned char* xs = xbase + (int64_t)t0 * a.ldx * 2;
    if (t0 + C::KT <= a.T) {
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) BLAST_GLDS16(ys + yoff[ni], slot + ni * 1024);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) BLAST_GLDS16(xs + xoff[ni], slot + C::TILE + ni * 1024);
    } else {
      const int last = a.T - 1 - t0;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const uint32_t row = (uint32_t)(crow[ni] < last ? crow[ni] : last);
        BLAST_GLDS16(ys + (row * (uint32_t)a.ldy * 2u + (uint32_t)cchunk[ni] * 16u), slot + ni * 1024);
      }
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const uint32_t row = (uint32_t)(crow[ni] < last ? crow[ni] : last);
        BLAST_GLDS16(xs + (row * (uint32_t)a.ldx * 2u + (uint32_t)cchunk[ni] * 16u), slot + C::TILE + ni * 1024);
      }
    }
  };

  // Fragments of a stage: fr[2*nq + h] = dY fragment half h of matrix tile nq, fr[2*NQ + 2*nq + h] the same
  // of X.  Half 1 lies four token rows below half 0 (same swizzle key), the X tile TILE bytes above.
  constexpr int NF = 4 * NQ;
  const uint32_t ring_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring;

  // ---- ring: NSTAGE - 1 stages of copies in flight behind the one being multiplied ------------------
#pragma unroll 1
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < n_stage) issue(s);

#pragma unroll 1
  for (int s = 0; s < n_stage; ++s) {
    // (the fragment reads of stage s - 1 returned inside their block: its slot goes back to the copier)
    if (s + NSTAGE - 1 < n_stage) issue(s + NSTAGE - 1);
    // copies retire in issue order: "at most (stages issued after s) * OPS outstanding" = stage s has landed
    const int later = (n_stage - 1 - s) < (NSTAGE - 1) ? (n_stage - 1 - s) : (NSTAGE - 1);
    sd_wait_vm(later, C::OPS);
    asm volatile("" ::: "memory");
    u32x2 fr[NF];
    const uint32_t base = ring_addr + (uint32_t)((s % NSTAGE) * C::STAGE);
    if constexpr (NQ == 2)
      sd_read_stage2<4 * C::ROWB, C::TILE>(base + foff[0][0], base + foff[1][0], fr);
    else
      sd_read_stage1<4 * C::ROWB, C::TILE>(base + foff[0][0], fr);
    // tokens of this stage that exist: all 16 except in the last stage of the last chunk
    const int valid = a.T - (t_lo + (wave + 4 * s) * C::KT);
    if (valid < C::KT) {
      const int k0 = 8 * (lane >> 5);  // first token of this lane's fragments inside the stage
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        const int kf = k0 + 4 * (f & 1);  // half 1 holds tokens k0 + 4 .. k0 + 7
#pragma unroll
        for (int w = 0; w < 2; ++w) {  // a register holds two tokens, the even one in its low half
          uint32_t v = fr[f][w];
          if (kf + 2 * w >= valid) v &= 0xFFFF0000u;
          if (kf + 2 * w + 1 >= valid) v &= 0x0000FFFFu;
          fr[f][w] = v;
        }
      }
    }
    bf16x8 fy[NQ], fx[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      const u32x4 yy = {fr[2 * nq][0], fr[2 * nq][1], fr[2 * nq + 1][0], fr[2 * nq + 1][1]};
      const u32x4 xx = {fr[2 * NQ + 2 * nq][0], fr[2 * NQ + 2 * nq][1], fr[2 * NQ + 2 * nq + 1][0],
                        fr[2 * NQ + 2 * nq + 1][1]};
      fy[nq] = __builtin_bit_cast(bf16x8, yy);
      fx[nq] = __builtin_bit_cast(bf16x8, xx);
    }
    // D[m][n] += sum_k A[m][k] B[k][n]: m = feature of dY (row of the block), n = feature of X (column)
#pragma unroll
    for (int mi = 0; mi < NQ; ++mi)
#pragma unroll
      for (int nj = 0; nj < NQ; ++nj)
        acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[mi], fx[nj], acc[mi][nj], 0, 0, 0);
  }

  // ---- the four partial sums meet in LDS (the rings are free once every wave has left its loop); wave w
  // then owns a quarter of the accumulator registers: adds the four copies in a fixed order and stores.
  constexpr int NACC = NQ * NQ * 16;
  float (*red)[NACC][64] = reinterpret_cast<float (*)[NACC][64]>(smem);
  static_assert(sizeof(float) * 4 * NACC * 64 <= C::LDS_BYTES, "the reduction reuses the ring memory");
  __syncthreads();
#pragma unroll
  for (int mi = 0; mi < NQ; ++mi)
#pragma unroll
    for (int nj = 0; nj < NQ; ++nj)
#pragma unroll
      for (int v = 0; v < 16; ++v) red[wave][(mi * NQ + nj) * 16 + v][lane] = acc[mi][nj][v];
  __syncthreads();
  // Result layout of a 32x32 tile: lane -> column n = lane % 32, register v -> row m = 8*(v/4) + 4*(lane/32) + v%4:
  // a store instruction writes two 128-byte row segments.
  float* out = a.dvals + (int64_t)q * (B * B) + (int64_t)(si * C::SB) * B + sj * C::SB;
  const int l32 = lane & 31, lh = lane >> 5;
  constexpr int PER_WAVE = NACC / 4;
#pragma unroll
  for (int e = 0; e < PER_WAVE; ++e) {
    const int id = wave * PER_WAVE + e;  // accumulator register (tile, v)
    const float sum = ((red[0][id][lane] + red[1][id][lane]) + red[2][id][lane]) + red[3][id][lane];
    const int tile = id >> 4, v = id & 15;
    const int mi = tile / NQ, nj = tile % NQ;
    const int m = 32 * mi + 8 * (v >> 2) + 4 * lh + (v & 3);
    float* dst = out + m * B + 32 * nj + l32;
    if (a.tsplit > 1)
      atomicAdd(dst, sum);
    else
      *dst = sum;
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
