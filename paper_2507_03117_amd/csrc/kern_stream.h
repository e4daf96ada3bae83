// Streaming tile kernel (fast path: token-major, 16-byte aligned activations).
//
// A persistent workgroup walks a static list of (block row, token tile) items and
// treats the stored blocks of all its items as ONE stream of steps (Listing 2's
// loop, flattened across output tiles).  A step is a KS-wide slice along the
// contraction dimension of one stored block: its weight slice and the matching
// activation slice are copied global -> LDS by the memory pipeline itself (no
// register staging) into a ring of NSTAGE stages.  While step i is multiplied out
// of stage i % NSTAGE, the copies of the following steps are in flight or being
// issued, also across item boundaries.  Two workgroups share a CU so that one
// computes while the other waits for its copies.
//
// LDS rows are stored unpadded (a copy instruction writes 1 KiB contiguous per
// wave); bank conflicts of the 16-byte fragment reads are avoided by XOR-ing the
// 16-byte chunk index with a key derived from the row, applied on the
// global-address side of the copy.
#pragma once
#include "kern_common.h"

namespace blast_dev {

#define BLAST_GLDS16(gptr, lptr)                                                                   \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gptr),          \
                                   (__attribute__((address_space(3))) void*)(lptr), 16, 0, 0)

// s_waitcnt immediate that waits for vmcnt <= n and nothing else (gfx9 encoding).
#define BLAST_VMCNT(n) (0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

// TW = waves along the token dimension (4: 256-token tiles, 2: 128-token tiles).  Wide tiles read each
// weight block once per 256 tokens; narrow tiles double the number of items, which matters when a
// matrix has fewer (block row, token tile) pairs than the chip has workgroup slots.
template <int B, int TW>
struct StreamCfg {
  static_assert(TW == 2 || TW == 4, "two or four waves along tokens");
  static_assert(B / (4 / TW) >= 32, "a wave needs at least 32 weight rows");
  static constexpr int TOKW = TW;                  // waves along tokens
  static constexpr int ROWW = 4 / TOKW;            // waves along weight rows
  static constexpr int WT_ROW = B / ROWW;          // weight rows per wave
  static constexpr int NI = WT_ROW / 32;
  static constexpr int MI = 2;
  static constexpr int TT = TOKW * 64;             // tokens per workgroup tile
  // Contraction slice per step.  The L1 path moves about one cache line per 2.5 clk whatever the
  // line's used fraction, so a row of a stage is a whole 128-byte line wherever the block allows.
  static constexpr int KS = (B >= 64) ? 64 : 32;
  static constexpr int NSLICE = B / KS;
  static constexpr int ROW_BYTES = 2 * KS;         // LDS row pitch
  static constexpr int CPR = KS / 8;               // 16-byte chunks per LDS row
  static constexpr int RPI = 1024 / ROW_BYTES;     // rows written by one wave-wide copy instruction
  static constexpr int W_BYTES = B * ROW_BYTES;
  static constexpr int X_BYTES = TT * ROW_BYTES;
  static constexpr int STAGE = W_BYTES + X_BYTES;
  // as many stages as fit in half of a CU's LDS (two workgroups per CU), at most 4
  static constexpr int NSTAGE_FIT = (80 * 1024) / STAGE;
  static constexpr int NSTAGE = NSTAGE_FIT >= 4 ? 4 : (NSTAGE_FIT >= 2 ? NSTAGE_FIT : 2);
  static constexpr int W_INSTR = W_BYTES / 1024;
  static constexpr int X_INSTR = X_BYTES / 1024;
  static constexpr int WQ = (W_INSTR + 3) / 4;     // copy instructions per wave and step (weights)
  static constexpr int XQ = X_INSTR / 4;           // (activations)
  static constexpr int LPS = WQ + XQ;              // copies per thread and step
  static constexpr int KSTEPS = KS / 16;
  static constexpr int KEY_MOD = (CPR >= 8) ? 8 : CPR;
  static constexpr int KEY_DIV = 8 / KEY_MOD;
  static constexpr size_t LDS_BYTES = (size_t)NSTAGE * STAGE;
  static constexpr int WG_PER_CU = (2 * LDS_BYTES <= 160 * 1024) ? 2 : 1;
  __device__ static __forceinline__ int key(int row) { return (row / KEY_DIV) % KEY_MOD; }
};

struct StreamArgs {
  TileArgs t;
  int n_items;    // nbr * ntt (without a chunk plan)
  int ntt_shift;  // log2(ntt) when ntt is a power of two, else -1
  // chunk plan written by the packer (CHUNK instances only): hdr[0] = number of chunks
  const int* hdr;
  const int* chunk_row;  // block row of the chunk; bit 31 set when the row has several chunks
  const int* chunk_kb;   // first stored block of the chunk
  const int* chunk_ke;   // one past its last stored block
};

// item -> (rank in the row schedule, token tile) without an integer division in the common case
__device__ __forceinline__ void split_item(int it, int ntt, int shift, int& rank, int& tile) {
  if (shift >= 0) {
    rank = it >> shift;
    tile = it & (ntt - 1);
  } else {
    rank = it / ntt;
    tile = it - rank * ntt;
  }
}

// Static schedule: items are ordered longest-first (row_order), workgroup w takes
// one item per round; odd rounds mirror the order of the groups of 8 so that long
// and short items pair up, while w % 8 (the XCD a workgroup lands on) keeps
// seeing the same token tiles.
__device__ __forceinline__ int item_of(int w, int round, int G) {
  const int ng = G >> 3, grp = w >> 3;
  const int g2 = (round & 1) ? (ng - 1 - grp) : grp;
  return round * G + (g2 << 3) + (w & 7);
}

// Position of the loader in the flattened stream of steps.
template <int NSLICE, bool DUAL, bool CHUNK>
struct StepCursor {
  int round, r, tile, phase, k, kend, slice;
  bool valid;

  __device__ __forceinline__ void enter_phase(const TileArgs& a) {
    const MatDev& m = (DUAL && phase == 1) ? a.m1 : a.m0;
    k = ld_idx(m.row_ptr, r);
    kend = ld_idx(m.row_ptr, r + 1);
  }
  // Move to the first step at or after the current position (skips empty phases and items).
  __device__ __forceinline__ void settle(const StreamArgs& sa, int n_items, int w, int G) {
    const TileArgs& a = sa.t;
    while (valid && k >= kend) {
      if (DUAL && phase == 0) {
        phase = 1;
        enter_phase(a);
      } else {
        ++round;
        const int it = item_of(w, round, G);
        if (it >= n_items) {
          valid = false;
          break;
        }
        int rank;
        split_item(it, a.ntt, sa.ntt_shift, rank, tile);
        phase = 0;
        if (CHUNK) {
          r = ld_idx(sa.chunk_row, rank) & 0x7FFFFFFF;
          k = ld_idx(sa.chunk_kb, rank);
          kend = ld_idx(sa.chunk_ke, rank);
        } else {
          r = a.row_order ? ld_idx(a.row_order, rank) : rank;
          enter_phase(a);
        }
      }
    }
  }
  __device__ __forceinline__ void advance(const StreamArgs& sa, int n_items, int w, int G) {
    if (++slice == NSLICE) {
      slice = 0;
      ++k;
      settle(sa, n_items, w, G);
    }
  }
};

// CHUNK: the items are (chunk of a block row, token tile) pairs from the packer's chunk plan instead of
// (block row, token tile); a row made of several chunks adds its partial sums into a zeroed fp32 output.
template <int B, bool DUAL, int TW, bool CHUNK>
__global__ __launch_bounds__(256, (StreamCfg<B, TW>::WG_PER_CU)) void k_spmm_stream(const StreamArgs sa) {
  static_assert(!(DUAL && CHUNK), "the activation needs complete sums: the gated product is never split");
  using C = StreamCfg<B, TW>;
  const TileArgs& a = sa.t;
  const int n_items = CHUNK ? ld_idx(sa.hdr, 0) * a.ntt : sa.n_items;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int w = blockIdx.x, G = gridDim.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
  const int tw = wave % C::TOKW, rw = wave / C::TOKW;

  // ---- per-lane constants --------------------------------------------------------------
  // copy side: lane -> (row inside the instruction, slot); the chunk fetched is slot ^ key(row)
  const int cp_rr = lane / C::CPR, cp_slot = lane % C::CPR;
  // fragment side: byte offset of the chunk for every k-step (same for the A and B operands)
  int frag_off[C::KSTEPS];
#pragma unroll
  for (int kk = 0; kk < C::KSTEPS; ++kk) frag_off[kk] = (((2 * kk + lh) ^ C::key(l32)) << 4);
  const int a_row0 = (tw * 64 + l32) * C::ROW_BYTES;         // + mi * 32 rows
  const int b_row0 = (rw * C::WT_ROW + l32) * C::ROW_BYTES;  // + ni * 32 rows

  // ---- loader: issues the copies of one step into an LDS stage --------------------------
  // Every copy is addressed as (uniform 64-bit base) + (per-lane 32-bit byte offset).  The
  // per-lane offsets do not depend on the block: the weight offsets never change, the
  // activation offsets change only when the loader moves to another token tile.
  uint32_t woff[C::WQ], xoff[C::XQ];
  int winstr[C::WQ];
#pragma unroll
  for (int q = 0; q < C::WQ; ++q) {
    winstr[q] = (q * 4 + wave) % C::W_INSTR;  // with fewer than 4 instructions, waves duplicate each other
    const int row = winstr[q] * C::RPI + cp_rr;
    woff[q] = (uint32_t)(row * B + ((cp_slot ^ C::key(row)) << 3)) * 2u;
  }
  int xoff_tile = -1;
  auto set_tile = [&](int tile) {
    if (tile == xoff_tile) return;
    xoff_tile = tile;
#pragma unroll
    for (int q = 0; q < C::XQ; ++q) {
      const int row = (q * 4 + wave) * C::RPI + cp_rr;
      int t = tile * C::TT + row;
      t = t < a.T ? t : a.T - 1;  // clamp: rows past T are never stored
      xoff[q] = ((uint32_t)t * (uint32_t)a.sxt + (uint32_t)((cp_slot ^ C::key(row)) << 3)) * 2u;
    }
  };
  auto issue = [&](const MatDev& m, int k, int c, int slice, int tile, int stage) {
    unsigned char* st = smem + stage * C::STAGE;
    const unsigned char* wblk =
        reinterpret_cast<const unsigned char*>(m.vals) + (int64_t)k * (B * B * 2) + slice * (C::KS * 2);
#pragma unroll
    for (int q = 0; q < C::WQ; ++q) BLAST_GLDS16(wblk + woff[q], st + winstr[q] * 1024);
    set_tile(tile);
    const unsigned char* xcol =
        reinterpret_cast<const unsigned char*>(a.X) + (int64_t)c * (B * 2) + slice * (C::KS * 2);
#pragma unroll
    for (int q = 0; q < C::XQ; ++q) BLAST_GLDS16(xcol + xoff[q], st + C::W_BYTES + (q * 4 + wave) * 1024);
  };

  StepCursor<C::NSLICE, DUAL, CHUNK> ld;
  ld.round = -1;
  ld.phase = DUAL ? 1 : 0;
  ld.k = ld.kend = 0;
  ld.r = 0;
  ld.tile = 0;
  ld.slice = 0;
  ld.valid = true;
  ld.settle(sa, n_items, w, G);
  int ld_c = 0;
  int issued = 0, done = 0;
  auto issue_next = [&]() {
    const MatDev& m = (DUAL && ld.phase == 1) ? a.m1 : a.m0;
    if (ld.slice == 0) ld_c = ld_idx(m.col_idx, ld.k);
    issue(m, ld.k, ld_c, ld.slice, ld.tile, issued % C::NSTAGE);
    ++issued;
    ld.advance(sa, n_items, w, G);
  };
#pragma unroll 1
  for (int p = 0; p < C::NSTAGE - 1; ++p)
    if (ld.valid) issue_next();

  // One step of the stream: wait for its data, let another step's copies go, multiply.
  auto do_step = [&](f32x16 (&acc)[C::MI][C::NI]) {
    // Copies retire in issue order, so "at most (later steps in flight) * LPS outstanding" means
    // this step's copies have landed (stores of an epilogue can only make the wait stricter).
    const int later = issued - done - 1;
    if (later >= 2)
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(2 * C::LPS));
    else if (later == 1)
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(C::LPS));
    else
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0));
    __builtin_amdgcn_s_barrier();  // everyone's copies have landed; nobody still reads the stage reused next
    asm volatile("" ::: "memory");
    const int stage = done % C::NSTAGE;
    if (ld.valid) issue_next();
    const unsigned char* st = smem + stage * C::STAGE;
    const unsigned char* Ws = st;
    const unsigned char* Xs = st + C::W_BYTES;
    bf16x8 af[C::KSTEPS][C::MI], bfg[C::KSTEPS][C::NI];
#pragma unroll
    for (int kk = 0; kk < C::KSTEPS; ++kk) {
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
        af[kk][mi] = *reinterpret_cast<const bf16x8*>(Xs + a_row0 + mi * 32 * C::ROW_BYTES + frag_off[kk]);
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        bfg[kk][ni] = *reinterpret_cast<const bf16x8*>(Ws + b_row0 + ni * 32 * C::ROW_BYTES + frag_off[kk]);
    }
#pragma unroll
    for (int kk = 0; kk < C::KSTEPS; ++kk)
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk][mi], bfg[kk][ni], acc[mi][ni], 0, 0, 0);
    asm volatile("" ::: "memory");
    ++done;
  };

  // ---- compute: item by item -------------------------------------------------------------
  for (int round = 0;; ++round) {
    const int it = item_of(w, round, G);
    if (it >= n_items) break;
    int rank, tile;
    split_item(it, a.ntt, sa.ntt_shift, rank, tile);
    int r, n0;
    bool shared_row = false;  // other chunks add into the same output rows
    if (CHUNK) {
      const int cr = ld_idx(sa.chunk_row, rank);
      r = cr & 0x7FFFFFFF;
      shared_row = cr < 0;
      n0 = (ld_idx(sa.chunk_ke, rank) - ld_idx(sa.chunk_kb, rank)) * C::NSLICE;
    } else {
      r = a.row_order ? ld_idx(a.row_order, rank) : rank;
      n0 = (ld_idx(a.m0.row_ptr, r + 1) - ld_idx(a.m0.row_ptr, r)) * C::NSLICE;
    }
    const int t0 = tile * C::TT;

    f32x16 acc0[C::MI][C::NI];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = 0.0f;
    for (int s = 0; s < n0; ++s) do_step(acc0);
    if (DUAL) {
      f32x16 acc1[C::MI][C::NI];
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
          for (int j = 0; j < 16; ++j) acc1[mi][ni][j] = 0.0f;
      const int n1 = (ld_idx(a.m1.row_ptr, r + 1) - ld_idx(a.m1.row_ptr, r)) * C::NSLICE;
      for (int s = 0; s < n1; ++s) do_step(acc1);
      if (a.act == BLAST_ACT_SILU) {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
            for (int j = 0; j < 16; ++j)
              acc0[mi][ni][j] = apply_act(BLAST_ACT_SILU, acc0[mi][ni][j]) * acc1[mi][ni][j];
      } else {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = apply_act(a.act, acc0[mi][ni][j]) * acc1[mi][ni][j];
      }
    }

    // Result layout: lane -> weight row l32 (+32 ni), register j -> token 8*(j/4) + 4*lh + j%4 (+32 mi).
    // A store instruction therefore writes 32 consecutive rows of one token: full 64/128-byte segments.
    const bool full = (t0 + C::TT <= a.T);
    auto put = [&](unsigned char* p, float v) {
      if (CHUNK && shared_row)
        atomicAdd(reinterpret_cast<float*>(p), v);  // fp32 output, zeroed before the launch
      else if (a.y_bf16)
        *reinterpret_cast<uint16_t*>(p) = f32_to_bf16_rne(v);
      else
        *reinterpret_cast<float*>(p) = v;
    };
    const int esz = a.y_bf16 ? 2 : 4;
    const int64_t tok_pitch = a.syt * esz;
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      const int64_t row = (int64_t)r * B + rw * C::WT_ROW + ni * 32 + l32;
      const int tokb = t0 + tw * 64 + 4 * lh;
      unsigned char* p0 = reinterpret_cast<unsigned char*>(a.Y) + (row * a.syi + (int64_t)tokb * a.syt) * esz;
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int dt = mi * 32 + 8 * (j / 4) + (j % 4);
          if (full || tokb + dt < a.T) put(p0 + dt * tok_pitch, acc0[mi][ni][j]);
        }
    }
  }
}

// Zeroes the fp32 output rows of every block row that is cut into several chunks (its chunks then add
// into them).  Grid: x = upper bound of the number of chunks, y = slabs of 64 tokens.
template <int B>
__global__ __launch_bounds__(256) void k_zero_shared_rows(const StreamArgs sa) {
  const TileArgs& a = sa.t;
  const int ci = blockIdx.x;
  if (ci >= ld_idx(sa.hdr, 0)) return;
  const int cr = ld_idx(sa.chunk_row, ci);
  if (cr >= 0) return;  // a single-chunk row is stored, not accumulated
  const int r = cr & 0x7FFFFFFF;
  if (ld_idx(sa.chunk_kb, ci) != ld_idx(a.m0.row_ptr, r)) return;  // only the first chunk of the row zeroes
  float* Y = reinterpret_cast<float*>(a.Y);
  const int t0 = blockIdx.y * 64;
  for (int e = threadIdx.x; e < 64 * B; e += 256) {
    const int t = t0 + e / B, i = e % B;
    if (t < a.T) Y[(int64_t)t * a.syt + ((int64_t)r * B + i) * a.syi] = 0.0f;
  }
}

}  // namespace blast_dev
