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
// NW = waves of a workgroup (4, or 8 for 128-wide blocks: a 256-token x 128-row output tile, one workgroup
// per CU, so that a weight slice is copied once per 256 tokens and 85 flop are done per byte copied
// instead of 64).
template <int B, int TW, int NW = 4>
struct StreamCfg {
  static_assert(TW == 2 || TW == 4, "two or four waves along tokens");
  static_assert(NW == 4 || NW == 8, "four or eight waves");
  static_assert(B / (NW / TW) >= 32, "a wave needs at least 32 weight rows");
  static constexpr int NWAVE = NW;
  static constexpr int TOKW = TW;                  // waves along tokens
  static constexpr int ROWW = NW / TOKW;           // waves along weight rows
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
  // as many stages as fit in a workgroup's share of a CU's LDS (two four-wave workgroups per CU, or one
  // eight-wave workgroup), at most 4
  static constexpr int NSTAGE_FIT = ((NW == 8 ? 160 : 80) * 1024) / STAGE;
  static constexpr int NSTAGE = NSTAGE_FIT >= 4 ? 4 : (NSTAGE_FIT >= 2 ? NSTAGE_FIT : 2);
  static constexpr int W_INSTR = W_BYTES / 1024;
  static constexpr int X_INSTR = X_BYTES / 1024;
  static constexpr int WQ = (W_INSTR + NW - 1) / NW;  // copy instructions per wave and step (weights)
  static constexpr int XQ = X_INSTR / NW;             // (activations)
  static_assert(X_INSTR % NW == 0, "the activation copies divide evenly among the waves");
  static constexpr int LPS = WQ + XQ;              // copies per thread and step
  static constexpr int KSTEPS = KS / 16;
  static constexpr int KEY_MOD = (CPR >= 8) ? 8 : CPR;
  static constexpr int KEY_DIV = 8 / KEY_MOD;
  static constexpr size_t LDS_BYTES = (size_t)NSTAGE * STAGE;
  static constexpr int WG_PER_CU = (NW == 4 && 2 * LDS_BYTES <= 160 * 1024) ? 2 : 1;
  static constexpr int WAVES_PER_SIMD = WG_PER_CU * NW / 4;
  __device__ static __forceinline__ int key(int row) { return (row / KEY_DIV) % KEY_MOD; }
};

struct StreamArgs {
  TileArgs t;
  int n_items;    // nbr * ntt (without a chunk plan)
  int ntt_shift;  // log2(ntt) when ntt is a power of two, else -1
  // Which items meet on an XCD (workgroup w runs on XCD w % 8, whose L2 its copies go through):
  // 0: a token tile stays on one XCD (its slab of activations is re-read from that L2, every XCD streams
  //    every weight block);
  // 1: a block row stays on one XCD, all its token tiles running side by side (every weight block leaves the
  //    memory side once; for activations too wide for an L2 to keep a slab of them anyway).  Needs
  //    (gridDim.x / 8) % ntt == 0.
  int row_pinned;
  // chunk plan written by the packer (CHUNK instances only): hdr[0] = number of chunks
  const int* hdr;
  const int* chunk_row;  // block row of the chunk; bit 31 set when the row has several chunks
  const int* chunk_kb;   // first stored block of the chunk
  const int* chunk_ke;   // one past its last stored block
  // Side job (z_hdr != null): before its own work this launch clears the fp32 rows that a LATER chunked
  // product accumulates into (the block rows cut into several chunks of that product's plan), so that
  // product needs no clearing launch of its own.  Units of (chunk slot, 64 tokens), dealt to all workgroups.
  const int* z_hdr;
  const int* z_chunk_row;
  const int* z_chunk_kb;
  const int* z_row_ptr;
  float* z_Y;
  int64_t z_syt, z_syi;
  int z_T;
  // Long rows of a gated product (LONG instances).  A block row that the first chunk plan of a matrix cuts
  // into several chunks has a slot in that matrix (the packer's row_slot, else -1); a row with a slot in
  // either matrix is "deferred": the launch leaves fp32 sums of its two sides (gate, up) in scratch and a
  // small launch after it adds them up, applies the activation and writes H.  The items of the launch are
  //   - the chunks of the first matrix' cut rows (the head of its plan: hdr points at their number),
  //   - those of the second matrix (hdr1, chunk_*1),
  //   - the block rows in schedule order: an ordinary row as ever; of a deferred row only the side that is
  //     not cut.
  // Every chunk stores its sums in a slice of its own (no atomics, nothing to clear): P0 / P1, indexed by
  // the chunk's place in the plan of the first / second matrix.  A side that is whole goes to W0 (the up
  // side of a row cut in the first matrix only, indexed by the row's slot there) or W1 (the gate side of a
  // row cut in the second matrix only, indexed by its slot there).  All four are fp32 [index][T][B]: the
  // tile an item stores is one contiguous piece.
  const int* slot0;
  const int* slot1;
  const int* chunk0_0;  // first chunk of a cut row in the first matrix' plan (the packer's row_chunk0)
  const int* chunk0_1;
  float* P0;
  float* P1;
  float* W0;
  float* W1;
  const int* hdr1;
  const int* chunk_row1;
  const int* chunk_kb1;
  const int* chunk_ke1;
};

constexpr int kLongChunk = 16;  // blocks per chunk of the plan that the LONG launch works from

// number of chunks of a matrix' cut rows (hdr points at that count, or is null)
__device__ __forceinline__ int long_chunks(const int* hdr) { return hdr ? ld_idx(hdr, 0) : 0; }

// What a LONG item that is not an ordinary row does with its sums (ItemTable::c1; bit 31 of r marks such items
// and the rest of r is the index in the destination).
constexpr int kLongSecond = 1;  // the blocks are the second matrix'
constexpr int kLongP = 2;       // destination P0 / P1 (a chunk), else W0 / W1 (a whole side); which: kLongSecond
constexpr int kLongNone = 4;    // nothing to do: both sides of the row are cut

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

// Descriptors of the items of one workgroup, one round per lane (every wave keeps its own copy, read
// with v_readlane).  They are fetched once at kernel start with ordinary vector loads, so that no
// dependent chain of index loads (schedule -> row pointers -> first column) is left on the path of the
// loader when it crosses an item or phase boundary.  The host sizes the grid so that a workgroup has at
// most 64 rounds.
struct ItemTable {
  int r;        // block row (bit 31: CHUNK row shared with other chunks)
  int tile;     // token tile
  int k0, e0;   // stored blocks [k0, e0) of the first matrix (or of the chunk)
  int k1, e1;   // of the second matrix (DUAL)
  int c0, c1;   // block column of the first stored block of each phase
  int n_rounds; // uniform: rounds of this workgroup
};

#define BLAST_LANE(v, j) __builtin_amdgcn_readlane((v), (j))

// Fills the descriptor of one item from its rank in the schedule (row_order, or the chunk plan) and its token tile.
template <bool DUAL, bool CHUNK, bool LONG>
__device__ __forceinline__ void describe_item(const StreamArgs& sa, int rank, int tile, ItemTable& t) {
  const TileArgs& a = sa.t;
  t.tile = tile;
  if constexpr (LONG) {
    const int n0 = long_chunks(sa.hdr), n1 = long_chunks(sa.hdr1);
    int index = 0, code = 0;
    bool special = true;
    t.k1 = t.e1 = 0;
    if (rank < n0) {  // a chunk of the first matrix
      index = rank;
      code = kLongP;
      t.k0 = sa.chunk_kb[rank];
      t.e0 = sa.chunk_ke[rank];
    } else if (rank < n0 + n1) {  // of the second
      index = rank - n0;
      code = kLongP | kLongSecond;
      t.k0 = sa.chunk_kb1[index];
      t.e0 = sa.chunk_ke1[index];
    } else {
      const int rr = rank - n0 - n1;
      const int r = a.row_order ? a.row_order[rr] : rr;
      const int s0 = sa.slot0 ? sa.slot0[r] : -1, s1 = sa.slot1 ? sa.slot1[r] : -1;
      if (s0 < 0 && s1 < 0) {  // an ordinary row
        special = false;
        t.r = r;
        t.k0 = a.m0.row_ptr[r];
        t.e0 = a.m0.row_ptr[r + 1];
        t.k1 = a.m1.row_ptr[r];
        t.e1 = a.m1.row_ptr[r + 1];
      } else if (s0 >= 0 && s1 >= 0) {
        code = kLongNone;
        t.k0 = t.e0 = 0;
      } else if (s0 >= 0) {  // the up side is whole: W0[s0]
        index = s0;
        code = kLongSecond;
        t.k0 = a.m1.row_ptr[r];
        t.e0 = a.m1.row_ptr[r + 1];
      } else {  // the gate side is whole: W1[s1]
        index = s1;
        code = 0;
        t.k0 = a.m0.row_ptr[r];
        t.e0 = a.m0.row_ptr[r + 1];
      }
    }
    if (special) {
      t.r = index | (int)0x80000000u;
      t.c1 = code;
      if (t.k0 < t.e0) t.c0 = ((code & kLongSecond) ? a.m1 : a.m0).col_idx[t.k0];
      return;
    }
  } else if (CHUNK) {
    t.r = sa.chunk_row[rank];
    t.k0 = sa.chunk_kb[rank];
    t.e0 = sa.chunk_ke[rank];
  } else {
    t.r = a.row_order ? a.row_order[rank] : rank;
    t.k0 = a.m0.row_ptr[t.r];
    t.e0 = a.m0.row_ptr[t.r + 1];
    if (DUAL) {
      t.k1 = a.m1.row_ptr[t.r];
      t.e1 = a.m1.row_ptr[t.r + 1];
    }
  }
  if (t.k0 < t.e0) t.c0 = a.m0.col_idx[t.k0];
  if (DUAL && t.k1 < t.e1) t.c1 = a.m1.col_idx[t.k1];
}

// Stored blocks that item `rank` of a LONG launch multiplies (see StreamArgs for the numbering).
__device__ __forceinline__ int long_item_blocks(const StreamArgs& sa, int rank) {
  const TileArgs& a = sa.t;
  const int n0 = long_chunks(sa.hdr), n1 = long_chunks(sa.hdr1);
  if (rank < n0) return sa.chunk_ke[rank] - sa.chunk_kb[rank];
  if (rank < n0 + n1) return sa.chunk_ke1[rank - n0] - sa.chunk_kb1[rank - n0];
  const int rr = rank - n0 - n1;
  const int r = a.row_order ? a.row_order[rr] : rr;
  int len = 0;
  if (!(sa.slot0 && sa.slot0[r] >= 0)) len += a.m0.row_ptr[r + 1] - a.m0.row_ptr[r];
  if (!(sa.slot1 && sa.slot1[r] >= 0)) len += a.m1.row_ptr[r + 1] - a.m1.row_ptr[r];
  return len;
}

template <bool DUAL, bool CHUNK, bool LONG>
__device__ __forceinline__ ItemTable load_item_table(const StreamArgs& sa, int n_items, int w, int G, int lane) {
  const TileArgs& a = sa.t;
  ItemTable t{};
  if (!sa.row_pinned) {
    const int it = item_of(w, lane, G);
    const bool ok = it < n_items;
    int rank = 0, tile = 0;
    if (ok) split_item(it, a.ntt, sa.ntt_shift, rank, tile);
    if (ok) describe_item<DUAL, CHUNK, LONG>(sa, rank, tile, t);
    // items of a workgroup grow with the round, so the valid rounds are a prefix
    t.n_rounds = __builtin_popcountll(__ballot(ok));
    return t;
  }
  // Row-pinned schedule.  The ranks (rows by population, fullest first) are dealt to the 8 XCDs in
  // octets, every other octet mirrored; on an XCD, `nslot` groups of ntt workgroups (one per token tile)
  // each take whole rows.  Which group takes which row is decided by every workgroup for itself, all
  // arriving at the same answer: rows in order, each to the group with the least work so far (work = stored
  // blocks + 2 for the output tile); with more rows per XCD than are dealt that way, or more than 8 groups,
  // rows are dealt round-robin, every other round mirrored.
  const int n_rows = n_items / a.ntt;
  const int x = w & 7, j = w >> 3, Gx = G >> 3;
  const int nslot = Gx / a.ntt, slot = j / a.ntt, tile = j - slot * a.ntt;
  const int octets = (n_rows + 7) >> 3;
  auto rank_of = [&](int o) { return (o << 3) + ((o & 1) ? 7 - x : x); };
  // rows of this XCD: octet o contributes rank_of(o) when that rank exists
  int nrx = octets;
  if (octets > 0 && rank_of(octets - 1) >= n_rows) --nrx;
  int mine = -1;  // per lane: the position (in the XCD's list) of the lane-th row of this group
  int n_mine = 0;
  // (LONG: up to 128 rows per XCD, the lengths two per lane, and no group is given more than the 64 rows a
  // descriptor table holds)
  constexpr int kDealt = LONG ? 128 : 64;
  if (nrx <= kDealt && nslot <= 8 && (nrx <= 64 || nslot >= 2)) {
    auto length_at = [&](int pos) {
      const int rank = rank_of(pos);
      int len;
      if (LONG) {
        len = long_item_blocks(sa, rank);
      } else if (CHUNK) {
        len = sa.chunk_ke[rank] - sa.chunk_kb[rank];
      } else {
        const int r = a.row_order ? a.row_order[rank] : rank;
        len = a.m0.row_ptr[r + 1] - a.m0.row_ptr[r];
        if (DUAL) len += a.m1.row_ptr[r + 1] - a.m1.row_ptr[r];
      }
      return len + 2;
    };
    int len = 0, len_hi = 0;
    if (lane < nrx) len = length_at(lane);
    if (LONG && lane + 64 < nrx) len_hi = length_at(lane + 64);
    int load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int cnt[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int k = 0; k < nrx; ++k) {
      const int l = (LONG && k >= 64) ? BLAST_LANE(len_hi, k - 64) : BLAST_LANE(len, k);
      int best = 0, bl = load[0];
      if (LONG && cnt[0] >= 64) bl = 0x7FFFFFFF;
#pragma unroll
      for (int q = 1; q < 8; ++q)
        if (q < nslot && load[q] < bl && !(LONG && cnt[q] >= 64)) {
          bl = load[q];
          best = q;
        }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        load[q] += (q == best) ? l : 0;
        if (LONG) cnt[q] += (q == best) ? 1 : 0;
      }
      if (best == slot) {
        if (lane == n_mine) mine = k;
        ++n_mine;
      }
    }
  } else {
    // round-robin: round q of group `slot` takes position q * nslot + (q odd ? nslot - 1 - slot : slot)
    const int pos = lane * nslot + ((lane & 1) ? nslot - 1 - slot : slot);
    if (pos < nrx) mine = pos;
    n_mine = __builtin_popcountll(__ballot(pos < nrx));
    // positions grow with the round except across a mirrored boundary, where validity can only end:
    // the valid rounds are a prefix
  }
  if (mine >= 0) describe_item<DUAL, CHUNK, LONG>(sa, rank_of(mine), tile, t);
  t.n_rounds = n_mine;
  return t;
}

// Position of the loader in the flattened stream of steps, kept as running addresses so that the
// common case (the next block of the same row) costs a handful of scalar additions: a "run" is the
// list of stored blocks of one (item, matrix) pair.
struct Loader {
  const unsigned char* wptr;  // first byte of the current block's values
  const int* cptr;            // its entry in the column index array
  int rem;                    // blocks left in the run, the current one included
  int c, c_next;              // block column of the current block / of the one after it
  int slice;                  // contraction slice of the current block
  int tile;                   // token tile of the run
  int round, phase;           // which run this is
  uint32_t stage_off;         // LDS byte offset of the stage the next step is copied into
  bool valid;
};

// The side job of StreamArgs: every lane looks at one unit (chunk slot, slab of 64 tokens) of the later
// product's plan, units being dealt to the workgroups round-robin; the units that are the first chunk of a
// row made of several chunks are then cleared by the whole workgroup, one after the other.
template <int B, int NTHREADS>
__device__ __forceinline__ void stream_zero_side(const StreamArgs& sa, int w, int G, int lane) {
  const int n_chunks = ld_idx(sa.z_hdr, 0);
  const int slabs = (sa.z_T + 63) >> 6;
  const int64_t total = (int64_t)n_chunks * slabs;
  for (int64_t base = 0; base < total; base += (int64_t)G * 64) {
    const int64_t u = base + (int64_t)lane * G + w;
    int r = -1, slab = 0;
    if (u < total) {
      const int ci = (int)(u / slabs);
      slab = (int)(u - (int64_t)ci * slabs);
      const int cr = sa.z_chunk_row[ci];
      if (cr < 0) {  // a row made of several chunks ...
        const int row = cr & 0x7FFFFFFF;
        if (sa.z_chunk_kb[ci] == sa.z_row_ptr[row]) r = row;  // ... and this is its first chunk
      }
    }
    unsigned long long todo = __ballot(r >= 0);
    while (todo) {
      const int l = __builtin_ctzll(todo);
      todo &= todo - 1;
      const int rr = BLAST_LANE(r, l), t0 = BLAST_LANE(slab, l) * 64;
      for (int e = threadIdx.x; e < 64 * B; e += NTHREADS) {
        const int t = t0 + e / B, i = e % B;
        if (t < sa.z_T) sa.z_Y[(int64_t)t * sa.z_syt + ((int64_t)rr * B + i) * sa.z_syi] = 0.0f;
      }
    }
  }
}

// CHUNK: the items are (chunk of a block row, token tile) pairs from the packer's chunk plan instead of
// (block row, token tile); a row made of several chunks adds its partial sums into a zeroed fp32 output.
// POST: a single-matrix product whose result goes through the activation a.act before it is stored
// (the first half of a two-matrix MLP).
// LONG: the gated product with its long rows cut into chunks and finished by a later launch, see StreamArgs.
template <int B, bool DUAL, int TW, bool CHUNK, bool POST = false, int NW = 4, bool LONG = false>
__global__ __launch_bounds__(64 * NW, (StreamCfg<B, TW, NW>::WAVES_PER_SIMD)) void k_spmm_stream(const StreamArgs sa) {
  static_assert(!(DUAL && CHUNK), "the activation needs complete sums: the gated product is never split");
  static_assert(!POST || (!DUAL && !CHUNK), "an activation on the output needs complete sums of a single matrix");
  static_assert(!LONG || (DUAL && !CHUNK), "long rows are a matter of the gated product");
  using C = StreamCfg<B, TW, NW>;
  const TileArgs& a = sa.t;
  const int n_items = LONG    ? (long_chunks(sa.hdr) + long_chunks(sa.hdr1) + a.nbr) * a.ntt
                      : CHUNK ? ld_idx(sa.hdr, 0) * a.ntt
                              : sa.n_items;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int w = blockIdx.x, G = gridDim.x;
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
  // the wave index is uniform: keeping it in a scalar register makes every LDS destination of the copy
  // instructions scalar arithmetic instead of vector arithmetic plus a lane read
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    winstr[q] = (q * NW + wave) % C::W_INSTR;  // with fewer instructions than waves, waves duplicate each other
    const int row = winstr[q] * C::RPI + cp_rr;
    woff[q] = (uint32_t)(row * B + ((cp_slot ^ C::key(row)) << 3)) * 2u;
  }
  int xoff_tile = -1;
  const uint32_t sxt32 = (uint32_t)a.sxt;
  auto set_tile = [&](int tile) {
    if (tile == xoff_tile) return;
    xoff_tile = tile;
#pragma unroll
    for (int q = 0; q < C::XQ; ++q) {
      const int row = (q * NW + wave) * C::RPI + cp_rr;
      int t = tile * C::TT + row;
      t = t < a.T ? t : a.T - 1;  // clamp: rows past T are never stored
      xoff[q] = ((uint32_t)t * sxt32 + (uint32_t)((cp_slot ^ C::key(row)) << 3)) * 2u;
    }
  };
  if (sa.z_hdr) stream_zero_side<B, 64 * NW>(sa, w, G, lane);
  const ItemTable tab = load_item_table<DUAL, CHUNK, LONG>(sa, n_items, w, G, lane);

  Loader ld;
  ld.round = -1;
  ld.phase = DUAL ? 1 : 0;
  ld.rem = 0;
  ld.slice = 0;
  ld.tile = 0;
  ld.c = ld.c_next = 0;
  ld.stage_off = 0;
  ld.wptr = nullptr;
  ld.cptr = nullptr;
  ld.valid = true;
  // Moves the loader to the first block of the next non-empty run (rare: once per row and matrix).
  auto next_run = [&]() {
    for (;;) {
      int k, e;
      const MatDev* m;
      if (DUAL && ld.phase == 0) {
        ld.phase = 1;
        k = BLAST_LANE(tab.k1, ld.round);
        e = BLAST_LANE(tab.e1, ld.round);
        ld.c = BLAST_LANE(tab.c1, ld.round);
        m = &a.m1;
      } else {
        ++ld.round;
        if (ld.round >= tab.n_rounds) {
          ld.valid = false;
          return;
        }
        ld.phase = 0;
        ld.tile = BLAST_LANE(tab.tile, ld.round);
        k = BLAST_LANE(tab.k0, ld.round);
        e = BLAST_LANE(tab.e0, ld.round);
        ld.c = BLAST_LANE(tab.c0, ld.round);
        m = &a.m0;
        if constexpr (LONG) {
          if (BLAST_LANE(tab.r, ld.round) < 0 && (BLAST_LANE(tab.c1, ld.round) & kLongSecond)) m = &a.m1;
        }
      }
      if (k < e) {
        ld.rem = e - k;
        ld.wptr = reinterpret_cast<const unsigned char*>(m->vals) + (int64_t)k * (B * B * 2);
        ld.cptr = m->col_idx + k;
        ld.c_next = ld_idx(ld.cptr, ld.rem > 1 ? 1 : 0);
        set_tile(ld.tile);
        return;
      }
    }
  };
  // Issues the copies of the loader's current step and moves it one step on.
  int ahead = 0;  // steps issued whose stage the multiplying side has not entered yet
  auto issue_next = [&]() {
    unsigned char* st = smem + ld.stage_off;
    const unsigned char* wblk = ld.wptr + ld.slice * (C::KS * 2);
#pragma unroll
    for (int q = 0; q < C::WQ; ++q) BLAST_GLDS16(wblk + woff[q], st + winstr[q] * 1024);
    const unsigned char* xcol =
        reinterpret_cast<const unsigned char*>(a.X) + (int64_t)ld.c * (B * 2) + ld.slice * (C::KS * 2);
#pragma unroll
    for (int q = 0; q < C::XQ; ++q) BLAST_GLDS16(xcol + xoff[q], st + C::W_BYTES + (q * NW + wave) * 1024);
    ld.stage_off = (ld.stage_off + C::STAGE == (uint32_t)C::LDS_BYTES) ? 0u : ld.stage_off + C::STAGE;
    ++ahead;
    if (C::NSLICE > 1) {
      if (++ld.slice < C::NSLICE) return;
      ld.slice = 0;
    }
    if (--ld.rem > 0) {
      ld.wptr += B * B * 2;
      ++ld.cptr;
      ld.c = ld.c_next;
      ld.c_next = ld_idx(ld.cptr, ld.rem > 1 ? 1 : 0);  // the last block of a run re-reads its own entry
    } else {
      next_run();
    }
  };
  next_run();
  // Two ways of running the ring.  With three or more stages (PIPE) every stage starts with a step in it and
  // the stream is software-pipelined at the grain of a k-step, see do_step.  With two stages the step that
  // refills a stage is issued before the wait for the current step's copies, two barriers per step: during
  // that wait two steps are then in flight instead of one, which matters more than the second barrier
  // (measured on the 1B- and 3B-shaped products, b = 64: 3 % faster than the pipelined form with two stages).
  constexpr bool PIPE = C::NSTAGE >= 3;
#pragma unroll 1
  for (int p = 0; p < (PIPE ? C::NSTAGE : C::NSTAGE - 1); ++p)
    if (ld.valid) issue_next();

  // Steps this workgroup will multiply (the consumer's view of the stream's length).
  int steps_left = 0;
  if (PIPE) {
    for (int q = 0; q < tab.n_rounds; ++q) {
      steps_left += (BLAST_LANE(tab.e0, q) - BLAST_LANE(tab.k0, q)) * C::NSLICE;
      if (DUAL) steps_left += (BLAST_LANE(tab.e1, q) - BLAST_LANE(tab.k1, q)) * C::NSLICE;
    }
  }

  // Operand fragments of one 16-wide k-step: MI token fragments, NI weight-row fragments.
  struct Frag {
    bf16x8 x[C::MI], w[C::NI];
  };
  auto read_frag = [&](Frag& f, const unsigned char* st, int kk) {
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
      f.x[mi] = *reinterpret_cast<const bf16x8*>(st + C::W_BYTES + a_row0 + mi * 32 * C::ROW_BYTES + frag_off[kk]);
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
      f.w[ni] = *reinterpret_cast<const bf16x8*>(st + b_row0 + ni * 32 * C::ROW_BYTES + frag_off[kk]);
  };
  auto mma = [&](f32x16 (&acc)[C::MI][C::NI], const Frag& f) {
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.x[mi], f.w[ni], acc[mi][ni], 0, 0, 0);
  };
  // A fragment read follows every matrix instruction: the wait for the fragments of this k-step then sits
  // in front of its first matrix instruction, where only reads issued a whole k-step ago are outstanding.
  auto pair_reads_with_mma = [&]() {
#pragma unroll
    for (int i = 0; i < C::MI * C::NI; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < C::MI + C::NI) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
  };

  uint32_t cstage_off = 0;
  Frag cur;
  if (PIPE && steps_left > 0) {
    if (ahead == C::NSTAGE)
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT((C::NSTAGE - 1) * C::LPS));
    else
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0));
    __builtin_amdgcn_s_barrier();  // everyone's copies of the first step have landed
    asm volatile("" ::: "memory");
    read_frag(cur, smem, 0);
    --ahead;  // from here on: steps issued beyond the one being multiplied
  }
  // PIPE: while the matrix instructions of one k-step run, the fragments of the next are on their way from
  // LDS, and `cur` always holds the fragments of the k-step that is multiplied next - at a step boundary
  // those of the first k-step of the following stage, across items too.  One barrier per step, placed before
  // the step's last k-step: by then every wave has issued the matrix work of the earlier k-steps, which keeps
  // the matrix cores fed while the waves meet.
  auto do_step_pipe = [&](f32x16 (&acc)[C::MI][C::NI]) {
    const unsigned char* st = smem + cstage_off;
    cstage_off = (cstage_off + C::STAGE == (uint32_t)C::LDS_BYTES) ? 0u : cstage_off + C::STAGE;
    Frag nxt;
#pragma unroll
    for (int kk = 0; kk + 1 < C::KSTEPS; ++kk) {
      read_frag(nxt, st, kk + 1);
      mma(acc, cur);
      pair_reads_with_mma();
      cur = nxt;
    }
    // Every read of this stage has been issued; once they have returned the stage can be handed back.
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    asm volatile("" ::: "memory");
    --steps_left;
    if (steps_left > 0) {
      // Copies retire in issue order, so "at most (steps issued after the next one) * LPS outstanding"
      // means the next step's copies have landed (stores of an epilogue can only make the wait stricter).
      // In the steady state NSTAGE-1 steps are issued beyond this one; the tail waits for all.
      if (ahead == C::NSTAGE - 1)
        __builtin_amdgcn_s_waitcnt(BLAST_VMCNT((C::NSTAGE - 2) * C::LPS));
      else
        __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0));
      // everyone's copies of the next step have landed, and everyone has left this step's stage
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      read_frag(nxt, smem + cstage_off, 0);
      --ahead;
    }
    mma(acc, cur);
    pair_reads_with_mma();
    cur = nxt;
    asm volatile("" ::: "memory");
    // the stage this step was multiplied out of takes the step NSTAGE further down the stream
    if (steps_left > 0 && ld.valid) issue_next();
  };
  // Two stages: wait for the step's data, let another step's copies go, multiply.
  auto do_step_two = [&](f32x16 (&acc)[C::MI][C::NI]) {
    // The stage that the previous step was multiplied out of is refilled first (once every wave has
    // left it), so that the copies of NSTAGE steps are in flight while this step's are awaited.
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (ld.valid) issue_next();
    // Copies retire in issue order, so "at most (later steps in flight) * LPS outstanding" means
    // this step's copies have landed (stores of an epilogue can only make the wait stricter).  In
    // the steady state NSTAGE-1 later steps are in flight at this point; the tail waits for all.
    if (ahead == C::NSTAGE)
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT((C::NSTAGE - 1) * C::LPS));
    else
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0));
    __builtin_amdgcn_s_barrier();  // everyone's copies of this step have landed
    asm volatile("" ::: "memory");
    const unsigned char* st = smem + cstage_off;
    cstage_off = (cstage_off + C::STAGE == (uint32_t)C::LDS_BYTES) ? 0u : cstage_off + C::STAGE;
    Frag f[C::KSTEPS];
#pragma unroll
    for (int kk = 0; kk < C::KSTEPS; ++kk) read_frag(f[kk], st, kk);
#pragma unroll
    for (int kk = 0; kk < C::KSTEPS; ++kk) mma(acc, f[kk]);
    // Shape of the schedule inside this block: the fragment reads of the first two k-steps go out
    // together, then every matrix instruction is paired with one read of the later k-steps, so that
    // LDS latency hides behind matrix work instead of being waited for read by read.
    constexpr int kReads = C::KSTEPS * (C::MI + C::NI), kMfma = C::KSTEPS * C::MI * C::NI;
    constexpr int kLead = kReads / 2;
    __builtin_amdgcn_sched_group_barrier(0x100, kLead, 0);
#pragma unroll
    for (int i = 0; i < kReads - kLead; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, kMfma - (kReads - kLead), 0);
    asm volatile("" ::: "memory");
    --ahead;
  };
  auto do_step = [&](f32x16 (&acc)[C::MI][C::NI]) {
    if constexpr (PIPE)
      do_step_pipe(acc);
    else
      do_step_two(acc);
  };

  // ---- compute: item by item -------------------------------------------------------------
  for (int round = 0; round < tab.n_rounds; ++round) {
    const int tile = BLAST_LANE(tab.tile, round);
    const int rr = BLAST_LANE(tab.r, round);
    const int r = CHUNK ? (rr & 0x7FFFFFFF) : rr;
    const bool shared_row = CHUNK && rr < 0;  // other chunks add into the same output rows
    const int n0 = (BLAST_LANE(tab.e0, round) - BLAST_LANE(tab.k0, round)) * C::NSLICE;
    const int t0 = tile * C::TT;

    f32x16 acc0[C::MI][C::NI];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = 0.0f;
    for (int s = 0; s < n0; ++s) do_step(acc0);
    if constexpr (LONG) {
      if (rr < 0) {  // a chunk, or the whole side of a deferred row: the sums go to scratch as they are
        const int code = BLAST_LANE(tab.c1, round);
        if (code & kLongNone) continue;
        // whole up side -> W0, whole gate side -> W1 (each indexed by the slot in the matrix that is cut)
        const bool second = (code & kLongSecond) != 0;
        float* S = (code & kLongP) ? (second ? sa.P1 : sa.P0) : (second ? sa.W0 : sa.W1);
        S += (int64_t)(rr & 0x7FFFFFFF) * a.T * B;
        const int tokb = t0 + tw * 64 + 4 * lh;
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni) {
          float* p0 = S + (int64_t)tokb * B + rw * C::WT_ROW + ni * 32 + l32;
#pragma unroll
          for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              const int dt = mi * 32 + 8 * (j / 4) + (j % 4);
              if (tokb + dt < a.T) p0[dt * B] = acc0[mi][ni][j];
            }
        }
        continue;
      }
    }
    if (DUAL) {
      f32x16 acc1[C::MI][C::NI];
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
          for (int j = 0; j < 16; ++j) acc1[mi][ni][j] = 0.0f;
      const int n1 = (BLAST_LANE(tab.e1, round) - BLAST_LANE(tab.k1, round)) * C::NSLICE;
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
    if (POST) {
      // the branch on the activation stays outside the unrolled loops: one copy of each function body
      if (a.act == BLAST_ACT_GELU) {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = apply_act(BLAST_ACT_GELU, acc0[mi][ni][j]);
      } else if (a.act == BLAST_ACT_SILU) {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = apply_act(BLAST_ACT_SILU, acc0[mi][ni][j]);
      } else {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = apply_act(BLAST_ACT_RELU, acc0[mi][ni][j]);
      }
    }

    // Result layout: lane -> weight row l32 (+32 ni), register j -> token 8*(j/4) + 4*lh + j%4 (+32 mi).
    // A store instruction therefore writes 32 consecutive rows of one token: full 64/128-byte segments.
    const bool full = (t0 + C::TT <= a.T);
    // Fast path (whole token tile, rows contiguous in memory, no atomics, offsets inside the tile fit 32
    // bits): one uniform 64-bit base per item and a 32-bit lane offset per store, so that a stored value
    // costs a conversion, an add and the store instead of 64-bit address arithmetic and predication.
    if (full && a.y_fast && !(CHUNK && shared_row)) {
      const uint32_t esz = a.y_bf16 ? 2u : 4u;
      uint32_t pitch = (uint32_t)a.syt * esz;
      // opaque to the optimiser: otherwise the 32 multiples of the pitch are computed once before the
      // loop over items and kept (spilled) for the whole kernel
      asm volatile("" : "+s"(pitch));
      unsigned char* base = reinterpret_cast<unsigned char*>(a.Y) + (int64_t)t0 * a.syt * esz;
      if (a.y_bf16) {
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni) {
          const uint32_t off0 = (uint32_t)(r * B + rw * C::WT_ROW + ni * 32 + l32) * 2u + (uint32_t)(tw * 64 + 4 * lh) * pitch;
#pragma unroll
          for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              const uint32_t dt = mi * 32 + 8 * (j / 4) + (j % 4);
              // the token step goes into the uniform base, the lane offset stays one register
              unsigned char* bj = base + __builtin_amdgcn_readfirstlane(dt * pitch);
              *reinterpret_cast<uint16_t*>(bj + off0) = f32_to_bf16_rne(acc0[mi][ni][j]);
            }
        }
      } else {
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni) {
          const uint32_t off0 = (uint32_t)(r * B + rw * C::WT_ROW + ni * 32 + l32) * 4u + (uint32_t)(tw * 64 + 4 * lh) * pitch;
#pragma unroll
          for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              const uint32_t dt = mi * 32 + 8 * (j / 4) + (j % 4);
              unsigned char* bj = base + __builtin_amdgcn_readfirstlane(dt * pitch);
              *reinterpret_cast<float*>(bj + off0) = acc0[mi][ni][j];
            }
        }
      }
      continue;
    }
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

// After a LONG launch: H = act(gate sums) * (up sums) for the deferred rows, each side either whole or the
// sum of the row's chunks, added in the order of the plan.
// Grid: x = groups of kLongFinishRows block rows, y = slabs of kLongFinishTokens tokens.  (A workgroup lives
// for at least the latency of the loads that tell it whether a row is deferred: one workgroup looks at several
// rows, so that the many rows that are not cost little.)
constexpr int kLongFinishTokens = 8, kLongFinishRows = 8;
template <int B>
__global__ __launch_bounds__(256) void k_long_finish(const StreamArgs sa) {
  const TileArgs& a = sa.t;
  int s0v[kLongFinishRows], s1v[kLongFinishRows];
#pragma unroll
  for (int q = 0; q < kLongFinishRows; ++q) {
    const int r = blockIdx.x * kLongFinishRows + q;
    s0v[q] = (r < a.nbr && sa.slot0) ? ld_idx(sa.slot0, r) : -1;
    s1v[q] = (r < a.nbr && sa.slot1) ? ld_idx(sa.slot1, r) : -1;
  }
  uint16_t* H = reinterpret_cast<uint16_t*>(a.Y);
  const int64_t slice = (int64_t)a.T * B;  // values of one chunk's or one side's sums
  // A thread takes four neighbouring rows of one token, 16 bytes per load; kAhead chunks of each side per
  // round, the loads of a round first.  Every load is unconditional (indices clamped, the surplus multiplied
  // by zero), so that they leave back to back.
  constexpr int kAhead = 8, kQuads = kLongFinishTokens * B / 4;
  const int e = threadIdx.x * 4;
  const bool mine = threadIdx.x < kQuads && blockIdx.y * kLongFinishTokens + e / B < a.T;
  const int t = mine ? blockIdx.y * kLongFinishTokens + e / B : 0, i = mine ? e % B : 0;
  using f32x4 = __attribute__((ext_vector_type(4))) float;
#pragma unroll 1
  for (int q = 0; q < kLongFinishRows; ++q) {
    const int s0 = s0v[q], s1 = s1v[q];
    if (s0 < 0 && s1 < 0) continue;
    const int r = blockIdx.x * kLongFinishRows + q;
    // gate side: the chunks of the row in P0, or the whole side in W1; up side: chunks in P1, or W0
    const float* G;
    const float* U;
    int nG = 1, nU = 1;
    if (s0 >= 0) {
      G = sa.P0 + ld_idx(sa.chunk0_0, r) * slice;
      nG = (ld_idx(a.m0.row_ptr, r + 1) - ld_idx(a.m0.row_ptr, r) + kLongChunk - 1) / kLongChunk;
    } else {
      G = sa.W1 + s1 * slice;
    }
    if (s1 >= 0) {
      U = sa.P1 + ld_idx(sa.chunk0_1, r) * slice;
      nU = (ld_idx(a.m1.row_ptr, r + 1) - ld_idx(a.m1.row_ptr, r) + kLongChunk - 1) / kLongChunk;
    } else {
      U = sa.W0 + s0 * slice;
    }
    G += (int64_t)t * B + i;
    U += (int64_t)t * B + i;
    f32x4 gv = {0.0f, 0.0f, 0.0f, 0.0f}, uv = gv;
    const int nmax = nG > nU ? nG : nU;
    for (int c0 = 0; c0 < nmax; c0 += kAhead) {
      f32x4 gl[kAhead], ul[kAhead];
#pragma unroll
      for (int cc = 0; cc < kAhead; ++cc) {
        const int c = c0 + cc;
        gl[cc] = *reinterpret_cast<const f32x4*>(G + (c < nG ? c : nG - 1) * slice);
        ul[cc] = *reinterpret_cast<const f32x4*>(U + (c < nU ? c : nU - 1) * slice);
      }
#pragma unroll
      for (int cc = 0; cc < kAhead; ++cc) {  // in the order of the plan
        const int c = c0 + cc;
        if (c < nG) gv += gl[cc];
        if (c < nU) uv += ul[cc];
      }
    }
    if (mine) {
      uint16_t* h = H + (int64_t)t * a.syt + ((int64_t)r * B + i) * a.syi;
#pragma unroll
      for (int k = 0; k < 4; ++k) h[k * a.syi] = f32_to_bf16_rne(apply_act(a.act, gv[k]) * uv[k]);
    }
  }
}

}  // namespace blast_dev
