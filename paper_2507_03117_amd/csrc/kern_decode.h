// Decode kernel: block-sparse product for a handful of tokens (T <= 128 or so).
//
// At these token counts the product is bound by streaming the stored blocks out
// of HBM once (the paper's abstract: data movement dominates), so the kernel is
// organised around the memory pipeline:
//  - one workgroup per (block row, 16-row slice), or per (chunk of a block row,
//    16-row slice) when the packer's chunk plan is in use; its four waves deal the
//    stored blocks among themselves, so even a row with a single block keeps a
//    wave busy and a long row is read by four waves at once;
//  - a 16-row slice of a block is contiguous in memory: a wave copies it
//    global -> LDS with wave-wide 1 KiB requests (whole 128-byte lines, the
//    request shape the L1 path handles best), and copies the matching activation
//    tile (16 tokens x B) the same way; nothing passes through registers, so the
//    only ordering device is the wave's own memory counter, which this code
//    controls completely;
//  - every wave owns a ring of NSLOT (slice + activation tile) slots in LDS: the
//    copies of the next NSLOT-1 blocks are in flight while one block is
//    multiplied; no other wave touches a wave's ring, so the loop has no barrier;
//  - 16-byte chunks are XOR-swizzled inside their row on the global-address side
//    of the copy, so that the operand-fragment reads do not pile onto one bank;
//  - the products run on v_mfma_f32_16x16x32_bf16, 16 tokens per instruction;
//  - the four partial sums meet in LDS (in a buffer laid over the rings, behind the kernel's only
//    barrier); wave 0 applies the epilogue;
//  - the single-launch MLP's variants at b = 128 and for 64-token units load the weight fragments
//    straight into registers instead (DecCfg::WREG): there the number of resident workgroups matters
//    more than the shape of the requests.
// Same arithmetic as the tile kernels: bf16 products, fp32 accumulation,
// activation on the fp32 sums, one rounding to bf16 where the output is bf16.
#pragma once
#include "kern_common.h"
#include "kern_stream.h"

namespace blast_dev {

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct DecArgs {
  MatDev m0, m1;         // m1 only for the dual (gate/up) kernel
  const int* row_order;  // block rows by population, fullest first (may be null)
  const uint16_t* X;
  int64_t sxt;           // elements between tokens (token-major, 16-byte aligned rows)
  void* Y;
  int64_t syt, syi;
  int y_bf16;
  int T;
  int act;       // as in TileArgs
  int n_units;   // (block rows or chunk slots) * slices
  int groups;    // token groups of NTT * 16 tokens
  // chunk plan written by the packer (CHUNK instances only): hdr[0] = number of chunks
  const int* hdr;
  const int* chunk_row;  // block row of the chunk; bit 31 set when the row has several chunks
  const int* chunk_kb;   // first stored block of the chunk
  const int* chunk_ke;   // one past its last stored block
  // single-launch MLP only: one 64-bit slot per (block row of H, 16-row slice); the producer of that
  // slice stores the launch's token there once its part of H is visible device-wide, consumers wait for it.
  // The token is `token` (drawn on the host, one per call) mixed with the epoch kept in ctl[1], see
  // handover_token(): a replay of a captured call differs from the previous replay in the epoch.
  unsigned long long* slots;
  unsigned long long token;
  unsigned long long* ctl;  // control block in the workspace (kCtlBytes): signature, epoch, status, arrival counters
  int total_waves;          // waves of the whole launch
  int ctl_shift;            // log2 of what a launch adds to each arrival counter (a power of two >= the largest group)
  int max_spins;            // polls before a wait gives up (never hang the GPU)
  int withhold;             // diagnostic: producers compute H but do not publish it
  int* sync_err;            // status word: kHandoverTimedOut / kHandoverInitTimedOut once a wait has given up
  // Side job of a launch (z_blocks > 0): workgroups [main_blocks, main_blocks + z_blocks) clear the fp32
  // rows that a LATER chunked product will accumulate into (the rows of block rows cut into several
  // chunks), so that product needs no clearing launch of its own.  One workgroup per chunk slot.
  int main_blocks, z_blocks;
  const int* z_hdr;
  const int* z_chunk_row;
  const int* z_chunk_kb;
  const int* z_row_ptr;
  float* z_Y;
  int64_t z_syt, z_syi;
  int z_T;
};

template <int B>
__device__ __forceinline__ void decode_zero_job(const DecArgs& a, int ci) {
  if (ci >= ld_idx(a.z_hdr, 0)) return;
  const int cr = ld_idx(a.z_chunk_row, ci);
  if (cr >= 0) return;  // a single-chunk row is stored, not accumulated
  const int r = cr & 0x7FFFFFFF;
  if (ld_idx(a.z_chunk_kb, ci) != ld_idx(a.z_row_ptr, r)) return;  // only the first chunk of the row clears
  for (int e = threadIdx.x; e < a.z_T * B; e += 256) {
    const int t = e / B, i = e % B;
    a.z_Y[(int64_t)t * a.z_syt + ((int64_t)r * B + i) * a.z_syi] = 0.0f;
  }
}

// Eight E5M2 codes -> eight bf16 values, exactly: the hardware conversion of the 8-bit type with 5 exponent bits
// (on gfx950 the format of Sec. 5.2: subnormals, infinities and NaN as in the upper byte of an IEEE half) widens
// two codes to fp32 at a time, and a value with two mantissa bits passes the conversion to bf16 unchanged.
__device__ __forceinline__ bf16x8 e5m2x8_to_bf16x8(uint2 raw) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  u32x4 out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned word = i < 2 ? raw.x : raw.y;
    const f32x2 f = (i & 1) ? __builtin_amdgcn_cvt_pk_f32_bf8(word, true) : __builtin_amdgcn_cvt_pk_f32_bf8(word, false);
    const bf16x2 h = {static_cast<__bf16>(f[0]), static_cast<__bf16>(f[1])};
    out[i] = __builtin_bit_cast(unsigned, h);
  }
  return __builtin_bit_cast(bf16x8, out);
}

enum DecRole { kDecAlone = 0, kDecProducer = 1, kDecConsumer = 2 };
constexpr int kDecMaxSpins = 1 << 19;  // polls of ~0.3 us each before a consumer gives up (never hang the GPU)
constexpr unsigned long long kCtlReady = 0xB1A57C7100D0C0DEull;  // the control block has been set up
constexpr unsigned long long kCtlBusy = 0xB1A57C71B0057EEDull;   // a wave is setting it up right now
constexpr int kHandoverTimedOut = 1, kHandoverInitTimedOut = 2;

constexpr int kCtlGroups = 64;        // arrival counters, each in a 128-byte line of its own
constexpr int kCtlLineWords = 16;     // 64-bit words per line
// Control block of the single-launch form, in 64-bit words (kCtlBytes bytes of the workspace):
//   [0] signature  [2] status (low 32 bits)  [(2 + g) * kCtlLineWords], g < kCtlGroups: arrival counters
constexpr int kCtlGroupWord0 = 2 * kCtlLineWords;
constexpr int kCtlBytes = (2 + kCtlGroups) * kCtlLineWords * 8;

// Every wave of a single-launch MLP calls handover_peek first thing, handover_begin once it needs the token
// and handover_leave as its last act.
//
// The token of a launch is the call's host-drawn token mixed with an epoch that must change from launch to
// launch on the same workspace (a call recorded into a graph is replayed with the same arguments).  The
// epoch is not stored anywhere: it is read off an arrival counter.  Wave number n belongs to group n % 64
// and, when it leaves, adds 1 to its group's counter - the group's first wave adds the rest up to a power
// of two P as well, so that a launch adds exactly P to every counter.  A counter therefore stays inside
// [epoch * P, (epoch + 1) * P) from the first to the last wave of a launch, whichever waves have already
// left, and counter >> log2(P) is the same number for every wave of the launch and one more for the next
// launch.  Nobody waits for anybody, no addition returns a value, and no address takes more than a few dozen
// additions per launch.  Launches on one workspace are ordered by their stream (overlapping calls need
// different workspaces), and what a launch added is visible when the next one starts.
//
// The control block needs no initialisation by the caller: a wave that does not find the signature of its
// launch shape (the number of waves is part of it) claims the set-up with a compare-and-swap on whatever it
// found there; the winner clears the counters and the status word, waits for those stores to be
// acknowledged and writes the signature; every other wave polls for the signature (the winner is running
// and waits for nothing, so that wait ends; it is bounded besides).
struct HandoverPeek {
  unsigned long long sig, count;
};
struct Handover {
  unsigned long long token;  // of this launch, the same in every wave
  unsigned long long add;    // what this wave adds to its group's counter when it leaves
  int group;
};
__device__ __forceinline__ int handover_group() { return (blockIdx.x * 4 + (threadIdx.x >> 6)) % kCtlGroups; }

// The signature as the scalar cache sees it (a stale value only sends the wave down the slow path of
// handover_begin) and this wave's counter read past the caches (a value from any moment of this launch
// gives the same epoch; one cached before the set-up of the control block would not).  Issued first thing
// in a wave, used later.
__device__ __forceinline__ HandoverPeek handover_peek(const DecArgs& a) {
  const __attribute__((address_space(4))) unsigned long long* c =
      reinterpret_cast<const __attribute__((address_space(4))) unsigned long long*>(reinterpret_cast<uintptr_t>(a.ctl));
  return HandoverPeek{c[0], __hip_atomic_load(a.ctl + kCtlGroupWord0 + handover_group() * kCtlLineWords, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT)};
}

__device__ __forceinline__ Handover handover_begin(const DecArgs& a, const HandoverPeek& pk) {
  Handover h{};
  const int wave_id = blockIdx.x * 4 + (threadIdx.x >> 6);
  h.group = wave_id % kCtlGroups;
  const int group_size = a.total_waves / kCtlGroups + (h.group < a.total_waves % kCtlGroups ? 1 : 0);
  h.add = wave_id < kCtlGroups ? (1ull << a.ctl_shift) - (unsigned long long)group_size + 1ull : 1ull;
  const unsigned long long ready = kCtlReady ^ (unsigned long long)(unsigned)a.total_waves;
  unsigned long long count = pk.count;
  if (pk.sig != ready) {
    if ((threadIdx.x & 63) == 0) {
      unsigned long long m = __hip_atomic_load(a.ctl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (m != ready) {
        bool won = false;
        if (m != kCtlBusy)
          won = __hip_atomic_compare_exchange_strong(a.ctl, &m, kCtlBusy, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
        if (won) {
          for (int i = 1; i < kCtlBytes / 8; i += (i < kCtlLineWords ? 1 : kCtlLineWords))
            __hip_atomic_store(a.ctl + i, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0));  // all acknowledged before the signature appears
          asm volatile("" ::: "memory");
          __hip_atomic_store(a.ctl, ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
          int spins = 0;
          while (__hip_atomic_load(a.ctl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != ready) {
            if (++spins > a.max_spins) {
              __hip_atomic_store(a.sync_err, kHandoverInitTimedOut, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              break;
            }
            __builtin_amdgcn_s_sleep(2);
          }
        }
      }
    }
    // the counter has just been cleared (waves that have left since may have added to it): read it afresh
    count = __hip_atomic_load(a.ctl + kCtlGroupWord0 + h.group * kCtlLineWords, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  const unsigned long long epoch = count >> a.ctl_shift;
  const unsigned elo = __builtin_amdgcn_readfirstlane((unsigned)epoch);
  const unsigned ehi = __builtin_amdgcn_readfirstlane((unsigned)(epoch >> 32));
  h.token = (a.token ^ ((((unsigned long long)ehi << 32) | elo) * 0x9E3779B97F4A7C15ull)) | 1ull;
  return h;
}

__device__ __forceinline__ void handover_leave(const DecArgs& a, const Handover& h) {
  if ((threadIdx.x & 63) == 0)
    (void)__hip_atomic_fetch_add(a.ctl + kCtlGroupWord0 + h.group * kCtlLineWords, h.add, __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_AGENT);
}

// XSMALL > 0: the activation tile of a block holds only as many token rows as XSMALL copy instructions
// bring (XSMALL * 512 / B); valid when T does not exceed that.  It shrinks a ring slot, hence allows more
// workgroups per CU at the token counts that matter most for decoding, and it lowers the activation bytes
// that travel with every weight slice.
// FUSED: the instance runs inside the single-launch MLP (same ring; kept as a separate configuration point).
// W8: the stored block values are E5M2 codes, one byte each (MatDev::vals8); a weight slice is half the
// bytes, its fragments are widened to bf16 (exactly) on the way into the matrix instruction.
template <int B, bool DUAL, int NTT, int XSMALL = 0, bool FUSED = false, bool W8 = false>
struct DecCfg {
  static_assert(!W8 || B >= 64, "one-byte weights: at least one whole copy instruction per slice");
  static_assert(!XSMALL || (NTT == 1 && B >= 64 && XSMALL * 512 / B < 16),
                "small activation tiles: one token group, at least 8 chunks per row, fewer than 16 token rows");
  static constexpr int SLICES = B / 16;       // 16-row slices per block row
  static constexpr int KST = B / 32;          // 32-wide k-steps per block
  static constexpr int SLB = 16 * B * 2;      // bytes of a 16-token activation tile (and of a 16-row slice of bf16 weights)
  static constexpr int WEB = W8 ? 1 : 2;      // bytes per stored weight
  static constexpr int SLW = 16 * B * WEB;    // bytes of one 16-row slice of a block
  static constexpr int NI = SLW / 1024;       // wave-wide copy instructions per slice
  static constexpr int CPRW = B / 8;          // 16-byte chunks per row (bf16)
  static constexpr int CPRW8 = B / 16;        // 16-byte chunks per row of one-byte weights
  static constexpr int XR = XSMALL ? XSMALL * 512 / B : 16 * NTT;  // token rows of the activation tile
  static constexpr int XB = XR * B * 2;                   // its bytes
  static constexpr int NIX = XB / 1024;                   // copy instructions per activation tile
  static constexpr int SLOT = SLW + XB;
  // XONE: one activation tile per wave instead of one per slot.  A block's fragments are moved to registers
  // before the next block's activation tile is copied over them, so only the weight slices need two slots.
  // Used where two 16-token tiles per slot would otherwise leave room for a single workgroup per CU
  // (b = 128 with 32 tokens per unit).
  // WREG: the weight fragments go from memory straight into registers (each lane fetches the 16 bytes it feeds
  // the matrix instruction with), no LDS for them.  Used by the single-launch MLP at b = 128: with weight
  // slots in LDS only three of its workgroups fit a CU (46 KiB each), so a layer of a thousand units ran in
  // two rounds and the consumers, dispatched last, started microseconds late (8B-shaped layer, one token: 768
  // resident of 1152), and by its 64-token units at b = 64.  The activation tile keeps one LDS tile per wave.
  // (Activation fragments in registers as well were measured: 112 VGPRs, four waves per SIMD, and the second
  // round is back.)  Only where latency rules: the ordinary launches of a large layer are bound by bandwidth, and
  // 16-byte loads scattered over 16 rows fetch less per request than the 1 KiB copies (405B-class layer, one
  // token: 61 against 51 us; 16 tokens: 72 against 64).
  static constexpr bool WREG = FUSED && !W8 && (B == 128 || NTT == 4);
  static constexpr bool XONE = !XSMALL && NTT == 2 && B == 128;
  // Two slots per wave: one block being multiplied, one in flight.  Deeper rings were measured and lose: what
  // hides the latency of the copies here is the number of resident workgroups (three per CU at b = 128 with
  // the small activation tile, four at b = 64, before the partial sums were laid over the ring; now one more
  // each), and every extra slot costs residents.
  // One-byte weights halve a slice: where a slot stays within 4 KiB the ring is four slots deep, so that the
  // bytes in flight per wave - what the HBM bandwidth reached follows - are those of the bf16 form.
  static constexpr int NSLOT = (W8 && SLOT <= 4096) ? 4 : 2;
  static constexpr int WAVE_LDS = WREG ? XB : (XONE ? NSLOT * SLW + XB : NSLOT * SLOT);
  static constexpr int OPS = NI + NIX;        // copy instructions per block and wave
  static constexpr int NM = DUAL ? 2 : 1;
  static constexpr int RING_LDS = 4 * WAVE_LDS;
  static constexpr int RED_LDS = 3 * NM * NTT * 4 * 64 * 4;
  // The buffer in which the four partial sums meet lies over the ring, which every wave is done with by then (a
  // barrier in front of it): every kilobyte counts towards how many workgroups fit a CU.  Measured where it
  // decides that number: 32-token units of the single launch at b = 64 (60 -> 48 KiB, three workgroups per CU,
  // the whole 1B-shaped launch resident: 13.2 -> 11.5 us), one-byte weights with their four-slot rings at
  // b = 128 (54 -> 48 KiB, three instead of two: 42.6 -> 37.7 us on the 405B-class layer with a uniform mask).
  static constexpr int RED_OFF = 0;
  static constexpr size_t LDS_BYTES = (size_t)(RING_LDS > RED_LDS ? RING_LDS : RED_LDS);
  static_assert(SLW % 1024 == 0 && (NSLOT - 1) * OPS < 64, "copy granularity / counter range");
  // swizzle key of a row (mod 16): distinct for rows that would otherwise share banks
  __device__ static __forceinline__ int key(int row) { return ((row & 15) / (16 / (CPRW < 16 ? CPRW : 16))) % CPRW; }
  // the same for rows of one-byte weights (B bytes per row: two rows of b = 64 share the 32 banks)
  __device__ static __forceinline__ int key8(int row) { return (B == 64 ? (row >> 1) : row) % CPRW8; }
};

// The work of one workgroup: unit = (block row or chunk, 16-row slice), tokens [t_base, t_base + 16 NTT).
// ROLE: alone (an ordinary launch); producer / consumer (the two halves of the single-launch MLP: the
// producer publishes its slice of H, the consumer waits for the slices of H its blocks will read).
// POST: a single-matrix product whose sums go through the activation a.act before they are stored (the
// first half of a two-matrix MLP).
template <int B, bool DUAL, int NTT, bool CHUNK, int XSMALL, int ROLE, bool POST = false, bool W8 = false>
__device__ __forceinline__ void decode_unit(const DecArgs& a, const int unit, const int t_base, unsigned char* smem) {
  static_assert(!W8 || ROLE == kDecAlone, "one-byte weights run as ordinary launches");
  static_assert(!(DUAL && CHUNK), "the activation needs complete sums: the gated product is never split");
  static_assert(!POST || (!DUAL && !CHUNK), "an activation on the output needs complete sums of a single matrix");
  static_assert(ROLE == kDecAlone || (ROLE == kDecProducer && !CHUNK && (DUAL || POST)) ||
                    (ROLE == kDecConsumer && !DUAL && !CHUNK && !POST),
                "producers compute the activated intermediate, consumers a plain product");
  using C = DecCfg<B, DUAL, NTT, XSMALL, ROLE != kDecAlone, W8>;
  constexpr int KST = C::KST, NM = C::NM, NI = C::NI, NSLOT = C::NSLOT;
  float (*red)[NM][NTT][4][64] = reinterpret_cast<float (*)[NM][NTT][4][64]>(smem + C::RED_OFF);
  const int q = unit % C::SLICES;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, l16 = lane & 15, g = lane >> 4;
  unsigned char* ring = smem + wave * C::WAVE_LDS;

  int r, kb0, n0, kb1 = 0, n1 = 0;
  bool shared_row = false;
  Handover hand{};  // single-launch MLP only
  HandoverPeek peek{};
  if (ROLE != kDecAlone) peek = handover_peek(a);
  if (CHUNK) {
    const int ci = unit / C::SLICES;
    if (ci >= ld_idx(a.hdr, 0)) return;  // the grid is sized by an upper bound of the number of chunks
    const int cr = ld_idx(a.chunk_row, ci);
    r = cr & 0x7FFFFFFF;
    shared_row = cr < 0;
    kb0 = ld_idx(a.chunk_kb, ci);
    n0 = ld_idx(a.chunk_ke, ci) - kb0;
  } else {
    const int rank = unit / C::SLICES;
    r = a.row_order ? ld_idx(a.row_order, rank) : rank;
    kb0 = ld_idx(a.m0.row_ptr, r);
    n0 = ld_idx(a.m0.row_ptr, r + 1) - kb0;
    if (DUAL) {
      kb1 = ld_idx(a.m1.row_ptr, r);
      n1 = ld_idx(a.m1.row_ptr, r + 1) - kb1;
    }
  }
  const int n = n0 + n1;
  // this wave's blocks are i = wave + 4 j, j < cnt
  const int cnt = n > wave ? (n - wave + 3) >> 2 : 0;

  f32x4 acc[NM][NTT];
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int tt = 0; tt < NTT; ++tt) acc[m][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- per-lane constants ----------------------------------------------------------------
  // Copy side: instruction ni of a tile writes LDS bytes [ni*1024 + lane*16, +16), i.e. position
  // p = ni*64 + lane in 16-byte units = (row p / CPRW, slot p % CPRW); it fetches chunk slot ^ key(row)
  // of that row.  Weight rows are B*2 bytes apart, activation rows sxt*2 bytes (clamped to the last token).
  uint32_t woff[NI], xoff[C::NIX];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    if (W8) {
      const int p = ni * 64 + lane, row = p / C::CPRW8, slot = p % C::CPRW8;
      woff[ni] = (uint32_t)(q * C::SLW + row * B + ((slot ^ C::key8(row)) << 4));
    } else {
      const int p = ni * 64 + lane, row = p / C::CPRW, slot = p % C::CPRW;
      woff[ni] = (uint32_t)(q * C::SLB + row * (B * 2) + ((slot ^ C::key(row)) << 4));
    }
  }
#pragma unroll
  for (int xi = 0; xi < C::NIX; ++xi) {
    const int p = xi * 64 + lane, row = p / C::CPRW, slot = p % C::CPRW;
    int t = t_base + row;
    t = t < a.T ? t : a.T - 1;
    xoff[xi] = (uint32_t)t * (uint32_t)a.sxt * 2u + (uint32_t)((slot ^ C::key(row)) << 4);
  }
  // Fragment side: row l16, chunk 4 s + g of a tile image.  A small activation tile has fewer rows than
  // the matrix instruction has token lanes: the lanes past it re-read rows whose results are never stored.
  uint32_t foff[KST], fxoff[KST];
  const int xrow = XSMALL ? (l16 % C::XR) : l16;
#pragma unroll
  for (int s = 0; s < KST; ++s) {
    // one-byte weights: the 8 values of k-step s, lane group g are bytes 32 s + 8 g ... of the row, i.e. half
    // g % 2 of the 16-byte chunk 2 s + g / 2
    foff[s] = W8 ? (uint32_t)(l16 * B + (((2 * s + (g >> 1)) ^ C::key8(l16)) << 4) + ((g & 1) << 3))
                 : (uint32_t)(l16 * (B * 2) + (((4 * s + g) ^ C::key(l16)) << 4));
    fxoff[s] = (uint32_t)(xrow * (B * 2) + (((4 * s + g) ^ C::key(xrow)) << 4));
  }
  // a weight fragment from its LDS image
  auto wfrag = [&](const unsigned char* p) -> bf16x8 {
    if constexpr (W8) {
      return e5m2x8_to_bf16x8(*reinterpret_cast<const uint2*>(p));
    } else {
      return *reinterpret_cast<const bf16x8*>(p);
    }
  };

  // ---- ring -----------------------------------------------------------------------------
  // where block j's weight slice and activation tile live in this wave's part of the ring
  auto wslot = [&](int j) { return ring + (j % NSLOT) * (C::XONE ? C::SLW : C::SLOT); };
  auto xslot = [&](int j) {
    return C::WREG ? ring : (C::XONE ? ring + NSLOT * C::SLW : ring + (j % NSLOT) * C::SLOT + C::SLW);
  };
  auto locate = [&](int j, const unsigned char*& wblk, const unsigned char*& xcol) {
    const int i = wave + 4 * j;
    const bool second = DUAL && i >= n0;
    const MatDev& m = second ? a.m1 : a.m0;
    const int k = second ? kb1 + (i - n0) : kb0 + i;
    wblk = W8 ? m.vals8 + (int64_t)k * (B * B)
              : reinterpret_cast<const unsigned char*>(m.vals) + (int64_t)k * (B * B * 2);
    xcol = reinterpret_cast<const unsigned char*>(a.X) + (int64_t)ld_idx(m.col_idx, k) * (B * 2);
  };
  auto issue_w = [&](int j) {
    const unsigned char *wblk, *xcol;
    locate(j, wblk, xcol);
    unsigned char* dst = wslot(j);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) BLAST_GLDS16(wblk + woff[ni], dst + ni * 1024);
  };
  auto issue_x = [&](int j) {
    const unsigned char *wblk, *xcol;
    locate(j, wblk, xcol);
    unsigned char* dst = xslot(j);
#pragma unroll
    for (int xi = 0; xi < C::NIX; ++xi) BLAST_GLDS16(xcol + xoff[xi], dst + xi * 1024);
  };
  auto issue = [&](int j) {
    issue_w(j);
    issue_x(j);
  };

  // Consumers: called once the copies of the first block's weights are on their way and before the first copy
  // of H.  Pulls the wave's other weight slices towards the L2 while H is still being produced (they do not
  // depend on it), then waits until every slice of H that its blocks read has been published.
  auto wait_for_h = [&]() {
    if (ROLE != kDecConsumer) return;
    uint32_t warm = 0;
#pragma unroll 1
    for (int j = 0; j < cnt; ++j) {
      const int k = kb0 + wave + 4 * j;
      const unsigned char* wblk = reinterpret_cast<const unsigned char*>(a.m0.vals) + (int64_t)k * (B * B * 2);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) warm ^= *reinterpret_cast<const uint32_t*>(wblk + woff[ni]);
    }
    hand = handover_begin(a, peek);
    const unsigned long long token = hand.token;
    bool gave_up = false;
    // One poll covers the slots of 64 / SLICES blocks: lane -> (block jb + lane / SLICES, slice lane % SLICES).
    // Polling block after block would cost a round trip to the memory side per block even when every
    // slice has long been published.
    constexpr int kPerPoll = 64 / C::SLICES;
#pragma unroll 1
    for (int jb = 0; jb < cnt && !gave_up; jb += kPerPoll) {
      const int jj = jb + lane / C::SLICES;
      const bool mine = jj < cnt;
      const int col = mine ? a.m0.col_idx[kb0 + wave + 4 * jj] : 0;
      const unsigned long long* sl = a.slots + (int64_t)col * C::SLICES + (lane % C::SLICES);
      int spins = 0;
      for (;;) {
        const unsigned long long v = mine ? __hip_atomic_load(sl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : token;
        if (__ballot(v != token) == 0) break;
        if (++spins > a.max_spins) {
          gave_up = true;
          break;
        }
        __builtin_amdgcn_s_sleep(2);
      }
    }
    if (gave_up) {
      // the output rows of this unit become NaN instead of plausible numbers, and the status word says why
      if (lane == 0) __hip_atomic_store(a.sync_err, kHandoverTimedOut, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
      for (int tt = 0; tt < NTT; ++tt) acc[0][tt] = f32x4{__builtin_nanf(""), __builtin_nanf(""), __builtin_nanf(""), __builtin_nanf("")};
    }
    // keeps the warming loads alive; the value never matches
    if (warm == 0x9E3779B9u && a.T < 0) a.sync_err[1] = 1;
    asm volatile("" ::: "memory");
  };

  // a producer draws the launch's token while its first copies are in flight; it needs it only to publish
  if constexpr (C::WREG) {
    // Fragment (k-step s, lane group g) of weight row l16 = bytes [(4 s + g) * 16, +16) of that row.  Two
    // register sets take turns: the fragments of the next block are on their way while one block is
    // multiplied (a third set was measured and changes nothing: with at most a few blocks per wave the time
    // is the memory's, not the ring's).  The activation tile still goes through LDS, one tile per wave,
    // copied a block ahead.
    bf16x8 w0s[KST], w1s[KST];
    const uint32_t wg0 = (uint32_t)(q * C::SLB + l16 * (B * 2) + g * 16);
    auto load_w = [&](bf16x8 (&dst)[KST], int j) {
      const unsigned char *wblk, *xcol;
      locate(j, wblk, xcol);
#pragma unroll
      for (int s = 0; s < KST; ++s) dst[s] = *reinterpret_cast<const bf16x8*>(wblk + wg0 + s * 64);
      asm volatile("" ::: "memory");  // issued here, not later
    };
    if (cnt > 0) load_w(w0s, 0);
    if (cnt > 1) load_w(w1s, 1);
    wait_for_h();
    if (cnt > 0) issue_x(0);
    if (ROLE == kDecProducer) hand = handover_begin(a, peek);
    // Requests retire in issue order: W 0, W 1, X 0, and then per block j: X j+1, W j+2.  When block j
    // starts, the only requests younger than its activation tile are the KST loads of W j+1 (j >= 1).
    auto block = [&](bf16x8 (&wcur)[KST], int j) {
      if (j >= 1 && j + 1 < cnt)
        __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(KST));
      else
        __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0));
      asm volatile("" ::: "memory");
      const unsigned char* xs = xslot(j);
      bf16x8 xf[KST][NTT];
#pragma unroll
      for (int s = 0; s < KST; ++s)
#pragma unroll
        for (int tt = 0; tt < NTT; ++tt) xf[s][tt] = *reinterpret_cast<const bf16x8*>(xs + C::SLB * tt + fxoff[s]);
      // the fragments are in registers before the next activation tile is copied over this one
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
      asm volatile("" ::: "memory");
      if (j + 1 < cnt) issue_x(j + 1);
      const bool second = DUAL && (wave + 4 * j) >= n0;
      const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KST; ++s) {
        const bf16x8 wg = second ? zero : wcur[s];
#pragma unroll
        for (int tt = 0; tt < NTT; ++tt) {
          acc[0][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[s][tt], wg, acc[0][tt], 0, 0, 0);
          if (DUAL) {
            const bf16x8 wu = second ? wcur[s] : zero;
            acc[NM - 1][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[s][tt], wu, acc[NM - 1][tt], 0, 0, 0);
          }
        }
      }
      asm volatile("" ::: "memory");
      if (j + 2 < cnt) load_w(wcur, j + 2);
    };
#pragma unroll 1
    for (int j = 0; j < cnt; j += 2) {
      block(w0s, j);
      if (j + 1 < cnt) block(w1s, j + 1);
    }
  } else if constexpr (C::XONE) {
    static_assert(!C::XONE || NSLOT == 2, "the single activation tile is written for two weight slots");
    if (cnt > 0) issue_w(0);
    wait_for_h();
    if (cnt > 0) issue_x(0);
    if (ROLE == kDecProducer) hand = handover_begin(a, peek);
#pragma unroll 1
    for (int j = 0; j < cnt; ++j) {
      const bool more = j + 1 < cnt;
      // The other weight slot is free: its fragments went to registers an iteration ago.  Copies retire in
      // issue order (..., W j, X j, W j+1), so "at most NI outstanding" means block j has landed whole.
      if (more) {
        issue_w(j + 1);
        __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(NI));
      } else {
        __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0));
      }
      asm volatile("" ::: "memory");
      const unsigned char* ws = wslot(j);
      const unsigned char* xs = xslot(j);
      bf16x8 wf[KST], xf[KST][NTT];
#pragma unroll
      for (int s = 0; s < KST; ++s) {
        wf[s] = wfrag(ws + foff[s]);
#pragma unroll
        for (int tt = 0; tt < NTT; ++tt) xf[s][tt] = *reinterpret_cast<const bf16x8*>(xs + C::SLB * tt + fxoff[s]);
      }
      // the fragments are in registers before the next activation tile is copied over this one
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
      asm volatile("" ::: "memory");
      if (more) issue_x(j + 1);
      const bool second = DUAL && (wave + 4 * j) >= n0;
      const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KST; ++s) {
        const bf16x8 w0 = second ? zero : wf[s];
#pragma unroll
        for (int tt = 0; tt < NTT; ++tt) {
          acc[0][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[s][tt], w0, acc[0][tt], 0, 0, 0);
          if (DUAL) {
            const bf16x8 w1 = second ? wf[s] : zero;
            acc[NM - 1][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[s][tt], w1, acc[NM - 1][tt], 0, 0, 0);
          }
        }
      }
      asm volatile("" ::: "memory");
    }
  } else {
  if constexpr (ROLE == kDecConsumer) {
    // the first block's weights are copied while the wait lasts (two slots: one block ahead, so the order
    // W 0, X 0, W 1, X 1, ... that the waits below count on is kept)
    static_assert(ROLE != kDecConsumer || NSLOT == 2, "the split first step is written for one block ahead");
    if (cnt > 0) issue_w(0);
    wait_for_h();
    if (cnt > 0) issue_x(0);
  } else {
#pragma unroll 1
    for (int j = 0; j < NSLOT - 1; ++j)
      if (j < cnt) issue(j);
  }
  if (ROLE == kDecProducer) hand = handover_begin(a, peek);

#pragma unroll 1
  for (int j = 0; j < cnt; ++j) {
    // fragment reads of the previous block have returned before its slot is handed back to the copier
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    asm volatile("" ::: "memory");
    if (j + NSLOT - 1 < cnt) issue(j + NSLOT - 1);
    // copies retire in issue order: "at most (blocks issued after j) * OPS outstanding" = block j has landed
    const int later = (cnt - 1 - j) < (NSLOT - 1) ? (cnt - 1 - j) : (NSLOT - 1);
    if (later >= 3)
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(3 * C::OPS < 63 ? 3 * C::OPS : 63));
    else if (later == 2)
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(2 * C::OPS));
    else if (later == 1)
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(C::OPS));
    else
      __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0));
    asm volatile("" ::: "memory");
    const unsigned char* slot = wslot(j);
    const bool second = DUAL && (wave + 4 * j) >= n0;
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    // Straight-line on purpose: a block of the other matrix multiplies a zeroed operand instead of
    // branching around the matrix instruction (adding 0 * x to an fp32 sum is exact, and matrix
    // instructions are not the bottleneck at these token counts).
#pragma unroll
    for (int s = 0; s < KST; ++s) {
      const bf16x8 wf = wfrag(slot + foff[s]);
      const bf16x8 w0 = second ? zero : wf;
#pragma unroll
      for (int tt = 0; tt < NTT; ++tt) {
        const bf16x8 xf = *reinterpret_cast<const bf16x8*>(slot + C::SLW + C::SLB * tt + fxoff[s]);
        acc[0][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf, w0, acc[0][tt], 0, 0, 0);
        if (DUAL) {
          const bf16x8 w1 = second ? wf : zero;
          acc[NM - 1][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf, w1, acc[NM - 1][tt], 0, 0, 0);
        }
      }
    }
    asm volatile("" ::: "memory");
  }

  }

  // ---- the four partial sums meet in LDS ---------------------------------------------------
  __syncthreads();  // every wave has read the last of its ring: the partial sums go over it
  if (wave > 0) {
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[wave - 1][m][tt][j][lane] = acc[m][tt][j];
  }
  __syncthreads();
  if (wave > 0) {
    if (ROLE != kDecAlone) handover_leave(a, hand);
    return;
  }
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[m][tt][j] += (red[0][m][tt][j][lane] + red[1][m][tt][j][lane]) + red[2][m][tt][j][lane];

  // ---- epilogue.  Result layout of the 16x16 tile: lane -> weight row l16, register j -> token 4*g + j.
  const int64_t row = (int64_t)r * B + q * 16 + l16;
#pragma unroll
  for (int tt = 0; tt < NTT; ++tt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int tok = t_base + tt * 16 + 4 * g + j;
      if (tok < a.T) {
        float v = acc[0][tt][j];
        if (DUAL) v = apply_act(a.act, v) * acc[NM - 1][tt][j];
        if (POST) v = apply_act(a.act, v);
        const int64_t off = (int64_t)tok * a.syt + row * a.syi;
        if (ROLE == kDecProducer)  // written through to where every XCD sees it
          __hip_atomic_store(reinterpret_cast<uint16_t*>(a.Y) + off, f32_to_bf16_rne(v), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        else if (CHUNK && shared_row)
          atomicAdd(reinterpret_cast<float*>(a.Y) + off, v);  // fp32 output, zeroed before the launch
        else if (a.y_bf16)
          reinterpret_cast<uint16_t*>(a.Y)[off] = f32_to_bf16_rne(v);
        else
          reinterpret_cast<float*>(a.Y)[off] = v;
      }
    }
  if (ROLE == kDecProducer) {
    // all of this wave's stores have been acknowledged before the slot says so
    __builtin_amdgcn_s_waitcnt(BLAST_VMCNT(0));
    asm volatile("" ::: "memory");
    if (lane == 0 && !a.withhold)
      __hip_atomic_store(a.slots + (int64_t)r * C::SLICES + q, hand.token, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (ROLE != kDecAlone) handover_leave(a, hand);
}

template <int B, bool DUAL, int NTT, bool CHUNK, int XSMALL, bool POST = false, bool W8 = false>
__global__ __launch_bounds__(256) void k_decode(const DecArgs a) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  // More tokens than one tile holds mean more workgroups per unit, each re-reading the unit's weight
  // slices.  Workgroup ids are dealt round-robin to the 8 XCDs, so the token groups of one unit are
  // placed 8 ids apart: same XCD, dispatched together - the re-reads hit that XCD's L2.
  const int blk = blockIdx.x, span = 8 * a.groups;
  if (a.z_blocks > 0 && blk >= a.main_blocks) {
    decode_zero_job<B>(a, blk - a.main_blocks);
    return;
  }
  const int rem = blk % span;
  const int unit = (blk / span) * 8 + (rem & 7);
  if (unit >= a.n_units) return;
  decode_unit<B, DUAL, NTT, CHUNK, XSMALL, kDecAlone, POST, W8>(a, unit, (rem >> 3) * (NTT * 16), smem);
}

// Single-launch MLP for one token tile (T <= 16 NTT): workgroups [0, n_units) compute H slice by slice
// (args `p`; H = act(G) (.) U with GATED, H = act(W1 X) without), workgroups [n_units, n_units + c.n_units)
// the last projection (args `c`, whose X is that H).  A consumer only ever waits for producers, which wait for
// nothing and have lower workgroup ids, hence are dispatched first: the wait always ends (and is bounded
// besides).  The grid is exactly p.n_units + c.n_units: every wave takes part in the arrival count.  (Two
// token tiles per launch, each with slots of its own, were measured on the 1B-shaped layer at 65-128
// tokens: 20.8-21.6 us against 19.4 for two launches - twice the workgroups no longer fit the chip at once.)
template <int B, int NTT, int XSMALL, bool GATED = true>
__global__ __launch_bounds__(256) void k_mlp_decode(const DecArgs p, const DecArgs c) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int blk = blockIdx.x;
  if (blk < p.n_units) {
    decode_unit<B, GATED, NTT, false, XSMALL, kDecProducer, !GATED>(p, blk, 0, smem);
  } else if (blk - p.n_units < c.n_units) {
    decode_unit<B, false, NTT, false, XSMALL, kDecConsumer>(c, blk - p.n_units, 0, smem);
  }
}

}  // namespace blast_dev
