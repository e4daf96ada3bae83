// Block-sparse product and fused block-sparse gated MLP for gfx950.
//
// BLaST Sec. 3.4 (Listing 2): every output tile loops over the stored blocks of
// its block row; the block's column index selects the slice of the dense
// operand.  Sec. 3.4.3 / Eq. (1): the nonlinearity is applied to the fp32
// accumulators inside the product kernel.
//
// Orientation on the matrix cores: tokens are the M dimension (A operand = X
// tile, K-contiguous because activations are token-major), weight rows are the
// N dimension (B operand = weight block, K-contiguous because blocks are
// row-major).  The fp32 result tile then has consecutive weight rows in
// consecutive lanes, so token-major stores are 128-byte coalesced.
#include "blast_common.h"

#include <atomic>

#include "kern_common.h"
#include "kern_tile.h"
#include "kern_stream.h"
#include "kern_decode.h"
#include "kern_b16.h"

using namespace blast_dev;

namespace {

// Raises a kernel's dynamic-LDS limit once per device (the attribute is per device; setting it again
// is harmless, so a race between host threads only repeats the call).
int ensure_lds_limit(const void* kernel, size_t bytes, blast::DeviceFlags& done) {
  int dev = 0;
  BLAST_HIP_TRY(hipGetDevice(&dev));
  if (done.test(dev)) return BLAST_OK;
  BLAST_HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  done.set(dev);
  return BLAST_OK;
}

template <int B, bool DUAL>
int launch_tile(TileArgs a, hipStream_t stream) {
  using C = TileCfg<B>;
  a.ntt = (a.T + C::TT - 1) / C::TT;
  const int64_t grid = (int64_t)a.ntt * a.nbr;
  if (grid <= 0) return BLAST_OK;
  if (grid > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  if constexpr (!DUAL) {
    if (a.act >= 0) {  // single matrix with an activation on the output
      static blast::DeviceFlags lds_set_post;
      if (int rc = ensure_lds_limit(reinterpret_cast<const void*>(&k_spmm_tile<B, false, true>), C::LDS_BYTES, lds_set_post))
        return rc;
      k_spmm_tile<B, false, true><<<dim3((unsigned)grid), dim3(256), C::LDS_BYTES, stream>>>(a);
      BLAST_LAUNCH_CHECK("k_spmm_tile");
      return BLAST_OK;
    }
  }
  static blast::DeviceFlags lds_set;
  if (int rc = ensure_lds_limit(reinterpret_cast<const void*>(&k_spmm_tile<B, DUAL>), C::LDS_BYTES, lds_set)) return rc;
  k_spmm_tile<B, DUAL><<<dim3((unsigned)grid), dim3(256), C::LDS_BYTES, stream>>>(a);
  BLAST_LAUNCH_CHECK("k_spmm_tile");
  return BLAST_OK;
}

// 16 x 16 blocks, token-major 16-byte-aligned activations: pairs of blocks on the 32-deep matrix instruction,
// operands straight from global memory.  A wave takes 16, 32 or 64 tokens of one block row.
int cu_count();

template <bool DUAL, bool POST, int NS, bool SPLIT, int NW = 4>
int launch_b16_ns(TileArgs a, int y_vec, hipStream_t stream) {
  a.ntt = (a.T + 16 * NS - 1) / (16 * NS);
  const int64_t items = (int64_t)a.ntt * a.nbr;
  const int64_t grid = SPLIT ? items : (items + 3) / 4;
  if (grid <= 0) return BLAST_OK;
  if (grid > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  k_spmm_b16<DUAL, POST, NS, SPLIT, NW><<<dim3((unsigned)grid), dim3(NW * 64), 0, stream>>>(a, y_vec);
  BLAST_LAUNCH_CHECK("k_spmm_b16");
  return BLAST_OK;
}

// A wave takes 16, 32 or 64 tokens of a block row.  While that makes fewer than eight waves per CU, a workgroup
// shares one (block row, token tile) and its waves deal the row's blocks: 1B-shaped layer, 128 tokens,
// 31 -> 19 us per MLP pass, 512 tokens 39 -> 32.  Up to 16 tokens, rows of more than 16 pairs on average go to
// sixteen waves instead of four (the 1B-shaped down projection: 128 rows of 51 blocks).
template <bool DUAL, bool POST>
int launch_b16_t(const TileArgs& a, int64_t nnz, int y_vec, hipStream_t stream) {
  if (a.T <= 16) {
    if (nnz > (int64_t)32 * a.nbr) return launch_b16_ns<DUAL, POST, 1, true, 16>(a, y_vec, stream);
    return launch_b16_ns<DUAL, POST, 1, true>(a, y_vec, stream);
  }
  if (a.T <= 32) return launch_b16_ns<DUAL, POST, 2, true>(a, y_vec, stream);
  if ((int64_t)((a.T + 63) / 64) * a.nbr < 8 * cu_count()) return launch_b16_ns<DUAL, POST, 4, true>(a, y_vec, stream);
  return launch_b16_ns<DUAL, POST, 4, false>(a, y_vec, stream);
}

template <bool DUAL>
int launch_b16(const TileArgs& a, int64_t nnz, hipStream_t stream) {
  const int y_vec = a.y_grp16 || (a.syi == 1 && a.syt % 4 == 0 && blast::aligned(a.Y, a.y_bf16 ? 8 : 16));
  if constexpr (!DUAL) {
    if (a.act >= 0) return launch_b16_t<false, true>(a, nnz, y_vec, stream);  // an activation on the output
  }
  return launch_b16_t<DUAL, false>(a, nnz, y_vec, stream);
}

// From this many tokens on, a product with 16-wide blocks reads its activations from column groups of 16
// features ([K/16][T][16], see kern_b16.h) when the caller's workspace has room for the regrouped copy.
constexpr int64_t kGroup16MinTokens = 33;
size_t group16_bytes(int64_t K, int64_t T) { return blast::align_up((size_t)K * (size_t)T * 2, 256); }
bool group16_applies(int32_t b, int32_t x_layout, const void* X, int64_t ldx, int64_t T) {
  return b == 16 && T >= kGroup16MinTokens && x_layout == BLAST_TOKEN_MAJOR && ldx % 8 == 0 && blast::aligned(X, 16);
}
int enqueue_group16(const uint16_t* X, int64_t ldx, int64_t T, int64_t K, uint16_t* Xg, hipStream_t stream) {
  const int64_t nbc = K / 16;
  if (T <= 0 || nbc <= 0) return BLAST_OK;
  if ((nbc + 7) / 8 > 65535) return BLAST_ERR_INVALID_ARG;
  k_group16<<<dim3((unsigned)((T + 15) / 16), (unsigned)((nbc + 7) / 8)), dim3(256), 0, stream>>>(X, ldx, (int)T, (int)nbc, Xg);
  BLAST_LAUNCH_CHECK("k_group16");
  return BLAST_OK;
}

int cu_count() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// Rows of an fp32 output that a later chunked product accumulates into; a launch before it can clear them
// on the side (see DecArgs) and says so in `done`.
struct ZeroJob {
  const int* hdr = nullptr;
  const int* chunk_row = nullptr;
  const int* chunk_kb = nullptr;
  const int* row_ptr = nullptr;
  float* Y = nullptr;
  int64_t syt = 0, syi = 0;
  int T = 0;
  int64_t max_chunks = 0;
  bool wide = false;  // the plan is the one of kWideChunkBlocks (its cut rows are a subset of the other plan's)
  bool done = false;
};

// Chunk plan of a packed matrix, as pointers into its aux buffer (null when it is not to be used).
struct ChunkPlan {
  const int* hdr = nullptr;
  const int* chunk_row = nullptr;
  const int* chunk_kb = nullptr;
  const int* chunk_ke = nullptr;
  int64_t max_chunks = 0;  // host-side upper bound of hdr[0]
  // the same rows in chunks of kWideChunkBlocks, for the streaming kernels
  const int* w_hdr = nullptr;
  const int* w_chunk_row = nullptr;
  const int* w_chunk_kb = nullptr;
  const int* w_chunk_ke = nullptr;
  int64_t w_max_chunks = 0;
  int max_row_blocks = 0;  // stored blocks of the fullest block row
  ZeroJob* zero_job = nullptr;  // a side job this launch may take along (decode launches: the first plan's only)
  bool pre_zeroed = false;      // the shared rows of the output have been cleared by an earlier launch ...
  bool zeroed_wide = false;     // ... those of the wide plan only (a subset of the other plan's)
  bool stream_narrow = false;   // the streaming kernels take the chunks of kChunkBlocks too (few token tiles)
  // long rows of a gated product cut into chunks (see StreamArgs)
  const int* slot0 = nullptr;
  const int* slot1 = nullptr;
  const int* chunk0_0 = nullptr;
  const int* chunk0_1 = nullptr;
  float* P0 = nullptr;
  float* P1 = nullptr;
  float* W0 = nullptr;
  float* W1 = nullptr;
  const int* hdr1 = nullptr;  // the second matrix' plan (the first one's is hdr, chunk_*)
  const int* chunk_row1 = nullptr;
  const int* chunk_kb1 = nullptr;
  const int* chunk_ke1 = nullptr;
  int64_t max_chunks1 = 0;
};

// An XCD's L2 (4 MB) keeps the slab of activations of the token tiles it works on only while that slab is a
// few megabytes.  Beyond that every stored block fetches its activation tile from the memory side whatever the
// schedule does, and what is left to save is the weights: with a block row pinned to one XCD they leave the
// memory side once instead of once per XCD (measured on the 405B-class layer, 16384 / 53248 features wide: 3.6
// and 2.2 GB per launch cross the fabric with token tiles pinned, at the 6 - 7.5 TB/s it delivers).
constexpr int64_t kRowPinnedSlabBytes = (int64_t)6 << 20;

template <int B, bool DUAL, int TW, bool CHUNK, int NW = 4, bool LONG = false>
int launch_stream_tw(TileArgs a, const ChunkPlan& plan, int64_t k_features, hipStream_t stream) {
  using C = StreamCfg<B, TW, NW>;
  a.ntt = (a.T + C::TT - 1) / C::TT;
  const int64_t n_rows = CHUNK ? plan.max_chunks : (int64_t)a.nbr + (LONG ? plan.max_chunks + plan.max_chunks1 : 0);
  const int64_t n_items = (int64_t)a.ntt * n_rows;
  if (n_items <= 0) return BLAST_OK;
  if (n_items > INT32_MAX / 2) return BLAST_ERR_INVALID_ARG;
  int shift = -1;
  for (int q = 0; q < 31; ++q)
    if ((1 << q) == a.ntt) shift = q;
  int64_t grid = (n_items + 7) / 8 * 8;
  const int64_t resident = (int64_t)cu_count() * C::WG_PER_CU / 8 * 8;
  if (grid > resident) grid = resident;
  // a workgroup keeps the descriptors of its items one per lane: at most 64 rounds
  if (grid * 64 < n_items) grid = ((n_items + 63) / 64 + 7) / 8 * 8;
  // row-pinned schedule: every token tile of a row on one XCD, side by side
  int row_pinned = 0;
  const int64_t slab = ((int64_t)a.ntt + 7) / 8 * C::TT * k_features * 2;
  if (B == 128 && slab > kRowPinnedSlabBytes && grid == resident && a.ntt <= grid / 8 && (grid / 8) % a.ntt == 0 &&
      n_rows / 8 + 1 <= 64 * ((grid / 8) / a.ntt))
    row_pinned = 1;
  StreamArgs sa{a, (int)n_items, shift, row_pinned, plan.hdr, plan.chunk_row, plan.chunk_kb, plan.chunk_ke};
  if constexpr (LONG) {
    sa.hdr1 = plan.hdr1;
    sa.chunk_row1 = plan.chunk_row1;
    sa.chunk_kb1 = plan.chunk_kb1;
    sa.chunk_ke1 = plan.chunk_ke1;
    sa.slot0 = plan.slot0;
    sa.slot1 = plan.slot1;
    sa.chunk0_0 = plan.chunk0_0;
    sa.chunk0_1 = plan.chunk0_1;
    sa.P0 = plan.P0;
    sa.P1 = plan.P1;
    sa.W0 = plan.W0;
    sa.W1 = plan.W1;
  }
  if (!CHUNK && plan.zero_job && plan.zero_job->hdr && !plan.zero_job->done) {
    // a later chunked product's rows are cleared by this launch on the side
    ZeroJob& z = *plan.zero_job;
    sa.z_hdr = z.hdr;
    sa.z_chunk_row = z.chunk_row;
    sa.z_chunk_kb = z.chunk_kb;
    sa.z_row_ptr = z.row_ptr;
    sa.z_Y = z.Y;
    sa.z_syt = z.syt;
    sa.z_syi = z.syi;
    sa.z_T = z.T;
    z.done = true;
  }
  if (CHUNK && !plan.pre_zeroed) {
    k_zero_shared_rows<B><<<dim3((unsigned)plan.max_chunks, (unsigned)((a.T + 63) / 64)), dim3(256), 0, stream>>>(sa);
    BLAST_LAUNCH_CHECK("k_zero_shared_rows");
  }
  if constexpr (!DUAL && !CHUNK && !LONG) {
    if (a.act >= 0) {  // single matrix with an activation on the output
      static blast::DeviceFlags lds_set_post;
      if (int rc = ensure_lds_limit(reinterpret_cast<const void*>(&k_spmm_stream<B, false, TW, false, true, NW>),
                                    C::LDS_BYTES, lds_set_post))
        return rc;
      k_spmm_stream<B, false, TW, false, true, NW><<<dim3((unsigned)grid), dim3(64 * NW), C::LDS_BYTES, stream>>>(sa);
      BLAST_LAUNCH_CHECK("k_spmm_stream");
      return BLAST_OK;
    }
  }
  static blast::DeviceFlags lds_set;
  if (int rc = ensure_lds_limit(reinterpret_cast<const void*>(&k_spmm_stream<B, DUAL, TW, CHUNK, false, NW, LONG>),
                                C::LDS_BYTES, lds_set))
    return rc;
  k_spmm_stream<B, DUAL, TW, CHUNK, false, NW, LONG><<<dim3((unsigned)grid), dim3(64 * NW), C::LDS_BYTES, stream>>>(sa);
  BLAST_LAUNCH_CHECK("k_spmm_stream");
  if constexpr (LONG) {
    k_long_finish<B><<<dim3((unsigned)((a.nbr + kLongFinishRows - 1) / kLongFinishRows),
                            (unsigned)((a.T + kLongFinishTokens - 1) / kLongFinishTokens)),
                       dim3(256), 0, stream>>>(sa);
    BLAST_LAUNCH_CHECK("k_long_finish");
  }
  return BLAST_OK;
}

template <int B, bool DUAL, bool CHUNK>
int launch_stream_c(const TileArgs& a, const ChunkPlan& plan, int64_t k_features, hipStream_t stream) {
  if constexpr (B == 128) {
    // 256-token x 128-row tiles (eight waves, one workgroup per CU) once every CU gets at least two of them;
    // below that, 128-token tiles in four-wave workgroups, two per CU (8B-shaped down projection at 2048
    // tokens, 256 wide tiles: 24.9 against 28.2 us)
    const int64_t n_rows = CHUNK ? plan.max_chunks : (int64_t)a.nbr;
    const int64_t wide_items = (int64_t)((a.T + 255) / 256) * n_rows;
    if (wide_items >= 2 * (int64_t)cu_count())
      return launch_stream_tw<B, DUAL, 4, CHUNK, 8>(a, plan, k_features, stream);
    return launch_stream_tw<B, DUAL, 2, CHUNK>(a, plan, k_features, stream);
  } else if constexpr (B == 64) {
    // 128-token tiles when 256-token tiles would leave workgroup slots empty
    const int64_t wide_items = (int64_t)((a.T + 255) / 256) * a.nbr;
    if (wide_items < (int64_t)cu_count() * 2)
      return launch_stream_tw<B, DUAL, 2, CHUNK>(a, plan, k_features, stream);
    return launch_stream_tw<B, DUAL, 4, CHUNK>(a, plan, k_features, stream);
  } else {
    return launch_stream_tw<B, DUAL, 4, CHUNK>(a, plan, k_features, stream);
  }
}

template <int B, bool DUAL>
int launch_stream(const TileArgs& a, const ChunkPlan& plan, int64_t k_features, hipStream_t stream) {
  if constexpr (!DUAL) {
    // rows cut into chunks accumulate with fp32 atomics: only for fp32 output without an activation
    if (plan.hdr && plan.stream_narrow && !a.y_bf16 && a.act < 0) {
      ChunkPlan narrow{};
      narrow.hdr = plan.hdr;
      narrow.chunk_row = plan.chunk_row;
      narrow.chunk_kb = plan.chunk_kb;
      narrow.chunk_ke = plan.chunk_ke;
      narrow.max_chunks = plan.max_chunks;
      narrow.max_row_blocks = plan.max_row_blocks;
      narrow.pre_zeroed = plan.pre_zeroed && !plan.zeroed_wide;
      return launch_stream_c<B, false, true>(a, narrow, k_features, stream);
    }
    if (plan.w_hdr && !a.y_bf16 && a.act < 0) {
      ChunkPlan wide{};
      wide.hdr = plan.w_hdr;
      wide.chunk_row = plan.w_chunk_row;
      wide.chunk_kb = plan.w_chunk_kb;
      wide.chunk_ke = plan.w_chunk_ke;
      wide.max_chunks = plan.w_max_chunks;
      wide.max_row_blocks = plan.max_row_blocks;
      wide.pre_zeroed = plan.pre_zeroed;  // either plan's rows cleared covers these
      return launch_stream_c<B, false, true>(a, wide, k_features, stream);
    }
  }
  ChunkPlan side{};  // no chunks; only the side job travels on
  side.zero_job = plan.zero_job;
  return launch_stream_c<B, DUAL, false>(a, side, k_features, stream);
}

template <int B, bool DUAL, int NTT, bool CHUNK, int XSMALL = 0>
int launch_decode_ntt(const TileArgs& a, const ChunkPlan& plan, hipStream_t stream) {
  DecArgs d{};
  d.m0 = a.m0;
  d.m1 = a.m1;
  d.row_order = a.row_order;
  d.X = a.X;
  d.sxt = a.sxt;
  d.Y = a.Y;
  d.syt = a.syt;
  d.syi = a.syi;
  d.y_bf16 = a.y_bf16;
  d.T = a.T;
  d.act = a.act;
  d.hdr = plan.hdr;
  d.chunk_row = plan.chunk_row;
  d.chunk_kb = plan.chunk_kb;
  d.chunk_ke = plan.chunk_ke;
  const int64_t units = (CHUNK ? plan.max_chunks : (int64_t)a.nbr) * (B / 16);
  if (units <= 0) return BLAST_OK;
  const int64_t groups = (a.T + NTT * 16 - 1) / (NTT * 16);
  const int64_t grid = (units + 7) / 8 * 8 * groups;
  if (grid > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  d.n_units = (int)units;
  d.groups = (int)groups;
  int64_t total = grid;
  if (plan.zero_job && plan.zero_job->hdr && !plan.zero_job->wide && plan.zero_job->max_chunks > 0 &&
      grid + plan.zero_job->max_chunks <= INT32_MAX) {
    ZeroJob& z = *plan.zero_job;
    d.main_blocks = (int)grid;
    d.z_blocks = (int)z.max_chunks;
    d.z_hdr = z.hdr;
    d.z_chunk_row = z.chunk_row;
    d.z_chunk_kb = z.chunk_kb;
    d.z_row_ptr = z.row_ptr;
    d.z_Y = z.Y;
    d.z_syt = z.syt;
    d.z_syi = z.syi;
    d.z_T = z.T;
    total = grid + z.max_chunks;
    z.done = true;
  }
  using C = DecCfg<B, DUAL, NTT, XSMALL>;
  if constexpr (!DUAL && !CHUNK) {
    if (a.act >= 0) {  // single matrix with an activation on the output
      static blast::DeviceFlags lds_set_post;
      if (int rc = ensure_lds_limit(reinterpret_cast<const void*>(&k_decode<B, false, NTT, false, XSMALL, true>),
                                    C::LDS_BYTES, lds_set_post))
        return rc;
      k_decode<B, false, NTT, false, XSMALL, true><<<dim3((unsigned)total), dim3(256), C::LDS_BYTES, stream>>>(d);
      BLAST_LAUNCH_CHECK("k_decode");
      return BLAST_OK;
    }
  }
  static blast::DeviceFlags lds_set;
  if (int rc = ensure_lds_limit(reinterpret_cast<const void*>(&k_decode<B, DUAL, NTT, CHUNK, XSMALL>), C::LDS_BYTES,
                                lds_set))
    return rc;
  if (CHUNK && !(plan.pre_zeroed && !plan.zeroed_wide)) {
    StreamArgs sa{a, 0, -1, 0, plan.hdr, plan.chunk_row, plan.chunk_kb, plan.chunk_ke};
    k_zero_shared_rows<B><<<dim3((unsigned)plan.max_chunks, (unsigned)((a.T + 63) / 64)), dim3(256), 0, stream>>>(sa);
    BLAST_LAUNCH_CHECK("k_zero_shared_rows");
  }
  k_decode<B, DUAL, NTT, CHUNK, XSMALL><<<dim3((unsigned)total), dim3(256), C::LDS_BYTES, stream>>>(d);
  BLAST_LAUNCH_CHECK("k_decode");
  return BLAST_OK;
}

template <int B, bool DUAL>
int launch_decode(const TileArgs& a, const ChunkPlan& plan, hipStream_t stream) {
  if constexpr (!DUAL) {
    // rows cut into chunks accumulate with fp32 atomics: only for fp32 output without an activation
    if (plan.hdr && !a.y_bf16 && a.act < 0) {
      if constexpr (B >= 64) {
        if (a.T <= 512 / B) return launch_decode_ntt<B, false, 1, true, 1>(a, plan, stream);
      }
      if constexpr (B == 128) {
        if (a.T <= 8) return launch_decode_ntt<B, false, 1, true, 2>(a, plan, stream);
      }
      if (a.T <= 16) return launch_decode_ntt<B, false, 1, true>(a, plan, stream);
      return launch_decode_ntt<B, false, 2, true>(a, plan, stream);
    }
  }
  ChunkPlan side{};  // no chunks; only the side job travels on
  side.zero_job = plan.zero_job;
  // the smallest activation tile that holds T token rows: 512 / B rows, at b = 128 also twice that
  if constexpr (B >= 64) {
    if (a.T <= 512 / B) return launch_decode_ntt<B, DUAL, 1, false, 1>(a, side, stream);
  }
  if constexpr (B == 128) {
    if (a.T <= 8) return launch_decode_ntt<B, DUAL, 1, false, 2>(a, side, stream);
  }
  if (a.T <= 16) return launch_decode_ntt<B, DUAL, 1, false>(a, side, stream);
  // groups of 32 tokens along gridDim.y (128-wide blocks: with a single activation tile per wave, see DecCfg)
  return launch_decode_ntt<B, DUAL, 2, false>(a, side, stream);
}

// Crossover with the streaming kernel, from token sweeps on the 1B-shaped MLP.  The decode kernel
// re-reads a matrix once per group of 16 or 32 tokens (from cache), the streaming kernel once per 256:
//  - up to 32 tokens the decode kernel always wins;
//  - the single-matrix product stays ahead up to 256 tokens as long as those re-reads are small
//    (the launch is latency bound; 13.8 us against 16.5 us at 256 tokens on a 3.3 MB matrix);
//  - the gated product (two matrices, twice the blocks per workgroup) crosses over at about 64 tokens,
//    unless its fullest block row is so long that the streaming kernel, which walks a whole row of the
//    gated product in one workgroup (the activation needs complete sums, so the row cannot be cut), would
//    spend longer on that one row than the decode kernel spends on everything (it deals a row's blocks to
//    the four waves of b/16 workgroups).  Measured on the 405B-class layer with the Zipf mask (fullest joint
//    row 256 blocks of 128 x 128): 183 us in the streaming kernel at 33-64 tokens, 0.7 us per block of that
//    row; the decode kernel takes about 42 us per group of 32 tokens there (174 MB of blocks per group):
//    84-93 us at 33-64 tokens, 120-127 us at 65-96, 168 us at 128.
constexpr int kDecodeAlwaysTokens = 32;
constexpr int kDecodeMaxTokens = 256;
constexpr int64_t kDecodeMaxRereadBytes = (int64_t)64 << 20;

template <bool DUAL>
bool decode_applies(int b, const TileArgs& a, int64_t nnz, int64_t max_row_blocks) {
  if (a.T <= kDecodeAlwaysTokens) return true;
  if (a.T > kDecodeMaxTokens) return false;
  const int64_t group = 32;  // tokens per unit of the decode kernel beyond 16 tokens
  const int64_t groups = (a.T + group - 1) / group;
  const int64_t reread = nnz * b * b * 2 * groups;
  if (DUAL) {
    // small products are a chain of latencies either way; the decode kernel's chain is the shorter one for up
    // to 64 tokens (1B / 3B shapes, b = 64: 17-19 us per MLP pass against 21-22 at 33-64 tokens; 8B shape,
    // b = 128: 25-28 against 29-32; from 96 tokens on the streaming kernel is ahead)
    if (groups <= 2 && reread <= kDecodeMaxRereadBytes) return true;
    if (max_row_blocks <= 0 || groups > 8) return false;
    const double row_us = (double)max_row_blocks * 0.7 * ((double)b * b / (128.0 * 128.0));  // streaming kernel, fullest row
    const double all_us = (double)reread / 4.1e6;                                            // decode kernel, whole product
    // only where that row is long against the fixed latencies of a launch (tens of microseconds)
    return row_us >= 30.0 && all_us < row_us;
  }
  return reread <= kDecodeMaxRereadBytes;
}

template <bool DUAL>
int dispatch_tile(int b, const TileArgs& a, int64_t nnz, hipStream_t stream, const ChunkPlan& plan = ChunkPlan{}) {
  // the streaming kernel addresses activations with 32-bit byte offsets inside one column block
  const bool small_x = (int64_t)a.T * a.sxt * 2 < ((int64_t)1 << 32);
  if (a.x_vec && a.T > 0 && small_x && decode_applies<DUAL>(b, a, nnz, plan.max_row_blocks)) {
    // The decode kernel already spreads a block row over b/16 workgroups of four waves each, so a row of n
    // blocks is n/4 block steps deep.  Chunks (a zero-fill launch plus atomics, about 8 us on the 405B-class
    // gate matrix) only pay when that depth exceeds four times the average load of a workgroup slot
    // (measured there: fullest row 128 blocks, 20.8 us without chunks against 28.8 us with; 416 blocks, 42.0
    // against 23.3).
    ChunkPlan dplan = plan;
    if (dplan.hdr) {
      double ref = (double)nnz * (b / 16) / (4.0 * 2.0 * cu_count());
      if (ref < blast::kChunkBlocks) ref = blast::kChunkBlocks;
      if ((double)dplan.max_row_blocks / 4.0 <= 4.0 * ref) {
        dplan = ChunkPlan{};
        dplan.zero_job = plan.zero_job;
      }
    }
    switch (b) {
      case 32: return launch_decode<32, DUAL>(a, dplan, stream);
      case 64: return launch_decode<64, DUAL>(a, dplan, stream);
      case 128: return launch_decode<128, DUAL>(a, dplan, stream);
      default: break;
    }
  }
  if (a.x_vec && a.T > 0 && !small_x && b >= 32) {
    // More tokens than 32-bit offsets reach: the same kernels over token ranges that each fit (whole
    // 256-token tiles, so no range ends inside a tile of the next one).
    const int64_t range = (((int64_t)1 << 32) - 1) / (a.sxt * 2) / 256 * 256;
    if (range >= 256) {
      for (int64_t t0 = 0; t0 < a.T; t0 += range) {
        TileArgs part = a;
        part.T = (int)((a.T - t0 < range) ? a.T - t0 : range);
        part.X = a.X + t0 * a.sxt;
        part.Y = static_cast<char*>(a.Y) + t0 * a.syt * (a.y_bf16 ? 2 : 4);
        if (int rc = dispatch_tile<DUAL>(b, part, nnz, stream, plan)) return rc;
      }
      return BLAST_OK;
    }
  }
  if (a.x_vec && a.T > 0 && small_x) {
    switch (b) {
      case 32: return launch_stream<32, DUAL>(a, plan, a.kdim, stream);
      case 64: return launch_stream<64, DUAL>(a, plan, a.kdim, stream);
      case 128: return launch_stream<128, DUAL>(a, plan, a.kdim, stream);
      default: break;
    }
  }
  if (b == 16 && (a.x_vec || a.x_grp16) && a.T > 0) return launch_b16<DUAL>(a, nnz, stream);
  switch (b) {
    case 16: return launch_tile<16, DUAL>(a, stream);
    case 32: return launch_tile<32, DUAL>(a, stream);
    case 64: return launch_tile<64, DUAL>(a, stream);
    case 128: return launch_tile<128, DUAL>(a, stream);
    default: return BLAST_ERR_UNSUPPORTED_BLOCK;
  }
}

int check_view(const blast_bsr_view* v) {
  if (!v) return BLAST_ERR_INVALID_ARG;
  if (v->rows < 0 || v->cols < 0 || v->nnz < 0) return BLAST_ERR_INVALID_ARG;
  if (!blast::supported_block(v->b)) return BLAST_ERR_UNSUPPORTED_BLOCK;
  if (v->rows % v->b || v->cols % v->b) return BLAST_ERR_SHAPE;
  if (v->rows / v->b > INT32_MAX / 2 || v->cols / v->b > INT32_MAX / 2 || v->nnz > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  if (!v->row_ptr) return BLAST_ERR_INVALID_ARG;
  if (v->nnz > 0 && (!v->col_idx || !v->vals || !blast::aligned(v->vals, 16))) return BLAST_ERR_INVALID_ARG;
  return BLAST_OK;
}

int check_dense(const void* p, int64_t ld, int32_t layout, int64_t feat, int64_t T) {
  if (layout != BLAST_TOKEN_MAJOR && layout != BLAST_FEATURE_MAJOR) return BLAST_ERR_INVALID_ARG;
  if (T > 0 && feat > 0) {
    if (!p) return BLAST_ERR_INVALID_ARG;
    if (ld < (layout == BLAST_TOKEN_MAJOR ? feat : T)) return BLAST_ERR_INVALID_ARG;
  }
  return BLAST_OK;
}

void set_x(TileArgs& a, const uint16_t* X, int64_t ldx, int32_t layout) {
  a.X = X;
  if (layout == BLAST_TOKEN_MAJOR) {
    a.sxt = ldx;
    a.sxk = 1;
    a.x_vec = (ldx % 8 == 0 && blast::aligned(X, 16)) ? 1 : 0;
  } else {
    a.sxt = 1;
    a.sxk = ldx;
    a.x_vec = 0;
  }
}

void set_y(TileArgs& a, void* Y, int64_t ldy, int32_t layout, int32_t y_dtype) {
  a.Y = Y;
  a.y_bf16 = (y_dtype == BLAST_BF16) ? 1 : 0;
  a.y_fast = 0;
  if (layout == BLAST_TOKEN_MAJOR) {
    a.syt = ldy;
    a.syi = 1;
    a.y_fast = ((int64_t)256 * ldy * 4 + ldy * 4 < ((int64_t)1 << 31)) ? 1 : 0;
  } else {
    a.syt = 1;
    a.syi = ldy;
  }
}

MatDev mat_of(const blast_bsr_view* v) { return MatDev{v->row_ptr, v->col_idx, v->vals}; }

// The chunk plan costs a zero-fill launch and fp32 atomics on the split rows (measured: about 9 us on
// the 1B-shaped down projection, where it does not pay).  It is used only when the fullest block row,
// taken as one work item, would outlast four times the average load of a workgroup slot (and four
// chunks): then that row is the critical path of the launch by a wide margin.
ChunkPlan plan_of(const blast_bsr_view* v, int64_t T) {
  ChunkPlan p;
  if (!v->aux || v->max_row_blocks <= blast::kChunkBlocks) return p;
  const int64_t nbr = v->rows / v->b, nbc = v->cols / v->b;
  const int64_t tiles = (T + 255) / 256;
  double ref = (double)v->nnz * (double)tiles / (2.0 * cu_count());
  if (ref < blast::kChunkBlocks) ref = blast::kChunkBlocks;
  if ((double)v->max_row_blocks <= 4.0 * ref) return p;
  const blast::AuxLayout L = blast::aux_layout(nbr, nbc, v->nnz);
  const char* ab = static_cast<const char*>(v->aux);
  p.hdr = reinterpret_cast<const int*>(ab + L.hdr_off);
  p.chunk_row = reinterpret_cast<const int*>(ab + L.chunk_row_off);
  p.chunk_kb = reinterpret_cast<const int*>(ab + L.chunk_kb_off);
  p.chunk_ke = reinterpret_cast<const int*>(ab + L.chunk_ke_off);
  p.max_chunks = nbr + v->nnz / blast::kChunkBlocks;
  if (v->max_row_blocks > blast::kWideChunkBlocks) {  // otherwise every row is one wide chunk: no plan needed
    p.w_hdr = reinterpret_cast<const int*>(ab + L.whdr_off);
    p.w_chunk_row = reinterpret_cast<const int*>(ab + L.wchunk_row_off);
    p.w_chunk_kb = reinterpret_cast<const int*>(ab + L.wchunk_kb_off);
    p.w_chunk_ke = reinterpret_cast<const int*>(ab + L.wchunk_ke_off);
    p.w_max_chunks = nbr + v->nnz / blast::kWideChunkBlocks;
  }
  p.max_row_blocks = v->max_row_blocks;
  {
    // blocks per CU with 256-token tiles: below half a wide chunk, wide chunks are too coarse to balance
    const double per_cu = (double)v->nnz * (double)tiles / cu_count();
    p.stream_narrow = per_cu < blast::kWideChunkBlocks / 2;
  }
  return p;
}

}  // namespace

extern "C" int blast_bsr_spmm_workspace(const blast_bsr_view* W, int64_t T, size_t* ws_bytes) {
  if (int rc = check_view(W)) return rc;
  if (T < 0 || !ws_bytes) return BLAST_ERR_INVALID_ARG;
  // 16-wide blocks at many tokens: room for the activations regrouped by block column (optional: without it the
  // product reads the caller's tensor as it lies)
  *ws_bytes = (W->b == 16 && T >= kGroup16MinTokens) ? group16_bytes(W->cols, T) : 0;
  return BLAST_OK;
}

extern "C" int blast_bsr_spmm(const blast_bsr_view* W, const uint16_t* X, int64_t ldx, int32_t x_layout, int64_t T,
                              void* Y, int64_t ldy, int32_t y_dtype, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (int rc = check_view(W)) return rc;
  if (T < 0 || T > INT32_MAX / 2) return BLAST_ERR_INVALID_ARG;
  if (y_dtype != BLAST_F32 && y_dtype != BLAST_BF16) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_dense(X, ldx, x_layout, W->cols, T)) return rc;
  if (int rc = check_dense(Y, ldy, x_layout, W->rows, T)) return rc;
  if (T == 0 || W->rows == 0) return BLAST_OK;
  TileArgs a{};
  a.m0 = mat_of(W);
  a.row_order = W->row_order;
  set_x(a, X, ldx, x_layout);
  set_y(a, Y, ldy, x_layout, y_dtype);
  a.T = (int)T;
  a.nbr = (int)(W->rows / W->b);
  a.kdim = W->cols;
  a.act = -1;
  if (group16_applies(W->b, x_layout, X, ldx, T) && ws && blast::aligned(ws, 16) &&
      ws_bytes >= group16_bytes(W->cols, T)) {
    uint16_t* Xg = static_cast<uint16_t*>(ws);
    if (int rc = enqueue_group16(X, ldx, T, W->cols, Xg, stream)) return rc;
    a.X = Xg;
    a.x_grp16 = 1;
  }
  return dispatch_tile<false>(W->b, a, W->nnz, stream, plan_of(W, T));
}

namespace {

// H in bf16, token-major [T][I]; then the publication slots of the single-launch form (one 64-bit word
// per 16 rows of H) and the control block of the hand-over: signature, epoch, status word, arrival counters
size_t mlp_h_bytes(int64_t I, int64_t T) { return blast::align_up((size_t)T * (size_t)I * 2, 256); }
size_t mlp_slot_bytes(int64_t I) { return blast::align_up((size_t)(I / 16) * 8, 256); }
size_t mlp_workspace_bytes(int64_t I, int64_t T) { return mlp_h_bytes(I, T) + mlp_slot_bytes(I) + kCtlBytes; }
constexpr size_t kCtlStatusOffset = 16;  // byte offset of the status word inside the control block

// ---- long rows of a gated product ---------------------------------------------------------------------
// The gated product cannot cut a block row (the activation needs complete sums), so at a few hundred tokens
// - one to four token tiles per row - the workgroup that walks the fullest joint row alone sets the time of
// the launch when the row lengths are skewed.  There the rows that the first chunk plan of either matrix cuts
// (more than kChunkBlocks stored blocks) are taken in chunks after all: the launch stores the fp32 sums of
// every chunk, and of the side of such a row that is not cut, in scratch slices of their own, and a small
// launch after it adds the slices of a row in plan order, applies the activation and writes those rows of H
// (see StreamArgs; no atomics, the result does not depend on the schedule).  Measured on the 405B-class layer
// with the Zipf mask (fullest rows: all 128 blocks of gate or of up, 133 joint), gate/up product in
// microseconds without / with: 128 tokens 160 / 90, 256: 199 / 125, 384: 264 / 187, 512: 275 / 198,
// 640: 317 / 272, 768: 325 / 296; at 1024 tokens 300 / 349 (the chunks' fp32 slices are written and read
// again, 64 us of the launch at 2048 tokens, and the finishing launch reads them at 2-2.5 TB/s only).
constexpr int kLongMinTokens = 64;  // up to here the decode kernels are at least as fast (81 against 88 us at 64)
constexpr int kLongWideTokens = 384;  // 512 tokens: 198 us with 256-token tiles (row-pinned schedule), 218 with 128-token tiles

// upper bound of the number of rows with more than kChunkBlocks stored blocks (0: none, or no plan at hand)
int64_t long_slots(const blast_bsr_view* v) {
  if (!v->aux || v->max_row_blocks <= blast::kChunkBlocks) return 0;
  const int64_t nbr = v->rows / v->b, by_blocks = v->nnz / (blast::kChunkBlocks + 1);
  return by_blocks < nbr ? by_blocks : nbr;
}

// upper bound of the number of chunks of the cut rows: sum of ceil(len / chunk) over those rows, at most
int64_t long_max_chunks(const blast_bsr_view* v) {
  const int64_t slots = long_slots(v);
  return slots ? v->nnz / blast::kChunkBlocks + slots : 0;
}

// fp32 scratch of one matrix in the long-row path, [chunks + slots][T][b]: a slice per chunk of its cut rows,
// and a slice per cut row for the whole side of that row in the other matrix
size_t long_scratch_bytes(const blast_bsr_view* v, int64_t T) {
  return blast::align_up((size_t)(long_max_chunks(v) + long_slots(v)) * (size_t)v->b * (size_t)T * 4, 256);
}

// Where it pays (host-side estimate from the counts the views carry).
bool long_rows_pay(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, int64_t T) {
  if (!Wup || Wgate->b < 32) return false;
  if (long_slots(Wgate) + long_slots(Wup) == 0) return false;
  if (T <= kLongMinTokens) return false;
  // the fullest row of either matrix (a lower bound of the fullest joint row) against the blocks a CU gets when
  // the product is dealt evenly, in 256-token tiles
  const int64_t tiles = (T + 255) / 256;
  const double avg = (double)(Wgate->nnz + Wup->nnz) * (double)tiles / cu_count();
  const int64_t fullest = Wgate->max_row_blocks > Wup->max_row_blocks ? Wgate->max_row_blocks : Wup->max_row_blocks;
  return fullest >= 2 * blast::kChunkBlocks && (double)fullest > 1.75 * avg;
}

// scratch of the long-row path behind the MLP workspace proper (0 where the path is not taken)
size_t mlp_long_bytes(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, int64_t T) {
  if (!Wup || !long_rows_pay(Wgate, Wup, T)) return 0;
  return long_scratch_bytes(Wgate, T) + long_scratch_bytes(Wup, T);
}

// Knobs of the hand-over inside the single-launch form; the defaults are what every ordinary call uses.
struct HandoverKnobs {
  int max_spins = kDecMaxSpins;
  int withhold = 0;
};

}  // namespace

extern "C" int blast_sparse_mlp_workspace(const blast_bsr_view* Wgate, const blast_bsr_view* Wup,
                                          const blast_bsr_view* Wdown, int64_t T, size_t* ws_bytes) {
  if (int rc = check_view(Wgate)) return rc;
  if (int rc = check_view(Wup)) return rc;
  if (int rc = check_view(Wdown)) return rc;
  if (T < 0 || !ws_bytes) return BLAST_ERR_INVALID_ARG;
  *ws_bytes = mlp_workspace_bytes(Wgate->rows, T) + mlp_long_bytes(Wgate, Wup, T) +
              ((Wgate->b == 16 && T >= kGroup16MinTokens) ? group16_bytes(Wgate->cols, T) : 0);
  return BLAST_OK;
}

extern "C" int blast_sparse_mlp2_workspace(const blast_bsr_view* W1, const blast_bsr_view* W2, int64_t T,
                                           size_t* ws_bytes) {
  if (int rc = check_view(W1)) return rc;
  if (int rc = check_view(W2)) return rc;
  if (T < 0 || !ws_bytes) return BLAST_ERR_INVALID_ARG;
  *ws_bytes = mlp_workspace_bytes(W1->rows, T) +
              ((W1->b == 16 && T >= kGroup16MinTokens) ? group16_bytes(W1->cols, T) : 0);
  return BLAST_OK;
}

namespace {

int check_mlp(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown, const uint16_t* X,
              int64_t ldx, int32_t x_layout, int64_t T, int32_t act, void* Y, int64_t ldy, int32_t y_dtype) {
  if (int rc = check_view(Wgate)) return rc;
  if (Wup)
    if (int rc = check_view(Wup)) return rc;
  if (int rc = check_view(Wdown)) return rc;
  const int64_t I = Wgate->rows, E = Wgate->cols;
  const int32_t b = Wgate->b;
  if (Wup && (Wup->rows != I || Wup->cols != E || Wup->b != b)) return BLAST_ERR_SHAPE;
  if (Wdown->rows != E || Wdown->cols != I || Wdown->b != b) return BLAST_ERR_SHAPE;
  if (T < 0 || T > INT32_MAX / 2) return BLAST_ERR_INVALID_ARG;
  if (act != BLAST_ACT_SILU && act != BLAST_ACT_GELU && act != BLAST_ACT_RELU) return BLAST_ERR_INVALID_ARG;
  if (y_dtype != BLAST_F32 && y_dtype != BLAST_BF16) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_dense(X, ldx, x_layout, E, T)) return rc;
  if (int rc = check_dense(Y, ldy, x_layout, E, T)) return rc;
  return BLAST_OK;
}

static_assert(kLongChunk == blast::kChunkBlocks, "the long-row launch works from the first chunk plan");

struct LongScratch {
  float* S0 = nullptr;  // long_scratch_bytes() of the first matrix: its chunk slices, then its rows' other sides
  float* S1 = nullptr;  // of the second
};

template <int B>
int enqueue_gated_long(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const TileArgs& g,
                       const LongScratch& ls, ZeroJob* side_job, hipStream_t stream) {
  ChunkPlan p{};
  p.zero_job = side_job;
  const blast_bsr_view* mats[2] = {Wgate, Wup};
  for (int m = 0; m < 2; ++m) {
    const blast_bsr_view* v = mats[m];
    const int64_t slots = long_slots(v);
    if (slots == 0) continue;
    const blast::AuxLayout L = blast::aux_layout(v->rows / v->b, v->cols / v->b, v->nnz);
    const char* ab = static_cast<const char*>(v->aux);
    const int* row_slot = reinterpret_cast<const int*>(ab + L.row_slot_off);
    const int* row_chunk0 = reinterpret_cast<const int*>(ab + L.row_chunk0_off);
    const int* hdr = reinterpret_cast<const int*>(ab + L.hdr_off) + 3;  // the chunks of the cut rows head the plan
    const int* chunk_row = reinterpret_cast<const int*>(ab + L.chunk_row_off);
    const int* chunk_kb = reinterpret_cast<const int*>(ab + L.chunk_kb_off);
    const int* chunk_ke = reinterpret_cast<const int*>(ab + L.chunk_ke_off);
    const int64_t most = long_max_chunks(v);
    if (m == 0) {
      p.hdr = hdr;
      p.chunk_row = chunk_row;
      p.chunk_kb = chunk_kb;
      p.chunk_ke = chunk_ke;
      p.max_chunks = most;
      p.slot0 = row_slot;
      p.chunk0_0 = row_chunk0;
      p.P0 = ls.S0;
      p.W0 = ls.S0 + most * g.T * B;
    } else {
      p.hdr1 = hdr;
      p.chunk_row1 = chunk_row;
      p.chunk_kb1 = chunk_kb;
      p.chunk_ke1 = chunk_ke;
      p.max_chunks1 = most;
      p.slot1 = row_slot;
      p.chunk0_1 = row_chunk0;
      p.P1 = ls.S1;
      p.W1 = ls.S1 + most * g.T * B;
    }
  }
  // 128-token tiles (more and shorter items) up to kLongWideTokens, the eight-wave 256-token tile beyond
  if constexpr (B == 128) {
    if (g.T > kLongWideTokens) return launch_stream_tw<B, true, 4, false, 8, true>(g, p, g.kdim, stream);
  }
  if constexpr (B >= 64) {
    return launch_stream_tw<B, true, 2, false, 4, true>(g, p, g.kdim, stream);
  } else {
    return launch_stream_tw<B, true, 4, false, 4, true>(g, p, g.kdim, stream);
  }
}

// H = act(Wgate X) (.) (Wup X), or H = act(Wgate X) when Wup is null; bf16, strides given by (h_layout, ldh).
// `ls` (may be null): scratch for the long rows, long_scratch_bytes() per matrix.
int enqueue_gated(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const uint16_t* X, int64_t ldx,
                  int32_t x_layout, int64_t T, int32_t act, uint16_t* H, int64_t ldh, int32_t h_layout,
                  hipStream_t stream, ZeroJob* side_job = nullptr, const LongScratch* ls = nullptr,
                  const uint16_t* Xg16 = nullptr, bool h_grp16 = false) {
  ChunkPlan side{};
  side.zero_job = side_job;
  // upper bound of the fullest joint row (exact when the same row is the fullest of both matrices)
  side.max_row_blocks = Wgate->max_row_blocks + (Wup ? Wup->max_row_blocks : 0);
  TileArgs g{};
  g.m0 = mat_of(Wgate);
  if (Wup) g.m1 = mat_of(Wup);
  g.row_order = Wgate->row_order;
  set_x(g, X, ldx, x_layout);
  set_y(g, H, ldh, h_layout, BLAST_BF16);
  g.T = (int)T;
  g.nbr = (int)(Wgate->rows / Wgate->b);
  g.kdim = Wgate->cols;
  g.act = act;
  if (Xg16) {  // 16-wide blocks: X regrouped by block column, H kept that way
    g.X = Xg16;
    g.x_grp16 = 1;
  }
  g.y_grp16 = h_grp16 ? 1 : 0;
  if (!Wup) return dispatch_tile<false>(Wgate->b, g, Wgate->nnz, stream, side);
  if (ls && g.x_vec && T > 0 && (int64_t)T * g.sxt * 2 < ((int64_t)1 << 32) && long_rows_pay(Wgate, Wup, T)) {
    switch (Wgate->b) {
      case 32: return enqueue_gated_long<32>(Wgate, Wup, g, *ls, side_job, stream);
      case 64: return enqueue_gated_long<64>(Wgate, Wup, g, *ls, side_job, stream);
      case 128: return enqueue_gated_long<128>(Wgate, Wup, g, *ls, side_job, stream);
      default: break;
    }
  }
  return dispatch_tile<true>(Wgate->b, g, Wgate->nnz + Wup->nnz, stream, side);
}

// Every single-launch MLP call gets its own token (never 0), which the kernel mixes with an epoch it keeps in
// the workspace: a slot says "published" only when it holds the token of the running launch, so the slots
// need no clearing between launches and no initialisation (a stale or random word equals a fresh 64-bit
// token with probability 2^-64), and a call recorded into a graph differs from replay to replay in the epoch.
unsigned long long next_token() {
  static std::atomic<unsigned long long> counter{0x243F6A8885A308D3ull};
  return counter.fetch_add(0x9E3779B97F4A7C15ull) | 1ull;
}

template <int B, int NTT, int XSMALL, bool GATED>
int launch_mlp_decode(const DecArgs& p, const DecArgs& c, hipStream_t stream) {
  using CP = DecCfg<B, GATED, NTT, XSMALL, true>;  // the producer's footprint is never below the consumer's
  static blast::DeviceFlags lds_set;
  if (int rc = ensure_lds_limit(reinterpret_cast<const void*>(&k_mlp_decode<B, NTT, XSMALL, GATED>), CP::LDS_BYTES,
                                lds_set))
    return rc;
  const int64_t grid = (int64_t)p.n_units + c.n_units;
  if (grid > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  k_mlp_decode<B, NTT, XSMALL, GATED><<<dim3((unsigned)grid), dim3(256), CP::LDS_BYTES, stream>>>(p, c);
  BLAST_LAUNCH_CHECK("k_mlp_decode");
  return BLAST_OK;
}

// The single-launch form of the MLP for one token tile.  Applies when both products would take the
// decode kernel's fast path anyway and no row of Wdown is cut into chunks.
template <int B, bool GATED>
int enqueue_mlp_decode(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown,
                       const TileArgs& g, const TileArgs& d, uint16_t* H, unsigned long long* slots,
                       unsigned long long* ctl, const HandoverKnobs& knobs, hipStream_t stream) {
  DecArgs p{}, c{};
  p.m0 = g.m0;
  p.m1 = g.m1;
  p.row_order = g.row_order;
  p.X = g.X;
  p.sxt = g.sxt;
  p.Y = H;
  p.syt = Wgate->rows;
  p.syi = 1;
  p.y_bf16 = 1;
  p.T = g.T;
  p.act = g.act;
  p.n_units = (int)(Wgate->rows / B) * (B / 16);
  p.slots = slots;
  p.token = next_token();
  p.ctl = ctl;
  p.max_spins = knobs.max_spins;
  p.withhold = knobs.withhold;
  p.sync_err = reinterpret_cast<int*>(reinterpret_cast<char*>(ctl) + kCtlStatusOffset);
  c.m0 = d.m0;
  c.row_order = d.row_order;
  c.X = H;
  c.sxt = Wgate->rows;
  c.Y = d.Y;
  c.syt = d.syt;
  c.syi = d.syi;
  c.y_bf16 = d.y_bf16;
  c.T = d.T;
  c.act = -1;
  c.n_units = (int)(Wdown->rows / B) * (B / 16);
  c.slots = slots;
  c.token = p.token;
  c.ctl = ctl;
  c.max_spins = knobs.max_spins;
  c.withhold = knobs.withhold;
  c.sync_err = p.sync_err;
  p.groups = c.groups = 1;
  p.total_waves = c.total_waves = (p.n_units + c.n_units) * 4;
  {  // a launch adds 2^shift to each of the 64 arrival counters: the smallest power of two >= the largest group
    const int largest = (p.total_waves + kCtlGroups - 1) / kCtlGroups;
    int shift = 0;
    while ((1 << shift) < largest) ++shift;
    p.ctl_shift = c.ctl_shift = shift;
  }
  (void)Wup;
  if constexpr (B >= 64) {
    if (g.T <= 512 / B) return launch_mlp_decode<B, 1, true, GATED>(p, c, stream);
  }
  if (g.T <= 16) return launch_mlp_decode<B, 1, false, GATED>(p, c, stream);
  if (g.T <= 32) return launch_mlp_decode<B, 2, false, GATED>(p, c, stream);
  if constexpr (B == 64) return launch_mlp_decode<B, 4, false, GATED>(p, c, stream);
  return BLAST_ERR_INVALID_ARG;
}

int enqueue_mlp(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown,
                const uint16_t* X, int64_t ldx, int32_t x_layout, int64_t T, int32_t act, void* Y, int64_t ldy,
                int32_t y_dtype, void* ws, size_t ws_bytes, hipStream_t stream, void* const* events,
                const HandoverKnobs& knobs = HandoverKnobs{}) {
  if (int rc = check_mlp(Wgate, Wup, Wdown, X, ldx, x_layout, T, act, Y, ldy, y_dtype)) return rc;
  const int64_t I = Wgate->rows, E = Wgate->cols;
  const int32_t b = Wgate->b;
  if (T == 0 || E == 0) return BLAST_OK;
  const size_t need = mlp_workspace_bytes(I, T);
  if (need > 0 && (!ws || ws_bytes < need || !blast::aligned(ws, 256))) return BLAST_ERR_WORKSPACE;
  uint16_t* H = static_cast<uint16_t*>(ws);

  if (events) BLAST_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(events[0]), stream));
  const int64_t one_tile = (b == 64) ? 64 : 32;  // 64-token units exist for 64-wide blocks only
  // One launch saves a dispatch gap and the second kernel's ramp, a few microseconds; its smaller copy rings
  // (producers and consumers share the CUs) cost bandwidth.  Measured with uniform masks and cold weights:
  // about even up to 18 MB of stored blocks, 63 us against 55 us on the 405B-class layer (262 MB).
  const int64_t stored_bytes = (Wgate->nnz + (Wup ? Wup->nnz : 0) + Wdown->nnz) * (int64_t)b * b * 2;
  const bool fused_pays = stored_bytes <= ((int64_t)32 << 20);
  // (b >= 64: a token's slice of one block column of H then fills whole 128-byte lines, so a line is never
  // read by one consumer while the producers of a neighbouring column are still writing the rest of it)
  if (I > 0 && T <= one_tile && (b == 64 || b == 128) && fused_pays && (I / 16 + E / 16) * 4 < INT32_MAX / 2 &&
      x_layout == BLAST_TOKEN_MAJOR && ldx % 8 == 0 &&
      blast::aligned(X, 16) && T * ldx * 2 < ((int64_t)1 << 32) && !plan_of(Wdown, T).hdr) {
    TileArgs g{}, d{};
    g.m0 = mat_of(Wgate);
    if (Wup) g.m1 = mat_of(Wup);
    g.row_order = Wgate->row_order;
    set_x(g, X, ldx, x_layout);
    g.T = (int)T;
    g.act = act;
    d.m0 = mat_of(Wdown);
    d.row_order = Wdown->row_order;
    set_y(d, Y, ldy, x_layout, y_dtype);
    d.T = (int)T;
    char* wsb = static_cast<char*>(ws);
    unsigned long long* slots = reinterpret_cast<unsigned long long*>(wsb + mlp_h_bytes(I, T));
    unsigned long long* ctl = reinterpret_cast<unsigned long long*>(wsb + mlp_h_bytes(I, T) + mlp_slot_bytes(I));
    // one kernel does both phases: events[1] falls before it
    if (events) BLAST_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(events[1]), stream));
    int rc;
    if (Wup) {
      rc = (b == 64) ? enqueue_mlp_decode<64, true>(Wgate, Wup, Wdown, g, d, H, slots, ctl, knobs, stream)
                     : enqueue_mlp_decode<128, true>(Wgate, Wup, Wdown, g, d, H, slots, ctl, knobs, stream);
    } else {
      rc = (b == 64) ? enqueue_mlp_decode<64, false>(Wgate, Wup, Wdown, g, d, H, slots, ctl, knobs, stream)
                     : enqueue_mlp_decode<128, false>(Wgate, Wup, Wdown, g, d, H, slots, ctl, knobs, stream);
    }
    if (rc) return rc;
    if (events) BLAST_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(events[2]), stream));
    return BLAST_OK;
  }
  TileArgs d{};
  d.m0 = mat_of(Wdown);
  d.row_order = Wdown->row_order;
  set_x(d, H, I, BLAST_TOKEN_MAJOR);
  set_y(d, Y, ldy, x_layout, y_dtype);
  d.T = (int)T;
  d.nbr = (int)(E / b);
  d.kdim = I;
  d.act = -1;
  ChunkPlan dplan = plan_of(Wdown, T);
  // At decode token counts the rows of Y that the chunked second product accumulates into are cleared on
  // the side by the first product's launch (extra workgroups of the same kernel) instead of by a launch
  // of their own between the two products.
  // Beyond them the streaming kernels do the same, with the rows of the plan that the second product will take
  // (the first plan's rows include the other's, so clearing those serves either).
  ZeroJob zj{};
  if (dplan.hdr && y_dtype == BLAST_F32 && (T <= kDecodeMaxTokens || dplan.stream_narrow) && I > 0) {
    zj.hdr = dplan.hdr;
    zj.chunk_row = dplan.chunk_row;
    zj.chunk_kb = dplan.chunk_kb;
    zj.max_chunks = dplan.max_chunks;
  } else if (dplan.w_hdr && y_dtype == BLAST_F32 && T > kDecodeMaxTokens && I > 0) {
    zj.hdr = dplan.w_hdr;
    zj.chunk_row = dplan.w_chunk_row;
    zj.chunk_kb = dplan.w_chunk_kb;
    zj.max_chunks = dplan.w_max_chunks;
    zj.wide = true;
  }
  if (zj.hdr) {
    zj.row_ptr = Wdown->row_ptr;
    zj.Y = static_cast<float*>(Y);
    zj.syt = d.syt;
    zj.syi = d.syi;
    zj.T = (int)T;
  }
  if (I > 0) {
    // room behind the workspace proper (blast_sparse_mlp_workspace asks for it where it pays): the long rows
    // of the gated product are cut into chunks
    LongScratch ls{};
    const size_t extra = Wup ? mlp_long_bytes(Wgate, Wup, T) : 0;
    const bool have_ls = extra > 0 && ws_bytes >= need + extra;
    if (have_ls) {
      ls.S0 = reinterpret_cast<float*>(static_cast<char*>(ws) + need);
      ls.S1 = reinterpret_cast<float*>(static_cast<char*>(ws) + need + long_scratch_bytes(Wgate, T));
    }
    // 16-wide blocks at many tokens: X is regrouped by block column behind the workspace proper (where the
    // caller left room for it), and H is written and read in the same form
    const uint16_t* Xg16 = nullptr;
    if (group16_applies(b, x_layout, X, ldx, T) && ws_bytes >= need + extra + group16_bytes(E, T)) {
      uint16_t* xg = reinterpret_cast<uint16_t*>(static_cast<char*>(ws) + need + extra);
      if (int rc = enqueue_group16(X, ldx, T, E, xg, stream)) return rc;
      Xg16 = xg;
      d.x_grp16 = 1;
    }
    if (int rc = enqueue_gated(Wgate, Wup, X, ldx, x_layout, T, act, H, I, BLAST_TOKEN_MAJOR, stream,
                               zj.hdr ? &zj : nullptr, have_ls ? &ls : nullptr, Xg16, Xg16 != nullptr))
      return rc;
  }
  if (events) BLAST_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(events[1]), stream));
  dplan.pre_zeroed = zj.done;
  dplan.zeroed_wide = zj.wide;
  if (int rc = dispatch_tile<false>(b, d, Wdown->nnz, stream, dplan)) return rc;
  if (events) BLAST_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(events[2]), stream));
  return BLAST_OK;
}

}  // namespace

extern "C" int blast_sparse_mlp(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown,
                                const uint16_t* X, int64_t ldx, int32_t x_layout, int64_t T, int32_t act, void* Y,
                                int64_t ldy, int32_t y_dtype, void* ws, size_t ws_bytes, void* stream_) {
  if (!Wup) return BLAST_ERR_INVALID_ARG;
  return enqueue_mlp(Wgate, Wup, Wdown, X, ldx, x_layout, T, act, Y, ldy, y_dtype, ws, ws_bytes,
                     static_cast<hipStream_t>(stream_), nullptr);
}

// ---- entry point for callers that cannot allocate ---------------------------------------------------
// Same work as blast_sparse_mlp, with the scratch (H, the publication slots of the single-launch form and
// the status words) in a device array that belongs to the library instead of a caller's workspace.
constexpr size_t kStaticScratchBytes = BLAST_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// Device address of `scratch` on the current device, looked up once per device (the array's name is only a
// host-side handle; every GPU holds its own copy at its own address).
int static_scratch(void** out) {
  static std::atomic<void*> addr[64];
  int dev = 0;
  BLAST_HIP_TRY(hipGetDevice(&dev));
  const bool tracked = dev >= 0 && dev < 64;
  void* p = tracked ? addr[dev].load(std::memory_order_acquire) : nullptr;
  if (!p) {
    BLAST_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return BLAST_ERR_HIP;
    if (tracked) addr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return BLAST_OK;
}

}  // namespace

extern "C" size_t blast_sparse_mlp_static_limit(void) { return kStaticScratchBytes; }

extern "C" int blast_sparse_mlp_static(const blast_bsr_view* Wgate, const blast_bsr_view* Wup,
                                       const blast_bsr_view* Wdown, const uint16_t* X, int64_t ldx, int32_t x_layout,
                                       int64_t T, int32_t act, void* Y, int64_t ldy, int32_t y_dtype, void* stream_) {
  if (!Wup) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_mlp(Wgate, Wup, Wdown, X, ldx, x_layout, T, act, Y, ldy, y_dtype)) return rc;
  if (T == 0 || Wgate->cols == 0) return BLAST_OK;
  if (mlp_workspace_bytes(Wgate->rows, T) > kStaticScratchBytes) return BLAST_ERR_WORKSPACE;
  void* ws = nullptr;
  if (int rc = static_scratch(&ws)) return rc;
  return enqueue_mlp(Wgate, Wup, Wdown, X, ldx, x_layout, T, act, Y, ldy, y_dtype, ws, kStaticScratchBytes,
                     static_cast<hipStream_t>(stream_), nullptr);
}

extern "C" int blast_sparse_mlp_handover_test(const blast_bsr_view* Wgate, const blast_bsr_view* Wup,
                                              const blast_bsr_view* Wdown, const uint16_t* X, int64_t ldx,
                                              int32_t x_layout, int64_t T, int32_t act, void* Y, int64_t ldy,
                                              int32_t y_dtype, void* ws, size_t ws_bytes, void* stream_,
                                              int32_t spin_limit, int32_t withhold_publication) {
  if (!Wup || spin_limit < 1) return BLAST_ERR_INVALID_ARG;
  HandoverKnobs knobs;
  knobs.max_spins = spin_limit;
  knobs.withhold = withhold_publication ? 1 : 0;
  return enqueue_mlp(Wgate, Wup, Wdown, X, ldx, x_layout, T, act, Y, ldy, y_dtype, ws, ws_bytes,
                     static_cast<hipStream_t>(stream_), nullptr, knobs);
}

extern "C" int blast_sparse_mlp_status(const blast_bsr_view* Wgate, int64_t T, const void* ws, size_t ws_bytes,
                                       int32_t* status, void* stream_) {
  if (int rc = check_view(Wgate)) return rc;
  if (T < 0 || !status) return BLAST_ERR_INVALID_ARG;
  *status = 0;
  const int64_t I = Wgate->rows;
  const void* base = ws;
  size_t have = ws_bytes;
  if (!base) {  // the library's own scratch array (blast_sparse_mlp_static)
    void* p = nullptr;
    if (int rc = static_scratch(&p)) return rc;
    base = p;
    have = kStaticScratchBytes;
  }
  if (have < mlp_workspace_bytes(I, T) || !blast::aligned(base, 256)) return BLAST_ERR_WORKSPACE;
  const char* ctl = static_cast<const char*>(base) + mlp_h_bytes(I, T) + mlp_slot_bytes(I);
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  BLAST_HIP_TRY(hipStreamSynchronize(stream));
  unsigned long long sig = 0;
  BLAST_HIP_TRY(hipMemcpy(&sig, ctl, sizeof(sig), hipMemcpyDeviceToHost));
  // the signature carries the wave count of the launch shape in its low bits
  if ((sig ^ kCtlReady) >> 32) return BLAST_OK;  // no single-launch call has used this workspace at this shape
  int32_t word = 0;
  BLAST_HIP_TRY(hipMemcpy(&word, ctl + kCtlStatusOffset, sizeof(word), hipMemcpyDeviceToHost));
  *status = word;
  if (word != 0) {
    const int32_t zero = 0;
    BLAST_HIP_TRY(hipMemcpy(const_cast<char*>(ctl) + kCtlStatusOffset, &zero, sizeof(zero), hipMemcpyHostToDevice));
  }
  return BLAST_OK;
}

// ---- E5M2 weights, bf16 activations: the decode form of the 8-bit run (Sec. 5.2) ------------------------
namespace {

template <int B, bool DUAL, int NTT, int XSMALL, bool CHUNK>
int launch_decode_w8_ntt(const TileArgs& a, const ChunkPlan& plan, hipStream_t stream) {
  DecArgs d{};
  d.m0 = a.m0;
  d.m1 = a.m1;
  d.row_order = a.row_order;
  d.X = a.X;
  d.sxt = a.sxt;
  d.Y = a.Y;
  d.syt = a.syt;
  d.syi = a.syi;
  d.y_bf16 = a.y_bf16;
  d.T = a.T;
  d.act = a.act;
  d.hdr = plan.hdr;
  d.chunk_row = plan.chunk_row;
  d.chunk_kb = plan.chunk_kb;
  d.chunk_ke = plan.chunk_ke;
  const int64_t units = (CHUNK ? plan.max_chunks : (int64_t)a.nbr) * (B / 16);
  if (units <= 0) return BLAST_OK;
  const int64_t groups = (a.T + NTT * 16 - 1) / (NTT * 16);
  const int64_t grid = (units + 7) / 8 * 8 * groups;
  if (grid > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  d.n_units = (int)units;
  d.groups = (int)groups;
  using C = DecCfg<B, DUAL, NTT, XSMALL, false, true>;
  static blast::DeviceFlags lds_set;
  if (int rc = ensure_lds_limit(reinterpret_cast<const void*>(&k_decode<B, DUAL, NTT, CHUNK, XSMALL, false, true>),
                                C::LDS_BYTES, lds_set))
    return rc;
  if (CHUNK) {  // rows cut into several chunks are accumulated: clear them first
    StreamArgs sa{a, 0, -1, 0, plan.hdr, plan.chunk_row, plan.chunk_kb, plan.chunk_ke};
    k_zero_shared_rows<B><<<dim3((unsigned)plan.max_chunks, (unsigned)((a.T + 63) / 64)), dim3(256), 0, stream>>>(sa);
    BLAST_LAUNCH_CHECK("k_zero_shared_rows");
  }
  k_decode<B, DUAL, NTT, CHUNK, XSMALL, false, true><<<dim3((unsigned)grid), dim3(256), C::LDS_BYTES, stream>>>(d);
  BLAST_LAUNCH_CHECK("k_decode (E5M2 weights)");
  return BLAST_OK;
}

template <int B, bool DUAL, bool CHUNK>
int launch_decode_w8_c(const TileArgs& a, const ChunkPlan& plan, hipStream_t stream) {
  // the smallest activation tile that holds T token rows, as in launch_decode
  if (a.T <= 512 / B) return launch_decode_w8_ntt<B, DUAL, 1, 1, CHUNK>(a, plan, stream);
  if constexpr (B == 128) {
    if (a.T <= 8) return launch_decode_w8_ntt<B, DUAL, 1, 2, CHUNK>(a, plan, stream);
  }
  if (a.T <= 16) return launch_decode_w8_ntt<B, DUAL, 1, 0, CHUNK>(a, plan, stream);
  return launch_decode_w8_ntt<B, DUAL, 2, 0, CHUNK>(a, plan, stream);
}

// `plan`: the chunk plan of the matrix (single matrix, fp32 output only); taken under the rule of the bf16
// decode path: when the fullest row, dealt to four waves, is deeper than four times a workgroup slot's share.
template <int B, bool DUAL>
int launch_decode_w8(const TileArgs& a, int64_t nnz, const ChunkPlan& plan, hipStream_t stream) {
  if constexpr (!DUAL) {
    if (plan.hdr && !a.y_bf16 && a.T <= kDecodeMaxTokens) {
      double ref = (double)nnz * (B / 16) / (4.0 * 2.0 * cu_count());
      if (ref < blast::kChunkBlocks) ref = blast::kChunkBlocks;
      if ((double)plan.max_row_blocks / 4.0 > 4.0 * ref) return launch_decode_w8_c<B, false, true>(a, plan, stream);
    }
  }
  return launch_decode_w8_c<B, DUAL, false>(a, ChunkPlan{}, stream);
}

}  // namespace

extern "C" int blast_sparse_mlp_e5m2w_workspace(const blast_bsr_view* Wgate, int64_t T, size_t* ws_bytes) {
  if (int rc = check_view(Wgate)) return rc;
  if (T < 0 || !ws_bytes) return BLAST_ERR_INVALID_ARG;
  *ws_bytes = mlp_h_bytes(Wgate->rows, T);
  return BLAST_OK;
}

extern "C" int blast_sparse_mlp_e5m2w(const blast_bsr_view* Wgate, const uint8_t* gate8, const blast_bsr_view* Wup,
                                      const uint8_t* up8, const blast_bsr_view* Wdown, const uint8_t* down8,
                                      const uint16_t* X, int64_t ldx, int64_t T, int32_t act, void* Y, int64_t ldy,
                                      int32_t y_dtype, void* ws, size_t ws_bytes, void* stream_) {
  if (!Wup) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_mlp(Wgate, Wup, Wdown, X, ldx, BLAST_TOKEN_MAJOR, T, act, Y, ldy, y_dtype)) return rc;
  const int64_t I = Wgate->rows, E = Wgate->cols;
  const int32_t b = Wgate->b;
  if (b != 64 && b != 128) return BLAST_ERR_UNSUPPORTED_BLOCK;
  if ((Wgate->nnz > 0 && !gate8) || (Wup->nnz > 0 && !up8) || (Wdown->nnz > 0 && !down8)) return BLAST_ERR_INVALID_ARG;
  if (!blast::aligned(gate8, 16) || !blast::aligned(up8, 16) || !blast::aligned(down8, 16)) return BLAST_ERR_INVALID_ARG;
  if (T == 0 || E == 0) return BLAST_OK;
  // the copies address a block column of the activations with 32-bit byte offsets and fetch 16 bytes at a time
  if (ldx % 8 != 0 || !blast::aligned(X, 16) || T * ldx * 2 >= ((int64_t)1 << 32) || T * I * 2 >= ((int64_t)1 << 32))
    return BLAST_ERR_INVALID_ARG;
  const size_t need = mlp_h_bytes(I, T);
  if (need > 0 && (!ws || ws_bytes < need || !blast::aligned(ws, 256))) return BLAST_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  uint16_t* H = static_cast<uint16_t*>(ws);
  TileArgs g{};
  g.m0 = mat_of(Wgate);
  g.m0.vals8 = gate8;
  g.m1 = mat_of(Wup);
  g.m1.vals8 = up8;
  g.row_order = Wgate->row_order;
  set_x(g, X, ldx, BLAST_TOKEN_MAJOR);
  set_y(g, H, I, BLAST_TOKEN_MAJOR, BLAST_BF16);
  g.T = (int)T;
  g.nbr = (int)(I / b);
  g.kdim = E;
  g.act = act;
  TileArgs d{};
  d.m0 = mat_of(Wdown);
  d.m0.vals8 = down8;
  d.row_order = Wdown->row_order;
  set_x(d, H, I, BLAST_TOKEN_MAJOR);
  set_y(d, Y, ldy, BLAST_TOKEN_MAJOR, y_dtype);
  d.T = (int)T;
  d.nbr = (int)(E / b);
  d.kdim = I;
  d.act = -1;
  if (I > 0) {
    const int64_t nnz_gu = Wgate->nnz + Wup->nnz;
    if (int rc = (b == 64) ? launch_decode_w8<64, true>(g, nnz_gu, ChunkPlan{}, stream)
                           : launch_decode_w8<128, true>(g, nnz_gu, ChunkPlan{}, stream))
      return rc;
  }
  const ChunkPlan dplan = plan_of(Wdown, T);
  return (b == 64) ? launch_decode_w8<64, false>(d, Wdown->nnz, dplan, stream)
                   : launch_decode_w8<128, false>(d, Wdown->nnz, dplan, stream);
}

extern "C" int blast_sparse_mlp2(const blast_bsr_view* W1, const blast_bsr_view* W2, const uint16_t* X, int64_t ldx,
                                 int32_t x_layout, int64_t T, int32_t act, void* Y, int64_t ldy, int32_t y_dtype,
                                 void* ws, size_t ws_bytes, void* stream_) {
  return enqueue_mlp(W1, nullptr, W2, X, ldx, x_layout, T, act, Y, ldy, y_dtype, ws, ws_bytes,
                     static_cast<hipStream_t>(stream_), nullptr);
}

extern "C" int blast_sparse_mlp_events(const blast_bsr_view* Wgate, const blast_bsr_view* Wup,
                                       const blast_bsr_view* Wdown, const uint16_t* X, int64_t ldx, int32_t x_layout,
                                       int64_t T, int32_t act, void* Y, int64_t ldy, int32_t y_dtype, void* ws,
                                       size_t ws_bytes, void* stream_, void* const* events) {
  if (!Wup || !events || !events[0] || !events[1] || !events[2]) return BLAST_ERR_INVALID_ARG;
  return enqueue_mlp(Wgate, Wup, Wdown, X, ldx, x_layout, T, act, Y, ldy, y_dtype, ws, ws_bytes,
                     static_cast<hipStream_t>(stream_), events);
}

extern "C" int blast_bsr_gated_spmm(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const uint16_t* X,
                                    int64_t ldx, int32_t x_layout, int64_t T, int32_t act, uint16_t* H, int64_t ldh,
                                    void* stream_) {
  if (int rc = check_view(Wgate)) return rc;
  if (int rc = check_view(Wup)) return rc;
  if (Wup->rows != Wgate->rows || Wup->cols != Wgate->cols || Wup->b != Wgate->b) return BLAST_ERR_SHAPE;
  if (T < 0 || T > INT32_MAX / 2) return BLAST_ERR_INVALID_ARG;
  if (act != BLAST_ACT_SILU && act != BLAST_ACT_GELU && act != BLAST_ACT_RELU) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_dense(X, ldx, x_layout, Wgate->cols, T)) return rc;
  if (int rc = check_dense(H, ldh, x_layout, Wgate->rows, T)) return rc;
  if (T == 0 || Wgate->rows == 0) return BLAST_OK;
  return enqueue_gated(Wgate, Wup, X, ldx, x_layout, T, act, H, ldh, x_layout, static_cast<hipStream_t>(stream_));
}
