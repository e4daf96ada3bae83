// Internal helpers shared by the translation units of the HIP library (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/blast.h"

namespace blast {

// Records the text of a HIP failure for blast_strerror (per host thread).
void note_hip_error(hipError_t e, const char* where);

inline bool supported_block(int32_t b) { return b == 16 || b == 32 || b == 64 || b == 128; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Block rows holding more than kChunkBlocks stored blocks are cut into chunks of at most that many
// blocks; a chunk is the unit of work of the decode kernels, so one very long row cannot become the
// critical path of a launch (its chunks add their partial sums into the output atomically).  The
// streaming (prefill) kernels take the same rows in chunks of kWideChunkBlocks: every chunk pays for
// an output tile added atomically, which at 256 tokens per tile is worth about ten block steps
// (measured on a 16384 x 53248 layer with Zipf row lengths, b = 128, 2048 tokens: 331 us with chunks of
// 16 blocks, 280 with 32, 267 with 64, 310 with 128).
constexpr int kChunkBlocks = 16;
constexpr int kWideChunkBlocks = 64;

// Layout of the "aux" buffer that pack writes for a matrix with NBr block rows, NBc block columns and
// nnz stored blocks (every offset can be recomputed from the packed view alone):
//   chunk plan:            hdr[4] = {n_chunks, max_row_blocks, kChunkBlocks, n_split_chunks} |
//                          chunk_row[cap] (bit 31: the row has several chunks) | chunk_kb[cap] | chunk_ke[cap]
//                          in schedule order (rows by population, descending), cap = NBr + NBr*NBc/kChunkBlocks + 1;
//                          the rows with several chunks come first in that order, so their n_split_chunks chunks
//                          are the head of the plan
//   wide chunk plan:       the same with kWideChunkBlocks: whdr[4] | wchunk_row[wcap] | wchunk_kb[wcap] | wchunk_ke[wcap]
//   row_slot[NBr]:         for a row with several chunks in the first plan, its rank in the schedule order
//                          (0, 1, ... : a dense numbering of those rows), else -1
//   row_chunk0[NBr]:       for such a row the index of its first chunk in the first plan, else -1
//   column-grouped index:  col_ptr[NBc+1] | csc_row[nnz] | csc_blk[nnz]
// The buffer is sized with nnz = nnz_cap; the arrays are placed with the actual nnz.
struct AuxLayout {
  size_t hdr_off, chunk_row_off, chunk_kb_off, chunk_ke_off;
  size_t whdr_off, wchunk_row_off, wchunk_kb_off, wchunk_ke_off;
  size_t row_slot_off, row_chunk0_off, col_ptr_off, csc_row_off, csc_blk_off, bytes;
  int64_t chunk_cap, wchunk_cap;
};
inline AuxLayout aux_layout(int64_t nbr, int64_t nbc, int64_t nnz) {
  AuxLayout L;
  L.chunk_cap = nbr + (nbr * nbc) / kChunkBlocks + 1;
  L.wchunk_cap = nbr + (nbr * nbc) / kWideChunkBlocks + 1;
  const size_t cb = align_up(sizeof(int32_t) * (size_t)L.chunk_cap, 16);
  const size_t wb = align_up(sizeof(int32_t) * (size_t)L.wchunk_cap, 16);
  L.hdr_off = 0;
  L.chunk_row_off = 16;
  L.chunk_kb_off = L.chunk_row_off + cb;
  L.chunk_ke_off = L.chunk_kb_off + cb;
  L.whdr_off = L.chunk_ke_off + cb;
  L.wchunk_row_off = L.whdr_off + 16;
  L.wchunk_kb_off = L.wchunk_row_off + wb;
  L.wchunk_ke_off = L.wchunk_kb_off + wb;
  L.row_slot_off = L.wchunk_ke_off + wb;
  L.row_chunk0_off = L.row_slot_off + align_up(sizeof(int32_t) * (size_t)nbr, 16);
  L.col_ptr_off = L.row_chunk0_off + align_up(sizeof(int32_t) * (size_t)nbr, 16);
  L.csc_row_off = L.col_ptr_off + align_up(sizeof(int32_t) * (size_t)(nbc + 1), 16);
  L.csc_blk_off = L.csc_row_off + align_up(sizeof(int32_t) * (size_t)nnz, 16);
  L.bytes = L.csc_blk_off + align_up(sizeof(int32_t) * (size_t)nnz, 16);
  return L;
}

// One flag per device, set once something per-device has been done.  Host threads may race on it: the
// worst outcome is that the (idempotent) action runs twice.
struct DeviceFlags {
  std::atomic<bool> done[64];
  bool test(int dev) const { return dev >= 0 && dev < 64 && done[dev].load(std::memory_order_acquire); }
  void set(int dev) {
    if (dev >= 0 && dev < 64) done[dev].store(true, std::memory_order_release);
  }
};

}  // namespace blast

#define BLAST_HIP_TRY(expr)                        \
  do {                                             \
    hipError_t e__ = (expr);                       \
    if (e__ != hipSuccess) {                       \
      ::blast::note_hip_error(e__, #expr);         \
      return BLAST_ERR_HIP;                        \
    }                                              \
  } while (0)

#define BLAST_LAUNCH_CHECK(name)                   \
  do {                                             \
    hipError_t e__ = hipGetLastError();            \
    if (e__ != hipSuccess) {                       \
      ::blast::note_hip_error(e__, name);          \
      return BLAST_ERR_HIP;                        \
    }                                              \
  } while (0)
