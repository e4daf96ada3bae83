// Internal helpers shared by the translation units of the HIP library (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/blast.h"

namespace blast {

// Records the text of a HIP failure for blast_strerror (per host thread).
void note_hip_error(hipError_t e, const char* where);

inline bool supported_block(int32_t b) { return b == 16 || b == 32 || b == 64 || b == 128; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Layout of the column-grouped index ("aux") that pack writes for a matrix with
// NBc block columns and capacity nnz_cap:  col_ptr[NBc+1] | csc_row[nnz_cap] | csc_blk[nnz_cap]
struct AuxLayout {
  size_t col_ptr_off, csc_row_off, csc_blk_off, bytes;
};
inline AuxLayout aux_layout(int64_t nbc, int64_t nnz_cap) {
  AuxLayout L;
  L.col_ptr_off = 0;
  L.csc_row_off = align_up(sizeof(int32_t) * (size_t)(nbc + 1), 16);
  L.csc_blk_off = L.csc_row_off + align_up(sizeof(int32_t) * (size_t)nnz_cap, 16);
  L.bytes = L.csc_blk_off + align_up(sizeof(int32_t) * (size_t)nnz_cap, 16);
  return L;
}

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
