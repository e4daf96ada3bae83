// Error text for the C ABI.
#include <stdio.h>
#include <string.h>

#include "blast_common.h"

namespace {
thread_local char g_hip_text[256] = "";
thread_local char g_msg[384];
}  // namespace

namespace blast {
void note_hip_error(hipError_t e, const char* where) {
  snprintf(g_hip_text, sizeof(g_hip_text), "%s at %s", hipGetErrorString(e), where);
}
}  // namespace blast

extern "C" const char* blast_strerror(int code) {
  switch (code) {
    case BLAST_OK: return "ok";
    case BLAST_ERR_INVALID_ARG: return "invalid argument (null pointer, negative size, leading dimension, enum or alignment)";
    case BLAST_ERR_SHAPE: return "shape error (rows/cols not a multiple of the block size, or inconsistent MLP matrices)";
    case BLAST_ERR_UNSUPPORTED_BLOCK: return "unsupported block size (expected 16, 32, 64 or 128)";
    case BLAST_ERR_CAPACITY: return "nnz_cap is smaller than the number of kept blocks";
    case BLAST_ERR_WORKSPACE: return "workspace or aux buffer missing, misaligned or too small (blast_sparse_mlp_static: the call needs more scratch than the library's array holds)";
    case BLAST_ERR_HIP:
      snprintf(g_msg, sizeof(g_msg), "HIP runtime error: %s", g_hip_text[0] ? g_hip_text : "(no detail recorded)");
      return g_msg;
    default: return "unknown error code";
  }
}
