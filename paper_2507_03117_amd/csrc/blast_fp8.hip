// E5M2 entry points: quantisation of bf16 data and the block-sparse product on E5M2 operands
// (BLaST Sec. 5.2 runs the kernel in float8_e5m2 as well as in 16-bit types).
#include "blast_common.h"

#include "kern_common.h"
#include "kern_fp8.h"

using namespace blast_dev;

namespace {

template <int B, bool KSPLIT, bool CHUNK = false>
int launch_fp8(Fp8Args a, hipStream_t stream) {
  using C = Fp8Cfg<B>;
  static blast::DeviceFlags lds_set;
  int dev = 0;
  BLAST_HIP_TRY(hipGetDevice(&dev));
  if (!lds_set.test(dev)) {
    BLAST_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_spmm_fp8<B, KSPLIT, CHUNK>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES));
    lds_set.set(dev);
  }
  const int64_t tokens_per_group = KSPLIT ? 64 : 256;
  const int64_t groups = (a.T + tokens_per_group - 1) / tokens_per_group;
  const int64_t grid = ((int64_t)a.n_units + 7) / 8 * 8 * groups;
  if (grid <= 0) return BLAST_OK;
  if (grid > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  a.groups = (int)groups;
  if (CHUNK) {
    // rows cut into several chunks are accumulated: clear them first (the kernel of the bf16 path; it only
    // reads the output description, the row pointers and the plan)
    StreamArgs sa{};
    sa.t.m0.row_ptr = a.row_ptr;
    sa.t.Y = a.Y;
    sa.t.syt = a.ldy;
    sa.t.syi = 1;
    sa.t.T = a.T;
    sa.hdr = a.hdr;
    sa.chunk_row = a.chunk_row;
    sa.chunk_kb = a.chunk_kb;
    sa.chunk_ke = a.chunk_ke;
    k_zero_shared_rows<B><<<dim3((unsigned)(a.n_units / C::SUB), (unsigned)((a.T + 63) / 64)), dim3(256), 0, stream>>>(sa);
    BLAST_LAUNCH_CHECK("k_zero_shared_rows");
  }
  k_spmm_fp8<B, KSPLIT, CHUNK><<<dim3((unsigned)grid), dim3(256), C::LDS_BYTES, stream>>>(a);
  BLAST_LAUNCH_CHECK("k_spmm_fp8");
  return BLAST_OK;
}

template <int B>
int launch_fp8_b(const Fp8Args& a, const blast_bsr_view* W, hipStream_t stream) {
  // up to two token tiles the stages of a row are dealt to the four waves (every wave streams weights);
  // beyond that a wave owns a token tile of its own and walks the whole row
  if (a.T <= 128) {
    // A row of n blocks is n * (B / 64) / 4 stages deep per wave.  When the fullest row is deeper than four
    // chunks' worth, take the packer's chunk plan (fp32 output only: chunks of a row add atomically).
    if (W->aux && !a.y_bf16 && W->max_row_blocks > 4 * blast::kChunkBlocks) {
      const int64_t nbr = W->rows / B, nbc = W->cols / B;
      const blast::AuxLayout L = blast::aux_layout(nbr, nbc, W->nnz);
      const char* ab = static_cast<const char*>(W->aux);
      Fp8Args c = a;
      c.hdr = reinterpret_cast<const int*>(ab + L.hdr_off);
      c.chunk_row = reinterpret_cast<const int*>(ab + L.chunk_row_off);
      c.chunk_kb = reinterpret_cast<const int*>(ab + L.chunk_kb_off);
      c.chunk_ke = reinterpret_cast<const int*>(ab + L.chunk_ke_off);
      const int64_t max_chunks = nbr + W->nnz / blast::kChunkBlocks;
      if (max_chunks * (B / 64) > INT32_MAX / 2) return BLAST_ERR_INVALID_ARG;
      c.n_units = (int)(max_chunks * (B / 64));
      return launch_fp8<B, true, true>(c, stream);
    }
    return launch_fp8<B, true>(a, stream);
  }
  return launch_fp8<B, false>(a, stream);
}

}  // namespace

extern "C" int blast_quantize_e5m2(const uint16_t* in_bf16, int64_t n, uint8_t* out, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (n < 0) return BLAST_ERR_INVALID_ARG;
  if (n == 0) return BLAST_OK;
  if (!in_bf16 || !out) return BLAST_ERR_INVALID_ARG;
  const int64_t blocks = ((n + 7) / 8 + 255) / 256;
  if (blocks > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  k_quantize_e5m2<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(in_bf16, n, out);
  BLAST_LAUNCH_CHECK("k_quantize_e5m2");
  return BLAST_OK;
}

extern "C" int blast_quantize_e5m2_groups(const uint16_t* X_bf16, int64_t ldx, int64_t T, int64_t K, uint8_t* out,
                                          void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (T < 0 || K < 0 || K % 64 != 0) return BLAST_ERR_INVALID_ARG;
  if (T == 0 || K == 0) return BLAST_OK;
  if (!X_bf16 || !out || ldx < K || !blast::aligned(out, 16)) return BLAST_ERR_INVALID_ARG;
  const int64_t blocks = (T * (K / 8) + 255) / 256;
  if (blocks > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  k_quantize_e5m2_groups<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(X_bf16, ldx, T, K, out);
  BLAST_LAUNCH_CHECK("k_quantize_e5m2_groups");
  return BLAST_OK;
}

extern "C" int blast_bsr_spmm_e5m2(const blast_bsr_view* W, const uint8_t* vals8, const uint8_t* X8, int64_t ldx,
                                   int32_t x_layout, int64_t T, void* Y, int64_t ldy, int32_t y_dtype,
                                   void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!W || !W->row_ptr) return BLAST_ERR_INVALID_ARG;
  if (W->rows < 0 || W->cols < 0 || W->nnz < 0 || W->nnz > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  if (!blast::supported_block(W->b)) return BLAST_ERR_UNSUPPORTED_BLOCK;
  if (W->rows % W->b || W->cols % W->b) return BLAST_ERR_SHAPE;
  if (W->rows / W->b > INT32_MAX / 4 || W->cols / W->b > INT32_MAX / 4) return BLAST_ERR_INVALID_ARG;
  if (x_layout != BLAST_TOKEN_MAJOR && x_layout != BLAST_FEATURE_MAJOR && x_layout != BLAST_COLUMN_GROUPS_64)
    return BLAST_ERR_INVALID_ARG;
  if (y_dtype != BLAST_F32 && y_dtype != BLAST_BF16) return BLAST_ERR_INVALID_ARG;
  if (T < 0 || T > INT32_MAX / 2) return BLAST_ERR_INVALID_ARG;
  if (T == 0 || W->rows == 0) return BLAST_OK;
  const bool cg = x_layout == BLAST_COLUMN_GROUPS_64;  // activations in column groups; the output is token-major
  const bool tm = x_layout == BLAST_TOKEN_MAJOR || cg;
  if (!Y || ldy < (tm ? W->rows : T)) return BLAST_ERR_INVALID_ARG;
  if (W->cols > 0 && (!X8 || (!cg && ldx < (tm ? W->cols : T)))) return BLAST_ERR_INVALID_ARG;
  if (W->nnz > 0 && (!W->col_idx || !vals8)) return BLAST_ERR_INVALID_ARG;
  const int b = W->b;
  if (cg) {
    // only the tiled kernel reads this layout: 64-wide groups need b >= 64, offsets inside a group 32 bits
    if (b < 64 || !blast::aligned(X8, 16) || !blast::aligned(vals8, 16) || T * 64 >= ((int64_t)1 << 32))
      return BLAST_ERR_INVALID_ARG;
  }
  const bool fast = cg || (tm && b >= 64 && ldx % 16 == 0 && blast::aligned(X8, 16) && blast::aligned(vals8, 16) &&
                           T * ldx < ((int64_t)1 << 32));
  if (fast) {
    Fp8Args a{};
    a.row_ptr = W->row_ptr;
    a.col_idx = W->col_idx;
    a.row_order = W->row_order;
    a.vals = vals8;
    a.X = X8;
    a.ldx = cg ? 64 : ldx;
    a.x_cg = cg ? T * 64 : 0;
    a.Y = Y;
    a.ldy = ldy;
    a.y_bf16 = y_dtype == BLAST_BF16 ? 1 : 0;
    a.y_fast = ((int64_t)64 * ldy * 4 + ldy * 4 < ((int64_t)1 << 31)) ? 1 : 0;
    a.T = (int)T;
    a.n_units = (int)(W->rows / b) * (b / 64);
    return b == 64 ? launch_fp8_b<64>(a, W, stream) : launch_fp8_b<128>(a, W, stream);
  }
  Fp8GenericArgs g{};
  g.row_ptr = W->row_ptr;
  g.col_idx = W->col_idx;
  g.vals = vals8;
  g.X = X8;
  g.sxk = tm ? 1 : ldx;
  g.sxt = tm ? ldx : 1;
  g.Y = Y;
  g.syt = tm ? ldy : 1;
  g.syi = tm ? 1 : ldy;
  g.y_bf16 = y_dtype == BLAST_BF16 ? 1 : 0;
  g.T = (int)T;
  g.b = b;
  const int64_t nbr = W->rows / b, tiles = (T + 63) / 64;
  if (tiles > 65535) return BLAST_ERR_INVALID_ARG;
  k_spmm_fp8_generic<<<dim3((unsigned)nbr, (unsigned)tiles), dim3(256), 0, stream>>>(g);
  BLAST_LAUNCH_CHECK("k_spmm_fp8_generic");
  return BLAST_OK;
}
