// Backward-pass products on the packed weight (BLaST Sec. 3.2: the pruned matrix serves forward and
// backward propagation alike).
//
//   dX = W~^T dY   runs as the forward product on the packed transpose that blast_bsr_transpose builds
//                  (the BCSC view of the same blocks, Sec. 3.4.1), so it has no kernel of its own;
//   dW~            the gradient of the stored blocks, a block-sampled dense-dense product: kern_sddmm.h.
#include "blast_common.h"

#include "kern_common.h"
#include "kern_sddmm.h"

using namespace blast_dev;

namespace {

int cu_count_bwd() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
  return n;
}

template <int B>
int launch_sddmm(SddmmArgs a, hipStream_t stream) {
  using C = SdCfg<B>;
  static blast::DeviceFlags lds_set;
  int dev = 0;
  BLAST_HIP_TRY(hipGetDevice(&dev));
  if (!lds_set.test(dev)) {
    BLAST_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_sddmm<B>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES));
    lds_set.set(dev);
  }
  const int64_t sub_units = (int64_t)a.nnz * C::SUB * C::SUB;
  // Token chunks across workgroups (on top of the four waves of a workgroup): only when there are fewer
  // units than CUs, and never below 512 tokens per chunk - the atomics on the output cost more than
  // idle workgroup slots otherwise.
  const int64_t want = (int64_t)cu_count_bwd();
  int64_t tsplit = (want + sub_units - 1) / sub_units;
  const int64_t max_split = (a.T + 511) / 512;
  if (tsplit > max_split) tsplit = max_split;
  if (tsplit < 1) tsplit = 1;
  int64_t chunk = ((a.T + tsplit - 1) / tsplit + C::KT - 1) / C::KT * C::KT;
  tsplit = (a.T + chunk - 1) / chunk;
  const int64_t units = sub_units * tsplit;
  if (units > INT32_MAX / 2) return BLAST_ERR_INVALID_ARG;
  a.tsplit = (int)tsplit;
  a.chunk_tokens = (int)chunk;
  a.n_units = (int)units;
  if (tsplit > 1) {
    const int64_t n = (int64_t)a.nnz * B * B;
    k_zero_f32<<<dim3((unsigned)((n / 4 + 255) / 256 + 1)), dim3(256), 0, stream>>>(a.dvals, n);
    BLAST_LAUNCH_CHECK("k_zero_f32");
  }
  k_sddmm<B><<<dim3((unsigned)((units + 7) / 8 * 8)), dim3(256), C::LDS_BYTES, stream>>>(a);
  BLAST_LAUNCH_CHECK("k_sddmm");
  return BLAST_OK;
}

}  // namespace

extern "C" int blast_bsr_sddmm(const blast_bsr_view* W, const uint16_t* dY, int64_t ldy, const uint16_t* X,
                               int64_t ldx, int32_t layout, int64_t T, float* dvals, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!W || !W->row_ptr) return BLAST_ERR_INVALID_ARG;
  if (W->rows < 0 || W->cols < 0 || W->nnz < 0 || W->nnz > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  if (!blast::supported_block(W->b)) return BLAST_ERR_UNSUPPORTED_BLOCK;
  if (W->rows % W->b || W->cols % W->b) return BLAST_ERR_SHAPE;
  if (W->rows / W->b > INT32_MAX / 2 || W->cols / W->b > INT32_MAX / 2) return BLAST_ERR_INVALID_ARG;
  if (layout != BLAST_TOKEN_MAJOR && layout != BLAST_FEATURE_MAJOR) return BLAST_ERR_INVALID_ARG;
  if (T < 0 || T > INT32_MAX / 2) return BLAST_ERR_INVALID_ARG;
  if (W->nnz == 0) return BLAST_OK;
  if (!W->col_idx || !dvals || !blast::aligned(dvals, 16)) return BLAST_ERR_INVALID_ARG;
  const int b = W->b;
  const int64_t n_out = W->nnz * b * b;
  if (T == 0) {  // an empty sum
    k_zero_f32<<<dim3((unsigned)((n_out / 4 + 255) / 256 + 1)), dim3(256), 0, stream>>>(dvals, n_out);
    BLAST_LAUNCH_CHECK("k_zero_f32");
    return BLAST_OK;
  }
  if (!dY || !X) return BLAST_ERR_INVALID_ARG;
  if (ldy < (layout == BLAST_TOKEN_MAJOR ? W->rows : T) || ldx < (layout == BLAST_TOKEN_MAJOR ? W->cols : T))
    return BLAST_ERR_INVALID_ARG;

  const bool fast = layout == BLAST_TOKEN_MAJOR && b >= 32 && ldy % 8 == 0 && ldx % 8 == 0 &&
                    blast::aligned(dY, 16) && blast::aligned(X, 16);
  if (fast) {
    SddmmArgs a{};
    a.row_ptr = W->row_ptr;
    a.col_idx = W->col_idx;
    a.dY = dY;
    a.X = X;
    a.ldy = ldy;
    a.ldx = ldx;
    a.dvals = dvals;
    a.T = (int)T;
    a.nbr = (int)(W->rows / b);
    a.nnz = (int)W->nnz;
    switch (b) {
      case 32: return launch_sddmm<32>(a, stream);
      case 64: return launch_sddmm<64>(a, stream);
      default: return launch_sddmm<128>(a, stream);
    }
  }
  SddmmGenericArgs g{};
  g.row_ptr = W->row_ptr;
  g.col_idx = W->col_idx;
  g.dY = dY;
  g.X = X;
  if (layout == BLAST_TOKEN_MAJOR) {
    g.syt = ldy; g.syi = 1; g.sxt = ldx; g.sxk = 1;
  } else {
    g.syt = 1; g.syi = ldy; g.sxt = 1; g.sxk = ldx;
  }
  g.dvals = dvals;
  g.T = (int)T;
  g.nbr = (int)(W->rows / b);
  g.b = b;
  k_sddmm_generic<<<dim3((unsigned)W->nnz), dim3(256), 0, stream>>>(g);
  BLAST_LAUNCH_CHECK("k_sddmm_generic");
  return BLAST_OK;
}
