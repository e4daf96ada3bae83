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

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct MatDev {
  const int* row_ptr;
  const int* col_idx;
  const uint16_t* vals;
};

struct TileArgs {
  MatDev m0, m1;         // m1 only for the dual (gate/up) kernel
  const int* row_order;  // may be null
  const uint16_t* X;
  int64_t sxt, sxk;      // element strides of X along tokens / features
  void* Y;
  int64_t syt, syi;      // element strides of Y along tokens / rows
  int y_bf16;
  int T;
  int nbr;               // block rows of the output
  int ntt;               // token tiles
  int act;
  int x_vec;             // 1: 16-byte loads of X are legal (sxk == 1, aligned)
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float apply_act(int act, float g) {
  if (act == BLAST_ACT_SILU) return g / (1.0f + __expf(-g));
  if (act == BLAST_ACT_GELU) return 0.5f * g * (1.0f + erff(g * 0.70710678118654752440f));
  return g > 0.0f ? g : 0.0f;
}

template <int B>
struct TileCfg {
  static constexpr int TOKW = (B == 128) ? 2 : 4;       // waves along tokens
  static constexpr int ROWW = 4 / TOKW;                 // waves along weight rows
  static constexpr int WT_ROW = (B >= 64) ? 64 : B;     // weight rows per wave
  static constexpr int NI = (WT_ROW + 31) / 32;         // 32-row MFMA tiles per wave
  static constexpr int MI = 2;                          // 32-token MFMA tiles per wave
  static constexpr int TT = TOKW * 64;                  // tokens per workgroup tile
  static constexpr int LD = B + 8;                      // LDS row pitch in bf16 (16-byte pad: conflict-free b128 reads)
  static constexpr int CPR = B / 8;                     // 16-byte chunks per row
  static constexpr int NCHW = B * CPR;                  // chunks in a weight block
  static constexpr int NCHX = TT * CPR;                 // chunks in an X tile
  static constexpr int WPT = (NCHW + 255) / 256;
  static constexpr int XPT = (NCHX + 255) / 256;
  static constexpr int KSTEPS = B / 16;
  static constexpr size_t LDS_BYTES = (size_t)(TT + B) * LD * 2;
};

template <int B>
struct Staged {
  uint4 w[TileCfg<B>::WPT];
  uint4 x[TileCfg<B>::XPT];
};

// Global -> registers for stored block k of a matrix (its values and the X slice it selects).
template <int B>
__device__ __forceinline__ void load_stage(const TileArgs& a, const MatDev& m, int k, int t0, Staged<B>& s) {
  using C = TileCfg<B>;
  const int tid = threadIdx.x;
  const uint16_t* wblk = m.vals + (int64_t)k * B * B;
  const int64_t c = m.col_idx[k];
#pragma unroll
  for (int j = 0; j < C::WPT; ++j) {
    const int idx = tid + 256 * j;
    if (C::NCHW % 256 == 0 || idx < C::NCHW) s.w[j] = *reinterpret_cast<const uint4*>(wblk + (int64_t)idx * 8);
  }
#pragma unroll
  for (int j = 0; j < C::XPT; ++j) {
    const int idx = tid + 256 * j;
    const int tok = idx / C::CPR, c8 = idx % C::CPR;
    const int t = t0 + tok;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (t < a.T) {
      if (a.x_vec) {
        v = *reinterpret_cast<const uint4*>(a.X + (int64_t)t * a.sxt + c * B + c8 * 8);
      } else {
        const uint16_t* p = a.X + (int64_t)t * a.sxt + (c * B + c8 * 8) * a.sxk;
        uint32_t e[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) e[q] = p[q * a.sxk];
        v = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
      }
    }
    s.x[j] = v;
  }
}

template <int B>
__device__ __forceinline__ void store_stage(uint16_t* Xs, uint16_t* Ws, const Staged<B>& s) {
  using C = TileCfg<B>;
  const int tid = threadIdx.x;
#pragma unroll
  for (int j = 0; j < C::WPT; ++j) {
    const int idx = tid + 256 * j;
    if (C::NCHW % 256 == 0 || idx < C::NCHW)
      *reinterpret_cast<uint4*>(Ws + (idx / C::CPR) * C::LD + (idx % C::CPR) * 8) = s.w[j];
  }
#pragma unroll
  for (int j = 0; j < C::XPT; ++j) {
    const int idx = tid + 256 * j;
    *reinterpret_cast<uint4*>(Xs + (idx / C::CPR) * C::LD + (idx % C::CPR) * 8) = s.x[j];
  }
}

// acc[mi][ni] += Xtile(wave's 64 tokens) * Wblock(wave's rows)^T from LDS.
template <int B>
__device__ __forceinline__ void mma_stage(const uint16_t* Xs, const uint16_t* Ws, int tw, int rw,
                                          f32x16 (&acc)[TileCfg<B>::MI][TileCfg<B>::NI]) {
  using C = TileCfg<B>;
  const int lane = threadIdx.x & 63, l32 = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int kk = 0; kk < C::KSTEPS; ++kk) {
    bf16x8 af[C::MI], bfg[C::NI];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
      af[mi] = *reinterpret_cast<const bf16x8*>(Xs + (tw * 64 + mi * 32 + l32) * C::LD + kk * 16 + lh * 8);
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      if (C::WT_ROW >= 32 || l32 < C::WT_ROW) {
        bfg[ni] = *reinterpret_cast<const bf16x8*>(Ws + (rw * C::WT_ROW + ni * 32 + l32) * C::LD + kk * 16 + lh * 8);
      } else {
        bfg[ni] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      }
    }
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfg[ni], acc[mi][ni], 0, 0, 0);
  }
}

// All stored blocks of block row r of matrix m, register-prefetched one block ahead.
template <int B>
__device__ __forceinline__ void run_row(const TileArgs& a, const MatDev& m, int r, int t0, uint16_t* Xs, uint16_t* Ws,
                                        int tw, int rw, f32x16 (&acc)[TileCfg<B>::MI][TileCfg<B>::NI]) {
  const int kb = m.row_ptr[r], ke = m.row_ptr[r + 1];
  Staged<B> st;
  if (kb < ke) load_stage<B>(a, m, kb, t0, st);
  for (int k = kb; k < ke; ++k) {
    __syncthreads();  // everyone is done reading the previous stage
    store_stage<B>(Xs, Ws, st);
    __syncthreads();
    if (k + 1 < ke) load_stage<B>(a, m, k + 1, t0, st);
    mma_stage<B>(Xs, Ws, tw, rw, acc);
  }
}

// One workgroup = one (block row, token tile).  DUAL: two matrices with the same
// shape share the tile; the epilogue writes bf16 act(acc0) * acc1.
template <int B, bool DUAL>
__global__ __launch_bounds__(256) void k_spmm_tile(const TileArgs a) {
  using C = TileCfg<B>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Xs = reinterpret_cast<uint16_t*>(smem);
  uint16_t* Ws = Xs + C::TT * C::LD;

  const int wg = blockIdx.x;
  const int rank = wg / a.ntt, tt = wg % a.ntt;
  const int r = a.row_order ? a.row_order[rank] : rank;
  const int t0 = tt * C::TT;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l32 = lane & 31, lh = lane >> 5;
  const int tw = wave % C::TOKW, rw = wave / C::TOKW;

  f32x16 acc0[C::MI][C::NI];
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = 0.0f;
  run_row<B>(a, a.m0, r, t0, Xs, Ws, tw, rw, acc0);

  if (DUAL) {
    f32x16 acc1[C::MI][C::NI];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc1[mi][ni][j] = 0.0f;
    run_row<B>(a, a.m1, r, t0, Xs, Ws, tw, rw, acc1);
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc0[mi][ni][j] = apply_act(a.act, acc0[mi][ni][j]) * acc1[mi][ni][j];
  }

  // Result layout of the 32x32 MFMA: lane -> column (weight row) l32, register j -> token 8*(j/4) + 4*lh + j%4.
  if (C::WT_ROW < 32 && l32 >= C::WT_ROW) return;
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      const int64_t row = (int64_t)r * B + rw * C::WT_ROW + ni * 32 + l32;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int tok = t0 + tw * 64 + mi * 32 + 8 * (j / 4) + 4 * lh + (j % 4);
        if (tok < a.T) {
          const float v = acc0[mi][ni][j];
          const int64_t off = (int64_t)tok * a.syt + row * a.syi;
          if (a.y_bf16)
            reinterpret_cast<uint16_t*>(a.Y)[off] = f32_to_bf16_rne(v);
          else
            reinterpret_cast<float*>(a.Y)[off] = v;
        }
      }
    }
}

template <int B, bool DUAL>
int launch_tile(TileArgs a, hipStream_t stream) {
  using C = TileCfg<B>;
  static bool attr_set = false;  // raising the dynamic-LDS limit is idempotent; a race only repeats it
  if (!attr_set) {
    BLAST_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_spmm_tile<B, DUAL>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES));
    attr_set = true;
  }
  a.ntt = (a.T + C::TT - 1) / C::TT;
  const int64_t grid = (int64_t)a.ntt * a.nbr;
  if (grid <= 0) return BLAST_OK;
  if (grid > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  k_spmm_tile<B, DUAL><<<dim3((unsigned)grid), dim3(256), C::LDS_BYTES, stream>>>(a);
  BLAST_LAUNCH_CHECK("k_spmm_tile");
  return BLAST_OK;
}

template <bool DUAL>
int dispatch_tile(int b, const TileArgs& a, hipStream_t stream) {
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
  if (layout == BLAST_TOKEN_MAJOR) {
    a.syt = ldy;
    a.syi = 1;
  } else {
    a.syt = 1;
    a.syi = ldy;
  }
}

MatDev mat_of(const blast_bsr_view* v) { return MatDev{v->row_ptr, v->col_idx, v->vals}; }

}  // namespace

extern "C" int blast_bsr_spmm_workspace(const blast_bsr_view* W, int64_t T, size_t* ws_bytes) {
  if (int rc = check_view(W)) return rc;
  if (T < 0 || !ws_bytes) return BLAST_ERR_INVALID_ARG;
  *ws_bytes = 0;
  return BLAST_OK;
}

extern "C" int blast_bsr_spmm(const blast_bsr_view* W, const uint16_t* X, int64_t ldx, int32_t x_layout, int64_t T,
                              void* Y, int64_t ldy, int32_t y_dtype, void* ws, size_t ws_bytes, void* stream_) {
  (void)ws;
  (void)ws_bytes;
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
  a.act = 0;
  return dispatch_tile<false>(W->b, a, stream);
}

extern "C" int blast_sparse_mlp_workspace(const blast_bsr_view* Wgate, const blast_bsr_view* Wup,
                                          const blast_bsr_view* Wdown, int64_t T, size_t* ws_bytes) {
  if (int rc = check_view(Wgate)) return rc;
  if (int rc = check_view(Wup)) return rc;
  if (int rc = check_view(Wdown)) return rc;
  if (T < 0 || !ws_bytes) return BLAST_ERR_INVALID_ARG;
  // H = act(G) * U in bf16, token-major [T][I]
  *ws_bytes = blast::align_up((size_t)T * (size_t)Wgate->rows * 2, 256);
  return BLAST_OK;
}

namespace {

int check_mlp(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown, const uint16_t* X,
              int64_t ldx, int32_t x_layout, int64_t T, int32_t act, void* Y, int64_t ldy, int32_t y_dtype) {
  if (int rc = check_view(Wgate)) return rc;
  if (int rc = check_view(Wup)) return rc;
  if (int rc = check_view(Wdown)) return rc;
  const int64_t I = Wgate->rows, E = Wgate->cols;
  const int32_t b = Wgate->b;
  if (Wup->rows != I || Wup->cols != E || Wdown->rows != E || Wdown->cols != I || Wup->b != b || Wdown->b != b)
    return BLAST_ERR_SHAPE;
  if (T < 0 || T > INT32_MAX / 2) return BLAST_ERR_INVALID_ARG;
  if (act != BLAST_ACT_SILU && act != BLAST_ACT_GELU && act != BLAST_ACT_RELU) return BLAST_ERR_INVALID_ARG;
  if (y_dtype != BLAST_F32 && y_dtype != BLAST_BF16) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_dense(X, ldx, x_layout, E, T)) return rc;
  if (int rc = check_dense(Y, ldy, x_layout, E, T)) return rc;
  return BLAST_OK;
}

// H = act(Wgate X) (.) (Wup X), bf16, strides given by (h_layout, ldh).
int enqueue_gated(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const uint16_t* X, int64_t ldx,
                  int32_t x_layout, int64_t T, int32_t act, uint16_t* H, int64_t ldh, int32_t h_layout,
                  hipStream_t stream) {
  TileArgs g{};
  g.m0 = mat_of(Wgate);
  g.m1 = mat_of(Wup);
  g.row_order = Wgate->row_order;
  set_x(g, X, ldx, x_layout);
  set_y(g, H, ldh, h_layout, BLAST_BF16);
  g.T = (int)T;
  g.nbr = (int)(Wgate->rows / Wgate->b);
  g.act = act;
  return dispatch_tile<true>(Wgate->b, g, stream);
}

int enqueue_mlp(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown,
                const uint16_t* X, int64_t ldx, int32_t x_layout, int64_t T, int32_t act, void* Y, int64_t ldy,
                int32_t y_dtype, void* ws, size_t ws_bytes, hipStream_t stream, void* const* events) {
  if (int rc = check_mlp(Wgate, Wup, Wdown, X, ldx, x_layout, T, act, Y, ldy, y_dtype)) return rc;
  const int64_t I = Wgate->rows, E = Wgate->cols;
  const int32_t b = Wgate->b;
  if (T == 0 || E == 0) return BLAST_OK;
  size_t need = 0;
  blast_sparse_mlp_workspace(Wgate, Wup, Wdown, T, &need);
  if (need > 0 && (!ws || ws_bytes < need || !blast::aligned(ws, 256))) return BLAST_ERR_WORKSPACE;
  uint16_t* H = static_cast<uint16_t*>(ws);

  if (events) BLAST_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(events[0]), stream));
  if (I > 0) {
    if (int rc = enqueue_gated(Wgate, Wup, X, ldx, x_layout, T, act, H, I, BLAST_TOKEN_MAJOR, stream)) return rc;
  }
  if (events) BLAST_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(events[1]), stream));
  TileArgs d{};
  d.m0 = mat_of(Wdown);
  d.row_order = Wdown->row_order;
  set_x(d, H, I, BLAST_TOKEN_MAJOR);
  set_y(d, Y, ldy, x_layout, y_dtype);
  d.T = (int)T;
  d.nbr = (int)(E / b);
  d.act = 0;
  if (int rc = dispatch_tile<false>(b, d, stream)) return rc;
  if (events) BLAST_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(events[2]), stream));
  return BLAST_OK;
}

}  // namespace

extern "C" int blast_sparse_mlp(const blast_bsr_view* Wgate, const blast_bsr_view* Wup, const blast_bsr_view* Wdown,
                                const uint16_t* X, int64_t ldx, int32_t x_layout, int64_t T, int32_t act, void* Y,
                                int64_t ldy, int32_t y_dtype, void* ws, size_t ws_bytes, void* stream_) {
  return enqueue_mlp(Wgate, Wup, Wdown, X, ldx, x_layout, T, act, Y, ldy, y_dtype, ws, ws_bytes,
                     static_cast<hipStream_t>(stream_), nullptr);
}

extern "C" int blast_sparse_mlp_events(const blast_bsr_view* Wgate, const blast_bsr_view* Wup,
                                       const blast_bsr_view* Wdown, const uint16_t* X, int64_t ldx, int32_t x_layout,
                                       int64_t T, int32_t act, void* Y, int64_t ldy, int32_t y_dtype, void* ws,
                                       size_t ws_bytes, void* stream_, void* const* events) {
  if (!events || !events[0] || !events[1] || !events[2]) return BLAST_ERR_INVALID_ARG;
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
