// Device-side helpers shared by the product kernels.
#pragma once
#include "blast_common.h"

namespace blast_dev {


typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct MatDev {
  const int* row_ptr;
  const int* col_idx;
  const uint16_t* vals;
  const uint8_t* vals8 = nullptr;  // E5M2 codes of the same blocks (kernels instantiated for one-byte weights)
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
  int64_t kdim;          // features contracted over (columns of the matrix); host-side scheduling only
  int ntt;               // token tiles
  int act;               // gated product: the activation of the gate; single matrix: < 0 none, else applied to the output
  int x_vec;             // 1: 16-byte loads of X are legal (sxk == 1, aligned)
  int y_fast;            // 1: syi == 1 and every byte offset inside a 256-token slab of Y fits 31 bits
  int x_grp16;           // 16-wide blocks only: X is stored in column groups of 16 features, [kdim/16][T][16]
  int y_grp16;           // ... and so is Y, [rows/16][T][16]
};

// Index arrays are read-only for the lifetime of a launch: reading them through the
// constant address space lets uniform loads go through the scalar unit, so they never
// sit in the vector-memory counter that the DMA pipeline is tracked with.
__device__ __forceinline__ int ld_idx(const int* p, int i) {
  return reinterpret_cast<const __attribute__((address_space(4))) int*>(reinterpret_cast<uintptr_t>(p))[i];
}

// fp32 -> bf16, round to nearest even (the hardware conversion of gfx950).
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  const __bf16 h = static_cast<__bf16>(f);
  return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float apply_act(int act, float g) {
  if (act == BLAST_ACT_SILU) return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g));
  if (act == BLAST_ACT_GELU) return 0.5f * g * (1.0f + erff(g * 0.70710678118654752440f));
  return g > 0.0f ? g : 0.0f;
}


}  // namespace blast_dev
