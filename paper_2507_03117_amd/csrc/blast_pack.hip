// Block-norm pruning and packing of a dense bf16 weight into the block-compressed
// format (BLaST Sec. 3.2: score each b x b block by its Frobenius norm, drop the
// lowest until the target sparsity is reached; Sec. 3.4.1: compressed block
// storage from which the product kernel derives its work).
//
// Everything runs on the device, on the caller's stream:
//   score  -> one workgroup per block, 16-byte loads, fp64 sum of squares
//   select -> exact radix select on the fp64 bit patterns + index-ordered tie-break
//   count  -> per block-row / block-column populations, exclusive scans
//   fill   -> ordered compaction of column indices, gather of block values
//   order  -> rank block rows by population (schedule for load balance)
//   csc    -> column-grouped index of the same blocks (used by the fused MLP)
#include "blast_common.h"

namespace {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Workgroup barrier.  LDS_ONLY: only the workgroup's LDS traffic is ordered - global stores still in flight are
// not waited for (the plain barrier waits for their acknowledgement, a trip to the memory side every time).
template <bool LDS_ONLY>
__device__ __forceinline__ void wg_barrier() {
  if (LDS_ONLY)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  else
    __syncthreads();
}

// Exclusive scan of one int per thread over the whole workgroup (blockDim.x a
// multiple of 64, at most 1024).  `wave_tot` is LDS scratch of >= 16 ints.
// Returns the exclusive prefix; `total` receives the workgroup sum.
template <bool LDS_ONLY = false>
__device__ __forceinline__ int block_exscan(int v, int* wave_tot, int& total) {
  const int lane = lane_id(), wave = threadIdx.x / kWave, nw = blockDim.x / kWave;
  int inc = v;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int o = __shfl_up(inc, d, kWave);
    if (lane >= d) inc += o;
  }
  wg_barrier<LDS_ONLY>();  // protect wave_tot from the previous use
  if (lane == kWave - 1) wave_tot[wave] = inc;
  wg_barrier<LDS_ONLY>();
  int base = 0, tot = 0;
  for (int w = 0; w < nw; ++w) {
    int t = wave_tot[w];
    if (w < wave) base += t;
    tot += t;
  }
  total = tot;
  return base + inc - v;
}

__device__ __forceinline__ double sq_bf16_pair(uint32_t w) {
  // two bf16 packed in a dword; each widened exactly to fp32, squared in fp64
  double lo = (double)__uint_as_float(w << 16);
  double hi = (double)__uint_as_float(w & 0xFFFF0000u);
  return lo * lo + hi * hi;
}

// One workgroup per block: squared Frobenius norm in fp64.  The summation tree
// depends only on b, so equal blocks get equal scores wherever they sit.
// blockIdx.y == 1: a second matrix of the same shape (the gradient of the mask update) into a second score array.
__global__ __launch_bounds__(256) void k_block_scores(const uint16_t* __restrict__ W, int64_t ldw, int nbc, int b,
                                                      double* __restrict__ score,
                                                      const uint16_t* __restrict__ W1 = nullptr, int64_t ldw1 = 0,
                                                      double* __restrict__ score1 = nullptr) {
  __shared__ double red[256];
  if (blockIdx.y == 1) {
    W = W1;
    ldw = ldw1;
    score = score1;
  }
  const int64_t blk = blockIdx.x;
  const int64_t br = blk / nbc, bc = blk % nbc;
  const uint16_t* base = W + br * b * ldw + bc * b;
  const int cpr = b / 8, nchunks = b * cpr;
  double s = 0.0;
  for (int c = threadIdx.x; c < nchunks; c += 256) {
    const int i = c / cpr, j8 = c % cpr;
    const uint4 v = *reinterpret_cast<const uint4*>(base + (int64_t)i * ldw + j8 * 8);
    s += (sq_bf16_pair(v.x) + sq_bf16_pair(v.y)) + (sq_bf16_pair(v.z) + sq_bf16_pair(v.w));
  }
  red[threadIdx.x] = s;
  __syncthreads();
  for (int d = 128; d > 0; d >>= 1) {
    if ((int)threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
    __syncthreads();
  }
  if (threadIdx.x == 0) score[blk] = red[0];
}

// One workgroup per block: mean of an fp32 sensitivity matrix over the block (2D average pooling,
// BLaST Sec. 3.3), accumulated in fp64 with the same tree as the Frobenius scores.
__global__ __launch_bounds__(256) void k_pooled_scores(const float* __restrict__ S, int64_t lds, int nbc, int b,
                                                       double* __restrict__ score) {
  __shared__ double red[256];
  const int64_t blk = blockIdx.x;
  const int64_t br = blk / nbc, bc = blk % nbc;
  const float* base = S + br * b * lds + bc * b;
  const int cpr = b / 4, nchunks = b * cpr;
  double s = 0.0;
  for (int c = threadIdx.x; c < nchunks; c += 256) {
    const int i = c / cpr, j4 = c % cpr;
    const float4 v = *reinterpret_cast<const float4*>(base + (int64_t)i * lds + j4 * 4);
    s += ((double)v.x + (double)v.y) + ((double)v.z + (double)v.w);
  }
  red[threadIdx.x] = s;
  __syncthreads();
  for (int d = 128; d > 0; d >>= 1) {
    if ((int)threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
    __syncthreads();
  }
  if (threadIdx.x == 0) score[blk] = red[0] / ((double)b * (double)b) + 0.0;  // + 0.0: no negative zero
}

__global__ void k_fill_u8(uint8_t* p, int64_t n, uint8_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ void k_fill_i32(int* p, int64_t n, int v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Bit pattern of a double mapped to an unsigned integer with the same order (any finite sign; -0.0 is
// canonicalised to +0.0 by the scoring kernels, so equal scores have equal keys).
__device__ __forceinline__ unsigned long long order_key(unsigned long long bits) {
  return (bits >> 63) ? ~bits : (bits | 0x8000000000000000ull);
}

// Exact selection of the n_keep highest scores (0 < n_keep < n), compared through
// order-preserving integer keys.
// An 8-pass most-significant-digit radix select finds the n_keep-th largest
// pattern; everything above it is kept, and of the entries equal to it the
// first ones in index order fill the remaining quota.
// The passes read the keys from global memory only until the keys that still share the selected prefix
// fit in LDS (kSelectCand of them); those are then collected once and the remaining passes run on LDS.
constexpr int kSelectCand = 4096;

// Workgroup 1 of a two-workgroup launch selects from a second score array into a second mask (the mask update
// of prune-and-grow ranks the weight and the gradient at the same sparsity: the two selections run side by side).
__global__ __launch_bounds__(1024) void k_select_topk(const double* __restrict__ score0, int64_t n, int64_t n_keep,
                                                      uint8_t* __restrict__ mask0,
                                                      const double* __restrict__ score1 = nullptr,
                                                      uint8_t* __restrict__ mask1 = nullptr) {
  const double* __restrict__ score = blockIdx.x == 0 ? score0 : score1;
  uint8_t* __restrict__ mask = blockIdx.x == 0 ? mask0 : mask1;
  __shared__ unsigned long long cand[kSelectCand];
  __shared__ unsigned hist[256];
  __shared__ unsigned long long s_prefix;
  __shared__ long long s_remaining;
  __shared__ int wave_tot[16];
  __shared__ long long s_running;
  __shared__ long long s_eq_total;
  __shared__ int s_ncand;  // < 0: the candidates are still the whole array
  __shared__ int s_fill;
  __shared__ unsigned s_h;
  const unsigned long long* key = reinterpret_cast<const unsigned long long*>(score);
  const int lane = lane_id();
  const bool pairs_ok = (reinterpret_cast<uintptr_t>(score) & 15u) == 0;
  if (threadIdx.x == 0) {
    s_prefix = 0ull;
    s_remaining = n_keep;
    s_running = 0;
    s_eq_total = 0;
    s_ncand = n <= kSelectCand ? (int)n : -1;
    s_fill = 0;
    s_h = 0u;
  }
  if (n <= kSelectCand)
    for (int i = threadIdx.x; i < (int)n; i += blockDim.x) cand[i] = order_key(key[i]);
  for (int pass = 7; pass >= 0; --pass) {
    if (threadIdx.x < 256) hist[threadIdx.x] = 0u;
    __syncthreads();
    const unsigned long long prefix = s_prefix;
    const unsigned long long himask = (pass == 7) ? 0ull : (~0ull << (8 * (pass + 1)));
    const int ncand = s_ncand;
    if (ncand >= 0) {
      for (int i = threadIdx.x; i < ncand; i += blockDim.x) {
        const unsigned long long k = cand[i];
        if ((k & himask) == prefix) atomicAdd(&hist[(unsigned)(k >> (8 * pass)) & 255u], 1u);
      }
    } else {
      // A thread adds a run of equal digits with one atomic: in the leading passes, where scores of similar
      // magnitude all carry the same digit, every key would otherwise hit the same LDS word.
      unsigned run_bin = 0u, run_len = 0u;
      auto count = [&](unsigned long long raw) {
        const unsigned long long k = order_key(raw);
        if ((k & himask) == prefix) {
          const unsigned bin = (unsigned)(k >> (8 * pass)) & 255u;
          if (run_len != 0u && bin != run_bin) {
            atomicAdd(&hist[run_bin], run_len);
            run_len = 0u;
          }
          run_bin = bin;
          ++run_len;
        }
      };
      // two keys per load, eight loads in flight: one workgroup walks the whole array, so the walk is
      // bound by how many bytes it keeps in flight
      const int64_t npair = pairs_ok ? n / 2 : 0;
      const ulonglong2* key2 = reinterpret_cast<const ulonglong2*>(key);
#pragma unroll 8
      for (int64_t p = threadIdx.x; p < npair; p += blockDim.x) {
        const ulonglong2 kk = key2[p];
        count(kk.x);
        count(kk.y);
      }
      for (int64_t i = 2 * npair + threadIdx.x; i < n; i += blockDim.x) count(key[i]);
      if (run_len != 0u) atomicAdd(&hist[run_bin], run_len);
    }
    __syncthreads();
    // Digit d of this pass: the bin where the count of larger digits, S(d), first satisfies
    // S(d) < remaining <= S(d) + hist[d].  One thread per bin; the suffix sums come from a scan of the
    // bins in descending order.
    {
      const long long rem = s_remaining;
      const int d = 255 - (int)threadIdx.x;  // thread t looks at bin 255 - t
      const int h = (threadIdx.x < 256) ? (int)hist[d & 255] : 0;
      int total;
      const int larger = block_exscan(h, wave_tot, total);  // sum of hist over digits > d
      __syncthreads();
      if (threadIdx.x < 256 && (long long)larger < rem && rem <= (long long)larger + h) {
        s_remaining = rem - larger;
        s_prefix = prefix | ((unsigned long long)d << (8 * pass));
        s_h = (unsigned)h;              // keys that share the prefix including this digit
        if (pass == 0) s_eq_total = h;  // entries equal to the n_keep-th largest
      }
    }
    __syncthreads();
    if (ncand < 0 && pass > 0 && s_h <= (unsigned)kSelectCand) {
      // collect the keys that carry the new prefix (exactly s_h of them); their order does not matter
      const unsigned long long newmask = ~0ull << (8 * pass), newprefix = s_prefix;
      for (int64_t base = 0; base < n; base += 4 * (int64_t)blockDim.x) {
        unsigned long long k[4];
        bool in[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int64_t i = base + u * (int64_t)blockDim.x + threadIdx.x;
          in[u] = i < n;
          k[u] = in[u] ? order_key(key[i]) : 0ull;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const bool take = in[u] && (k[u] & newmask) == newprefix;
          const unsigned long long bal = __ballot(take);
          int wbase = 0;
          if (lane == 0 && bal != 0ull) wbase = atomicAdd(&s_fill, __popcll(bal));
          wbase = __shfl(wbase, 0, kWave);
          if (take) cand[wbase + __popcll(bal & ((1ull << lane) - 1ull))] = k[u];
        }
      }
      __syncthreads();
      if (threadIdx.x == 0) s_ncand = s_fill;
      __syncthreads();
    }
  }
  const unsigned long long kth = s_prefix;
  const long long need_eq = s_remaining;
  if (need_eq == s_eq_total) {
    // every entry equal to the threshold is kept (always so when the scores are distinct): no ordering needed
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) mask[i] = order_key(key[i]) >= kth ? 1 : 0;
    return;
  }
  for (int64_t base = 0; base < n; base += blockDim.x) {
    const int64_t i = base + threadIdx.x;
    const unsigned long long k = (i < n) ? order_key(key[i]) : 0ull;
    const int eq = (i < n && k == kth) ? 1 : 0;
    int total;
    const long long pos = s_running + block_exscan(eq, wave_tot, total);
    if (i < n) mask[i] = (k > kth || (eq && pos < need_eq)) ? 1 : 0;
    __syncthreads();
    if (threadIdx.x == 0) s_running += total;
    __syncthreads();
  }
}

// One wave per line: population of mask along a row (stride 1) or a column (stride nbc).
__global__ __launch_bounds__(256) void k_line_counts(const uint8_t* __restrict__ mask, int n_lines, int line_len,
                                                     int64_t line_stride, int64_t elem_stride, int* __restrict__ cnt) {
  const int line = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (line >= n_lines) return;
  int c = 0;
  for (int j = lane_id(); j < line_len; j += kWave) c += mask[line * line_stride + j * elem_stride] ? 1 : 0;
#pragma unroll
  for (int d = kWave / 2; d > 0; d >>= 1) c += __shfl_xor(c, d, kWave);
  if (lane_id() == 0) cnt[line] = c;
}

// Single workgroup: ptr[0..n] = exclusive scan of cnt[0..n).  total_out (may be null) gets ptr[n].
__global__ __launch_bounds__(1024) void k_exscan(const int* __restrict__ cnt, int n, int* __restrict__ ptr,
                                                 int* __restrict__ total_out) {
  __shared__ int wave_tot[16];
  __shared__ int s_running;
  if (threadIdx.x == 0) s_running = 0;
  __syncthreads();
  for (int base = 0; base < n; base += blockDim.x) {
    const int i = base + threadIdx.x;
    const int v = (i < n) ? cnt[i] : 0;
    int total;
    const int ex = s_running + block_exscan(v, wave_tot, total);
    if (i < n) ptr[i] = ex;
    __syncthreads();
    if (threadIdx.x == 0) s_running += total;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    ptr[n] = s_running;
    if (total_out) *total_out = s_running;
  }
}

// One workgroup per block row: kept block columns, ascending, into col_idx; the
// owning block row of every stored block into blk_row (for the gather).
__global__ __launch_bounds__(256) void k_fill_cols(const uint8_t* __restrict__ mask, int nbc,
                                                   const int* __restrict__ row_ptr, int* __restrict__ col_idx,
                                                   int* __restrict__ blk_row, int64_t nnz_cap) {
  __shared__ int wave_tot[16];
  const int br = blockIdx.x;
  const int start = row_ptr[br];
  int running = 0;
  for (int base = 0; base < nbc; base += blockDim.x) {
    const int c = base + threadIdx.x;
    const int f = (c < nbc && mask[(int64_t)br * nbc + c]) ? 1 : 0;
    int total;
    const int pos = running + block_exscan(f, wave_tot, total);
    if (f) {
      const int64_t k = (int64_t)start + pos;
      if (k < nnz_cap) {
        col_idx[k] = c;
        blk_row[k] = br;
      }
    }
    running += total;
  }
}

// One workgroup per stored block: copy its b x b values, row-major, 16 bytes per lane.  A block whose mask
// code is 2 (regrown, BLaST Sec. 3.2) is stored as zeros: it joins the structure without changing the product.
// (The grid is sized by the capacity: workgroups past the number of stored blocks leave.)
__global__ __launch_bounds__(256) void k_gather_blocks(const uint16_t* __restrict__ W, int64_t ldw, int b,
                                                       const int* __restrict__ col_idx, const int* __restrict__ blk_row,
                                                       const uint8_t* __restrict__ mask, int nbc,
                                                       uint16_t* __restrict__ vals, const int* __restrict__ nnz_dev) {
  const int64_t k = blockIdx.x;
  if (k >= *nnz_dev) return;
  const int64_t br = blk_row[k], bc = col_idx[k];
  const uint16_t* src = W + br * b * ldw + bc * b;
  uint16_t* dst = vals + k * b * b;
  const int cpr = b / 8, nchunks = b * cpr;
  const bool zero = mask[br * nbc + bc] == 2;
  for (int c = threadIdx.x; c < nchunks; c += 256) {
    const int i = c / cpr, j8 = c % cpr;
    *reinterpret_cast<uint4*>(dst + (int64_t)c * 8) =
        zero ? uint4{0u, 0u, 0u, 0u} : *reinterpret_cast<const uint4*>(src + (int64_t)i * ldw + j8 * 8);
  }
}

// out = 1 where the weight's own selection keeps the block, 2 where only the gradient's does, else 0
__global__ __launch_bounds__(256) void k_merge_masks(const uint8_t* __restrict__ mw, const uint8_t* __restrict__ mg,
                                                     int64_t n, uint8_t* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = mw[i] ? 1 : (mg[i] ? 2 : 0);
}

// row_order[rank] = r with rank = number of rows that sort before r under
// (population descending, row index ascending) -- a stable sort by counting.
// row_ptr2 (may be null) adds the populations of a second matrix with the same block rows.
__global__ __launch_bounds__(256) void k_row_order(const int* __restrict__ row_ptr, const int* __restrict__ row_ptr2,
                                                   int nbr, int* __restrict__ row_order) {
  // the populations pass through LDS in slabs: every thread compares its row with all of them
  constexpr int kSlab = 2048;
  __shared__ __attribute__((aligned(16))) int cnt[kSlab];
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  int cr = 0;
  if (r < nbr) {
    cr = row_ptr[r + 1] - row_ptr[r];
    if (row_ptr2) cr += row_ptr2[r + 1] - row_ptr2[r];
  }
  int rank = 0;
  for (int base = 0; base < nbr; base += kSlab) {
    const int m = nbr - base < kSlab ? nbr - base : kSlab;
    __syncthreads();
    for (int q = threadIdx.x; q < m; q += blockDim.x) {
      int cq = row_ptr[base + q + 1] - row_ptr[base + q];
      if (row_ptr2) cq += row_ptr2[base + q + 1] - row_ptr2[base + q];
      cnt[q] = cq;
    }
    __syncthreads();
    if (r < nbr) {
      // four populations per LDS read, several reads in flight: a serial chain of single reads would cost
      // one LDS round trip per row
      int q = 0;
#pragma unroll 4
      for (; q + 4 <= m; q += 4) {
        const int4 c4 = *reinterpret_cast<const int4*>(&cnt[q]);
        rank += (c4.x > cr || (c4.x == cr && base + q < r)) ? 1 : 0;
        rank += (c4.y > cr || (c4.y == cr && base + q + 1 < r)) ? 1 : 0;
        rank += (c4.z > cr || (c4.z == cr && base + q + 2 < r)) ? 1 : 0;
        rank += (c4.w > cr || (c4.w == cr && base + q + 3 < r)) ? 1 : 0;
      }
      for (; q < m; ++q) {
        const int cq = cnt[q];
        rank += (cq > cr || (cq == cr && base + q < r)) ? 1 : 0;
      }
    }
  }
  if (r < nbr) row_order[rank] = r;
}

// One workgroup per block column: its stored blocks by ascending block row; for
// each, the block row and the position k of the block in vals / col_idx.
// csc_blk null: it follows csc_row at the next 16-byte boundary after nnz entries, nnz read from nnz_dev (the
// layout of the aux buffer; nothing is written when nnz exceeds the capacity).
__global__ __launch_bounds__(256) void k_fill_csc(const uint8_t* __restrict__ mask, int nbr, int nbc,
                                                  const int* __restrict__ row_ptr, const int* __restrict__ col_idx,
                                                  const int* __restrict__ col_ptr, int* __restrict__ csc_row,
                                                  int* __restrict__ csc_blk, int64_t nnz_cap,
                                                  const int* __restrict__ nnz_dev) {
  __shared__ int wave_tot[16];
  if (!csc_blk) {
    const int64_t nnz = *nnz_dev;
    if (nnz > nnz_cap) return;
    csc_blk = csc_row + (nnz + 3) / 4 * 4;
  }
  const int c = blockIdx.x;
  const int start = col_ptr[c];
  int running = 0;
  for (int base = 0; base < nbr; base += blockDim.x) {
    const int r = base + threadIdx.x;
    const int f = (r < nbr && mask[(int64_t)r * nbc + c]) ? 1 : 0;
    int total;
    const int pos = running + block_exscan(f, wave_tot, total);
    if (f) {
      int lo = row_ptr[r], hi = row_ptr[r + 1] - 1;  // col_idx ascending in the row: find c
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (col_idx[mid] < c) lo = mid + 1; else hi = mid;
      }
      const int64_t e = (int64_t)start + pos;
      if (e < nnz_cap) {
        csc_row[e] = r;
        csc_blk[e] = lo;
      }
    }
    running += total;
  }
}

// Where one chunk plan goes.
struct PlanOut {
  int chunk;        // blocks per chunk, at most
  int* hdr;         // {n_chunks, max_row_blocks, chunk, chunks of the rows that have several}
  int* chunk_row;
  int* chunk_kb;
  int* chunk_ke;
  int64_t cap;
  int* row_slot;    // may be null: per row, its rank if it has several chunks, else -1
  int* row_chunk0;  // may be null: per row, the index of its first chunk if it has several, else -1
};

// Cuts the block rows, in schedule order, into chunks of at most `chunk` blocks, once per requested plan; run by
// every thread of one workgroup.  An empty row still gets one (empty) chunk: its output has to be written.
// `sh` is LDS scratch of 3 ints.
__device__ __forceinline__ void chunk_plans(const int* row_ptr, const int* row_order, int nbr, const PlanOut& narrow,
                                            const PlanOut& wide, int* __restrict__ max_row_out, int* wave_tot,
                                            int* sh) {
  int& s_running = sh[0];
  int& s_heavy = sh[1];
  int& s_split = sh[2];
  for (int which = 0; which < 2; ++which) {
    const PlanOut o = which ? wide : narrow;
    const int chunk = o.chunk;
    __syncthreads();
    if (threadIdx.x == 0) {
      s_running = 0;
      s_heavy = 0;
      s_split = 0;
    }
    __syncthreads();
    for (int base = 0; base < nbr; base += blockDim.x) {
      const int rank = base + threadIdx.x;
      int r = 0, kb = 0, ke = 0, nch = 0;
      if (rank < nbr) {
        r = row_order[rank];
        kb = row_ptr[r];
        ke = row_ptr[r + 1];
        nch = (ke - kb + chunk - 1) / chunk;
        if (nch < 1) nch = 1;
        atomicMax(&s_heavy, ke - kb);
        if (nch > 1) atomicAdd(&s_split, nch);
        if (o.row_slot) o.row_slot[r] = nch > 1 ? rank : -1;
      }
      int total;
      const int first = s_running + block_exscan(nch, wave_tot, total);
      if (rank < nbr && o.row_chunk0) o.row_chunk0[r] = nch > 1 ? first : -1;
      for (int j = 0; j < nch; ++j) {
        const int64_t e = (int64_t)first + j;
        if (e < o.cap) {
          o.chunk_row[e] = r | (nch > 1 ? (int)0x80000000u : 0);
          const int b0 = kb + j * chunk;
          o.chunk_kb[e] = b0;
          o.chunk_ke[e] = (b0 + chunk < ke) ? b0 + chunk : ke;
        }
      }
      __syncthreads();
      if (threadIdx.x == 0) s_running += total;
      __syncthreads();
    }
    if (threadIdx.x == 0) {
      o.hdr[0] = s_running;
      o.hdr[1] = s_heavy;
      if (which == 0) *max_row_out = s_heavy;  // next to nnz, so that one copy brings both to the host
      o.hdr[2] = chunk;
      o.hdr[3] = s_split;
    }
  }
}

// Single workgroup: both chunk plans of a matrix.
__global__ __launch_bounds__(1024) void k_chunk_plan(const int* __restrict__ row_ptr, const int* __restrict__ row_order,
                                                     int nbr, PlanOut narrow, PlanOut wide,
                                                     int* __restrict__ max_row_out) {
  __shared__ int wave_tot[16];
  __shared__ int sh[3];
  chunk_plans(row_ptr, row_order, nbr, narrow, wide, max_row_out, wave_tot, sh);
}

// Both plans of a matrix, placed in its aux buffer.
inline void plan_outputs(char* ab, const blast::AuxLayout& A, PlanOut& narrow, PlanOut& wide) {
  narrow = PlanOut{blast::kChunkBlocks, reinterpret_cast<int*>(ab + A.hdr_off), reinterpret_cast<int*>(ab + A.chunk_row_off),
                   reinterpret_cast<int*>(ab + A.chunk_kb_off), reinterpret_cast<int*>(ab + A.chunk_ke_off), A.chunk_cap,
                   reinterpret_cast<int*>(ab + A.row_slot_off), reinterpret_cast<int*>(ab + A.row_chunk0_off)};
  wide = PlanOut{blast::kWideChunkBlocks, reinterpret_cast<int*>(ab + A.whdr_off), reinterpret_cast<int*>(ab + A.wchunk_row_off),
                 reinterpret_cast<int*>(ab + A.wchunk_kb_off), reinterpret_cast<int*>(ab + A.wchunk_ke_off), A.wchunk_cap,
                 nullptr, nullptr};
}

// ---- small matrices: selection and every index array in one workgroup ----
//
// A layer-sized matrix has a few thousand blocks; scored, the rest of the packing is a few thousand integer
// operations, and as a dozen dependent launches it costs a dozen launch latencies.  For at most kSmallN blocks
// (and at most 1024 block rows and block columns) one workgroup does it all: a thread owns `per` consecutive
// blocks in row-major order and keeps their keys in registers; the mask, the position of every stored block and
// the per-line populations live in LDS.  The workgroup's 16 waves share one compute unit, so what the kernel
// costs is instructions per thread: no integer division per block, both scans of a pair in one (two 16-bit
// counts in one word: no sum here exceeds kSmallN + 1024), barriers that do not wait for global stores.
constexpr int kSmallPer = 8;
constexpr int kSmallN = 1024 * kSmallPer;
static_assert(kSmallN + 1024 < 65536, "two counts share a 32-bit word");
static_assert((blast::kChunkBlocks & (blast::kChunkBlocks - 1)) == 0 &&
              (blast::kWideChunkBlocks & (blast::kWideChunkBlocks - 1)) == 0, "chunk sizes are powers of two");

// LDS scratch of select_small.
struct SelectShared {
  unsigned hist[256];
  int wave_tot[16];
  unsigned long long prefix, kth;
  long long remaining;
  unsigned h;
};

// Exact selection of the n_keep highest of n <= kSmallN scores by one workgroup of 1024 threads: thread t owns
// scores t * per ... t * per + per - 1 (per = ceil(n / 1024)) and returns their keep flags (bit j: score
// t * per + j is kept).  Equal scores are kept in index order.
__device__ __forceinline__ unsigned select_small(const double* __restrict__ score, int n, long long n_keep, int per,
                                                 SelectShared& sh) {
  const int tid = threadIdx.x, lane = lane_id();
  const int e0 = tid * per;
  unsigned* hist = sh.hist;
  int* wave_tot = sh.wave_tot;
  unsigned long long& s_prefix = sh.prefix;
  unsigned long long& s_kth = sh.kth;
  long long& s_remaining = sh.remaining;
  unsigned& s_h = sh.h;
  unsigned keep = 0u;
  {
    unsigned long long key[kSmallPer];
#pragma unroll
    for (int j = 0; j < kSmallPer; ++j)
      key[j] = (j < per && e0 + j < n) ? order_key(reinterpret_cast<const unsigned long long*>(score)[e0 + j]) : 0ull;
    if (n_keep <= 0 || n_keep >= n) {
#pragma unroll
      for (int j = 0; j < kSmallPer; ++j) keep |= (j < per && e0 + j < n && n_keep > 0) ? 1u << j : 0u;
    } else {
      // Most-significant-digit radix select of the n_keep-th largest key.  Scores of one matrix share their
      // leading bits (sign, exponent, often the first mantissa bits), and a digit that every key carries would
      // send every count to one LDS word: the bits above the highest one in which any two keys differ are taken
      // as they are, the passes start below them, eight bits at a time, and stop as soon as a single key
      // carries the selected prefix.
      unsigned long long diff = 0ull;
      const unsigned long long key0 = order_key(reinterpret_cast<const unsigned long long*>(score)[0]);
#pragma unroll
      for (int j = 0; j < kSmallPer; ++j)
        if (j < per && e0 + j < n) diff |= key[j] ^ key0;
#pragma unroll
      for (int d = kWave / 2; d > 0; d >>= 1) diff |= __shfl_xor(diff, d, kWave);
      if (tid == 0) s_kth = 0ull;
      wg_barrier<true>();
      if (lane == 0 && diff != 0ull) atomicOr(&s_kth, diff);
      wg_barrier<true>();
      diff = s_kth;
      int fixed = diff == 0ull ? 0 : 64 - __clzll(diff);  // bits at and above this position are decided
      unsigned long long prefix = fixed == 64 ? 0ull : (key0 >> fixed) << fixed;
      long long rem = n_keep;
      unsigned eq_total = (unsigned)n;  // keys that carry the decided bits
      while (fixed > 0) {
        const int sft = fixed > 8 ? fixed - 8 : 0, width = fixed - sft;
        if (tid < 256) hist[tid] = 0u;
        wg_barrier<true>();
#pragma unroll
        for (int j = 0; j < kSmallPer; ++j) {
          if (j < per) {
            const bool in = e0 + j < n && (fixed == 64 || (key[j] >> fixed) == (prefix >> fixed));
            if (in) atomicAdd(&hist[(unsigned)(key[j] >> sft) & ((1u << width) - 1u)], 1u);
          }
        }
        wg_barrier<true>();
        if (tid < kWave) {
          // lane l looks at bins 255 - 4l ... 252 - 4l; `larger` = keys in bins above the one looked at
          unsigned h4[4], sum = 0u;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            h4[u] = hist[255 - 4 * lane - u];
            sum += h4[u];
          }
          unsigned inc = sum;
#pragma unroll
          for (int d = 1; d < kWave; d <<= 1) {
            const unsigned v = __shfl_up(inc, d, kWave);
            if (lane >= d) inc += v;
          }
          long long larger = (long long)(inc - sum);
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const long long h = h4[u];
            if (larger < rem && rem <= larger + h) {
              s_remaining = rem - larger;
              s_prefix = prefix | ((unsigned long long)(255 - 4 * lane - u) << sft);
              s_h = (unsigned)h;
            }
            larger += h;
          }
        }
        wg_barrier<true>();
        prefix = s_prefix;
        rem = s_remaining;
        eq_total = s_h;
        fixed = sft;
        if (eq_total == 1u && fixed > 0) {
#pragma unroll
          for (int j = 0; j < kSmallPer; ++j)
            if (j < per && e0 + j < n && (key[j] >> fixed) == (prefix >> fixed)) s_kth = key[j];
          wg_barrier<true>();
          prefix = s_kth;
          break;
        }
      }
      const unsigned long long kth = prefix;
      if (rem == (long long)eq_total) {
#pragma unroll
        for (int j = 0; j < kSmallPer; ++j) keep |= (j < per && e0 + j < n && key[j] >= kth) ? 1u << j : 0u;
      } else {
        // of the keys equal to the threshold the first `rem` in index order are kept
        int neq = 0;
#pragma unroll
        for (int j = 0; j < kSmallPer; ++j) neq += (j < per && e0 + j < n && key[j] == kth) ? 1 : 0;
        int total;
        long long pos = block_exscan<true>(neq, wave_tot, total);
#pragma unroll
        for (int j = 0; j < kSmallPer; ++j) {
          if (j < per && e0 + j < n) {
            const bool eq = key[j] == kth;
            if (key[j] > kth || (eq && pos < rem)) keep |= 1u << j;
            pos += eq ? 1 : 0;
          }
        }
      }
    }
  }
  return keep;
}

// One workgroup: mask[i] = 1 for the n_keep highest of n <= kSmallN scores, else 0.
__global__ __launch_bounds__(1024) void k_select_small(const double* __restrict__ score, int n, long long n_keep,
                                                       uint8_t* __restrict__ mask) {
  __shared__ SelectShared ssh;
  const int per = (n + 1023) >> 10, e0 = threadIdx.x * per;
  const unsigned keep = select_small(score, n, n_keep, per, ssh);
#pragma unroll
  for (int j = 0; j < kSmallPer; ++j)
    if (j < per && e0 + j < n) mask[e0 + j] = (keep >> j) & 1u;
}

// One workgroup: the mask update of prune-and-grow on n <= kSmallN blocks - both selections and their merge
// (1 where the weight's selection keeps the block, 2 where only the gradient's does, else 0).
__global__ __launch_bounds__(1024) void k_masks_small(const double* __restrict__ score_w,
                                                      const double* __restrict__ score_g, int n, long long n_keep,
                                                      uint8_t* __restrict__ mask) {
  __shared__ SelectShared ssh;
  const int per = (n + 1023) >> 10, e0 = threadIdx.x * per;
  const unsigned keep_w = select_small(score_w, n, n_keep, per, ssh);
  wg_barrier<true>();  // the scratch is used again
  const unsigned keep_g = select_small(score_g, n, n_keep, per, ssh);
#pragma unroll
  for (int j = 0; j < kSmallPer; ++j)
    if (j < per && e0 + j < n) mask[e0 + j] = ((keep_w >> j) & 1u) ? 1 : (((keep_g >> j) & 1u) ? 2 : 0);
}

struct SmallOut {
  int* row_ptr;
  int* col_idx;
  int* blk_row;
  int* row_order;
  uint8_t* mask_out;  // may be null (the caller's mask is the mask)
  int* col_ptr;       // null without aux
  int* csc_row;       // csc_blk follows at the next 16-byte boundary after nnz entries
  int* scalars;       // {nnz, max_row_blocks}
  int64_t nnz_cap;
};

template <bool TOPK>
__global__ __launch_bounds__(1024) void k_pack_small(const double* __restrict__ score,
                                                     const uint8_t* __restrict__ mask_in, int nbr, int nbc,
                                                     long long n_keep, SmallOut o, PlanOut narrow, PlanOut wide) {
  __shared__ int kpos[kSmallN];  // position of a stored block in col_idx / vals, by row-major block index
  __shared__ uint8_t m[kSmallN];
  __shared__ __attribute__((aligned(16))) int rcnt[1024];
  __shared__ int ccnt[1024];
  __shared__ int rptr[1025];
  __shared__ int rord[1024];
  __shared__ SelectShared ssh;
  __shared__ int sh[3];
  int* wave_tot = ssh.wave_tot;
  const int tid = threadIdx.x;
  const int n = nbr * nbc;
  const int per = (n + 1023) >> 10;  // blocks per thread (uniform); the loops below are unrolled to kSmallPer
  const int e0 = tid * per;
  rcnt[tid] = 0;
  ccnt[tid] = 0;
  unsigned keep = 0u;  // bit j: block e0 + j is kept
  if (TOPK) {
    keep = select_small(score, n, n_keep, per, ssh);
  } else {
#pragma unroll
    for (int j = 0; j < kSmallPer; ++j) keep |= (j < per && e0 + j < n && mask_in[e0 + j] != 0) ? 1u << j : 0u;
  }

  // stored blocks in row-major order: the position of a block is the number of kept blocks before it
  int nnz;
  int k = block_exscan<true>(__popc(keep), wave_tot, nnz);  // (its barriers also cover the clearing of rcnt / ccnt)
  {
    int r = e0 / nbc, c = e0 - r * nbc;
#pragma unroll
    for (int j = 0; j < kSmallPer; ++j) {
      if (j < per && e0 + j < n) {
        const bool kp = (keep >> j) & 1u;
        m[e0 + j] = kp ? 1 : 0;
        if (o.mask_out) o.mask_out[e0 + j] = kp ? 1 : 0;
        if (kp) {
          kpos[e0 + j] = k;
          if (k < o.nnz_cap) {
            o.col_idx[k] = c;
            o.blk_row[k] = r;
          }
          atomicAdd(&rcnt[r], 1);
          atomicAdd(&ccnt[c], 1);
          ++k;
        }
        if (++c == nbc) {
          c = 0;
          ++r;
        }
      }
    }
  }
  wg_barrier<true>();

  // row pointers and column pointers: one scan of both populations
  {
    const int v = (tid < nbr ? rcnt[tid] : 0) | ((tid < nbc ? ccnt[tid] : 0) << 16);
    int total;
    const int ex = block_exscan<true>(v, wave_tot, total);
    if (tid < nbr) {
      rptr[tid] = ex & 0xFFFF;
      o.row_ptr[tid] = ex & 0xFFFF;
    }
    if (o.col_ptr && tid < nbc) o.col_ptr[tid] = ex >> 16;
    if (tid == 0) {
      rptr[nbr] = nnz;
      o.row_ptr[nbr] = nnz;
      if (o.col_ptr) o.col_ptr[nbc] = nnz;
      o.scalars[0] = nnz;
      if (!o.col_ptr) o.scalars[1] = 0;
    }
  }
  // schedule: rows by population, descending, stable.  P threads share a row, each comparing it with a
  // contiguous part of the rows (four populations per LDS read; the array is zero beyond nbr, which never counts).
  {
    const int pl = 31 - __clz(1024 / nbr);         // log2 P, P = largest power of two <= 1024 / nbr ...
    const int lp = pl > 6 ? 6 : pl, P = 1 << lp;   // ... and <= 64, so that the P threads sit in one wave
    const int r = tid >> lp, part = tid & (P - 1);
    const int len = (((nbr + P - 1) >> lp) + 3) & ~3;
    const int cr = r < nbr ? rcnt[r] : 0;
    int rank = 0;
    const int q0 = part * len;
#pragma unroll 4
    for (int q = q0; q < q0 + len; q += 4) {
      const int4 c4 = *reinterpret_cast<const int4*>(&rcnt[q]);
      rank += (c4.x > cr || (c4.x == cr && q < r)) ? 1 : 0;
      rank += (c4.y > cr || (c4.y == cr && q + 1 < r)) ? 1 : 0;
      rank += (c4.z > cr || (c4.z == cr && q + 2 < r)) ? 1 : 0;
      rank += (c4.w > cr || (c4.w == cr && q + 3 < r)) ? 1 : 0;
    }
    for (int d = P >> 1; d > 0; d >>= 1) rank += __shfl_xor(rank, d, kWave);
    if (r < nbr && part == 0) {
      rord[rank] = r;
      o.row_order[rank] = r;
    }
  }
  wg_barrier<true>();
  if (!o.col_ptr) return;

  // both chunk plans: rows in schedule order, cut into chunks of at most 16 / 64 blocks (an empty row still gets
  // one chunk: its output has to be written)
  {
    if (tid == 0) {
      sh[0] = 0;  // fullest row
      sh[1] = 0;  // chunks of the rows that the first plan cuts
      sh[2] = 0;  // ... the second plan
    }
    wg_barrier<true>();
    constexpr int ls0 = __builtin_ctz(blast::kChunkBlocks), ls1 = __builtin_ctz(blast::kWideChunkBlocks);
    int r = 0, kb = 0, ke = 0, n0 = 0, n1 = 0;
    if (tid < nbr) {
      r = rord[tid];
      kb = rptr[r];
      ke = rptr[r + 1];
      n0 = (ke - kb + (1 << ls0) - 1) >> ls0;
      n1 = (ke - kb + (1 << ls1) - 1) >> ls1;
      n0 = n0 < 1 ? 1 : n0;
      n1 = n1 < 1 ? 1 : n1;
      atomicMax(&sh[0], ke - kb);
      if (n0 > 1) atomicAdd(&sh[1], n0);
      if (n1 > 1) atomicAdd(&sh[2], n1);
      narrow.row_slot[r] = n0 > 1 ? tid : -1;
    }
    int total;
    const int first = block_exscan<true>(n0 | (n1 << 16), wave_tot, total);
    if (tid < nbr) {
      const int f0 = first & 0xFFFF, f1 = first >> 16;
      narrow.row_chunk0[r] = n0 > 1 ? f0 : -1;
      for (int j = 0; j < n0; ++j) {
        const int e = f0 + j, b0 = kb + (j << ls0);
        if (e < narrow.cap) {
          narrow.chunk_row[e] = r | (n0 > 1 ? (int)0x80000000u : 0);
          narrow.chunk_kb[e] = b0;
          narrow.chunk_ke[e] = (b0 + (1 << ls0) < ke) ? b0 + (1 << ls0) : ke;
        }
      }
      for (int j = 0; j < n1; ++j) {
        const int e = f1 + j, b0 = kb + (j << ls1);
        if (e < wide.cap) {
          wide.chunk_row[e] = r | (n1 > 1 ? (int)0x80000000u : 0);
          wide.chunk_kb[e] = b0;
          wide.chunk_ke[e] = (b0 + (1 << ls1) < ke) ? b0 + (1 << ls1) : ke;
        }
      }
    }
    if (tid == 0) {
      const int heavy = sh[0];
      narrow.hdr[0] = total & 0xFFFF;
      narrow.hdr[1] = heavy;
      narrow.hdr[2] = 1 << ls0;
      narrow.hdr[3] = sh[1];
      wide.hdr[0] = total >> 16;
      wide.hdr[1] = heavy;
      wide.hdr[2] = 1 << ls1;
      wide.hdr[3] = sh[2];
      o.scalars[1] = heavy;
    }
  }

  // column-grouped index: the same count with the blocks taken in column-major order
  if (nnz > o.nnz_cap) return;
  {
    int* csc_blk = o.csc_row + (nnz + 3) / 4 * 4;
    unsigned keep_c = 0u;
    const int c0 = e0 / nbr, r0 = e0 - c0 * nbr;
    {
      int r = r0, at = r0 * nbc + c0;
#pragma unroll
      for (int j = 0; j < kSmallPer; ++j) {
        if (j < per && e0 + j < n) {
          keep_c |= m[at] ? 1u << j : 0u;
          at += nbc;
          if (++r == nbr) {
            r = 0;
            at = at - n + 1;  // top of the next column
          }
        }
      }
    }
    int total;
    int e = block_exscan<true>(__popc(keep_c), wave_tot, total);
    int r = r0, at = r0 * nbc + c0;
#pragma unroll
    for (int j = 0; j < kSmallPer; ++j) {
      if (j < per && e0 + j < n) {
        if ((keep_c >> j) & 1u) {
          o.csc_row[e] = r;
          csc_blk[e] = kpos[at];
          ++e;
        }
        at += nbc;
        if (++r == nbr) {
          r = 0;
          at = at - n + 1;
        }
      }
    }
  }
}

// One workgroup per stored block of the transposed matrix: block e of the output is the transpose of
// block src_blk[e] of the input.  Rows are read and written whole; the turn happens in LDS (row pitch
// b + 2 elements, so that a column walk does not stay on one bank).
__global__ __launch_bounds__(256) void k_transpose_blocks(const uint16_t* __restrict__ vals, int b,
                                                          const int* __restrict__ src_blk,
                                                          uint16_t* __restrict__ vals_t) {
  extern __shared__ uint16_t tile[];
  const int pitch = b + 2;
  const uint16_t* src = vals + (int64_t)src_blk[blockIdx.x] * b * b;
  uint16_t* dst = vals_t + (int64_t)blockIdx.x * b * b;
  for (int idx = threadIdx.x; idx < b * b; idx += blockDim.x) tile[(idx / b) * pitch + idx % b] = src[idx];
  __syncthreads();
  for (int idx = threadIdx.x; idx < b * b; idx += blockDim.x) dst[idx] = tile[(idx % b) * pitch + idx / b];
}

// One workgroup per block of the dense matrix: copies the stored block there, or writes zeros where the
// block row's column list (ascending) has no entry for it.
__global__ __launch_bounds__(256) void k_unpack_blocks(const int* __restrict__ row_ptr, const int* __restrict__ col_idx,
                                                       const uint16_t* __restrict__ vals, int nbc, int b,
                                                       uint16_t* __restrict__ W, int64_t ldw) {
  const int64_t blk = blockIdx.x;
  const int br = (int)(blk / nbc), bc = (int)(blk % nbc);
  int lo = row_ptr[br], hi = row_ptr[br + 1];
  int k = -1;
  while (lo < hi) {  // binary search for bc in [lo, hi)
    const int mid = (lo + hi) >> 1;
    const int c = col_idx[mid];
    if (c == bc) {
      k = mid;
      break;
    }
    if (c < bc) lo = mid + 1; else hi = mid;
  }
  uint16_t* dst = W + (int64_t)br * b * ldw + (int64_t)bc * b;
  const uint16_t* src = k >= 0 ? vals + (int64_t)k * b * b : nullptr;
  const int cpr = b / 8, nchunks = b * cpr;
  for (int c = threadIdx.x; c < nchunks; c += 256) {
    const int i = c / cpr, j8 = c % cpr;
    *reinterpret_cast<uint4*>(dst + (int64_t)i * ldw + j8 * 8) =
        src ? *reinterpret_cast<const uint4*>(src + (int64_t)c * 8) : uint4{0u, 0u, 0u, 0u};
  }
}

// out[i] = in[i]
__global__ __launch_bounds__(256) void k_copy_i32(const int* __restrict__ in, int64_t n, int* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = in[i];
}

// inv[perm[e]] = e
__global__ __launch_bounds__(256) void k_invert_perm(const int* __restrict__ perm, int64_t n, int* __restrict__ inv) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < n) inv[perm[e]] = (int)e;
}

struct PackWs {
  size_t scores_off, mask_off, rcnt_off, ccnt_off, blk_row_off, scalars_off, bytes;
};

PackWs pack_ws_layout(int64_t nbr, int64_t nbc, int32_t mode, int64_t nnz_cap) {
  using blast::align_up;
  const size_t n = (size_t)nbr * (size_t)nbc;
  PackWs L;
  size_t off = 0;
  L.scores_off = off;
  if (mode == BLAST_PACK_TOPK_FROBENIUS) off += align_up(8 * n, 256);
  L.mask_off = off;
  if (mode == BLAST_PACK_TOPK_FROBENIUS) off += align_up(n, 256);
  L.rcnt_off = off;
  off += align_up(4 * (size_t)nbr, 256);
  L.ccnt_off = off;
  off += align_up(4 * (size_t)nbc, 256);
  L.blk_row_off = off;
  off += align_up(4 * (size_t)(nnz_cap > 0 ? nnz_cap : 1), 256);
  L.scalars_off = off;
  off += 256;
  L.bytes = off;
  return L;
}

int check_shape(int64_t rows, int64_t cols, int32_t b) {
  if (rows < 0 || cols < 0) return BLAST_ERR_INVALID_ARG;
  if (!blast::supported_block(b)) return BLAST_ERR_UNSUPPORTED_BLOCK;
  if (rows % b || cols % b) return BLAST_ERR_SHAPE;
  if (rows / b > INT32_MAX / 2 || cols / b > INT32_MAX / 2 || (rows / b) * (cols / b) > (int64_t)INT32_MAX)
    return BLAST_ERR_INVALID_ARG;
  return BLAST_OK;
}

}  // namespace

extern "C" int64_t blast_n_keep(int64_t n_blocks, double sparsity) {
  if (n_blocks < 0 || !(sparsity >= 0.0 && sparsity <= 1.0)) return -1;
  const int64_t s_bp = (int64_t)(sparsity * 10000.0 + 0.5);
  const int64_t n_zero = (int64_t)(((__int128)s_bp * n_blocks + 9999) / 10000);
  return n_blocks - (n_zero > n_blocks ? n_blocks : n_zero);
}

extern "C" size_t blast_bsr_aux_bytes(int64_t rows, int64_t cols, int32_t b, int64_t nnz_cap) {
  if (check_shape(rows, cols, b) != BLAST_OK || nnz_cap < 0) return 0;
  return blast::aux_layout(rows / b, cols / b, nnz_cap).bytes;
}

extern "C" int blast_bsr_pack_bound(int64_t rows, int64_t cols, int32_t b, int32_t mode, double sparsity,
                                    int64_t* nnz_cap, size_t* aux_bytes, size_t* ws_bytes) {
  if (mode != BLAST_PACK_MASK && mode != BLAST_PACK_TOPK_FROBENIUS) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_shape(rows, cols, b)) return rc;
  const int64_t nbr = rows / b, nbc = cols / b, n = nbr * nbc;
  int64_t cap = n;
  if (mode == BLAST_PACK_TOPK_FROBENIUS) {
    cap = blast_n_keep(n, sparsity);
    if (cap < 0) return BLAST_ERR_INVALID_ARG;
  }
  if (nnz_cap) *nnz_cap = cap;
  if (aux_bytes) *aux_bytes = blast::aux_layout(nbr, nbc, cap).bytes;
  if (ws_bytes) *ws_bytes = pack_ws_layout(nbr, nbc, mode, cap).bytes;
  return BLAST_OK;
}

namespace {

// Validates the arguments of a packing call and enqueues all of its work.  The two result scalars {number of
// stored blocks, stored blocks of the fullest row} are left at *scalars_out (device memory: `result` when the
// caller gave one, else a slot of the workspace); n_keep_out gets the number of blocks the scoring mode keeps
// (-1 in mask mode).
int pack_enqueue(const uint16_t* W, int64_t ldw, int64_t rows, int64_t cols, int32_t b, int32_t mode,
                 const uint8_t* block_mask, double sparsity, int32_t* row_ptr, int32_t* col_idx, uint16_t* vals,
                 int32_t* row_order, void* aux, size_t aux_bytes, int64_t nnz_cap, int32_t* result, void* ws,
                 size_t ws_bytes, hipStream_t stream, int** scalars_out) {
  if (mode != BLAST_PACK_MASK && mode != BLAST_PACK_TOPK_FROBENIUS) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_shape(rows, cols, b)) return rc;
  if (!row_ptr || nnz_cap < 0) return BLAST_ERR_INVALID_ARG;
  const int64_t nbr = rows / b, nbc = cols / b, n = nbr * nbc;
  if (n > 0 && (!W || ldw < cols || ldw % 8 || !blast::aligned(W, 16))) return BLAST_ERR_INVALID_ARG;
  if (mode == BLAST_PACK_MASK && n > 0 && !block_mask) return BLAST_ERR_INVALID_ARG;
  int64_t n_keep = -1;
  if (mode == BLAST_PACK_TOPK_FROBENIUS) {
    n_keep = blast_n_keep(n, sparsity);
    if (n_keep < 0) return BLAST_ERR_INVALID_ARG;
  }
  if (nnz_cap > 0 && (!col_idx || !vals || !blast::aligned(vals, 16))) return BLAST_ERR_INVALID_ARG;
  if (nbr > 0 && !row_order) return BLAST_ERR_INVALID_ARG;
  const PackWs L = pack_ws_layout(nbr, nbc, mode, nnz_cap);
  if (!ws || ws_bytes < L.bytes || !blast::aligned(ws, 16)) return BLAST_ERR_WORKSPACE;
  const blast::AuxLayout A = blast::aux_layout(nbr, nbc, nnz_cap);
  if (aux && (aux_bytes < A.bytes || !blast::aligned(aux, 16))) return BLAST_ERR_WORKSPACE;
  const int64_t gather_grid = (mode == BLAST_PACK_TOPK_FROBENIUS && n_keep < nnz_cap) ? n_keep : nnz_cap;
  if (gather_grid > INT32_MAX) return BLAST_ERR_INVALID_ARG;

  char* wsb = static_cast<char*>(ws);
  double* scores = reinterpret_cast<double*>(wsb + L.scores_off);
  int* rcnt = reinterpret_cast<int*>(wsb + L.rcnt_off);
  int* ccnt = reinterpret_cast<int*>(wsb + L.ccnt_off);
  int* blk_row = reinterpret_cast<int*>(wsb + L.blk_row_off);
  int* nnz_dev = result ? result : reinterpret_cast<int*>(wsb + L.scalars_off);
  *scalars_out = nnz_dev;
  const uint8_t* mask = block_mask;
  uint8_t* m = mode == BLAST_PACK_TOPK_FROBENIUS ? reinterpret_cast<uint8_t*>(wsb + L.mask_off) : nullptr;
  if (m) mask = m;
  char* ab = static_cast<char*>(aux);
  PlanOut narrow{}, wide{};
  if (aux) plan_outputs(ab, A, narrow, wide);
  int* col_ptr = aux ? reinterpret_cast<int*>(ab + A.col_ptr_off) : nullptr;  // (this offset does not depend on nnz)
  int* csc_row = aux ? reinterpret_cast<int*>(ab + A.csc_row_off) : nullptr;
  const bool scored = mode == BLAST_PACK_TOPK_FROBENIUS && n > 0 && n_keep > 0 && n_keep < n;
  if (scored) {
    k_block_scores<<<dim3((unsigned)n), dim3(256), 0, stream>>>(W, ldw, (int)nbc, b, scores);
    BLAST_LAUNCH_CHECK("k_block_scores");
  }

  if (n > 0 && n <= kSmallN && nbr <= 1024 && nbc <= 1024) {
    // selection, row pointers, column indices, schedule, chunk plans and column-grouped index: one launch
    const SmallOut o{row_ptr, col_idx, blk_row, row_order, m, col_ptr, csc_row, nnz_dev, nnz_cap};
    if (mode == BLAST_PACK_TOPK_FROBENIUS)
      k_pack_small<true><<<dim3(1), dim3(1024), 0, stream>>>(scores, nullptr, (int)nbr, (int)nbc, (long long)n_keep, o,
                                                             narrow, wide);
    else
      k_pack_small<false><<<dim3(1), dim3(1024), 0, stream>>>(nullptr, mask, (int)nbr, (int)nbc, 0ll, o, narrow, wide);
    BLAST_LAUNCH_CHECK("k_pack_small");
  } else {
    if (m && n > 0) {
      if (!scored) {
        k_fill_u8<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(m, n, n_keep == n ? 1 : 0);
        BLAST_LAUNCH_CHECK("k_fill_u8");
      } else {
        k_select_topk<<<dim3(1), dim3(1024), 0, stream>>>(scores, n, n_keep, m);
        BLAST_LAUNCH_CHECK("k_select_topk");
      }
    }
    if (nbr > 0) {
      k_line_counts<<<dim3((unsigned)((nbr + 3) / 4)), dim3(256), 0, stream>>>(mask, (int)nbr, (int)nbc, nbc, 1, rcnt);
      BLAST_LAUNCH_CHECK("k_line_counts(rows)");
    }
    k_exscan<<<dim3(1), dim3(1024), 0, stream>>>(rcnt, (int)nbr, row_ptr, nnz_dev);
    BLAST_LAUNCH_CHECK("k_exscan(rows)");
    if (nbr > 0) {
      k_row_order<<<dim3((unsigned)((nbr + 255) / 256)), dim3(256), 0, stream>>>(row_ptr, nullptr, (int)nbr, row_order);
      BLAST_LAUNCH_CHECK("k_row_order");
    }
    if (aux) {
      k_chunk_plan<<<dim3(1), dim3(1024), 0, stream>>>(row_ptr, row_order, (int)nbr, narrow, wide, nnz_dev + 1);
      BLAST_LAUNCH_CHECK("k_chunk_plan");
    } else {
      k_fill_i32<<<dim3(1), dim3(64), 0, stream>>>(nnz_dev + 1, 1, 0);
      BLAST_LAUNCH_CHECK("k_fill_i32");
    }
    if (nbr > 0) {
      k_fill_cols<<<dim3((unsigned)nbr), dim3(256), 0, stream>>>(mask, (int)nbc, row_ptr, col_idx, blk_row, nnz_cap);
      BLAST_LAUNCH_CHECK("k_fill_cols");
    }
    if (aux) {
      if (nbc > 0 && nbr > 0) {
        k_line_counts<<<dim3((unsigned)((nbc + 3) / 4)), dim3(256), 0, stream>>>(mask, (int)nbc, (int)nbr, 1, nbc, ccnt);
        BLAST_LAUNCH_CHECK("k_line_counts(cols)");
      } else if (nbc > 0) {
        k_fill_i32<<<dim3((unsigned)((nbc + 255) / 256)), dim3(256), 0, stream>>>(ccnt, nbc, 0);
        BLAST_LAUNCH_CHECK("k_fill_i32(cols)");
      }
      k_exscan<<<dim3(1), dim3(1024), 0, stream>>>(ccnt, (int)nbc, col_ptr, nullptr);
      BLAST_LAUNCH_CHECK("k_exscan(cols)");
      if (nbc > 0 && nbr > 0 && nnz_cap > 0) {
        k_fill_csc<<<dim3((unsigned)nbc), dim3(256), 0, stream>>>(mask, (int)nbr, (int)nbc, row_ptr, col_idx, col_ptr,
                                                                  csc_row, nullptr, nnz_cap, nnz_dev);
        BLAST_LAUNCH_CHECK("k_fill_csc");
      }
    }
  }
  // Nothing needs the number of stored blocks on the host: the gather's grid is the capacity (workgroups past
  // the device's count leave), and the column-grouped index is placed by the device's count.
  if (gather_grid > 0) {
    k_gather_blocks<<<dim3((unsigned)gather_grid), dim3(256), 0, stream>>>(W, ldw, b, col_idx, blk_row, mask, (int)nbc,
                                                                         vals, nnz_dev);
    BLAST_LAUNCH_CHECK("k_gather_blocks");
  }
  return BLAST_OK;
}

}  // namespace

extern "C" int blast_bsr_pack_enqueue(const uint16_t* W, int64_t ldw, int64_t rows, int64_t cols, int32_t b,
                                      int32_t mode, const uint8_t* block_mask, double sparsity, int32_t* row_ptr,
                                      int32_t* col_idx, uint16_t* vals, int32_t* row_order, void* aux, size_t aux_bytes,
                                      int64_t nnz_cap, int32_t* result, void* ws, size_t ws_bytes, void* stream_) {
  if (!result || !blast::aligned(result, 8)) return BLAST_ERR_INVALID_ARG;
  int* scalars = nullptr;
  return pack_enqueue(W, ldw, rows, cols, b, mode, block_mask, sparsity, row_ptr, col_idx, vals, row_order, aux,
                      aux_bytes, nnz_cap, result, ws, ws_bytes, static_cast<hipStream_t>(stream_), &scalars);
}

extern "C" int blast_bsr_pack(const uint16_t* W, int64_t ldw, int64_t rows, int64_t cols, int32_t b, int32_t mode,
                              const uint8_t* block_mask, double sparsity, int32_t* row_ptr, int32_t* col_idx,
                              uint16_t* vals, int32_t* row_order, void* aux, size_t aux_bytes, int64_t nnz_cap,
                              int64_t* nnz_out, int32_t* max_row_blocks_out, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!nnz_out) return BLAST_ERR_INVALID_ARG;
  int* scalars = nullptr;
  if (int rc = pack_enqueue(W, ldw, rows, cols, b, mode, block_mask, sparsity, row_ptr, col_idx, vals, row_order, aux,
                            aux_bytes, nnz_cap, nullptr, ws, ws_bytes, stream, &scalars))
    return rc;
  // The two scalars come back through a small pinned buffer (one per host thread, allocated on first use
  // and kept): a copy into pageable memory costs the call tens of microseconds more.
  int host_vals[2] = {0, 0};
  static thread_local int* pinned = nullptr;
  if (!pinned) {
    void* p = nullptr;
    if (hipHostMalloc(&p, 64, hipHostMallocDefault) == hipSuccess) {
      pinned = static_cast<int*>(p);
    } else {
      (void)hipGetLastError();
    }
  }
  int* landing = pinned ? pinned : host_vals;
  BLAST_HIP_TRY(hipMemcpyAsync(landing, scalars, 2 * sizeof(int), hipMemcpyDeviceToHost, stream));
  BLAST_HIP_TRY(hipStreamSynchronize(stream));
  host_vals[0] = landing[0];
  host_vals[1] = landing[1];
  *nnz_out = host_vals[0];
  if (max_row_blocks_out) *max_row_blocks_out = aux ? host_vals[1] : 0;
  if (host_vals[0] > nnz_cap) return BLAST_ERR_CAPACITY;
  return BLAST_OK;
}

extern "C" int blast_bsr_joint_row_order(const blast_bsr_view* A, const blast_bsr_view* Bm, int32_t* row_order,
                                         void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!A || !Bm || !A->row_ptr || !Bm->row_ptr) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_shape(A->rows, A->cols, A->b)) return rc;
  if (A->rows != Bm->rows || A->b != Bm->b) return BLAST_ERR_SHAPE;
  const int64_t nbr = A->rows / A->b;
  if (nbr == 0) return BLAST_OK;
  if (!row_order) return BLAST_ERR_INVALID_ARG;
  k_row_order<<<dim3((unsigned)((nbr + 255) / 256)), dim3(256), 0, stream>>>(A->row_ptr, Bm->row_ptr, (int)nbr,
                                                                              row_order);
  BLAST_LAUNCH_CHECK("k_row_order(joint)");
  return BLAST_OK;
}

extern "C" int blast_bsr_transpose(const blast_bsr_view* W, int32_t* row_ptr_t, int32_t* col_idx_t, uint16_t* vals_t,
                                   int32_t* row_order_t, void* aux_t, size_t aux_t_bytes,
                                   int32_t* max_row_blocks_t_out, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!W || !W->row_ptr || W->nnz < 0 || W->nnz > INT32_MAX) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_shape(W->rows, W->cols, W->b)) return rc;
  const int64_t nbr = W->rows / W->b, nbc = W->cols / W->b, nnz = W->nnz;
  const int b = W->b;
  if (!W->aux) return BLAST_ERR_WORKSPACE;  // the column-grouped index of the packer is the input here
  if (!row_ptr_t || (nbc > 0 && !row_order_t)) return BLAST_ERR_INVALID_ARG;
  if (nnz > 0 && (!W->col_idx || !W->vals || !col_idx_t || !vals_t || !blast::aligned(vals_t, 16) ||
                  !blast::aligned(W->vals, 16)))
    return BLAST_ERR_INVALID_ARG;
  const blast::AuxLayout A = blast::aux_layout(nbr, nbc, nnz);   // of the input
  const blast::AuxLayout At = blast::aux_layout(nbc, nbr, nnz);  // of the output
  if (aux_t && (aux_t_bytes < At.bytes || !blast::aligned(aux_t, 16))) return BLAST_ERR_WORKSPACE;
  const char* ab = static_cast<const char*>(W->aux);
  const int* col_ptr = reinterpret_cast<const int*>(ab + A.col_ptr_off);
  const int* csc_row = reinterpret_cast<const int*>(ab + A.csc_row_off);
  const int* csc_blk = reinterpret_cast<const int*>(ab + A.csc_blk_off);
  auto blocks_for = [](int64_t n) { return dim3((unsigned)((n + 255) / 256)); };

  // BSR of the transpose = the column-grouped (BCSC) view of the input, with every block turned
  k_copy_i32<<<blocks_for(nbc + 1), dim3(256), 0, stream>>>(col_ptr, nbc + 1, row_ptr_t);
  BLAST_LAUNCH_CHECK("k_copy_i32(row_ptr_t)");
  if (nnz > 0) {
    k_copy_i32<<<blocks_for(nnz), dim3(256), 0, stream>>>(csc_row, nnz, col_idx_t);
    BLAST_LAUNCH_CHECK("k_copy_i32(col_idx_t)");
    k_transpose_blocks<<<dim3((unsigned)nnz), dim3(256), (size_t)b * (b + 2) * 2, stream>>>(W->vals, b, csc_blk, vals_t);
    BLAST_LAUNCH_CHECK("k_transpose_blocks");
  }
  if (nbc > 0) {
    k_row_order<<<blocks_for(nbc), dim3(256), 0, stream>>>(row_ptr_t, nullptr, (int)nbc, row_order_t);
    BLAST_LAUNCH_CHECK("k_row_order(transpose)");
  }
  int heavy = 0;
  if (aux_t) {
    char* at = static_cast<char*>(aux_t);
    int* hdr = reinterpret_cast<int*>(at + At.hdr_off);
    PlanOut narrow, wide;
    plan_outputs(at, At, narrow, wide);
    k_chunk_plan<<<dim3(1), dim3(1024), 0, stream>>>(row_ptr_t, row_order_t, (int)nbc, narrow, wide, hdr + 1);
    BLAST_LAUNCH_CHECK("k_chunk_plan(transpose)");
    // the column-grouped index of the transpose is the row-grouped one of the input
    k_copy_i32<<<blocks_for(nbr + 1), dim3(256), 0, stream>>>(W->row_ptr, nbr + 1,
                                                              reinterpret_cast<int*>(at + At.col_ptr_off));
    BLAST_LAUNCH_CHECK("k_copy_i32(col_ptr_t)");
    if (nnz > 0) {
      k_copy_i32<<<blocks_for(nnz), dim3(256), 0, stream>>>(W->col_idx, nnz, reinterpret_cast<int*>(at + At.csc_row_off));
      BLAST_LAUNCH_CHECK("k_copy_i32(csc_row_t)");
      k_invert_perm<<<blocks_for(nnz), dim3(256), 0, stream>>>(csc_blk, nnz, reinterpret_cast<int*>(at + At.csc_blk_off));
      BLAST_LAUNCH_CHECK("k_invert_perm");
    }
    if (max_row_blocks_t_out) {
      BLAST_HIP_TRY(hipMemcpyAsync(&heavy, hdr + 1, sizeof(int), hipMemcpyDeviceToHost, stream));
      BLAST_HIP_TRY(hipStreamSynchronize(stream));
    }
  }
  if (max_row_blocks_t_out) *max_row_blocks_t_out = heavy;
  return BLAST_OK;
}

// ---- one mask update of blocked prune-and-grow (BLaST Sec. 3.2, generate_masks()) ----

extern "C" size_t blast_generate_masks_workspace(int64_t rows, int64_t cols, int32_t b) {
  if (check_shape(rows, cols, b) != BLAST_OK) return 0;
  const size_t n = (size_t)(rows / b) * (size_t)(cols / b);
  return 2 * blast::align_up(8 * (n > 0 ? n : 1), 256) + 2 * blast::align_up(n > 0 ? n : 1, 256);
}

extern "C" int blast_generate_masks(const uint16_t* W, int64_t ldw, const uint16_t* G, int64_t ldg, int64_t rows,
                                    int64_t cols, int32_t b, double sparsity, uint8_t* mask_out, void* ws,
                                    size_t ws_bytes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (int rc = check_shape(rows, cols, b)) return rc;
  const int64_t nbc = cols / b, n = (rows / b) * nbc;
  const int64_t n_keep = blast_n_keep(n, sparsity);
  if (n_keep < 0) return BLAST_ERR_INVALID_ARG;
  if (n == 0) return BLAST_OK;
  if (!W || !G || !mask_out || ldw < cols || ldg < cols || ldw % 8 || ldg % 8 || !blast::aligned(W, 16) ||
      !blast::aligned(G, 16))
    return BLAST_ERR_INVALID_ARG;
  if (!ws || ws_bytes < blast_generate_masks_workspace(rows, cols, b) || !blast::aligned(ws, 16))
    return BLAST_ERR_WORKSPACE;
  char* wsb = static_cast<char*>(ws);
  double* scores = reinterpret_cast<double*>(wsb);
  double* scores_g = reinterpret_cast<double*>(wsb + blast::align_up(8 * (size_t)n, 256));
  uint8_t* mw = reinterpret_cast<uint8_t*>(wsb + 2 * blast::align_up(8 * (size_t)n, 256));
  uint8_t* mg = mw + blast::align_up((size_t)n, 256);
  const dim3 per_elem((unsigned)((n + 255) / 256));
  if (n_keep == 0 || n_keep == n) {  // nothing survives and nothing regrows, or everything is kept by W itself
    k_fill_u8<<<per_elem, dim3(256), 0, stream>>>(mask_out, n, n_keep == n ? 1 : 0);
    BLAST_LAUNCH_CHECK("k_fill_u8");
    return BLAST_OK;
  }
  k_block_scores<<<dim3((unsigned)n, 2), dim3(256), 0, stream>>>(W, ldw, (int)nbc, b, scores, G, ldg, scores_g);
  BLAST_LAUNCH_CHECK("k_block_scores(W, G)");
  if (n <= kSmallN) {  // both selections and the merge in one workgroup
    k_masks_small<<<dim3(1), dim3(1024), 0, stream>>>(scores, scores_g, (int)n, (long long)n_keep, mask_out);
    BLAST_LAUNCH_CHECK("k_masks_small");
    return BLAST_OK;
  }
  k_select_topk<<<dim3(2), dim3(1024), 0, stream>>>(scores, n, n_keep, mw, scores_g, mg);
  BLAST_LAUNCH_CHECK("k_select_topk(W, G)");
  k_merge_masks<<<per_elem, dim3(256), 0, stream>>>(mw, mg, n, mask_out);
  BLAST_LAUNCH_CHECK("k_merge_masks");
  return BLAST_OK;
}

// Eq. (2).  Past i = m - d the cube would turn negative and push s above s_max; the iteration is held
// inside [0, m - d].
extern "C" double blast_sparsity_schedule(int64_t i, int64_t m, int64_t d, double s_init, double s_max) {
  const int64_t span = m - d;
  if (span <= 0) return s_max;
  if (i < 0) i = 0;
  if (i > span) i = span;
  const double f = 1.0 - (double)i / (double)span;
  return s_max + (s_init - s_max) * f * f * f;
}

// ---- block selection from a sensitivity matrix (BLaST Sec. 3.3) ----

extern "C" size_t blast_pooled_topk_mask_workspace(int64_t rows, int64_t cols, int32_t b) {
  if (check_shape(rows, cols, b) != BLAST_OK) return 0;
  const size_t n = (size_t)(rows / b) * (size_t)(cols / b);
  return blast::align_up(8 * (n > 0 ? n : 1), 256);
}

extern "C" int blast_pooled_topk_mask(const float* S, int64_t lds, int64_t rows, int64_t cols, int32_t b,
                                      double sparsity, uint8_t* mask_out, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (int rc = check_shape(rows, cols, b)) return rc;
  const int64_t nbc = cols / b, n = (rows / b) * nbc;
  const int64_t n_keep = blast_n_keep(n, sparsity);
  if (n_keep < 0) return BLAST_ERR_INVALID_ARG;
  if (n == 0) return BLAST_OK;
  if (!S || !mask_out || lds < cols || lds % 4 || !blast::aligned(S, 16)) return BLAST_ERR_INVALID_ARG;
  if (!ws || ws_bytes < blast_pooled_topk_mask_workspace(rows, cols, b) || !blast::aligned(ws, 16))
    return BLAST_ERR_WORKSPACE;
  if (n_keep == 0 || n_keep == n) {
    k_fill_u8<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(mask_out, n, n_keep == n ? 1 : 0);
    BLAST_LAUNCH_CHECK("k_fill_u8");
    return BLAST_OK;
  }
  double* scores = static_cast<double*>(ws);
  k_pooled_scores<<<dim3((unsigned)n), dim3(256), 0, stream>>>(S, lds, (int)nbc, b, scores);
  BLAST_LAUNCH_CHECK("k_pooled_scores");
  if (n <= kSmallN) {
    k_select_small<<<dim3(1), dim3(1024), 0, stream>>>(scores, (int)n, (long long)n_keep, mask_out);
    BLAST_LAUNCH_CHECK("k_select_small(pooled)");
    return BLAST_OK;
  }
  k_select_topk<<<dim3(1), dim3(1024), 0, stream>>>(scores, n, n_keep, mask_out);
  BLAST_LAUNCH_CHECK("k_select_topk(pooled)");
  return BLAST_OK;
}

// The dense form of a packed matrix: W_new of prune_weights() (BLaST Sec. 3.2), zeros outside the stored blocks.
extern "C" int blast_bsr_unpack(const blast_bsr_view* Wp, uint16_t* W, int64_t ldw, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!Wp || !Wp->row_ptr || Wp->nnz < 0) return BLAST_ERR_INVALID_ARG;
  if (int rc = check_shape(Wp->rows, Wp->cols, Wp->b)) return rc;
  const int64_t nbr = Wp->rows / Wp->b, nbc = Wp->cols / Wp->b, n = nbr * nbc;
  if (n == 0) return BLAST_OK;
  if (!W || ldw < Wp->cols || ldw % 8 || !blast::aligned(W, 16)) return BLAST_ERR_INVALID_ARG;
  if (Wp->nnz > 0 && (!Wp->col_idx || !Wp->vals || !blast::aligned(Wp->vals, 16))) return BLAST_ERR_INVALID_ARG;
  k_unpack_blocks<<<dim3((unsigned)n), dim3(256), 0, stream>>>(Wp->row_ptr, Wp->col_idx, Wp->vals, (int)nbc, Wp->b, W, ldw);
  BLAST_LAUNCH_CHECK("k_unpack_blocks");
  return BLAST_OK;
}
