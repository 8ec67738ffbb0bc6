// Compaction of the surviving K/V rows into the packed per-head cache (Alg. 1, last loop:
// K^ = K (.) I, V^ = V (.) I, stored without the evicted rows).  A pure gather: every row is
// moved with 128-bit loads and stores, one row per group of (row bytes / 16) lanes.
#include "common.h"

namespace lava {

constexpr int kCompactThreads = 256;
constexpr int kCompactMaxHeads = 64;

// LPR = lanes per row = row bytes / 16.  The source is either dense ([n_heads][n] rows, src_offsets
// null) or itself packed (head g owns source rows src_offsets[g] .. src_offsets[g+1]-1), which is
// what a re-eviction of an already compressed layer reads (Alg. 2, inner loop).  pos_out, if
// given, receives the token position of every surviving row: pos_src[source row] for a packed
// source, the index itself for a dense one.
template <int LPR>
__global__ void __launch_bounds__(kCompactThreads)
compact_kernel(int n_heads, long long n, const int64_t* __restrict__ src_offsets, const uint4* __restrict__ k,
               const uint4* __restrict__ v, const int32_t* __restrict__ pos_src,
               const int64_t* __restrict__ head_offsets, const int32_t* __restrict__ kept_idx,
               long long capacity, uint4* __restrict__ k_out, uint4* __restrict__ v_out,
               int32_t* __restrict__ pos_out) {
  __shared__ long long s_off[kCompactMaxHeads + 1];
  __shared__ long long s_src[kCompactMaxHeads + 1];
  if (threadIdx.x <= n_heads) {
    s_off[threadIdx.x] = (long long)head_offsets[threadIdx.x];
    s_src[threadIdx.x] = src_offsets ? (long long)src_offsets[threadIdx.x] : (long long)threadIdx.x * n;
  }
  __syncthreads();
  constexpr int kRowsPerBlock = kCompactThreads / LPR;
  const long long t = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / LPR;
  const int c = threadIdx.x % LPR;
  long long kept = s_off[n_heads];
  if (kept > capacity) kept = capacity;
  if (t >= kept) return;
  int g = 0;
  while (g + 1 < n_heads && t >= s_off[g + 1]) ++g;
  const long long src = (long long)kept_idx[t];
  const long long len = s_src[g + 1] - s_src[g];
  // never dereference an index outside the head; a packed source must also stay inside its pool (n rows)
  if (src < 0 || src >= len || s_src[g] < 0 || (src_offsets != nullptr && s_src[g + 1] > n)) return;
  const long long row = s_src[g] + src;
  const long long in = row * LPR + c;
  const long long out = t * LPR + c;
  const uint4 kv = k[in];
  const uint4 vv = v[in];
  k_out[out] = kv;
  v_out[out] = vv;
  if (pos_out != nullptr && c == 0) pos_out[t] = pos_src ? pos_src[row] : (int32_t)src;
}

int32_t launch_compact(const lava_layer_desc& d, int64_t n, const int64_t* src_offsets, const void* k,
                       const void* v, const int32_t* pos_src, const int64_t* head_offsets,
                       const int32_t* kept_idx, int64_t capacity, void* k_out, void* v_out, int32_t* pos_out,
                       hipStream_t s) {
  if (capacity == 0) return LAVA_OK;
  const int row_bytes = d.head_dim * (d.dtype == LAVA_BF16 ? 2 : 4);
  const int lpr = row_bytes / 16;
  const int rows_per_block = kCompactThreads / lpr;
  const dim3 grid((unsigned)((capacity + rows_per_block - 1) / rows_per_block)), block(kCompactThreads);
  ProfScope ps(KID_COMPACT, s);
#define LAVA_COMPACT(L)                                                                          \
  hipLaunchKernelGGL(compact_kernel<L>, grid, block, 0, s, d.n_kv_heads, (long long)n, src_offsets, \
                     static_cast<const uint4*>(k), static_cast<const uint4*>(v), pos_src, head_offsets, \
                     kept_idx, (long long)capacity, static_cast<uint4*>(k_out),                  \
                     static_cast<uint4*>(v_out), pos_out)
  switch (lpr) {
    case 8: LAVA_COMPACT(8); break;
    case 16: LAVA_COMPACT(16); break;
    case 32: LAVA_COMPACT(32); break;
    default: return LAVA_ERR_SHAPE;
  }
#undef LAVA_COMPACT
  return launch_status();
}

}  // namespace lava
