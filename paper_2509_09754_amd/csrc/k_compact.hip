// Compaction of the surviving K/V rows into the packed per-head cache (Alg. 1, last loop:
// K^ = K (.) I, V^ = V (.) I, stored without the evicted rows).  A pure gather: every row is
// moved with 128-bit loads and stores, one row per group of (row bytes / 16) lanes.
#include "common.h"

namespace lava {

constexpr int kCompactThreads = 256;
constexpr int kCompactMaxHeads = 64;

// LPR = lanes per row = row bytes / 16.
template <int LPR>
__global__ void __launch_bounds__(kCompactThreads)
compact_kernel(int n_heads, long long n, const uint4* __restrict__ k, const uint4* __restrict__ v,
               const int64_t* __restrict__ head_offsets, const int32_t* __restrict__ kept_idx,
               long long capacity, uint4* __restrict__ k_out, uint4* __restrict__ v_out) {
  __shared__ long long s_off[kCompactMaxHeads + 1];
  if (threadIdx.x <= n_heads) s_off[threadIdx.x] = (long long)head_offsets[threadIdx.x];
  __syncthreads();
  constexpr int kRowsPerBlock = kCompactThreads / LPR;
  const long long t = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / LPR;
  const int c = threadIdx.x % LPR;
  long long kept = s_off[n_heads];
  if (kept > capacity) kept = capacity;
  if (t >= kept) return;
  int g = 0;
  while (g + 1 < n_heads && t >= s_off[g + 1]) ++g;
  long long src = (long long)kept_idx[t];
  if (src < 0 || src >= n) return;   // never dereference an index outside the head
  const long long in = ((long long)g * n + src) * LPR + c;
  const long long out = t * LPR + c;
  const uint4 kv = k[in];
  const uint4 vv = v[in];
  k_out[out] = kv;
  v_out[out] = vv;
}

int32_t launch_compact(const lava_layer_desc& d, int64_t n, const void* k, const void* v,
                       const int64_t* head_offsets, const int32_t* kept_idx, int64_t capacity,
                       void* k_out, void* v_out, hipStream_t s) {
  if (capacity == 0) return LAVA_OK;
  const int row_bytes = d.head_dim * (d.dtype == LAVA_BF16 ? 2 : 4);
  const int lpr = row_bytes / 16;
  const int rows_per_block = kCompactThreads / lpr;
  const dim3 grid((unsigned)((capacity + rows_per_block - 1) / rows_per_block)), block(kCompactThreads);
  ProfScope ps(KID_COMPACT, s);
#define LAVA_COMPACT(L)                                                                          \
  hipLaunchKernelGGL(compact_kernel<L>, grid, block, 0, s, d.n_kv_heads, (long long)n,           \
                     static_cast<const uint4*>(k), static_cast<const uint4*>(v), head_offsets,   \
                     kept_idx, (long long)capacity, static_cast<uint4*>(k_out),                  \
                     static_cast<uint4*>(v_out))
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
