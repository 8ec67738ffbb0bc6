// Compaction of the surviving K/V rows into the packed per-head cache (Alg. 1, last loop:
// K^ = K (.) I, V^ = V (.) I, stored without the evicted rows).  A pure gather: every row is
// moved with 128-bit loads and stores, one row per group of (row bytes / 16) lanes.
#include "common.h"

namespace lava {

constexpr int kCompactThreads = 256;
constexpr int kCompactMaxHeads = 64;

struct CompactBatch {
  int n_heads;
  int n_problems;
  lava_compact_problem p[kMaxSelProblems];
};

// LPR = lanes per row = row bytes / 16.  The source is either dense ([n_heads][n] rows, src_offsets
// null) or itself packed (head g owns source rows src_offsets[g] .. src_offsets[g+1]-1), which is
// what a re-eviction of an already compressed layer reads (Alg. 2, inner loop).  pos_out, if
// given, receives the token position of every surviving row: pos_src[source row] for a packed
// source, the index itself for a dense one.  A packed source and the output may each start at a
// row offset that is read on the device (layers packed back to back in one pool).
// blockIdx.y = problem of the table; the workgroups of a problem walk over its surviving rows,
// whose number is only known on the device, a grid's worth of rows at a time (kCompactBlocks
// workgroups per problem of a table, four times as many for a problem alone).
constexpr int kCompactBlocks = 256;

template <int LPR>
__global__ void __launch_bounds__(kCompactThreads) compact_kernel(const CompactBatch a) {
  const lava_compact_problem pr = a.p[blockIdx.y];
  const int n_heads = a.n_heads;
  const long long n = pr.src_rows;
  const int64_t* __restrict__ src_offsets = pr.src_offsets;
  constexpr int kRowsPerBlock = kCompactThreads / LPR;
  if ((long long)blockIdx.x * kRowsPerBlock >= pr.capacity) return;
  const long long src_off = pr.src_offset_dev ? (long long)*pr.src_offset_dev : 0;
  const long long out_off = pr.out_offset_dev ? (long long)*pr.out_offset_dev : 0;
  const int32_t* __restrict__ pos_src = pr.pos_src;
  const int32_t* __restrict__ kept_idx = pr.kept_idx + out_off;
  const uint4* __restrict__ k = static_cast<const uint4*>(pr.k_src);
  const uint4* __restrict__ v = static_cast<const uint4*>(pr.v_src);
  uint4* __restrict__ k_out = static_cast<uint4*>(pr.k_out);
  uint4* __restrict__ v_out = static_cast<uint4*>(pr.v_out);
  int32_t* __restrict__ pos_out = pr.pos_out;
  __shared__ long long s_off[kCompactMaxHeads + 1];
  __shared__ long long s_src[kCompactMaxHeads + 1];
  if (threadIdx.x <= n_heads) {
    s_off[threadIdx.x] = (long long)pr.head_offsets[threadIdx.x];
    s_src[threadIdx.x] = src_offsets ? (long long)src_offsets[threadIdx.x] : (long long)threadIdx.x * n;
  }
  __syncthreads();
  // rows that exist and fit: never write at or beyond row `capacity` of the output pool
  long long kept = s_off[n_heads];
  if (out_off < 0 || src_off < 0) kept = 0;
  if (kept > pr.capacity - out_off) kept = pr.capacity - out_off;
  const int c = threadIdx.x % LPR;
  for (long long t = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / LPR; t < kept;
       t += (long long)gridDim.x * kRowsPerBlock) {
    int g = 0;
    while (g + 1 < n_heads && t >= s_off[g + 1]) ++g;
    const long long src = (long long)kept_idx[t];
    const long long len = s_src[g + 1] - s_src[g];
    // never dereference an index outside the head; a packed source must also stay inside its pool (n rows)
    if (src < 0 || src >= len || s_src[g] < 0 || (src_offsets != nullptr && src_off + s_src[g + 1] > n)) continue;
    const long long row = src_off + s_src[g] + src;
    const long long in = row * LPR + c;
    const long long out = (out_off + t) * LPR + c;
    const uint4 kv = k[in];
    const uint4 vv = v[in];
    k_out[out] = kv;
    v_out[out] = vv;
    if (pos_out != nullptr && c == 0) pos_out[out_off + t] = pos_src ? pos_src[row] : (int32_t)src;
  }
}

int32_t launch_compact_batch(const lava_layer_desc& d, int n_problems, const lava_compact_problem* problems,
                             hipStream_t s) {
  const int row_bytes = d.head_dim * (d.dtype == LAVA_BF16 ? 2 : 4);
  const int lpr = row_bytes / 16;
  const int rows_per_block = kCompactThreads / lpr;
  CompactBatch a;
  a.n_heads = d.n_kv_heads;
  for (int first = 0; first < n_problems; first += kMaxSelProblems) {
    const int count = n_problems - first < kMaxSelProblems ? n_problems - first : kMaxSelProblems;
    int64_t widest = 0;
    for (int i = 0; i < count; ++i) {
      a.p[i] = problems[first + i];
      if (a.p[i].capacity > widest) widest = a.p[i].capacity;
    }
    if (widest == 0) continue;
    a.n_problems = count;
    int64_t bx = (widest + rows_per_block - 1) / rows_per_block;
    const int64_t most = count > 1 ? kCompactBlocks : 4 * kCompactBlocks;   // a problem alone: one pass for up to 16K rows
    if (bx > most) bx = most;
    const dim3 grid((unsigned)bx, count), block(kCompactThreads);
    ProfScope ps(KID_COMPACT, s);
    switch (lpr) {
      case 8: hipLaunchKernelGGL(compact_kernel<8>, grid, block, 0, s, a); break;
      case 16: hipLaunchKernelGGL(compact_kernel<16>, grid, block, 0, s, a); break;
      case 32: hipLaunchKernelGGL(compact_kernel<32>, grid, block, 0, s, a); break;
      default: return LAVA_ERR_SHAPE;
    }
    const int32_t st = launch_status();
    if (st != LAVA_OK) return st;
  }
  return LAVA_OK;
}

int32_t launch_compact(const lava_layer_desc& d, int64_t n, const int64_t* src_offsets, const void* k,
                       const void* v, const int32_t* pos_src, const int64_t* head_offsets,
                       const int32_t* kept_idx, int64_t capacity, void* k_out, void* v_out, int32_t* pos_out,
                       hipStream_t s) {
  lava_compact_problem pr;
  pr.src_rows = n;
  pr.src_offsets = src_offsets;
  pr.k_src = k;
  pr.v_src = v;
  pr.pos_src = pos_src;
  pr.head_offsets = head_offsets;
  pr.kept_idx = kept_idx;
  pr.capacity = capacity;
  pr.k_out = k_out;
  pr.v_out = v_out;
  pr.pos_out = pos_out;
  pr.src_offset_dev = nullptr;
  pr.out_offset_dev = nullptr;
  return launch_compact_batch(d, 1, &pr, s);
}

}  // namespace lava
