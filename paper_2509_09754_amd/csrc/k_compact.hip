// Compaction of the surviving K/V rows into the packed per-head cache (Alg. 1, last loop:
// K^ = K (.) I, V^ = V (.) I, stored without the evicted rows).  A pure gather: every row is
// moved with 128-bit loads and stores, one row per group of (row bytes / 16) lanes.
#include "common.h"
#include "xblock.h"

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

// ------------------------------------------------------------------------------------------
// In-place re-compaction of the earlier layers of a cascade arena (Alg. 2, inner loop, without a
// second arena for K and V).
//
// After a step's selections every surviving row's new place is at or before its old one: layers
// only shrink (a layer keeps min(budget, rows it holds)), so every layer starts at or before
// where it started; inside a layer every head keeps a subset of its rows, so every head starts at
// or before where it started; and inside a head the survivors keep their order.  A gather that
// overwrites its own source is then safe if rows are taken in passes of increasing NEW position
// and, within a pass, every row is read before any row is written: what a pass overwrites lies
// before everything later passes still have to read, and what it reads has not been overwritten
// by earlier passes.  A pass therefore loads its rows into registers, the whole grid meets at a
// barrier, and the pass stores them.  The grid is sized to stay resident (the barrier's wait is
// bounded like the selection's: if it gives up the state's error word is set).
// ------------------------------------------------------------------------------------------
constexpr int kInplaceThreads = 1024;   // few, large workgroups: the grid barrier costs per workgroup
constexpr int kInplaceRows = 8;          // rows a lane group holds in registers per pass
constexpr int kInplaceMaxLayers = 1024;
constexpr int kInplaceStaged = 2304;     // head offsets (layers x (heads + 1)) kept in LDS: 256 layers of 8 heads, 35 of 64

struct InplaceArgs {
  int n_layers, n_heads;
  const int64_t* start_cur;   // [>= n_layers]
  const int64_t* start_new;   // [>= n_layers + 1]
  const int64_t* offs_cur;    // [n_layers][n_heads + 1]
  const int64_t* offs_new;
  const int32_t* kept_idx;    // by new arena row
  uint4* k;
  uint4* v;
  const int32_t* pos_src;
  int32_t* pos_dst;
  long long capacity;
  unsigned int* sync;         // kArriveWords zeroed words: arrivals (monotonic)
  int32_t* error;             // set to 1 if a wait gave up, or null
  unsigned int spin_limit;
};

template <int LPR>
__global__ void __launch_bounds__(kInplaceThreads) compact_inplace_kernel(const InplaceArgs a) {
  __shared__ long long s_new[kInplaceMaxLayers + 1], s_cur[kInplaceMaxLayers];
  __shared__ long long s_on[kInplaceStaged], s_oc[kInplaceStaged];
  for (int i = threadIdx.x; i <= a.n_layers; i += kInplaceThreads) {
    s_new[i] = (long long)a.start_new[i];
    if (i < a.n_layers) s_cur[i] = (long long)a.start_cur[i];
  }
  // the head offsets of every layer, old and new: a row's head is found by a search that would otherwise
  // be a chain of dependent loads from memory per row (stacks too deep for the table read them from memory)
  const int n_offs = a.n_layers * (a.n_heads + 1);
  const bool staged = n_offs <= kInplaceStaged;               // uniform
  if (staged)
    for (int i = threadIdx.x; i < n_offs; i += kInplaceThreads) {
      s_on[i] = (long long)a.offs_new[i];
      s_oc[i] = (long long)a.offs_cur[i];
    }
  __syncthreads();
  long long rows = s_new[a.n_layers];                         // rows the earlier layers keep
  if (rows > a.capacity) rows = a.capacity;
  constexpr int kGroups = kInplaceThreads / LPR;
  const int c = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  const long long per_pass = (long long)gridDim.x * kGroups * kInplaceRows;
  const int H = a.n_heads;
  unsigned int round = 0u;
  for (long long base = 0; base < rows; base += per_pass) {
    uint4 kv[kInplaceRows], vv[kInplaceRows];
    unsigned int moves = 0u;                                  // bit u: row u of this pass is moved by this lane group
#pragma unroll
    for (int u = 0; u < kInplaceRows; ++u) {
      const long long r = base + ((long long)u * gridDim.x + blockIdx.x) * kGroups + grp;
      long long src = 0;                                      // a row that is not moved reads row 0 and stores nothing
      if (r < rows) {
        int lo = 0, hi = a.n_layers - 1;                      // the layer: largest t with s_new[t] <= r
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if (s_new[mid] <= r) lo = mid; else hi = mid - 1;
        }
        const int t = lo;
        const long long j = r - s_new[t];
        const long long idx = (long long)a.kept_idx[r];
        long long kept_t, oc0, oc1;                           // rows layer t keeps; the head's old segment
        if (staged) {
          const long long* on = s_on + t * (H + 1);
          int g = 0;
          while (g + 1 < H && j >= on[g + 1]) ++g;
          kept_t = on[H];
          oc0 = s_oc[t * (H + 1) + g];
          oc1 = s_oc[t * (H + 1) + g + 1];
        } else {
          const int64_t* on = a.offs_new + (long long)t * (H + 1);
          int g = 0;
          while (g + 1 < H && j >= (long long)on[g + 1]) ++g;
          kept_t = (long long)on[H];
          oc0 = (long long)a.offs_cur[(long long)t * (H + 1) + g];
          oc1 = (long long)a.offs_cur[(long long)t * (H + 1) + g + 1];
        }
        const long long from = s_cur[t] + oc0 + idx;
        // never follow an index outside the head's old segment, never move a row backwards
        if (j < kept_t && idx >= 0 && idx < oc1 - oc0 && from >= r && from < a.capacity) {
          src = from;
          moves |= 1u << u;
          if (c == 0) a.pos_dst[r] = a.pos_src[from];
        }
      }
      kv[u] = a.k[src * LPR + c];
      vv[u] = a.v[src * LPR + c];
    }
    // every row of the pass is in registers before any is written
    drain_vmem();
    __syncthreads();
    if (threadIdx.x == 0) {
      // arrivals in two levels (hundreds of atomics on one address would serialise), then a bounded wait
      // for the top counter: one increment per completed group and round
      ++round;
      arrive_two_level(a.sync, gridDim.x, blockIdx.x, round);
      const unsigned int target = round * arrive_groups(gridDim.x);
      unsigned int spins = 0u;
      while (ld_dev(&a.sync[0]) < target) {
        __builtin_amdgcn_s_sleep(16);                          // polls are device-scope loads of one address: keep them rare
        if (++spins > a.spin_limit) {
          if (a.error != nullptr) *a.error = 1;
          break;
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kInplaceRows; ++u) {
      if (moves & (1u << u)) {
        const long long r = base + ((long long)u * gridDim.x + blockIdx.x) * kGroups + grp;
        a.k[r * LPR + c] = kv[u];
        a.v[r * LPR + c] = vv[u];
      }
    }
  }
}

int32_t launch_compact_inplace(const lava_layer_desc& d, int n_layers, const int64_t* layer_start_cur,
                               const int64_t* layer_start_new, const int64_t* offs_cur, const int64_t* offs_new,
                               const int32_t* kept_idx, void* k, void* v, const int32_t* pos_src, int32_t* pos_dst,
                               int64_t capacity, unsigned int* sync, int32_t* error, hipStream_t s) {
  if (n_layers < 1) return LAVA_OK;
  if (n_layers > kInplaceMaxLayers) return LAVA_ERR_SHAPE;
  const int lpr = d.head_dim * (d.dtype == LAVA_BF16 ? 2 : 4) / 16;
  InplaceArgs a;
  a.n_layers = n_layers;
  a.n_heads = d.n_kv_heads;
  a.start_cur = layer_start_cur;
  a.start_new = layer_start_new;
  a.offs_cur = offs_cur;
  a.offs_new = offs_new;
  a.kept_idx = kept_idx;
  a.k = static_cast<uint4*>(k);
  a.v = static_cast<uint4*>(v);
  a.pos_src = pos_src;
  a.pos_dst = pos_dst;
  a.capacity = capacity;
  a.sync = sync;
  a.error = error;
  a.spin_limit = tuning().barrier_spin_limit > 0 ? (unsigned int)tuning().barrier_spin_limit : 1u << 18;
  // all workgroups have to be resident at once: one per compute unit at most, fewer for a small arena
  int cus = 0, dev = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    cus = 256;
  const int64_t rows_per_wg = (int64_t)(kInplaceThreads / lpr) * kInplaceRows;
  int64_t wgs = (capacity + rows_per_wg - 1) / rows_per_wg;
  if (wgs > (int64_t)cus) wgs = (int64_t)cus;
  if (wgs < 1) wgs = 1;
  const dim3 grid((unsigned)wgs), block(kInplaceThreads);
  ProfScope ps(KID_COMPACT, s);
  switch (lpr) {
    case 8: hipLaunchKernelGGL(compact_inplace_kernel<8>, grid, block, 0, s, a); break;
    case 16: hipLaunchKernelGGL(compact_inplace_kernel<16>, grid, block, 0, s, a); break;
    case 32: hipLaunchKernelGGL(compact_inplace_kernel<32>, grid, block, 0, s, a); break;
    default: return LAVA_ERR_SHAPE;
  }
  return launch_status();
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
