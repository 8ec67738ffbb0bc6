// Top-B selection over the flattened heads of a layer (Alg. 1, "B_l largest entries based on
// s_l"; the per-head survivor counts are the dynamic head budgets of Sec. 4.1).
//
// The paper's cost statement assumes a min-heap, O(H N log B_l); on a GPU the same result
// comes from a most-significant-digit radix select: three histogram passes (11 + 11 + 10 bits
// of an order-preserving integer image of the score) find the exact threshold key T and how
// many entries equal to T must still be taken; ties are resolved by ascending flat index with
// an ordered scan, so the survivor set is unique and the output needs no floating-point
// comparison at all.  Survivors are written in flat order, which is exactly "heads
// concatenated, ascending position inside each head".
#include "common.h"

namespace lava {

constexpr int kSelThreads = 256;
constexpr int kSelPerThread = 16;
constexpr int kSelChunk = kSelThreads * kSelPerThread;  // entries per workgroup
constexpr int kBins = 2048;
constexpr int kMaxHeads = 64;

struct SelectState {
  unsigned int prefix;       // digits of the threshold key decided so far
  unsigned int reserved;
  long long need;            // survivors still to take among keys that match `prefix`
  long long budget_eff;      // number of survivors
  unsigned int ticket[8];    // "last workgroup done" counters: 0-2 histogram passes, 3 count, 4 write
};

SelectWorkspace make_select_workspace(int64_t total) {
  SelectWorkspace w;
  w.n_blocks = (int)((total + kSelChunk - 1) / kSelChunk);
  if (w.n_blocks < 1) w.n_blocks = 1;
  size_t off = 0;
  w.off_hist = off;  off += align_up(sizeof(unsigned int) * 3 * kBins);
  w.off_state = off; off += align_up(sizeof(SelectState));
  w.off_blk = off;   off += align_up(sizeof(unsigned int) * 4 * (size_t)w.n_blocks);
  w.bytes = off;
  return w;
}

// Order-preserving map float -> uint32 (larger score = larger key); -0 and +0 coincide.
__device__ __forceinline__ unsigned int score_key(float f) {
  unsigned int b = __float_as_uint(f);
  if ((b << 1) == 0u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ unsigned int ld_agent(const unsigned int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Returns true in every thread of the workgroup that finishes last.
__device__ __forceinline__ bool last_block_done(unsigned int* ticket, unsigned int n_blocks) {
  __shared__ unsigned int s_last;
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned int t = atomicAdd(ticket, 1u);
    s_last = (t == n_blocks - 1) ? 1u : 0u;
  }
  __syncthreads();
  const bool last = s_last != 0u;
  if (last) __threadfence();
  return last;
}

__global__ void __launch_bounds__(kSelThreads)
sel_init_kernel(unsigned int* __restrict__ hist, SelectState* __restrict__ st,
                int32_t* __restrict__ head_counts, int n_heads, long long total, long long budget,
                const int64_t* __restrict__ budget_dev) {
  for (int i = threadIdx.x; i < 3 * kBins; i += kSelThreads) hist[i] = 0u;
  if (threadIdx.x < n_heads) head_counts[threadIdx.x] = 0;
  if (threadIdx.x == 0) {
    long long b = budget;
    if (budget_dev != nullptr) {
      const long long d = (long long)*budget_dev;
      b = d < b ? d : b;
    }
    if (b > total) b = total;
    if (b < 0) b = 0;
    st->prefix = 0u;
    st->reserved = 0u;
    st->need = b;
    st->budget_eff = b;
    for (int i = 0; i < 8; ++i) st->ticket[i] = 0u;
  }
}

// One radix pass: histogram of digit PASS among the keys whose higher digits equal the prefix
// found so far; the last workgroup to finish then picks the digit that holds the need-th
// largest key and updates (prefix, need).
template <int PASS>
__global__ void __launch_bounds__(kSelThreads)
sel_hist_kernel(const float* __restrict__ scores, long long total, unsigned int* __restrict__ hist,
                SelectState* __restrict__ st) {
  constexpr int kShift = PASS == 0 ? 21 : (PASS == 1 ? 10 : 0);
  constexpr int kDigitBits = PASS == 2 ? 10 : 11;
  constexpr int kNumBins = 1 << kDigitBits;
  constexpr int kHiShift = kShift + kDigitBits;   // bits above this digit
  __shared__ unsigned int s_hist[kBins];
  __shared__ unsigned int s_sum[kSelThreads];
  unsigned int* ghist = hist + PASS * kBins;

  for (int i = threadIdx.x; i < kNumBins; i += kSelThreads) s_hist[i] = 0u;
  const unsigned int prefix = PASS == 0 ? 0u : st->prefix;
  __syncthreads();

  const long long base = (long long)blockIdx.x * kSelChunk;
#pragma unroll 4
  for (int j = 0; j < kSelPerThread; ++j) {
    const long long p = base + j * kSelThreads + threadIdx.x;
    if (p < total) {
      const unsigned int key = score_key(scores[p]);
      const bool match = PASS == 0 ? true : ((key >> kHiShift) == prefix);
      if (match) atomicAdd(&s_hist[(key >> kShift) & (kNumBins - 1)], 1u);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kNumBins; i += kSelThreads) {
    const unsigned int c = s_hist[i];
    if (c) atomicAdd(&ghist[i], c);
  }

  if (!last_block_done(&st->ticket[PASS], gridDim.x)) return;

  // ---- digit pick (one workgroup): thread t owns bins [t*per, (t+1)*per), scanned from the top
  constexpr int kPer = kNumBins / kSelThreads;
  unsigned int cnt[kPer];
  unsigned int mine = 0u;
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    cnt[j] = ld_agent(&ghist[threadIdx.x * kPer + j]);
    mine += cnt[j];
  }
  // inclusive suffix sums over threads (Hillis-Steele in LDS)
  s_sum[threadIdx.x] = mine;
  __syncthreads();
  for (int off = 1; off < kSelThreads; off <<= 1) {
    unsigned int add = (threadIdx.x + off < kSelThreads) ? s_sum[threadIdx.x + off] : 0u;
    __syncthreads();
    s_sum[threadIdx.x] += add;
    __syncthreads();
  }
  const long long need = st->need;
  const long long above_me = (long long)s_sum[threadIdx.x] - mine;  // keys in bins owned by higher threads
  __syncthreads();
  if (need <= 0) {
    if (threadIdx.x == 0) st->prefix = (prefix << kDigitBits) | (unsigned int)(kNumBins - 1);
    return;
  }
  if (above_me < need && need <= above_me + (long long)mine) {
    long long above = above_me;
    for (int j = kPer - 1; j >= 0; --j) {
      if (need <= above + (long long)cnt[j]) {
        st->prefix = (prefix << kDigitBits) | (unsigned int)(threadIdx.x * kPer + j);
        st->need = need - above;
        break;
      }
      above += cnt[j];
    }
  }
}

// Per-workgroup counts of keys above / equal to the threshold; the last workgroup turns them
// into output offsets and the number of threshold-equal entries each workgroup may keep.
__global__ void __launch_bounds__(kSelThreads)
sel_count_kernel(const float* __restrict__ scores, long long total, SelectState* __restrict__ st,
                 unsigned int* __restrict__ blk, int n_blocks) {
  __shared__ unsigned int s_gt[kSelThreads / 64], s_eq[kSelThreads / 64];
  __shared__ unsigned long long s_scan[kSelThreads];
  const unsigned int T = st->prefix;
  const long long base = (long long)blockIdx.x * kSelChunk;
  unsigned int gt = 0u, eq = 0u;
#pragma unroll 4
  for (int j = 0; j < kSelPerThread; ++j) {
    const long long p = base + j * kSelThreads + threadIdx.x;
    if (p < total) {
      const unsigned int key = score_key(scores[p]);
      gt += key > T;
      eq += key == T;
    }
  }
  for (int off = 32; off > 0; off >>= 1) {
    gt += __shfl_down(gt, off);
    eq += __shfl_down(eq, off);
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { s_gt[wave] = gt; s_eq[wave] = eq; }
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned int g = 0u, e = 0u;
    for (int i = 0; i < kSelThreads / 64; ++i) { g += s_gt[i]; e += s_eq[i]; }
    blk[blockIdx.x] = g;
    blk[n_blocks + blockIdx.x] = e;
  }

  if (!last_block_done(&st->ticket[3], gridDim.x)) return;

  // ---- scan over workgroups (one workgroup): thread t owns a contiguous run of workgroups
  const long long need = st->need;
  const int per = (n_blocks + kSelThreads - 1) / kSelThreads;
  const int b0 = threadIdx.x * per;
  const int b1 = b0 + per < n_blocks ? b0 + per : n_blocks;
  unsigned long long sum_gt = 0ull, sum_eq = 0ull;
  for (int b = b0; b < b1; ++b) {
    sum_gt += ld_agent(&blk[b]);
    sum_eq += ld_agent(&blk[n_blocks + b]);
  }
  // exclusive prefix of (gt, eq) over threads; both fit 32 bits, packed in one 64-bit word
  s_scan[threadIdx.x] = (sum_gt << 32) | sum_eq;
  __syncthreads();
  for (int off = 1; off < kSelThreads; off <<= 1) {
    unsigned long long add = (threadIdx.x >= (unsigned)off) ? s_scan[threadIdx.x - off] : 0ull;
    __syncthreads();
    s_scan[threadIdx.x] += add;
    __syncthreads();
  }
  const unsigned long long incl = s_scan[threadIdx.x];
  long long gt_before = (long long)(incl >> 32) - (long long)sum_gt;
  long long eq_before = (long long)(incl & 0xffffffffull) - (long long)sum_eq;
  for (int b = b0; b < b1; ++b) {
    const long long g = ld_agent(&blk[b]);
    const long long e = ld_agent(&blk[n_blocks + b]);
    const long long taken_before = eq_before < need ? eq_before : need;
    blk[2 * n_blocks + b] = (unsigned int)(gt_before + taken_before);   // first output slot
    blk[3 * n_blocks + b] = (unsigned int)(eq_before < 0xffffffffll ? eq_before : 0xffffffffll);
    gt_before += g;
    eq_before += e;
  }
}

// Ordered write of the survivors of one chunk.
__global__ void __launch_bounds__(kSelThreads)
sel_write_kernel(const float* __restrict__ scores, long long total, int n_heads,
                 const int64_t* __restrict__ seg_offsets, SelectState* __restrict__ st,
                 const unsigned int* __restrict__ blk, int n_blocks,
                 int32_t* __restrict__ head_counts, int64_t* __restrict__ head_offsets,
                 int32_t* __restrict__ kept_idx, float* __restrict__ kept_scores) {
  __shared__ float s_val[kSelChunk + 64];
  __shared__ long long s_off[kMaxHeads + 1];
  __shared__ unsigned int s_cnt[kMaxHeads];
  __shared__ unsigned int s_wave[kSelThreads / 64];

  const long long base = (long long)blockIdx.x * kSelChunk;
  for (int j = 0; j < kSelPerThread; ++j) {
    const int i = j * kSelThreads + threadIdx.x;
    const long long p = base + i;
    s_val[i + (i >> 6)] = p < total ? scores[p] : 0.0f;   // one pad word per 64 against bank clashes
  }
  if (threadIdx.x <= n_heads) {
    const long long seg = total / n_heads;
    s_off[threadIdx.x] = seg_offsets ? (long long)seg_offsets[threadIdx.x]
                                     : (threadIdx.x == n_heads ? total : seg * threadIdx.x);
  }
  if (threadIdx.x < kMaxHeads) s_cnt[threadIdx.x] = 0u;
  const unsigned int T = st->prefix;
  const long long need = st->need;
  const unsigned int out0 = blk[2 * n_blocks + blockIdx.x];
  const long long eq0 = (long long)blk[3 * n_blocks + blockIdx.x];
  __syncthreads();

  // this thread's 16 consecutive entries
  float val[kSelPerThread];
  unsigned int gt_mask = 0u, eq_mask = 0u;
  const int first = threadIdx.x * kSelPerThread;
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    const int i = first + j;
    val[j] = s_val[i + (i >> 6)];
    if (base + i < total) {
      const unsigned int key = score_key(val[j]);
      gt_mask |= (key > T ? 1u : 0u) << j;
      eq_mask |= (key == T ? 1u : 0u) << j;
    }
  }
  // exclusive scan of packed (gt << 16 | eq) over the workgroup
  const unsigned int mine = ((unsigned int)__popc(gt_mask) << 16) | (unsigned int)__popc(eq_mask);
  unsigned int incl = mine;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned int up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  unsigned int wave_base = 0u;
  for (int i = 0; i < wave; ++i) wave_base += s_wave[i];
  const unsigned int excl = wave_base + incl - mine;
  long long gt_before = (long long)(excl >> 16);
  long long eq_before = eq0 + (long long)(excl & 0xffffu);

  // walk the entries in flat order
  int g = 0;
  {
    const long long p0 = base + first;
    while (g + 1 < n_heads && p0 >= s_off[g + 1]) ++g;
  }
  unsigned int local_cnt = 0u;
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    const long long p = base + first + j;
    while (g + 1 < n_heads && p >= s_off[g + 1]) {
      if (local_cnt) atomicAdd(&s_cnt[g], local_cnt);
      local_cnt = 0u;
      ++g;
    }
    const bool is_gt = (gt_mask >> j) & 1u;
    const bool is_eq = (eq_mask >> j) & 1u;
    const bool keep = is_gt || (is_eq && eq_before < need);
    if (keep) {
      const long long taken_before = eq_before < need ? eq_before : need;
      const long long slot = (long long)out0 + gt_before + (taken_before - (eq0 < need ? eq0 : need));
      kept_idx[slot] = (int32_t)(p - s_off[g]);
      if (kept_scores) kept_scores[slot] = val[j];
      ++local_cnt;
    }
    gt_before += is_gt;
    eq_before += is_eq;
  }
  if (local_cnt) atomicAdd(&s_cnt[g], local_cnt);
  __syncthreads();
  if (threadIdx.x < n_heads) {
    const unsigned int c = s_cnt[threadIdx.x];
    if (c) atomicAdd(reinterpret_cast<unsigned int*>(&head_counts[threadIdx.x]), c);
  }

  if (!last_block_done(&st->ticket[4], gridDim.x)) return;
  if (threadIdx.x == 0) {
    long long acc = 0;
    for (int h = 0; h < n_heads; ++h) {
      head_offsets[h] = acc;
      acc += (long long)ld_agent(reinterpret_cast<const unsigned int*>(&head_counts[h]));
    }
    head_offsets[n_heads] = acc;
  }
}

int32_t launch_select(int n_heads, const float* scores, const int64_t* seg_offsets, int64_t total,
                      int64_t budget, const int64_t* budget_dev, int32_t* head_counts,
                      int64_t* head_offsets, int32_t* kept_idx, float* kept_scores, void* ws,
                      hipStream_t s) {
  const SelectWorkspace w = make_select_workspace(total);
  char* base = static_cast<char*>(ws);
  unsigned int* hist = reinterpret_cast<unsigned int*>(base + w.off_hist);
  SelectState* st = reinterpret_cast<SelectState*>(base + w.off_state);
  unsigned int* blk = reinterpret_cast<unsigned int*>(base + w.off_blk);
  const dim3 grid(w.n_blocks), block(kSelThreads);
  {
    ProfScope ps(KID_SEL_INIT, s);
    hipLaunchKernelGGL(sel_init_kernel, dim3(1), block, 0, s, hist, st, head_counts, n_heads,
                       (long long)total, (long long)budget, budget_dev);
  }
  {
    ProfScope ps(KID_SEL_HIST, s);
    hipLaunchKernelGGL(sel_hist_kernel<0>, grid, block, 0, s, scores, (long long)total, hist, st);
    hipLaunchKernelGGL(sel_hist_kernel<1>, grid, block, 0, s, scores, (long long)total, hist, st);
    hipLaunchKernelGGL(sel_hist_kernel<2>, grid, block, 0, s, scores, (long long)total, hist, st);
  }
  {
    ProfScope ps(KID_SEL_COUNT, s);
    hipLaunchKernelGGL(sel_count_kernel, grid, block, 0, s, scores, (long long)total, st, blk,
                       w.n_blocks);
  }
  {
    ProfScope ps(KID_SEL_WRITE, s);
    hipLaunchKernelGGL(sel_write_kernel, grid, block, 0, s, scores, (long long)total, n_heads,
                       seg_offsets, st, blk, w.n_blocks, head_counts, head_offsets, kept_idx,
                       kept_scores);
  }
  return launch_status();
}

}  // namespace lava
