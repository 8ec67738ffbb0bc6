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
//
// The whole selection is latency-bound (a few MiB of scores), so it runs as ONE kernel whose
// workgroups (1024 lanes, 16 scores per lane in registers) meet at four grid-wide barriers; every
// workgroup derives the digit picks and its output offset redundantly from the shared
// histograms / per-workgroup counts, so no workgroup waits for a "leader".  Inputs too large for
// all workgroups to be resident at once fall back to the same phases as separate kernels.
#include "common.h"
#include "xblock.h"

namespace lava {

constexpr int kSelThreads = 1024;   // few, large workgroups: grid-wide barriers and histogram merges cost per workgroup
constexpr int kSelPerThread = 16;
constexpr int kSelChunk = kSelThreads * kSelPerThread;  // entries per workgroup
constexpr int kBins = kSelBins;
constexpr int kMaxHeads = 64;
constexpr unsigned int kSpinLimit = 1u << 18;           // polls of a grid barrier before giving up (default)

// The fused kernel's last histogram pass also publishes, per workgroup, how many of its keys lie
// above each possible last digit (kPubWords = 1024 digits + 1), so that the counts every
// workgroup needs from those before it are two loads once the threshold is known.
constexpr int kPubWords = 1025;
constexpr int kFusedMaxBlocks = 1024;   // more workgroups than any device keeps resident

struct SelectState {
  unsigned int barrier;      // arrivals at the grid barriers of the fused kernel (monotonic)
  unsigned int error;        // set when a barrier wait gave up (results are then invalid)
  unsigned int done;         // workgroups of the fused kernel that have written their results
  unsigned int reserved[5];
};
static_assert(sizeof(SelectState) == kSelStateWords * sizeof(unsigned int), "cleared word by word by the score kernels");

// Layout of a selection's workspace for `total` entries (also evaluated at compile time, for the
// built-in scratch array of lava_select_topk_static).
static constexpr SelectWorkspace select_layout(int64_t total) {
  SelectWorkspace w{};
  w.n_blocks = (int)((total + kSelChunk - 1) / kSelChunk);
  if (w.n_blocks < 1) w.n_blocks = 1;
  size_t off = 0;
  w.off_hist = off;  off += align_up(sizeof(unsigned int) * 3 * kBins);
  w.off_state = off; off += align_up(sizeof(SelectState));
  // per-workgroup counts: two words per workgroup for the step launches; the fused kernel publishes
  // kPubWords per workgroup (it serves problems of up to kFusedMaxBlocks workgroups)
  size_t words = 2 * (size_t)w.n_blocks;
  const size_t fused = (size_t)(w.n_blocks < kFusedMaxBlocks ? w.n_blocks : kFusedMaxBlocks) * kPubWords;
  if (fused > words) words = fused;
  w.off_blk = off;   off += align_up(sizeof(unsigned int) * words);
  w.bytes = off;
  return w;
}

SelectWorkspace make_select_workspace(int64_t total) { return select_layout(total); }

struct SelShared {
  union {
    float val[kSelChunk + 64];        // staging of the chunk (one pad word per 64 entries)
    unsigned int hist[kBins];         // per-workgroup digit histogram
  };
  long long off[kMaxHeads + 1];       // segment starts
  unsigned int cnt[kMaxHeads];        // survivors per head in this workgroup
  unsigned int wave[kSelThreads / 64];
  unsigned long long wave64[kSelThreads / 64];
  unsigned int pick_digit;
  long long pick_need;
};

// Where the selection stands: digits of the threshold key found so far and how many survivors
// must still come from the keys that match them.
struct Pick {
  unsigned int prefix;
  long long need;
};

__device__ __forceinline__ long long effective_budget(long long budget, const int64_t* budget_dev,
                                                      long long total) {
  long long b = budget;
  if (budget_dev != nullptr) {
    const long long d = (long long)*budget_dev;
    b = d < b ? d : b;
  }
  if (b > total) b = total;
  if (b < 0) b = 0;
  return b;
}

// Chunk -> registers: coalesced reads through shared memory, then 16 consecutive entries per lane
// (flat order inside the workgroup = lane order, which the ordered write needs).
__device__ __forceinline__ void load_chunk(int bx, const float* __restrict__ scores, long long total,
                                           SelShared& sh, float (&val)[kSelPerThread]) {
  const long long base = (long long)bx * kSelChunk;
  float tmp[kSelPerThread];
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {        // all loads in flight before the first use
    const long long p = base + j * kSelThreads + threadIdx.x;
    tmp[j] = p < total ? scores[p] : 0.0f;
  }
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    const int i = j * kSelThreads + threadIdx.x;
    sh.val[i + (i >> 6)] = tmp[j];
  }
  __syncthreads();
  const int first = threadIdx.x * kSelPerThread;
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) val[j] = sh.val[first + j + ((first + j) >> 6)];
  __syncthreads();
}

template <int PASS> struct Digit {
  static constexpr int kShift = PASS == 0 ? 21 : (PASS == 1 ? 10 : 0);
  static constexpr int kBits = PASS == 2 ? 10 : 11;
  static constexpr int kNum = 1 << kBits;
  static constexpr int kHiShift = kShift + kBits;
};

// Histogram of digit PASS over this workgroup's keys that match the prefix; merged into the
// global histogram with integer atomics.
template <int PASS>
__device__ __forceinline__ void hist_phase(int bx, const float (&val)[kSelPerThread], long long total,
                                           unsigned int prefix, SelShared& sh,
                                           unsigned int* __restrict__ ghist) {
  using Dg = Digit<PASS>;
  for (int i = threadIdx.x; i < Dg::kNum; i += kSelThreads) sh.hist[i] = 0u;
  __syncthreads();
  const long long p0 = (long long)bx * kSelChunk + threadIdx.x * kSelPerThread;
  // neighbouring entries mostly share a digit (pooling makes plateaus, magnitudes vary slowly), so a
  // lane adds one count per run of equal digits instead of one per entry
  unsigned int run_digit = 0xffffffffu, run_len = 0u;
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    unsigned int digit = 0xffffffffu;
    if (p0 + j < total) {
      const unsigned int key = score_key(val[j]);
      const bool match = PASS == 0 ? true : ((key >> Dg::kHiShift) == prefix);
      if (match) digit = (key >> Dg::kShift) & (Dg::kNum - 1);
    }
    if (digit != run_digit) {
      if (run_len != 0u && run_digit != 0xffffffffu) atomicAdd(&sh.hist[run_digit], run_len);
      run_digit = digit;
      run_len = 0u;
    }
    ++run_len;
  }
  if (run_digit != 0xffffffffu) atomicAdd(&sh.hist[run_digit], run_len);
  __syncthreads();
  for (int i = threadIdx.x; i < Dg::kNum; i += kSelThreads) {
    const unsigned int c = sh.hist[i];
    if (c) __hip_atomic_fetch_add(&ghist[i], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// Digit of the threshold key: the bin, counted from the top, in which the cumulative count
// reaches `need`.  Every workgroup computes it for itself from the complete global histogram.
template <int PASS>
__device__ __forceinline__ Pick pick_phase(const unsigned int* __restrict__ ghist, Pick in,
                                           SelShared& sh) {
  using Dg = Digit<PASS>;
  constexpr int kPer = Dg::kNum / kSelThreads;
  // thread t owns the bins kNum-1 - t*kPer - j (descending), so a prefix scan over t runs from the top
  unsigned int cnt[kPer];
  unsigned int mine = 0u;
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    cnt[j] = ld_dev(&ghist[Dg::kNum - 1 - (threadIdx.x * kPer + j)]);
    mine += cnt[j];
  }
  unsigned int incl = mine;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned int up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  if (lane == 63) sh.wave[wave] = incl;
  if (threadIdx.x == 0) {
    sh.pick_digit = (unsigned int)(Dg::kNum - 1);     // taken when need == 0: nothing matches below
    sh.pick_need = 0;
  }
  __syncthreads();
  long long above = 0;
  for (int i = 0; i < wave; ++i) above += sh.wave[i];
  above += (long long)incl - mine;                     // keys in bins above this thread's bins
  if (in.need > 0 && above < in.need && in.need <= above + (long long)mine) {
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      if (in.need <= above + (long long)cnt[j]) {
        sh.pick_digit = (unsigned int)(Dg::kNum - 1 - (threadIdx.x * kPer + j));
        sh.pick_need = in.need - above;
        break;
      }
      above += cnt[j];
    }
  }
  __syncthreads();
  Pick out;
  out.prefix = (in.prefix << Dg::kBits) | sh.pick_digit;
  out.need = sh.pick_need;
  __syncthreads();
  return out;
}

// Keys above / equal to the threshold in this workgroup, published for the other workgroups.
__device__ __forceinline__ void count_phase(int bx, const float (&val)[kSelPerThread], long long total,
                                            unsigned int T, SelShared& sh, unsigned int* __restrict__ blk,
                                            int n_blocks, unsigned int& gt_mask, unsigned int& eq_mask) {
  const long long p0 = (long long)bx * kSelChunk + threadIdx.x * kSelPerThread;
  gt_mask = 0u;
  eq_mask = 0u;
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    if (p0 + j < total) {
      const unsigned int key = score_key(val[j]);
      gt_mask |= (key > T ? 1u : 0u) << j;
      eq_mask |= (key == T ? 1u : 0u) << j;
    }
  }
  unsigned int packed = ((unsigned int)__popc(gt_mask) << 16) | (unsigned int)__popc(eq_mask);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) packed += __shfl_xor(packed, off);
  if ((threadIdx.x & 63) == 0) sh.wave[threadIdx.x >> 6] = packed;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned int tot = 0u;
    for (int i = 0; i < kSelThreads / 64; ++i) tot += sh.wave[i];
    st_dev(&blk[bx], tot >> 16);
    st_dev(&blk[n_blocks + bx], tot & 0xffffu);
  }
  __syncthreads();
}

// Sums of (gt, eq) over the workgroups before this one.
__device__ __forceinline__ void prefix_phase(int bx, const unsigned int* __restrict__ blk, int n_blocks,
                                             SelShared& sh, long long& gt_before, long long& eq_before) {
  unsigned long long acc = 0ull;   // gt in the high word, eq in the low word (each < 2^31)
  for (int b = threadIdx.x; b < bx; b += kSelThreads)
    acc += ((unsigned long long)ld_dev(&blk[b]) << 32) | (unsigned long long)ld_dev(&blk[n_blocks + b]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if ((threadIdx.x & 63) == 0) sh.wave64[threadIdx.x >> 6] = acc;
  __syncthreads();
  unsigned long long tot = 0ull;
  for (int i = 0; i < kSelThreads / 64; ++i) tot += sh.wave64[i];
  gt_before = (long long)(tot >> 32);
  eq_before = (long long)(tot & 0xffffffffull);
  __syncthreads();
}

// Ordered write of this workgroup's survivors; survivors per head are added to head_counts and the
// head offsets are written by the lanes that own the first entry of each head.
__device__ __forceinline__ void write_phase(int bx, const float (&val)[kSelPerThread], long long total, int n_heads,
                                            const int64_t* __restrict__ seg_offsets, unsigned int gt_mask,
                                            unsigned int eq_mask, long long need, long long capacity,
                                            long long gt_blocks_before, long long eq_blocks_before,
                                            long long need_total, SelShared& sh,
                                            int32_t* __restrict__ head_counts, int64_t* __restrict__ head_offsets,
                                            int32_t* __restrict__ kept_idx, float* __restrict__ kept_scores) {
  if (threadIdx.x <= n_heads) {
    const long long seg = total / n_heads;
    sh.off[threadIdx.x] = seg_offsets ? (long long)seg_offsets[threadIdx.x]
                                      : (threadIdx.x == n_heads ? total : seg * threadIdx.x);
  }
  if (threadIdx.x < kMaxHeads) sh.cnt[threadIdx.x] = 0u;
  // exclusive scan of packed (gt << 16 | eq) over the workgroup
  const unsigned int mine = ((unsigned int)__popc(gt_mask) << 16) | (unsigned int)__popc(eq_mask);
  unsigned int incl = mine;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned int up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  if (lane == 63) sh.wave[wave] = incl;
  __syncthreads();
  unsigned int wave_base = 0u;
  for (int i = 0; i < wave; ++i) wave_base += sh.wave[i];
  const unsigned int excl = wave_base + incl - mine;
  long long gt_before = gt_blocks_before + (long long)(excl >> 16);
  long long eq_before = eq_blocks_before + (long long)(excl & 0xffffu);

  const long long first = (long long)bx * kSelChunk + threadIdx.x * kSelPerThread;
  // head_offsets[h] = survivors before the first entry of head h: written by the lane that owns that
  // entry; segments starting at or beyond the end (empty trailing heads) and the two ends by lane 0
  if (bx == 0 && threadIdx.x == 0) {
    const long long kept = need_total;
    head_offsets[0] = 0;
    head_offsets[n_heads] = kept;
    for (int h = 1; h < n_heads; ++h)
      if (sh.off[h] >= total) head_offsets[h] = kept;
  }
  int g = 0;
  while (g + 1 < n_heads && sh.off[g + 1] < first) ++g;     // segment starts equal to `first` are crossed below
  // most lanes never cross a segment start: the next start and this head's start stay in registers
  constexpr long long kNever = 0x7fffffffffffffffll;
  long long next_start = g + 1 < n_heads ? sh.off[g + 1] : kNever;
  long long head_start = sh.off[g];
  unsigned int local_cnt = 0u;
  // most lanes hold no survivor and no segment start (a fraction of a per cent of the entries survive):
  // they have nothing to write
  const bool idle = gt_mask == 0u && (eq_mask == 0u || eq_before >= need) && next_start >= first + kSelPerThread;
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    if (idle) break;
    const long long p = first + j;
    while (p >= next_start) {
      if (local_cnt) atomicAdd(&sh.cnt[g], local_cnt);
      local_cnt = 0u;
      ++g;
      head_start = next_start;
      if (p == head_start && p < total) head_offsets[g] = gt_before + (eq_before < need ? eq_before : need);
      next_start = g + 1 < n_heads ? sh.off[g + 1] : kNever;
    }
    const bool is_gt = (gt_mask >> j) & 1u;
    const bool is_eq = (eq_mask >> j) & 1u;
    if (is_gt || (is_eq && eq_before < need)) {
      // survivors before this entry in flat order: all larger keys plus the threshold-equal ones taken
      const long long slot = gt_before + (eq_before < need ? eq_before : need);
      if (slot < capacity) {
        kept_idx[slot] = (int32_t)(p - head_start);
        if (kept_scores) kept_scores[slot] = val[j];
      }
      ++local_cnt;
    }
    gt_before += is_gt;
    eq_before += is_eq;
  }
  if (local_cnt) atomicAdd(&sh.cnt[g], local_cnt);
  __syncthreads();
  if (threadIdx.x < n_heads) {
    const unsigned int c = sh.cnt[threadIdx.x];
    if (c) __hip_atomic_fetch_add(reinterpret_cast<unsigned int*>(&head_counts[threadIdx.x]), c,
                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// Last histogram pass of the fused kernel.  Besides merging the workgroup's histogram of the last
// digit (keys matching the 22 digits found so far) into the global one, it publishes
//   pub[d] = #keys of this workgroup above every key that matches the prefix and has last digit < d
//          = #keys whose first 22 bits exceed the prefix + #matching keys with last digit >= d,
// d = 0 .. 1024, so that for a threshold with last digit t the workgroup holds pub[t + 1] keys above
// it and pub[t] - pub[t + 1] equal to it.
__device__ __forceinline__ void hist_publish_phase(int bx, const float (&val)[kSelPerThread], long long total,
                                                   unsigned int prefix, SelShared& sh,
                                                   unsigned int* __restrict__ ghist,
                                                   unsigned int* __restrict__ pub) {
  using Dg = Digit<2>;
  static_assert(Dg::kNum == kSelThreads && Dg::kNum + 1 == kPubWords, "one last digit per thread");
  sh.hist[threadIdx.x] = 0u;
  __syncthreads();
  const long long p0 = (long long)bx * kSelChunk + threadIdx.x * kSelPerThread;
  unsigned int run_digit = 0xffffffffu, run_len = 0u, above = 0u;
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    unsigned int digit = 0xffffffffu;
    if (p0 + j < total) {
      const unsigned int key = score_key(val[j]);
      const unsigned int hi = key >> Dg::kHiShift;
      above += hi > prefix ? 1u : 0u;
      if (hi == prefix) digit = key & (Dg::kNum - 1);
    }
    if (digit != run_digit) {
      if (run_len != 0u && run_digit != 0xffffffffu) atomicAdd(&sh.hist[run_digit], run_len);
      run_digit = digit;
      run_len = 0u;
    }
    ++run_len;
  }
  if (run_digit != 0xffffffffu) atomicAdd(&sh.hist[run_digit], run_len);
  __syncthreads();
  // thread t owns digit kNum - 1 - t: an inclusive scan over t is a suffix sum over the digits
  const int d = Dg::kNum - 1 - (int)threadIdx.x;
  const unsigned int c = sh.hist[d];
  if (c) __hip_atomic_fetch_add(&ghist[d], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  unsigned int incl = c;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned int up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) above += __shfl_xor(above, off);
  if (lane == 63) sh.wave[wave] = incl;
  if (lane == 0) sh.wave64[wave] = above;
  __syncthreads();
  unsigned int base = 0u, above_all = 0u;
  for (int i = 0; i < kSelThreads / 64; ++i) {
    if (i < wave) base += sh.wave[i];
    above_all += (unsigned int)sh.wave64[i];
  }
  st_dev(&pub[d], above_all + base + incl);
  if (threadIdx.x == 0) st_dev(&pub[Dg::kNum], above_all);
  __syncthreads();
}

// This lane's keys above / equal to the threshold.
__device__ __forceinline__ void mask_phase(int bx, const float (&val)[kSelPerThread], long long total,
                                           unsigned int T, unsigned int& gt_mask, unsigned int& eq_mask) {
  const long long p0 = (long long)bx * kSelChunk + threadIdx.x * kSelPerThread;
  gt_mask = 0u;
  eq_mask = 0u;
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    if (p0 + j < total) {
      const unsigned int key = score_key(val[j]);
      gt_mask |= (key > T ? 1u : 0u) << j;
      eq_mask |= (key == T ? 1u : 0u) << j;
    }
  }
}

// Sums of (above, equal) over the workgroups before this one, from what they published.
__device__ __forceinline__ void prefix_published_phase(int bx, const unsigned int* __restrict__ pub_all,
                                                       unsigned int T, SelShared& sh, long long& gt_before,
                                                       long long& eq_before) {
  const unsigned int t = T & (unsigned int)(Digit<2>::kNum - 1);
  unsigned long long acc = 0ull;   // above in the high word, equal in the low word (each < 2^31)
  for (int b = threadIdx.x; b < bx; b += kSelThreads) {
    const unsigned int ge = ld_dev(&pub_all[(size_t)b * kPubWords + t]);
    const unsigned int gt = ld_dev(&pub_all[(size_t)b * kPubWords + t + 1]);
    acc += ((unsigned long long)gt << 32) | (unsigned long long)(ge - gt);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if ((threadIdx.x & 63) == 0) sh.wave64[threadIdx.x >> 6] = acc;
  __syncthreads();
  unsigned long long tot = 0ull;
  for (int i = 0; i < kSelThreads / 64; ++i) tot += sh.wave64[i];
  gt_before = (long long)(tot >> 32);
  eq_before = (long long)(tot & 0xffffffffull);
  __syncthreads();
}

// Grid-wide barrier of the fused kernel: all of its workgroups are resident (the host checks the
// grid against the device's capacity), arrivals are counted monotonically, and the wait is
// bounded: if it ever gives up, the error word is set and the kernel still runs to completion.
__device__ __forceinline__ void grid_sync(SelectState* __restrict__ st, unsigned int round, unsigned int n_blocks,
                                          unsigned int spin_limit) {
  drain_vmem();
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(&st->barrier, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned int target = round * n_blocks;
    unsigned int spins = 0u;
    while (ld_dev(&st->barrier) < target) {
      __builtin_amdgcn_s_sleep(2);
      if (++spins > spin_limit) {
        st_dev(&st->error, 1u);
        break;
      }
    }
  }
  __syncthreads();
}

// One launch serves up to kMaxSelProblems independent selections: the table travels in the kernel
// arguments, and the workgroups of all problems are numbered through (first_block), so every
// workgroup of the grid has work.  Every problem has its own histograms, barrier counter and
// per-workgroup counts in its own region of the workspace, so problems never wait for each other.
struct SelectBatch {
  int n_heads;
  int n_problems;
  int first_block[kMaxSelProblems + 1];   // workgroups of problem p: first_block[p] .. first_block[p + 1] - 1
  char* ws;                      // region of problem p at ws + p * ws_stride
  size_t ws_stride, off_hist, off_state, off_blk;
  int blk_stride;                // n_blocks the regions were laid out for
  unsigned int spin_limit;       // polls of a grid barrier before it gives up
  unsigned int primed_mask;      // bit p: problem p's region was prepared by the score kernels (first histogram
                                 // complete, the rest cleared)
  lava_select_problem p[kMaxSelProblems];
};

__device__ __forceinline__ int problem_blocks(const lava_select_problem& pr) {
  const long long nb = (pr.total_entries + kSelChunk - 1) / kSelChunk;
  return nb < 1 ? 1 : (int)nb;
}

// Problem of this workgroup (uniform over the workgroup).
__device__ __forceinline__ int problem_of_block(const SelectBatch& a) {
  int p = 0;
  while (p + 1 < a.n_problems && (int)blockIdx.x >= a.first_block[p + 1]) ++p;
  return p;
}

__global__ void __launch_bounds__(kSelThreads) sel_init_kernel(const SelectBatch a) {
  const lava_select_problem pr = a.p[blockIdx.x];
  char* region = a.ws + blockIdx.x * a.ws_stride;
  unsigned int* hist = reinterpret_cast<unsigned int*>(region + a.off_hist);
  SelectState* st = reinterpret_cast<SelectState*>(region + a.off_state);
  if (threadIdx.x < a.n_heads) pr.head_counts[threadIdx.x] = 0;
  if ((a.primed_mask >> blockIdx.x) & 1u) return;           // histograms and state are as the score kernels left them
  for (int i = threadIdx.x; i < 3 * kBins; i += kSelThreads) hist[i] = 0u;
  if (threadIdx.x == 0) {
    st->barrier = 0u;
    st->error = 0u;
    st->done = 0u;
  }
}

// With explicit segments the number of entries is whatever the last offset says (read on the
// device, so that a caller can chain selections without a host round trip); the host value is then
// an upper bound that sized the grid and the workspace.
__device__ __forceinline__ long long device_total(long long bound, const int64_t* __restrict__ seg_offsets,
                                                  int n_heads) {
  if (seg_offsets == nullptr) return bound;
  long long t = (long long)seg_offsets[n_heads];
  t = t < 0 ? 0 : t;
  return t < bound ? t : bound;
}

// The whole selection in one launch.
__global__ void __launch_bounds__(kSelThreads) sel_fused_kernel(const SelectBatch a) {
  const int prob = problem_of_block(a);
  const lava_select_problem pr = a.p[prob];
  const unsigned int nb = (unsigned int)problem_blocks(pr);
  const int bx = (int)blockIdx.x - a.first_block[prob];
  char* region = a.ws + prob * a.ws_stride;
  unsigned int* hist = reinterpret_cast<unsigned int*>(region + a.off_hist);
  SelectState* st = reinterpret_cast<SelectState*>(region + a.off_state);
  unsigned int* blk = reinterpret_cast<unsigned int*>(region + a.off_blk);
  const long long in_off = pr.in_offset_dev ? (long long)*pr.in_offset_dev : 0;
  const long long out_off = pr.out_offset_dev ? (long long)*pr.out_offset_dev : 0;
  const float* __restrict__ scores = pr.scores + in_off;
  const int64_t* __restrict__ seg_offsets = pr.seg_offsets;
  const int n_heads = a.n_heads;
  const long long budget = pr.budget;

  __shared__ SelShared sh;
  const long long total = device_total(pr.total_entries, seg_offsets, n_heads);
  float val[kSelPerThread];
  load_chunk(bx, scores, total, sh, val);
  Pick pk;
  pk.prefix = 0u;
  pk.need = effective_budget(budget, pr.budget_dev, total);
  const long long kept_total = pk.need;

  // A primed problem arrives with its first histogram complete (the score kernels built it from the
  // scores they wrote) and everything else cleared: no init launch, no first pass, one barrier fewer.
  // Its survivor counts are cleared here, by a workgroup that passes two barriers before anybody adds to them.
  const bool primed = (a.primed_mask >> prob) & 1u;
  unsigned int round = 0u;
  if (primed) {
    if (bx == 0 && threadIdx.x < (unsigned)n_heads)        // device-scope store: the counts are added to with device-scope atomics
      st_dev(reinterpret_cast<unsigned int*>(&pr.head_counts[threadIdx.x]), 0u);
  } else {
    hist_phase<0>(bx, val, total, pk.prefix, sh, hist);
    grid_sync(st, ++round, nb, a.spin_limit);
  }
  pk = pick_phase<0>(hist, pk, sh);
  hist_phase<1>(bx, val, total, pk.prefix, sh, hist + kBins);
  grid_sync(st, ++round, nb, a.spin_limit);
  pk = pick_phase<1>(hist + kBins, pk, sh);
  hist_publish_phase(bx, val, total, pk.prefix, sh, hist + 2 * kBins, blk + (size_t)bx * kPubWords);
  grid_sync(st, ++round, nb, a.spin_limit);
  pk = pick_phase<2>(hist + 2 * kBins, pk, sh);

  // the counts of the workgroups before this one were published with the last histogram: no
  // further pass over the keys and no fourth barrier
  unsigned int gt_mask, eq_mask;
  mask_phase(bx, val, total, pk.prefix, gt_mask, eq_mask);
  long long gt_before, eq_before;
  prefix_published_phase(bx, blk, pk.prefix, sh, gt_before, eq_before);
  write_phase(bx, val, total, n_heads, seg_offsets, gt_mask, eq_mask, pk.need, budget, gt_before, eq_before,
              kept_total, sh, pr.head_counts, pr.head_offsets, pr.kept_idx + out_off,
              pr.kept_scores ? pr.kept_scores + out_off : nullptr);

  // A wait that gave up leaves results computed from incomplete histograms.  The workgroup that
  // finishes last (every other one has completed its writes before taking its ticket) then replaces
  // them by a mark no consumer can mistake for a selection: no survivors anywhere, counts -1.
  drain_vmem();
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned int t = __hip_atomic_fetch_add(&st->done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sh.wave[0] = (t + 1u == nb && ld_dev(&st->error) != 0u) ? 1u : 0u;
  }
  __syncthreads();
  if (sh.wave[0] != 0u) {
    if (threadIdx.x < (unsigned)n_heads) pr.head_counts[threadIdx.x] = -1;
    if (threadIdx.x <= (unsigned)n_heads) pr.head_offsets[threadIdx.x] = 0;
    if (threadIdx.x == 0 && pr.error_dev != nullptr) *pr.error_dev = 1;
  }
}

// The same phases as separate launches (kernel boundaries take the place of the grid barriers),
// for a problem too large to keep its whole grid resident.  STEP 0..2: histogram pass STEP; 3: counts; 4: write.
template <int STEP>
__global__ void __launch_bounds__(kSelThreads) sel_step_kernel(const SelectBatch a) {
  const int prob = problem_of_block(a);
  const lava_select_problem pr = a.p[prob];
  const int bx = (int)blockIdx.x - a.first_block[prob];
  char* region = a.ws + prob * a.ws_stride;
  unsigned int* hist = reinterpret_cast<unsigned int*>(region + a.off_hist);
  unsigned int* blk = reinterpret_cast<unsigned int*>(region + a.off_blk);
  const int64_t* __restrict__ seg_offsets = pr.seg_offsets;
  const int n_heads = a.n_heads;
  const long long budget = pr.budget;
  __shared__ SelShared sh;
  {
    const long long total = device_total(pr.total_entries, seg_offsets, n_heads);
    float val[kSelPerThread];
    const long long in_off = pr.in_offset_dev ? (long long)*pr.in_offset_dev : 0;
    const long long out_off = pr.out_offset_dev ? (long long)*pr.out_offset_dev : 0;
    load_chunk(bx, pr.scores + in_off, total, sh, val);
    Pick pk;
    pk.prefix = 0u;
    pk.need = effective_budget(budget, pr.budget_dev, total);
    const long long kept_total = pk.need;
    if constexpr (STEP >= 1) pk = pick_phase<0>(hist, pk, sh);
    if constexpr (STEP >= 2) pk = pick_phase<1>(hist + kBins, pk, sh);
    if constexpr (STEP >= 3) pk = pick_phase<2>(hist + 2 * kBins, pk, sh);
    if constexpr (STEP <= 2) {
      hist_phase<STEP>(bx, val, total, pk.prefix, sh, hist + STEP * kBins);
    } else {
      unsigned int gt_mask, eq_mask;
      // counts are recomputed in the write step (cheap) so that both steps share count_phase
      count_phase(bx, val, total, pk.prefix, sh, blk, a.blk_stride, gt_mask, eq_mask);
      if constexpr (STEP == 4) {
        long long gt_before, eq_before;
        prefix_phase(bx, blk, a.blk_stride, sh, gt_before, eq_before);
        write_phase(bx, val, total, n_heads, seg_offsets, gt_mask, eq_mask, pk.need, budget, gt_before, eq_before,
                    kept_total, sh, pr.head_counts, pr.head_offsets, pr.kept_idx + out_off,
                    pr.kept_scores ? pr.kept_scores + out_off : nullptr);
      }
    }
  }
}

// Workgroups of the fused kernel that can be resident at once on the current device.
static int fused_capacity() {
  static int cached[64];
  static bool known[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  if (!known[dev]) {
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, sel_fused_kernel, kSelThreads, 0) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      return 0;
    cached[dev] = per_cu * cus;
    known[dev] = true;
  }
  return cached[dev];
}

// Selections of a batch: consecutive problems are packed into launches of the fused kernel as long
// as their workgroups fit into half of the device together (they all have to be resident: each
// problem meets at its own grid barriers; should another stream hold compute units for so long that
// a bounded wait gives up, the kernel marks the outputs and the status call reports it).  A single
// problem wider than that runs as step launches.
int32_t launch_select_batch(int n_heads, int n_problems, const lava_select_problem* problems, int64_t max_total,
                            void* ws, hipStream_t s, bool cleared) {
  const SelectWorkspace w = make_select_workspace(max_total);
  SelectBatch a;
  a.n_heads = n_heads;
  a.ws_stride = w.bytes;
  a.off_hist = w.off_hist;
  a.off_state = w.off_state;
  a.off_blk = w.off_blk;
  a.blk_stride = w.n_blocks;
  const dim3 block(kSelThreads);
  // Half of what the device can keep resident: the grid barriers need every workgroup of a launch
  // on the device at once, and the margin leaves room for whatever else is running there.
  const int cap = (fused_capacity() < kFusedMaxBlocks ? fused_capacity() : kFusedMaxBlocks) / 2;
  a.spin_limit = tuning().barrier_spin_limit > 0 ? (unsigned int)tuning().barrier_spin_limit : kSpinLimit;
  int first = 0;
  while (first < n_problems) {
    int count = 0, blocks = 0;
    while (first + count < n_problems && count < kMaxSelProblems) {
      const int64_t t = problems[first + count].total_entries;
      const int nb = (int)((t + kSelChunk - 1) / kSelChunk) < 1 ? 1 : (int)((t + kSelChunk - 1) / kSelChunk);
      if (count > 0 && blocks + nb > cap) break;
      a.first_block[count] = blocks;
      blocks += nb;
      a.p[count] = problems[first + count];
      ++count;
    }
    a.n_problems = count;
    a.first_block[count] = blocks;
    a.ws = static_cast<char*>(ws) + (size_t)first * w.bytes;
    a.primed_mask = 0u;
    for (int i = 0; i < count; ++i)
      if (a.p[i].primed) a.primed_mask |= 1u << i;
    const bool all_primed = a.primed_mask == (count == 32 ? 0xffffffffu : (1u << count) - 1u);
    const bool fused = blocks <= cap;
    if (!(fused && (all_primed || cleared))) {             // the one-launch selection clears a primed problem's counts itself
      ProfScope ps(KID_SEL_INIT, s);
      hipLaunchKernelGGL(sel_init_kernel, dim3(count), block, 0, s, a);
    }
    if (fused) {
      ProfScope ps(KID_SEL_FUSED, s);
      hipLaunchKernelGGL(sel_fused_kernel, dim3(blocks), block, 0, s, a);
    } else {                                               // a single problem wider than the device allows
      ProfScope ps(KID_SEL_STEPS, s);
      const dim3 grid(blocks);
      if (!all_primed) hipLaunchKernelGGL(sel_step_kernel<0>, grid, block, 0, s, a);
      hipLaunchKernelGGL(sel_step_kernel<1>, grid, block, 0, s, a);
      hipLaunchKernelGGL(sel_step_kernel<2>, grid, block, 0, s, a);
      hipLaunchKernelGGL(sel_step_kernel<3>, grid, block, 0, s, a);
      hipLaunchKernelGGL(sel_step_kernel<4>, grid, block, 0, s, a);
    }
    const int32_t st = launch_status();
    if (st != LAVA_OK) return st;
    first += count;
  }
  return LAVA_OK;
}

int32_t launch_select(int n_heads, const float* scores, const int64_t* seg_offsets, int64_t total,
                      int64_t budget, const int64_t* budget_dev, int32_t* head_counts,
                      int64_t* head_offsets, int32_t* kept_idx, float* kept_scores, void* ws,
                      hipStream_t s) {
  lava_select_problem pr;
  pr.scores = scores;
  pr.seg_offsets = seg_offsets;
  pr.total_entries = total;
  pr.budget = budget;
  pr.budget_dev = budget_dev;
  pr.head_counts = head_counts;
  pr.head_offsets = head_offsets;
  pr.kept_idx = kept_idx;
  pr.kept_scores = kept_scores;
  pr.in_offset_dev = nullptr;
  pr.out_offset_dev = nullptr;
  pr.error_dev = nullptr;
  pr.primed = 0;
  return launch_select_batch(n_heads, 1, &pr, total, ws, s);
}

// Error words of the first n_problems regions laid out for max_total: flag = OR of them.
int32_t select_error_flag(const void* ws, int64_t max_total, int n_problems, hipStream_t s, int* flag) {
  const SelectWorkspace w = make_select_workspace(max_total);
  *flag = 0;
  for (int p = 0; p < n_problems; ++p) {
    const SelectState* st = reinterpret_cast<const SelectState*>(static_cast<const char*>(ws) + (size_t)p * w.bytes +
                                                                 w.off_state);
    unsigned int host = 0u;
    if (hipMemcpyAsync(&host, &st->error, sizeof(host), hipMemcpyDeviceToHost, s) != hipSuccess) return LAVA_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return LAVA_ERR_HIP;
    *flag |= (int)host;
  }
  return LAVA_OK;
}

}  // namespace lava

// ------------------------------------------------------------------------------------------
// lava_select_topk for callers that cannot allocate (code under HIP graph capture, serving loops
// and harnesses that forbid hipMalloc): the selection's workspace is a fixed array in the
// library's own device image instead of a caller buffer.  Every GPU holds its own copy of the
// array at its own address; the address is looked up once per device and the kernels receive it
// as an ordinary pointer argument, exactly as they receive a caller's workspace.
// ------------------------------------------------------------------------------------------
namespace {
constexpr int64_t kStaticMaxEntries = LAVA_SELECT_STATIC_MAX_ENTRIES;
constexpr size_t kStaticScratchBytes = lava::select_layout(kStaticMaxEntries).bytes;
static_assert(kStaticScratchBytes <= ((size_t)2 << 20), "the built-in scratch array is meant to stay small");
}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];       // device address of `scratch` on each GPU, once known
bool g_scratch_known[kMaxDevices];

// Device address of this GPU's copy of the array (the array's name is a host-side handle, never a
// device address).
int32_t scratch_of_current_device(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LAVA_ERR_HIP;
  if (!g_scratch_known[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return LAVA_ERR_HIP;
    g_scratch_ptr[dev] = p;
    g_scratch_known[dev] = true;
  }
  *out = g_scratch_ptr[dev];
  return LAVA_OK;
}
}  // namespace

extern "C" int32_t lava_select_topk_static(int32_t n_heads, const float* scores, const int64_t* seg_offsets,
                                           int64_t total_entries, int64_t budget, const int64_t* budget_dev,
                                           int32_t* head_counts, int64_t* head_offsets, int32_t* kept_idx,
                                           float* kept_scores, void* hip_stream) {
  if (n_heads < 1) return LAVA_ERR_INVALID_ARG;
  if (n_heads > lava::kMaxHeads) return LAVA_ERR_SHAPE;
  const lava_select_problem p = {scores,      seg_offsets,  total_entries, budget,     budget_dev,
                                 head_counts, head_offsets, kept_idx,      kept_scores, nullptr, nullptr, nullptr, 0};
  const int32_t st = lava::check_select_problem(n_heads, p);
  if (st != LAVA_OK) return st;
  if (total_entries > kStaticMaxEntries) return LAVA_ERR_WORKSPACE;   // beyond what the built-in array holds
  void* ws = nullptr;
  const int32_t sw = scratch_of_current_device(&ws);
  if (sw != LAVA_OK) return sw;
  lava::discard_stale_error();
  // histograms, barrier counter and error word are cleared by the selection's own first kernel
  return lava::launch_select_batch(n_heads, 1, &p, total_entries, ws, static_cast<hipStream_t>(hip_stream));
}

