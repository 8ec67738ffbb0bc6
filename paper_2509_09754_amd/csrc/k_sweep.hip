// The three sweeps over a layer's cache (Def. 1 / Eq. 3 with the attention rows of Sec. 2):
//
//   vnorm   V once:  per-row L1 norms, per-workgroup maxima                 -> Vbar (Thm. 1)
//   stats   K once:  logits of the w window rows against every key on the matrix cores, online
//                    row max / row sum per workgroup                        -> softmax normaliser
//   scores  K again: the same logits, exp2 against the merged normaliser, mean over the window
//                    rows, max over the query heads of the KV group (Sec. 4.3)
//
// The window product is the one dense contraction of the path: per KV head a
// [G*w] x d_h x N GEMM.  Each wavefront owns 32-key tiles.  A tile travels HBM -> LDS with
// coalesced 128-bit direct-to-LDS loads (no staging registers) into a wavefront-private ring of
// XOR-swizzled buffers, several tiles ahead of the one being multiplied; it is then read in MFMA
// operand layout and multiplied against the group's query rows, which stay in registers for the
// whole sweep.  The ring is private to the wavefront, so the sweep needs no workgroup barrier:
// arrival of a tile is a vmcnt wait that leaves the younger tiles in flight.
//
// MFMA 32x32 layouts used below (wave64): operand lane l supplies row/column l%32 and k-slice
// l/32; result register v of lane l is element (8*(v/4) + 4*(l/32) + v%4, l%32).
//   stats  : D = K_tile * Q^T  -> a lane holds 16 keys of ONE query row: row reductions stay in-lane
//   scores : D = Q * K_tile^T  -> a lane holds 16 query rows of ONE key: the window mean stays in-lane
#include <math.h>

#include "budget_wave.h"
#include "common.h"
#include "tile_ring.h"
#include "xblock.h"

namespace lava {

// "last workgroup done" tickets in the workspace (zeroed by the first kernel of every call)
constexpr int kCounterPool = 0;                         // poolstat: one two-level ticket
// control words of the persistent sweep, behind the ticket (a sequence's counter region)
constexpr int kCtlError = kArriveWords;                 // a wait for other workgroups gave up (first sequence's region)
constexpr int kCtlDoneA = kArriveWords + 1;             // [64] statistics units completed, per KV head of the sequence
constexpr int kCtlUnitA = kCtlDoneA + 64;               // [H_kv * blocks_x] claim word of every statistics unit of the sequence

// Wavefronts per workgroup and ring depth.  Kernels whose registers fit twice into a SIMD come in two
// shapes.  Wide (W = 8): 8 wavefronts (2 per SIMD: one wavefront's exponentials overlap the
// other's MFMAs and waits), a 128 KiB ring, so a CU holds one workgroup: the shape for a launch
// whose workgroups all start together (one sequence).  Narrow (W = 4): 4 wavefronts and a 64 KiB
// ring, two workgroups per CU with the same registers, wavefronts and bytes in flight per CU: in a
// launch of several rounds of workgroups (a batch) the two run out of phase, and one's set-up and
// tail hide behind the other's streaming.  The f32 / d_h 128 kernels need more than 256 registers:
// 4 wavefronts and the whole ring in either case.
constexpr int kFusedTilesWide = 128;
constexpr int kFusedTilesNarrow = 96;
template <int DT, int D, int W>
struct Shape {
  static_assert(W == 4 || W == 8, "wavefronts per workgroup");
  static constexpr bool kBig = DT == LAVA_F32 && D == 128;
  static constexpr bool kNarrow = W == 4 && !kBig;
  static constexpr int kWaves = kBig ? 4 : W;
  static constexpr int kThreads = kWaves * 64;
  static constexpr int kMinWaves = kNarrow ? 2 : 1;      // per SIMD, for the register allocator
  static constexpr int kRingBytes = kNarrow ? 64 * 1024 : 128 * 1024;
  static constexpr int kStagesRaw = kRingBytes / (kWaves * Tile<DT, D>::kTileBytes);
  static constexpr int kStages = kStagesRaw > 4 ? 4 : kStagesRaw;
  static constexpr int kFusedTiles = kNarrow ? kFusedTilesNarrow : kFusedTilesWide;   // span of raw scores kept in LDS
  static_assert(kStages >= 2 && kStages <= kMaxRingStages, "ring depth");
};

// Layer statistic from per-lane partial sums S = sum s, T = sum s ln s (fp64): fixed-order reduction
// over lanes (xor tree), wavefronts and, by the last workgroup to arrive, workgroups; then
// e = (ln S - T / S) / n_entries  (Eq. 4-5 in closed form).  Contains workgroup barriers.  Returns true in
// every thread of that last workgroup, whose thread 0 has then also left the statistic (as stored,
// rounded to fp32) in s_t[0] for whatever the workgroup does next with it (not yet published by a barrier).
template <int THREADS>
__device__ __forceinline__ bool entropy_finish(double acc_s, double acc_t, double2* __restrict__ ent_part,
                                               uint32_t* __restrict__ counters, unsigned int n_blocks,
                                               unsigned int block_id, double n_entries,
                                               float* __restrict__ layer_stat, double* s_s, double* s_t,
                                               unsigned int* s_last, const uint32_t* error_word = nullptr) {
  constexpr int kW = THREADS / 64;
  for (int off = 32; off > 0; off >>= 1) {
    acc_s += __shfl_xor(acc_s, off);
    acc_t += __shfl_xor(acc_t, off);
  }
  if ((threadIdx.x & 63) == 0) { s_s[threadIdx.x >> 6] = acc_s; s_t[threadIdx.x >> 6] = acc_t; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double S = 0.0, Tt = 0.0;
    for (int i = 0; i < kW; ++i) { S += s_s[i]; Tt += s_t[i]; }
    double2* mine = &ent_part[block_id];
    st_dev_f64(&mine->x, S);
    st_dev_f64(&mine->y, Tt);
  }
  if (!arrive_last(&counters[kCounterPool], n_blocks, block_id, s_last)) return false;
  // last workgroup: thread t sums partials t, t + THREADS, ... then the same fixed tree as above
  double S = 0.0, Tt = 0.0;
  for (unsigned int i = threadIdx.x; i < n_blocks; i += THREADS) {
    S += ld_dev_f64(&ent_part[i].x);
    Tt += ld_dev_f64(&ent_part[i].y);
  }
  for (int off = 32; off > 0; off >>= 1) {
    S += __shfl_xor(S, off);
    Tt += __shfl_xor(Tt, off);
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { s_s[threadIdx.x >> 6] = S; s_t[threadIdx.x >> 6] = Tt; }
  __syncthreads();
  if (threadIdx.x != 0) return true;
  S = 0.0; Tt = 0.0;
  for (int i = 0; i < kW; ++i) { S += s_s[i]; Tt += s_t[i]; }
  double e = 0.0;
  if (S > 0.0) e = (log(S) - Tt / S) / n_entries;
  if (error_word != nullptr && ld_dev(error_word) != 0u) e = (double)NAN;   // scores of this call are not to be used
  layer_stat[0] = (float)e;
  s_t[0] = (double)(float)e;
  return true;
}

// What the budget rule reads, fetched by the lanes of wavefront 0 well before the statistic exists (any
// workgroup may turn out to be the one that forms it; the loads are few and hit in L2): layers lane and
// lane + 64 of sequence b's rows.
struct PlanInputs {
  long long lo[2], hi[2], total;
  float e[2];
};
static_assert(kMaxPlannedLayers <= 128, "two layers per lane");
__device__ __forceinline__ PlanInputs plan_prefetch(const BudgetPlanArgs& plan, int b) {
  PlanInputs in = {};
  if (plan.e == nullptr || threadIdx.x >= 64) return in;
  const long long row = (long long)b * plan.n_layers;
  in.total = (long long)plan.total[b];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int i = (int)threadIdx.x + 64 * j;
    if (i < plan.n_layers) {
      in.lo[j] = (long long)plan.lo[row + i];
      in.hi[j] = (long long)plan.hi[row + i];
      if (i != plan.layer) in.e[j] = plan.e[row + i];
    }
  }
  return in;
}

// Budgets of sequence b of the batch from the statistics of its layers (Alg. 2, inner loop), by
// wavefront 0 of the workgroup that has just formed the statistic e_new of layer plan.layer: the same
// routine, on the same values, as the budgets kernel.  `lds`: sizeof(BudgetScratchT<kMaxPlannedLayers>)
// bytes, 8-aligned, that no other wavefront of the workgroup touches meanwhile.  A NaN statistic (a
// failed launch) leaves all budgets of the sequence at -1.
__device__ __forceinline__ void plan_budgets(const BudgetPlanArgs& plan, const PlanInputs& in, int b, float e_new,
                                             void* lds) {
  if (threadIdx.x >= 64) return;
  using Scratch = BudgetScratchT<kMaxPlannedLayers>;
  Scratch* sc = static_cast<Scratch*>(lds);
  const int lane = (int)threadIdx.x, n = plan.n_layers;
  const long long row = (long long)b * n;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int i = lane + 64 * j;
    if (i < n) {
      sc->ed[i] = i == plan.layer ? (double)e_new : (double)in.e[j];
      sc->lo[i] = in.lo[j];
      sc->hi[i] = in.hi[j];
    }
  }
  if (lane == 0) plan.e[row + plan.layer] = e_new;
  WaveSync::sync();
  long long* out_b = reinterpret_cast<long long*>(plan.out) + row;
  int bad = e_new != e_new ? 1 : 0;
  if (n == 1) {
    // a single layer takes the whole total (its quota is total * e / e, exactly), if the bounds allow it:
    // what the rule below returns, without its reductions across the wavefront
    const long long lo0 = __shfl(in.lo[0], 0), hi0 = __shfl(in.hi[0], 0);
    if (lane == 0) out_b[0] = (!bad && lo0 >= 0 && lo0 <= in.total && in.total <= hi0) ? in.total : -1;
    return;
  }
  if (!bad)
    bad = allocate_budgets_wave<WaveSync>(lane, n, sc->ed, in.total, sc->lo, sc->hi, out_b, sc->quota, sc->base,
                                          sc->freel, sc->frac, sc->state);
  if (bad)
    for (int i = lane; i < n; i += 64) out_b[i] = -1;
}

// The statistics sweep of one wavefront: tiles first, first + WAVES, ... (cnt of them) of the head
// at kg, whose first STAGES - 1 tiles have already been requested into `ring`.  Returns, per head of
// the chunk, this lane's running maximum of the raw dot products of its query row (lane % 32) and
// the sum of exp2((dot - max) * c2) over the keys this lane saw (the two lane halves see different
// keys of the same rows).  The assignment of tiles to wavefronts is static: the sums depend on the
// order, and results must not depend on timing.  Tile `it` sits in ring slot (it + slot0) % STAGES
// (slot0 != 0 when another sweep of the same wavefront used the ring just before and requested these tiles).
template <int DT, int D, int GT, int WAVES, int STAGES>
__device__ __forceinline__ void stats_tiles(const TileDma<DT, D>& dma, const FragReader<DT, D>& frags,
                                            const char* __restrict__ kg, long long n, int w, int bph, float c2,
                                            long long first, int cnt, u32x4* ring,
                                            const u32x4 (&qf)[GT][Tile<DT, D>::kSteps], int lane,
                                            float (&m_run)[GT], float (&z_run)[GT], int slot0 = 0) {
  using T = Tile<DT, D>;
  static_assert((STAGES & (STAGES - 1)) == 0, "ring slots are taken modulo a power of two");
#pragma unroll
  for (int t = 0; t < GT; ++t) { m_run[t] = -INFINITY; z_run[t] = 0.0f; }
  const int r = lane & 31, half = lane >> 5;
  const unsigned int ring_addr = lds_addr(ring);
  for (int it = 0; it < cnt; ++it) {
    const long long tile = first + (long long)it * WAVES;
    const int ahead = it + STAGES - 1;
    if (ahead < cnt)
      dma.issue(kg, first + (long long)ahead * WAVES, n, lane, ring + ((ahead + slot0) % STAGES) * T::kTileChunks);
    const int younger = cnt - 1 - it < STAGES - 1 ? cnt - 1 - it : STAGES - 1;
    wait_tile<DT, D>(younger);
    u32x4 kf[T::kSteps];
    frags.read(ring_addr + ((it + slot0) % STAGES) * T::kTileBytes, kf);

    const long long key0 = tile * kTileKeys;
    if (key0 + kTileKeys - 1 <= n - w) {
      // every row sees every key of the tile: straight-line code, the next head's MFMAs are
      // independent of this head's exponentials
      f32x16 acc = dot_tile<DT, D, true>(kf, qf[0]);
#pragma unroll
      for (int t = 0; t < GT; ++t) {
        f32x16 nxt = acc;
        if (t + 1 < GT) nxt = dot_tile<DT, D, true>(kf, qf[t + 1]);
        float tmax = fmaxf(acc[0], acc[1]);
#pragma unroll
        for (int v = 2; v < 16; ++v) tmax = fmaxf(tmax, acc[v]);
        const float mn = fmaxf(m_run[t], tmax);
        const float mc = mn * c2;
        float zs = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) zs += fast_exp2(fmaf(acc[v], c2, -mc));
        z_run[t] = z_run[t] * fast_exp2((m_run[t] - mn) * c2) + zs;   // exp2(-inf) = 0 on the first tile
        m_run[t] = mn;
        acc = nxt;
      }
    } else {
      // tile touches the window or the end of the sequence: mask what a row may not see
      const int rel0 = (int)(key0 - (n - w));                // position of the tile's first key relative to N - w
#pragma unroll
      for (int t = 0; t < GT; ++t) {
        // window row of this lane in block t (a chunk starts at an even block when heads have two blocks);
        // row rr sees relative positions <= min(rr, w - 1)
        const int rr = r + ((bph == 2 && (t & 1)) ? 32 : 0);
        const int row_limit = rr < w - 1 ? rr : w - 1;
        f32x16 acc = dot_tile<DT, D, true>(kf, qf[t]);
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (rel0 + 8 * (v / 4) + 4 * half + (v % 4) > row_limit) acc[v] = -INFINITY;
        float tmax = acc[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, acc[v]);
        if (tmax > -INFINITY) {
          const float mn = fmaxf(m_run[t], tmax);
          const float mc = mn * c2;
          float zs = 0.0f;
#pragma unroll
          for (int v = 0; v < 16; ++v) zs += fast_exp2(fmaf(acc[v], c2, -mc));
          const float f = (m_run[t] == mn) ? 1.0f : fast_exp2((m_run[t] - mn) * c2);
          z_run[t] = z_run[t] * f + zs;
          m_run[t] = mn;
        }
      }
    }
  }
}

// Merge of the two lane halves (same row, different keys), then of the wavefronts in wavefront order.
// Thread (head * 32 + row) of the workgroup returns true and the merged (max, sum) of its row.
// Contains a workgroup barrier.
template <int GT, int WAVES>
__device__ __forceinline__ bool stats_merge_waves(float (&m_run)[GT], float (&z_run)[GT], float c2, int lane, int wave,
                                                  float2 (*s_red)[kMaxChunkHeads * 32], float2& out) {
  const int r = lane & 31, half = lane >> 5;
#pragma unroll
  for (int t = 0; t < GT; ++t) {
    const float m2 = __shfl_xor(m_run[t], 32);
    const float z2 = __shfl_xor(z_run[t], 32);
    merge_stat(m_run[t], z_run[t], m2, z2, c2);
    if (half == 0) s_red[wave][t * 32 + r] = make_float2(m_run[t], z_run[t]);
  }
  __syncthreads();
  if (threadIdx.x >= GT * 32) return false;
  float m = -INFINITY, z = 0.0f;
#pragma unroll
  for (int wv = 0; wv < WAVES; ++wv) {
    const float2 p = s_red[wv][threadIdx.x];
    merge_stat(m, z, p.x, p.y, c2);
  }
  out = make_float2(m, z);
  return true;
}

// sum of |x| over 16 bytes, added to s
template <int DT>
__device__ __forceinline__ float abs_sum16(const u32x4& x, float s) {
  const unsigned int u[4] = {x.x, x.y, x.z, x.w};
  if constexpr (DT == LAVA_BF16) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int i = 0; i < 4; ++i)   // clear both sign bits, then a.x * 1 + a.y * 1 + s in one instruction
      s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, u[i] & 0x7fff7fffu), ones, s, false);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) s += fabsf(__uint_as_float(u[i]));
  }
  return s;
}

// The selection region a primed call prepares for sequence z of the launch: histograms and state to zero
// (the score kernels of the same call then fill the first histogram).  Called by one workgroup.
__device__ __forceinline__ void clear_selection_region(const SweepArgs& a, int z, int threads) {
  if (a.sel_ws == nullptr) return;
  char* region = a.sel_ws + (size_t)(a.first_seq + z) * a.sel_stride;
  unsigned int* hist = reinterpret_cast<unsigned int*>(region + a.sel_off_hist);
  unsigned int* state = reinterpret_cast<unsigned int*>(region + a.sel_off_state);
  for (int i = threadIdx.x; i < 3 * kSelBins; i += threads) hist[i] = 0u;
  if (threadIdx.x < kSelStateWords) state[threadIdx.x] = 0u;
}

// The value-norm sweep of one wavefront: tiles first, first + WAVES, ... (cnt of them) of the head at
// vg, whose first STAGES - 1 tiles have already been requested into `ring`.  Returns this lane's maximum
// over its rows (row lane % 32 of every tile) of sum_c |V[row, c]|; with token_norm the rows' own norms
// also go to row_norm (indexed by position).  CHAIN: as the ring drains, the first STAGES - 1 tiles
// of the same numbers at `next` (the head's keys) are requested into the slots that follow, so that the
// statistics sweep continues without a gap: its tile `it` is in slot (cnt + it) % STAGES.
template <int DT, int D, int WAVES, int STAGES, bool CHAIN>
__device__ __forceinline__ float vnorm_tiles(const TileDma<DT, D>& dma, const FragReader<DT, D>& frags,
                                             const char* __restrict__ vg, const char* __restrict__ next, long long n,
                                             long long first, int cnt, u32x4* ring, int lane, bool token_norm,
                                             float* __restrict__ row_norm) {
  using T = Tile<DT, D>;
  static_assert((STAGES & (STAGES - 1)) == 0, "ring slots are taken modulo a power of two");
  const unsigned int ring_addr = lds_addr(ring);
  const int total = CHAIN ? 2 * cnt : cnt;                   // tiles this wavefront requests through the ring
  float best = 0.0f;
  for (int it = 0; it < cnt; ++it) {
    const int ahead = it + STAGES - 1;
    if (ahead < cnt)
      dma.issue(vg, first + (long long)ahead * WAVES, n, lane, ring + (ahead % STAGES) * T::kTileChunks);
    else if (CHAIN && ahead < total)
      dma.issue(next, first + (long long)(ahead - cnt) * WAVES, n, lane, ring + (ahead % STAGES) * T::kTileChunks);
    const int younger = total - 1 - it < STAGES - 1 ? total - 1 - it : STAGES - 1;
    wait_tile<DT, D>(younger);
    // each lane sums the half row it holds (row lane % 32; rows past n repeat row n - 1), the two
    // halves are added across lanes
    u32x4 f[T::kSteps];
    frags.read(ring_addr + (it % STAGES) * T::kTileBytes, f);
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < T::kSteps; ++j) s = abs_sum16<DT>(f[j], s);
    s += __shfl_xor(s, 32);
    best = fmaxf(best, s);
    if (token_norm) {                                          // uniform: the rows' own norms, for the pooling step
      const long long row = (first + (long long)it * WAVES) * kTileKeys + (lane & 31);
      if (lane < 32 && row < n) row_norm[row] = s;
    }
  }
  return best;
}

// ------------------------------------------------------------------------------------------
// stats: per workgroup and per (head of the chunk, window row) the running maximum of the raw
// dot products and sum of exp2((dot - max) * c2) over the workgroup's keys, c2 = scale * log2 e.
// Row r may see keys 0 .. n - w + r only (each window row is normalised over the keys up to
// and including its own position).
// ------------------------------------------------------------------------------------------
//
// VN: the workgroup of a head's first chunk first sweeps the same span of the head's VALUE rows for their
// L1 norms (what vnorm_kernel does in a launch of its own, cut here like the statistics: vnorm_blocks ==
// blocks_x), through the same ring, and runs on into the keys without draining it.  One launch instead of
// two: one start-up and one tail for both streams.  Workgroup (0, 0) also clears what vnorm_kernel clears.
template <int DT, int D, int GT, int W, bool VN>
__global__ void __launch_bounds__((Shape<DT, D, W>::kThreads), (Shape<DT, D, W>::kMinWaves))
stats_kernel(const SweepArgs a) {
  using T = Tile<DT, D>;
  const SweepSeq sq = a.s[blockIdx.z];
  if (blockIdx.x >= (unsigned int)sq.blocks_x) return;
  const long long n = sq.n;
  const int w = a.w, G = a.G, n_chunks = a.n_chunks, tiles_per_block = sq.tiles_per_block;
  const float c2 = a.c2;
  const u32x4* __restrict__ q_win =
      static_cast<const u32x4*>(a.q_win) + (long long)(a.first_seq + blockIdx.z) * a.H * w * T::kCpr;
  const u32x4* __restrict__ k = static_cast<const u32x4*>(a.k) + (long long)a.H_kv * sq.tok * T::kCpr;
  float2* __restrict__ stat_part = reinterpret_cast<float2*>(a.ws + sq.ws_off + a.off_stat_part);
  constexpr int kWaves = Shape<DT, D, W>::kWaves;
  constexpr int kStages = Shape<DT, D, W>::kStages;
  __shared__ u32x4 s_tile[kWaves][kStages][T::kTileChunks];
  __shared__ float2 s_red[kWaves][kMaxChunkHeads * 32];   // [wave][head*32+row]

  const int lane = threadIdx.x & 63, wave = wave_index();
  const int g = blockIdx.y / n_chunks, chunk = blockIdx.y % n_chunks;
  const int h0 = g * G + chunk * GT;
  const int nh = (G - chunk * GT) < GT ? (G - chunk * GT) : GT;
  const char* kg = reinterpret_cast<const char*>(k) + (long long)g * n * T::kRowBytes;

  TileDma<DT, D> dma;
  dma.init(lane);
  FragReader<DT, D> frags;
  frags.init(lane);

  const long long n_tiles = (n + kTileKeys - 1) / kTileKeys;
  const long long t_begin = (long long)blockIdx.x * tiles_per_block;
  long long t_end = t_begin + tiles_per_block;
  if (t_end > n_tiles) t_end = n_tiles;

  // this wavefront's tiles: t_begin + wave, + kWaves, ...; ring of kStages buffers, kStages-1 tiles ahead
  const long long first = t_begin + wave;
  const int cnt = first < t_end ? (int)((t_end - first + kWaves - 1) / kWaves) : 0;
  u32x4* ring = s_tile[wave][0];
  const bool with_v = VN && chunk == 0;                        // uniform
  const char* first_stream = kg;
  if constexpr (VN) {
    if (with_v) {
      const u32x4* __restrict__ v = static_cast<const u32x4*>(a.v) + (long long)a.H_kv * sq.tok * T::kCpr;
      first_stream = reinterpret_cast<const char*>(v) + (long long)g * n * T::kRowBytes;
    }
    if (blockIdx.x == 0 && blockIdx.y == 0) {
      uint32_t* __restrict__ counters = reinterpret_cast<uint32_t*>(a.ws + sq.ws_off + a.off_counter);
      const int n_counter_words = kCtlUnitA + a.H_kv * sq.blocks_x;
      for (int i = threadIdx.x; i < n_counter_words; i += Shape<DT, D, W>::kThreads) counters[i] = 0u;
      clear_selection_region(a, (int)blockIdx.z, Shape<DT, D, W>::kThreads);
    }
  }
  // with the value rows first, the ring holds both streams in turn: the wavefront's cnt value tiles, then
  // its cnt key tiles (a wavefront with few tiles already requests keys here)
#pragma unroll
  for (int p = 0; p < kStages - 1; ++p) {
    if (p < cnt) dma.issue(first_stream, first + (long long)p * kWaves, n, lane, ring + p * T::kTileChunks);
    else if (with_v && p < 2 * cnt) dma.issue(kg, first + (long long)(p - cnt) * kWaves, n, lane, ring + p * T::kTileChunks);
  }
  // Every wavefront fetches its own copy of the query rows, after its first tiles so that the two
  // latencies overlap.  (Staging them once per workgroup through LDS, as the scores kernel does, was
  // measured slower here: the wavefronts then leave the barrier in step and the sweep loses more
  // than the set-up gains.)  Both are in before the loop: otherwise the compiler, which cannot count
  // the ring's loads across iterations, waits for everything in flight before each tile's products.
  u32x4 qf[GT][T::kSteps];
  load_q<DT, D, GT>(q_win, h0, nh, w, a.bph, lane, qf);
  wait_vmcnt<0>();
  float v_best = 0.0f;
  int slot0 = 0;
  if constexpr (VN) {
    if (with_v) {
      v_best = vnorm_tiles<DT, D, kWaves, kStages, true>(dma, frags, first_stream, kg, n, first, cnt, ring, lane,
                                                         a.token_norm != 0,
                                                         a.scores + (long long)a.H_kv * sq.tok + (long long)g * n);
      slot0 = cnt % kStages;
    }
  }
  float m_run[GT], z_run[GT];
  stats_tiles<DT, D, GT, kWaves, kStages>(dma, frags, kg, n, w, a.bph, c2, first, cnt, ring, qf, lane, m_run, z_run,
                                          slot0);
  if constexpr (VN) {
    __shared__ float s_vmax[kWaves];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v_best = fmaxf(v_best, __shfl_xor(v_best, off));
    if (lane == 0) s_vmax[wave] = v_best;                      // read after the barrier of the merge below
    float2 mine;
    const bool owner = stats_merge_waves<GT, kWaves>(m_run, z_run, c2, lane, wave, s_red, mine);
    if (owner) stat_part[((long long)blockIdx.y * sq.blocks_x + blockIdx.x) * (GT * 32) + threadIdx.x] = mine;
    if (with_v && threadIdx.x == 0) {
      float m = s_vmax[0];
#pragma unroll
      for (int i = 1; i < kWaves; ++i) m = fmaxf(m, s_vmax[i]);
      float* __restrict__ vnorm_part = reinterpret_cast<float*>(a.ws + sq.ws_off + a.off_vnorm_part);
      vnorm_part[(long long)g * sq.vnorm_blocks + blockIdx.x] = m;
    }
  } else {
    float2 mine;
    if (stats_merge_waves<GT, kWaves>(m_run, z_run, c2, lane, wave, s_red, mine))
      stat_part[((long long)blockIdx.y * sq.blocks_x + blockIdx.x) * (GT * 32) + threadIdx.x] = mine;
  }
}

// ------------------------------------------------------------------------------------------
// scores: s_raw[g, i] = max over the heads h of group g of (1/w) sum_r softmax_r[h, i], i < n'.
// The normaliser of each (head, row) is merged from the stats partials by every workgroup, always
// in the same fixed order (deterministic) and with independent loads, or taken from a
// caller-supplied log-sum-exp.
// ------------------------------------------------------------------------------------------
//
// FUSED (all heads of the group in one workgroup, at most Shape::kFusedTiles tiles per workgroup): the
// workgroup keeps the raw scores of its key span in LDS, recomputes one tile on either side of
// the span (the pooling halo; 2 extra tiles per workgroup instead of a trip through HBM and
// another launch), and finishes the scores itself: max-pool, value factor, +inf for the window
// entries, and the layer statistic.  Otherwise the raw scores go to s_raw for poolstat_kernel.
constexpr int kPoolMaxHalf = 7;   // pooling kernels up to 15

struct PoolArgs {
  const float* vnorm_part;   // [H_kv][vnorm_blocks] value-norm partials
  int vnorm_blocks;
  int pool_half;
  int token_norm;            // scores[g][i] holds ||V[g, i]||_1 on entry: the value factor of entry i
  float* scores;             // [H_kv][n]
  float* vbar;               // [H_kv]
  float* layer_stat;         // [1]
  double2* ent_part;         // [workgroups]
  uint32_t* counters;
  const uint32_t* error_word; // persistent launch: non-zero once a wait for other workgroups gave up (statistic -> NaN); else null
  unsigned int* sel_hist0;    // first-digit histogram of the selection that will rank these scores, or null
  BudgetPlanArgs plan;        // budgets right after the statistic (e == nullptr: none)
  int plan_seq;               // the sequence's row in the plan's tables
};

// Histogram of the selection's first digit over the scores a workgroup has just written, for a selection
// workspace prepared alongside (lava_window_scores_primed): per-workgroup counts in `bins` (kSelBins words
// of LDS, zeroed and published by a barrier before the first call), then one device-scope add per
// non-empty bin.  Runs of equal digits (pooling makes plateaus) are counted once per run by the caller.
__device__ __forceinline__ void digit0_count(unsigned int* bins, float score, unsigned int& run_digit,
                                             unsigned int& run_len) {
  const unsigned int digit = score_key(score) >> kSelDigit0Shift;
  if (digit != run_digit) {
    if (run_len != 0u) atomicAdd(&bins[run_digit], run_len);
    run_digit = digit;
    run_len = 0u;
  }
  ++run_len;
}
template <int THREADS>
__device__ __forceinline__ void digit0_flush(unsigned int* bins, unsigned int run_digit, unsigned int run_len,
                                             unsigned int* __restrict__ global_hist) {
  if (run_len != 0u) atomicAdd(&bins[run_digit], run_len);
  __syncthreads();
  for (int i = threadIdx.x; i < kSelBins; i += THREADS) {
    const unsigned int c = bins[i];
    if (c) __hip_atomic_fetch_add(&global_hist[i], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// Exponent bias of every (head, row) of a scores workgroup, step 1: thread (row, slice) merges its slice
// of the head's statistics partials in workgroup order into s_merge[slice][row] (always the same fixed
// order, independent loads: deterministic, no tickets).  DEVICE_SCOPE: the partials were written by
// other workgroups of the SAME launch (device-scope stores), so they are read with device-scope loads.
// `part` points at partial 0 of the head's (chunk's) rows.  The caller synchronises afterwards.
template <int GT, int THREADS, bool DEVICE_SCOPE>
__device__ __forceinline__ void merge_partials(const float2* __restrict__ part, int stat_blocks, bool have_lse,
                                               float c2, float2* s_merge) {
  constexpr int kRows = GT * 32;
  constexpr int kSlices = THREADS / kRows;
  const int row = threadIdx.x % kRows, slice = threadIdx.x / kRows;
  float m = -INFINITY, z = 0.0f;
  if (!have_lse) {
    const int per = (stat_blocks + kSlices - 1) / kSlices;
    const int b_begin = slice * per, b_end = (b_begin + per < stat_blocks) ? b_begin + per : stat_blocks;
    const float2* p = part + row;
    for (int b0 = b_begin; b0 < b_end; b0 += 16) {
      float2 x[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        if (b0 + u < b_end)
          x[u] = DEVICE_SCOPE ? ld_dev_f2(&p[(long long)(b0 + u) * kRows]) : p[(long long)(b0 + u) * kRows];
        else
          x[u] = make_float2(-INFINITY, 0.0f);
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) merge_stat(m, z, x[u].x, x[u].y, c2);
    }
  }
  s_merge[slice * kRows + row] = make_float2(m, z);
}

// Step 2: the slices are merged in slice order; bias = log2(row normaliser * w) in the exp2 domain,
// +inf for padding rows (their exponentials vanish).
template <int GT, int THREADS>
__device__ __forceinline__ void write_bias(const float2* s_merge, const float* __restrict__ lse, int h0, int nh, int w,
                                           int bph, float c2, float* s_bias) {
  constexpr int kRows = GT * 32;
  constexpr int kSlices = THREADS / kRows;
  if (threadIdx.x < kRows) {
    const int t = threadIdx.x >> 5;
    const int head = (h0 + t) / bph, rr = ((h0 + t) % bph) * 32 + (int)(threadIdx.x & 31);   // head and window row of this block row
    float bias = INFINITY;
    if (t < nh && rr < w) {
      if (lse != nullptr) {
        bias = lse[(long long)head * w + rr] * kLog2e;
      } else {
        float m = -INFINITY, z = 0.0f;
#pragma unroll
        for (int sl = 0; sl < kSlices; ++sl) {
          const float2 x = s_merge[sl * kRows + threadIdx.x];
          merge_stat(m, z, x.x, x.y, c2);
        }
        bias = m * c2 + log2f(z);
      }
      bias += log2f((float)w);
    }
    s_bias[threadIdx.x] = bias;
  }
}

// The score sweep of one wavefront over the jobs of its workgroup: the workgroup's own tiles
// t_begin .. t_end - 1, then (FUSED) the pooling halo, i.e. the tile before and the tile after the
// span.  fifo[] holds the jobs this wavefront has already requested into its ring (the first
// STAGES - 1 are fixed); the rest are taken from the shared counter *next_job as wavefronts become
// free, because the wavefronts of a workgroup do not run at the same speed.  Which wavefront
// computes a tile does not change its result, so the scores stay deterministic.
// FUSED: raw scores go to s_span (position p of the prefix at s_span[p - (t_begin - 1) * 32]);
// otherwise to raw_head[position] (atomic maximum when the group is split over workgroups).
template <int DT, int D, int GT, int WAVES, int STAGES, bool FUSED>
__device__ __forceinline__ void scores_tiles(const TileDma<DT, D>& dma, const FragReader<DT, D>& frags,
                                             const char* __restrict__ kg, long long n, long long n_prefix, float c2,
                                             long long t_begin, long long t_end, int n_own, bool halo_left,
                                             bool halo_right, int n_jobs, int (&fifo)[STAGES], u32x4* ring,
                                             unsigned int* next_job, const float* s_bias, float* s_span,
                                             const u32x4 (&qf)[GT][Tile<DT, D>::kSteps], int lane,
                                             float* __restrict__ raw_head, int n_chunks, int bph) {
  using T = Tile<DT, D>;
  auto job_tile = [&](int j) -> long long {
    if (j < n_own) return t_begin + j;
    return (j == n_own && halo_left) ? t_begin - 1 : t_end;
  };
  (void)halo_right;
  const int half = lane >> 5;
  const unsigned int ring_addr = lds_addr(ring);
  const unsigned int next_job_addr = lds_addr(next_job);
  // rows held by this lane in result register v: 8 * (v / 4) + 4 * half + v % 4 -> four float4 per head
  const unsigned int bias_addr = lds_addr(s_bias) + half * 16;
  const unsigned int span_base = lds_addr(s_span);

  // The result of a tile is stored one iteration later, right after the next tile's arrival wait:
  // the store then has a whole iteration to complete before a wait counts it among the older
  // operations, instead of stalling every iteration on its acknowledgement.
  float pend = 0.0f;
  int pend_key = -1;                 // n < 2^31
  auto store_result = [&](int key, float value) {
    if (half == 0 && key >= 0 && key < n_prefix) {
      float* dst = raw_head + key;
      if (n_chunks == 1) {
        *dst = value;
      } else {   // heads of the group are split over workgroups: non-negative floats order as integers
        atomicMax(reinterpret_cast<unsigned int*>(dst), __float_as_uint(value));
      }
    }
  };
  bool more = true;                                             // the counter has not run out yet
  for (int it = 0; fifo[0] >= 0; ++it) {
    const long long tile = job_tile(fifo[0]);
    if (more) {
      unsigned int j = 0;
      if (lane == 0) j = lds_fetch_inc(next_job_addr);
      j = __builtin_amdgcn_readfirstlane(j);
      more = j < (unsigned int)n_jobs;
      if (more) {
        fifo[STAGES - 1] = (int)j;
        dma.issue(kg, job_tile((int)j), n, lane, ring + ((it + STAGES - 1) % STAGES) * T::kTileChunks);
      }
    }
    int younger = 0;
#pragma unroll
    for (int p = 1; p < STAGES; ++p) younger += fifo[p] >= 0 ? 1 : 0;
    wait_tile<DT, D>(younger);
#pragma unroll
    for (int p = 0; p + 1 < STAGES; ++p) fifo[p] = fifo[p + 1];
    fifo[STAGES - 1] = -1;
    if constexpr (!FUSED) store_result(pend_key, pend);
    u32x4 kf[T::kSteps];
    frags.read(ring_addr + (it % STAGES) * T::kTileBytes, kf);

    float best = 0.0f, pair = 0.0f;
    f32x16 acc = dot_tile<DT, D, false>(kf, qf[0]);
#pragma unroll
    for (int t = 0; t < GT; ++t) {
      f32x16 nxt = acc;
      if (t + 1 < GT) nxt = dot_tile<DT, D, false>(kf, qf[t + 1]);
      float ps = 0.0f;
      u32x4 bb[4];                       // biases of rows 8*jj + 4*half + 0..3 of head t
      lds_read128x4_strided<32>(bias_addr + t * 128, bb[0], bb[1], bb[2], bb[3]);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        ps += fast_exp2(fmaf(acc[4 * jj + 0], c2, -__uint_as_float(bb[jj].x)));
        ps += fast_exp2(fmaf(acc[4 * jj + 1], c2, -__uint_as_float(bb[jj].y)));
        ps += fast_exp2(fmaf(acc[4 * jj + 2], c2, -__uint_as_float(bb[jj].z)));
        ps += fast_exp2(fmaf(acc[4 * jj + 3], c2, -__uint_as_float(bb[jj].w)));
      }
      ps += __shfl_xor(ps, 32);
      if (bph == 2) {                    // uniform: a head's window mean is the sum over its two row blocks
        if (t & 1) best = fmaxf(best, pair + ps);
        else pair = ps;
      } else {
        best = fmaxf(best, ps);
      }
      acc = nxt;
    }
    if constexpr (FUSED) {
      // the lane's slot in the span is formed here from the lane counter instead of living in a register
      // across the loop, which has none to spare
      unsigned int l;
      asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
      if (l < 32u) lds_write32(span_base + (unsigned int)(tile - t_begin + 1) * (kTileKeys * 4) + l * 4u, best);
    } else {
      pend = best;
      pend_key = (int)(tile * kTileKeys) + (lane & 31);
    }
  }
  if constexpr (!FUSED) store_result(pend_key, pend);
}

// Finishes the scores of a workgroup's span from the raw scores in s_span (FUSED): Vbar of the head
// (vb: this thread's share of the head's value-norm partials), max-pool over the prefix, the value
// factor, +inf for the window entries, and the workgroup's share of the layer statistic; the last
// workgroup of the sequence to arrive (block_id of n_blocks) forms e.  Contains workgroup barriers.
template <int THREADS>
__device__ __forceinline__ void scores_finish(const PoolArgs& pa, float vb, int g, long long n, long long n_prefix, int w,
                                              long long t_begin, long long t_end, long long n_tiles,
                                              const float* s_span, float* s_vb, double* s_s, double* s_t,
                                              unsigned int* s_last, unsigned int n_blocks, unsigned int block_id,
                                              int n_heads, bool writes_vbar, int wave, unsigned int* bins) {
  constexpr int kWaves = THREADS / 64;
  // `bins`: kSelBins words of LDS that only wavefront 0 has used since the workgroup's last barrier (the
  // start of its own tile ring, which it is done with)
  const bool count_digits = pa.sel_hist0 != nullptr;
  const PlanInputs plan_in = plan_prefetch(pa.plan, pa.plan_seq);
  if (count_digits && wave == 0)
    for (int i = threadIdx.x; i < kSelBins; i += 64) bins[i] = 0u;
  unsigned int run_digit = 0u, run_len = 0u;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) vb = fmaxf(vb, __shfl_xor(vb, off));
  if ((threadIdx.x & 63) == 0) s_vb[wave] = vb;
  lds_reads_done();                      // this wavefront's span entries are written
  __syncthreads();                       // s_span complete, s_vb visible
  vb = s_vb[0];
#pragma unroll
  for (int i = 1; i < kWaves; ++i) vb = fmaxf(vb, s_vb[i]);
  if (writes_vbar && threadIdx.x == 0) pa.vbar[g] = vb;

  const long long p_begin = t_begin * kTileKeys;
  long long p_end = t_end * kTileKeys;
  if (p_end > n_prefix) p_end = n_prefix;
  const long long span0 = (t_begin - 1) * kTileKeys;      // position held by s_span[0]
  // Eight consecutive positions per thread: 24 raw scores (positions base-8 .. base+15, six
  // 128-bit reads) cover every tap of a pooling window of up to 15; positions outside the prefix
  // do not take part in the maximum (the window is clipped, not padded).
  double acc_s = 0.0, acc_t = 0.0;
  constexpr int kPer = 8;
  static_assert(kPoolMaxHalf <= kPer - 1, "taps must stay inside the 24 values read");
  const float* out_head = pa.scores + (long long)g * n;
  for (long long base = p_begin + (long long)threadIdx.x * kPer; base < p_end; base += (long long)THREADS * kPer) {
    float raw[3 * kPer];
    const float4* src = reinterpret_cast<const float4*>(&s_span[(int)(base - kPer - span0)]);
#pragma unroll
    for (int i = 0; i < 3 * kPer / 4; ++i) {
      const float4 x = src[i];
      raw[4 * i + 0] = x.x; raw[4 * i + 1] = x.y; raw[4 * i + 2] = x.z; raw[4 * i + 3] = x.w;
    }
#pragma unroll
    for (int i = 0; i < 3 * kPer; ++i) {
      const long long pos = base - kPer + i;
      if (pos < 0 || pos >= n_prefix) raw[i] = -INFINITY;
    }
    float sc[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) sc[j] = raw[kPer + j];
#pragma unroll
    for (int dd = 1; dd <= kPoolMaxHalf; ++dd) {
      if (dd <= pa.pool_half) {                              // uniform
#pragma unroll
        for (int j = 0; j < kPer; ++j) sc[j] = fmaxf(sc[j], fmaxf(raw[kPer + j - dd], raw[kPer + j + dd]));
      }
    }
    float fac[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) fac[j] = vb;
    if (pa.token_norm) {                                     // uniform
#pragma unroll
      for (int j = 0; j < kPer; ++j)
        if (base + j < p_end) fac[j] = out_head[base + j];
    }
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      sc[j] *= fac[j];
      if (base + j < p_end) {
        acc_s += (double)sc[j];
        if (sc[j] > 0.0f) acc_t += (double)sc[j] * (double)logf(sc[j]);
        if (count_digits) digit0_count(bins, sc[j], run_digit, run_len);
      }
    }
    if (base + kPer <= p_end && (reinterpret_cast<uintptr_t>(out_head + base) & 15) == 0) {
      float4* dst = reinterpret_cast<float4*>(const_cast<float*>(out_head) + base);
      dst[0] = make_float4(sc[0], sc[1], sc[2], sc[3]);
      dst[1] = make_float4(sc[4], sc[5], sc[6], sc[7]);
    } else {
#pragma unroll
      for (int j = 0; j < kPer; ++j)
        if (base + j < p_end) pa.scores[(long long)g * n + base + j] = sc[j];
    }
  }
  // the workgroup that owns the head's last prefix tile also writes the window entries
  if (t_begin < t_end && t_end == n_tiles && threadIdx.x < (unsigned)w) {
    pa.scores[(long long)g * n + n_prefix + threadIdx.x] = INFINITY;
    if (count_digits) digit0_count(bins, INFINITY, run_digit, run_len);
  }
  if (count_digits) digit0_flush<THREADS>(bins, run_digit, run_len, pa.sel_hist0);
  const bool last = entropy_finish<THREADS>(acc_s, acc_t, pa.ent_part, pa.counters, n_blocks, block_id,
                                            (double)n_heads * (double)n_prefix, pa.layer_stat, s_s, s_t, s_last,
                                            pa.error_word);
  if (last && pa.plan.e != nullptr) {                        // uniform
    __syncthreads();                                         // s_t[0]; every wavefront is done with `bins`
    // scratch: what is left of wavefront 0's own tile ring behind the bins
    static_assert(kSelBins * 4 + sizeof(BudgetScratchT<kMaxPlannedLayers>) <= 16 * 1024, "wavefront 0's ring");
    plan_budgets(pa.plan, plan_in, pa.plan_seq, (float)s_t[0], bins + kSelBins);
  }
}

template <int DT, int D, int GT, bool FUSED, int W>
__global__ void __launch_bounds__((Shape<DT, D, W>::kThreads), (Shape<DT, D, W>::kMinWaves))
scores_kernel(const SweepArgs a) {
  using T = Tile<DT, D>;
  const SweepSeq sq = a.s[blockIdx.z];
  if (blockIdx.x >= (unsigned int)sq.blocks_x) return;
  const int seq = a.first_seq + (int)blockIdx.z;
  const long long n = sq.n;
  const int w = a.w, G = a.G, n_chunks = a.n_chunks, tiles_per_block = sq.tiles_per_block;
  const int stat_blocks = sq.blocks_x;
  const float c2 = a.c2;
  const u32x4* __restrict__ q_win = static_cast<const u32x4*>(a.q_win) + (long long)seq * a.H * w * T::kCpr;
  const u32x4* __restrict__ k = static_cast<const u32x4*>(a.k) + (long long)a.H_kv * sq.tok * T::kCpr;
  char* region = a.ws + sq.ws_off;
  const float2* __restrict__ stat_part = reinterpret_cast<const float2*>(region + a.off_stat_part);
  const float* __restrict__ lse = a.lse ? a.lse + (long long)seq * a.H * w : nullptr;
  float* __restrict__ s_raw = reinterpret_cast<float*>(region + a.off_sraw);
  PoolArgs pa;
  pa.vnorm_part = reinterpret_cast<const float*>(region + a.off_vnorm_part);
  pa.vnorm_blocks = sq.vnorm_blocks;
  pa.pool_half = a.pool_half;
  pa.scores = a.scores + (long long)a.H_kv * sq.tok;
  pa.vbar = a.vbar + (long long)seq * a.H_kv;
  pa.token_norm = a.token_norm;
  pa.layer_stat = a.layer_stat + seq;
  pa.ent_part = reinterpret_cast<double2*>(region + a.off_ent_part);
  pa.counters = reinterpret_cast<uint32_t*>(region + a.off_counter);
  pa.error_word = nullptr;
  pa.sel_hist0 = a.sel_ws ? reinterpret_cast<unsigned int*>(a.sel_ws + (size_t)seq * a.sel_stride + a.sel_off_hist) : nullptr;
  pa.plan = a.plan;
  pa.plan_seq = seq;
  constexpr int kWaves = Shape<DT, D, W>::kWaves;
  constexpr int kStages = Shape<DT, D, W>::kStages;
  __shared__ u32x4 s_tile[kWaves][kStages][T::kTileChunks];
  __shared__ __attribute__((aligned(16))) float s_bias[GT * 32];
  __shared__ __attribute__((aligned(16))) float s_span[FUSED ? (Shape<DT, D, W>::kFusedTiles + 2) * kTileKeys : 4];   // raw scores of the span + halo tiles

  const int lane = threadIdx.x & 63, wave = wave_index();
  const int g = blockIdx.y / n_chunks, chunk = blockIdx.y % n_chunks;
  const int h0 = g * G + chunk * GT;
  const int nh = (G - chunk * GT) < GT ? (G - chunk * GT) : GT;
  const char* kg = reinterpret_cast<const char*>(k) + (long long)g * n * T::kRowBytes;
  const long long n_prefix = n - w;

  float vb = 0.0f;   // this thread's share of the head's value-norm partials (reduced after the sweep)
  if constexpr (FUSED) {
    for (int i = threadIdx.x; i < pa.vnorm_blocks; i += Shape<DT, D, W>::kThreads)
      vb = fmaxf(vb, pa.vnorm_part[(long long)g * pa.vnorm_blocks + i]);
  }

  constexpr int kThreads = Shape<DT, D, W>::kThreads;
  constexpr int kRows = GT * 32;
  __shared__ float2 s_merge[kThreads];

  // start the ring first: these loads only need the key pointer
  TileDma<DT, D> dma;
  dma.init(lane);
  FragReader<DT, D> frags;
  frags.init(lane);
  const long long n_tiles = (n_prefix + kTileKeys - 1) / kTileKeys;
  const long long t_begin = (long long)blockIdx.x * tiles_per_block;
  long long t_end = t_begin + tiles_per_block;
  if (t_end > n_tiles) t_end = n_tiles;
  // Jobs of the workgroup: its own tiles, then (FUSED) the pooling halo, i.e. the tile before and the
  // tile after the span.  The first kStages - 1 jobs of every wavefront are fixed; the rest are taken
  // from a shared counter as wavefronts become free, because the wavefronts of a workgroup do not
  // run at the same speed (two share each SIMD and the older one wins the arbitration).  Which
  // wavefront computes a tile does not change its result, so the scores stay deterministic.
  const int n_own = t_begin < t_end ? (int)(t_end - t_begin) : 0;
  const bool halo_left = FUSED && n_own > 0 && t_begin > 0;
  const bool halo_right = FUSED && n_own > 0 && t_end < n_tiles;
  const int n_jobs = n_own + (halo_left ? 1 : 0) + (halo_right ? 1 : 0);
  auto job_tile = [&](int j) -> long long {
    if (j < n_own) return t_begin + j;
    return (j == n_own && halo_left) ? t_begin - 1 : t_end;
  };
  __shared__ unsigned int s_next_job;
  if (threadIdx.x == 0) s_next_job = kWaves * (kStages - 1);   // published by the barriers below
  int fifo[kStages];                                            // jobs requested and not yet computed; -1: none
#pragma unroll
  for (int p = 0; p < kStages; ++p) {
    const int j = wave + p * kWaves;
    fifo[p] = (p < kStages - 1 && j < n_jobs) ? j : -1;
  }
  u32x4* ring = s_tile[wave][0];
#pragma unroll
  for (int p = 0; p < kStages - 1; ++p)
    if (fifo[p] >= 0) dma.issue(kg, job_tile(fifo[p]), n, lane, ring + p * T::kTileChunks);

  // the query rows go through the last stage of the first GT wavefronts' rings (idle until the loop
  // starts); their loads are in flight together with the normaliser partials below
  static_assert(kWaves >= GT, "one staging buffer per head");
  stage_q<DT, D, GT, kThreads>(q_win, h0, nh, w, a.bph, [&](int t) { return &s_tile[t][kStages - 1][0]; });

  // exponent bias of every (head, row), from the statistics partials or the caller's log-sum-exp
  merge_partials<GT, kThreads, false>(stat_part + (long long)blockIdx.y * stat_blocks * kRows, stat_blocks,
                                      lse != nullptr, c2, s_merge);
  __syncthreads();
  write_bias<GT, kThreads>(s_merge, lse, h0, nh, w, a.bph, c2, s_bias);
  u32x4 qf[GT][T::kSteps];
#pragma unroll
  for (int t = 0; t < GT; ++t) frags.read(lds_addr(&s_tile[t][kStages - 1][0]), qf[t]);
  __syncthreads();

  scores_tiles<DT, D, GT, kWaves, kStages, FUSED>(dma, frags, kg, n, n_prefix, c2, t_begin, t_end, n_own, halo_left,
                                                  halo_right, n_jobs, fifo, ring, &s_next_job, s_bias, s_span,
                                                  qf, lane, s_raw + (long long)g * n_prefix, n_chunks, a.bph);
  if constexpr (FUSED) {
    __shared__ float s_vb[kWaves];
    __shared__ double s_s[kWaves], s_t[kWaves];
    __shared__ unsigned int s_last;
    scores_finish<kThreads>(pa, vb, g, n, n_prefix, w, t_begin, t_end, n_tiles, s_span, s_vb, s_s, s_t, &s_last,
                            sq.blocks_x * gridDim.y, blockIdx.y * sq.blocks_x + blockIdx.x, (int)gridDim.y,
                            blockIdx.x == 0, wave, reinterpret_cast<unsigned int*>(&s_tile[0][0][0]));
  }
}

// ------------------------------------------------------------------------------------------
// sweep: statistics and scores of a launch's sequences in ONE persistent launch.
//
// Work units are (sequence, KV head, span of keys): the same spans the two separate kernels give
// their workgroups.  Workgroup b of a grid of `grid` workgroups owns units b, b + grid, ... : it
// first runs their statistics passes, then their score passes.  A score unit needs the statistics
// of all spans of its head: it waits for the head's completion count.  So that this wait cannot
// depend on the whole grid being resident, every statistics unit carries a claim word: its owner
// claims it (a compare-and-swap on a word nobody else touches, in flight while the unit's first
// tiles are requested), and a workgroup whose wait lasts long looks for unclaimed statistics units
// of the head it waits for and runs them itself (it already holds that head's query rows).  A
// claimed unit is being run by a resident workgroup that waits for nothing, so every wait ends.
// (The waits are bounded all the same; one that gives up sets an error word and the layer
// statistic becomes NaN.)
// What the single launch saves over two: the query rows are fetched once, the second pass of a
// head starts as soon as that head's statistics are complete instead of after the slowest
// workgroup of the whole device, its first tiles are requested before the statistics are even
// published, and there is no second launch.  Results are bit-identical to the separate kernels:
// the same tiles are combined in the same order.
// ------------------------------------------------------------------------------------------
template <int DT, int D, int GT, int W>
struct SweepSmem {
  using T = Tile<DT, D>;
  using S = Shape<DT, D, W>;
  u32x4 tile[S::kWaves][S::kStages][T::kTileChunks];
  __attribute__((aligned(16))) float bias[GT * 32];
  union {
    float2 red[S::kWaves][kMaxChunkHeads * 32];            // statistics units: per-wavefront results
    struct {
      float2 merge[S::kThreads];                           // score units: slices of the partial merge
      __attribute__((aligned(16))) float span[(S::kFusedTiles + 2) * kTileKeys];   // raw scores of the span + halo
    } sc;
  };
  float vb[S::kWaves];
  double ss[S::kWaves], st[S::kWaves];
  unsigned int last, next_job;
  int claim[4];                                             // words handed from thread 0 to the workgroup
};

__device__ __forceinline__ void lds_write128(unsigned int a, const u32x4& x) {
  asm volatile("ds_write_b128 %0, %1" : : "v"(a), "v"(x) : "memory");
}

template <int DT, int D, int GT, int W>
__global__ void __launch_bounds__((Shape<DT, D, W>::kThreads), (Shape<DT, D, W>::kMinWaves))
sweep_kernel(const SweepArgs a) {
  using T = Tile<DT, D>;
  using S = Shape<DT, D, W>;
  constexpr int kWaves = S::kWaves, kStages = S::kStages, kThreads = S::kThreads, kRows = GT * 32;
  static_assert(kWaves >= GT, "one staging buffer per head");
  __shared__ SweepSmem<DT, D, GT, W> sm;
  const int lane = threadIdx.x & 63, wave = wave_index();
  const int w = a.w, G = a.G, H_kv = a.H_kv;
  const float c2 = a.c2;
  uint32_t* __restrict__ ctl0 = reinterpret_cast<uint32_t*>(a.ws + a.s[0].ws_off + a.off_counter);
  TileDma<DT, D> dma;
  dma.init(lane);
  FragReader<DT, D> frags;
  frags.init(lane);
  u32x4* ring = sm.tile[wave][0];

  // Query rows of (sequence si, head g), once per workgroup and unit.  The w rows of a head are one
  // contiguous run of q_win, i.e. a key tile of w rows: wavefront t requests head t's rows straight into
  // its idle last ring stage with the same direct-to-LDS loads (rows beyond the window repeat row w - 1,
  // heads beyond the group repeat its last head: their results are never used), AHEAD of the unit's first
  // key tiles, so that q_commit only waits for the older loads and the tiles stay in flight.
  // (Keeping the rows in registers from one unit to the next costs more registers than the two
  // passes leave.)  The workgroup is past a barrier since it last used those stages.
  auto q_request = [&](int si, int g) {
    if (wave < GT) {
      const int nh = G < GT ? G : GT;
      const int h = g * G + (wave < nh ? wave : nh - 1);
      const char* rows = static_cast<const char*>(a.q_win) +
                         ((long long)(a.first_seq + si) * a.H + h) * w * (long long)T::kRowBytes;
      dma.issue_clamped(rows, 0, w, lane, ring + (kStages - 1) * T::kTileChunks);
    }
  };
  // `younger`: key tiles this wavefront has requested since q_request
  auto q_commit = [&](u32x4 (&qf)[GT][T::kSteps], int younger) {
    if (wave < GT) wait_tile<DT, D>(younger);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < GT; ++t) frags.read(lds_addr(&sm.tile[t][kStages - 1][0]), qf[t]);
    __syncthreads();
  };
  auto seq_of_unit = [&](int u) {
    int si = 0;
    while (si + 1 < a.n_seq && u >= a.s[si + 1].unit_base) ++si;
    return si;
  };

  // The workgroup's own units: u_a walks its statistics units, then u_b its score units.  A score unit
  // whose wait for its head's statistics lasts may hand a statistics unit of that head to the top of
  // the loop (help_bx >= 0) and is set up again afterwards; there is one copy of each pass's code.
  int u_a = (int)blockIdx.x, u_b = (int)blockIdx.x;
  int help_si = 0, help_g = 0, help_bx = -1;
  for (;;) {
    // ------------------------------------------------------------ a statistics unit, if there is one to run
    int si = 0, g = 0, bx = -1;
    if (help_bx >= 0) {
      si = help_si; g = help_g; bx = help_bx;
      help_bx = -1;
    } else if (u_a < a.n_units) {
      const int u = u_a;
      u_a += (int)gridDim.x;
      // testing aid: every orphan_mod-th unit is left alone by its owner, as if the owner were not resident;
      // somebody waiting for the unit's head has to run it (the helping path below)
      if (a.orphan_mod != 0 && (u % a.orphan_mod) == 0) continue;
      si = seq_of_unit(u);
      const int rel = u - a.s[si].unit_base;
      g = rel / a.s[si].blocks_x;
      bx = rel % a.s[si].blocks_x;
    }
    if (bx >= 0) {
      const SweepSeq sq = a.s[si];
      const long long n = sq.n;
      const char* kg = static_cast<const char*>(a.k) + ((long long)H_kv * sq.tok + (long long)g * n) * T::kRowBytes;
      char* region = a.ws + sq.ws_off;
      float2* __restrict__ stat_part = reinterpret_cast<float2*>(region + a.off_stat_part);
      uint32_t* __restrict__ ctl = reinterpret_cast<uint32_t*>(region + a.off_counter);
      const long long n_tiles = (n + kTileKeys - 1) / kTileKeys;
      const long long t_begin = (long long)bx * sq.tiles_per_block;
      long long t_end = t_begin + sq.tiles_per_block;
      if (t_end > n_tiles) t_end = n_tiles;
      const long long first = t_begin + wave;
      const int cnt = first < t_end ? (int)((t_end - first + kWaves - 1) / kWaves) : 0;
      // Exactly the statistics kernel's pass: every wavefront fetches its own copy of the query rows after
      // its first tiles and enters the loop when both are in, without a workgroup barrier in front of
      // the loop (one there costs the pass a fifth of its speed, measured).
#pragma unroll
      for (int p = 0; p < kStages - 1; ++p)
        if (p < cnt) dma.issue(kg, first + (long long)p * kWaves, n, lane, ring + p * T::kTileChunks);
      u32x4 qf[GT][T::kSteps];
      load_q<DT, D, GT>(static_cast<const u32x4*>(a.q_win) + (long long)(a.first_seq + si) * a.H * w * T::kCpr, g * G,
                        G < GT ? G : GT, w, a.bph, lane, qf);
      wait_vmcnt<0>();
      float m_run[GT], z_run[GT];
      stats_tiles<DT, D, GT, kWaves, kStages>(dma, frags, kg, n, w, a.bph, c2, first, cnt, ring, qf, lane, m_run, z_run);
      float2 mine;
      if (stats_merge_waves<GT, kWaves>(m_run, z_run, c2, lane, wave, sm.red, mine))
        st_dev_f2(&stat_part[((long long)g * sq.blocks_x + bx) * kRows + threadIdx.x], mine.x, mine.y);
      // published: the partials are device-visible before the head's completion count moves.  The unit's
      // word goes to "done" (2); should a helper and the owner both have run the unit (their partials are
      // bit-identical), only the first to finish counts it.
      drain_vmem();
      __syncthreads();
      if (threadIdx.x == 0) {
        uint32_t* word = &ctl[kCtlUnitA + g * sq.blocks_x + bx];
        if (__hip_atomic_exchange(word, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 2u)
          __hip_atomic_fetch_add(&ctl[kCtlDoneA + g], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      continue;
    }

    // ------------------------------------------------------------ a score unit
    if (u_b >= a.n_units) break;
    si = seq_of_unit(u_b);
    const SweepSeq sq = a.s[si];
    const int rel = u_b - sq.unit_base;
    g = rel / sq.blocks_x;
    bx = rel % sq.blocks_x;
    const int seq = a.first_seq + si;
    const long long n = sq.n, n_prefix = n - w;
    const char* kg = static_cast<const char*>(a.k) + ((long long)H_kv * sq.tok + (long long)g * n) * T::kRowBytes;
    char* region = a.ws + sq.ws_off;
    const float2* __restrict__ stat_part = reinterpret_cast<const float2*>(region + a.off_stat_part);
    uint32_t* __restrict__ ctl = reinterpret_cast<uint32_t*>(region + a.off_counter);

    const long long n_tiles = (n_prefix + kTileKeys - 1) / kTileKeys;
    const long long t_begin = (long long)bx * sq.tiles_per_block;
    long long t_end = t_begin + sq.tiles_per_block;
    if (t_end > n_tiles) t_end = n_tiles;
    const int n_own = t_begin < t_end ? (int)(t_end - t_begin) : 0;
    const bool halo_left = n_own > 0 && t_begin > 0;
    const bool halo_right = n_own > 0 && t_end < n_tiles;
    const int n_jobs = n_own + (halo_left ? 1 : 0) + (halo_right ? 1 : 0);
    auto job_tile = [&](int j) -> long long {
      if (j < n_own) return t_begin + j;
      return (j == n_own && halo_left) ? t_begin - 1 : t_end;
    };
    __syncthreads();                                   // every wavefront is done with the previous unit's LDS
    // The unit's first tiles are requested before anything else, so that they travel while the head's
    // statistics are awaited and merged.
    q_request(si, g);
    if (threadIdx.x == 0) sm.next_job = kWaves * (kStages - 1);   // published by the barriers below
    int fifo[kStages];
#pragma unroll
    for (int p = 0; p < kStages; ++p) {
      const int j = wave + p * kWaves;
      fifo[p] = (p < kStages - 1 && j < n_jobs) ? j : -1;
    }
    int primed = 0;
#pragma unroll
    for (int p = 0; p < kStages - 1; ++p)
      if (fifo[p] >= 0) {
        dma.issue(kg, job_tile(fifo[p]), n, lane, ring + p * T::kTileChunks);
        ++primed;
      }
    u32x4 qf[GT][T::kSteps];
    q_commit(qf, primed);

    // The head's statistics.  A wait that lasts looks for statistics units of this head nobody has
    // claimed (their owners are not resident yet); one is then run above and this unit set up again.
    if (threadIdx.x == 0) {
      unsigned int spins = 0u;
      int verdict = -1;                                // -1: complete (or gave up), else: span of the unit to run
      while (ld_dev(&ctl[kCtlDoneA + g]) < (unsigned int)sq.blocks_x) {
        __builtin_amdgcn_s_sleep(4);
        ++spins;
        if (spins > a.spin_limit) {
          st_dev(&ctl0[kCtlError], 1u);
          break;
        }
        if ((spins % a.help_after) == 0u) {
          for (int x = 0; x < sq.blocks_x && verdict < 0; ++x) {
            uint32_t* word = &ctl[kCtlUnitA + g * sq.blocks_x + x];
            if (ld_dev(word) == 0u && atomicCAS(word, 0u, 1u) == 0u) verdict = x;
          }
          if (verdict >= 0) break;
        }
      }
      sm.claim[0] = verdict;
    }
    __syncthreads();
    help_bx = sm.claim[0];
    __syncthreads();
    if (help_bx >= 0) {
      help_si = si;
      help_g = g;
      wait_vmcnt<0>();                                 // the tiles requested for this unit have landed; they are asked for again
      __syncthreads();
      continue;
    }
    PoolArgs pa;
    pa.vnorm_part = reinterpret_cast<const float*>(region + a.off_vnorm_part);
    pa.vnorm_blocks = sq.vnorm_blocks;
    pa.pool_half = a.pool_half;
    pa.scores = a.scores + (long long)H_kv * sq.tok;
    pa.vbar = a.vbar + (long long)seq * H_kv;
    pa.token_norm = a.token_norm;
    pa.layer_stat = a.layer_stat + seq;
    pa.ent_part = reinterpret_cast<double2*>(region + a.off_ent_part);
    pa.counters = ctl;
    pa.error_word = &ctl0[kCtlError];
    pa.sel_hist0 = a.sel_ws ? reinterpret_cast<unsigned int*>(a.sel_ws + (size_t)seq * a.sel_stride + a.sel_off_hist) : nullptr;
    pa.plan = a.plan;
    pa.plan_seq = seq;
    float vb = 0.0f;   // this thread's share of the head's value-norm partials (an earlier launch wrote them)
    for (int i = threadIdx.x; i < pa.vnorm_blocks; i += kThreads)
      vb = fmaxf(vb, pa.vnorm_part[(long long)g * pa.vnorm_blocks + i]);
    merge_partials<GT, kThreads, true>(stat_part + (long long)g * sq.blocks_x * kRows, sq.blocks_x, false, c2,
                                       sm.sc.merge);
    __syncthreads();
    write_bias<GT, kThreads>(sm.sc.merge, nullptr, g * G, G < GT ? G : GT, w, a.bph, c2, sm.bias);
    __syncthreads();
    scores_tiles<DT, D, GT, kWaves, kStages, true>(dma, frags, kg, n, n_prefix, c2, t_begin, t_end, n_own, halo_left,
                                                   halo_right, n_jobs, fifo, ring, &sm.next_job, sm.bias, sm.sc.span,
                                                   qf, lane, nullptr, 1, 1);
    scores_finish<kThreads>(pa, vb, g, n, n_prefix, w, t_begin, t_end, n_tiles, sm.sc.span, sm.vb, sm.ss, sm.st,
                            &sm.last, (unsigned int)(sq.blocks_x * H_kv), (unsigned int)(g * sq.blocks_x + bx), H_kv,
                            bx == 0, wave, reinterpret_cast<unsigned int*>(&sm.tile[0][0][0]));
    u_b += (int)gridDim.x;
  }
}

// ------------------------------------------------------------------------------------------
// vnorm: per-workgroup maximum over rows of sum_c |V[g, k, c]|, all n rows.  Pure streaming: the
// same direct-to-LDS tile ring as the key sweeps (it sustains more bandwidth than loads into
// registers), 32-row tiles, no matrix work.
// ------------------------------------------------------------------------------------------

template <int DT, int D>
struct VShape {
  static constexpr int kWaves = Tile<DT, D>::kTileBytes > 8192 ? 4 : 8;
  static constexpr int kThreads = kWaves * 64;
  static constexpr int kStagesRaw = (128 * 1024) / (kWaves * Tile<DT, D>::kTileBytes);
  static constexpr int kStages = kStagesRaw > 4 ? 4 : kStagesRaw;
  static_assert(kStages >= 1, "tile too large for the ring");
};

template <int DT, int D>
__global__ void __launch_bounds__((VShape<DT, D>::kThreads))
vnorm_kernel(const SweepArgs a) {
  using T = Tile<DT, D>;
  const SweepSeq sq = a.s[blockIdx.z];
  if (blockIdx.x >= (unsigned int)sq.vnorm_blocks) return;
  const long long n = sq.n;
  const int tiles_per_block = sq.vnorm_tiles_per_block;
  const u32x4* __restrict__ v = static_cast<const u32x4*>(a.v) + (long long)a.H_kv * sq.tok * T::kCpr;
  float* __restrict__ vnorm_part = reinterpret_cast<float*>(a.ws + sq.ws_off + a.off_vnorm_part);
  float* __restrict__ row_norm = a.scores + (long long)a.H_kv * sq.tok;
  uint32_t* __restrict__ counters = reinterpret_cast<uint32_t*>(a.ws + sq.ws_off + a.off_counter);
  const int n_counter_words = kCtlUnitA + a.H_kv * sq.blocks_x;
  constexpr int kWaves = VShape<DT, D>::kWaves;
  constexpr int kStages = VShape<DT, D>::kStages < 2 ? 2 : VShape<DT, D>::kStages;
  __shared__ u32x4 s_tile[kWaves][kStages][T::kTileChunks];
  __shared__ float s_max[kWaves];
  if (blockIdx.x == 0 && blockIdx.y == 0) {
    for (int i = threadIdx.x; i < n_counter_words; i += VShape<DT, D>::kThreads) counters[i] = 0u;
    clear_selection_region(a, (int)blockIdx.z, VShape<DT, D>::kThreads);
  }

  const int lane = threadIdx.x & 63, wave = wave_index();
  const int g = blockIdx.y;
  const char* vg = reinterpret_cast<const char*>(v) + (long long)g * n * T::kRowBytes;
  TileDma<DT, D> dma;
  dma.init(lane);
  FragReader<DT, D> frags;
  frags.init(lane);

  const long long n_tiles = (n + kTileKeys - 1) / kTileKeys;
  const long long t_begin = (long long)blockIdx.x * tiles_per_block;
  long long t_end = t_begin + tiles_per_block;
  if (t_end > n_tiles) t_end = n_tiles;
  const long long first = t_begin + wave;
  const int cnt = first < t_end ? (int)((t_end - first + kWaves - 1) / kWaves) : 0;
  u32x4* ring = s_tile[wave][0];
#pragma unroll
  for (int p = 0; p < kStages - 1; ++p)
    if (p < cnt) dma.issue(vg, first + (long long)p * kWaves, n, lane, ring + p * T::kTileChunks);
  const float best = vnorm_tiles<DT, D, kWaves, kStages, false>(dma, frags, vg, nullptr, n, first, cnt, ring, lane,
                                                                 a.token_norm != 0, row_norm + (long long)g * n);
  float wave_best = best;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) wave_best = fmaxf(wave_best, __shfl_xor(wave_best, off));
  if ((threadIdx.x & 63) == 0) s_max[wave] = wave_best;
  __syncthreads();
  if (threadIdx.x == 0) {
    float m = s_max[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) m = fmaxf(m, s_max[i]);
    vnorm_part[(long long)g * sq.vnorm_blocks + blockIdx.x] = m;
  }
}

// ------------------------------------------------------------------------------------------
// poolstat: scores[g, i] = Vbar[g] * max_{|i'-i| <= half, i' in prefix} s_raw[g, i'] for the
// prefix, +inf for the window entries; S = sum s, T = sum s ln s in double with a fixed
// reduction order; the last workgroup to finish forms e = (ln S - T / S) / (H_kv * n')  (Eq. 4-5).
// ------------------------------------------------------------------------------------------
constexpr int kPoolThreads = 256;
constexpr int kPoolPerThread = 8;
constexpr int kPoolChunk = kPoolThreads * kPoolPerThread;

__global__ void __launch_bounds__(kPoolThreads)
poolstat_kernel(const float* __restrict__ s_raw, long long n, int w, int pool_half, int token_norm,
                const float* __restrict__ vnorm_part, int vnorm_blocks, float* __restrict__ scores,
                float* __restrict__ vbar, float* __restrict__ layer_stat,
                double2* __restrict__ ent_part, uint32_t* __restrict__ counters, unsigned int* __restrict__ sel_hist0,
                const BudgetPlanArgs plan, int plan_seq) {
  __shared__ float s_in[kPoolChunk + 2 * kPoolMaxHalf];
  __shared__ BudgetScratchT<kMaxPlannedLayers> s_plan;
  __shared__ unsigned int s_bins[kSelBins];
  const PlanInputs plan_in = plan_prefetch(plan, plan_seq);
  if (sel_hist0 != nullptr)
    for (int i = threadIdx.x; i < kSelBins; i += kPoolThreads) s_bins[i] = 0u;      // published by the barrier below
  unsigned int run_digit = 0u, run_len = 0u;
  __shared__ float s_vmax[kPoolThreads / 64];
  __shared__ double s_s[kPoolThreads / 64], s_t[kPoolThreads / 64];
  __shared__ unsigned int s_last;
  const int g = blockIdx.y;
  const long long n_prefix = n - w;
  const long long i0 = (long long)blockIdx.x * kPoolChunk;

  // Vbar of this head from the value-norm partials
  float vb = 0.0f;
  for (int i = threadIdx.x; i < vnorm_blocks; i += kPoolThreads)
    vb = fmaxf(vb, vnorm_part[(long long)g * vnorm_blocks + i]);
  for (int off = 32; off > 0; off >>= 1) vb = fmaxf(vb, __shfl_xor(vb, off));
  if ((threadIdx.x & 63) == 0) s_vmax[threadIdx.x >> 6] = vb;

  for (int i = threadIdx.x; i < kPoolChunk + 2 * pool_half; i += kPoolThreads) {
    const long long p = i0 + i - pool_half;
    s_in[i] = (p >= 0 && p < n_prefix) ? s_raw[(long long)g * n_prefix + p] : -INFINITY;
  }
  __syncthreads();
  vb = s_vmax[0];
  for (int i = 1; i < kPoolThreads / 64; ++i) vb = fmaxf(vb, s_vmax[i]);
  if (blockIdx.x == 0 && threadIdx.x == 0) vbar[g] = vb;

  double acc_s = 0.0, acc_t = 0.0;
#pragma unroll
  for (int j = 0; j < kPoolPerThread; ++j) {
    const int i = j * kPoolThreads + threadIdx.x;
    const long long p = i0 + i;
    if (p < n_prefix) {
      float m = s_in[i + pool_half];
      for (int d = 1; d <= pool_half; ++d) m = fmaxf(m, fmaxf(s_in[i + pool_half - d], s_in[i + pool_half + d]));
      const float s = (token_norm ? scores[(long long)g * n + p] : vb) * m;   // the entry's own value norm, left there by vnorm
      scores[(long long)g * n + p] = s;
      acc_s += (double)s;
      if (s > 0.0f) acc_t += (double)s * (double)logf(s);
      if (sel_hist0 != nullptr) digit0_count(s_bins, s, run_digit, run_len);
    } else if (p < n) {
      scores[(long long)g * n + p] = INFINITY;
      if (sel_hist0 != nullptr) digit0_count(s_bins, INFINITY, run_digit, run_len);
    }
  }
  if (sel_hist0 != nullptr) digit0_flush<kPoolThreads>(s_bins, run_digit, run_len, sel_hist0);
  const bool last = entropy_finish<kPoolThreads>(acc_s, acc_t, ent_part, counters, gridDim.x * gridDim.y,
                                                 blockIdx.y * gridDim.x + blockIdx.x,
                                                 (double)gridDim.y * (double)n_prefix, layer_stat, s_s, s_t, &s_last);
  if (last && plan.e != nullptr) {
    __syncthreads();
    plan_budgets(plan, plan_in, plan_seq, (float)s_t[0], &s_plan);
  }
}

__global__ void __launch_bounds__(256) fill_zero_kernel(float* __restrict__ p, long long count) {
  const long long i0 = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
  for (int j = 0; j < 4; ++j)
    if (i0 + j < count) p[i0 + j] = 0.0f;
}

// ------------------------------------------------------------------------------------------ host
static int compute_units() {
  static int cached = 0;
  if (cached == 0) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      cached = cus;
    else
      cached = 256;   // MI355X
  }
  return cached;
}

int sweep_device_wgs() { return compute_units(); }

int sweep_blocks_per_head(const lava_layer_desc& d) { return d.window > 32 ? 2 : 1; }

bool sweep_has_narrow_shape(const lava_layer_desc& d) { return !(d.dtype == LAVA_F32 && d.head_dim == 128); }

SweepPlan make_sweep_plan(const lava_layer_desc& d, int64_t n, int64_t batch_tokens, bool narrow) {
  SweepPlan p;
  const int G = (d.n_q_heads / d.n_kv_heads) * sweep_blocks_per_head(d);   // row blocks of 32 window rows per group
  int gt = kMaxChunkHeads;
  if (d.dtype == LAVA_F32 && d.head_dim == 128) gt = 2;
  p.chunk_heads = G < gt ? G : gt;     // even whenever heads have two blocks: a head's blocks stay in one chunk
  if (p.chunk_heads == 3) p.chunk_heads = 4;   // kernels are built for 1, 2 and 4 heads per chunk
  p.n_chunks = (G + p.chunk_heads - 1) / p.chunk_heads;
  p.narrow = narrow && sweep_has_narrow_shape(d);
  const int64_t n_tiles = (n + kTileKeys - 1) / kTileKeys;
  // One resident workgroup per slot of the device (one per CU for the wide shape, two for the
  // narrow one): the sweeps keep the group's query rows in registers and a tile ring in LDS, and
  // per-workgroup set-up (query load, partial results) is amortised over as many tiles as possible.
  const int64_t device_wgs = compute_units();
  int64_t target_wgs = p.narrow ? 2 * device_wgs : device_wgs;
  if (tuning().sweep_workgroups > 0) target_wgs = tuning().sweep_workgroups;   // forced by the caller's tuning
  // a sequence that shares its launches with others gets its share of the device, so that the
  // batch as a whole is cut into the longest runs the kernels allow
  const bool shared = batch_tokens > n;
  const auto share = [&](int64_t wgs) { return shared ? (wgs * n + batch_tokens - 1) / batch_tokens : wgs; };
  int64_t max_bx = share(target_wgs) / ((int64_t)d.n_kv_heads * p.n_chunks);
  if (max_bx < 1) max_bx = 1;
  int64_t tpb = (n_tiles + max_bx - 1) / max_bx;
  if (tpb < 16) tpb = 16;
  // all heads of a group in one workgroup -> the scores kernel can finish the scores itself, which
  // needs the workgroup's span of raw scores in LDS: a bounded number of tiles per workgroup
  p.fused_pool = p.n_chunks == 1;
  const int64_t fused_cap = p.narrow ? kFusedTilesNarrow : kFusedTilesWide;
  if (p.fused_pool && tpb > fused_cap) tpb = fused_cap;
  p.tiles_per_block = (int)tpb;
  p.blocks_x = (int)((n_tiles + tpb - 1) / tpb);
  // bounds that hold for either shape, alone or in a batch, and never shrink when n grows: a
  // workspace sized for the longest sequence of a batch must also hold the (differently split)
  // partials of every shorter one
  int64_t bx_alone = 2 * device_wgs / ((int64_t)d.n_kv_heads * p.n_chunks);
  if (target_wgs / ((int64_t)d.n_kv_heads * p.n_chunks) > bx_alone) bx_alone = target_wgs / ((int64_t)d.n_kv_heads * p.n_chunks);
  if (bx_alone < 1) bx_alone = 1;
  const int64_t capped = (n_tiles + kFusedTilesNarrow - 1) / kFusedTilesNarrow;
  p.blocks_x_bound = (int)(bx_alone > capped ? bx_alone : capped);
  // value norms: one workgroup per CU for a sequence alone, at least 8 tiles (one per wavefront)
  // each.  Sequences of a batch keep that cut (no share): the kernel's set-up is short, and many
  // small workgroups even out the unequal lengths better than few long ones.
  int64_t vb = (p.narrow ? device_wgs : target_wgs) / d.n_kv_heads;
  if (vb < 1) vb = 1;
  int64_t vtpb = (n_tiles + vb - 1) / vb;
  if (vtpb < 8) vtpb = 8;
  p.vnorm_tiles_per_block = (int)vtpb;
  p.vnorm_blocks = (int)((n_tiles + vtpb - 1) / vtpb);
  const int64_t vb_bound = (target_wgs > device_wgs ? target_wgs : device_wgs) / d.n_kv_heads;
  p.vnorm_blocks_bound = (int)(vb_bound > 1 ? vb_bound : 1);
  if (p.vnorm_blocks_bound < p.blocks_x_bound) p.vnorm_blocks_bound = p.blocks_x_bound;   // value norms cut like the statistics
  return p;
}

int pool_blocks(const lava_layer_desc& d, int64_t n) {
  (void)d;
  return (int)((n + kPoolChunk - 1) / kPoolChunk);
}

ScoreWorkspace make_score_workspace(const lava_layer_desc& d, int64_t n) {
  const SweepPlan p = make_sweep_plan(d, n);
  ScoreWorkspace w;
  size_t off = 0;
  w.off_stat_part = off;
  off += align_up(sizeof(float2) * (size_t)d.n_kv_heads * p.n_chunks * p.blocks_x_bound * p.chunk_heads * 32);
  w.off_vnorm_part = off;
  off += align_up(sizeof(float) * (size_t)d.n_kv_heads * p.vnorm_blocks_bound);
  w.off_sraw = off;          // only a group split into chunks goes through raw scores in memory
  if (!p.fused_pool) off += align_up(sizeof(float) * (size_t)d.n_kv_heads * (size_t)(n - d.window));
  w.off_ent_part = off;
  const size_t ent_blocks = (size_t)pool_blocks(d, n) > (size_t)p.blocks_x_bound * p.n_chunks
                                ? (size_t)pool_blocks(d, n) : (size_t)p.blocks_x_bound * p.n_chunks;
  off += align_up(sizeof(double2) * (size_t)d.n_kv_heads * ent_blocks);
  w.off_counter = off;
  off += align_up(sizeof(uint32_t) * ((size_t)kCtlUnitA + (size_t)d.n_kv_heads * p.blocks_x_bound));
  w.bytes = off;
  return w;
}

int32_t launch_vnorm(const lava_layer_desc& d, const SweepArgs& a, int max_vnorm_blocks, hipStream_t s) {
  const dim3 grid(max_vnorm_blocks, d.n_kv_heads, a.n_seq);
  ProfScope ps(KID_VNORM, s);
#define LAVA_VNORM(DTV, DV) \
  hipLaunchKernelGGL((vnorm_kernel<DTV, DV>), grid, dim3(VShape<DTV, DV>::kThreads), 0, s, a)
  if (d.dtype == LAVA_BF16 && d.head_dim == 128) LAVA_VNORM(LAVA_BF16, 128);
  else if (d.dtype == LAVA_BF16 && d.head_dim == 64) LAVA_VNORM(LAVA_BF16, 64);
  else if (d.dtype == LAVA_F32 && d.head_dim == 64) LAVA_VNORM(LAVA_F32, 64);
  else if (d.dtype == LAVA_F32 && d.head_dim == 128) LAVA_VNORM(LAVA_F32, 128);
  else return LAVA_ERR_SHAPE;
#undef LAVA_VNORM
  return launch_status();
}

__global__ void __launch_bounds__(256) unit_vnorm_kernel(const SweepArgs a) {
  const SweepSeq sq = a.s[blockIdx.z];
  float* vnorm_part = reinterpret_cast<float*>(a.ws + sq.ws_off + a.off_vnorm_part);
  uint32_t* counters = reinterpret_cast<uint32_t*>(a.ws + sq.ws_off + a.off_counter);
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < a.H_kv * sq.vnorm_blocks) vnorm_part[i] = 1.0f;
  for (int j = i; j < kCtlUnitA + a.H_kv * sq.blocks_x; j += (int)gridDim.x * 256) counters[j] = 0u;
  if (blockIdx.x == 0) clear_selection_region(a, (int)blockIdx.z, 256);
}

int32_t launch_unit_vnorm(const lava_layer_desc& d, const SweepArgs& a, int max_vnorm_blocks, hipStream_t s) {
  const int n_part = d.n_kv_heads * max_vnorm_blocks;
  const int n = n_part > kCtlUnitA ? n_part : kCtlUnitA;
  ProfScope ps(KID_VNORM, s);
  hipLaunchKernelGGL(unit_vnorm_kernel, dim3((n + 255) / 256, 1, a.n_seq), dim3(256), 0, s, a);
  return launch_status();
}

float sweep_exp2_scale(const lava_layer_desc& d) {
  const float scale = d.softmax_scale > 0.0f ? d.softmax_scale : 1.0f / sqrtf((float)d.head_dim);
  return scale * kLog2e;
}

// Dispatch over (dtype, head_dim, heads per chunk).
#define LAVA_SWEEP_DISPATCH(CALL)                                                   \
  do {                                                                              \
    const int gt = p.chunk_heads;                                                   \
    if (d.dtype == LAVA_BF16 && d.head_dim == 128) {                                \
      if (gt == 4) CALL(LAVA_BF16, 128, 4); else if (gt == 2) CALL(LAVA_BF16, 128, 2); \
      else CALL(LAVA_BF16, 128, 1);                                                 \
    } else if (d.dtype == LAVA_BF16 && d.head_dim == 64) {                          \
      if (gt == 4) CALL(LAVA_BF16, 64, 4); else if (gt == 2) CALL(LAVA_BF16, 64, 2); \
      else CALL(LAVA_BF16, 64, 1);                                                  \
    } else if (d.dtype == LAVA_F32 && d.head_dim == 64) {                           \
      if (gt == 4) CALL(LAVA_F32, 64, 4); else if (gt == 2) CALL(LAVA_F32, 64, 2);  \
      else CALL(LAVA_F32, 64, 1);                                                   \
    } else if (d.dtype == LAVA_F32 && d.head_dim == 128) {                          \
      if (gt == 2) CALL(LAVA_F32, 128, 2); else CALL(LAVA_F32, 128, 1);             \
    } else {                                                                        \
      return LAVA_ERR_SHAPE;                                                        \
    }                                                                               \
  } while (0)

int32_t launch_stats(const lava_layer_desc& d, const SweepArgs& a, int max_blocks_x, const SweepPlan& p,
                     bool with_vnorm, hipStream_t s) {
  const dim3 grid(max_blocks_x, d.n_kv_heads * p.n_chunks, a.n_seq);
  ProfScope ps(with_vnorm ? KID_PREPASS : KID_STATS, s);
#define LAVA_STATS_W(DTV, DV, GTV, WV)                                                                             \
  do {                                                                                                             \
    if (with_vnorm)                                                                                                \
      hipLaunchKernelGGL((stats_kernel<DTV, DV, GTV, WV, true>), grid, dim3(Shape<DTV, DV, WV>::kThreads), 0, s, a); \
    else                                                                                                           \
      hipLaunchKernelGGL((stats_kernel<DTV, DV, GTV, WV, false>), grid, dim3(Shape<DTV, DV, WV>::kThreads), 0, s, a); \
  } while (0)
#define LAVA_STATS(DTV, DV, GTV)                                               \
  do {                                                                         \
    if (Shape<DTV, DV, 4>::kNarrow && p.narrow) LAVA_STATS_W(DTV, DV, GTV, (Shape<DTV, DV, 4>::kNarrow ? 4 : 8)); \
    else LAVA_STATS_W(DTV, DV, GTV, 8);                                        \
  } while (0)
  LAVA_SWEEP_DISPATCH(LAVA_STATS);
#undef LAVA_STATS
#undef LAVA_STATS_W
  return launch_status();
}

int32_t launch_sweep(const lava_layer_desc& d, const SweepArgs& a, const SweepPlan& p, hipStream_t s) {
  if (!p.fused_pool || a.lse != nullptr || a.bph != 1) return LAVA_ERR_INVALID_ARG;
  // persistent workgroups: as many as the device keeps resident for this shape, at most one per unit
  const int slots = compute_units() * ((p.narrow && sweep_has_narrow_shape(d)) ? 2 : 1);
  const dim3 grid(a.n_units < slots ? a.n_units : slots);
  ProfScope ps(KID_SWEEP, s);
#define LAVA_SWEEP_W(DTV, DV, GTV, WV) \
  hipLaunchKernelGGL((sweep_kernel<DTV, DV, GTV, WV>), grid, dim3(Shape<DTV, DV, WV>::kThreads), 0, s, a)
#define LAVA_SWEEP(DTV, DV, GTV)                                               \
  do {                                                                         \
    if (Shape<DTV, DV, 4>::kNarrow && p.narrow) LAVA_SWEEP_W(DTV, DV, GTV, (Shape<DTV, DV, 4>::kNarrow ? 4 : 8)); \
    else LAVA_SWEEP_W(DTV, DV, GTV, 8);                                        \
  } while (0)
  LAVA_SWEEP_DISPATCH(LAVA_SWEEP);
#undef LAVA_SWEEP
#undef LAVA_SWEEP_W
  return launch_status();
}

int32_t launch_scores(const lava_layer_desc& d, const SweepArgs& a, int max_blocks_x, const SweepPlan& p,
                      hipStream_t s) {
  const dim3 grid(max_blocks_x, d.n_kv_heads * p.n_chunks, a.n_seq);
  ProfScope ps(KID_SCORES, s);
  if (p.n_chunks > 1) {
    // partial group maxima are combined with integer atomicMax; start from +0 (a fill kernel,
    // not a memset node, so the call sequence can be captured in a HIP graph).  One sequence per launch here.
    const long long count = (long long)d.n_kv_heads * (a.s[0].n - d.window);
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((count + 1023) / 1024)), dim3(256), 0, s,
                       reinterpret_cast<float*>(a.ws + a.s[0].ws_off + a.off_sraw), count);
  }
#define LAVA_SCORES_W(DTV, DV, GTV, WV)                                                                     \
  do {                                                                                                      \
    if (p.fused_pool)                                                                                       \
      hipLaunchKernelGGL((scores_kernel<DTV, DV, GTV, true, WV>), grid, dim3(Shape<DTV, DV, WV>::kThreads), \
                         0, s, a);                                                                          \
    else                                                                                                    \
      hipLaunchKernelGGL((scores_kernel<DTV, DV, GTV, false, WV>), grid, dim3(Shape<DTV, DV, WV>::kThreads), \
                         0, s, a);                                                                          \
  } while (0)
#define LAVA_SCORES(DTV, DV, GTV)                                               \
  do {                                                                          \
    if (Shape<DTV, DV, 4>::kNarrow && p.narrow) LAVA_SCORES_W(DTV, DV, GTV, (Shape<DTV, DV, 4>::kNarrow ? 4 : 8)); \
    else LAVA_SCORES_W(DTV, DV, GTV, 8);                                        \
  } while (0)
  LAVA_SWEEP_DISPATCH(LAVA_SCORES);
#undef LAVA_SCORES
#undef LAVA_SCORES_W
  return launch_status();
}

int32_t launch_poolstat(const lava_layer_desc& d, int64_t n, const float* s_raw,
                        const float* vnorm_part, int vnorm_blocks, float* scores, float* vbar,
                        float* layer_stat, double2* ent_part, uint32_t* counters, unsigned int* sel_hist0,
                        const BudgetPlanArgs& plan, int plan_seq, hipStream_t s) {
  const dim3 grid(pool_blocks(d, n), d.n_kv_heads), block(kPoolThreads);
  ProfScope ps(KID_POOLSTAT, s);
  hipLaunchKernelGGL(poolstat_kernel, grid, block, 0, s, s_raw, (long long)n, d.window,
                     d.pool_kernel / 2, d.score_kind == LAVA_SCORE_TOKEN_NORM ? 1 : 0, vnorm_part, vnorm_blocks, scores, vbar, layer_stat, ent_part,
                     counters, sel_hist0, plan, plan_seq);
  return launch_status();
}

}  // namespace lava
