// Shared declarations of the HIP library: kernel launchers, the per-kernel timing hook and a
// few device helpers.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/lava.h"

namespace lava {

// ---------------------------------------------------------------- kernel ids (timing hook)
enum KernelId : int {
  KID_VNORM = 0,      // value-row L1 norms, per-block maxima
  KID_STATS,          // window softmax statistics (row max, row sum) per block
  KID_SCORES,         // window scores: group-max of window-mean attention
  KID_SWEEP,          // statistics and scores of a layer in one persistent launch
  KID_PREPASS,        // value-row norms and window softmax statistics in one launch
  KID_POOLSTAT,       // max-pool, value factor, +inf window entries, entropy statistic
  KID_SEL_INIT,       // selection: clear histograms and counters
  KID_SEL_FUSED,      // selection: radix select + ordered write in one launch
  KID_SEL_STEPS,      // selection: the same phases as separate launches (very large inputs)
  KID_COMPACT,        // K/V row gather
  KID_BUDGETS,        // layer budgets on the device
  KID_DECODE,         // decode attention over the packed cache: per-unit partials
  KID_DECODE_MERGE,   // decode attention: merge of the units of each head
  KID_COUNT
};

// Brackets a launch with events when timing is enabled (no-ops otherwise).
void prof_begin(int kid, hipStream_t s);
void prof_end(int kid, hipStream_t s);

struct ProfScope {
  int kid;
  hipStream_t s;
  ProfScope(int k, hipStream_t st) : kid(k), s(st) { prof_begin(kid, s); }
  ~ProfScope() { prof_end(kid, s); }
};

inline int32_t hip_ok(hipError_t e) { return e == hipSuccess ? LAVA_OK : LAVA_ERR_HIP; }
inline int32_t launch_status() { return hip_ok(hipGetLastError()); }

// Discards an error left in the thread by earlier HIP calls that are none of this library's, so that
// the launch checks below report this call's launches only.
inline void discard_stale_error() { (void)hipGetLastError(); }

// The process-wide launch-shape tuning (lava_set_tuning); all-zero = the library's own choices.
const lava_tuning& tuning();

// Order-preserving map float -> uint32 used by the selection (larger score = larger key); -0 and +0
// coincide.  The selection's first digit is the key's top kSelDigit0Bits bits.
__device__ __forceinline__ unsigned int score_key(float f) {
  unsigned int b = __float_as_uint(f);
  if ((b << 1) == 0u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
constexpr int kSelBins = 2048;
constexpr int kSelDigit0Shift = 21;

constexpr size_t kAlign = 256;
constexpr size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------- sweep (K, V) kernels
constexpr int kTileKeys = 32;        // keys per MFMA tile
constexpr int kMaxChunkHeads = 4;    // query heads a wavefront keeps in registers

struct SweepPlan {
  int chunk_heads;     // GT: row blocks (32 window rows of one head) per chunk (<= kMaxChunkHeads; <= 2 for f32 with d_h 128)
  int n_chunks;        // ceil(G * blocks per head / GT)
  int blocks_x;        // workgroups along the key axis per (KV head, chunk)
  int tiles_per_block; // key tiles per workgroup
  int vnorm_blocks;    // workgroups per KV head of the value-norm kernel
  int vnorm_tiles_per_block;
  int blocks_x_bound, vnorm_blocks_bound;   // upper bounds of blocks_x / vnorm_blocks for any shorter sequence
  bool fused_pool;     // the scores kernel also pools, scales and forms the layer statistic
  bool narrow;         // 4-wavefront workgroups, two per CU (launches of several rounds of workgroups)
};
// batch_tokens: tokens of all sequences that share the launches (0 or n: the sequence is alone);
// narrow: ask for the two-per-CU shape (ignored where the kernels have only one shape)
SweepPlan make_sweep_plan(const lava_layer_desc& d, int64_t n, int64_t batch_tokens = 0, bool narrow = false);
bool sweep_has_narrow_shape(const lava_layer_desc& d);
int sweep_device_wgs();   // compute units of the current device
int sweep_blocks_per_head(const lava_layer_desc& d);   // 32-row blocks a head's window rows take: 1 or 2

// Workspace of lava_window_scores for one sequence (all offsets 256-byte aligned).
struct ScoreWorkspace {
  size_t off_stat_part;   // float2 [H_kv*n_chunks][blocks_x][GT*32]  (row max, row sum)
  size_t off_vnorm_part;  // float  [H_kv][vnorm_blocks]
  size_t off_sraw;        // float  [H_kv][N']  group-max of window-mean attention
  size_t off_ent_part;    // double2[pool blocks]  partial (S, T)
  size_t off_counter;     // uint32 "last workgroup done" tickets
  size_t bytes;
};
ScoreWorkspace make_score_workspace(const lava_layer_desc& d, int64_t n);
int pool_blocks(const lava_layer_desc& d, int64_t n);

int32_t launch_vnorm(const lava_layer_desc& d, int64_t n, const void* v, float* vnorm_part,
                     uint32_t* counters, const SweepPlan& p, hipStream_t s);
// Arguments of a sweep launch.  One launch covers up to kMaxSeqPerLaunch sequences of a batch
// (blockIdx.z picks the sequence): the whole table travels in the kernel arguments, so nothing is
// copied to the device and the call stays capturable.  Workgroups beyond a sequence's own count
// (the grid is sized for the longest sequence) return at once.
constexpr int kMaxSeqPerLaunch = 32;

struct SweepSeq {
  long long n;               // cached tokens of the sequence
  long long tok;             // tokens of the batch before it (K, V and the scores are packed)
  long long ws_off;          // byte offset of the sequence's region in the workspace
  int blocks_x;              // stats / scores workgroups along the key axis
  int tiles_per_block;
  int vnorm_blocks;          // value-norm partials per KV head the scores kernel finds
  int vnorm_tiles_per_block;
  int unit_base;             // persistent launch: work units of the sequences before this one (H_kv * blocks_x each)
};

// Budgets formed right after the layer statistic, by the workgroup that formed it (e == nullptr: none).
// Sequence b of the batch uses row b of every table.
struct BudgetPlanArgs {
  float* e;                  // [batch][n_layers] statistics; column `layer` is written by this call
  const int64_t* total;      // [batch]
  const int64_t* lo;         // [batch][n_layers]
  const int64_t* hi;         // [batch][n_layers]
  int64_t* out;              // [batch][n_layers] budgets (-1 everywhere for infeasible bounds)
  int n_layers, layer;
};

struct SweepArgs {
  const void* q_win;         // [batch][H][w][d_h]
  const void* k;             // packed, [H_kv][n][d_h] per sequence
  const void* v;
  const float* lse;          // [batch][H][w] or null
  float* scores;             // packed, [H_kv][n] per sequence
  float* vbar;               // [batch][H_kv]
  float* layer_stat;         // [batch]
  char* ws;
  size_t off_stat_part, off_vnorm_part, off_sraw, off_ent_part, off_counter;   // inside a sequence's region
  int H, H_kv, w, G, n_chunks, pool_half;   // G: row blocks of 32 window rows per KV group = (H / H_kv) * bph
  int bph;                   // row blocks per query head: 1 (w <= 32) or 2
  int token_norm;            // value factor per token: vnorm leaves ||V[g, i]||_1 in scores[g][i], the pooling step multiplies by it
  float c2;
  int first_seq;             // index in the batch of s[0]
  int n_seq;
  // lava_window_scores_primed: the selection workspace whose region (first_seq + z) the launch prepares
  // (null: none): region stride and the offsets of the histograms / the state inside a region
  char* sel_ws;
  size_t sel_stride, sel_off_hist, sel_off_state;
  BudgetPlanArgs plan;
  int n_units;               // persistent launch: H_kv * sum of blocks_x over the table
  unsigned int spin_limit;   // persistent launch: polls of a wait for other workgroups before it gives up
  unsigned int help_after;   // persistent launch: polls after which a waiting workgroup looks for unclaimed units (>= 1)
  int orphan_mod;            // persistent launch, testing aid: owners leave every orphan_mod-th statistics unit unclaimed (0: none)
  SweepSeq s[kMaxSeqPerLaunch];
};

// grid.x of the launches below: the largest blocks_x / vnorm_blocks in the table
int32_t launch_vnorm(const lava_layer_desc& d, const SweepArgs& a, int max_vnorm_blocks, hipStream_t s);
// value factor 1 for every head (scores without the value norm): fills the partials, clears the tickets
int32_t launch_unit_vnorm(const lava_layer_desc& d, const SweepArgs& a, int max_vnorm_blocks, hipStream_t s);
// with_vnorm: the launch also sweeps the value rows (SweepSeq::vnorm_blocks == blocks_x, no launch_vnorm)
int32_t launch_stats(const lava_layer_desc& d, const SweepArgs& a, int max_blocks_x, const SweepPlan& p,
                     bool with_vnorm, hipStream_t s);
// statistics and scores in one persistent launch (all heads of a group in one workgroup, no caller LSE)
int32_t launch_sweep(const lava_layer_desc& d, const SweepArgs& a, const SweepPlan& p, hipStream_t s);
// not fused (a group split into chunks): one sequence per launch, raw scores to the region's s_raw
int32_t launch_scores(const lava_layer_desc& d, const SweepArgs& a, int max_blocks_x, const SweepPlan& p,
                      hipStream_t s);
float sweep_exp2_scale(const lava_layer_desc& d);
int32_t launch_poolstat(const lava_layer_desc& d, int64_t n, const float* s_raw,
                        const float* vnorm_part, int vnorm_blocks, float* scores, float* vbar,
                        float* layer_stat, double2* ent_part, uint32_t* counters, unsigned int* sel_hist0,
                        const BudgetPlanArgs& plan, int plan_seq, hipStream_t s);
// words of a selection's state block (cleared together with its histograms)
constexpr int kSelStateWords = 8;

// ---------------------------------------------------------------- selection / compaction
struct SelectWorkspace {
  size_t off_hist;      // uint32 [3][2048]
  size_t off_state;     // SelectState
  size_t off_blk;       // uint32 [2][n_blocks]: keys above / equal to the threshold per workgroup
  int n_blocks;
  size_t bytes;
};
SelectWorkspace make_select_workspace(int64_t total);

int32_t launch_select(int n_heads, const float* scores, const int64_t* seg_offsets, int64_t total,
                      int64_t budget, const int64_t* budget_dev, int32_t* head_counts,
                      int64_t* head_offsets, int32_t* kept_idx, float* kept_scores, void* ws,
                      hipStream_t s);
// independent selections in as few launches as the device's capacity allows; problem p uses the
// p-th region of the workspace, regions laid out for max_total entries
constexpr int kMaxSelProblems = 32;
// cleared: an earlier kernel on the stream has zeroed every problem's region and survivor counts (what the
// selection's own init kernel does), so launches that fit the one-kernel path skip that kernel
int32_t launch_select_batch(int n_heads, int n_problems, const lava_select_problem* problems, int64_t max_total,
                            void* ws, hipStream_t s, bool cleared = false);

int32_t select_error_flag(const void* ws, int64_t max_total, int n_problems, hipStream_t s, int* flag);
// host-side argument checks of one selection (shared by every entry point that takes one)
int32_t check_select_problem(int32_t n_heads, const lava_select_problem& p);

// src_offsets null: dense source [H_kv][n]; otherwise a packed source inside a pool of n rows.
int32_t launch_compact(const lava_layer_desc& d, int64_t n, const int64_t* src_offsets, const void* k,
                       const void* v, const int32_t* pos_src, const int64_t* head_offsets,
                       const int32_t* kept_idx, int64_t capacity, void* k_out, void* v_out, int32_t* pos_out,
                       hipStream_t s);
int32_t launch_compact_batch(const lava_layer_desc& d, int n_problems, const lava_compact_problem* problems,
                             hipStream_t s);
// Re-compaction of layers 0..n_layers-1 of a cascade arena IN PLACE (K and V rows move inside k / v; token
// positions go from pos_src to pos_dst): row r of the new layout (layer_start_new, offs_new [layer][H_kv+1],
// kept_idx[r] = index in the head's old segment) comes from the old layout (layer_start_cur, offs_cur).
// Every row moves towards the front or stays, which is what makes it possible.  `sync`: 128 zeroed words.
int32_t launch_compact_inplace(const lava_layer_desc& d, int n_layers, const int64_t* layer_start_cur,
                               const int64_t* layer_start_new, const int64_t* offs_cur, const int64_t* offs_new,
                               const int32_t* kept_idx, void* k, void* v, const int32_t* pos_src, int32_t* pos_dst,
                               int64_t capacity, unsigned int* sync, int32_t* error, hipStream_t s);

// ---------------------------------------------------------------- decode attention
struct DecodePlan {
  int rows_per_unit;     // rows of one head a workgroup handles
  int group_pad;         // G rounded up to 1, 2, 4 or 8
  int64_t units_bound;   // units a sequence can have at most (grid.x)
  size_t off_ml, off_acc, bytes;
};
DecodePlan make_decode_plan(const lava_layer_desc& d, int32_t batch, int64_t rows_capacity, int64_t tail_len);
int32_t launch_decode(const lava_layer_desc& d, int32_t batch, const void* q, const void* k_hat,
                      const void* v_hat, const int64_t* head_offsets, const int64_t* seq_base,
                      int64_t rows_capacity, const void* k_tail, const void* v_tail, int64_t tail_len,
                      int64_t tail_capacity, float* out, float* lse, void* ws, const DecodePlan& p,
                      hipStream_t s);

// ---------------------------------------------------------------- layer budgets
// The host path runs the sequential allocation, the device kernel the same arithmetic spread over
// one wavefront per sequence: bit-identical integers.
int32_t budgets_host(int32_t batch, int32_t n_layers, const float* e, const int64_t* total,
                     const int64_t* lo, const int64_t* hi, int64_t* out);
int32_t launch_budgets(int32_t batch, int32_t n_layers, const float* e, const int64_t* total,
                       const int64_t* lo, const int64_t* hi, int64_t* out, hipStream_t s);
// A cascade step's plan for one sequence: budgets of layers 0..n_layers-1 (bounds lo / hi for every
// layer), the rows each keeps = min(budget, bound, rows it holds: head_offsets_cur[t][n_heads]
// for t < n_layers - 1, hi for the newest), and layer_start[0..n_layers] = their prefix sums.
// gather_sync: 128 words the kernel sets to zero for launch_compact_inplace later in the step, or null.
// regions (ws != null): the workspace regions of the step's n_layers selections and their survivor counts
// [n_layers][n_heads], cleared by extra workgroups of the same launch (launch_select_batch(cleared = true)).
struct SelectRegions {
  char* ws;
  size_t stride, off_hist, off_state;
  int32_t* head_counts;
};
int32_t launch_cascade_plan(int32_t n_layers, int32_t n_heads, const float* e, int64_t total, int64_t lo, int64_t hi,
                            int64_t bound, const int64_t* head_offsets_cur, int64_t* budgets, int64_t* layer_start,
                            unsigned int* gather_sync, const SelectRegions& regions, hipStream_t s);

}  // namespace lava
