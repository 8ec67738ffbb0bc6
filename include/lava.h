/*
 * lava.h — C ABI of the MI355X (gfx950) implementation of LAVa's prefill-end KV-cache
 * eviction path (arXiv 2509.09754).
 *
 * For one transformer layer the path is, in order:
 *   lava_window_scores   attention of the last w queries against every cached key, reduced to
 *                        the pooled, head-comparable LAVa score of every cache entry, plus the
 *                        layer's normalised-entropy statistic          (Def. 1 / Eq. 3, Sec. 4.3,
 *                                                                       Sec. 5.1 pooling, Eq. 4-5)
 *   lava_layer_budgets   dynamic layer budgets from the statistics of the layers seen so far
 *                                                                      (Alg. 2, inner loop)
 *   lava_select_topk     one top-B selection over the flattened heads of the layer; the number
 *                        of survivors per head is the dynamic head budget   (Alg. 1, Sec. 4.1)
 *   lava_compact_kv      packs the surviving K/V rows per head              (Alg. 1, last loop)
 * and, after the path, lava_decode_attention reads the packed cache (Sec. 2 decoding step).
 * Around the path: lava_select_topk_batch / lava_compact_batch run tables of independent
 * selections / compactions in one launch each (the sequences of a ragged batch, the layers of a
 * stack), and lava_cascade_step is Algorithm 2 as a driver over a stack's compressed caches.
 *
 * Conventions common to all calls
 *   - "device" pointers are HIP device memory of the current device, "host" pointers are
 *     ordinary host memory.  The library never allocates, frees or keeps any buffer; the
 *     caller owns everything, including the workspace.  Outputs must not alias inputs.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = default stream)
 *     and the call returns without synchronising, unless stated otherwise.
 *   - All argument checks happen on the host before anything is launched: a call that returns
 *     an argument error (INVALID_ARG, SHAPE, BUDGET, WORKSPACE) has launched nothing.
 *     LAVA_ERR_HIP means a launch failed; kernels of the same call enqueued before it may still
 *     run.  An error left behind by earlier, unrelated HIP calls of the thread is discarded, not
 *     reported.  Errors are reported by return code only.
 *   - Layouts are row-major with the last index fastest.  K and V are head-major per layer as
 *     in the paper's layer-wise view (App. A): [H_kv][N][d_h].
 *   - Notation: H query heads, H_kv KV heads, G = H / H_kv (query head h reads KV head
 *     h / G), d_h head dimension, N cached tokens, w window, N' = N - w prefix length.
 */
#ifndef LAVA_H
#define LAVA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LAVA_OK = 0,
  LAVA_ERR_INVALID_ARG = 1, /* null pointer, negative count, unknown enum value            */
  LAVA_ERR_SHAPE = 2,       /* a shape the kernels are not built for (see lava_layer_desc) */
  LAVA_ERR_BUDGET = 3,      /* budget outside its feasible range                           */
  LAVA_ERR_WORKSPACE = 4,   /* workspace missing, misaligned (256 B) or too small          */
  LAVA_ERR_HIP = 5          /* a HIP runtime call or kernel launch failed                  */
} lava_status;

typedef enum { LAVA_F32 = 0, LAVA_BF16 = 1 } lava_dtype;

/* Which score lava_window_scores writes.
 *   LAVA_SCORE_LAVA       window-mean attention times max_k ||V[k]||_1 (Def. 1 / Eq. 3)
 *   LAVA_SCORE_ATTENTION  window-mean attention alone: the value factor is 1 and V is not read
 *                         (the recent-window attention score of the SnapKV / Ada-KV rows of
 *                         Table 4, and the paper's ablation without the value norm); vbar = 1
 *   LAVA_SCORE_TOKEN_NORM the pooled window-mean attention times the token's own ||V[i]||_1
 *                         (the VATP comparison of the appendix and of Table 4: a factor per
 *                         token where LAVa has one per head); vbar is still max_k ||V[k]||_1
 * Group-max, pooling and the layer statistic are the same for all. */
typedef enum { LAVA_SCORE_LAVA = 0, LAVA_SCORE_ATTENTION = 1, LAVA_SCORE_TOKEN_NORM = 2 } lava_score_kind;

/* One layer of one model.  Plain data, read during the call only. */
typedef struct lava_layer_desc {
  int32_t n_q_heads;    /* H                                                                  */
  int32_t n_kv_heads;   /* H_kv <= 64; H % H_kv == 0 and G = H / H_kv <= 16 (decode step: <= 8)   */
  int32_t head_dim;     /* d_h: 64 or 128                                                     */
  int32_t window;       /* w, 1 <= w <= 64: number of observation-window query rows           */
  int32_t pool_kernel;  /* odd, 1..15; the paper uses 7 (Sec. 5.1); 1 disables pooling        */
  int32_t dtype;        /* lava_dtype of q_win, k, v, k_out, v_out                            */
  float softmax_scale;  /* logits are scale * <q, k>; 0 selects 1 / sqrt(d_h) (Sec. 2)        */
  int32_t score_kind;   /* lava_score_kind; 0 = the LAVa score                                */
} lava_layer_desc;

const char* lava_status_string(int32_t status);

/*
 * Launch-shape tuning, for tests and benchmarks: how the sweeps of lava_window_scores and the
 * units of lava_decode_attention are cut, and how long a grid-wide wait polls.  A zero field
 * means "the library's own choice", which is what production callers want.  The setting is
 * process-wide and read at every call: set it while no call is in progress, and ask the
 * *_workspace_bytes functions again after changing it (decode_rows_per_unit and
 * sweep_workgroups change workspace sizes).  lava_set_tuning(NULL) restores the defaults.
 * Results never depend on the tuning (scores: up to floating-point summation order of the
 * softmax statistics; everything else bit for bit).
 */
typedef struct lava_tuning {
  int32_t sweep_shape;          /* 0 library's choice, 1 wide (one workgroup per compute unit),
                                   2 narrow (two per compute unit), where the kernels have both */
  int32_t sweep_workgroups;     /* workgroups a sweep launch aims for, 1..65536                */
  int32_t sweep_schedule;       /* 0 library's choice (today: 3 for a launch of one sequence, else
                                   1), 1 three launches (value norms, statistics, scores), 2 value
                                   norms, then one persistent launch for statistics and scores
                                   where the shape allows it, 3 value norms inside the statistics
                                   launch, then scores.  All give bit-identical results          */
  int32_t decode_rows_per_unit; /* rows of one head per decode work unit, 128..8192            */
  int32_t barrier_spin_limit;   /* polls of a grid-wide wait before it gives up (default 2^18) */
  int32_t sweep_orphan_units;   /* testing aid for the persistent sweep: the owners leave every n-th
                                   statistics unit unclaimed, as if their workgroup were not resident,
                                   so that a workgroup waiting for that head has to run it; 0 = none */
  int32_t reserved[2];          /* must be zero                                                */
} lava_tuning;
int32_t lava_set_tuning(const lava_tuning* tuning);
int32_t lava_get_tuning(lava_tuning* tuning);

/* Bytes of device workspace lava_window_scores needs for `batch` sequences holding
 * `total_tokens` cached tokens in all.  Returns 0 for an invalid descriptor. */
size_t lava_window_scores_workspace_bytes(const lava_layer_desc* desc, int32_t batch,
                                          int64_t total_tokens);

/*
 * Scores of every cache entry of one layer (Def. 1 / Eq. 3; GQA group-max, Sec. 4.3; max-pool,
 * Sec. 5.1) and the layer statistic e_l (Eq. 4-5).
 *
 *   seq_lens   host  [batch]            N_b > w for every sequence
 *   q_win      device [batch][H][w][d_h]      queries of the last w positions, row r is the
 *                                             query at position N_b - w + r
 *   k, v       device, sequences packed back to back; sequence b starts at element
 *              H_kv * d_h * sum_{b' < b} N_b' and is laid out [H_kv][N_b][d_h]
 *   lse        device [batch][H][w] or NULL   natural-log log-sum-exp of each window row's
 *                                             logits over keys 0..N_b-w+r, if the prefill
 *                                             attention kept it; skips the statistics pass
 *   scores     device, float, packed like k without the d_h axis: [H_kv][N_b] per sequence.
 *              Prefix entries hold the pooled group score; the w window entries of each head
 *              hold +inf (they are always retained, Eq. 1)
 *   vbar       device [batch][H_kv] float     max_k ||V[k]||_1 over all N_b rows (Thm. 1)
 *   layer_stat device [batch] float           e_l of Eq. 5 over the H_kv * N' prefix scores
 *
 * Each window row is normalised over all keys up to and including its own position.
 * Results are deterministic (no floating-point atomics).  Scores carry fp32 accumulation
 * error only (inputs are used exactly as stored).
 */
int32_t lava_window_scores(const lava_layer_desc* desc, int32_t batch, const int64_t* seq_lens,
                           const void* q_win, const void* k, const void* v, const float* lse,
                           float* scores, float* vbar, float* layer_stat, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

/*
 * lava_window_scores that also prepares the workspace of the selection which will rank the scores it
 * writes (Alg. 1 runs the two back to back): while the final scores are still in registers the score
 * kernels count the selection's first radix digit, so that the selection needs neither its clearing
 * launch nor its first pass over the scores nor the grid-wide wait behind that pass.  Results of both
 * calls are unchanged bit for bit.
 *
 *   select_workspace  device, 256-byte aligned, laid out as for lava_select_topk_batch with `batch`
 *                     problems and max_total_entries = H_kv * max_b N_b (for batch = 1 that is the
 *                     workspace of lava_select_topk for H_kv * N entries): region b belongs to
 *                     sequence b.  Too small -> LAVA_ERR_WORKSPACE.
 * Afterwards rank sequence b's scores ([H_kv][N_b], equal segments, all H_kv * N_b entries) ONCE with
 * lava_select_topk_primed, or with lava_select_topk_batch where problem b has primed = 1 and
 * max_total_entries is the same H_kv * max_b N_b.  A prepared region is used up by that selection; a
 * selection with primed = 0 ignores what was prepared and clears the region itself.
 */
int32_t lava_window_scores_primed(const lava_layer_desc* desc, int32_t batch, const int64_t* seq_lens,
                                  const void* q_win, const void* k, const void* v, const float* lse,
                                  float* scores, float* vbar, float* layer_stat, void* workspace,
                                  size_t workspace_bytes, void* select_workspace,
                                  size_t select_workspace_bytes, void* hip_stream);

/*
 * Budgets formed by the scores call itself (Alg. 2 computes them from the statistic the scores have
 * just produced; the workgroup that forms e_l goes on to run the budget rule, which saves the small
 * launch of lava_layer_budgets).  All pointers are device memory; sequence b uses row b of each table.
 *
 *   n_layers   layers that share each sequence's total, this call's layer included; 1..128
 *              (LAVA_PLAN_MAX_LAYERS; deeper stacks call lava_layer_budgets)
 *   layer      0 <= layer < n_layers: the column of `e` this call's statistic belongs to
 *   e          [batch][n_layers] float   statistics; the call writes column `layer` (the same value
 *                                        as layer_stat[b]) and reads the other columns
 *   total      [batch] int64             total budget of each sequence
 *   lo, hi     [batch][n_layers] int64   bounds, as for lava_layer_budgets
 *   budgets    [batch][n_layers] int64   out: exactly what lava_layer_budgets(on_device = 1) returns
 *                                        for these tables, -1 everywhere for infeasible bounds
 */
#define LAVA_PLAN_MAX_LAYERS 128
typedef struct lava_budget_plan {
  int32_t n_layers;
  int32_t layer;
  float* e;
  const int64_t* total;
  const int64_t* lo;
  const int64_t* hi;
  int64_t* budgets;
} lava_budget_plan;

/*
 * lava_window_scores with both optional extras: select_workspace as for lava_window_scores_primed
 * (NULL with 0 bytes: the selection is not prepared) and `plan` (NULL: no budgets).  A plan with
 * n_layers or layer out of range or a null table returns LAVA_ERR_INVALID_ARG.
 */
int32_t lava_window_scores_planned(const lava_layer_desc* desc, int32_t batch, const int64_t* seq_lens,
                                   const void* q_win, const void* k, const void* v, const float* lse,
                                   float* scores, float* vbar, float* layer_stat, void* workspace,
                                   size_t workspace_bytes, void* select_workspace,
                                   size_t select_workspace_bytes, const lava_budget_plan* plan,
                                   void* hip_stream);

/*
 * Layer budgets B_l = e_l / sum_l e_l * total (Alg. 2, inner loop) as integers.
 *
 *   e          [batch][n_layers] float   statistics of the layers prefilled so far
 *   total      [batch] int64             total budget of each sequence
 *   lo, hi     [batch][n_layers] int64   bounds of each layer's budget (H_kv * w and the
 *                                        number of entries the layer still holds)
 *   budgets    [batch][n_layers] int64   out; sums to total[b], lo <= B <= hi
 *
 * Rounding: real quotas are floored and the leftover units go to the largest fractional parts
 * (lower layer first on ties); layers that violate a bound are pinned to it and the remainder
 * is split again among the others.  All-zero statistics give a uniform split.
 *
 * on_device == 0: every pointer is host memory; pure host arithmetic, synchronous, the stream
 * is ignored; infeasible bounds (sum lo > total or sum hi < total) return LAVA_ERR_BUDGET.
 * on_device != 0: every pointer is device memory; one small kernel on the stream; a sequence
 * with infeasible bounds gets all budgets = -1.  n_layers <= 1024.
 * Calling it with n_layers = 1, 2, ... reproduces the cascade of Alg. 2.
 */
int32_t lava_layer_budgets(int32_t batch, int32_t n_layers, const float* e, const int64_t* total,
                           const int64_t* lo, const int64_t* hi, int64_t* budgets,
                           int32_t on_device, void* hip_stream);

/* Bytes of device workspace lava_select_topk needs for `total_entries` scores. */
size_t lava_select_workspace_bytes(int64_t total_entries);

/*
 * Top-`budget` selection over the concatenated per-head score segments of a layer (Alg. 1,
 * "B_l largest entries based on s_l").  An entry precedes another if its score is larger, or
 * the scores are equal and its flat index is smaller; the first `budget` entries survive.
 *
 *   scores        device float [total_entries], heads concatenated.  No NaN; -0 == +0.
 *   seg_offsets   device int64 [n_heads + 1] segment starts, or NULL for equal segments of
 *                 total_entries / n_heads.  With explicit segments the number of entries is
 *                 seg_offsets[n_heads] as read on the device (clamped to total_entries, which is
 *                 then an upper bound: it sizes the launch and the workspace), so that selections
 *                 can be chained without a host round trip
 *   budget        entries to keep, 0 <= budget <= total_entries; when budget_dev != NULL the
 *                 value is read on the device from *budget_dev instead (clamped to
 *                 [0, min(budget, total_entries)]) and `budget` is the capacity of the outputs
 *   head_counts   device int32 [n_heads]      survivors per head (the dynamic head budget)
 *   head_offsets  device int64 [n_heads + 1]  exclusive prefix sums of head_counts
 *   kept_idx      device int32 [budget]       position of each survivor inside its head,
 *                                             ascending per head, heads concatenated
 *   kept_scores   device float [budget] or NULL   the survivors' scores, same order (what a
 *                                             later re-selection with a smaller budget needs)
 * Integer-exact and deterministic.  n_heads <= 64, total_entries < 2^31.
 *
 * Up to half of the device's resident-workgroup capacity the selection is one launch whose
 * workgroups meet at grid-wide barriers with bounded waits.  If a wait ever gives up (the device
 * could not keep the workgroups resident together, e.g. because another stream held its compute
 * units), the call's results are replaced by an unmistakable mark before the kernel ends:
 * head_counts[h] = -1 for every head and head_offsets[0..n_heads] = 0, so that a compaction or a
 * decode step fed with them moves and reads nothing; lava_select_status reports it on the host.
 */
int32_t lava_select_topk(int32_t n_heads, const float* scores, const int64_t* seg_offsets,
                         int64_t total_entries, int64_t budget, const int64_t* budget_dev,
                         int32_t* head_counts, int64_t* head_offsets, int32_t* kept_idx,
                         float* kept_scores, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/* lava_select_topk over a score array whose workspace lava_window_scores_primed prepared (equal
 * segments of total_entries / n_heads; total_entries = H_kv * N of that sequence). */
int32_t lava_select_topk_primed(int32_t n_heads, const float* scores, int64_t total_entries, int64_t budget,
                                const int64_t* budget_dev, int32_t* head_counts, int64_t* head_offsets,
                                int32_t* kept_idx, float* kept_scores, void* workspace,
                                size_t workspace_bytes, void* hip_stream);

/*
 * Synchronises the stream and reports whether the last lava_select_topk that used `workspace`
 * (with the same total_entries) completed normally.  The selection meets at grid-wide barriers
 * whose waits are bounded; LAVA_ERR_HIP means a wait gave up (the device could not keep the
 * kernel's workgroups resident together) and the outputs of that call must not be used.
 */
int32_t lava_select_status(const void* workspace, int64_t total_entries, void* hip_stream);

/*
 * lava_select_topk without a workspace argument, for callers that cannot allocate device memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same results bit for bit, same kernels; the selection's scratch memory (histograms,
 * barrier counter, per-workgroup counts) is a fixed array of about 1 MiB inside the library's
 * device image, which every GPU the library runs on holds until the process ends.  The call
 * allocates and frees nothing.
 *   total_entries <= LAVA_SELECT_STATIC_MAX_ENTRIES, else LAVA_ERR_WORKSPACE (nothing launched).
 * All calls on one GPU share that GPU's array (it is cleared by the call's own first kernel, so
 * a call does not depend on what the previous one left): calls that overlap in time on one GPU,
 * on different streams or from different threads, race and must be serialised by the caller.
 * A failed bounded wait cannot be queried with lava_select_status for this variant (there is no
 * workspace to pass); the outputs carry the mark described for lava_select_topk.
 */
#define LAVA_SELECT_STATIC_MAX_ENTRIES ((int64_t)1 << 22)
int32_t lava_select_topk_static(int32_t n_heads, const float* scores, const int64_t* seg_offsets,
                                int64_t total_entries, int64_t budget, const int64_t* budget_dev,
                                int32_t* head_counts, int64_t* head_offsets, int32_t* kept_idx,
                                float* kept_scores, void* hip_stream);

/*
 * Packed surviving rows (Alg. 1: K^ = K (.) I, V^ = V (.) I, stored without the evicted rows):
 *   k_out[head_offsets[g] + t][:] = k[g][kept_idx[head_offsets[g] + t]][:], same for v.
 *
 *   k, v          device [H_kv][n][d_h]   one sequence's layer cache
 *   head_offsets  device int64 [H_kv + 1], kept_idx device int32 [>= head_offsets[H_kv]]
 *   capacity      rows available in k_out / v_out; rows beyond head_offsets[H_kv] are left
 *                 untouched, and no more than `capacity` rows are ever written
 *   k_out, v_out  device [capacity][d_h], dtype of the descriptor; bit copies of the rows
 */
int32_t lava_compact_kv(const lava_layer_desc* desc, int64_t n, const void* k, const void* v,
                        const int64_t* head_offsets, const int32_t* kept_idx, int64_t capacity,
                        void* k_out, void* v_out, void* hip_stream);

/*
 * The same gather from an already packed source: what a re-eviction of a compressed layer does
 * (Alg. 2, inner loop: layers below the one just prefilled are evicted again, from what they still
 * hold, with a smaller budget).
 *
 *   src_offsets   device int64 [H_kv + 1]: head g owns source rows src_offsets[g] .. src_offsets[g+1]-1
 *   src_rows      rows in the source pool; offsets beyond it are never followed
 *   k_src, v_src  device [src_rows][d_h];  pos_src device int32 [src_rows] or NULL
 *   head_offsets, kept_idx   as written by lava_select_topk run on the source's segments
 *                 (kept_idx counts from the start of the head's source segment)
 *   k_out, v_out  device [capacity][d_h]; pos_out device int32 [capacity] or NULL: the token
 *                 position of every surviving row (pos_src of its source row)
 * Out of place: outputs must not overlap the source.
 */
int32_t lava_compact_packed(const lava_layer_desc* desc, const int64_t* src_offsets, int64_t src_rows,
                            const void* k_src, const void* v_src, const int32_t* pos_src,
                            const int64_t* head_offsets, const int32_t* kept_idx, int64_t capacity,
                            void* k_out, void* v_out, int32_t* pos_out, void* hip_stream);

/*
 * Several independent selections / compactions in as few launches as the device allows: the layers
 * an outer iteration of Alg. 2 evicts again, or the sequences of a ragged batch (Alg. 1 per
 * sequence).  Each problem is exactly one lava_select_topk / lava_compact_packed call (same
 * meaning, layout and limits of every field); results are identical to calling them one by one.
 * The tables are host arrays, read during the call.  The optional *_offset_dev fields let a
 * problem's data start at a position inside its buffers that only the device knows (layers packed
 * back to back in one pool whose split was decided on the device); the caller guarantees that the
 * offsets, plus what the problem reads and writes, stay inside the buffers.
 */
typedef struct lava_select_problem {
  const float* scores;
  const int64_t* seg_offsets;   /* or NULL: equal segments                                     */
  int64_t total_entries;
  int64_t budget;
  const int64_t* budget_dev;    /* or NULL                                                     */
  int32_t* head_counts;
  int64_t* head_offsets;
  int32_t* kept_idx;
  float* kept_scores;           /* or NULL                                                     */
  const int64_t* in_offset_dev; /* or NULL: device int64, entries added to `scores` (the problem's
                                   scores start there)                                          */
  const int64_t* out_offset_dev;/* or NULL: device int64, entries added to kept_idx / kept_scores */
  int32_t* error_dev;           /* or NULL: device int32 set to 1 if this selection gave up at a
                                   bounded wait (never cleared by the library, so one word can
                                   collect the failures of many selections)                     */
  int32_t primed;               /* non-zero: this problem's workspace region was prepared by
                                   lava_window_scores_primed for exactly these scores (seg_offsets
                                   and in_offset_dev must be NULL)                              */
} lava_select_problem;

typedef struct lava_compact_problem {
  int64_t src_rows;             /* src_offsets != NULL: rows of the packed source pool;
                                   src_offsets == NULL: rows per head of a dense [H_kv][n] source */
  const int64_t* src_offsets;
  const void* k_src;
  const void* v_src;
  const int32_t* pos_src;       /* or NULL (dense source: the position is the index itself)    */
  const int64_t* head_offsets;
  const int32_t* kept_idx;
  int64_t capacity;
  void* k_out;
  void* v_out;
  int32_t* pos_out;             /* or NULL                                                     */
  const int64_t* src_offset_dev;/* or NULL: device int64, first row of a packed source inside
                                   k_src / v_src / pos_src (src_rows counts from their base)   */
  const int64_t* out_offset_dev;/* or NULL: device int64, first output row inside k_out / v_out /
                                   pos_out and first entry inside kept_idx (capacity counts from
                                   their base)                                                 */
} lava_compact_problem;

/* Workspace of a batch: n_problems regions, each sized for max_total_entries.  0 if invalid. */
size_t lava_select_batch_workspace_bytes(int32_t n_problems, int64_t max_total_entries);

/*
 * n_problems >= 1 selections with n_heads heads each.  max_total_entries >= every problem's
 * total_entries fixes the region size (problem p uses region p of the workspace).  Problems are
 * packed into one launch while their workgroups can be resident together, otherwise into several.
 */
int32_t lava_select_topk_batch(int32_t n_heads, int32_t n_problems, const lava_select_problem* problems,
                               int64_t max_total_entries, void* workspace, size_t workspace_bytes,
                               void* hip_stream);

/* lava_select_status over the regions of a batch: LAVA_ERR_HIP if any selection gave up. */
int32_t lava_select_batch_status(const void* workspace, int32_t n_problems, int64_t max_total_entries,
                                 void* hip_stream);

/* n_problems >= 1 compactions of layers of the descriptor's shape, one launch per 32 problems. */
int32_t lava_compact_batch(const lava_layer_desc* desc, int32_t n_problems,
                           const lava_compact_problem* problems, void* hip_stream);

/*
 * Algorithm 2 as a driver: the compressed caches of all layers between cascade steps.  Every
 * pointer is device memory owned by the caller.  The layers sit back to back in one pool ("arena")
 * of `capacity` rows: their sizes change at every step but always sum to at most the total budget,
 * so the whole state needs capacity >= total budget rows, whatever the number of layers.  A step
 * gathers every layer from the current arena into the other one (a re-eviction is out of place),
 * hence two arenas; `cur` (host) says which one holds the state.  K and V, which are nearly all of
 * the state's bytes, may instead share ONE arena: pass k[1] == k[0] and v[1] == v[0] and the step
 * moves the earlier layers' rows inside that arena (every surviving row moves towards the front or
 * stays, which makes that possible) at the price of one more launch per step; pos, scores,
 * head_offsets and layer_start stay double-buffered either way.
 *   layer t occupies arena rows layer_start[cur][t] .. layer_start[cur][t + 1] - 1; inside them
 *   head g owns rows head_offsets[cur][t][g] .. head_offsets[cur][t][g + 1] - 1 (relative to the
 *   layer's first row), in ascending token position.
 * lava_decode_attention reads a layer in place: k_hat / v_hat = the arena, head_offsets =
 * head_offsets[cur] + t * (H_kv + 1), seq_base = layer_start[cur] + t, rows_capacity = capacity.
 */
typedef struct lava_cascade_state {
  void* k[2];               /* [capacity][d_h] packed keys                                      */
  void* v[2];               /* [capacity][d_h] packed values                                    */
  int32_t* pos[2];          /* [capacity] token position of each retained row                   */
  float* scores[2];         /* [capacity] retained scores (what the next re-eviction ranks)     */
  int64_t* head_offsets[2]; /* [max_layers][H_kv + 1]                                           */
  int64_t* layer_start[2];  /* [max_layers + 1]                                                 */
  int32_t* head_counts;     /* [max_layers][H_kv] dynamic head budgets after the latest step    */
  int32_t* kept_idx;        /* [capacity] scratch                                               */
  int32_t* error;           /* [1] or NULL: set to 1 by any step one of whose selections gave up
                               at a bounded wait (that layer is then marked empty: head_counts
                               -1, no rows); never cleared by the library: the state is invalid
                               from then on, zero the word when the state is reset              */
  int64_t capacity;         /* rows per arena, >= total budget                                  */
  int32_t max_layers;
  int32_t cur;              /* 0 or 1; flipped by every lava_cascade_step                       */
} lava_cascade_state;

/*
 * Bytes of device workspace lava_cascade_step needs for up to n_layers layers of H_kv * n entries
 * and a total budget (all layers of a step are evicted by one batched selection, one workspace
 * region per layer).  Returns 0 for invalid arguments.
 */
size_t lava_cascade_workspace_bytes(const lava_layer_desc* desc, int64_t n, int32_t n_layers,
                                    int64_t total_budget);

/*
 * One outer iteration of Algorithm 2, after layer `layer` (0-based) has been prefilled and scored:
 *   budgets  B_t = e_t / sum_{t' <= layer} e_t' * total_budget for t = 0..layer (device, bounds
 *            H_kv * w and H_kv * n, rounding as lava_layer_budgets); the budget applied to a
 *            layer is min(B_t, entries it still holds)
 *   layer    first eviction of the new layer from its dense cache k_new, v_new [H_kv][n][d_h] by
 *            its scores [H_kv][n] (as written by lava_window_scores)
 *   t<layer  re-eviction of every earlier layer from what it holds, ranked by the scores it
 *            retained
 * All layers are written into the other arena, back to back in layer order; state->cur flips.
 *
 *   e        device float [>= layer + 1]: statistics of layers 0..layer (point layer_stat of
 *            lava_window_scores at e + layer)
 *   budgets  device int64 [>= layer + 1] out
 * Three launches (four with a shared K/V arena), whatever the number of layers; everything is enqueued on the stream, nothing
 * is read back.  Selection is integer-exact, rows are bit copies, so the state after every step
 * equals the literal algorithm's.  layer < state->max_layers; total_budget <= state->capacity and
 * within [H_kv * w, H_kv * n] * (layer + 1).
 */
int32_t lava_cascade_step(const lava_layer_desc* desc, int32_t layer, int64_t n, const void* k_new,
                          const void* v_new, const float* scores_new, const float* e,
                          int64_t total_budget, lava_cascade_state* state, int64_t* budgets,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of device workspace lava_decode_attention needs.  Returns 0 for invalid arguments. */
size_t lava_decode_workspace_bytes(const lava_layer_desc* desc, int32_t batch, int64_t rows_capacity,
                                   int64_t tail_len);

/*
 * The step after the path: attention of ONE new token per sequence over the compressed layer
 * cache (decoding step of Sec. 2, restricted to the retained entries, i.e. under the mask of
 * Sec. 3):  out[h] = Softmax(scale * q[h] K_g^T) V_g,  g = h / G, where K_g, V_g are the rows
 * head g retained, followed by the rows appended since the eviction (Cat[K, K^N] of Sec. 2).
 * It consumes the packed variable-length layout lava_select_topk / lava_compact_kv produce.
 *
 *   q             device [batch][H][d_h], dtype of the descriptor
 *   k_hat, v_hat  device, packed rows [..][d_h], dtype of the descriptor
 *   head_offsets  device int64 [batch][H_kv + 1]; head g of sequence b owns packed rows
 *                 base_b + head_offsets[b][g] .. base_b + head_offsets[b][g+1] - 1
 *   seq_base      device int64 [batch] first packed row of each sequence, or NULL for
 *                 base_b = b * rows_capacity
 *   rows_capacity upper bound of head_offsets[b][H_kv] for every b (>= 0)
 *   k_tail,v_tail device [batch][H_kv][tail_capacity][d_h] rows appended after the eviction, the
 *                 first tail_len of them valid; NULL when tail_len == 0
 *   out           device float [batch][H][d_h]
 *   lse           device float [batch][H] natural-log log-sum-exp of the scaled logits, or NULL
 *
 * A head without any row gives zeros (lse = -inf).  If a sequence's offsets exceed rows_capacity
 * its outputs are NaN.  fp32 accumulation, deterministic (fixed merge order).  Uses n_q_heads,
 * n_kv_heads (<= 64, G <= 8), head_dim, dtype and softmax_scale of the descriptor; window and
 * pool_kernel are ignored.
 */
int32_t lava_decode_attention(const lava_layer_desc* desc, int32_t batch, const void* q,
                              const void* k_hat, const void* v_hat, const int64_t* head_offsets,
                              const int64_t* seq_base, int64_t rows_capacity, const void* k_tail,
                              const void* v_tail, int64_t tail_len, int64_t tail_capacity,
                              float* out, float* lse, void* workspace, size_t workspace_bytes,
                              void* hip_stream);

/*
 * Per-kernel timing for benchmarks.  When enabled, every kernel the library launches is
 * bracketed by HIP events on the stream it is launched on.  lava_prof_read synchronises the
 * device and returns the accumulated time of kernel `id` since the last reset.  Kernel ids run
 * from 0 to lava_prof_kernel_count() - 1.  Not thread-safe; leave disabled in production.
 */
int32_t lava_prof_kernel_count(void);
const char* lava_prof_kernel_name(int32_t id);
int32_t lava_prof_enable(int32_t on);
int32_t lava_prof_reset(void);
int32_t lava_prof_read(int32_t id, double* total_ms, int64_t* launches);

/*
 * Measurement aid: a plain streaming kernel over `bytes` (multiple of 16) of device memory, used
 * to calibrate the profiler's HBM byte counters and to measure the streaming ceiling the sweep
 * kernels are compared with.  mode 0: copy src -> dst (both `bytes` long); mode 1: read src only
 * (dst: at least 4 bytes, effectively never written).  `blocks` workgroups of 256 lanes.
 */
int32_t lava_probe_stream(const void* src, void* dst, int64_t bytes, int32_t mode, int32_t blocks,
                          void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LAVA_H */
