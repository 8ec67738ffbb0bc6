// C ABI of the library: argument checks on the host, then kernel launches on the caller's
// stream.  Nothing here allocates device memory.
#include <string.h>

#include <vector>

#include "budget_wave.h"
#include "common.h"

namespace lava {

// ------------------------------------------------------------------ per-kernel timing hook
namespace {
struct ProfState {
  bool enabled = false;
  std::vector<hipEvent_t> start[KID_COUNT], stop[KID_COUNT];
  size_t used[KID_COUNT] = {};
  double total_ms[KID_COUNT] = {};
  int64_t launches[KID_COUNT] = {};
} g_prof;

const char* const kKernelNames[KID_COUNT] = {
    "vnorm", "stats", "scores", "sweep", "prepass", "poolstat", "sel_init", "sel_fused", "sel_steps", "compact", "budgets",
    "decode", "decode_merge"};

void prof_collect() {
  (void)hipDeviceSynchronize();
  for (int k = 0; k < KID_COUNT; ++k) {
    for (size_t i = 0; i < g_prof.used[k]; ++i) {
      float ms = 0.0f;
      if (hipEventElapsedTime(&ms, g_prof.start[k][i], g_prof.stop[k][i]) == hipSuccess) {
        g_prof.total_ms[k] += ms;
        g_prof.launches[k] += 1;
      }
    }
    g_prof.used[k] = 0;
  }
}
}  // namespace

void prof_begin(int kid, hipStream_t s) {
  if (!g_prof.enabled) return;
  if (g_prof.used[kid] == g_prof.start[kid].size()) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
    g_prof.start[kid].push_back(a);
    g_prof.stop[kid].push_back(b);
  }
  (void)hipEventRecord(g_prof.start[kid][g_prof.used[kid]], s);
}

void prof_end(int kid, hipStream_t s) {
  if (!g_prof.enabled) return;
  if (g_prof.used[kid] >= g_prof.start[kid].size()) return;
  (void)hipEventRecord(g_prof.stop[kid][g_prof.used[kid]], s);
  g_prof.used[kid] += 1;
  if (g_prof.used[kid] >= 4096) prof_collect();   // bound the number of live events
}

// ------------------------------------------------------------------ launch-shape tuning
namespace {
lava_tuning g_tuning = {};
}
const lava_tuning& tuning() { return g_tuning; }

// ------------------------------------------------------------------ descriptor checks
static int32_t check_desc(const lava_layer_desc* d) {
  if (d == nullptr) return LAVA_ERR_INVALID_ARG;
  if (d->dtype != LAVA_F32 && d->dtype != LAVA_BF16) return LAVA_ERR_INVALID_ARG;
  if (d->n_q_heads < 1 || d->n_kv_heads < 1 || d->window < 1 || d->pool_kernel < 1)
    return LAVA_ERR_INVALID_ARG;
  if (!(d->softmax_scale >= 0.0f) || d->softmax_scale > 1e30f) return LAVA_ERR_INVALID_ARG;
  if (d->score_kind < LAVA_SCORE_LAVA || d->score_kind > LAVA_SCORE_TOKEN_NORM) return LAVA_ERR_INVALID_ARG;
  if (d->n_q_heads % d->n_kv_heads != 0) return LAVA_ERR_SHAPE;
  if (d->n_q_heads / d->n_kv_heads > 16 || d->n_kv_heads > 64) return LAVA_ERR_SHAPE;
  if (d->head_dim != 64 && d->head_dim != 128) return LAVA_ERR_SHAPE;
  if (d->window > 64) return LAVA_ERR_SHAPE;
  if (d->pool_kernel % 2 == 0 || d->pool_kernel > 15) return LAVA_ERR_SHAPE;
  return LAVA_OK;
}

int32_t check_select_problem(int32_t n_heads, const lava_select_problem& p) {
  if (p.scores == nullptr || p.head_counts == nullptr || p.head_offsets == nullptr || p.kept_idx == nullptr ||
      p.total_entries < 1)
    return LAVA_ERR_INVALID_ARG;
  if (p.total_entries >= (int64_t)1 << 31) return LAVA_ERR_SHAPE;
  if (p.seg_offsets == nullptr && p.total_entries % n_heads != 0) return LAVA_ERR_SHAPE;
  if (p.budget < 0 || p.budget > p.total_entries) return LAVA_ERR_BUDGET;
  // a prepared workspace holds the histogram of a whole score array as lava_window_scores_primed wrote it
  if (p.primed != 0 && (p.seg_offsets != nullptr || p.in_offset_dev != nullptr)) return LAVA_ERR_INVALID_ARG;
  return LAVA_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace lava

using namespace lava;

extern "C" {

const char* lava_status_string(int32_t status) {
  switch (status) {
    case LAVA_OK: return "ok";
    case LAVA_ERR_INVALID_ARG: return "invalid argument";
    case LAVA_ERR_SHAPE: return "unsupported shape";
    case LAVA_ERR_BUDGET: return "budget out of range";
    case LAVA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case LAVA_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int32_t lava_set_tuning(const lava_tuning* t) {
  if (t == nullptr) {
    g_tuning = lava_tuning{};
    return LAVA_OK;
  }
  if (t->sweep_shape < 0 || t->sweep_shape > 2 || t->sweep_schedule < 0 || t->sweep_schedule > 3 ||
      t->sweep_workgroups < 0 || t->sweep_workgroups > 65536 || t->barrier_spin_limit < 0 ||
      (t->decode_rows_per_unit != 0 && (t->decode_rows_per_unit < 128 || t->decode_rows_per_unit > 8192)) ||
      t->sweep_orphan_units < 0 || t->reserved[0] != 0 || t->reserved[1] != 0)
    return LAVA_ERR_INVALID_ARG;
  g_tuning = *t;
  return LAVA_OK;
}

int32_t lava_get_tuning(lava_tuning* t) {
  if (t == nullptr) return LAVA_ERR_INVALID_ARG;
  *t = g_tuning;
  return LAVA_OK;
}

size_t lava_window_scores_workspace_bytes(const lava_layer_desc* desc, int32_t batch,
                                          int64_t total_tokens) {
  if (check_desc(desc) != LAVA_OK || batch < 1 || total_tokens <= desc->window) return 0;
  // the longest sequence the batch can contain bounds every sequence's region (the size of a region
  // never shrinks with the length)
  const int64_t max_n = total_tokens - (int64_t)(batch - 1) * (desc->window + 1);
  if (max_n <= desc->window) return 0;
  const size_t region = make_score_workspace(*desc, max_n).bytes;
  // sequences of a batch are swept together, each in its own region; when a KV group has to be
  // split into chunks they are processed one after another and share one region
  return make_sweep_plan(*desc, max_n).fused_pool ? region * (size_t)batch : region;
}

// lava_window_scores, optionally preparing a selection workspace (select_ws != null) for the selections
// that will rank the scores it writes.
static int32_t window_scores(const lava_layer_desc* desc, int32_t batch, const int64_t* seq_lens,
                             const void* q_win, const void* k, const void* v, const float* lse,
                             float* scores, float* vbar, float* layer_stat, void* workspace,
                             size_t workspace_bytes, void* select_ws, size_t select_ws_bytes, bool primed,
                             const lava_budget_plan* budget_plan, void* hip_stream) {
  int32_t st = check_desc(desc);
  if (st != LAVA_OK) return st;
  if (budget_plan != nullptr &&
      (budget_plan->n_layers < 1 || budget_plan->n_layers > LAVA_PLAN_MAX_LAYERS || budget_plan->layer < 0 ||
       budget_plan->layer >= budget_plan->n_layers || budget_plan->e == nullptr || budget_plan->total == nullptr ||
       budget_plan->lo == nullptr || budget_plan->hi == nullptr || budget_plan->budgets == nullptr))
    return LAVA_ERR_INVALID_ARG;
  if (batch < 1 || seq_lens == nullptr || q_win == nullptr || k == nullptr || v == nullptr ||
      scores == nullptr || vbar == nullptr || layer_stat == nullptr)
    return LAVA_ERR_INVALID_ARG;
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(v)) return LAVA_ERR_INVALID_ARG;
  int64_t max_n = 0;
  for (int b = 0; b < batch; ++b) {
    if (seq_lens[b] <= desc->window) return LAVA_ERR_SHAPE;
    if (seq_lens[b] >= (int64_t)1 << 31) return LAVA_ERR_SHAPE;
    if (seq_lens[b] > max_n) max_n = seq_lens[b];
  }
  const lava_layer_desc& d = *desc;
  const SweepPlan plan_max = make_sweep_plan(d, max_n);
  const ScoreWorkspace region = make_score_workspace(d, max_n);
  const bool together = plan_max.fused_pool;                 // property of the descriptor, not of the length
  const size_t need = together ? region.bytes * (size_t)batch : region.bytes;
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 ||
      workspace_bytes < need)
    return LAVA_ERR_WORKSPACE;
  SelectWorkspace sel_layout = {};
  if (primed) {
    if ((int64_t)desc->n_kv_heads * max_n >= (int64_t)1 << 31) return LAVA_ERR_SHAPE;
    sel_layout = make_select_workspace((int64_t)desc->n_kv_heads * max_n);
    if (select_ws == nullptr || (reinterpret_cast<uintptr_t>(select_ws) % kAlign) != 0 ||
        select_ws_bytes < sel_layout.bytes * (size_t)batch)
      return LAVA_ERR_WORKSPACE;
  }

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  discard_stale_error();
  SweepArgs a;
  a.sel_ws = primed ? static_cast<char*>(select_ws) : nullptr;
  a.sel_stride = sel_layout.bytes;
  a.sel_off_hist = sel_layout.off_hist;
  a.sel_off_state = sel_layout.off_state;
  a.plan = BudgetPlanArgs{};
  if (budget_plan != nullptr)
    a.plan = BudgetPlanArgs{budget_plan->e,  budget_plan->total,    budget_plan->lo,   budget_plan->hi,
                            budget_plan->budgets, budget_plan->n_layers, budget_plan->layer};
  a.q_win = q_win;
  a.k = k;
  a.v = v;
  a.lse = lse;
  a.scores = scores;
  a.vbar = vbar;
  a.layer_stat = layer_stat;
  a.ws = static_cast<char*>(workspace);
  a.off_stat_part = region.off_stat_part;
  a.off_vnorm_part = region.off_vnorm_part;
  a.off_sraw = region.off_sraw;
  a.off_ent_part = region.off_ent_part;
  a.off_counter = region.off_counter;
  a.H = d.n_q_heads;
  a.H_kv = d.n_kv_heads;
  a.w = d.window;
  a.bph = sweep_blocks_per_head(d);
  a.G = (d.n_q_heads / d.n_kv_heads) * a.bph;
  a.n_chunks = plan_max.n_chunks;
  a.pool_half = d.pool_kernel / 2;
  a.token_norm = d.score_kind == LAVA_SCORE_TOKEN_NORM ? 1 : 0;
  a.c2 = sweep_exp2_scale(d);

  const int per_launch = together ? kMaxSeqPerLaunch : 1;
  int64_t tok = 0;
  for (int b0 = 0; b0 < batch; b0 += per_launch) {
    a.first_seq = b0;
    a.n_seq = batch - b0 < per_launch ? batch - b0 : per_launch;
    int max_bx = 0, max_vb = 0;
    SweepPlan plan = plan_max;
    int64_t launch_tokens = 0;
    for (int i = 0; i < a.n_seq; ++i) launch_tokens += seq_lens[b0 + i];
    // Several sequences whose workgroups do not all fit on the device at once: the narrow shape
    // (two workgroups per CU, out of phase) hides the per-workgroup set-up that a launch of
    // several rounds of one-per-CU workgroups would pay once per round.
    bool narrow = false;
    if (a.n_seq > 1) {
      int64_t wide_wgs = 0;
      for (int i = 0; i < a.n_seq; ++i)
        wide_wgs += (int64_t)make_sweep_plan(d, seq_lens[b0 + i], launch_tokens).blocks_x * d.n_kv_heads * plan_max.n_chunks;
      narrow = wide_wgs > sweep_device_wgs();
    }
    if (tuning().sweep_shape == 1) narrow = false;           // forced by the caller's tuning
    else if (tuning().sweep_shape == 2) narrow = true;
    SweepPlan plan_launch = plan_max;
    plan_launch.narrow = narrow && sweep_has_narrow_shape(d);
    for (int i = 0; i < a.n_seq; ++i) {
      const int64_t n = seq_lens[b0 + i];
      plan = make_sweep_plan(d, n, launch_tokens, narrow);
      SweepSeq& sq = a.s[i];
      sq.n = n;
      sq.tok = tok;
      sq.ws_off = together ? (long long)(region.bytes * (size_t)(b0 + i)) : 0;
      sq.blocks_x = plan.blocks_x;
      sq.tiles_per_block = plan.tiles_per_block;
      sq.vnorm_blocks = plan.vnorm_blocks;
      sq.vnorm_tiles_per_block = plan.vnorm_tiles_per_block;
      if (plan.blocks_x > max_bx) max_bx = plan.blocks_x;
      if (plan.vnorm_blocks > max_vb) max_vb = plan.vnorm_blocks;
      tok += n;
    }
    // Statistics and scores: two launches, or (when the caller's tuning asks for it, all heads of a group
    // fit one workgroup and the statistics pass is needed) one persistent launch that runs both passes.
    // The persistent launch measured a few per cent slower on this device, so it is not the default.
    const bool persistent = together && lse == nullptr && a.bph == 1 && tuning().sweep_schedule == 2;
    // Value norms: a launch of their own, or, where a statistics launch follows anyway, inside it (its
    // workgroups sweep the value rows of their span before the keys: one launch fewer).  Measured: a gain
    // for one sequence per launch (4 % of the whole path at 32K tokens, none at 128K), a loss of about 3 %
    // for a launch of many sequences, whose value norms do better with their own, finer cut.
    const bool prepass = lse == nullptr && !persistent && d.score_kind != LAVA_SCORE_ATTENTION &&
                         (tuning().sweep_schedule == 3 || (tuning().sweep_schedule == 0 && a.n_seq == 1));
    if (prepass) {
      for (int i = 0; i < a.n_seq; ++i) {
        a.s[i].vnorm_blocks = a.s[i].blocks_x;
        a.s[i].vnorm_tiles_per_block = a.s[i].tiles_per_block;
      }
    } else {
      st = d.score_kind == LAVA_SCORE_ATTENTION ? launch_unit_vnorm(d, a, max_vb, s) : launch_vnorm(d, a, max_vb, s);
      if (st != LAVA_OK) return st;
    }
    if (persistent) {
      int units = 0;
      for (int i = 0; i < a.n_seq; ++i) {
        a.s[i].unit_base = units;
        units += d.n_kv_heads * a.s[i].blocks_x;
      }
      a.n_units = units;
      a.spin_limit = tuning().barrier_spin_limit > 0 ? (unsigned int)tuning().barrier_spin_limit : 1u << 18;
      a.help_after = a.spin_limit / 4 < 64u ? (a.spin_limit / 4 > 0u ? a.spin_limit / 4 : 1u) : 64u;
      a.orphan_mod = tuning().sweep_orphan_units;
      st = launch_sweep(d, a, plan_launch, s);
      if (st != LAVA_OK) return st;
      continue;
    }
    if (lse == nullptr) {
      st = launch_stats(d, a, max_bx, plan_launch, prepass, s);
      if (st != LAVA_OK) return st;
    }
    st = launch_scores(d, a, max_bx, plan_launch, s);
    if (st != LAVA_OK) return st;
    if (!together) {                                         // one sequence: `plan` is its plan
      const SweepSeq& sq = a.s[0];
      char* reg = a.ws + sq.ws_off;
      st = launch_poolstat(d, sq.n, reinterpret_cast<const float*>(reg + a.off_sraw),
                           reinterpret_cast<const float*>(reg + a.off_vnorm_part), sq.vnorm_blocks,
                           scores + (size_t)d.n_kv_heads * sq.tok, vbar + (size_t)b0 * d.n_kv_heads,
                           layer_stat + b0, reinterpret_cast<double2*>(reg + a.off_ent_part),
                           reinterpret_cast<uint32_t*>(reg + a.off_counter),
                           a.sel_ws ? reinterpret_cast<unsigned int*>(a.sel_ws + (size_t)b0 * a.sel_stride + a.sel_off_hist)
                                    : nullptr,
                           a.plan, b0, s);
      if (st != LAVA_OK) return st;
    }
  }
  return LAVA_OK;
}

int32_t lava_window_scores(const lava_layer_desc* desc, int32_t batch, const int64_t* seq_lens,
                           const void* q_win, const void* k, const void* v, const float* lse,
                           float* scores, float* vbar, float* layer_stat, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  return window_scores(desc, batch, seq_lens, q_win, k, v, lse, scores, vbar, layer_stat, workspace, workspace_bytes,
                       nullptr, 0, false, nullptr, hip_stream);
}

int32_t lava_window_scores_primed(const lava_layer_desc* desc, int32_t batch, const int64_t* seq_lens,
                                  const void* q_win, const void* k, const void* v, const float* lse,
                                  float* scores, float* vbar, float* layer_stat, void* workspace,
                                  size_t workspace_bytes, void* select_workspace, size_t select_workspace_bytes,
                                  void* hip_stream) {
  return window_scores(desc, batch, seq_lens, q_win, k, v, lse, scores, vbar, layer_stat, workspace, workspace_bytes,
                       select_workspace, select_workspace_bytes, true, nullptr, hip_stream);
}

int32_t lava_window_scores_planned(const lava_layer_desc* desc, int32_t batch, const int64_t* seq_lens,
                                   const void* q_win, const void* k, const void* v, const float* lse,
                                   float* scores, float* vbar, float* layer_stat, void* workspace,
                                   size_t workspace_bytes, void* select_workspace, size_t select_workspace_bytes,
                                   const lava_budget_plan* plan, void* hip_stream) {
  static_assert(LAVA_PLAN_MAX_LAYERS == kMaxPlannedLayers, "header and kernels agree on the plan's depth");
  const bool primed = select_workspace != nullptr || select_workspace_bytes != 0;
  return window_scores(desc, batch, seq_lens, q_win, k, v, lse, scores, vbar, layer_stat, workspace, workspace_bytes,
                       select_workspace, select_workspace_bytes, primed, plan, hip_stream);
}

int32_t lava_layer_budgets(int32_t batch, int32_t n_layers, const float* e, const int64_t* total,
                           const int64_t* lo, const int64_t* hi, int64_t* budgets,
                           int32_t on_device, void* hip_stream) {
  if (batch < 1 || n_layers < 1 || e == nullptr || total == nullptr || lo == nullptr ||
      hi == nullptr || budgets == nullptr)
    return LAVA_ERR_INVALID_ARG;
  if (n_layers > 1024) return LAVA_ERR_SHAPE;
  if (on_device) discard_stale_error();
  if (on_device)
    return launch_budgets(batch, n_layers, e, total, lo, hi, budgets,
                          static_cast<hipStream_t>(hip_stream));
  return budgets_host(batch, n_layers, e, total, lo, hi, budgets);
}

size_t lava_select_workspace_bytes(int64_t total_entries) {
  if (total_entries < 1 || total_entries >= (int64_t)1 << 31) return 0;
  return make_select_workspace(total_entries).bytes;
}

size_t lava_select_batch_workspace_bytes(int32_t n_problems, int64_t max_total_entries) {
  if (n_problems < 1 || max_total_entries < 1 || max_total_entries >= (int64_t)1 << 31) return 0;
  return make_select_workspace(max_total_entries).bytes * (size_t)n_problems;
}

int32_t lava_select_topk_batch(int32_t n_heads, int32_t n_problems, const lava_select_problem* problems,
                               int64_t max_total_entries, void* workspace, size_t workspace_bytes,
                               void* hip_stream) {
  if (n_heads < 1 || n_problems < 1 || problems == nullptr || max_total_entries < 1) return LAVA_ERR_INVALID_ARG;
  if (n_heads > 64 || max_total_entries >= (int64_t)1 << 31) return LAVA_ERR_SHAPE;
  for (int p = 0; p < n_problems; ++p) {
    const int32_t st = check_select_problem(n_heads, problems[p]);
    if (st != LAVA_OK) return st;
    if (problems[p].total_entries > max_total_entries) return LAVA_ERR_SHAPE;
  }
  const size_t need = make_select_workspace(max_total_entries).bytes * (size_t)n_problems;
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < need)
    return LAVA_ERR_WORKSPACE;
  discard_stale_error();
  return launch_select_batch(n_heads, n_problems, problems, max_total_entries, workspace,
                             static_cast<hipStream_t>(hip_stream));
}

int32_t lava_select_topk(int32_t n_heads, const float* scores, const int64_t* seg_offsets,
                         int64_t total_entries, int64_t budget, const int64_t* budget_dev,
                         int32_t* head_counts, int64_t* head_offsets, int32_t* kept_idx,
                         float* kept_scores, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  if (n_heads < 1) return LAVA_ERR_INVALID_ARG;
  const lava_select_problem p = {scores,      seg_offsets,  total_entries, budget,     budget_dev,
                                 head_counts, head_offsets, kept_idx,      kept_scores, nullptr, nullptr, nullptr, 0};
  return lava_select_topk_batch(n_heads, 1, &p, total_entries, workspace, workspace_bytes, hip_stream);
}

int32_t lava_select_topk_primed(int32_t n_heads, const float* scores, int64_t total_entries, int64_t budget,
                                const int64_t* budget_dev, int32_t* head_counts, int64_t* head_offsets,
                                int32_t* kept_idx, float* kept_scores, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
  if (n_heads < 1) return LAVA_ERR_INVALID_ARG;
  const lava_select_problem p = {scores,      nullptr,      total_entries, budget,      budget_dev,
                                 head_counts, head_offsets, kept_idx,      kept_scores, nullptr, nullptr, nullptr, 1};
  return lava_select_topk_batch(n_heads, 1, &p, total_entries, workspace, workspace_bytes, hip_stream);
}

int32_t lava_select_batch_status(const void* workspace, int32_t n_problems, int64_t max_total_entries,
                                 void* hip_stream) {
  if (workspace == nullptr || n_problems < 1 || max_total_entries < 1 || max_total_entries >= (int64_t)1 << 31)
    return LAVA_ERR_INVALID_ARG;
  int flag = 0;
  const int32_t st = select_error_flag(workspace, max_total_entries, n_problems,
                                       static_cast<hipStream_t>(hip_stream), &flag);
  if (st != LAVA_OK) return st;
  return flag ? LAVA_ERR_HIP : LAVA_OK;
}

int32_t lava_select_status(const void* workspace, int64_t total_entries, void* hip_stream) {
  return lava_select_batch_status(workspace, 1, total_entries, hip_stream);
}

static int32_t check_compact_problem(const lava_layer_desc& d, const lava_compact_problem& p) {
  if (p.k_src == nullptr || p.v_src == nullptr || p.head_offsets == nullptr || p.kept_idx == nullptr ||
      p.k_out == nullptr || p.v_out == nullptr || p.src_rows < 1 || p.capacity < 0)
    return LAVA_ERR_INVALID_ARG;
  if (!aligned16(p.k_src) || !aligned16(p.v_src) || !aligned16(p.k_out) || !aligned16(p.v_out))
    return LAVA_ERR_INVALID_ARG;
  const int64_t rows = p.src_offsets ? p.src_rows : (int64_t)d.n_kv_heads * p.src_rows;
  if (p.capacity > rows) return LAVA_ERR_BUDGET;
  return LAVA_OK;
}

int32_t lava_compact_batch(const lava_layer_desc* desc, int32_t n_problems,
                           const lava_compact_problem* problems, void* hip_stream) {
  int32_t st = check_desc(desc);
  if (st != LAVA_OK) return st;
  if (n_problems < 1 || problems == nullptr) return LAVA_ERR_INVALID_ARG;
  for (int p = 0; p < n_problems; ++p) {
    st = check_compact_problem(*desc, problems[p]);
    if (st != LAVA_OK) return st;
  }
  discard_stale_error();
  return launch_compact_batch(*desc, n_problems, problems, static_cast<hipStream_t>(hip_stream));
}

int32_t lava_compact_kv(const lava_layer_desc* desc, int64_t n, const void* k, const void* v,
                        const int64_t* head_offsets, const int32_t* kept_idx, int64_t capacity,
                        void* k_out, void* v_out, void* hip_stream) {
  const lava_compact_problem p = {n, nullptr, k, v, nullptr, head_offsets, kept_idx, capacity, k_out, v_out, nullptr};
  return lava_compact_batch(desc, 1, &p, hip_stream);
}

int32_t lava_compact_packed(const lava_layer_desc* desc, const int64_t* src_offsets, int64_t src_rows,
                            const void* k_src, const void* v_src, const int32_t* pos_src,
                            const int64_t* head_offsets, const int32_t* kept_idx, int64_t capacity,
                            void* k_out, void* v_out, int32_t* pos_out, void* hip_stream) {
  const int32_t st = check_desc(desc);
  if (st != LAVA_OK) return st;
  if (src_offsets == nullptr) return LAVA_ERR_INVALID_ARG;
  const lava_compact_problem p = {src_rows, src_offsets, k_src, v_src, pos_src, head_offsets,
                                  kept_idx, capacity,    k_out, v_out, pos_out};
  return lava_compact_batch(desc, 1, &p, hip_stream);
}

// Entries a layer can hold when a step starts: the dense layer, or at most the whole budget.
static int64_t cascade_layer_bound(int64_t dense, int64_t total_budget) {
  return total_budget < dense ? total_budget : dense;
}

size_t lava_cascade_workspace_bytes(const lava_layer_desc* desc, int64_t n, int32_t n_layers, int64_t total_budget) {
  if (check_desc(desc) != LAVA_OK || n <= desc->window || n_layers < 1 || n_layers > 1024 || total_budget < 1)
    return 0;
  const int64_t dense = (int64_t)desc->n_kv_heads * n;
  if (dense >= (int64_t)1 << 31) return 0;
  return make_select_workspace(dense).bytes * (size_t)n_layers + 2 * kAlign;   // + the in-place gather's barrier words
}

int32_t lava_cascade_step(const lava_layer_desc* desc, int32_t layer, int64_t n, const void* k_new,
                          const void* v_new, const float* scores_new, const float* e,
                          int64_t total_budget, lava_cascade_state* state, int64_t* budgets,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  int32_t st = check_desc(desc);
  if (st != LAVA_OK) return st;
  if (layer < 0 || k_new == nullptr || v_new == nullptr || scores_new == nullptr || e == nullptr ||
      state == nullptr || budgets == nullptr)
    return LAVA_ERR_INVALID_ARG;
  if (n <= desc->window || layer >= 1024) return LAVA_ERR_SHAPE;
  const int64_t dense = (int64_t)desc->n_kv_heads * n;
  if (dense >= (int64_t)1 << 31) return LAVA_ERR_SHAPE;
  const int64_t lo = (int64_t)desc->n_kv_heads * desc->window;
  if (total_budget < lo * (layer + 1) || total_budget > dense * (layer + 1)) return LAVA_ERR_BUDGET;
  if (!aligned16(k_new) || !aligned16(v_new)) return LAVA_ERR_INVALID_ARG;
  lava_cascade_state& S = *state;
  for (int i = 0; i < 2; ++i)
    if (S.k[i] == nullptr || S.v[i] == nullptr || S.pos[i] == nullptr || S.scores[i] == nullptr ||
        S.head_offsets[i] == nullptr || S.layer_start[i] == nullptr || !aligned16(S.k[i]) || !aligned16(S.v[i]))
      return LAVA_ERR_INVALID_ARG;
  if (S.head_counts == nullptr || S.kept_idx == nullptr || (S.cur != 0 && S.cur != 1) || S.max_layers < 1)
    return LAVA_ERR_INVALID_ARG;
  if (layer >= S.max_layers) return LAVA_ERR_SHAPE;
  if (S.capacity < total_budget || S.capacity >= (int64_t)1 << 31) return LAVA_ERR_BUDGET;
  // one arena for K and V (both pairs of pointers equal): the earlier layers are re-compacted in place
  const bool in_place = S.k[0] == S.k[1];
  if ((S.v[0] == S.v[1]) != in_place) return LAVA_ERR_INVALID_ARG;
  const int64_t bound = cascade_layer_bound(dense, total_budget);
  const size_t select_bytes = make_select_workspace(dense).bytes * (size_t)(layer + 1);
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 ||
      workspace_bytes < select_bytes + (in_place ? 2 * kAlign : 0))
    return LAVA_ERR_WORKSPACE;
  unsigned int* gather_sync = in_place ? reinterpret_cast<unsigned int*>(static_cast<char*>(workspace) + select_bytes) : nullptr;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  discard_stale_error();
  const int H1 = desc->n_kv_heads + 1;
  const int a = S.cur, b = 1 - S.cur;

  // budgets of the layers seen so far, and from them where every layer will start in the other arena
  // (its extra workgroups clear the regions of the step's selections and their survivor counts)
  const SelectWorkspace sel_layout = make_select_workspace(dense);
  const SelectRegions regions = {static_cast<char*>(workspace), sel_layout.bytes, sel_layout.off_hist,
                                 sel_layout.off_state, S.head_counts};
  st = launch_cascade_plan(layer + 1, desc->n_kv_heads, e, total_budget, lo, dense, bound, S.head_offsets[a],
                           budgets, S.layer_start[b], gather_sync, regions, s);
  if (st != LAVA_OK) return st;

  // One table of selections and one of compactions: every earlier layer from what it holds in the
  // current arena, ranked by the scores it retained, then the new layer from its dense cache.
  std::vector<lava_select_problem> sel(layer + 1);
  std::vector<lava_compact_problem> cmp(layer + 1);
  for (int t = 0; t <= layer; ++t) {
    int32_t* counts = S.head_counts + (size_t)t * desc->n_kv_heads;
    int64_t* offs_new = S.head_offsets[b] + (size_t)t * H1;
    const int64_t* start_new = S.layer_start[b] + t;
    if (t < layer) {
      const int64_t* offs_cur = S.head_offsets[a] + (size_t)t * H1;
      const int64_t* start_cur = S.layer_start[a] + t;
      sel[t] = {S.scores[a], offs_cur, bound,      bound,       budgets + t, counts,
                offs_new,    S.kept_idx, S.scores[b], start_cur, start_new, S.error, 0};
      cmp[t] = {S.capacity, offs_cur, S.k[a], S.v[a], S.pos[a],  offs_new,  S.kept_idx,
                S.capacity, S.k[b],   S.v[b], S.pos[b], start_cur, start_new};
    } else {
      sel[t] = {scores_new, nullptr,    dense,       bound,   budgets + t, counts,
                offs_new,   S.kept_idx, S.scores[b], nullptr, start_new, S.error, 0};
      cmp[t] = {n,          nullptr, k_new,  v_new,    nullptr, offs_new, S.kept_idx,
                S.capacity, S.k[b],  S.v[b], S.pos[b], nullptr, start_new};
    }
  }
  st = launch_select_batch(desc->n_kv_heads, layer + 1, sel.data(), dense, workspace, s, /*cleared=*/true);
  if (st != LAVA_OK) return st;
  if (in_place) {
    // the earlier layers move inside the arena first; the new layer's rows land behind them afterwards
    // (its place may still hold rows of the old layout until then)
    st = launch_compact_inplace(*desc, layer, S.layer_start[a], S.layer_start[b], S.head_offsets[a], S.head_offsets[b],
                                S.kept_idx, S.k[a], S.v[a], S.pos[a], S.pos[b], S.capacity, gather_sync, S.error, s);
    if (st != LAVA_OK) return st;
    st = launch_compact_batch(*desc, 1, &cmp[layer], s);
  } else {
    st = launch_compact_batch(*desc, layer + 1, cmp.data(), s);
  }
  if (st != LAVA_OK) return st;
  S.cur = b;
  return LAVA_OK;
}

// Descriptor checks for the decode step: window and pool_kernel play no role there.
static int32_t check_desc_decode(const lava_layer_desc* desc, lava_layer_desc* out) {
  if (desc == nullptr) return LAVA_ERR_INVALID_ARG;
  *out = *desc;
  out->window = 1;
  out->pool_kernel = 1;
  const int32_t st = check_desc(out);
  if (st != LAVA_OK) return st;
  return out->n_q_heads / out->n_kv_heads > 8 ? LAVA_ERR_SHAPE : LAVA_OK;   // the step's operand holds 8 heads of a group
}

size_t lava_decode_workspace_bytes(const lava_layer_desc* desc, int32_t batch, int64_t rows_capacity,
                                   int64_t tail_len) {
  lava_layer_desc d;
  if (check_desc_decode(desc, &d) != LAVA_OK || batch < 1 || rows_capacity < 0 || tail_len < 0) return 0;
  if (rows_capacity >= (int64_t)1 << 31 || tail_len >= (int64_t)1 << 31) return 0;
  return make_decode_plan(d, batch, rows_capacity, tail_len).bytes;
}

int32_t lava_decode_attention(const lava_layer_desc* desc, int32_t batch, const void* q,
                              const void* k_hat, const void* v_hat, const int64_t* head_offsets,
                              const int64_t* seq_base, int64_t rows_capacity, const void* k_tail,
                              const void* v_tail, int64_t tail_len, int64_t tail_capacity,
                              float* out, float* lse, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  lava_layer_desc d;
  int32_t st = check_desc_decode(desc, &d);
  if (st != LAVA_OK) return st;
  if (batch < 1 || q == nullptr || head_offsets == nullptr || out == nullptr || rows_capacity < 0 ||
      tail_len < 0 || tail_capacity < tail_len)
    return LAVA_ERR_INVALID_ARG;
  if (batch > 65535) return LAVA_ERR_SHAPE;
  if (rows_capacity >= (int64_t)1 << 31 || tail_len >= (int64_t)1 << 31) return LAVA_ERR_SHAPE;
  if (rows_capacity > 0 && (k_hat == nullptr || v_hat == nullptr)) return LAVA_ERR_INVALID_ARG;
  if (tail_len > 0 && (k_tail == nullptr || v_tail == nullptr)) return LAVA_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_hat) || !aligned16(v_hat) || !aligned16(k_tail) || !aligned16(v_tail))
    return LAVA_ERR_INVALID_ARG;
  const DecodePlan p = make_decode_plan(d, batch, rows_capacity, tail_len);
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 ||
      workspace_bytes < p.bytes)
    return LAVA_ERR_WORKSPACE;
  discard_stale_error();
  return launch_decode(d, batch, q, k_hat, v_hat, head_offsets, seq_base, rows_capacity, k_tail, v_tail,
                       tail_len, tail_capacity, out, lse, workspace, p, static_cast<hipStream_t>(hip_stream));
}

int32_t lava_prof_kernel_count(void) { return KID_COUNT; }

const char* lava_prof_kernel_name(int32_t id) {
  return (id >= 0 && id < KID_COUNT) ? kKernelNames[id] : "";
}

int32_t lava_prof_enable(int32_t on) {
  if (!on && g_prof.enabled) prof_collect();
  g_prof.enabled = on != 0;
  return LAVA_OK;
}

int32_t lava_prof_reset(void) {
  prof_collect();
  for (int k = 0; k < KID_COUNT; ++k) {
    g_prof.total_ms[k] = 0.0;
    g_prof.launches[k] = 0;
  }
  return LAVA_OK;
}

int32_t lava_prof_read(int32_t id, double* total_ms, int64_t* launches) {
  if (id < 0 || id >= KID_COUNT || total_ms == nullptr || launches == nullptr)
    return LAVA_ERR_INVALID_ARG;
  prof_collect();
  *total_ms = g_prof.total_ms[id];
  *launches = g_prof.launches[id];
  return LAVA_OK;
}

}  // extern "C"
