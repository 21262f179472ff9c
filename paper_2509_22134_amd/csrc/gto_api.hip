// C ABI of libgto: argument validation on the host, then kernel launches on the caller's
// stream.  No allocation, no synchronisation, no retained pointers.
#include <hip/hip_runtime.h>
#include <string.h>

#include <string>
#include <vector>

#include "../../include/gto.h"
#include "gto_kernels.h"

namespace {

thread_local std::string t_hip_error;

int hip_status() {
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) return GTO_OK;
  t_hip_error = std::string("HIP error: ") + hipGetErrorString(e);
  return GTO_E_HIP;
}

// ------------------------------------------------------------------------- profiling
struct ProfRecord {
  const char *name;
  hipEvent_t start, stop;
};
thread_local bool t_prof_on = false;
thread_local std::vector<ProfRecord> t_prof;

struct ProfScope {
  hipStream_t st;
  bool on;
  ProfRecord rec;
  ProfScope(const char *name, hipStream_t s) : st(s), on(t_prof_on) {
    if (!on) return;
    rec.name = name;
    (void)hipEventCreate(&rec.start);
    (void)hipEventCreate(&rec.stop);
    (void)hipEventRecord(rec.start, st);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(rec.stop, st);
    t_prof.push_back(rec);
  }
};

// ------------------------------------------------------------------------- validation
constexpr int kMaxK = 64, kMaxD = 32, kMaxPool = 4096;

int elem_size(int dtype) { return dtype == GTO_BF16 ? 2 : 4; }

int check_cfg(const gto_config *c, bool need_group) {
  if (!c) return GTO_E_NULL;
  if (c->dtype != GTO_BF16 && c->dtype != GTO_F32) return GTO_E_DTYPE;
  if (c->R < 1 || c->d < 1 || c->d > kMaxD || c->k < 1 || c->k > kMaxK || c->g < 1) return GTO_E_SHAPE;
  if (c->V < c->k || (int64_t)c->V > 2147483647ll - 65536ll) return GTO_E_SHAPE;
  const int64_t C = (int64_t)c->k + (int64_t)(c->d - 1) * c->k * c->k;
  if (C > kMaxPool) return GTO_E_SHAPE;
  if (c->row_stride < c->V) return GTO_E_SHAPE;
  const int64_t rho = 1 + (int64_t)(c->d - 1) * c->k;
  if ((int64_t)c->R * rho > 2147483647ll || (int64_t)c->R * c->d > 2147483647ll) return GTO_E_SHAPE;
  if ((c->row_stride * elem_size(c->dtype)) % 16 != 0) return GTO_E_ALIGN;
  if (c->reward_mode < GTO_REWARD_LSE || c->reward_mode > GTO_REWARD_NODESUM) return GTO_E_MODE;
  if (!(c->eta > 0.f) || !(c->eps >= 0.f) || !(c->delta >= 0.f)) return GTO_E_MODE;
  if (c->reserved != 0) return GTO_E_MODE;
  if (need_group && (c->group_size < 1 || c->R % c->group_size != 0)) return GTO_E_SHAPE;
  return GTO_OK;
}

int check_logits(const void *p) {
  if (!p) return GTO_E_NULL;
  if (reinterpret_cast<uintptr_t>(p) & 15) return GTO_E_ALIGN;
  return GTO_OK;
}

bool any_null(std::initializer_list<const void *> ps) {
  for (const void *p : ps)
    if (!p) return true;
  return false;
}

int pool_size(const gto_config *c) { return c->k + (c->d - 1) * c->k * c->k; }
int rows_per_root(const gto_config *c) { return 1 + (c->d - 1) * c->k; }

#define GTO_TRY(expr)             \
  do {                            \
    int _s = (expr);              \
    if (_s != GTO_OK) return _s;  \
  } while (0)

int check_draft_stats(const gto_draft_stats *s) {
  if (!s || any_null({s->row_max, s->row_lse, s->top_tok, s->top_logp})) return GTO_E_NULL;
  return GTO_OK;
}
int check_target_stats(const gto_target_stats *s) {
  if (!s || any_null({s->t_max, s->t_lse, s->t_argmax})) return GTO_E_NULL;
  return GTO_OK;
}
int check_pool(const gto_pool *p) {
  if (!p || any_null({p->cand_tok, p->cand_parent, p->cand_depth, p->cand_pslot, p->cand_slot, p->cand_score,
                      p->slot_cand}))
    return GTO_E_NULL;
  return GTO_OK;
}
int check_tree(const gto_tree *t) {
  if (!t || any_null({t->sel_cand, t->sel_tok, t->sel_parent, t->sel_depth, t->sel_pslot, t->sel_slot,
                      t->sel_leaf, t->sel_score, t->n_sel, t->slot_need}))
    return GTO_E_NULL;
  return GTO_OK;
}
int check_reward(const gto_reward *w) {
  if (!w || any_null({w->node_q, w->node_cum, w->reward, w->reward_aux, w->n_leaves, w->path_len,
                      w->path_node, w->path_slot}))
    return GTO_E_NULL;
  return GTO_OK;
}
int check_ppo(const gto_ppo *p) {
  if (!p || any_null({p->logM, p->logM0, p->ratio, p->term, p->active, p->coef, p->loss_group, p->loss}))
    return GTO_E_NULL;
  return GTO_OK;
}

// ------------------------------------------------------------------------- launch helpers
void run_draft_rows(const gto_config *c, const void *logits, const gto_draft_stats *s, hipStream_t st) {
  gto::RowStatsArgs a{};
  a.logits = logits;
  a.row_stride = c->row_stride;
  a.V = c->V; a.d = c->d; a.kslots = c->k; a.ktop = c->k; a.rho = rows_per_root(c);
  a.path_slot = nullptr;
  a.row_max = s->row_max; a.row_lse = s->row_lse; a.top_tok = s->top_tok; a.top_logp = s->top_logp;
  ProfScope ps("row_stats_draft", st);
  gto::launch_row_stats(a, c->dtype, c->R * a.rho, st);
}

void run_target_rows(const gto_config *c, const void *logits, const gto_target_stats *s,
                     const int32_t *row_need, hipStream_t st) {
  gto::RowStatsArgs a{};
  a.logits = logits;
  a.row_stride = c->row_stride;
  a.V = c->V; a.d = c->d; a.kslots = c->k; a.ktop = 1; a.rho = rows_per_root(c);
  a.path_slot = nullptr;
  a.row_need = row_need;
  a.row_max = s->t_max; a.row_lse = s->t_lse; a.top_tok = s->t_argmax; a.top_logp = nullptr;
  ProfScope ps("row_stats_target", st);
  gto::launch_row_stats(a, c->dtype, c->R * a.rho, st);
}

void run_expand(const gto_config *c, const gto_draft_stats *s, const gto_pool *p, hipStream_t st) {
  gto::ExpandArgs a{};
  a.R = c->R; a.d = c->d; a.k = c->k; a.C = pool_size(c);
  a.top_tok = s->top_tok; a.top_logp = s->top_logp;
  a.cand_tok = p->cand_tok; a.cand_parent = p->cand_parent; a.cand_depth = p->cand_depth;
  a.cand_pslot = p->cand_pslot; a.cand_slot = p->cand_slot; a.cand_score = p->cand_score;
  a.slot_cand = p->slot_cand;
  ProfScope ps("expand", st);
  gto::launch_expand(a, st);
}

void run_reward(const gto_config *c, const gto_tree *t, const void *logits, const gto_target_stats *s,
                const gto_reward *w, hipStream_t st) {
  gto::RewardArgs a{};
  a.R = c->R; a.d = c->d; a.k = c->k; a.g = c->g; a.dtype = c->dtype; a.reward_mode = c->reward_mode;
  a.row_stride = c->row_stride; a.eta = c->eta;
  a.target_logits = logits; a.t_lse = s->t_lse; a.t_argmax = s->t_argmax;
  a.sel_tok = t->sel_tok; a.sel_parent = t->sel_parent; a.sel_depth = t->sel_depth;
  a.sel_pslot = t->sel_pslot; a.sel_slot = t->sel_slot; a.sel_leaf = t->sel_leaf; a.n_sel = t->n_sel;
  a.node_q = w->node_q; a.node_cum = w->node_cum; a.reward = w->reward; a.reward_aux = w->reward_aux;
  a.n_leaves = w->n_leaves; a.path_len = w->path_len; a.path_node = w->path_node; a.path_slot = w->path_slot;
  ProfScope ps("reward_path", st);
  gto::launch_reward(a, st);
}

}  // namespace

extern "C" {

int gto_version(void) { return 100; }

const char *gto_strerror(int status) {
  switch (status) {
    case GTO_OK: return "ok";
    case GTO_E_NULL: return "a required pointer is NULL";
    case GTO_E_SHAPE: return "a size is outside the supported limits";
    case GTO_E_ALIGN: return "logits base or row stride is not 16-byte aligned";
    case GTO_E_DTYPE: return "unknown logits dtype";
    case GTO_E_MODE: return "unknown reward mode or unusable eta/eps/delta";
    case GTO_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case GTO_E_HIP: return t_hip_error.empty() ? "HIP error" : t_hip_error.c_str();
    default: return "unknown status";
  }
}

int gto_workspace_bytes(const gto_config *cfg, size_t *bytes_out) {
  if (!bytes_out) return GTO_E_NULL;
  GTO_TRY(check_cfg(cfg, false));
  const size_t raw = (size_t)cfg->R * cfg->d * sizeof(float);  // reference lse of the path rows
  *bytes_out = (raw + 255) & ~(size_t)255;
  return GTO_OK;
}

int gto_draft_row_stats(const gto_config *cfg, const void *draft_logits, const gto_draft_stats *stats_out,
                        void *hip_stream) {
  GTO_TRY(check_cfg(cfg, false));
  GTO_TRY(check_logits(draft_logits));
  GTO_TRY(check_draft_stats(stats_out));
  run_draft_rows(cfg, draft_logits, stats_out, (hipStream_t)hip_stream);
  return hip_status();
}

int gto_target_row_stats(const gto_config *cfg, const void *target_logits, const gto_target_stats *stats_out,
                         void *hip_stream) {
  GTO_TRY(check_cfg(cfg, false));
  GTO_TRY(check_logits(target_logits));
  GTO_TRY(check_target_stats(stats_out));
  run_target_rows(cfg, target_logits, stats_out, nullptr, (hipStream_t)hip_stream);
  return hip_status();
}

int gto_expand_from_stats(const gto_config *cfg, const gto_draft_stats *stats, const gto_pool *pool_out,
                          void *hip_stream) {
  GTO_TRY(check_cfg(cfg, false));
  GTO_TRY(check_draft_stats(stats));
  GTO_TRY(check_pool(pool_out));
  run_expand(cfg, stats, pool_out, (hipStream_t)hip_stream);
  return hip_status();
}

int gto_expand_tree(const gto_config *cfg, const void *draft_logits, const gto_draft_stats *stats_out,
                    const gto_pool *pool_out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  GTO_TRY(check_cfg(cfg, false));
  GTO_TRY(check_logits(draft_logits));
  GTO_TRY(check_draft_stats(stats_out));
  GTO_TRY(check_pool(pool_out));
  run_draft_rows(cfg, draft_logits, stats_out, (hipStream_t)hip_stream);
  run_expand(cfg, stats_out, pool_out, (hipStream_t)hip_stream);
  return hip_status();
}

int gto_select_topg(const gto_config *cfg, const gto_pool *pool, const gto_tree *tree_out, void *hip_stream) {
  GTO_TRY(check_cfg(cfg, false));
  GTO_TRY(check_pool(pool));
  GTO_TRY(check_tree(tree_out));
  gto::SelectArgs a{};
  a.R = cfg->R; a.C = pool_size(cfg); a.g = cfg->g; a.d = cfg->d; a.k = cfg->k;
  a.cand_tok = pool->cand_tok; a.cand_parent = pool->cand_parent; a.cand_depth = pool->cand_depth;
  a.cand_pslot = pool->cand_pslot; a.cand_slot = pool->cand_slot; a.cand_score = pool->cand_score;
  a.sel_cand = tree_out->sel_cand; a.sel_tok = tree_out->sel_tok; a.sel_parent = tree_out->sel_parent;
  a.sel_depth = tree_out->sel_depth; a.sel_pslot = tree_out->sel_pslot; a.sel_slot = tree_out->sel_slot;
  a.sel_leaf = tree_out->sel_leaf; a.sel_score = tree_out->sel_score; a.n_sel = tree_out->n_sel;
  a.slot_need = tree_out->slot_need;
  {
    ProfScope ps("select_topg", (hipStream_t)hip_stream);
    gto::launch_select(a, (hipStream_t)hip_stream);
  }
  return hip_status();
}

int gto_reward_from_stats(const gto_config *cfg, const gto_tree *tree, const void *target_logits,
                          const gto_target_stats *stats, const gto_reward *reward_out, void *hip_stream) {
  GTO_TRY(check_cfg(cfg, false));
  GTO_TRY(check_logits(target_logits));
  GTO_TRY(check_tree(tree));
  GTO_TRY(check_target_stats(stats));
  GTO_TRY(check_reward(reward_out));
  run_reward(cfg, tree, target_logits, stats, reward_out, (hipStream_t)hip_stream);
  return hip_status();
}

int gto_tree_reward(const gto_config *cfg, const gto_tree *tree, const void *target_logits,
                    const gto_target_stats *stats_out, const gto_reward *reward_out, void *workspace,
                    size_t workspace_bytes, void *hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  GTO_TRY(check_cfg(cfg, false));
  GTO_TRY(check_logits(target_logits));
  GTO_TRY(check_tree(tree));
  GTO_TRY(check_target_stats(stats_out));
  GTO_TRY(check_reward(reward_out));
  run_target_rows(cfg, target_logits, stats_out,
                  (cfg->flags & GTO_FLAG_TARGET_PRUNE) ? tree->slot_need : nullptr, (hipStream_t)hip_stream);
  run_reward(cfg, tree, target_logits, stats_out, reward_out, (hipStream_t)hip_stream);
  return hip_status();
}

int gto_group_advantage(const gto_config *cfg, const float *reward_cur, const float *reward_ref, float *adv_out,
                        void *hip_stream) {
  GTO_TRY(check_cfg(cfg, true));
  if (!reward_cur || !adv_out) return GTO_E_NULL;
  gto::AdvArgs a{};
  a.R = cfg->R; a.m = cfg->group_size; a.delta = cfg->delta;
  a.r_cur = reward_cur; a.r_ref = reward_ref; a.adv = adv_out;
  {
    ProfScope ps("group_advantage", (hipStream_t)hip_stream);
    gto::launch_advantage(a, (hipStream_t)hip_stream);
  }
  return hip_status();
}

int gto_ppo_surrogate_fwd(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                          const void *draft_logits_cur, const gto_draft_stats *draft_stats_cur,
                          const void *ref_logits_on_cur, const gto_draft_stats *ref_stats, const float *adv,
                          const gto_ppo *out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  GTO_TRY(check_cfg(cfg, true));
  GTO_TRY(check_logits(draft_logits_cur));
  GTO_TRY(check_logits(ref_logits_on_cur));
  GTO_TRY(check_tree(tree_cur));
  GTO_TRY(check_reward(path_cur));
  if (!draft_stats_cur || !draft_stats_cur->row_lse || !adv) return GTO_E_NULL;
  GTO_TRY(check_ppo(out));
  hipStream_t st = (hipStream_t)hip_stream;
  const float *ref_lse = nullptr;
  int by_step = 0;
  if (ref_stats) {
    if (!ref_stats->row_lse) return GTO_E_NULL;
    ref_lse = ref_stats->row_lse;
  } else {
    size_t need = 0;
    GTO_TRY(gto_workspace_bytes(cfg, &need));
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255))
      return GTO_E_WORKSPACE;
    gto::RowStatsArgs a{};
    a.logits = ref_logits_on_cur;
    a.row_stride = cfg->row_stride;
    a.V = cfg->V; a.d = cfg->d; a.kslots = cfg->k; a.ktop = 1; a.rho = rows_per_root(cfg);
    a.path_slot = path_cur->path_slot;
    a.row_max = nullptr; a.row_lse = static_cast<float *>(workspace); a.top_tok = nullptr; a.top_logp = nullptr;
    ProfScope ps("row_stats_ref_path", st);
    gto::launch_row_stats(a, cfg->dtype, cfg->R * cfg->d, st);
    ref_lse = static_cast<const float *>(workspace);
    by_step = 1;
  }
  gto::PpoFwdArgs a{};
  a.R = cfg->R; a.d = cfg->d; a.k = cfg->k; a.g = cfg->g; a.m = cfg->group_size; a.dtype = cfg->dtype;
  a.row_stride = cfg->row_stride; a.eps = cfg->eps; a.grad_scale = cfg->grad_scale;
  a.draft_logits = draft_logits_cur; a.ref_logits = ref_logits_on_cur;
  a.draft_lse = draft_stats_cur->row_lse; a.ref_lse = ref_lse; a.ref_lse_by_step = by_step;
  a.sel_tok = tree_cur->sel_tok; a.path_len = path_cur->path_len; a.path_node = path_cur->path_node;
  a.path_slot = path_cur->path_slot; a.adv = adv;
  a.logM = out->logM; a.logM0 = out->logM0; a.ratio = out->ratio; a.term = out->term; a.coef = out->coef;
  a.loss_group = out->loss_group; a.loss = out->loss; a.active = out->active;
  {
    ProfScope ps("ppo_fwd", st);
    gto::launch_ppo_fwd(a, st);
  }
  return hip_status();
}

int gto_ppo_surrogate_bwd(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                          const gto_ppo *fwd, const void *draft_logits_cur, const gto_draft_stats *draft_stats_cur,
                          float *grad_rows, int32_t *grad_slot, void *hip_stream) {
  GTO_TRY(check_cfg(cfg, true));
  GTO_TRY(check_logits(draft_logits_cur));
  GTO_TRY(check_tree(tree_cur));
  GTO_TRY(check_reward(path_cur));
  GTO_TRY(check_ppo(fwd));
  if (!draft_stats_cur || !draft_stats_cur->row_lse || !grad_rows || !grad_slot) return GTO_E_NULL;
  gto::PpoBwdArgs a{};
  a.logits = draft_logits_cur;
  a.row_stride = cfg->row_stride;
  a.V = cfg->V; a.d = cfg->d; a.k = cfg->k; a.g = cfg->g;
  a.path_slot = path_cur->path_slot; a.path_node = path_cur->path_node; a.sel_tok = tree_cur->sel_tok;
  a.coef = fwd->coef; a.row_lse = draft_stats_cur->row_lse;
  a.grad_rows = grad_rows; a.grad_slot = grad_slot;
  a.zero_fill = (cfg->flags & GTO_FLAG_GRAD_ZERO_FILL) ? 1 : 0;
  {
    ProfScope ps("ppo_bwd", (hipStream_t)hip_stream);
    gto::launch_ppo_bwd(a, cfg->dtype, cfg->R * cfg->d, (hipStream_t)hip_stream);
  }
  return hip_status();
}

int gto_calibration_copy(const void *src, void *dst, size_t bytes, void *hip_stream) {
  if (!src || !dst) return GTO_E_NULL;
  if (bytes == 0 || bytes % 16 != 0) return GTO_E_SHAPE;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) return GTO_E_ALIGN;
  {
    ProfScope ps("calibration_copy", (hipStream_t)hip_stream);
    gto::launch_copy16(src, dst, (int64_t)bytes, (hipStream_t)hip_stream);
  }
  return hip_status();
}

int gto_set_waves_per_row(int waves) {
  gto::set_waves_per_row(waves);
  return gto::get_waves_per_row();
}

int gto_profile_enable(int on) {
  t_prof_on = (on != 0);
  return GTO_OK;
}

int gto_profile_read(const char **names, int32_t *launches, double *total_ms, int cap) {
  if (!names || !launches || !total_ms || cap < 1) return GTO_E_NULL;
  int n = 0;
  for (ProfRecord &rec : t_prof) {
    (void)hipEventSynchronize(rec.stop);
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, rec.start, rec.stop);
    (void)hipEventDestroy(rec.start);
    (void)hipEventDestroy(rec.stop);
    int slot = -1;
    for (int i = 0; i < n; ++i)
      if (strcmp(names[i], rec.name) == 0) slot = i;
    if (slot < 0) {
      if (n >= cap) continue;
      slot = n++;
      names[slot] = rec.name;
      launches[slot] = 0;
      total_ms[slot] = 0.0;
    }
    launches[slot] += 1;
    total_ms[slot] += (double)ms;
  }
  t_prof.clear();
  return n;
}

}  // extern "C"
