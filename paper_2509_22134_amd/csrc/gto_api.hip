// C ABI of libgto: argument validation on the host, then kernel launches on the caller's
// stream.  No allocation, no synchronisation, no retained pointers.
#include <hip/hip_runtime.h>
#include <string.h>

#include <mutex>
#include <string>
#include <utility>
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
// Per calling thread: a pool of event pairs filled by gto_profile_enable(1) and recycled by
// gto_profile_read, so that a launch under profiling only records two events.
struct ProfRecord {
  const char *name;
  hipEvent_t start, stop;
};
constexpr size_t kProfInitialPairs = 1024, kProfMaxRecords = 16384;
struct ProfState {
  bool on = false;
  std::string only;      // empty: every kernel is timed; else only the kernel of this name
  std::vector<ProfRecord> used;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> free_pairs;
  size_t created = 0;
  bool grow(size_t n) {
    for (size_t i = 0; i < n && created < kProfMaxRecords; ++i) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess) return false;
      if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return false; }
      free_pairs.emplace_back(a, b);
      ++created;
    }
    return true;
  }
  ~ProfState() {
    // events are left to the runtime's own teardown: the device may already be gone when a thread ends
  }
};
thread_local ProfState t_prof;

struct ProfScope {
  hipStream_t st;
  bool on;
  ProfRecord rec;
  ProfScope(const char *name, hipStream_t s) : st(s), on(t_prof.on) {
    if (on && !t_prof.only.empty() && t_prof.only != name) on = false;
    if (!on) return;
    if (t_prof.free_pairs.empty() && !t_prof.grow(256)) { on = false; return; }
    if (t_prof.free_pairs.empty()) { on = false; return; }      // cap reached: this launch is not timed
    rec.name = name;
    rec.start = t_prof.free_pairs.back().first;
    rec.stop = t_prof.free_pairs.back().second;
    t_prof.free_pairs.pop_back();
    (void)hipEventRecord(rec.start, st);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(rec.stop, st);
    t_prof.used.push_back(rec);
  }
};

// ------------------------------------------------------------------------- static scratch
// Scratch memory of gto_ppo_surrogate_fwd_noalloc: the log-sum-exp of the reference model's rows on the
// accepted paths, [R, d] floats.  Every GPU the library runs on holds its own copy of this array at its
// own address until the process ends; host code must only ever use the per-device address obtained from
// hipGetSymbolAddress below, never the array's name.
constexpr int kNoAllocMaxRows = 65536;                    // R * d of one call; 256 KiB per GPU
static __device__ __align__(256) float scratch[kNoAllocMaxRows];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float *g_scratch_ptr[kMaxDevices] = {};                   // written once per device, under the mutex

// Address of `scratch` on the current device (resolved on the first call on that device).
int scratch_on_current_device(float **out) {
  int dev = -1;
  const hipError_t ed = hipGetDevice(&dev);
  if (ed != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    t_hip_error = std::string("HIP error: ") + (ed != hipSuccess ? hipGetErrorString(ed) : "device ordinal out of range");
    (void)hipGetLastError();
    return GTO_E_HIP;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      t_hip_error = std::string("HIP error: ") + hipGetErrorString(e);
      (void)hipGetLastError();
      return GTO_E_HIP;
    }
    g_scratch_ptr[dev] = static_cast<float *>(p);
  }
  *out = g_scratch_ptr[dev];
  return GTO_OK;
}

// ------------------------------------------------------------------------- validation
constexpr int kMaxK = 64, kMaxD = 32, kMaxPool = 4096;

int elem_size(int dtype) { return dtype == GTO_BF16 ? 2 : 4; }

// Tests on the bit pattern: this file is compiled with the same floating-point flags as the kernels
// (NaNs not honoured), so a comparison is not a reliable way to reject a NaN argument here.
bool finite_at_least(float x, bool allow_zero) {
  uint32_t u;
  memcpy(&u, &x, sizeof u);
  if ((u & 0x7f800000u) == 0x7f800000u) return false;          // inf or NaN
  if ((u & 0x7fffffffu) == 0u) return allow_zero;               // +0 or -0
  return (u & 0x80000000u) == 0u;                               // positive
}
bool is_finite(float x) {
  uint32_t u;
  memcpy(&u, &x, sizeof u);
  return (u & 0x7f800000u) != 0x7f800000u;
}

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
  if (!finite_at_least(c->eta, false) || !finite_at_least(c->eps, true) || !finite_at_least(c->delta, true) ||
      !is_finite(c->grad_scale))
    return GTO_E_MODE;
  const int wpr = c->waves_per_row;
  if (!(wpr == 0 || wpr == 1 || wpr == 2 || wpr == 4 || wpr == 8)) return GTO_E_MODE;
  if (c->fused_layout != 0 && c->fused_layout != 1) return GTO_E_MODE;
  if (c->fused_groups < 0 || c->fused_groups > (c->fused_layout == 0 ? 16 : 8) || c->reserved != 0) return GTO_E_MODE;
  if (c->path_mode != GTO_PATH_GREEDY && c->path_mode != GTO_PATH_MAX_L && c->path_mode != GTO_PATH_SAMPLED)
    return GTO_E_MODE;
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
// the entry points that take the verification walk also need the uniform numbers in the sampled mode
int check_reward_out(const gto_config *c, const gto_reward *w) {
  GTO_TRY(check_reward(w));
  if (c->path_mode == GTO_PATH_SAMPLED && w->accept_u == nullptr) return GTO_E_NULL;
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
  a.waves = c->waves_per_row;
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
  a.waves = c->waves_per_row;
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
  a.R = c->R; a.d = c->d; a.k = c->k; a.g = c->g; a.V = c->V; a.dtype = c->dtype; a.reward_mode = c->reward_mode;
  a.path_mode = c->path_mode;
  a.row_stride = c->row_stride; a.eta = c->eta;
  a.target_logits = logits; a.t_lse = s->t_lse; a.t_argmax = s->t_argmax; a.accept_u = w->accept_u;
  a.sel_tok = t->sel_tok; a.sel_parent = t->sel_parent; a.sel_depth = t->sel_depth;
  a.sel_pslot = t->sel_pslot; a.sel_slot = t->sel_slot; a.sel_leaf = t->sel_leaf; a.n_sel = t->n_sel;
  a.node_q = w->node_q; a.node_cum = w->node_cum; a.reward = w->reward; a.reward_aux = w->reward_aux;
  a.n_leaves = w->n_leaves; a.path_len = w->path_len; a.path_node = w->path_node; a.path_slot = w->path_slot;
  ProfScope ps("reward_path", st);
  gto::launch_reward(a, st);
}

int check_ppo_fwd_args(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                       const void *draft_logits_cur, const gto_draft_stats *draft_stats_cur,
                       const void *ref_logits_on_cur, const float *adv, const gto_ppo *out) {
  GTO_TRY(check_cfg(cfg, true));
  GTO_TRY(check_logits(draft_logits_cur));
  GTO_TRY(check_logits(ref_logits_on_cur));
  GTO_TRY(check_tree(tree_cur));
  GTO_TRY(check_reward(path_cur));
  if (!draft_stats_cur || !draft_stats_cur->row_lse || !adv) return GTO_E_NULL;
  GTO_TRY(check_ppo(out));
  return GTO_OK;
}

// Eq. 11-12.  The reference rows' log-sum-exp comes either from statistics of the whole tensor
// (`ref_lse_by_slot`, [R, d, k]) or is computed here for the rows on the accepted paths into
// `lse_by_step` ([R, d] floats of scratch memory).
void run_ppo_fwd(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                 const void *draft_logits_cur, const gto_draft_stats *draft_stats_cur, const void *ref_logits_on_cur,
                 const float *ref_lse_by_slot, float *lse_by_step, const float *adv, const gto_ppo *out,
                 hipStream_t st) {
  if (!ref_lse_by_slot) {
    gto::RowStatsArgs a{};
    a.logits = ref_logits_on_cur;
    a.row_stride = cfg->row_stride;
    a.V = cfg->V; a.d = cfg->d; a.kslots = cfg->k; a.ktop = 1; a.rho = rows_per_root(cfg);
    a.waves = cfg->waves_per_row;
    a.path_slot = path_cur->path_slot;
    a.row_max = nullptr; a.row_lse = lse_by_step; a.top_tok = nullptr; a.top_logp = nullptr;
    ProfScope ps("row_stats_ref_path", st);
    gto::launch_row_stats(a, cfg->dtype, cfg->R * cfg->d, st);
  }
  gto::PpoFwdArgs a{};
  a.R = cfg->R; a.d = cfg->d; a.k = cfg->k; a.g = cfg->g; a.m = cfg->group_size; a.dtype = cfg->dtype; a.V = cfg->V;
  a.row_stride = cfg->row_stride; a.eps = cfg->eps; a.grad_scale = cfg->grad_scale;
  a.draft_logits = draft_logits_cur; a.ref_logits = ref_logits_on_cur;
  a.draft_lse = draft_stats_cur->row_lse;
  a.ref_lse = ref_lse_by_slot ? ref_lse_by_slot : lse_by_step;
  a.ref_lse_by_step = ref_lse_by_slot ? 0 : 1;
  a.sel_tok = tree_cur->sel_tok; a.path_len = path_cur->path_len; a.path_node = path_cur->path_node;
  a.path_slot = path_cur->path_slot; a.adv = adv;
  a.logM = out->logM; a.logM0 = out->logM0; a.ratio = out->ratio; a.term = out->term; a.coef = out->coef;
  a.loss_group = out->loss_group; a.loss = out->loss; a.active = out->active;
  ProfScope ps("ppo_fwd", st);
  gto::launch_ppo_fwd(a, st);
}

// ------------------------------------------------------------------------- fused LM-head variant
constexpr int kFusedMaxK = 16;

struct FusedPlan {
  int64_t M;
  int n_tiles, groups, patch_rows, patch_cols, n_slots;
  size_t off_s, off_m, off_c, off_v, off_i, bytes;
};

int check_fused(const gto_config *c, const void *hidden, int hidden_dim, const void *w) {
  GTO_TRY(check_cfg(c, false));
  if (c->dtype != GTO_BF16) return GTO_E_DTYPE;
  if (c->k > kFusedMaxK || hidden_dim < 64 || hidden_dim % 64 != 0) return GTO_E_SHAPE;
  GTO_TRY(check_logits(hidden));
  GTO_TRY(check_logits(w));
  return GTO_OK;
}

// Launch geometry of the row pass (see the work distribution in gto_fused.hip): `groups` groups of
// patch_rows x patch_cols workgroups, each row with groups * patch_cols partial results.  By default 8 groups
// of 8 x 4: one group per XCD, one workgroup per compute unit (8 x 4 and 4 x 8 take the same time; 8 x 4 streams
// the head half as often, fetches a quarter less from the fabric and leaves half as many partial results).
FusedPlan fused_plan(const gto_config *c, int64_t M, int ktop) {
  FusedPlan p{};
  p.M = M;
  p.n_tiles = (c->V + 255) / 256;
  p.groups = c->fused_groups > 0 ? c->fused_groups : 8;
  p.patch_rows = c->fused_layout == 0 ? 8 : 4;
  p.patch_cols = c->fused_layout == 0 ? 4 : 8;
  p.n_slots = p.groups * p.patch_cols;
  const size_t rows = (size_t)M * p.n_slots;
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  p.off_s = 0;
  p.off_m = up(p.off_s + rows * sizeof(double));
  p.off_c = up(p.off_m + rows * sizeof(float));
  p.off_v = up(p.off_c + rows * sizeof(float));
  p.off_i = up(p.off_v + rows * ktop * sizeof(float));
  p.bytes = up(p.off_i + rows * ktop * sizeof(int32_t));
  return p;
}

void set_geometry(gto::FusedArgs &a, const FusedPlan &p) {
  a.n_tiles = p.n_tiles; a.groups = p.groups; a.patch_rows = p.patch_rows; a.patch_cols = p.patch_cols;
}

// Workspace of the fused calls: [partials of the row pass | gathered single logits].
struct FusedWs {
  size_t partial_bytes, off_slot, off_tok, off_out0, off_out1, off_list, off_count, bytes;
};
FusedWs fused_ws(const gto_config *c) {
  FusedWs w{};
  const int64_t M = (int64_t)c->R * rows_per_root(c);
  size_t b = fused_plan(c, M, c->k).bytes;
  const size_t b1 = fused_plan(c, M, 1).bytes;
  w.partial_bytes = b1 > b ? b1 : b;
  const size_t n = (size_t)c->R * (size_t)(c->g > c->d ? c->g : c->d);
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  w.off_slot = w.partial_bytes;
  w.off_tok = up(w.off_slot + n * sizeof(int64_t));
  w.off_out0 = up(w.off_tok + n * sizeof(int32_t));
  w.off_out1 = up(w.off_out0 + n * sizeof(float));
  w.off_list = up(w.off_out1 + n * sizeof(float));            // compacted slot list of a pruned target pass
  w.off_count = up(w.off_list + (size_t)c->R * c->d * c->k * sizeof(int32_t));
  w.bytes = w.off_count + 256;
  // the backward pass lays the same memory out differently
  const size_t rd = (size_t)c->R * c->d;
  const size_t bwd = fused_plan(c, (int64_t)rd, 1).bytes + 2 * up(rd * sizeof(int32_t)) + 256;
  if (bwd > w.bytes) w.bytes = bwd;
  return w;
}

int check_ws(const void *ws, size_t ws_bytes, size_t need) {
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255)) return GTO_E_WORKSPACE;
  return GTO_OK;
}

// single logits hidden[slot] . w[tok] for the kept nodes (mode 0) or the path steps (mode 1)
void run_gather(const gto_config *c, const gto_tree *t, const gto_reward *path, int mode, const void *hidden,
                int hidden_dim, const void *w, void *ws, const FusedWs &L, float *out, hipStream_t st) {
  char *base = static_cast<char *>(ws);
  gto::PairArgs pa{};
  pa.R = c->R; pa.d = c->d; pa.k = c->k; pa.g = c->g;
  pa.sel_tok = t->sel_tok; pa.sel_depth = t->sel_depth; pa.sel_pslot = t->sel_pslot; pa.n_sel = t->n_sel;
  pa.path_slot = path ? path->path_slot : nullptr; pa.path_node = path ? path->path_node : nullptr;
  pa.slot = reinterpret_cast<int64_t *>(base + L.off_slot);
  pa.tok = reinterpret_cast<int32_t *>(base + L.off_tok);
  gto::GatherDotArgs ga{};
  ga.hidden = hidden; ga.w = w; ga.hidden_dim = hidden_dim; ga.V = c->V;
  ga.n = (int64_t)c->R * (mode == 0 ? c->g : c->d);
  ga.slot = pa.slot; ga.tok = pa.tok; ga.out = out;
  ProfScope ps(mode == 0 ? "gather_nodes" : "gather_path", st);
  gto::launch_pairs(pa, mode, st);
  gto::launch_gather_dot(ga, st);
}

int run_fused_rows(const gto_config *c, const void *hidden, int hidden_dim, const void *w, int ktop,
                   const int32_t *row_list, int64_t n_list, const int32_t *n_dev, int out_by_list, float *row_max,
                   float *row_lse,
                   int32_t *top_tok, float *top_logp, float *top_logit, void *ws, size_t ws_bytes,
                   const char *name, hipStream_t st) {
  const int64_t M = row_list ? n_list : (int64_t)c->R * rows_per_root(c);
  const FusedPlan p = fused_plan(c, M, ktop);
  if (!ws || ws_bytes < p.bytes || (reinterpret_cast<uintptr_t>(ws) & 255)) return GTO_E_WORKSPACE;
  char *base = static_cast<char *>(ws);
  gto::FusedArgs a{};
  a.hidden = hidden; a.w = w; a.hidden_dim = hidden_dim; a.V = c->V; a.rho = rows_per_root(c); a.d = c->d;
  a.kslots = c->k; a.ktop = ktop; a.M = M; a.m_dev = n_dev; a.row_list = row_list; a.out_by_list = out_by_list;
  set_geometry(a, p);
  a.part_s = reinterpret_cast<double *>(base + p.off_s);
  a.part_m = reinterpret_cast<float *>(base + p.off_m);
  a.part_c = reinterpret_cast<float *>(base + p.off_c);
  a.part_v = reinterpret_cast<float *>(base + p.off_v);
  a.part_i = reinterpret_cast<int32_t *>(base + p.off_i);
  a.row_max = row_max; a.row_lse = row_lse; a.top_tok = top_tok; a.top_logp = top_logp; a.top_logit = top_logit;
  {
    ProfScope ps(name, st);
    gto::launch_fused_rows(a, st);
  }
  {
    ProfScope ps("fused_merge", st);
    gto::launch_fused_merge(a, st);
  }
  return GTO_OK;
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
    case GTO_E_WORKSPACE: return "workspace missing, misaligned or too small (for a no-alloc call: size beyond the static scratch array)";
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
  GTO_TRY(check_reward_out(cfg, reward_out));
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
  GTO_TRY(check_reward_out(cfg, reward_out));
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
  GTO_TRY(check_ppo_fwd_args(cfg, tree_cur, path_cur, draft_logits_cur, draft_stats_cur, ref_logits_on_cur, adv, out));
  float *lse_by_step = nullptr;
  if (ref_stats) {
    if (!ref_stats->row_lse) return GTO_E_NULL;
  } else {
    size_t need = 0;
    GTO_TRY(gto_workspace_bytes(cfg, &need));
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255))
      return GTO_E_WORKSPACE;
    lse_by_step = static_cast<float *>(workspace);
  }
  run_ppo_fwd(cfg, tree_cur, path_cur, draft_logits_cur, draft_stats_cur, ref_logits_on_cur,
              ref_stats ? ref_stats->row_lse : nullptr, lse_by_step, adv, out, (hipStream_t)hip_stream);
  return hip_status();
}

int gto_ppo_surrogate_fwd_noalloc(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                                  const void *draft_logits_cur, const gto_draft_stats *draft_stats_cur,
                                  const void *ref_logits_on_cur, const float *adv, const gto_ppo *out,
                                  void *hip_stream) {
  GTO_TRY(check_ppo_fwd_args(cfg, tree_cur, path_cur, draft_logits_cur, draft_stats_cur, ref_logits_on_cur, adv, out));
  if ((int64_t)cfg->R * cfg->d > kNoAllocMaxRows) return GTO_E_WORKSPACE;
  float *lse_by_step = nullptr;
  GTO_TRY(scratch_on_current_device(&lse_by_step));
  // nothing in the scratch needs clearing: the row pass writes the entry of every (root, step) on an
  // accepted path before the surrogate kernel reads exactly those entries, on the same stream
  run_ppo_fwd(cfg, tree_cur, path_cur, draft_logits_cur, draft_stats_cur, ref_logits_on_cur, nullptr, lse_by_step,
              adv, out, (hipStream_t)hip_stream);
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

int gto_fused_workspace_bytes(const gto_config *cfg, int32_t hidden_dim, size_t *bytes_out) {
  if (!bytes_out) return GTO_E_NULL;
  GTO_TRY(check_cfg(cfg, false));
  if (cfg->k > kFusedMaxK || hidden_dim < 64 || hidden_dim % 64 != 0) return GTO_E_SHAPE;
  *bytes_out = fused_ws(cfg).bytes;
  return GTO_OK;
}

int gto_fused_draft_row_stats(const gto_config *cfg, const void *hidden, int32_t hidden_dim, const void *w_vh,
                              const gto_draft_stats *stats_out, float *top_logit_or_null, void *workspace,
                              size_t workspace_bytes, void *hip_stream) {
  GTO_TRY(check_fused(cfg, hidden, hidden_dim, w_vh));
  GTO_TRY(check_draft_stats(stats_out));
  GTO_TRY(run_fused_rows(cfg, hidden, hidden_dim, w_vh, cfg->k, nullptr, 0, nullptr, 0, stats_out->row_max,
                         stats_out->row_lse, stats_out->top_tok, stats_out->top_logp, top_logit_or_null,
                         workspace, workspace_bytes, "fused_rows_draft", (hipStream_t)hip_stream));
  return hip_status();
}

int gto_fused_target_row_stats(const gto_config *cfg, const void *hidden, int32_t hidden_dim, const void *w_vh,
                               const gto_target_stats *stats_out, void *workspace, size_t workspace_bytes,
                               void *hip_stream) {
  GTO_TRY(check_fused(cfg, hidden, hidden_dim, w_vh));
  GTO_TRY(check_target_stats(stats_out));
  GTO_TRY(run_fused_rows(cfg, hidden, hidden_dim, w_vh, 1, nullptr, 0, nullptr, 0, stats_out->t_max, stats_out->t_lse,
                         stats_out->t_argmax, nullptr, nullptr, workspace, workspace_bytes, "fused_rows_target",
                         (hipStream_t)hip_stream));
  return hip_status();
}

int gto_expand_tree_fused(const gto_config *cfg, const void *hidden, int32_t hidden_dim, const void *w_draft_vh,
                          const gto_draft_stats *stats_out, const gto_pool *pool_out, void *workspace,
                          size_t workspace_bytes, void *hip_stream) {
  GTO_TRY(check_fused(cfg, hidden, hidden_dim, w_draft_vh));
  GTO_TRY(check_draft_stats(stats_out));
  GTO_TRY(check_pool(pool_out));
  GTO_TRY(check_ws(workspace, workspace_bytes, fused_ws(cfg).bytes));
  hipStream_t st = (hipStream_t)hip_stream;
  GTO_TRY(run_fused_rows(cfg, hidden, hidden_dim, w_draft_vh, cfg->k, nullptr, 0, nullptr, 0, stats_out->row_max,
                         stats_out->row_lse, stats_out->top_tok, stats_out->top_logp, nullptr, workspace,
                         workspace_bytes, "fused_rows_draft", st));
  run_expand(cfg, stats_out, pool_out, st);
  return hip_status();
}

int gto_tree_reward_fused(const gto_config *cfg, const gto_tree *tree, const void *hidden, int32_t hidden_dim,
                          const void *w_target_vh, const gto_target_stats *stats_out,
                          const gto_reward *reward_out, void *workspace, size_t workspace_bytes,
                          void *hip_stream) {
  GTO_TRY(check_fused(cfg, hidden, hidden_dim, w_target_vh));
  GTO_TRY(check_tree(tree));
  GTO_TRY(check_target_stats(stats_out));
  GTO_TRY(check_reward_out(cfg, reward_out));
  const FusedWs L = fused_ws(cfg);
  GTO_TRY(check_ws(workspace, workspace_bytes, L.bytes));
  hipStream_t st = (hipStream_t)hip_stream;
  const int32_t *list = nullptr, *count = nullptr;
  int64_t cap = 0;
  if (cfg->flags & GTO_FLAG_TARGET_PRUNE) {
    // only the slots whose node has a kept child are multiplied: compact them into a row list
    int32_t *l = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + L.off_list);
    int32_t *c = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + L.off_count);
    ProfScope ps("compact_needed_slots", st);
    gto::launch_compact_flags(tree->slot_need, cfg->R * cfg->d * cfg->k, l, c, st);
    list = l; count = c; cap = (int64_t)cfg->R * rows_per_root(cfg);
  }
  GTO_TRY(run_fused_rows(cfg, hidden, hidden_dim, w_target_vh, 1, list, cap, count, 0, stats_out->t_max,
                         stats_out->t_lse, stats_out->t_argmax, nullptr, nullptr, workspace, workspace_bytes,
                         "fused_rows_target", st));
  float *node_logit = reinterpret_cast<float *>(static_cast<char *>(workspace) + L.off_out0);
  run_gather(cfg, tree, nullptr, 0, hidden, hidden_dim, w_target_vh, workspace, L, node_logit, st);
  {
    gto::RewardArgs a{};
    a.R = cfg->R; a.d = cfg->d; a.k = cfg->k; a.g = cfg->g; a.V = cfg->V; a.dtype = cfg->dtype;
    a.reward_mode = cfg->reward_mode;
    a.path_mode = cfg->path_mode;
    a.row_stride = 0; a.eta = cfg->eta;
    a.target_logits = nullptr; a.node_logit = node_logit; a.t_lse = stats_out->t_lse; a.t_argmax = stats_out->t_argmax;
    a.accept_u = reward_out->accept_u;
    a.sel_tok = tree->sel_tok; a.sel_parent = tree->sel_parent; a.sel_depth = tree->sel_depth;
    a.sel_pslot = tree->sel_pslot; a.sel_slot = tree->sel_slot; a.sel_leaf = tree->sel_leaf; a.n_sel = tree->n_sel;
    a.node_q = reward_out->node_q; a.node_cum = reward_out->node_cum; a.reward = reward_out->reward;
    a.reward_aux = reward_out->reward_aux; a.n_leaves = reward_out->n_leaves; a.path_len = reward_out->path_len;
    a.path_node = reward_out->path_node; a.path_slot = reward_out->path_slot;
    ProfScope ps("reward_path", st);
    gto::launch_reward(a, st);
  }
  return hip_status();
}

int gto_ppo_surrogate_fwd_fused(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                                const void *hidden_cur, const void *hidden_ref_on_cur, int32_t hidden_dim,
                                const void *w_draft_vh, const gto_draft_stats *draft_stats_cur,
                                const gto_draft_stats *ref_stats, const float *adv, const gto_ppo *out,
                                void *workspace, size_t workspace_bytes, void *hip_stream) {
  GTO_TRY(check_cfg(cfg, true));
  GTO_TRY(check_fused(cfg, hidden_cur, hidden_dim, w_draft_vh));
  GTO_TRY(check_logits(hidden_ref_on_cur));
  GTO_TRY(check_tree(tree_cur));
  GTO_TRY(check_reward(path_cur));
  if (!draft_stats_cur || !draft_stats_cur->row_lse || !ref_stats || !ref_stats->row_lse || !adv) return GTO_E_NULL;
  GTO_TRY(check_ppo(out));
  const FusedWs L = fused_ws(cfg);
  GTO_TRY(check_ws(workspace, workspace_bytes, L.bytes));
  hipStream_t st = (hipStream_t)hip_stream;
  float *lc = reinterpret_cast<float *>(static_cast<char *>(workspace) + L.off_out0);
  float *lr = reinterpret_cast<float *>(static_cast<char *>(workspace) + L.off_out1);
  run_gather(cfg, tree_cur, path_cur, 1, hidden_cur, hidden_dim, w_draft_vh, workspace, L, lc, st);
  run_gather(cfg, tree_cur, path_cur, 1, hidden_ref_on_cur, hidden_dim, w_draft_vh, workspace, L, lr, st);
  gto::PpoFwdArgs a{};
  a.R = cfg->R; a.d = cfg->d; a.k = cfg->k; a.g = cfg->g; a.m = cfg->group_size; a.dtype = cfg->dtype; a.V = cfg->V;
  a.row_stride = 0; a.eps = cfg->eps; a.grad_scale = cfg->grad_scale;
  a.draft_logits = nullptr; a.ref_logits = nullptr; a.path_logit_cur = lc; a.path_logit_ref = lr;
  a.draft_lse = draft_stats_cur->row_lse; a.ref_lse = ref_stats->row_lse; a.ref_lse_by_step = 0;
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

int gto_ppo_surrogate_bwd_fused(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                                const gto_ppo *fwd, const void *hidden_cur, int32_t hidden_dim,
                                const void *w_draft_vh, const gto_draft_stats *draft_stats_cur, float *grad_rows,
                                int32_t *grad_slot, void *workspace, size_t workspace_bytes, void *hip_stream) {
  GTO_TRY(check_cfg(cfg, true));
  GTO_TRY(check_fused(cfg, hidden_cur, hidden_dim, w_draft_vh));
  GTO_TRY(check_tree(tree_cur));
  GTO_TRY(check_reward(path_cur));
  GTO_TRY(check_ppo(fwd));
  if (!draft_stats_cur || !draft_stats_cur->row_lse || !grad_rows || !grad_slot) return GTO_E_NULL;
  GTO_TRY(check_ws(workspace, workspace_bytes, fused_ws(cfg).bytes));
  hipStream_t st = (hipStream_t)hip_stream;
  const int64_t rd = (int64_t)cfg->R * cfg->d;
  const FusedPlan p = fused_plan(cfg, rd, 1);
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  char *base = static_cast<char *>(workspace);
  int32_t *list_p = reinterpret_cast<int32_t *>(base + p.bytes);
  int32_t *list_slot = reinterpret_cast<int32_t *>(base + p.bytes + up(rd * sizeof(int32_t)));
  int32_t *count = reinterpret_cast<int32_t *>(base + p.bytes + 2 * up(rd * sizeof(int32_t)));
  {
    gto::BwdRowsArgs b{};
    b.R = cfg->R; b.d = cfg->d; b.k = cfg->k;
    b.path_slot = path_cur->path_slot; b.coef = fwd->coef;
    b.grad_slot = grad_slot; b.list_p = list_p; b.list_slot = list_slot; b.count = count;
    ProfScope ps("bwd_rows", st);
    gto::launch_bwd_rows(b, st);
    if (cfg->flags & GTO_FLAG_GRAD_ZERO_FILL) gto::launch_zero_rows(grad_rows, grad_slot, (int)rd, cfg->V, st);
  }
  gto::FusedArgs a{};
  a.hidden = hidden_cur; a.w = w_draft_vh; a.hidden_dim = hidden_dim; a.V = cfg->V; a.rho = rows_per_root(cfg);
  a.d = cfg->d; a.kslots = cfg->k; a.ktop = 1; a.M = rd; a.m_dev = count; a.row_list = list_slot; a.out_by_list = 1;
  set_geometry(a, p);
  a.part_s = reinterpret_cast<double *>(base + p.off_s);
  a.list_p = list_p; a.sel_tok = tree_cur->sel_tok; a.path_node = path_cur->path_node; a.coef = fwd->coef;
  a.lse_by_slot = draft_stats_cur->row_lse; a.g = cfg->g; a.grad_rows = grad_rows;
  {
    ProfScope ps("fused_rows_bwd", st);
    gto::launch_fused_rows(a, st);
    gto::launch_fused_bwd_fixup(a, st);
  }
  return hip_status();
}

// workspace of the hidden-state backward: the forward-style partial area is not needed; row lists and
// count, the two bf16 planes [R d, V], the split partials [splits, R d, hidden]
struct DhWs {
  int n_splits, slabs_per_split, m_blocks, h_blocks;
  size_t off_list_p, off_list_slot, off_count, off_s, off_hi, off_lo, off_partial, bytes;
};
DhWs dh_ws(const gto_config *c, int hidden_dim) {
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  DhWs L{};
  const size_t rd = (size_t)c->R * c->d;
  const int slabs = 2 * (c->V / 32);
  const int want = 8;                               // splits of the contraction, so that few rows still fill the chip
  L.slabs_per_split = (slabs + want - 1) / want;
  L.n_splits = (slabs + L.slabs_per_split - 1) / L.slabs_per_split;
  L.m_blocks = (int)((rd + 255) / 256);
  L.h_blocks = (hidden_dim + 255) / 256;
  size_t off = 0;
  L.off_list_p = off; off += up(rd * sizeof(int32_t));
  L.off_list_slot = off; off += up(rd * sizeof(int32_t));
  L.off_count = off; off += 256;
  L.off_s = off; off += up(rd * 64 * sizeof(double));     // at most 64 partial results per row
  L.off_hi = off; off += up(rd * (size_t)c->V * sizeof(uint16_t));
  L.off_lo = off; off += up(rd * (size_t)c->V * sizeof(uint16_t));
  L.off_partial = off; off += up((size_t)L.n_splits * rd * hidden_dim * sizeof(float));
  L.bytes = off;
  return L;
}

int gto_fused_dh_workspace_bytes(const gto_config *cfg, int32_t hidden_dim, size_t *bytes_out) {
  if (!cfg || !bytes_out) return GTO_E_NULL;
  GTO_TRY(check_cfg(cfg, true));
  if (cfg->k > kFusedMaxK || hidden_dim < 64 || hidden_dim % 64 != 0 || cfg->V % 32 != 0) return GTO_E_SHAPE;
  *bytes_out = dh_ws(cfg, hidden_dim).bytes;
  return GTO_OK;
}

int gto_ppo_surrogate_bwd_fused_dh(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                                   const gto_ppo *fwd, const void *hidden_cur, int32_t hidden_dim,
                                   const void *w_draft_vh, const void *w_draft_hv,
                                   const gto_draft_stats *draft_stats_cur, float *dh_rows, int32_t *grad_slot,
                                   void *workspace, size_t workspace_bytes, void *hip_stream) {
  GTO_TRY(check_cfg(cfg, true));
  GTO_TRY(check_fused(cfg, hidden_cur, hidden_dim, w_draft_vh));
  GTO_TRY(check_logits(w_draft_hv));
  if (cfg->V % 32 != 0) return GTO_E_SHAPE;
  GTO_TRY(check_tree(tree_cur));
  GTO_TRY(check_reward(path_cur));
  GTO_TRY(check_ppo(fwd));
  if (!draft_stats_cur || !draft_stats_cur->row_lse || !dh_rows || !grad_slot) return GTO_E_NULL;
  const DhWs L = dh_ws(cfg, hidden_dim);
  GTO_TRY(check_ws(workspace, workspace_bytes, L.bytes));
  hipStream_t st = (hipStream_t)hip_stream;
  const int64_t rd = (int64_t)cfg->R * cfg->d;
  char *base = static_cast<char *>(workspace);
  int32_t *list_p = reinterpret_cast<int32_t *>(base + L.off_list_p);
  int32_t *list_slot = reinterpret_cast<int32_t *>(base + L.off_list_slot);
  int32_t *count = reinterpret_cast<int32_t *>(base + L.off_count);
  uint16_t *hi = reinterpret_cast<uint16_t *>(base + L.off_hi);
  uint16_t *lo = reinterpret_cast<uint16_t *>(base + L.off_lo);
  {
    gto::BwdRowsArgs b{};
    b.R = cfg->R; b.d = cfg->d; b.k = cfg->k;
    b.path_slot = path_cur->path_slot; b.coef = fwd->coef;
    b.grad_slot = grad_slot; b.list_p = list_p; b.list_slot = list_slot; b.count = count;
    ProfScope ps("bwd_rows", st);
    gto::launch_bwd_rows(b, st);
    if (cfg->flags & GTO_FLAG_GRAD_ZERO_FILL) gto::launch_zero_rows(dh_rows, grad_slot, (int)rd, hidden_dim, st);
  }
  {
    // -coef * softmax of every path row, as two bf16 planes
    const FusedPlan p = fused_plan(cfg, rd, 1);
    gto::FusedArgs a{};
    a.hidden = hidden_cur; a.w = w_draft_vh; a.hidden_dim = hidden_dim; a.V = cfg->V; a.rho = rows_per_root(cfg);
    a.d = cfg->d; a.kslots = cfg->k; a.ktop = 1; a.M = rd; a.m_dev = count; a.row_list = list_slot; a.out_by_list = 1;
    set_geometry(a, p);
    a.list_p = list_p; a.coef = fwd->coef; a.lse_by_slot = draft_stats_cur->row_lse; a.g = cfg->g;
    a.plane_hi = hi; a.plane_lo = lo; a.sel_tok = tree_cur->sel_tok; a.path_node = path_cur->path_node;
    a.part_s = reinterpret_cast<double *>(base + L.off_s);
    ProfScope ps("fused_rows_bwd_planes", st);
    gto::launch_fused_rows(a, st);
  }
  {
    gto::FusedDhArgs a{};
    a.plane_hi = hi; a.plane_lo = lo; a.w_hv = w_draft_hv; a.w_vh = w_draft_vh;
    a.hidden_dim = hidden_dim; a.V = cfg->V; a.d = cfg->d; a.g = cfg->g; a.M = rd; a.m_dev = count;
    a.m_blocks = L.m_blocks; a.h_blocks = L.h_blocks; a.n_splits = L.n_splits; a.slabs_per_split = L.slabs_per_split;
    a.partial = reinterpret_cast<float *>(base + L.off_partial);
    a.part_s = reinterpret_cast<const double *>(base + L.off_s);
    {
      const FusedPlan p = fused_plan(cfg, rd, 1);
      a.n_tiles = p.n_tiles; a.groups = p.groups; a.patch_rows = p.patch_rows; a.patch_cols = p.patch_cols;
    }
    a.list_p = list_p; a.sel_tok = tree_cur->sel_tok; a.path_node = path_cur->path_node; a.coef = fwd->coef;
    a.dh_rows = dh_rows;
    ProfScope ps("fused_dh", st);
    gto::launch_fused_dh(a, st);
  }
  return hip_status();
}

int gto_token_loss_fwd(const gto_config *cfg, const void *draft_logits, const void *target_logits,
                       const gto_draft_stats *draft_stats, const gto_target_stats *target_stats,
                       const float *weight_or_null, float *loss_rows, float *loss, float *inv_count,
                       void *hip_stream) {
  GTO_TRY(check_cfg(cfg, false));
  GTO_TRY(check_logits(draft_logits));
  GTO_TRY(check_logits(target_logits));
  if (!draft_stats || !draft_stats->row_lse || !target_stats || !target_stats->t_lse || !loss_rows || !loss ||
      !inv_count)
    return GTO_E_NULL;
  gto::TokenLossArgs a{};
  a.R = cfg->R; a.d = cfg->d; a.k = cfg->k; a.V = cfg->V; a.row_stride = cfg->row_stride;
  a.draft_logits = draft_logits; a.target_logits = target_logits;
  a.d_lse = draft_stats->row_lse; a.t_lse = target_stats->t_lse; a.weight = weight_or_null;
  a.loss_rows = loss_rows; a.loss = loss; a.inv_count_out = inv_count;
  {
    ProfScope ps("token_loss_fwd", (hipStream_t)hip_stream);
    gto::launch_token_loss(a, cfg->dtype, false, (hipStream_t)hip_stream);
  }
  return hip_status();
}

int gto_token_loss_bwd(const gto_config *cfg, const void *draft_logits, const void *target_logits,
                       const gto_draft_stats *draft_stats, const gto_target_stats *target_stats,
                       const float *weight_or_null, const float *inv_count, float grad_scale, float *grad_rows0,
                       void *hip_stream) {
  GTO_TRY(check_cfg(cfg, false));
  GTO_TRY(check_logits(draft_logits));
  GTO_TRY(check_logits(target_logits));
  if (!draft_stats || !draft_stats->row_lse || !target_stats || !target_stats->t_lse || !inv_count || !grad_rows0)
    return GTO_E_NULL;
  gto::TokenLossArgs a{};
  a.R = cfg->R; a.d = cfg->d; a.k = cfg->k; a.V = cfg->V; a.row_stride = cfg->row_stride;
  a.draft_logits = draft_logits; a.target_logits = target_logits;
  a.d_lse = draft_stats->row_lse; a.t_lse = target_stats->t_lse; a.weight = weight_or_null;
  a.grad_scale = grad_scale; a.inv_count = inv_count; a.grad = grad_rows0;
  {
    ProfScope ps("token_loss_bwd", (hipStream_t)hip_stream);
    gto::launch_token_loss(a, cfg->dtype, true, (hipStream_t)hip_stream);
  }
  return hip_status();
}

// fused token loss: workspace = [draft root logits | target root logits], fp32 [R, pitch] each
struct TokWs {
  int64_t pitch;
  size_t off_d, off_t, bytes;
};
TokWs tok_ws(const gto_config *c) {
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  TokWs L{};
  L.pitch = ((int64_t)c->V + 3) & ~(int64_t)3;
  L.off_d = 0;
  L.off_t = up((size_t)c->R * L.pitch * sizeof(float));
  L.bytes = L.off_t + up((size_t)c->R * L.pitch * sizeof(float));
  return L;
}

int gto_fused_token_loss_workspace_bytes(const gto_config *cfg, int32_t hidden_dim, size_t *bytes_out) {
  if (!cfg || !bytes_out) return GTO_E_NULL;
  GTO_TRY(check_cfg(cfg, false));
  if (cfg->k > kFusedMaxK || hidden_dim < 64 || hidden_dim % 64 != 0) return GTO_E_SHAPE;
  *bytes_out = tok_ws(cfg).bytes;
  return GTO_OK;
}

int gto_token_loss_fwd_fused(const gto_config *cfg, const void *hidden, int32_t hidden_dim, const void *w_draft_vh,
                             const void *w_target_vh, const gto_draft_stats *draft_stats,
                             const gto_target_stats *target_stats, const float *weight_or_null, float *loss_rows,
                             float *loss, float *inv_count, void *workspace, size_t workspace_bytes,
                             void *hip_stream) {
  GTO_TRY(check_cfg(cfg, false));
  GTO_TRY(check_fused(cfg, hidden, hidden_dim, w_draft_vh));
  GTO_TRY(check_logits(w_target_vh));
  if (!draft_stats || !draft_stats->row_lse || !target_stats || !target_stats->t_lse || !loss_rows || !loss ||
      !inv_count)
    return GTO_E_NULL;
  const TokWs L = tok_ws(cfg);
  GTO_TRY(check_ws(workspace, workspace_bytes, L.bytes));
  hipStream_t st = (hipStream_t)hip_stream;
  char *base = static_cast<char *>(workspace);
  float *dl = reinterpret_cast<float *>(base + L.off_d), *tl = reinterpret_cast<float *>(base + L.off_t);
  for (int which = 0; which < 2; ++which) {
    // root rows only: with one used row per root, row i of the pass is slot (0,0) of root i
    const FusedPlan p = fused_plan(cfg, cfg->R, 1);
    gto::FusedArgs a{};
    a.hidden = hidden; a.w = which ? w_target_vh : w_draft_vh; a.hidden_dim = hidden_dim; a.V = cfg->V; a.rho = 1;
    a.d = cfg->d; a.kslots = cfg->k; a.ktop = 1; a.M = cfg->R;
    set_geometry(a, p);
    a.store_rows = which ? tl : dl; a.store_pitch = L.pitch;
    ProfScope ps(which ? "fused_root_logits_target" : "fused_root_logits_draft", st);
    gto::launch_fused_rows(a, st);
  }
  gto::TokenLossArgs a{};
  a.R = cfg->R; a.d = cfg->d; a.k = cfg->k; a.V = cfg->V; a.row_stride = L.pitch; a.root_stride = L.pitch;
  a.draft_logits = dl; a.target_logits = tl;
  a.d_lse = draft_stats->row_lse; a.t_lse = target_stats->t_lse; a.weight = weight_or_null;
  a.loss_rows = loss_rows; a.loss = loss; a.inv_count_out = inv_count;
  {
    ProfScope ps("token_loss_fwd", st);
    gto::launch_token_loss(a, GTO_F32, false, st);
  }
  return hip_status();
}

int gto_token_loss_bwd_fused(const gto_config *cfg, const gto_draft_stats *draft_stats,
                             const gto_target_stats *target_stats, const float *weight_or_null,
                             const float *inv_count, float grad_scale, float *grad_rows0, const void *workspace,
                             size_t workspace_bytes, void *hip_stream) {
  GTO_TRY(check_cfg(cfg, false));
  if (!draft_stats || !draft_stats->row_lse || !target_stats || !target_stats->t_lse || !inv_count || !grad_rows0)
    return GTO_E_NULL;
  const TokWs L = tok_ws(cfg);
  GTO_TRY(check_ws(const_cast<void *>(workspace), workspace_bytes, L.bytes));
  const char *base = static_cast<const char *>(workspace);
  gto::TokenLossArgs a{};
  a.R = cfg->R; a.d = cfg->d; a.k = cfg->k; a.V = cfg->V; a.row_stride = L.pitch; a.root_stride = L.pitch;
  a.draft_logits = base + L.off_d; a.target_logits = base + L.off_t;
  a.d_lse = draft_stats->row_lse; a.t_lse = target_stats->t_lse; a.weight = weight_or_null;
  a.grad_scale = grad_scale; a.inv_count = inv_count; a.grad = grad_rows0;
  {
    ProfScope ps("token_loss_bwd", (hipStream_t)hip_stream);
    gto::launch_token_loss(a, GTO_F32, true, (hipStream_t)hip_stream);
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

int gto_profile_enable(int on) {
  if (on && t_prof.created == 0 && !t_prof.grow(kProfInitialPairs)) return hip_status();
  t_prof.on = (on != 0);
  return GTO_OK;
}

int gto_profile_filter(const char *kernel_name_or_null) {
  t_prof.only = kernel_name_or_null ? kernel_name_or_null : "";
  return GTO_OK;
}

int gto_profile_read(const char **names, int32_t *launches, double *total_ms, int cap) {
  if (!names || !launches || !total_ms || cap < 1) return GTO_E_NULL;
  int n = 0;
  for (ProfRecord &rec : t_prof.used) {
    (void)hipEventSynchronize(rec.stop);
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, rec.start, rec.stop);
    t_prof.free_pairs.emplace_back(rec.start, rec.stop);
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
  t_prof.used.clear();
  return n;
}

}  // extern "C"
