/*
 * gto.h - C ABI of the MI355X (gfx950) implementation of the data-parallel core of
 * Group Tree Optimization (GTO): batched draft-tree construction, the sampling-free
 * Draft Tree Reward, group-standardised advantages and the clipped likelihood-ratio
 * surrogate (forward and gradient w.r.t. the draft logits).
 *
 * Paper: "Bridging Draft Policy Misalignment: Group Tree Optimization for Speculative
 * Decoding".  Each entry point cites the passage that defines what it computes.
 *
 * Conventions that hold for every call
 *   - All tensor pointers are DEVICE pointers owned by the caller; `cfg` and the small
 *     structs that bundle pointers are HOST memory, read during the call only.
 *   - The library never allocates, frees or keeps device memory, never synchronises, and
 *     enqueues all work on `hip_stream` (a hipStream_t passed as void*, NULL = default
 *     stream).  Outputs are valid once that stream has reached the end of the call.
 *   - Inputs are never modified.  Results are deterministic run to run.
 *   - Return value: GTO_OK (0) or a negative gto_status.  Arguments are validated on the
 *     host before anything is launched, so a failing call has no side effect.
 *   - The library keeps no mutable process-wide state: every tuning choice travels in `cfg`.
 *     Calls may come from several host threads; the optional kernel timing is per calling
 *     thread.  Calls that share output buffers or a workspace must be ordered by the caller
 *     (same stream, or events).
 *   - Logits are finite or -inf (probability 0).  A row that is entirely -inf, or holds a
 *     NaN, gives unspecified VALUES for that root, but never a fault: every token id the
 *     library writes is in [0, V), every index it follows is range-checked, and the other
 *     roots are not affected.
 *
 * Shapes.  R roots, d levels, k branching, g kept nodes, V vocabulary,
 * C = k + (d-1) k^2 generated candidates per root.
 *   logits [R, d, k, row_stride] : slot (l, j) holds the next-token logits at the j-th
 *       expanded node of level l (level 0 = the root, only slot (0,0) is used; slots
 *       (0, 1..k-1) are padding and are never read).  Element type cfg->dtype.  Every row
 *       starts 16-byte aligned (base pointer aligned, row_stride * sizeof(elem) % 16 == 0).
 *   pool index c of a candidate: c = r for the root's r-th best child; for l >= 1 the
 *       r-th best child of slot (l, j) is c = k + (l-1) k^2 + j k + r.
 * Limits (GTO_E_SHAPE otherwise): 1 <= k <= 64, 1 <= d <= 32, C <= 4096, g >= 1, V >= k,
 *       V < 2^31 - 64K, R * (1 + (d-1) k) < 2^31, R % group_size == 0 for the group-wise calls.
 */
#ifndef GTO_H
#define GTO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum gto_status {
  GTO_OK = 0,
  GTO_E_NULL = -1,      /* a required pointer is NULL                                   */
  GTO_E_SHAPE = -2,     /* a size is outside the limits above                           */
  GTO_E_ALIGN = -3,     /* logits base or row stride not 16-byte aligned                */
  GTO_E_DTYPE = -4,     /* cfg->dtype is not GTO_BF16 / GTO_F32                         */
  GTO_E_MODE = -5,      /* cfg->reward_mode / path_mode unknown, or eta/eps/delta not usable */
  GTO_E_WORKSPACE = -6, /* workspace missing, misaligned or smaller than required       */
  GTO_E_HIP = -7        /* a launch failed; gto_strerror(GTO_E_HIP) has the HIP message */
} gto_status;

enum { GTO_BF16 = 0, GTO_F32 = 1 };
/* Longest accepted sequence (Sec. 3.2): GREEDY = the sequence greedy (T = 0) target verification
 * accepts (default); MAX_L = the root-to-leaf sequence with the largest expected acceptance length;
 * SAMPLED = the sequence lossless verification at temperature 1 accepts (Sec. 4 evaluates at T = 1
 * too): at each node the kept children are tried in kept order, child x being accepted with
 * probability p_T(x) / (1 - target mass of the children already rejected at that node), decided by
 * the caller's uniform numbers gto_reward.accept_u (child x ends up accepted with probability
 * p_T(x), so the expected length is the node-sum reward of App. A Eq. (2)). */
enum { GTO_PATH_GREEDY = 0, GTO_PATH_MAX_L = 1, GTO_PATH_SAMPLED = 2 };
enum { GTO_REWARD_LSE = 0, GTO_REWARD_MAX = 1, GTO_REWARD_MEAN = 2, GTO_REWARD_NODESUM = 3 };
enum {
  GTO_FLAG_GRAD_ZERO_FILL = 1, /* bwd also writes zeros into rows that carry no gradient                */
  GTO_FLAG_TARGET_PRUNE = 2    /* gto_tree_reward streams only the target rows the kept tree refers to:
                                  slots with tree->slot_need == 0 are skipped and their entries in the
                                  target statistics are left untouched                                 */
};

typedef struct gto_config {
  int32_t R, d, k, g, V;
  int32_t dtype;        /* element type of all logits tensors                              */
  int64_t row_stride;   /* elements between consecutive rows, >= V                         */
  int32_t group_size;   /* m of Eq. 6: consecutive roots per group                         */
  int32_t reward_mode;  /* which aggregate feeds `reward` (all four are always computed)   */
  float eta;            /* smooth-max temperature of Eq. 5 (paper: 1)                      */
  float eps;            /* clip range of Eq. 12                                            */
  float delta;          /* std floor of Eq. 10                                             */
  float grad_scale;     /* upstream dL/dL_GTO (the paper's omega = 0.5 in Eq. 13)          */
  int32_t flags;        /* GTO_FLAG_*                                                      */
  int32_t path_mode;    /* GTO_PATH_*: which sequence the surrogate is taken along           */
  /* Tuning, per call; 0 everywhere = the library's own choice.  Results never depend on these
   * (bit for bit for ids; the fused variant's floats within its usual tolerance).            */
  int32_t waves_per_row;  /* wavefronts sharing one logits row in the row kernels: 0 (chosen per
                             launch from V and the number of rows), 1, 2, 4 or 8; else GTO_E_MODE */
  int32_t fused_groups;   /* fused variant: groups of workgroups the row pass is launched with, 0 (= 8: one
                             group per XCD, one workgroup per compute unit) .. 16 (8 with fused_layout 1);
                             else GTO_E_MODE.  Sizes the fused workspace.                          */
  int32_t fused_layout;   /* fused variant: a group is 0 = 8 row blocks x 4 column tiles of workgroups
                             (the library's choice), 1 = 4 x 8                                     */
  int32_t reserved;       /* must be 0                                                          */
} gto_config;

/* Row statistics of a draft-logits tensor.  Entries of padding slots are not written. */
typedef struct gto_draft_stats {
  float *row_max;    /* [R, d, k]     max logit of the row                                  */
  float *row_lse;    /* [R, d, k]     log sum exp of the row                                */
  int32_t *top_tok;  /* [R, d, k, k]  k best tokens: logit descending, token id ascending   */
  float *top_logp;   /* [R, d, k, k]  their log-probabilities (full-vocabulary softmax)     */
} gto_draft_stats;

typedef struct gto_target_stats {
  float *t_max;      /* [R, d, k] */
  float *t_lse;      /* [R, d, k] */
  int32_t *t_argmax; /* [R, d, k] lowest token id attaining the max */
} gto_target_stats;

/* Candidate pool of one expansion, all [R, C] unless noted. */
typedef struct gto_pool {
  int32_t *cand_tok;
  int32_t *cand_parent; /* pool index of the parent, -1 for depth-1 nodes                  */
  int32_t *cand_depth;  /* 1..d                                                             */
  int32_t *cand_pslot;  /* slot j (within level depth-1) of the parent                      */
  int32_t *cand_slot;   /* slot the node itself occupies at level depth if expanded, else -1 */
  float *cand_score;    /* cumulative draft log-probability from the root (fp32 adds)       */
  int32_t *slot_cand;   /* [R, d, k] pool index expanded in each slot; level 0: -1          */
} gto_pool;

/* Kept tree, all [R, g]; positions >= n_sel hold -1 (ints) / 0 (score). */
typedef struct gto_tree {
  int32_t *sel_cand;   /* pool index                                                       */
  int32_t *sel_tok;
  int32_t *sel_parent; /* position of the parent in this list, -1 for depth-1 nodes        */
  int32_t *sel_depth;
  int32_t *sel_pslot;
  int32_t *sel_slot;
  int32_t *sel_leaf;   /* 1 if no kept child                                               */
  float *sel_score;
  int32_t *n_sel;      /* [R] = min(g, C)                                                  */
  int32_t *slot_need;  /* [R, d, k] 1 if the slot's node has a kept child (its target row is needed) */
} gto_tree;

typedef struct gto_reward {
  float *node_q;       /* [R, g] target probability that the path up to the node is accepted */
  float *node_cum;     /* [R, g] sum of node_q along the path = L of Eq. 3 at a leaf        */
  float *reward;       /* [R]    the aggregate chosen by cfg->reward_mode                   */
  float *reward_aux;   /* [R, 4] lse (Eq. 5), max, mean, nodesum, in GTO_REWARD_* order     */
  int32_t *n_leaves;   /* [R]    number of root-to-leaf sequences N                         */
  int32_t *path_len;   /* [R]    length l of the longest accepted sequence, 0..d            */
  int32_t *path_node;  /* [R, d] its nodes as positions in the kept list, -1 beyond l       */
  int32_t *path_slot;  /* [R, d] slot (within level t) of the node whose row produced step t */
  const float *accept_u; /* in, [R, d, k]: uniform numbers in [0, 1) for GTO_PATH_SAMPLED; entry (r, t, j)
                            decides the j-th child tried at step t.  Not read (may be NULL) in the other
                            path modes; GTO_E_NULL if it is NULL in that mode.                          */
} gto_reward;

typedef struct gto_ppo {
  float *logM;        /* [R] log-probability of the accepted sequence under the current draft */
  float *logM0;       /* [R] ... under the reference draft                                  */
  float *ratio;       /* [R] s_i of Eq. 11                                                  */
  float *term;        /* [R] min(s A, clip(s) A)                                            */
  int32_t *active;    /* [R] 1 if a gradient flows (l > 0 and the unclipped branch is the min) */
  float *coef;        /* [R] c_i multiplying (onehot - softmax) in the backward             */
  float *loss_group;  /* [R / group_size] Eq. 12 per group                                  */
  float *loss;        /* [1] mean of the group losses                                       */
} gto_ppo;

int gto_version(void);
/* Static text for a status; for GTO_E_HIP the text of the last HIP error seen by this thread. */
const char *gto_strerror(int status);
/* Host only.  Bytes of device workspace the calls below may need for `cfg` (256-byte aligned). */
int gto_workspace_bytes(const gto_config *cfg, size_t *bytes_out);

/* Per-row statistics of draft logits: max, log-sum-exp, and the k most probable tokens with
 * their log-probabilities under the full-vocabulary softmax (Fig. 1 caption: the number on an
 * edge is the draft probability of that token; App. B.3: top-k per node, k = 10).  One pass
 * over every used row. */
int gto_draft_row_stats(const gto_config *cfg, const void *draft_logits,
                        const gto_draft_stats *stats_out, void *hip_stream);

/* Per-row statistics of target logits needed by Eq. 3-4 and by greedy verification. */
int gto_target_row_stats(const gto_config *cfg, const void *target_logits,
                         const gto_target_stats *stats_out, void *hip_stream);

/* Stage (i) of the decoding policy G (Sec. 3.1, "Layer-wise expansion"; Fig. 1 caption for
 * the score): gto_draft_row_stats, then the level-by-level expansion.  A candidate's global
 * acceptance score is score(parent) + log-probability (fp32 add; root = 0); at every level
 * below the last the k best of the k^2 children (score descending, pool index ascending)
 * become the next level's slots, in that order.  `workspace` is unused by this call (no scratch
 * memory is needed): it may be NULL and workspace_bytes 0; the pair is there so that every one of
 * the six calls has the same shape. */
int gto_expand_tree(const gto_config *cfg, const void *draft_logits,
                    const gto_draft_stats *stats_out, const gto_pool *pool_out,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* The expansion alone, from row statistics already on the device. */
int gto_expand_from_stats(const gto_config *cfg, const gto_draft_stats *stats,
                          const gto_pool *pool_out, void *hip_stream);

/* Stage (ii) of G (Sec. 3.1, "Global pruning and re-ranking"; App. B.1: budget of 60
 * draft tokens): rank all C candidates by (score descending, pool index ascending), keep the
 * first min(g, C) in that order, remap parents, flag leaves. */
int gto_select_topg(const gto_config *cfg, const gto_pool *pool, const gto_tree *tree_out,
                    void *hip_stream);

/* Draft Tree Reward (Eq. 2-5; Max / Mean of the aggregation ablation; App. A Eq. (2) as
 * `nodesum`) and the longest accepted sequence under greedy target verification (Sec. 3.2,
 * Algorithm 1; App. A case T = 0).  Runs gto_target_row_stats, then the per-root scan.
 * `workspace` is unused by this call: it may be NULL and workspace_bytes 0. */
int gto_tree_reward(const gto_config *cfg, const gto_tree *tree, const void *target_logits,
                    const gto_target_stats *stats_out, const gto_reward *reward_out,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* The per-root reward scan alone, from target statistics already on the device. */
int gto_reward_from_stats(const gto_config *cfg, const gto_tree *tree, const void *target_logits,
                          const gto_target_stats *stats, const gto_reward *reward_out,
                          void *hip_stream);

/* Eq. 9-10: adv = (Rdeb - mean) / (std + delta) within groups of cfg->group_size consecutive
 * roots, Rdeb = reward_cur - reward_ref, population std.  reward_ref == NULL skips the
 * debiasing (the paper's "w/o Debiasing" ablation). */
int gto_group_advantage(const gto_config *cfg, const float *reward_cur, const float *reward_ref,
                        float *adv_out, void *hip_stream);

/* Eq. 11-12 on the longest accepted sequence of the current tree.  `ref_logits_on_cur` holds
 * the reference draft model's logits at the same slot coordinates as `draft_logits_cur`.
 * `ref_stats` may be NULL: then the log-sum-exp of the (at most d) reference rows on each path
 * is computed here into `workspace`. */
int gto_ppo_surrogate_fwd(const gto_config *cfg, const gto_tree *tree_cur,
                          const gto_reward *path_cur, const void *draft_logits_cur,
                          const gto_draft_stats *draft_stats_cur, const void *ref_logits_on_cur,
                          const gto_draft_stats *ref_stats, const float *adv,
                          const gto_ppo *out, void *workspace, size_t workspace_bytes,
                          void *hip_stream);

/* gto_ppo_surrogate_fwd for callers that cannot allocate device memory and therefore have no
 * workspace to pass: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same outputs as gto_ppo_surrogate_fwd called with ref_stats == NULL (the reference
 * rows' log-sum-exps are recomputed for the rows on the accepted paths), bit for bit; the [R, d]
 * floats of scratch memory live in a static device array inside the library (256 KiB, held by every
 * GPU the library runs on until the process ends).  The call allocates nothing and frees nothing.
 *   - Limit: R * d <= 65536, else GTO_E_WORKSPACE (nothing is launched).
 *   - The first call on a device looks up the array's address on that device (a host-side query, no
 *     allocation); make one call on each device before recording calls into a graph.
 *   - All calls on one GPU share that GPU's array, which keeps the last call's contents.  Nothing
 *     in it has to start at zero: each call writes every entry it later reads.  Two calls that
 *     overlap in time on one GPU (different streams without ordering) race on it: order them. */
int gto_ppo_surrogate_fwd_noalloc(const gto_config *cfg, const gto_tree *tree_cur,
                                  const gto_reward *path_cur, const void *draft_logits_cur,
                                  const gto_draft_stats *draft_stats_cur, const void *ref_logits_on_cur,
                                  const float *adv, const gto_ppo *out, void *hip_stream);

/* Gradient of cfg->grad_scale * loss w.r.t. the current draft logits (derivative of Eq. 11-12
 * with the advantage and the tree held constant): for step t < l_i of root i,
 *   grad_rows[i, t, v] = coef_i * (1[v == token_t] - softmax(row)[v]),
 * the row being slot grad_slot[i, t] of level t.  grad_rows is [R, d, V] fp32 (dense, row
 * length V); grad_slot is [R, d], -1 where the row carries no gradient (t >= l_i or
 * coef_i == 0).  Such rows are left untouched unless GTO_FLAG_GRAD_ZERO_FILL is set. */
int gto_ppo_surrogate_bwd(const gto_config *cfg, const gto_tree *tree_cur,
                          const gto_reward *path_cur, const gto_ppo *fwd,
                          const void *draft_logits_cur, const gto_draft_stats *draft_stats_cur,
                          float *grad_rows, int32_t *grad_slot, void *hip_stream);

/* Token-level loss of Eq. 13 / App. B.2: mean over the supervised positions of the cross-entropy
 * H(p_T, p_M) = -sum_v p_T(v) log p_M(v) from the target's to the draft's next-token distribution under
 * the same teacher-forced prefix, i.e. at the root slot (0, 0) of every root.  The row statistics must
 * hold the lse of slot (0, 0) of both tensors (gto_expand_tree / gto_tree_reward leave them there, also
 * with target pruning).  `weight_or_null` [R] selects the supervised positions (1 / 0; NULL = all).
 * Forward: loss_rows [R], loss [1] and inv_count [1] = 1 / |I|.  Backward: grad_rows0 [R, V] fp32 =
 * grad_scale * weight / |I| * (softmax(draft) - softmax(target)), the gradient of grad_scale * loss
 * w.r.t. the draft logits of slot (0, 0). */
int gto_token_loss_fwd(const gto_config *cfg, const void *draft_logits, const void *target_logits,
                       const gto_draft_stats *draft_stats, const gto_target_stats *target_stats,
                       const float *weight_or_null, float *loss_rows, float *loss, float *inv_count,
                       void *hip_stream);
int gto_token_loss_bwd(const gto_config *cfg, const void *draft_logits, const void *target_logits,
                       const gto_draft_stats *draft_stats, const gto_target_stats *target_stats,
                       const float *weight_or_null, const float *inv_count, float grad_scale, float *grad_rows0,
                       void *hip_stream);

/* ---- Fused LM-head variant (the fifth workload: logits never reach HBM) -------------------------
 * The logits of slot (l, j) of root r are hidden[r, l, j, :] . w_vh[v, :] for v < V, accumulated in
 * fp32 on the matrix cores and consumed as fp32 (never rounded to bf16).  `hidden` is bf16
 * [R, d, k, hidden_dim]; `w_vh` is the LM-head weight bf16 [V, hidden_dim] (vocabulary-major, the
 * layout a linear layer stores).  Requirements: cfg->dtype == GTO_BF16, k <= 16, hidden_dim a
 * multiple of 64, both pointers 16-byte aligned.  `workspace` (device, 256-byte aligned) must hold
 * gto_fused_workspace_bytes(cfg, hidden_dim) bytes. */
int gto_fused_workspace_bytes(const gto_config *cfg, int32_t hidden_dim, size_t *bytes_out);

/* Same outputs as gto_draft_row_stats / gto_target_row_stats, from hidden states and the LM head.
 * `top_logit_or_null` [R, d, k, k] optionally receives the fp32 logits of the top-k tokens. */
int gto_fused_draft_row_stats(const gto_config *cfg, const void *hidden, int32_t hidden_dim, const void *w_vh,
                              const gto_draft_stats *stats_out, float *top_logit_or_null, void *workspace,
                              size_t workspace_bytes, void *hip_stream);
int gto_fused_target_row_stats(const gto_config *cfg, const void *hidden, int32_t hidden_dim, const void *w_vh,
                               const gto_target_stats *stats_out, void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/* gto_expand_tree / gto_tree_reward / gto_ppo_surrogate_fwd with the logits produced on the fly.
 * Single logits that the reward (kept tokens under the target) and the surrogate (path tokens under
 * the current and the reference draft) need are recomputed as fp32 dot products.  In the surrogate,
 * `hidden_ref_on_cur` holds the reference model's hidden states at the current tree's slot
 * coordinates and `ref_stats` (required) its row statistics under the same draft head. */
int gto_expand_tree_fused(const gto_config *cfg, const void *hidden, int32_t hidden_dim, const void *w_draft_vh,
                          const gto_draft_stats *stats_out, const gto_pool *pool_out, void *workspace,
                          size_t workspace_bytes, void *hip_stream);
int gto_tree_reward_fused(const gto_config *cfg, const gto_tree *tree, const void *hidden, int32_t hidden_dim,
                          const void *w_target_vh, const gto_target_stats *stats_out,
                          const gto_reward *reward_out, void *workspace, size_t workspace_bytes,
                          void *hip_stream);
int gto_ppo_surrogate_fwd_fused(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                                const void *hidden_cur, const void *hidden_ref_on_cur, int32_t hidden_dim,
                                const void *w_draft_vh, const gto_draft_stats *draft_stats_cur,
                                const gto_draft_stats *ref_stats, const float *adv, const gto_ppo *out,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/* gto_ppo_surrogate_bwd with the logits of the path rows recomputed on the matrix cores: same
 * grad_rows [R, d, V] / grad_slot [R, d] outputs and flag semantics.  Only the (root, step) pairs
 * that carry a gradient are multiplied. */
int gto_ppo_surrogate_bwd_fused(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                                const gto_ppo *fwd, const void *hidden_cur, int32_t hidden_dim,
                                const void *w_draft_vh, const gto_draft_stats *draft_stats_cur, float *grad_rows,
                                int32_t *grad_slot, void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same backward, carried on to the hidden states (the chain rule through logits = hidden . W^T;
 * Eq. 11-12 for the surrogate): dh_rows[r, t, :] = sum_v G[r, t, v] w_draft[v, :] with G the gradient
 * row gto_ppo_surrogate_bwd_fused would write, for the slot grad_slot[r, t] of level t.  The fp32
 * gradient rows are not written; -coef * softmax of each path row is staged in the workspace as two
 * bf16 planes (value = hi + lo, relative error <= 2^-16 per entry), contracted with the head on the
 * matrix cores in fp32; the accepted token's own term coef * (1 - p_token) * w_draft[token, :] is added
 * afterwards with 1 - p_token formed as the sum of the other probabilities (no cancellation).
 *   w_draft_hv : the same head, hidden-major: bf16 [hidden_dim, V] (w_draft_hv[h, v] = w_draft_vh[v, h]);
 *                the caller keeps this second copy so that both operands are contiguous along the vocabulary
 *   dh_rows    : out, fp32 [R, d, hidden_dim]; rows with grad_slot = -1 or a zero coefficient are left
 *                untouched (zeroed with GTO_FLAG_GRAD_ZERO_FILL)
 * Requires V % 32 == 0 (GTO_E_SHAPE otherwise) and a workspace of gto_fused_dh_workspace_bytes. */
int gto_fused_dh_workspace_bytes(const gto_config *cfg, int32_t hidden_dim, size_t *bytes_out);
int gto_ppo_surrogate_bwd_fused_dh(const gto_config *cfg, const gto_tree *tree_cur, const gto_reward *path_cur,
                                   const gto_ppo *fwd, const void *hidden_cur, int32_t hidden_dim,
                                   const void *w_draft_vh, const void *w_draft_hv,
                                   const gto_draft_stats *draft_stats_cur, float *dh_rows, int32_t *grad_slot,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/* Token-level loss (Eq. 13, App. B.2) of the fused variant.  The root-row logits of the draft and the
 * target head are produced on the matrix cores and kept in the workspace as fp32 [R, V] each (the
 * root rows are 1 / rho of all rows; every other logit still never reaches HBM), then reduced by the
 * kernels of gto_token_loss_fwd / _bwd.  draft_stats->row_lse and target_stats->t_lse must hold the
 * root slots' log-sum-exps (gto_expand_tree_fused / gto_tree_reward_fused write them).  The backward
 * reads the logits the forward left in `workspace`: same buffer, untouched in between.  Outputs and
 * weight / inv_count / grad_scale semantics as in the streaming calls. */
int gto_fused_token_loss_workspace_bytes(const gto_config *cfg, int32_t hidden_dim, size_t *bytes_out);
int gto_token_loss_fwd_fused(const gto_config *cfg, const void *hidden, int32_t hidden_dim, const void *w_draft_vh,
                             const void *w_target_vh, const gto_draft_stats *draft_stats,
                             const gto_target_stats *target_stats, const float *weight_or_null, float *loss_rows,
                             float *loss, float *inv_count, void *workspace, size_t workspace_bytes,
                             void *hip_stream);
int gto_token_loss_bwd_fused(const gto_config *cfg, const gto_draft_stats *draft_stats,
                             const gto_target_stats *target_stats, const float *weight_or_null,
                             const float *inv_count, float grad_scale, float *grad_rows0, const void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* Measurement aid, not part of the method: copies `bytes` (a multiple of 16; both device pointers
 * 16-byte aligned, non-overlapping) with a plain kernel.  Hardware HBM counters of the row kernels
 * are scaled by what the same counters report for this copy of known size. */
int gto_calibration_copy(const void *src, void *dst, size_t bytes, void *hip_stream);

/* Optional per-kernel timing.  While enabled, every kernel launch of the calling thread is
 * bracketed by two HIP events recorded on its stream; the events come from a per-thread pool
 * that gto_profile_enable(1) fills (the only place where events are created), so nothing is
 * created inside a timed region.  At most 16384 launches are kept between two reads; further
 * ones are not timed.  gto_profile_read synchronises the recorded events, returns them to the
 * pool and reports, for up to `cap` distinct kernels, the name, the number of launches and the
 * summed duration in milliseconds since the last read; it returns the number of kernels written.
 * gto_profile_enable(0) stops recording; the pool lives until the thread ends. */
int gto_profile_enable(int on);
int gto_profile_read(const char **names, int32_t *launches, double *total_ms, int cap);
/* Restricts the timing to the kernel of one name (the names gto_profile_read reports, e.g.
 * "row_stats_draft"); NULL = every kernel again.  Two event records per launch leave a few
 * microseconds between consecutive kernels, which a timed region that only needs one kernel's
 * duration can do without.  Per calling thread, like the rest of the profiling state. */
int gto_profile_filter(const char *kernel_name_or_null);

#ifdef __cplusplus
}
#endif
#endif /* GTO_H */
