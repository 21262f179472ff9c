// Kernel argument blocks and host-side launchers (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gto {

struct RowStatsArgs {
  const void *logits;
  int64_t row_stride;
  int V, d, kslots, ktop, rho;
  int waves;                 // wavefronts per row: 0 = chosen per launch, else 1, 2, 4 or 8
  const int32_t *path_slot;  // null: all used slots; else rows (root, step) on an accepted path
  const int32_t *row_need;   // optional [R, d, kslots]: rows whose flag is 0 are skipped
  float *row_max;            // may be null
  float *row_lse;
  int32_t *top_tok;          // may be null (then no top-k output)
  float *top_logp;           // may be null
};

struct PpoBwdArgs {
  const void *logits;
  int64_t row_stride;
  int V, d, k, g;
  const int32_t *path_slot, *path_node, *sel_tok;
  const float *coef, *row_lse;
  float *grad_rows;
  int32_t *grad_slot;
  int zero_fill;
};

struct ExpandArgs {
  int R, d, k, C;
  const int32_t *top_tok;
  const float *top_logp;
  int32_t *cand_tok, *cand_parent, *cand_depth, *cand_pslot, *cand_slot;
  float *cand_score;
  int32_t *slot_cand;
};

struct SelectArgs {
  int R, C, g, d, k;
  const int32_t *cand_tok, *cand_parent, *cand_depth, *cand_pslot, *cand_slot;
  const float *cand_score;
  int32_t *sel_cand, *sel_tok, *sel_parent, *sel_depth, *sel_pslot, *sel_slot, *sel_leaf;
  float *sel_score;
  int32_t *n_sel, *slot_need;
};

struct RewardArgs {
  int R, d, k, g, V, dtype, reward_mode, path_mode;
  int64_t row_stride;
  float eta;
  const void *target_logits;
  const float *node_logit;   // optional [R, g]: logits of the kept tokens gathered beforehand (fused variant)
  const float *t_lse;
  const int32_t *t_argmax;
  const float *accept_u;     // [R, d, k] uniform numbers of the sampled walk (path_mode 2 only)
  const int32_t *sel_tok, *sel_parent, *sel_depth, *sel_pslot, *sel_slot, *sel_leaf, *n_sel;
  float *node_q, *node_cum, *reward, *reward_aux;
  int32_t *n_leaves, *path_len, *path_node, *path_slot;
};

struct AdvArgs {
  int R, m;
  float delta;
  const float *r_cur, *r_ref;  // r_ref may be null
  float *adv;
};

struct PpoFwdArgs {
  int R, d, k, g, m, dtype, V;
  int64_t row_stride;
  float eps, grad_scale;
  const void *draft_logits, *ref_logits;
  const float *path_logit_cur, *path_logit_ref;   // optional [R, d]: gathered beforehand (fused variant)
  const float *draft_lse;   // [R, d, k]
  const float *ref_lse;     // [R, d, k] if ref_lse_by_step == 0, else [R, d]
  int ref_lse_by_step;
  const int32_t *sel_tok, *path_len, *path_node, *path_slot;
  const float *adv;
  float *logM, *logM0, *ratio, *term, *coef, *loss_group, *loss;
  int32_t *active;
};

struct FusedArgs {
  const void *hidden;        // bf16 [R, d, kslots, hidden_dim]
  const void *w;             // bf16 [V, hidden_dim]
  int hidden_dim, V, rho, d, kslots, ktop;
  int64_t M;                 // rows processed (used slots, or capacity of row_list)
  const int32_t *m_dev;      // optional: actual row count in device memory (<= M)
  const int32_t *row_list;   // optional: slot index of each processed row
  int out_by_list;           // with row_list: statistics are written at the list position, not at the slot
  int n_tiles;               // column tiles of 256 tokens
  int groups, patch_rows, patch_cols;   // launch geometry: groups x (patch_rows x patch_cols) workgroups;
                             // n_slots = groups * patch_cols partial results per row (<= 64)
  float *part_m, *part_c;    // [M, n_slots]
  double *part_s;            // [M, n_slots]
  float *part_v;             // [M, n_slots, ktop]
  int32_t *part_i;           // [M, n_slots, ktop]
  float *row_max, *row_lse;  // final statistics (row_max may be null)
  int32_t *top_tok;          // may be null
  float *top_logp, *top_logit;  // may be null
  // backward mode (grad_rows != null): rows come from row_list (hidden slots) / list_p ((root, step))
  const int32_t *list_p, *sel_tok, *path_node;
  const float *coef, *lse_by_slot;
  int g;
  float *grad_rows;          // [R, d, V]
  // plane mode (plane_hi != null, instead of grad_rows): -coef * softmax of row i of the list is split
  // into two bf16 planes [M, V] (value = hi + lo; zero at the accepted token), the row operand of the
  // hidden-state gradient; part_s receives the sum of the other probabilities as in the backward mode
  uint16_t *plane_hi, *plane_lo;
  // store mode (store_rows != null): the fp32 logits of row i of the processed rows go to store_rows[i, :V]
  float *store_rows;
  int64_t store_pitch;
};

// Hidden-state gradient dH = G . W of the fused variant: G = the two bf16 planes, W hidden-major.
struct FusedDhArgs {
  const uint16_t *plane_hi, *plane_lo;   // [M, V]
  const void *w_hv;          // bf16 [hidden_dim, V]
  const void *w_vh;          // bf16 [V, hidden_dim] (row of the accepted token, added exactly)
  int hidden_dim, V, d, g;
  int64_t M;                 // capacity of the row list
  const int32_t *m_dev;      // actual row count
  int m_blocks, h_blocks, n_splits, slabs_per_split;
  float *partial;            // [n_splits, M, hidden_dim]
  const double *part_s;      // [M, n_slots] sum of the non-token probabilities per segment of the plane pass
  int n_tiles, groups, patch_rows, patch_cols;   // geometry of the plane pass (which slots hold a result)
  const int32_t *list_p, *sel_tok, *path_node;
  const float *coef;
  float *dh_rows;            // [R, d, hidden_dim]
};

struct BwdRowsArgs {
  int R, d, k;
  const int32_t *path_slot;
  const float *coef;
  int32_t *grad_slot, *list_p, *list_slot, *count;
};

struct GatherDotArgs {
  const void *hidden, *w;
  int hidden_dim, V;
  int64_t n;
  const int64_t *slot;       // [n] slot index of the hidden row, < 0: skip
  const int32_t *tok;        // [n]
  float *out;                // [n]
};

struct PairArgs {
  int R, d, k, g;
  const int32_t *sel_tok, *sel_depth, *sel_pslot, *n_sel;      // kept nodes (mode 0)
  const int32_t *path_slot, *path_node;                       // path steps (mode 1)
  int64_t *slot;
  int32_t *tok;
};
void launch_pairs(const PairArgs &a, int mode, hipStream_t st);
void launch_fused_rows(const FusedArgs &a, hipStream_t st);
void launch_fused_bwd_fixup(const FusedArgs &a, hipStream_t st);
void launch_fused_dh(const FusedDhArgs &a, hipStream_t st);
void launch_bwd_rows(const BwdRowsArgs &a, hipStream_t st);
void launch_zero_rows(float *grad_rows, const int32_t *grad_slot, int rows, int V, hipStream_t st);
void launch_compact_flags(const int32_t *flags, int n, int32_t *list, int32_t *count, hipStream_t st);
void launch_fused_merge(const FusedArgs &a, hipStream_t st);
void launch_gather_dot(const GatherDotArgs &a, hipStream_t st);
struct TokenLossArgs {
  int R, d, k, V;
  int64_t row_stride;
  int64_t root_stride;             // 0: root rows sit at slot (0,0) of [R, d, k, row_stride]; else elements between
                                   // consecutive roots' rows in a compact [R, root_stride] layout
  const void *draft_logits, *target_logits;
  const float *d_lse, *t_lse;      // [R, d, k] statistics (entry of slot (0,0) is used)
  const float *weight;             // optional [R]
  float grad_scale;
  float *loss_rows, *loss, *inv_count_out;   // forward outputs: [R], [1], [1] = 1 / |I|
  const float *inv_count;          // backward input: the forward's 1 / |I|
  float *grad;                     // backward output [R, V]
};
void launch_token_loss(const TokenLossArgs &a, int dtype, bool bwd, hipStream_t st);
void launch_row_stats(const RowStatsArgs &a, int dtype, int blocks, hipStream_t st);
void launch_ppo_bwd(const PpoBwdArgs &a, int dtype, int blocks, hipStream_t st);
void launch_copy16(const void *src, void *dst, int64_t bytes, hipStream_t st);
void launch_expand(const ExpandArgs &a, hipStream_t st);
void launch_select(const SelectArgs &a, hipStream_t st);
void launch_reward(const RewardArgs &a, hipStream_t st);
void launch_advantage(const AdvArgs &a, hipStream_t st);
void launch_ppo_fwd(const PpoFwdArgs &a, hipStream_t st);

}  // namespace gto
