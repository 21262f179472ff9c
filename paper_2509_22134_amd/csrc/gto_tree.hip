// Per-root kernels of the GTO hot path: layer-wise expansion, global re-rank, reward scan and
// greedy verification walk, group advantage, clipped surrogate forward.  All of them work on a
// few KB per root that live in LDS; they are latency-bound and tiny next to the row kernels.
//
// Ranking everywhere is on a packed 64-bit key (order-preserving bits of the fp32 score, then the
// inverted index): keys are unique, so (score descending, index ascending) is realised exactly and
// deterministically whether a rank is found by counting the keys that beat mine (expansion: k^2
// keys per level) or by sorting (top-g: C keys).
#include "gto_device.h"
#include "gto_kernels.h"

namespace gto {

constexpr int kTreeThreads = 256;
constexpr int kMaxPool = 4096;        // C

__device__ __forceinline__ uint64_t rank_key(float score, int index) {
  return ((uint64_t)ordered_bits(score) << 32) | (uint32_t)(0xffffffffu - (uint32_t)index);
}

// ------------------------------------------------------------------------------ expansion
// Which rows feed which candidate is fixed by the shape (candidate c of the pool is child rk of slot j of
// level l), so every log-probability and token of the root is fetched up front in one round of loads; the
// level loop then runs out of LDS and only stores to memory.
// Dynamic LDS: k^2 keys rounded up to a multiple of eight (8 B each), C log-probabilities (4 B).
__global__ __launch_bounds__(kTreeThreads) void k_expand(ExpandArgs a) {
  const int r = blockIdx.x;
  const int k = a.k, d = a.d, kk = a.k * a.k, C = a.C;
  const int tid = threadIdx.x;
  extern __shared__ __align__(16) unsigned char s_dyn[];
  const int kk8 = (kk + 7) & ~7;
  uint64_t *s_key = reinterpret_cast<uint64_t *>(s_dyn);
  float *s_lp = reinterpret_cast<float *>(s_key + kk8);
  __shared__ float s_score[2][64];
  __shared__ int s_cand[2][64];
  const int64_t pool0 = (int64_t)r * C;
  const int64_t slot0 = (int64_t)r * d * k;

  for (int t = kk + tid; t < kk8; t += kTreeThreads) s_key[t] = 0ull;
  for (int c = tid; c < C; c += kTreeThreads) {
    int l = 0, j = 0, rk = c;
    if (c >= k) {
      const int q = c - k;
      l = 1 + q / kk;
      const int t = q - (l - 1) * kk;
      j = t / k;
      rk = t - j * k;
    }
    const int64_t si = stat_index(r, l, j, d, k) * k + rk;
    s_lp[c] = a.top_logp[si];
    a.cand_tok[pool0 + c] = a.top_tok[si];
    a.cand_depth[pool0 + c] = l + 1;
    a.cand_pslot[pool0 + c] = j;
  }
  __syncthreads();
  // level 0: the root's k children, all expanded at level 1 in rank order
  for (int t = tid; t < k; t += kTreeThreads) {
    const float sc = __fadd_rn(0.f, s_lp[t]);
    a.cand_parent[pool0 + t] = -1;
    a.cand_score[pool0 + t] = sc;
    a.cand_slot[pool0 + t] = (d > 1) ? t : -1;
    a.slot_cand[slot0 + t] = -1;
    if (d > 1) a.slot_cand[slot0 + k + t] = t;
    s_score[1][t] = sc;
    s_cand[1][t] = t;
  }
  __syncthreads();
  for (int l = 1; l < d; ++l) {
    const int cur = l & 1, nxt = cur ^ 1;
    const int base = k + (l - 1) * kk;
    for (int t = tid; t < kk; t += kTreeThreads) {
      const int j = t / k;
      const float sc = __fadd_rn(s_score[cur][j], s_lp[base + t]);
      const int c = base + t;
      a.cand_parent[pool0 + c] = s_cand[cur][j];
      a.cand_score[pool0 + c] = sc;
      s_key[t] = rank_key(sc, t);
      if (l == d - 1) a.cand_slot[pool0 + c] = -1;
    }
    if (l == d - 1) break;
    __syncthreads();
    for (int t = tid; t < kk; t += kTreeThreads) {
      const uint64_t mine = s_key[t];
      int rank = 0;
      // eight keys per trip (the list is padded with zeros, which beat nothing): the reads of a trip are
      // independent, one key per trip would pay the LDS latency kk times
      for (int u = 0; u < kk8; u += 8) {
        uint64_t q[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] = s_key[u + e];
#pragma unroll
        for (int e = 0; e < 8; ++e) rank += (q[e] > mine) ? 1 : 0;
      }
      const int c = base + t;
      if (rank < k) {
        // the same add as above gives the same bits; s_score[nxt] was last read before the previous barrier
        s_score[nxt][rank] = __fadd_rn(s_score[cur][t / k], s_lp[base + t]);
        s_cand[nxt][rank] = c;
        a.slot_cand[slot0 + (int64_t)(l + 1) * k + rank] = c;
        a.cand_slot[pool0 + c] = rank;
      } else {
        a.cand_slot[pool0 + c] = -1;
      }
    }
    __syncthreads();
  }
}

void launch_expand(const ExpandArgs &a, hipStream_t st) {
  const size_t lds = (size_t)((a.k * a.k + 7) & ~7) * 8 + (size_t)a.C * 4;
  hipLaunchKernelGGL(k_expand, dim3(a.R), dim3(kTreeThreads), lds, st, a);
}

// ------------------------------------------------------------------------------ top-g
// The C candidates of a root are sorted by their (unique) keys with a bitonic network over the next power of
// two, padded with key 0 (below every real key: the low word of a real key is never 0).  Position i of the
// sorted list is rank i; comparing every key with every other one, as the expansion does for its k^2 keys,
// costs C^2 = 260 k compares per root at C = 510 and made this kernel ALU bound.
// Dynamic LDS: n_pad keys (8 B), C ranks (4 B), n_keep leaf flags, d * k need flags.
__device__ __forceinline__ int select_pad(int C) {
  int n = 2;
  while (n < C) n <<= 1;
  return n;
}

__global__ __launch_bounds__(kTreeThreads) void k_select(SelectArgs a) {
  const int r = blockIdx.x, tid = threadIdx.x;
  const int C = a.C, g = a.g;
  const int n_keep = (g < C) ? g : C;
  const int n_pad = select_pad(C);
  extern __shared__ __align__(16) unsigned char s_dyn[];
  uint64_t *s_key = reinterpret_cast<uint64_t *>(s_dyn);
  int *s_rank = reinterpret_cast<int *>(s_key + n_pad);
  unsigned char *s_leaf = reinterpret_cast<unsigned char *>(s_rank + C);
  unsigned char *s_need = s_leaf + n_keep;
  const int64_t pool0 = (int64_t)r * C;
  const int64_t sel0 = (int64_t)r * g;
  for (int c = tid; c < n_pad; c += kTreeThreads) s_key[c] = (c < C) ? rank_key(a.cand_score[pool0 + c], c) : 0ull;
  for (int i = tid; i < n_keep; i += kTreeThreads) s_leaf[i] = 1;
  for (int i = tid; i < a.d * a.k; i += kTreeThreads) s_need[i] = 0;
  __syncthreads();
  // descending bitonic sort
  for (int size = 2; size <= n_pad; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = tid; t < (n_pad >> 1); t += kTreeThreads) {
        const int lo = 2 * t - (t & (stride - 1));
        const int hi = lo + stride;
        const bool desc = (lo & size) == 0;
        const uint64_t x = s_key[lo], y = s_key[hi];
        if ((x < y) == desc) {
          s_key[lo] = y;
          s_key[hi] = x;
        }
      }
      __syncthreads();
    }
  }
  for (int i = tid; i < C; i += kTreeThreads) s_rank[(int)(0xffffffffu - (uint32_t)s_key[i])] = i;
  __syncthreads();
  for (int c = tid; c < C; c += kTreeThreads) {
    const int p = a.cand_parent[pool0 + c];
    if (s_rank[c] < n_keep && p >= 0) {
      const int pr = s_rank[p];
      if (pr < n_keep) s_leaf[pr] = 0;  // a kept child: the parent is not a leaf
    }
    // the row that produced a kept node is needed by the reward
    if (s_rank[c] < n_keep) s_need[(a.cand_depth[pool0 + c] - 1) * a.k + a.cand_pslot[pool0 + c]] = 1;
  }
  __syncthreads();
  // the kept candidates, straight from the sorted list
  for (int i = tid; i < n_keep; i += kTreeThreads) {
    const int c = (int)(0xffffffffu - (uint32_t)s_key[i]);
    const int p = a.cand_parent[pool0 + c];
    a.sel_cand[sel0 + i] = c;
    a.sel_tok[sel0 + i] = a.cand_tok[pool0 + c];
    // a parent always outranks its child (log-probabilities are <= 0); the range check only matters for
    // rows that held NaNs, whose values are unspecified but whose indices must stay inside the list
    a.sel_parent[sel0 + i] = (p >= 0 && s_rank[p] < i) ? s_rank[p] : -1;
    a.sel_depth[sel0 + i] = a.cand_depth[pool0 + c];
    a.sel_pslot[sel0 + i] = a.cand_pslot[pool0 + c];
    a.sel_slot[sel0 + i] = a.cand_slot[pool0 + c];
    a.sel_score[sel0 + i] = a.cand_score[pool0 + c];
    a.sel_leaf[sel0 + i] = s_leaf[i];
  }
  for (int i = n_keep + tid; i < g; i += kTreeThreads) {
    a.sel_cand[sel0 + i] = -1;
    a.sel_tok[sel0 + i] = -1;
    a.sel_parent[sel0 + i] = -1;
    a.sel_depth[sel0 + i] = 0;
    a.sel_pslot[sel0 + i] = 0;
    a.sel_slot[sel0 + i] = -1;
    a.sel_score[sel0 + i] = 0.f;
    a.sel_leaf[sel0 + i] = 0;
  }
  for (int i = tid; i < a.d * a.k; i += kTreeThreads) a.slot_need[(int64_t)r * a.d * a.k + i] = s_need[i];
  if (tid == 0) a.n_sel[r] = n_keep;
}

void launch_select(const SelectArgs &a, hipStream_t st) {
  int n_pad = 2;
  while (n_pad < a.C) n_pad <<= 1;
  const int n_keep = (a.g < a.C) ? a.g : a.C;
  const size_t lds = (size_t)n_pad * 8 + (size_t)a.C * 4 + (size_t)n_keep + (size_t)a.d * a.k;
  hipLaunchKernelGGL(k_select, dim3(a.R), dim3(kTreeThreads), lds, st, a);
}

// ------------------------------------------------------------------------------ reward
constexpr int kRewardThreads = 128;
constexpr int kMaxDepth = 32;

__device__ __forceinline__ double block_reduce(double v, double *scratch, bool is_max) {
  const int tid = threadIdx.x;
  scratch[tid] = v;
  __syncthreads();
  for (int off = kRewardThreads / 2; off >= 1; off >>= 1) {
    if (tid < off) {
      const double o = scratch[tid + off];
      scratch[tid] = is_max ? fmax(scratch[tid], o) : scratch[tid] + o;
    }
    __syncthreads();
  }
  const double out = scratch[0];
  __syncthreads();
  return out;
}

// most nodes a root can keep: min(g, C)
__host__ __device__ inline int reward_nodes(const RewardArgs &a) {
  const int C = a.k + (a.d - 1) * a.k * a.k;
  return a.g < C ? a.g : C;
}

template <typename T>
__global__ __launch_bounds__(kRewardThreads) void k_reward(RewardArgs a) {
  const int r = blockIdx.x, tid = threadIdx.x;
  const int d = a.d, k = a.k, g = a.g;
  const int n = a.n_sel[r];
  const int64_t sel0 = (int64_t)r * g;
  extern __shared__ __align__(16) unsigned char s_dyn[];     // min(g, C) doubles, then as many ints
  double *s_logt = reinterpret_cast<double *>(s_dyn);
  int *s_parent = reinterpret_cast<int *>(s_logt + reward_nodes(a));
  __shared__ double s_red[kRewardThreads];
  __shared__ int s_found;
  const T *logits = static_cast<const T *>(a.target_logits);

  // target log-probability of every kept token (one gather each)
  for (int i = tid; i < n; i += kRewardThreads) {
    const int lvl = a.sel_depth[sel0 + i] - 1;
    const int js = a.sel_pslot[sel0 + i];
    const int tok = min(max(a.sel_tok[sel0 + i], 0), a.V - 1);     // ids come from the row kernels: always in range
    const int64_t si = stat_index(r, lvl, js, d, k);
    const float x = a.node_logit ? a.node_logit[sel0 + i] : Elem<T>::load1(logits + si * a.row_stride + tok);
    s_logt[i] = (double)x - (double)a.t_lse[si];
    s_parent[i] = a.sel_parent[sel0 + i];
  }
  __syncthreads();

  // prefix products along each node's own ancestor chain (root first), Eq. 3-4
  double v_max = -1.0, v_sumL = 0.0, v_cnt = 0.0, v_q = 0.0;
  double myL[ (kMaxPool + kRewardThreads - 1) / kRewardThreads ];
  int nmine = 0;
  for (int i = tid; i < n; i += kRewardThreads) {
    int chain[kMaxDepth];
    int len = 0;
    for (int p = i; p >= 0 && len < kMaxDepth; p = s_parent[p]) chain[len++] = p;
    double lq = 0.0, cum = 0.0, q = 0.0;
    for (int s = len - 1; s >= 0; --s) {
      lq += s_logt[chain[s]];
      q = exp(lq);
      cum += q;
    }
    a.node_q[sel0 + i] = (float)q;
    a.node_cum[sel0 + i] = (float)cum;
    v_q += q;
    const bool leaf = a.sel_leaf[sel0 + i] != 0;
    if (leaf) {
      v_max = fmax(v_max, cum);
      v_sumL += cum;
      v_cnt += 1.0;
    }
    myL[nmine++] = leaf ? cum : -1.0;
  }
  for (int i = n + tid; i < g; i += kRewardThreads) {
    a.node_q[sel0 + i] = 0.f;
    a.node_cum[sel0 + i] = 0.f;
  }
  const double Lmax = block_reduce(v_max, s_red, true);
  double v_exp = 0.0;
  for (int q = 0; q < nmine; ++q)
    if (myL[q] >= 0.0) v_exp += exp((double)a.eta * (myL[q] - Lmax));
  const double sum_exp = block_reduce(v_exp, s_red, false);
  const double sumL = block_reduce(v_sumL, s_red, false);
  const double cnt = block_reduce(v_cnt, s_red, false);
  const double nodesum = block_reduce(v_q, s_red, false);
  if (tid == 0) {
    const double lse = (cnt > 0.0) ? Lmax + log(sum_exp) / (double)a.eta : 0.0;
    const double mx = (cnt > 0.0) ? Lmax : 0.0;
    const double mean = (cnt > 0.0) ? sumL / cnt : 0.0;
    float *aux = a.reward_aux + (int64_t)r * 4;
    aux[0] = (float)lse;
    aux[1] = (float)mx;
    aux[2] = (float)mean;
    aux[3] = (float)nodesum;
    const double pick = (a.reward_mode == 0) ? lse : (a.reward_mode == 1) ? mx : (a.reward_mode == 2) ? mean : nodesum;
    a.reward[r] = (float)pick;
    a.n_leaves[r] = (int)cnt;
  }

  if (a.path_mode == 1) {
    // alternative reading of "longest accepted sequence": the root-to-leaf sequence with the largest
    // expected acceptance length L_i (first one in kept order among equals)
    __syncthreads();
    for (int q = 0, i = tid; i < n; i += kRewardThreads, ++q) s_logt[i] = myL[q];   // -1 for non-leaves
    __syncthreads();
    if (tid == 0) {
      int best = -1;
      double bl = -1.0;
      for (int i = 0; i < n; ++i)
        if (s_logt[i] > bl) { bl = s_logt[i]; best = i; }
      int chain[kMaxDepth];
      int len = 0;
      for (int p = best; p >= 0 && len < kMaxDepth; p = s_parent[p]) chain[len++] = p;
      for (int t = 0; t < d; ++t) {
        const bool on = t < len;
        const int node = on ? chain[len - 1 - t] : -1;
        a.path_node[(int64_t)r * d + t] = node;
        a.path_slot[(int64_t)r * d + t] = on ? a.sel_pslot[sel0 + node] : -1;
      }
      a.path_len[r] = len;
    }
    return;
  }
  if (a.path_mode == 2) {
    // verification at temperature 1: the kept children of the current node are tried in kept order,
    // child x accepted with probability p_T(x) / (target mass not yet rejected at this node), decided
    // by the caller's uniform numbers; s_logt still holds log p_T of every kept token
    __syncthreads();
    if (tid == 0) {
      int cur = -1, slot = 0, len = 0;
      for (int t = 0; t < d; ++t) {
        double rest = 1.0;
        int j = 0, nxt = -1;
        for (int i = 0; i < n; ++i) {
          if (s_parent[i] != cur || a.sel_depth[sel0 + i] != t + 1) continue;
          const double p_tok = exp(s_logt[i]);
          const double acc = (rest > 0.0) ? p_tok / rest : 1.0;
          const double u = (double)a.accept_u[((int64_t)r * d + t) * k + j];
          if (u < acc) { nxt = i; break; }
          rest -= p_tok;
          ++j;
        }
        if (nxt < 0) break;
        a.path_node[(int64_t)r * d + t] = nxt;
        a.path_slot[(int64_t)r * d + t] = slot;
        len = t + 1;
        const int own = a.sel_slot[sel0 + nxt];
        if (own < 0) break;
        cur = nxt;
        slot = own;
      }
      for (int t = len; t < d; ++t) {
        a.path_node[(int64_t)r * d + t] = -1;
        a.path_slot[(int64_t)r * d + t] = -1;
      }
      a.path_len[r] = len;
    }
    return;
  }
  // greedy verification walk (T = 0): follow the kept child that equals the target argmax
  int cur = -1, slot = 0, len = 0;
  bool alive = true;
  for (int t = 0; t < d; ++t) {
    if (tid == 0) s_found = -1;
    __syncthreads();
    if (alive) {
      const int want = a.t_argmax[stat_index(r, t, slot, d, k)];
      for (int i = tid; i < n; i += kRewardThreads)
        if (s_parent[i] == cur && a.sel_depth[sel0 + i] == t + 1 && a.sel_tok[sel0 + i] == want) s_found = i;
    }
    __syncthreads();
    const int nxt = alive ? s_found : -1;
    __syncthreads();
    if (nxt >= 0) {
      if (tid == 0) {
        a.path_node[(int64_t)r * d + t] = nxt;
        a.path_slot[(int64_t)r * d + t] = slot;
      }
      len = t + 1;
      const int own = a.sel_slot[sel0 + nxt];
      if (own < 0) alive = false;
      cur = nxt;
      slot = own;
    } else {
      alive = false;
      if (tid == 0) {
        a.path_node[(int64_t)r * d + t] = -1;
        a.path_slot[(int64_t)r * d + t] = -1;
      }
    }
  }
  if (tid == 0) a.path_len[r] = len;
}

void launch_reward(const RewardArgs &a, hipStream_t st) {
  const size_t lds = (size_t)reward_nodes(a) * 12;
  if (a.dtype == 0) hipLaunchKernelGGL(k_reward<uint16_t>, dim3(a.R), dim3(kRewardThreads), lds, st, a);
  else hipLaunchKernelGGL(k_reward<float>, dim3(a.R), dim3(kRewardThreads), lds, st, a);
}

// ------------------------------------------------------------------------------ advantage
// One wave per group: lane-strided fp64 sums and a fixed-shape wave reduction (deterministic for any m).
__global__ __launch_bounds__(64) void k_advantage(AdvArgs a) {
  const int grp = blockIdx.x, lane = threadIdx.x;
  const int i0 = grp * a.m;
  double sum = 0.0;
  for (int i = lane; i < a.m; i += 64)
    sum += (double)a.r_cur[i0 + i] - (a.r_ref ? (double)a.r_ref[i0 + i] : 0.0);
  const double mean = wave_sum(sum) / a.m;
  double var = 0.0;
  for (int i = lane; i < a.m; i += 64) {
    const double dv = ((double)a.r_cur[i0 + i] - (a.r_ref ? (double)a.r_ref[i0 + i] : 0.0)) - mean;
    var += dv * dv;
  }
  const double sd = sqrt(wave_sum(var) / a.m);
  for (int i = lane; i < a.m; i += 64) {
    const double dv = ((double)a.r_cur[i0 + i] - (a.r_ref ? (double)a.r_ref[i0 + i] : 0.0)) - mean;
    a.adv[i0 + i] = (float)(dv / (sd + (double)a.delta));
  }
}

void launch_advantage(const AdvArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(k_advantage, dim3(a.R / a.m), dim3(64), 0, st, a);
}

// ------------------------------------------------------------------------------ surrogate fwd
template <typename T>
__global__ void k_ppo_root(PpoFwdArgs a) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= a.R) return;
  const int d = a.d, k = a.k;
  const int l = a.path_len[r];
  const T *dl = static_cast<const T *>(a.draft_logits);
  const T *rl = static_cast<const T *>(a.ref_logits);
  double lm = 0.0, lm0 = 0.0;
  for (int t = 0; t < l; ++t) {
    const int64_t rt = (int64_t)r * d + t;
    const int j = a.path_slot[rt];
    const int tok = min(max(a.sel_tok[(int64_t)r * a.g + a.path_node[rt]], 0), a.V - 1);
    const int64_t si = stat_index(r, t, j, d, k);
    const float xc = a.path_logit_cur ? a.path_logit_cur[rt] : Elem<T>::load1(dl + si * a.row_stride + tok);
    lm += (double)xc - (double)a.draft_lse[si];
    const double rlse = a.ref_lse_by_step ? (double)a.ref_lse[rt] : (double)a.ref_lse[si];
    const float xr = a.path_logit_ref ? a.path_logit_ref[rt] : Elem<T>::load1(rl + si * a.row_stride + tok);
    lm0 += (double)xr - rlse;
  }
  const int lden = (l > 1) ? l : 1;
  const double s = exp((lm - lm0) / lden);
  const double A = (double)a.adv[r];
  const double lo = 1.0 - (double)a.eps, hi = 1.0 + (double)a.eps;
  const double clipped = fmax(lo, fmin(s, hi));
  const double term = fmin(s * A, clipped * A);
  const bool passes = (A >= 0.0) ? (s <= hi) : (s >= lo);
  const int active = (l > 0 && passes) ? 1 : 0;
  const int K = a.R / a.m;
  a.logM[r] = (float)lm;
  a.logM0[r] = (float)lm0;
  a.ratio[r] = (float)s;
  a.term[r] = (float)term;
  a.active[r] = active;
  a.coef[r] = (float)((double)a.grad_scale * (-A / ((double)a.m * K)) * active * s / lden);
}

__global__ __launch_bounds__(256) void k_ppo_loss(PpoFwdArgs a) {
  // single block: group losses (Eq. 12), then their mean; every sum has a fixed shape
  const int K = a.R / a.m;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __shared__ double s_red[256];
  double part = 0.0;
  if (a.m <= 16) {
    // small groups: one thread per group
    for (int grp = threadIdx.x; grp < K; grp += 256) {
      double sum = 0.0;
      for (int i = 0; i < a.m; ++i) sum += (double)a.term[grp * a.m + i];
      const double lg = -sum / a.m;
      a.loss_group[grp] = (float)lg;
      part += lg;
    }
  } else {
    // large groups: one wave per group, lane-strided sum and wave reduction
    for (int grp = wave; grp < K; grp += 4) {
      double sum = 0.0;
      for (int i = lane; i < a.m; i += 64) sum += (double)a.term[grp * a.m + i];
      const double lg = -wave_sum(sum) / a.m;
      if (lane == 0) {
        a.loss_group[grp] = (float)lg;
        part += lg;
      }
    }
  }
  s_red[threadIdx.x] = part;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {
    if ((int)threadIdx.x < off) s_red[threadIdx.x] += s_red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) a.loss[0] = (float)(s_red[0] / K);
}

// (slot, token) pairs whose single logits the fused variant computes as dot products
__global__ void k_pairs(PairArgs a, int mode) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int per = (mode == 0) ? a.g : a.d;
  if (p >= (int64_t)a.R * per) return;
  const int r = (int)(p / per), i = (int)(p - (int64_t)r * per);
  int64_t slot = -1;
  int tok = -1;
  if (mode == 0) {
    if (i < a.n_sel[r]) {
      slot = stat_index(r, a.sel_depth[p] - 1, a.sel_pslot[p], a.d, a.k);
      tok = a.sel_tok[p];
    }
  } else {
    const int j = a.path_slot[p];
    if (j >= 0) {
      slot = stat_index(r, i, j, a.d, a.k);
      tok = a.sel_tok[(int64_t)r * a.g + a.path_node[p]];
    }
  }
  a.slot[p] = slot;
  a.tok[p] = tok;
}

void launch_pairs(const PairArgs &a, int mode, hipStream_t st) {
  const int64_t n = (int64_t)a.R * ((mode == 0) ? a.g : a.d);
  hipLaunchKernelGGL(k_pairs, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a, mode);
}

void launch_ppo_fwd(const PpoFwdArgs &a, hipStream_t st) {
  const int blocks = (a.R + 63) / 64;
  if (a.dtype == 0) hipLaunchKernelGGL(k_ppo_root<uint16_t>, dim3(blocks), dim3(64), 0, st, a);
  else hipLaunchKernelGGL(k_ppo_root<float>, dim3(blocks), dim3(64), 0, st, a);
  hipLaunchKernelGGL(k_ppo_loss, dim3(1), dim3(256), 0, st, a);
}

}  // namespace gto
