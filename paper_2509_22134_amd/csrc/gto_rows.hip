// Row-streaming kernels of the GTO hot path (gfx950, wave64).
//
//  k_row_stats : one workgroup per logits row.  Streams the row once with 16-byte loads and
//                produces max, log-sum-exp and the exact top-k (value descending, token id
//                ascending).  Used for draft rows (k = branching), target rows (k = 1 gives
//                the argmax) and for the reference rows on an accepted path.
//  k_ppo_bwd   : one workgroup per (root, path step).  Re-streams one draft row and writes
//                one fp32 gradient row  coef * (onehot - softmax).
//
// Both are HBM-bandwidth bound by design: per element they spend one conversion, one fused
// multiply-add, one exp2 and one add; the top-k costs one max per element plus a rarely
// taken insertion path.
#include "gto_device.h"
#include "gto_kernels.h"

namespace gto {

constexpr int kRowLoads = 4;   // 16-byte loads in flight per lane and tile (2 and 8 measured about 1 % slower)

// ----------------------------------------------------------------------------- top-k list
// A wave keeps the 64 best (value, id) pairs it has seen, sorted, one per lane (lane 0 = best).
// Inserting shifts the tail down by one lane with a single DPP move per register.
struct TopList {
  float v;
  int id;
  __device__ __forceinline__ void init() { v = neg_inf(); id = kNoId; }
  __device__ __forceinline__ void insert(float cv, int ci) {
    const bool b = better(cv, ci, v, id);
    const float uv = wave_shr1(v, __builtin_inff());
    const int ui = wave_shr1(id, -1);
    const bool bu = better(cv, ci, uv, ui);
    v = b ? (bu ? uv : cv) : v;
    id = b ? (bu ? ui : ci) : id;
  }
};

// k-th largest of the 64 per-lane values (k <= 64), the same in every lane.
__device__ __forceinline__ float kth_largest_of_lanes(float x, int k) {
  int cnt = 0;
#pragma unroll
  for (int i = 0; i < kWave; ++i) cnt += (readlane(x, i) > x) ? 1 : 0;
  float cand = (cnt < k) ? x : __builtin_inff();
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) cand = fminf(cand, __shfl_xor(cand, off, kWave));
  return cand;
}

// Per-lane streaming state: running max m, log2-domain offset c = m*log2(e) and
// s = sum 2^(x*log2(e) - c) over the elements this lane has seen.  Each 16-byte vector is summed
// in fp32 and then added to s in fp64 (a full-rate add on this chip): an fp32 running sum that
// already holds a dominant term would silently drop the many tiny ones added after it.
struct LaneAcc {
  float m, c;
  double s;
  __device__ __forceinline__ void init() { m = neg_inf(); c = 0.f; s = 0.0; }
};

enum RowMode { kDraftTopK = 0, kTargetArgmax = 1, kLseOnly = 2 };

// Issues the LOADS 16-byte loads of one tile (lane l, load u: elements (u*64 + l)*EPV ...).
template <typename T, int LOADS, bool GUARD>
__device__ __forceinline__ void load_tile(const T *__restrict__ row, int tile_base, int V, int lane, u32x4 *q) {
  constexpr int EPV = Elem<T>::kPerVec;
#pragma unroll
  for (int u = 0; u < LOADS; ++u) {
    const int e0 = tile_base + (u * kWave + lane) * EPV;
    if (!GUARD || e0 < V) {
      q[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row + e0));
    } else {
      q[u] = u32x4{0u, 0u, 0u, 0u};
    }
  }
}

template <typename T, int LOADS, bool GUARD, int MODE>
__device__ __forceinline__ void scan_tile(const u32x4 *q, int tile_base, int V, int lane,
                                          int ktop_rt, bool &first, LaneAcc &acc, TopList &top,
                                          float &thr_v, int &thr_i) {
  const int ktop = (MODE == kTargetArgmax) ? 1 : ktop_rt;
  constexpr int EPV = Elem<T>::kPerVec;
  float x[LOADS][EPV];
#pragma unroll
  for (int u = 0; u < LOADS; ++u) {
    Elem<T>::unpack(q[u], x[u]);
    if (GUARD) {
      const int e0 = tile_base + (u * kWave + lane) * EPV;
#pragma unroll
      for (int e = 0; e < EPV; ++e)
        if (e0 + e >= V) x[u][e] = neg_inf();
    }
  }
  float mu[LOADS];
#pragma unroll
  for (int u = 0; u < LOADS; ++u) {
    mu[u] = x[u][0];
#pragma unroll
    for (int e = 1; e < EPV; ++e) mu[u] = fmaxf(mu[u], x[u][e]);
  }
  float cm = mu[0];
#pragma unroll
  for (int u = 1; u < LOADS; ++u) cm = fmaxf(cm, mu[u]);

  // online log-sum-exp in the log2 domain
  const float m_new = fmaxf(acc.m, cm);
  const float c_new = (m_new == neg_inf()) ? 0.f : m_new * kLog2e;
  const float scale = __builtin_amdgcn_exp2f(acc.c - c_new);
  double s = (acc.m == neg_inf()) ? 0.0 : acc.s * (double)scale;
#pragma unroll
  for (int u = 0; u < LOADS; ++u) {
    float p = 0.f;
#pragma unroll
    for (int e = 0; e < EPV; ++e) p += __builtin_amdgcn_exp2f(__builtin_fmaf(x[u][e], kLog2e, -c_new));
    s += (double)p;
  }
  acc.m = m_new;
  acc.c = c_new;
  acc.s = s;

  if (MODE == kLseOnly) return;
  // top-k: first tile of a wave seeds the threshold with the k-th largest lane maximum, a
  // value that at least k elements of this tile reach.
  if (first) {
    first = false;
    thr_v = kth_largest_of_lanes(cm, ktop);
    thr_i = kNoId;
  }
  const int lane_first = tile_base + lane * EPV;
  const bool hit = better(cm, lane_first, thr_v, thr_i);
  if (__builtin_amdgcn_ballot_w64(hit) == 0) return;

#pragma unroll
  for (int u = 0; u < LOADS; ++u) {
    // skip a whole vector position when no lane's vector maximum can enter the list
    if (__builtin_amdgcn_ballot_w64(better(mu[u], tile_base + (u * kWave + lane) * EPV, thr_v, thr_i)) == 0)
      continue;
#pragma unroll
    for (int e = 0; e < EPV; ++e) {
      const int my_id = tile_base + (u * kWave + lane) * EPV + e;
      bool p = better(x[u][e], my_id, thr_v, thr_i);
      if (GUARD) p = p && (my_id < V);
      uint64_t mask = __builtin_amdgcn_ballot_w64(p);
      while (mask) {
        const int src = __builtin_ctzll(mask);
        mask &= mask - 1;
        const float cv = readlane(x[u][e], src);
        const int ci = tile_base + (u * kWave + src) * EPV + e;
        if (better(cv, ci, thr_v, thr_i)) {
          top.insert(cv, ci);
          const float nv = readlane(top.v, ktop - 1);
          const int ni = readlane(top.id, ktop - 1);
          if (better(nv, ni, thr_v, thr_i)) {
            thr_v = nv;
            thr_i = ni;
          }
        }
      }
    }
  }
}

template <typename T, int WAVES, int LOADS, int MODE>
__global__ __launch_bounds__(WAVES *kWave) void k_row_stats(RowStatsArgs a) {
  constexpr int EPV = Elem<T>::kPerVec;
  constexpr int TILE = kWave * LOADS * EPV;
  const int lane = lane_id();
  const int wave = threadIdx.x / kWave;

  // which row
  int r, l, j;
  int64_t oi;
  if (a.path_slot == nullptr) {
    r = blockIdx.x / a.rho;
    const int qq = blockIdx.x - r * a.rho;
    l = (qq == 0) ? 0 : 1 + (qq - 1) / a.kslots;
    j = (qq == 0) ? 0 : (qq - 1) % a.kslots;
    oi = stat_index(r, l, j, a.d, a.kslots);
    if (a.row_need != nullptr && a.row_need[oi] == 0) return;
  } else {  // rows on an accepted path: block = (root, step)
    r = blockIdx.x / a.d;
    l = blockIdx.x - r * a.d;
    j = a.path_slot[(int64_t)r * a.d + l];
    if (j < 0) return;
    oi = (int64_t)r * a.d + l;
  }
  const T *row = static_cast<const T *>(a.logits) + stat_index(r, l, j, a.d, a.kslots) * a.row_stride;
  const int V = a.V;

  LaneAcc acc;
  acc.init();
  TopList top;
  top.init();
  float thr_v = neg_inf();
  int thr_i = kNoId;
  bool first = true;

  const int n_full = V / TILE;
  for (int t = wave; t < n_full; t += WAVES) {
    u32x4 q[LOADS];
    load_tile<T, LOADS, false>(row, t * TILE, V, lane, q);
    scan_tile<T, LOADS, false, MODE>(q, t * TILE, V, lane, a.ktop, first, acc, top, thr_v, thr_i);
  }
  if (n_full * TILE < V && (n_full % WAVES) == wave) {
    u32x4 q[LOADS];
    load_tile<T, LOADS, true>(row, n_full * TILE, V, lane, q);
    scan_tile<T, LOADS, true, MODE>(q, n_full * TILE, V, lane, a.ktop, first, acc, top, thr_v, thr_i);
  }

  // wave-level reduction of (max, offset, sum)
  const float Mw = wave_max(acc.m);
  const float Cw = wave_max(acc.m == neg_inf() ? neg_inf() : acc.c);
  const double contrib =
      (acc.m == neg_inf()) ? 0.0 : acc.s * (double)__builtin_amdgcn_exp2f(acc.c - Cw);
  const double Sw = wave_sum(contrib);

  __shared__ float sh_v[WAVES * kWave];
  __shared__ int sh_i[WAVES * kWave];
  __shared__ float sh_M[WAVES], sh_C[WAVES];
  __shared__ double sh_S[WAVES];
  __shared__ double sh_lse;
  sh_v[threadIdx.x] = top.v;
  sh_i[threadIdx.x] = top.id;
  if (lane == 0) {
    sh_M[wave] = Mw;
    sh_C[wave] = Cw;
    sh_S[wave] = Sw;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float M = sh_M[0], C = sh_C[0];
    bool any = (sh_M[0] != neg_inf());
#pragma unroll
    for (int w = 1; w < WAVES; ++w) {
      M = fmaxf(M, sh_M[w]);
      if (sh_M[w] != neg_inf()) {
        C = any ? fmaxf(C, sh_C[w]) : sh_C[w];
        any = true;
      }
    }
    double S = 0.0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w)
      if (sh_M[w] != neg_inf()) S += sh_S[w] * (double)__builtin_amdgcn_exp2f(sh_C[w] - C);
    // log2-domain total is C + log2(S); the row maximum contributes exactly M*log2e of it.
    const double lse = (double)M + kLn2 * (((double)C - (double)M * (double)kLog2e) + log2(S));
    sh_lse = lse;
    if (a.row_max) a.row_max[oi] = M;
    a.row_lse[oi] = (float)lse;
  }
  if (MODE == kLseOnly || a.top_tok == nullptr) return;
  __shared__ int sh_claimed[kWave];
  if (threadIdx.x < kWave) sh_claimed[threadIdx.x] = 0;
  __syncthreads();
  // merge the WAVES sorted lists: rank each of the first ktop entries of every wave
  if (lane < a.ktop) {
    const float v = top.v;
    const int id = top.id;
    int rank = 0;
    for (int w = 0; w < WAVES; ++w)
      for (int i = 0; i < a.ktop; ++i) rank += better(sh_v[w * kWave + i], sh_i[w * kWave + i], v, id) ? 1 : 0;
    if (rank < a.ktop && id != kNoId) {
      sh_claimed[rank] = 1;
      a.top_tok[oi * a.ktop + rank] = id;
      // clamped: rounding must never make a log-probability positive (a child may not outrank its parent)
      if (a.top_logp) a.top_logp[oi * a.ktop + rank] = fminf((float)((double)v - sh_lse), 0.f);
    }
  }
  __syncthreads();
  // A row that holds NaNs can leave ranks unclaimed (a NaN wins no comparison).  Such a row's values are
  // unspecified, but every id written must be a token of the vocabulary: unclaimed ranks get token `rank`
  // (V >= ktop) with probability zero.
  if (threadIdx.x < a.ktop && sh_claimed[threadIdx.x] == 0) {
    a.top_tok[oi * a.ktop + threadIdx.x] = threadIdx.x;
    if (a.top_logp) a.top_logp[oi * a.ktop + threadIdx.x] = neg_inf();
  }
}

// Four consecutive elements of a row, at element index 4 * q4, as fp32: one 8-byte (bf16) or 16-byte (fp32)
// nontemporal load.  A wave's 64 such loads are contiguous, and so are the 64 16-byte stores of the four
// fp32 results: every store instruction fills whole cache lines (two 16-byte stores per lane, 32 bytes
// apart between lanes, leave every line half written and cost ~1.7x the write traffic, measured).
template <typename T>
__device__ __forceinline__ void load4(const T *row, int q4, float *x);
template <>
__device__ __forceinline__ void load4<uint16_t>(const uint16_t *row, int q4, float *x) {
  const u32x2 q = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(row) + q4);
  x[0] = __uint_as_float(q.x << 16); x[1] = __uint_as_float(q.x & 0xffff0000u);
  x[2] = __uint_as_float(q.y << 16); x[3] = __uint_as_float(q.y & 0xffff0000u);
}
template <>
__device__ __forceinline__ void load4<float>(const float *row, int q4, float *x) {
  const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row) + q4);
  x[0] = __uint_as_float(q.x); x[1] = __uint_as_float(q.y); x[2] = __uint_as_float(q.z); x[3] = __uint_as_float(q.w);
}
// The same four elements as they come from memory (to be carried across loop trips without the unpacking
// being scheduled right behind the load), and their conversion.
template <typename T> struct Raw4;
template <> struct Raw4<uint16_t> {
  typedef u32x2 type;
  __device__ static __forceinline__ type load(const uint16_t *row, int q4) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(row) + q4);
  }
  __device__ static __forceinline__ void unpack(const type &q, float *x) {
    x[0] = __uint_as_float(q.x << 16); x[1] = __uint_as_float(q.x & 0xffff0000u);
    x[2] = __uint_as_float(q.y << 16); x[3] = __uint_as_float(q.y & 0xffff0000u);
  }
};
template <> struct Raw4<float> {
  typedef u32x4 type;
  __device__ static __forceinline__ type load(const float *row, int q4) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row) + q4);
  }
  __device__ static __forceinline__ void unpack(const type &q, float *x) {
    x[0] = __uint_as_float(q.x); x[1] = __uint_as_float(q.y); x[2] = __uint_as_float(q.z); x[3] = __uint_as_float(q.w);
  }
};

// N consecutive elements at element index N * idx: N == 4 as above; N == the elements of a 16-byte
// vector for kernels that only read (16-byte loads stream ~20 % faster than 8-byte ones, measured).
template <typename T, int N>
__device__ __forceinline__ void load_group(const T *row, int idx, float *x) {
  if constexpr (N == 4) {
    load4<T>(row, idx, x);
  } else {
    static_assert(N == Elem<T>::kPerVec, "group is four elements or one 16-byte vector");
    Elem<T>::unpack(__builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row) + idx), x);
  }
}

// ------------------------------------------------------------------------------- backward
// One workgroup of 16 waves per (root, step): only the few hundred rows on accepted paths do any work,
// so the parallelism has to come from inside the row.
constexpr int kBwdThreads = 1024;
template <typename T, bool VEC>
__global__ __launch_bounds__(kBwdThreads) void k_ppo_bwd(PpoBwdArgs a) {
  // step-major order: the rows that carry a gradient (short paths: mostly the first steps) then sit densely at
  // the front of the grid and spread over the compute units (root-major order: 106 us instead of 80)
  const int n_roots = gridDim.x / a.d;
  const int t = blockIdx.x / n_roots;
  const int r = blockIdx.x - t * n_roots;
  const int64_t rt = (int64_t)r * a.d + t;
  const int j = a.path_slot[rt];
  const float coef = a.coef[r];
  const bool valid = (j >= 0) && (coef != 0.f);
  if (threadIdx.x == 0) a.grad_slot[rt] = valid ? j : -1;
  float *__restrict__ out = a.grad_rows + rt * (int64_t)a.V;
  const int V = a.V;
  if (!valid) {
    if (a.zero_fill) {
      if (VEC) {
        f32x4 *o4 = reinterpret_cast<f32x4 *>(out);
        for (int i = threadIdx.x; i < V / 4; i += blockDim.x) o4[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      } else {
        for (int i = threadIdx.x; i < V; i += blockDim.x) out[i] = 0.f;
      }
    }
    return;
  }
  const int tok = a.sel_tok[(int64_t)r * a.g + a.path_node[rt]];
  const float lse = a.row_lse[stat_index(r, t, j, a.d, a.k)];
  const T *__restrict__ row = static_cast<const T *>(a.logits) + stat_index(r, t, j, a.d, a.k) * a.row_stride;
  // Every entry but the token's is -coef * p_v.  The token's entry coef * (1 - p_tok) is formed as
  // coef * (sum of the other probabilities): when p_tok is close to 1 the subtraction would cancel.
  float others = 0.f;
  bool own_tok = false;
  if (VEC) {
    // Groups of four elements, kBwdUnroll groups per step and lane.  The loads of the next step are issued
    // before the stores of this one: loads and stores share one in-order counter, so a wait for loads that
    // were issued after a batch of stores would also wait for those stores to be acknowledged by memory.
    constexpr int kBwdUnroll = 8;
    const int n4 = V / 4;
    typedef typename Raw4<T>::type raw_t;
    raw_t x[kBwdUnroll], xn[kBwdUnroll];
    // (past the end of the row the last group is fetched again: a branch around a load would end in a wait
    // for everything outstanding)
    auto fetch = [&](raw_t (&dst)[kBwdUnroll], int i0) {
#pragma unroll
      for (int u = 0; u < kBwdUnroll; ++u) dst[u] = Raw4<T>::load(row, min(i0 + u * kBwdThreads, n4 - 1));
    };
    auto emit = [&](const raw_t (&src)[kBwdUnroll], int i0) {
#pragma unroll
      for (int u = 0; u < kBwdUnroll; ++u) {
        const int i = i0 + u * kBwdThreads;
        if (i >= n4) continue;
        float xv[4];
        Raw4<T>::unpack(src[u], xv);
        float gq[4];
        float part = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p = __builtin_amdgcn_exp2f((xv[e] - lse) * kLog2e);
          gq[e] = -coef * p;
          const bool is_tok = (i * 4 + e == tok);
          own_tok = own_tok || is_tok;
          part += is_tok ? 0.f : p;
        }
        others += part;
        const f32x4 o = {gq[0], gq[1], gq[2], gq[3]};
        __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(out) + i);
      }
    };
    // two steps per trip, the two register sets swapping roles (no copies between them)
    constexpr int kStep = kBwdUnroll * kBwdThreads;
    fetch(x, threadIdx.x);
    for (int i0 = threadIdx.x; i0 < n4; i0 += 2 * kStep) {
      fetch(xn, i0 + kStep);
      emit(x, i0);
      fetch(x, i0 + 2 * kStep);
      emit(xn, i0 + kStep);
    }
  } else {
    for (int i = threadIdx.x; i < V; i += blockDim.x) {
      const float xv = Elem<T>::load1(row + i);
      const float p = __builtin_amdgcn_exp2f((xv - lse) * kLog2e);
      const bool is_tok = (i == tok);
      own_tok = own_tok || is_tok;
      others += is_tok ? 0.f : p;
      out[i] = -coef * p;
    }
  }
  __shared__ double s_part[kBwdThreads];
  s_part[threadIdx.x] = (double)others;
  __syncthreads();
  for (int off = kBwdThreads / 2; off >= 1; off >>= 1) {
    if ((int)threadIdx.x < off) s_part[threadIdx.x] += s_part[threadIdx.x + off];
    __syncthreads();
  }
  // the thread that stored the token's entry overwrites it (same thread, program order)
  if (own_tok) out[tok] = (float)((double)coef * s_part[0]);
}

// ------------------------------------------------------------------------------- token-level loss
// One workgroup per root: streams the root rows (slot (0,0)) of the draft and the target logits
// together.  Forward: H = lse_M - sum_v p_T(v) d_v.  Backward: scale * (p_M - p_T) as an fp32 row.
constexpr int kTokThreads = 256;
template <typename T, bool BWD, bool VEC>
__global__ __launch_bounds__(kTokThreads) void k_token_loss(TokenLossArgs a) {
  const int r = blockIdx.x;
  const float w = a.weight ? a.weight[r] : 1.f;
  const int64_t si = stat_index(r, 0, 0, a.d, a.k);
  const int64_t lo = a.root_stride ? (int64_t)r * a.root_stride : si * a.row_stride;
  const T *__restrict__ drow = static_cast<const T *>(a.draft_logits) + lo;
  const T *__restrict__ trow = static_cast<const T *>(a.target_logits) + lo;
  const float d_lse = a.d_lse[si], t_lse = a.t_lse[si];
  const int V = a.V;
  float *__restrict__ out = BWD ? a.grad + (int64_t)r * V : nullptr;
  const float scale = BWD ? a.grad_scale * w * a.inv_count[0] : 0.f;
  double acc = 0.0;
  // Groups of kGroup elements, kUnroll groups of each row in flight per lane.  The backward takes
  // groups of four so that its stores fill whole lines (see load4); the forward, which stores nothing,
  // takes whole 16-byte vectors.  VEC: V % kGroup == 0 and, for the backward, 16-byte aligned output
  // rows; otherwise one element at a time.
  constexpr int kGroup = BWD ? 4 : Elem<T>::kPerVec;
  constexpr int kUnroll = BWD ? 4 : 2;
  const int n4 = VEC ? V / kGroup : 0;
  for (int i0 = threadIdx.x; i0 < n4; i0 += kUnroll * kTokThreads) {
    float xd[kUnroll][kGroup], xt[kUnroll][kGroup];
    // past the end of the rows the last group is fetched again (a branch around a load would end in a wait
    // for everything outstanding)
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int i = min(i0 + u * kTokThreads, n4 - 1);
      load_group<T, kGroup>(drow, i, xd[u]);
      load_group<T, kGroup>(trow, i, xt[u]);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int i = i0 + u * kTokThreads;
      if (i >= n4) continue;
      if constexpr (BWD) {
        float gq[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float pm = __builtin_amdgcn_exp2f((xd[u][e] - d_lse) * kLog2e);
          const float pt = __builtin_amdgcn_exp2f((xt[u][e] - t_lse) * kLog2e);
          gq[e] = scale * (pm - pt);
        }
        const f32x4 o = {gq[0], gq[1], gq[2], gq[3]};
        __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(out) + i);
      } else {
        float part = 0.f;
#pragma unroll
        for (int e = 0; e < kGroup; ++e) {
          const float pt = __builtin_amdgcn_exp2f((xt[u][e] - t_lse) * kLog2e);
          part += (pt > 0.f) ? pt * (xd[u][e] - d_lse) : 0.f;      // 0 * log 0 := 0
        }
        acc += (double)part;
      }
    }
  }
  if (!VEC) {
    for (int i = threadIdx.x; i < V; i += kTokThreads) {
      const float dv = Elem<T>::load1(drow + i), tv = Elem<T>::load1(trow + i);
      const float pt = __builtin_amdgcn_exp2f((tv - t_lse) * kLog2e);
      if (BWD) out[i] = scale * (__builtin_amdgcn_exp2f((dv - d_lse) * kLog2e) - pt);
      else acc += (double)((pt > 0.f) ? pt * (dv - d_lse) : 0.f);
    }
  }
  if (BWD) return;
  __shared__ double s_red[kTokThreads];
  s_red[threadIdx.x] = acc;
  __syncthreads();
  for (int off = kTokThreads / 2; off >= 1; off >>= 1) {
    if ((int)threadIdx.x < off) s_red[threadIdx.x] += s_red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) a.loss_rows[r] = (float)(-(double)w * s_red[0]);
}

// single workgroup: |I| = sum of weights, loss = sum of rows / |I| (fixed-shape tree reductions)
__global__ __launch_bounds__(256) void k_token_loss_mean(TokenLossArgs a) {
  __shared__ double s_a[256], s_b[256];
  double sa = 0.0, sb = 0.0;
  for (int r = threadIdx.x; r < a.R; r += 256) {
    sa += (double)a.loss_rows[r];
    sb += a.weight ? (double)a.weight[r] : 1.0;
  }
  s_a[threadIdx.x] = sa;
  s_b[threadIdx.x] = sb;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {
    if ((int)threadIdx.x < off) {
      s_a[threadIdx.x] += s_a[threadIdx.x + off];
      s_b[threadIdx.x] += s_b[threadIdx.x + off];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double n = s_b[0];
    a.loss[0] = (n > 0.0) ? (float)(s_a[0] / n) : 0.f;
    a.inv_count_out[0] = (n > 0.0) ? (float)(1.0 / n) : 0.f;
  }
}

void launch_token_loss(const TokenLossArgs &a, int dtype, bool bwd, hipStream_t st) {
  const dim3 grid(a.R), block(kTokThreads);
  // rows start 16-byte aligned; the backward walks groups of four elements, the forward 16-byte vectors
  const int group = bwd ? 4 : (dtype == 0 ? 8 : 4);
  const bool vec = (a.V % group == 0) && (!bwd || (reinterpret_cast<uintptr_t>(a.grad) & 15) == 0);
  if (bwd) {
    if (dtype == 0) {
      if (vec) hipLaunchKernelGGL((k_token_loss<uint16_t, true, true>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((k_token_loss<uint16_t, true, false>), grid, block, 0, st, a);
    } else {
      if (vec) hipLaunchKernelGGL((k_token_loss<float, true, true>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((k_token_loss<float, true, false>), grid, block, 0, st, a);
    }
    return;
  }
  if (dtype == 0) {
    if (vec) hipLaunchKernelGGL((k_token_loss<uint16_t, false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((k_token_loss<uint16_t, false, false>), grid, block, 0, st, a);
  } else {
    if (vec) hipLaunchKernelGGL((k_token_loss<float, false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((k_token_loss<float, false, false>), grid, block, 0, st, a);
  }
  hipLaunchKernelGGL(k_token_loss_mean, dim3(1), dim3(256), 0, st, a);
}

// ------------------------------------------------------------------------------- calibration copy
// Plain 16-byte-per-lane copy of a known size: the yardstick that hardware HBM counters of the
// row kernels are scaled by.
__global__ __launch_bounds__(256) void k_copy16(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t nvec) {
  const int64_t step = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += step) dst[i] = src[i];
}

void launch_copy16(const void *src, void *dst, int64_t bytes, hipStream_t st) {
  hipLaunchKernelGGL(k_copy16, dim3(16384), dim3(256), 0, st, static_cast<const u32x4 *>(src),
                     static_cast<u32x4 *>(dst), bytes / 16);
}

// ------------------------------------------------------------------------------- launchers
// One wave per row streams best when rows are long and plentiful (one threshold, one list per
// row).  With few rows, or short ones, split a row over more waves so the chip stays full.
static int choose_waves(int forced, int V, int blocks, int elems_per_tile) {
  if (forced) return forced;
  const int64_t wave_slots = 256 * 28;   // CUs x resident waves per CU at this kernel's register use
  int w = 1;
  while (w < 8 && (int64_t)blocks * w < wave_slots && V / (2 * w) >= 2 * elems_per_tile) w *= 2;
  return w;
}


template <typename T, int MODE>
static void launch_row_stats_m(const RowStatsArgs &a, int blocks, hipStream_t st) {
  const int w = choose_waves(a.waves, a.V, blocks, kWave * kRowLoads * Elem<T>::kPerVec);
  switch (w) {
    case 1: hipLaunchKernelGGL((k_row_stats<T, 1, kRowLoads, MODE>), dim3(blocks), dim3(64), 0, st, a); break;
    case 2: hipLaunchKernelGGL((k_row_stats<T, 2, kRowLoads, MODE>), dim3(blocks), dim3(128), 0, st, a); break;
    case 8: hipLaunchKernelGGL((k_row_stats<T, 8, kRowLoads, MODE>), dim3(blocks), dim3(512), 0, st, a); break;
    default: hipLaunchKernelGGL((k_row_stats<T, 4, kRowLoads, MODE>), dim3(blocks), dim3(256), 0, st, a); break;
  }
}

template <typename T>
static void launch_row_stats_t(const RowStatsArgs &a, int blocks, hipStream_t st) {
  if (a.top_tok == nullptr) launch_row_stats_m<T, kLseOnly>(a, blocks, st);
  else if (a.ktop == 1) launch_row_stats_m<T, kTargetArgmax>(a, blocks, st);
  else launch_row_stats_m<T, kDraftTopK>(a, blocks, st);
}

void launch_row_stats(const RowStatsArgs &a, int dtype, int blocks, hipStream_t st) {
  if (dtype == 0) launch_row_stats_t<uint16_t>(a, blocks, st);
  else launch_row_stats_t<float>(a, blocks, st);
}

void launch_ppo_bwd(const PpoBwdArgs &a, int dtype, int blocks, hipStream_t st) {
  const bool vec = (a.V % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.grad_rows) & 15) == 0);
  if (dtype == 0) {
    if (vec) hipLaunchKernelGGL((k_ppo_bwd<uint16_t, true>), dim3(blocks), dim3(kBwdThreads), 0, st, a);
    else hipLaunchKernelGGL((k_ppo_bwd<uint16_t, false>), dim3(blocks), dim3(kBwdThreads), 0, st, a);
  } else {
    if (vec) hipLaunchKernelGGL((k_ppo_bwd<float, true>), dim3(blocks), dim3(kBwdThreads), 0, st, a);
    else hipLaunchKernelGGL((k_ppo_bwd<float, false>), dim3(blocks), dim3(kBwdThreads), 0, st, a);
  }
}

}  // namespace gto
