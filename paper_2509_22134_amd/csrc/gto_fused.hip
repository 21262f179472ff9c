// Fused LM-head variant: logits = hidden . W^T are produced tile by tile on the matrix cores and
// reduced to the row statistics (max, log-sum-exp, exact top-k) in the epilogue, so the logits
// never reach HBM.
//
//  k_fused_rows  : 256 x 256 output tile per workgroup iteration (4 waves, each 128 x 128 as 4 x 4
//                  MFMA 32x32x16 bf16 tiles, fp32 accumulators).  K slabs of 32 go from global
//                  memory straight into a ring of four LDS stages (no register staging), three
//                  slabs in flight while one is multiplied.  The launch is persistent (one
//                  workgroup per compute unit); a workgroup keeps its 256 rows while it moves
//                  along a patch row of the tile grid.  After each tile the accumulators are staged
//                  through LDS column-major; in the statistics passes thread t owns row t and folds
//                  its 256 new logits into its running (max, sum, top-k list) in registers; in the
//                  writing passes (gradient rows, bf16 planes, stored logits) the eight lanes of a
//                  row write contiguous bytes.
//  k_fused_merge : combines the partial results of a row (one per group and column phase) into the
//                  final statistics.
//  k_gather_dot  : single logits (hidden row . W row) for the few (row, token) pairs the reward
//                  and the surrogate need.
#include "gto_device.h"
#include "gto_kernels.h"

namespace gto {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int FBM = 256, FBN = 256;
constexpr int FBK = 32;                            // k extent of one LDS stage
constexpr int FROWB = FBK * 2;                     // bytes per staged row (bf16)
constexpr int FSTAGE_B = (FBM + FBN) * FROWB;      // bytes per stage: 256 hidden rows, then 256 W rows
constexpr int FNST = 4;                            // LDS stages: one being multiplied, FNST-1 landing (3 and 5 measured slower)
constexpr int FKT = 16;                            // capacity of the per-thread top list
constexpr int FSTG_CM = FBM + 4;                   // staging column stride (floats), column-major staging
constexpr size_t kFusedLdsBytes = (size_t)FNST * FSTAGE_B;
static_assert(kFusedLdsBytes >= (size_t)64 * FSTG_CM * sizeof(float), "staging area must fit");
static_assert(63 * FSTG_CM * sizeof(float) < 65536, "a row's 64 staged columns are reached with immediate offsets");
static_assert(FNST == 4, "the wait counts and the issue order of the main loop are written for this ring");

// wait until at most n of this wave's vector memory operations are outstanding (n known at compile time)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N == 0 || N == 8 || N == 16, "counts used by the slab ring");
  if (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  if (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
}

// 16 bytes per lane from global memory straight into LDS: lane l of the wave lands at lds_addr + 16 l
// (lds_addr is wave-uniform; the compiler moves it into M0); counted by vmcnt.
__device__ __forceinline__ void load_to_lds16(unsigned lds_addr, const void *g) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)g,
                                   (__attribute__((address_space(3))) void *)(uintptr_t)lds_addr, 16, 0, 0);
}

// index of the statistics entry (= logits slot) of the q-th used row of root r
__device__ __forceinline__ int64_t used_slot_index(int64_t gidx, int rho, int d, int k) {
  const int64_t r = gidx / rho;
  const int q = (int)(gidx - r * rho);
  return r * d * k + (q ? k + q - 1 : 0);
}

template <int KT>
struct RowState {
  float m, c;
  double s;
  float v[KT];
  int id[KT];
};

template <int KT>
__device__ __forceinline__ void list_insert(float (&v)[KT], int (&id)[KT], float x, int xi) {
  // v/id sorted best first; branch-free shift-insert
  bool prev = false;   // "x beats entry i-1"
  float pv = 0.f;
  int pi = 0;
#pragma unroll
  for (int i = 0; i < KT; ++i) {
    const bool b = better(x, xi, v[i], id[i]);
    const float cv = v[i];
    const int ci = id[i];
    v[i] = b ? (prev ? pv : x) : cv;
    id[i] = b ? (prev ? pi : xi) : ci;
    prev = b;
    pv = cv;
    pi = ci;
  }
}

// ---- the GEMM main loop: acc += A . B^T over kt_count k slabs of 32, for the 256 x 256 tile of the
// workgroup; wave (wm, wn) owns the 128 x 128 quadrant as 4 x 4 MFMA 32x32x16 tiles.
//
// K slab s lands in ring stage s % 4 (global memory -> LDS directly); every wave issues 4 loads per
// operand and slab (load j = the 16-row group 64 wave + 16 j).  The matrix pipe is the unit to keep busy
// and this wave is the only one on its SIMD, so the instruction stream is laid out by hand: every MFMA is
// followed by at most one memory instruction (pinned by scheduling barriers), which issues while the
// MFMA executes.  One slab:
//   first half  (k units 0, 1): after MFMA 0..7 the fragment reads of the second half (the four W
//               fragments first: its first MFMA row needs them all); then the wait until slab s+1 has
//               landed, and the barrier
//   second half (k units 2, 3): after MFMA 0..7 the first-half fragments of slab s+1; after MFMA 8..15
//               the loads of slab s+3 (hidden states, then W): a slab is requested two and a half slabs
//               (about 5000 clocks) before its first use, which is what a miss in the L2 needs here
struct SlabRing {
  unsigned wbase;              // LDS byte address of this wave's 4 KB landing area inside stage 0
  const unsigned char *ldsb;   // the ring
  int fa_base, fb_base;        // this lane's fragment byte offsets inside a stage (k units 0 / 1)
};

// LOAD3: slab s+3 exists and is requested here.  PEND2: slab s+2 exists (its 8 loads are in flight at the
// wait).  NEXT: slab s+1 exists.
template <bool LOAD3, bool PEND2, bool NEXT>
__device__ __forceinline__ void slab_step(f32x16 (&acc)[4][4], bf16x8 (&fa)[2][4], bf16x8 (&fb)[2][4],
                                          const SlabRing &r, const uint16_t *(&ap)[4], const uint16_t *(&bp)[4],
                                          int stage) {
  const int s1 = (stage + 1) % FNST, s3 = (stage + 3) % FNST;
  const unsigned char *sS = r.ldsb + stage * FSTAGE_B;
  const unsigned char *nS = r.ldsb + s1 * FSTAGE_B;
#pragma unroll
  for (int idx = 0; idx < 16; ++idx) {
    const int i = idx >> 2, j = (i & 1) ? 3 - (idx & 3) : (idx & 3);    // boustrophedon: one operand changes per MFMA
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][i], fb[0][j], acc[i][j], 0, 0, 0);
    if (idx < 4) {
      fb[1][idx] = *reinterpret_cast<const bf16x8 *>(sS + (r.fb_base ^ 32) + idx * 32 * FROWB);
    } else if (idx < 8) {
      fa[1][idx - 4] = *reinterpret_cast<const bf16x8 *>(sS + (r.fa_base ^ 32) + (idx - 4) * 32 * FROWB);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  if (NEXT) {
    // this wave's share of slab s+1 has landed when at most the 8 loads of slab s+2 are still out; the
    // barrier extends that to the other waves' shares, and tells that every wave is past its reads of
    // slab s-1, whose stage the loads below overwrite
    if (PEND2) wait_vmcnt<8>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int idx = 0; idx < 16; ++idx) {
    const int i = idx >> 2, j = (i & 1) ? 3 - (idx & 3) : (idx & 3);
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[1][i], fb[1][j], acc[i][j], 0, 0, 0);
    if (NEXT) {
      if (idx < 4) fb[0][idx] = *reinterpret_cast<const bf16x8 *>(nS + r.fb_base + idx * 32 * FROWB);
      else if (idx < 8) fa[0][idx - 4] = *reinterpret_cast<const bf16x8 *>(nS + r.fa_base + (idx - 4) * 32 * FROWB);
    }
    if (LOAD3) {
      if (idx >= 8 && idx < 12) {
        load_to_lds16(r.wbase + s3 * FSTAGE_B + (idx - 8) * 1024, ap[idx - 8]);
        ap[idx - 8] += FBK;
      } else if (idx >= 12) {
        load_to_lds16(r.wbase + s3 * FSTAGE_B + FBM * FROWB + (idx - 12) * 1024, bp[idx - 12]);
        bp[idx - 12] += FBK;
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// ap[j] / bp[j]: this lane's global address, in slab 0, for load j of the row operand / the column
// operand: the 16 bytes of row ld_row + 16 j at k unit ld_unit (see the callers); both advance by one slab
// per load.  Every wave of the workgroup calls this with the same kt_count >= 1; on return all fragment
// reads of the caller's wave are done and nothing of this call is in flight.
__device__ __forceinline__ void tile_mainloop(f32x16 (&acc)[4][4], uint16_t *lds, unsigned wbase, int lane, int wm,
                                              int wn, int kt_count, const uint16_t *(&ap)[4],
                                              const uint16_t *(&bp)[4]) {
  SlabRing r;
  r.wbase = wbase;
  r.ldsb = reinterpret_cast<const unsigned char *>(lds);
  // Fragment byte offsets of this lane inside a stage: row (lane & 31) of each 32-row tile; the
  // 16-byte unit 2 h + (lane >> 5) of k half h sits at unit ^ ((row / 4) % 4).
  const int fsw = ((lane >> 5) ^ ((lane >> 2) & 3)) * 16;
  r.fa_base = (wm * 128 + (lane & 31)) * FROWB + fsw;
  r.fb_base = (FBM + wn * 128 + (lane & 31)) * FROWB + fsw;
  __syncthreads();                           // the previous user of the ring (an epilogue's staging area) is done
  // prologue: slabs 0, 1 and 2
#pragma unroll
  for (int s_ = 0; s_ < 3; ++s_)
    if (s_ < kt_count) {
#pragma unroll
      for (int j = 0; j < 4; ++j) { load_to_lds16(wbase + s_ * FSTAGE_B + j * 1024, ap[j]); ap[j] += FBK; }
#pragma unroll
      for (int j = 0; j < 4; ++j) { load_to_lds16(wbase + s_ * FSTAGE_B + FBM * FROWB + j * 1024, bp[j]); bp[j] += FBK; }
    }
  // slab 0 landed; the later ones stay in flight
  if (kt_count > 2) wait_vmcnt<16>();
  else if (kt_count > 1) wait_vmcnt<8>();
  else wait_vmcnt<0>();
  __syncthreads();
  bf16x8 fa[2][4], fb[2][4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    fa[0][t] = *reinterpret_cast<const bf16x8 *>(r.ldsb + r.fa_base + t * 32 * FROWB);
    fb[0][t] = *reinterpret_cast<const bf16x8 *>(r.ldsb + r.fb_base + t * 32 * FROWB);
  }
  // slabs whose third successor exists request it; the last three request nothing
  int kt = 0;
  for (; kt + 3 < kt_count; ++kt) slab_step<true, true, true>(acc, fa, fb, r, ap, bp, kt & 3);
  if (kt + 2 < kt_count) { slab_step<false, true, true>(acc, fa, fb, r, ap, bp, kt & 3); ++kt; }
  if (kt + 1 < kt_count) { slab_step<false, false, true>(acc, fa, fb, r, ap, bp, kt & 3); ++kt; }
  slab_step<false, false, false>(acc, fa, fb, r, ap, bp, kt & 3);
}

// ---- work distribution of the row pass
// The 256 x 256 output tiles form an (m_blocks x n_tiles) grid; it is cut into patches of pr row blocks x
// pc column tiles: PR patch rows of QC patches ("patch steps").  The launch has G groups of pr * pc
// workgroups; workgroup (dr, dc) of a group computes tile (row block P pr + dr, column tile Q pc + dc) of
// every step (P, Q) its group owns, one after the other.  A group owns
//   - base = PR / G whole patch rows (group x: rows x base .. (x+1) base - 1), swept left to right, and
//   - an equal share of the steps of the remaining PR % G patch rows (row-major, contiguous).
// Consecutive steps of a patch row keep the row block, so a workgroup's 256 rows carry their statistics in
// registers from tile to tile and write one partial result per (row, group, dc) when a patch row (or the
// group's share of it) ends.
//   - Workgroup i of a launch runs on XCD i % 8, so with G = 8 a group is the 32 compute units of one XCD:
//     at any time its L2 serves pr row-operand streams and pc column-operand streams to pr * pc workgroups.
//   - While the groups sweep their whole patch rows they all sit at about the same column position, so a
//     column-operand tile is fetched from HBM by the first group and from the memory-side cache by the others.
//   - Every group gets the same number of steps to within one, whatever the shape: no tail of idle
//     compute units, and nothing depends on the row count being known on the host (a launch over a
//     device-side row list reads its count here).
struct RowSched {
  int m_blocks, n_tiles, PR, QC, pr, pc, G;
  int base;         // whole patch rows per group
  int64_t Tr;       // steps of the remaining patch rows, shared out evenly
};
__device__ __forceinline__ RowSched make_sched(int64_t M, int n_tiles, int G, int pr, int pc) {
  RowSched s;
  s.m_blocks = (int)((M + FBM - 1) / FBM);
  s.n_tiles = n_tiles;
  s.pr = pr; s.pc = pc; s.G = G;
  s.PR = (s.m_blocks + pr - 1) / pr;
  s.QC = (n_tiles + pc - 1) / pc;
  s.base = s.PR / G;
  s.Tr = (int64_t)(s.PR - s.base * G) * s.QC;
  return s;
}
__device__ __forceinline__ int64_t rest_begin(const RowSched &s, int x) { return s.Tr * x / s.G; }
// number of steps of group x, and its i-th step as (patch row, patch column)
__device__ __forceinline__ int64_t group_steps(const RowSched &s, int x) {
  return (int64_t)s.base * s.QC + (rest_begin(s, x + 1) - rest_begin(s, x));
}
__device__ __forceinline__ void group_step(const RowSched &s, int x, int64_t i, int &P, int &Q) {
  const int64_t n1 = (int64_t)s.base * s.QC;
  if (i < n1) {
    P = x * s.base + (int)(i / s.QC);
    Q = (int)(i % s.QC);
  } else {
    const int64_t r = rest_begin(s, x) + (i - n1);
    P = s.base * s.G + (int)(r / s.QC);
    Q = (int)(r % s.QC);
  }
}
// does partial slot (group x, column phase dc) of row block `mblock` hold a result?
__device__ __forceinline__ bool slot_valid(const RowSched &s, int mblock, int slot) {
  const int x = slot / s.pc, dc = slot - x * s.pc;
  if (x >= s.G) return false;
  const int P = mblock / s.pr;
  if (P < s.base * s.G) return x == P / s.base && dc < s.n_tiles;
  const int64_t row_lo = (int64_t)(P - s.base * s.G) * s.QC;
  const int64_t lo = max(rest_begin(s, x), row_lo), hi = min(rest_begin(s, x + 1), row_lo + s.QC);
  if (lo >= hi) return false;
  return (int)(lo - row_lo) * s.pc + dc < s.n_tiles;   // the first tile of the segment exists (later ones lie further right)
}

enum FusedMode { kFusedStats = 0, kFusedBwd = 1, kFusedPlanes = 2, kFusedStore = 3 };

template <int KT, int MODE>
__global__ __launch_bounds__(256) void k_fused_rows(FusedArgs a) {
  extern __shared__ __align__(16) uint16_t lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const int64_t M = a.m_dev ? min((int64_t)*a.m_dev, a.M) : a.M;   // row count may live on the device
  const RowSched sc = make_sched(M, a.n_tiles, a.groups, a.patch_rows, a.patch_cols);
  const int grp = blockIdx.x % sc.G, cell = blockIdx.x / sc.G;       // workgroup (dr, dc) of group grp
  const int dr = cell / sc.pc, dc = cell - dr * sc.pc;
  const int slot = grp * sc.pc + dc;                                  // partial-result slot of a row
  const int n_slots = sc.G * sc.pc;
  const int64_t n_steps = group_steps(sc, grp);
  const int HD = a.hidden_dim;
  const int kt_count = HD / FBK;
  const uint16_t *__restrict__ Hp = static_cast<const uint16_t *>(a.hidden);
  const uint16_t *__restrict__ Wp = static_cast<const uint16_t *>(a.w);

  // global -> LDS assignment: one wave instruction fills 16 rows x 64 bytes; wave w issues the
  // row groups 64 w + 16 j (j = 0..3) of both operands.  Lane l lands at row l/4, 16-byte unit
  // l%4 of its group; it fetches the unit (l%4) ^ ((row/4)%4) of that row, so that the fragment
  // reads (32 rows at one k unit) spread over all LDS banks.
  const int ld_row = 64 * wave + (lane >> 2);            // + 16 j
  const int ld_unit = (lane & 3) ^ ((lane >> 4) & 3);
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)lds;
  const unsigned wbase = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)wave * 4096u);
  // the list keeps the KT >= ktop best of the row; its last entry is the insertion threshold
  RowState<KT> st;
  const int ktop = a.ktop;
  // Writing modes (backward, planes, store): a wave writes the rows 64 wave .. 64 wave + 63 of the tile, eight
  // at a time; lane l then holds four consecutive columns (4 (l % 8) ..) of row 8 it + l / 8, so that the eight
  // lanes of a row write 128 contiguous bytes of an fp32 row (64 of a bf16 plane) per store instruction.  A
  // lane therefore keeps the parameters of its eight rows (it = 0..7) for the whole patch row.
  constexpr bool kWrites = (MODE != kFusedStats);
  constexpr int NR = kWrites ? 8 : 1;
  float e_lse[NR], e_coef[NR];
  int e_tok[NR];
  int64_t e_base[NR];        // element offset of the row in the output (gradient rows / planes / stored rows); -1: no row
  double e_others[NR];       // backward and planes: sum of the probabilities of all tokens but the accepted one
#pragma unroll
  for (int it = 0; it < NR; ++it) { e_lse[it] = 0.f; e_coef[it] = 0.f; e_tok[it] = -1; e_base[it] = -1; e_others[it] = 0.0; }
  const uint16_t *a_ptr[4] = {nullptr, nullptr, nullptr, nullptr};
  int64_t row0 = 0;
  int cur_P = -1;
  bool rows_live = false;      // this workgroup's row block of the current patch row exists

  // partial results of the row-block segment that ends (patch row finished, or the group's range did)
  auto flush = [&]() {
    if constexpr (MODE == kFusedStore) {
      return;
    } else if constexpr (kWrites) {
      // the eight lanes of a row add up their column groups (fixed order), lane 0 of the eight writes
#pragma unroll
      for (int it = 0; it < NR; ++it) {
        double v = e_others[it];
        v += __shfl_xor(v, 1, kWave);
        v += __shfl_xor(v, 2, kWave);
        v += __shfl_xor(v, 4, kWave);
        const int64_t g = row0 + wave * 64 + 8 * it + (lane >> 3);
        if ((lane & 7) == 0 && g < M) a.part_s[g * n_slots + slot] = v;
      }
    } else {
      const int64_t g = row0 + tid;
      if (g >= M) return;
      const int64_t pi = g * n_slots + slot;
      a.part_m[pi] = st.m;
      a.part_c[pi] = st.c;
      a.part_s[pi] = st.s;
#pragma unroll
      for (int i = 0; i < KT; ++i) {
        if (i < ktop) {
          a.part_v[pi * ktop + i] = st.v[i];
          a.part_i[pi * ktop + i] = st.id[i];
        }
      }
    }
  };

  for (int64_t step = 0; step < n_steps; ++step) {
    int P, Q;
    group_step(sc, grp, step, P, Q);
    if (P != cur_P) {
      if (rows_live) flush();
      cur_P = P;
      const int mblock = P * sc.pr + dr;
      rows_live = mblock < sc.m_blocks;
      row0 = (int64_t)mblock * FBM;
      st.m = neg_inf(); st.c = 0.f; st.s = 0.0;
#pragma unroll
      for (int i = 0; i < KT; ++i) { st.v[i] = neg_inf(); st.id[i] = kNoId; }
#pragma unroll
      for (int it = 0; it < NR; ++it) { e_base[it] = -1; e_others[it] = 0.0; e_tok[it] = -1; }
      if (rows_live) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          int64_t g = row0 + ld_row + 16 * j;
          if (g >= M) g = M - 1;
          const int64_t hs = a.row_list ? (int64_t)a.row_list[g] : used_slot_index(g, a.rho, a.d, a.kslots);
          a_ptr[j] = Hp + hs * HD + ld_unit * 8;
        }
        if constexpr (kWrites) {
#pragma unroll
          for (int it = 0; it < NR; ++it) {
            const int64_t gme = row0 + wave * 64 + 8 * it + (lane >> 3);
            if (gme < M) {
              if constexpr (MODE == kFusedStore) {
                e_base[it] = gme * a.store_pitch;
              } else {
                const int pidx = a.list_p[gme];
                const int rr = pidx / a.d;
                e_lse[it] = a.lse_by_slot[a.row_list[gme]];
                e_coef[it] = a.coef[rr];
                e_tok[it] = a.sel_tok[(int64_t)rr * a.g + a.path_node[pidx]];
                e_base[it] = (MODE == kFusedBwd) ? (int64_t)pidx * a.V : gme * (int64_t)a.V;
              }
            }
          }
        }
      }
    }
    const int tile = Q * sc.pc + dc;
    if (!rows_live || tile >= sc.n_tiles) continue;     // uniform over the workgroup
    const int n0 = tile * FBN;
    const uint16_t *b_ptr[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + ld_row + 16 * j;
      if (n >= a.V) n = a.V - 1;
      b_ptr[j] = Wp + (int64_t)n * HD + ld_unit * 8;
    }
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    {
      const uint16_t *ap[4], *bp[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) { ap[j] = a_ptr[j]; bp[j] = b_ptr[j]; }
      tile_mainloop(acc, lds, wbase, lane, wm, wn, kt_count, ap, bp);
    }
    __syncthreads();                           // all fragment reads done before the staging area is written

    float *stg = reinterpret_cast<float *>(lds);
    if constexpr (MODE == kFusedStats) {
      // ---- epilogue of the statistics pass: thread t owns row t.  Four phases; phase nt takes column
      // tile nt of both wave columns (64 columns, every wave takes part) through a column-major staging
      // area: the four consecutive rows a lane holds of a column leave as one 16-byte write (16 writes
      // per wave and phase, conflict-free with the column stride FSTG_CM), and a thread then reads its
      // row with one 4-byte read per column, all 64 issued back to back.
      const bool full_tile = (n0 + FBN <= a.V);
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        {
          float *wcol = stg + (wn * 32 + (lane & 31)) * FSTG_CM + wm * 128 + 4 * (lane >> 5);
#pragma unroll
          for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
              const f32x4 q = {acc[mt][nt][4 * g4], acc[mt][nt][4 * g4 + 1], acc[mt][nt][4 * g4 + 2],
                               acc[mt][nt][4 * g4 + 3]};
              *reinterpret_cast<f32x4 *>(wcol + mt * 32 + 8 * g4) = q;
            }
            __builtin_amdgcn_sched_barrier(0);   // 16 accumulator reads at a time keep the register pressure low
          }
        }
        __syncthreads();
        // staged column c is vocabulary entry n0 + 128 (c / 32) + 32 nt + c % 32
        const int cid0 = n0 + nt * 32;
        float x[64];
#pragma unroll
        for (int c = 0; c < 64; ++c) x[c] = stg[c * FSTG_CM + tid];
        if (!full_tile) {
#pragma unroll
          for (int c = 0; c < 64; ++c)
            if (cid0 + (c >> 5) * 128 + (c & 31) >= a.V) x[c] = neg_inf();     // adds nothing to max and sum
        }
        // One pass over the 64 new logits: maximum and sum of exp2 against the reference exponent the
        // row already has (st.c, at most 2 below its maximum in the log2 domain).  The sum is
        // re-referenced when the maximum has moved more than that above st.c, and recomputed in the rare
        // case that the old reference could have overflowed (or when the row has none yet).
        const bool have_ref = (st.m != neg_inf());
        const float c_ref = have_ref ? st.c : 0.f;
        float cm = neg_inf(), p = 0.f;
#pragma unroll
        for (int c = 0; c < 64; ++c) {
          cm = fmaxf(cm, x[c]);
          p += __builtin_amdgcn_exp2f(__builtin_fmaf(x[c], kLog2e, -c_ref));
        }
        // top-k insertions.  Some row of the workgroup reaches its threshold in almost every phase, and
        // the other waves wait for that wave at the barrier, so the search for the candidates must not walk
        // the 64 columns one by one: a row first marks, from registers, the columns that reach the threshold
        // it had on entry (later thresholds are higher), then visits only those (typically one or two).
        if (cm >= st.v[KT - 1]) {
          const float thr = st.v[KT - 1];
          uint32_t mask_lo = 0, mask_hi = 0;
#pragma unroll
          for (int c = 0; c < 32; ++c) {
            mask_lo |= (x[c] >= thr) ? (1u << c) : 0u;
            mask_hi |= (x[c + 32] >= thr) ? (1u << c) : 0u;
          }
          if (!full_tile) {      // masked columns hold -inf, which reaches the threshold of a list that is not full yet
            const int left = a.V - cid0;                      // valid columns from cid0 on (low half), from cid0 + 128 (high half)
            mask_lo &= (left >= 32) ? ~0u : (left <= 0 ? 0u : (1u << left) - 1u);
            const int left_hi = left - 128;
            mask_hi &= (left_hi >= 32) ? ~0u : (left_hi <= 0 ? 0u : (1u << left_hi) - 1u);
          }
          while ((mask_lo | mask_hi) != 0u) {
            int c;
            if (mask_lo != 0u) { c = __builtin_ctz(mask_lo); mask_lo &= mask_lo - 1u; }
            else { c = 32 + __builtin_ctz(mask_hi); mask_hi &= mask_hi - 1u; }
            const float xv = stg[c * FSTG_CM + tid];
            const int xi = cid0 + (c >> 5) * 128 + (c & 31);
            if (better(xv, xi, st.v[KT - 1], st.id[KT - 1])) list_insert<KT>(st.v, st.id, xv, xi);
          }
        }
        const float m_new = fmaxf(st.m, cm);
        const float over = __builtin_fmaf(cm, kLog2e, -c_ref);     // how far the new maximum is above the reference
        if (!have_ref || over > 100.f) {
          const float c_new = (m_new == neg_inf()) ? 0.f : m_new * kLog2e;
          float p2 = 0.f;
#pragma unroll
          for (int c = 0; c < 64; ++c) p2 += __builtin_amdgcn_exp2f(__builtin_fmaf(x[c], kLog2e, -c_new));
          const double s = have_ref ? st.s * (double)__builtin_amdgcn_exp2f(st.c - c_new) : 0.0;
          st.s = s + (double)p2;
          st.c = c_new;
        } else if (over > 1.f) {       // keep the dominant terms' exponents small: their rounding scales with |exponent|
          const float c_new = m_new * kLog2e;
          st.s = (st.s + (double)p) * (double)__builtin_amdgcn_exp2f(st.c - c_new);
          st.c = c_new;
        } else {
          st.s += (double)p;
        }
        st.m = m_new;
        __syncthreads();
      }
    } else {
      // ---- epilogue of the writing modes: the same four phases and the same column-major staging; then
      // every wave walks its 64 rows eight at a time (see the lane mapping above), two pieces of 32 columns each
      const bool vec4 = ((a.V & 3) == 0) && (MODE != kFusedStore || (a.store_pitch & 3) == 0);
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        {
          float *wcol = stg + (wn * 32 + (lane & 31)) * FSTG_CM + wm * 128 + 4 * (lane >> 5);
#pragma unroll
          for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
              const f32x4 q = {acc[mt][nt][4 * g4], acc[mt][nt][4 * g4 + 1], acc[mt][nt][4 * g4 + 2],
                               acc[mt][nt][4 * g4 + 3]};
              *reinterpret_cast<f32x4 *>(wcol + mt * 32 + 8 * g4) = q;
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < NR; ++it) {
          const float *src = stg + wave * 64 + 8 * it + (lane >> 3);
#pragma unroll
          for (int piece = 0; piece < 2; ++piece) {
            const int c0 = piece * 32 + 4 * (lane & 7);                       // staged column of this lane's first element
            const int col = n0 + piece * 128 + nt * 32 + 4 * (lane & 7);      // its vocabulary entry
            if (e_base[it] < 0 || col >= a.V) continue;
            float x[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = src[(c0 + e) * FSTG_CM];
            const bool whole = vec4 && (col + 3 < a.V);
            if constexpr (MODE == kFusedStore) {
              float *o = a.store_rows + e_base[it] + col;
              if (whole) {
                const f32x4 q = {x[0], x[1], x[2], x[3]};
                *reinterpret_cast<f32x4 *>(o) = q;
              } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                  if (col + e < a.V) o[e] = x[e];
              }
            } else {
              // -coef * softmax; the accepted token's probability is left out of the sum (and, in the planes, out
              // of the entry) so that its coefficient coef * (1 - p_token) can be formed without cancellation
              float gq[4], part = 0.f;
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const bool is_tok = (col + e == e_tok[it]);
                float pv = (col + e < a.V) ? __builtin_amdgcn_exp2f((x[e] - e_lse[it]) * kLog2e) : 0.f;
                if (MODE == kFusedPlanes && is_tok) pv = 0.f;
                part += is_tok ? 0.f : pv;
                gq[e] = -e_coef[it] * pv;
              }
              e_others[it] += (double)part;
              if constexpr (MODE == kFusedBwd) {
                float *o = a.grad_rows + e_base[it] + col;
                if (whole) {
                  const f32x4 q = {gq[0], gq[1], gq[2], gq[3]};
                  __builtin_nontemporal_store(q, reinterpret_cast<f32x4 *>(o));
                } else {
#pragma unroll
                  for (int e = 0; e < 4; ++e)
                    if (col + e < a.V) o[e] = gq[e];
                }
              } else {
                // planes: value = hi + lo in bf16 (V is a multiple of 32 in this mode: whole 8-byte stores)
                uint16_t hq[4], lq[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const __bf16 hb = (__bf16)gq[e];
                  const __bf16 lb = (__bf16)(gq[e] - (float)hb);
                  hq[e] = __builtin_bit_cast(uint16_t, hb);
                  lq[e] = __builtin_bit_cast(uint16_t, lb);
                }
                const u32x2 ho = {(uint32_t)hq[0] | ((uint32_t)hq[1] << 16), (uint32_t)hq[2] | ((uint32_t)hq[3] << 16)};
                const u32x2 lo = {(uint32_t)lq[0] | ((uint32_t)lq[1] << 16), (uint32_t)lq[2] | ((uint32_t)lq[3] << 16)};
                *reinterpret_cast<u32x2 *>(a.plane_hi + e_base[it] + col) = ho;
                *reinterpret_cast<u32x2 *>(a.plane_lo + e_base[it] + col) = lo;
              }
            }
          }
        }
        __syncthreads();
      }
    }
  }

  if (rows_live) flush();
}

// One wave per row: merge the partial results of the row's segments (one lane per slot) into the final
// statistics.  Which slots hold a result follows from the launch geometry alone (slot_valid).
__global__ __launch_bounds__(64) void k_fused_merge(FusedArgs a) {
  const int64_t g = blockIdx.x;
  const int64_t M = a.m_dev ? min((int64_t)*a.m_dev, a.M) : a.M;
  if (g >= M) return;
  const int lane = threadIdx.x;
  const int ktop = a.ktop;
  const RowSched sc = make_sched(M, a.n_tiles, a.groups, a.patch_rows, a.patch_cols);
  const int n_slots = sc.G * sc.pc;                       // <= 64: one lane per slot
  const int64_t oi = a.row_list ? (a.out_by_list ? g : (int64_t)a.row_list[g])
                                : used_slot_index(g, a.rho, a.d, a.kslots);
  __shared__ float s_v[64 * FKT];
  __shared__ int s_i[64 * FKT];
  __shared__ int s_claimed[FKT];
  const bool valid = lane < n_slots && slot_valid(sc, (int)(g / FBM), lane);
  float m = neg_inf(), c = neg_inf();
  double s = 0.0;
  if (valid) {
    m = a.part_m[g * n_slots + lane];
    if (m != neg_inf()) {
      c = a.part_c[g * n_slots + lane];
      s = a.part_s[g * n_slots + lane];
    }
  }
  const float Mx = wave_max(m);
  const float C = wave_max(c);
  const double S = wave_sum((m == neg_inf()) ? 0.0 : s * (double)__builtin_amdgcn_exp2f(c - C));
  const double lse = (double)Mx + kLn2 * (((double)C - (double)Mx * (double)kLog2e) + log2(S));
  if (lane == 0) {
    if (a.row_max) a.row_max[oi] = Mx;
    a.row_lse[oi] = (float)lse;
  }
  if (a.top_tok == nullptr) return;
  // the valid slots' lists, packed: slot j of the packed order is the j-th valid lane
  const uint64_t vmask = __builtin_amdgcn_ballot_w64(valid);
  const int n_valid = __builtin_popcountll(vmask);
  const int my_pos = __builtin_popcountll(vmask & ((1ull << lane) - 1ull));
  if (lane < FKT) s_claimed[lane] = 0;
  if (valid) {
    for (int i = 0; i < ktop; ++i) {
      s_v[my_pos * ktop + i] = a.part_v[(g * n_slots + lane) * ktop + i];
      s_i[my_pos * ktop + i] = a.part_i[(g * n_slots + lane) * ktop + i];
    }
  }
  __syncthreads();
  const int total = n_valid * ktop;
  for (int j = lane; j < total; j += 64) {
    const float v = s_v[j];
    const int id = s_i[j];
    if (id == kNoId) continue;
    int rank = 0;
    for (int u = 0; u < total; ++u) rank += better(s_v[u], s_i[u], v, id) ? 1 : 0;
    if (rank < ktop) {
      s_claimed[rank] = 1;
      a.top_tok[oi * ktop + rank] = id;
      if (a.top_logp) a.top_logp[oi * ktop + rank] = fminf((float)((double)v - lse), 0.f);
      if (a.top_logit) a.top_logit[oi * ktop + rank] = v;
    }
  }
  __syncthreads();
  // ranks no entry claimed (possible only when the row held NaNs): a valid token id with probability zero
  if (lane < ktop && s_claimed[lane] == 0) {
    a.top_tok[oi * ktop + lane] = lane;
    if (a.top_logp) a.top_logp[oi * ktop + lane] = neg_inf();
    if (a.top_logit) a.top_logit[oi * ktop + lane] = neg_inf();
  }
}

// sum, over the valid slots of row g in slot order, of the per-segment sums of the non-token probabilities
__device__ __forceinline__ double sum_others(const double *part_s, int64_t g, const RowSched &sc) {
  const int n_slots = sc.G * sc.pc;
  double tot = 0.0;
  for (int c = 0; c < n_slots; ++c)
    if (slot_valid(sc, (int)(g / FBM), c)) tot += part_s[g * n_slots + c];
  return tot;
}

// Backward fix-up, one thread per processed row: the accepted token's entry is coef times the sum
// of all other probabilities (summed over the vocabulary chunks in a fixed order).
__global__ void k_fused_bwd_fixup(FusedArgs a) {
  const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t M = a.m_dev ? min((int64_t)*a.m_dev, a.M) : a.M;
  if (g >= M) return;
  const double tot = sum_others(a.part_s, g, make_sched(M, a.n_tiles, a.groups, a.patch_rows, a.patch_cols));
  const int pidx = a.list_p[g];
  const int rr = pidx / a.d;
  const int tok = a.sel_tok[(int64_t)rr * a.g + a.path_node[pidx]];
  if (tok >= 0 && tok < a.V) a.grad_rows[(int64_t)pidx * a.V + tok] = (float)((double)a.coef[rr] * tot);
}

// Ordered compaction (single workgroup): the (root, step) pairs that carry a gradient, their
// hidden-row slots, and grad_slot for every pair.
__global__ __launch_bounds__(1024) void k_bwd_rows(BwdRowsArgs a) {
  __shared__ int s_wave[16];
  __shared__ int s_base;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) s_base = 0;
  __syncthreads();
  const int n = a.R * a.d;
  for (int p0 = 0; p0 < n; p0 += 1024) {
    const int p = p0 + tid;
    bool valid = false;
    int j = -1;
    if (p < n) {
      j = a.path_slot[p];
      valid = (j >= 0) && (a.coef[p / a.d] != 0.f);
      a.grad_slot[p] = valid ? j : -1;
    }
    const uint64_t bal = __builtin_amdgcn_ballot_w64(valid);
    const int before = __builtin_popcountll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) s_wave[wave] = __builtin_popcountll(bal);
    __syncthreads();
    int off = s_base;
    for (int w = 0; w < wave; ++w) off += s_wave[w];
    if (valid) {
      const int r = p / a.d, t = p - r * a.d;
      a.list_p[off + before] = p;
      a.list_slot[off + before] = (int)stat_index(r, t, j, a.d, a.k);
    }
    __syncthreads();
    if (tid == 0) {
      int tot = 0;
      for (int w = 0; w < 16; ++w) tot += s_wave[w];
      s_base += tot;
    }
    __syncthreads();
  }
  if (tid == 0) *a.count = s_base;
}

// Ordered compaction (single workgroup) of the slots whose flag is set: list of slot indices + count.
__global__ __launch_bounds__(1024) void k_compact_flags(const int32_t *flags, int n, int32_t *list, int32_t *count) {
  __shared__ int s_wave[16];
  __shared__ int s_base;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) s_base = 0;
  __syncthreads();
  for (int p0 = 0; p0 < n; p0 += 1024) {
    const int p = p0 + tid;
    const bool valid = (p < n) && (flags[p] != 0);
    const uint64_t bal = __builtin_amdgcn_ballot_w64(valid);
    const int before = __builtin_popcountll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) s_wave[wave] = __builtin_popcountll(bal);
    __syncthreads();
    int off = s_base;
    for (int w = 0; w < wave; ++w) off += s_wave[w];
    if (valid) list[off + before] = p;
    __syncthreads();
    if (tid == 0) {
      int tot = 0;
      for (int w = 0; w < 16; ++w) tot += s_wave[w];
      s_base += tot;
    }
    __syncthreads();
  }
  if (tid == 0) *count = s_base;
}

void launch_compact_flags(const int32_t *flags, int n, int32_t *list, int32_t *count, hipStream_t st) {
  hipLaunchKernelGGL(k_compact_flags, dim3(1), dim3(1024), 0, st, flags, n, list, count);
}

__global__ void k_zero_rows(float *grad_rows, const int32_t *grad_slot, int V) {
  if (grad_slot[blockIdx.x] >= 0) return;
  float *o = grad_rows + (int64_t)blockIdx.x * V;
  for (int i = threadIdx.x; i < V; i += blockDim.x) o[i] = 0.f;
}

// One wave per (row slot, token): fp32 dot product of a hidden row and a W row.
__global__ __launch_bounds__(64) void k_gather_dot(GatherDotArgs a) {
  const int64_t p = blockIdx.x;
  const int lane = threadIdx.x;
  const int64_t slot = a.slot[p];
  const int tok = a.tok[p];
  if (slot < 0 || tok < 0 || tok >= a.V) {
    if (lane == 0) a.out[p] = 0.f;
    return;
  }
  const uint16_t *h = static_cast<const uint16_t *>(a.hidden) + slot * a.hidden_dim;
  const uint16_t *w = static_cast<const uint16_t *>(a.w) + (int64_t)tok * a.hidden_dim;
  float acc = 0.f;
  for (int e0 = lane * 8; e0 < a.hidden_dim; e0 += 64 * 8) {
    const u32x4 hq = *reinterpret_cast<const u32x4 *>(h + e0);
    const u32x4 wq = *reinterpret_cast<const u32x4 *>(w + e0);
    float hx[8], wx[8];
    Elem<uint16_t>::unpack(hq, hx);
    Elem<uint16_t>::unpack(wq, wx);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(hx[e], wx[e], acc);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, kWave);
  if (lane == 0) a.out[p] = acc;
}

// Hidden-state gradient, one 256 (rows of the list) x 256 (hidden columns) tile per workgroup and split of
// the contraction: partial[split] = sum over the split's k slabs of G . W, G = [plane_hi | plane_lo]
// (contraction length 2 V), W hidden-major so that both operands are contiguous along the vocabulary.
__global__ __launch_bounds__(256) void k_fused_dh(FusedDhArgs a) {
  extern __shared__ __align__(16) uint16_t lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int split = blockIdx.x % a.n_splits;
  const int rest = blockIdx.x / a.n_splits;
  const int hblock = rest % a.h_blocks, mblock = rest / a.h_blocks;
  const int64_t M = min((int64_t)*a.m_dev, a.M);
  const int64_t row0 = (int64_t)mblock * FBM;
  if (row0 >= M) return;
  const int nks = a.V / FBK;                                  // slabs per plane
  const int s0 = split * a.slabs_per_split;
  const int kt_count = min(a.slabs_per_split, 2 * nks - s0);  // >= 1 by the launch geometry
  const int h0 = hblock * FBN;
  const int ld_row = 64 * wave + (lane >> 2);
  const int ld_unit = (lane & 3) ^ ((lane >> 4) & 3);
  const uint16_t *a_hi[4], *a_lo[4], *b_ptr[4];
  const uint16_t *Wp = static_cast<const uint16_t *>(a.w_hv);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int64_t g = row0 + ld_row + 16 * j;
    if (g >= M) g = M - 1;
    a_hi[j] = a.plane_hi + g * a.V + ld_unit * 8;
    a_lo[j] = a.plane_lo + g * a.V + ld_unit * 8;
    int n = h0 + ld_row + 16 * j;
    if (n >= a.hidden_dim) n = a.hidden_dim - 1;
    b_ptr[j] = Wp + (int64_t)n * a.V + ld_unit * 8;
  }
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)lds;
  const unsigned wbase = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)wave * 4096u);
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  // the split's slabs [s0, s0 + kt_count) of the contraction over [hi plane | lo plane]: the part inside the
  // hi plane, then the part inside the lo plane, each a contiguous k range of both operands
  const int n_hi = max(0, min(s0 + kt_count, nks) - s0);
  if (n_hi > 0) {
    const uint16_t *ap[4], *bp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { ap[j] = a_hi[j] + (int64_t)s0 * FBK; bp[j] = b_ptr[j] + (int64_t)s0 * FBK; }
    tile_mainloop(acc, lds, wbase, lane, wm, wn, n_hi, ap, bp);
  }
  if (kt_count - n_hi > 0) {
    const int l0 = max(s0, nks) - nks;
    const uint16_t *ap[4], *bp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { ap[j] = a_lo[j] + (int64_t)l0 * FBK; bp[j] = b_ptr[j] + (int64_t)l0 * FBK; }
    tile_mainloop(acc, lds, wbase, lane, wm, wn, kt_count - n_hi, ap, bp);
  }
  float *out = a.partial + (int64_t)split * a.M * a.hidden_dim;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t row = row0 + wm * 128 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        const int col = h0 + wn * 128 + j * 32 + (lane & 31);
        if (row < M && col < a.hidden_dim) out[row * a.hidden_dim + col] = acc[i][j][e];
      }
}

// dH row of list entry g: the splits in a fixed order, plus the accepted token's own term
// coef * (1 - p_token) * W[token, :], with 1 - p_token taken as the sum of the other probabilities.
__global__ __launch_bounds__(256) void k_fused_dh_reduce(FusedDhArgs a) {
  const int64_t g = blockIdx.x;
  if (g >= (int64_t)*a.m_dev) return;
  const int pidx = a.list_p[g];
  const int rr = pidx / a.d;
  const int tok = min(max(a.sel_tok[(int64_t)rr * a.g + a.path_node[pidx]], 0), a.V - 1);
  const float coef = a.coef[rr];
  const uint16_t *wrow = static_cast<const uint16_t *>(a.w_vh) + (int64_t)tok * a.hidden_dim;
  // sum of the probabilities of all tokens but the accepted one, from the plane pass's segments
  const int64_t M = min((int64_t)*a.m_dev, a.M);
  const double others = sum_others(a.part_s, g, make_sched(M, a.n_tiles, a.groups, a.patch_rows, a.patch_cols));
  const float ctok = (float)((double)coef * others);
  for (int h = threadIdx.x; h < a.hidden_dim; h += 256) {
    float sum = 0.f;
    for (int s = 0; s < a.n_splits; ++s) sum += a.partial[((int64_t)s * a.M + g) * a.hidden_dim + h];
    a.dh_rows[(int64_t)pidx * a.hidden_dim + h] = __builtin_fmaf(ctok, Elem<uint16_t>::load1(wrow + h), sum);
  }
}

template <typename K>
static void set_lds_attr(K kern) {
  (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kFusedLdsBytes);
}

static int fused_grid(const FusedArgs &a) { return a.groups * a.patch_rows * a.patch_cols; }

// the kernels that use the whole slab ring need the dynamic LDS limit raised once per process
// (initialisation of a function-local static is thread-safe)
static void ensure_lds_attrs() {
  static const bool done = [] {
    set_lds_attr(k_fused_rows<1, kFusedStats>);
    set_lds_attr(k_fused_rows<8, kFusedStats>);
    set_lds_attr(k_fused_rows<16, kFusedStats>);
    set_lds_attr(k_fused_rows<1, kFusedBwd>);
    set_lds_attr(k_fused_rows<1, kFusedPlanes>);
    set_lds_attr(k_fused_rows<1, kFusedStore>);
    set_lds_attr(k_fused_dh);
    return true;
  }();
  (void)done;
}

void launch_fused_rows(const FusedArgs &a, hipStream_t st) {
  ensure_lds_attrs();
  const int blocks = fused_grid(a);
  if (a.store_rows != nullptr)
    hipLaunchKernelGGL((k_fused_rows<1, kFusedStore>), dim3(blocks), dim3(256), kFusedLdsBytes, st, a);
  else if (a.plane_hi != nullptr)
    hipLaunchKernelGGL((k_fused_rows<1, kFusedPlanes>), dim3(blocks), dim3(256), kFusedLdsBytes, st, a);
  else if (a.grad_rows != nullptr)
    hipLaunchKernelGGL((k_fused_rows<1, kFusedBwd>), dim3(blocks), dim3(256), kFusedLdsBytes, st, a);
  else if (a.ktop <= 1)
    hipLaunchKernelGGL((k_fused_rows<1, kFusedStats>), dim3(blocks), dim3(256), kFusedLdsBytes, st, a);
  else if (a.ktop <= 8)
    hipLaunchKernelGGL((k_fused_rows<8, kFusedStats>), dim3(blocks), dim3(256), kFusedLdsBytes, st, a);
  else
    hipLaunchKernelGGL((k_fused_rows<16, kFusedStats>), dim3(blocks), dim3(256), kFusedLdsBytes, st, a);
}

void launch_fused_dh(const FusedDhArgs &a, hipStream_t st) {
  ensure_lds_attrs();
  hipLaunchKernelGGL(k_fused_dh, dim3((unsigned)(a.m_blocks * a.h_blocks * a.n_splits)), dim3(256), kFusedLdsBytes, st, a);
  hipLaunchKernelGGL(k_fused_dh_reduce, dim3((unsigned)a.M), dim3(256), 0, st, a);
}

void launch_fused_bwd_fixup(const FusedArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(k_fused_bwd_fixup, dim3((unsigned)((a.M + 255) / 256)), dim3(256), 0, st, a);
}

void launch_bwd_rows(const BwdRowsArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(k_bwd_rows, dim3(1), dim3(1024), 0, st, a);
}

void launch_zero_rows(float *grad_rows, const int32_t *grad_slot, int rows, int V, hipStream_t st) {
  hipLaunchKernelGGL(k_zero_rows, dim3(rows), dim3(256), 0, st, grad_rows, grad_slot, V);
}

void launch_fused_merge(const FusedArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(k_fused_merge, dim3((unsigned)a.M), dim3(64), 0, st, a);
}

void launch_gather_dot(const GatherDotArgs &a, hipStream_t st) {
  if (a.n > 0) hipLaunchKernelGGL(k_gather_dot, dim3((unsigned)a.n), dim3(64), 0, st, a);
}

}  // namespace gto
