// Reward composition, group normalisation, routing through phi and reward placement.
//
// The thin graph arrives as host arrays (the controller's view: role ids, routing ids,
// reward metadata); it is validated on the host, staged to the device and every step after
// that runs in kernels: per-turn reward r_v = lam_node r_node + lam_turn r_turn + lam_traj
// r_traj (Section "Agent-Specific Reward Interface"), the stable partition of turns by
// phi(role) into model-local streams (Sections "Agent--LLM Mapping", "Model-Local Buffers")
// and the alignment of each turn's reward with its token sequence (paragraph "Batch
// construction").
//
// Three kernels (four with normalisation groups).  k_turn_plan does everything that is per turn: one thread walks
// one trajectory's turns (a trajectory's turns are consecutive, and everything a turn needs from its neighbours -
// whether it opens or closes the trajectory's run inside its model's stream, how many steps lie between it and the
// run's next turn - lies inside its trajectory), blocks of 256 trajectories publish their per-model totals and read
// everybody else's to place themselves.  k_tokens writes everything that is per token in one pass over the streams
// (22 bytes per token, the mask read once); k_rowsel compacts the positions of the scored tokens (the gathered mask
// read again, 4 bytes per scored token written).
#include <algorithm>
#include <vector>

#include "umas_common.h"

namespace umas {

namespace {

constexpr int kPlanThreads = 256;  // trajectories per chunk of the plan kernel
constexpr int kPlanPerCu = 2;      // its workgroups per compute unit at most (one with more than two models): a fraction of what
                                   // the device holds at once, so all of them are resident, also next to a second call's
constexpr int kCnt = 3;            // per model and chunk: turns, tokens, trajectory runs
constexpr int kPlanWords = UMAS_MAX_MODELS * kCnt;
constexpr int kTokThreads = 256;
constexpr int kTokPerThread = 4;   // consecutive tokens of one thread in one round
constexpr int kTokRounds = 4;      // rounds of a block, kTokThreads * kTokPerThread tokens apart
constexpr int kTokRound = kTokThreads * kTokPerThread;
constexpr int kTokBlock = kTokRound * kTokRounds;
constexpr unsigned long long kMark = 1ull << 63;          // ready mark of a published count

// What the token kernel needs to know about one turn segment of a model-local stream.
struct __attribute__((aligned(16))) SegMeta {
  int64_t src;         // global index of the segment's first token
  int32_t turn;
  int32_t role;
  float rho;           // composed reward of the turn
  int32_t end_flags;   // flag bits of the segment's last token besides the mask bit
  int64_t pad;
};
static_assert(sizeof(SegMeta) == 32, "two 16-byte loads");

struct RouteWs {
  // the thin arrays, staged from the host in one copy (everything up to traj_norm)
  int32_t* role_to_model;
  int32_t* traj_turn_off;
  int32_t* turn_role;
  int64_t* turn_tok_off;
  int32_t* group_off;
  int32_t* group_members;
  float* role_reward;
  float* turn_reward;
  float* traj_reward;
  float* weights;       // [3 * n_roles]: role, turn, traj
  unsigned long long* plan_part;   // [n_chunks][kPlanWords] per-chunk totals of the plan kernel; zeros come with the staged copy
  // written on the device
  float* traj_norm;     // [n_traj]
  SegMeta* seg_meta;    // [n_turns] per segment slot
  int32_t* blk_first;   // [nblk_tok] segment that holds the first token of each token block
  unsigned long long* tok_count;   // [nblk_tok + groups] scored tokens of the token kernel's blocks, then of its groups of blocks
};

// Blocks of the token kernel are grouped 2^shift to a group, about the square root of their number and at least 64.
inline int group_shift(size_t nbk) {
  int sh = 6;
  while ((size_t{1} << (2 * sh)) < nbk) ++sh;
  return sh;
}
inline int plan_chunks(int n_traj) { return static_cast<int>(cdiv(n_traj > 0 ? n_traj : 1, kPlanThreads)); }

size_t carve(Carver& c, RouteWs& w, int n_roles, int n_traj, int n_turns, int64_t n_tokens) {
  const size_t nbk = cdiv(n_tokens > 0 ? n_tokens : 1, kTokBlock);
  w.role_to_model = c.take<int32_t>(n_roles);
  w.traj_turn_off = c.take<int32_t>(n_traj + 1);
  w.turn_role = c.take<int32_t>(n_turns);
  w.turn_tok_off = c.take<int64_t>(n_turns + 1);
  w.group_off = c.take<int32_t>(n_traj + 2);
  w.group_members = c.take<int32_t>(n_traj);
  w.role_reward = c.take<float>(static_cast<size_t>(n_traj) * n_roles);
  w.turn_reward = c.take<float>(n_turns);
  w.traj_reward = c.take<float>(n_traj);
  w.weights = c.take<float>(3 * n_roles);
  w.plan_part = c.take<unsigned long long>(static_cast<size_t>(plan_chunks(n_traj)) * kPlanWords);
  w.traj_norm = c.take<float>(n_traj);
  w.seg_meta = c.take<SegMeta>(n_turns);
  w.blk_first = c.take<int32_t>(nbk);
  w.tok_count = c.take<unsigned long long>(nbk + (nbk >> group_shift(nbk)) + 1);
  return c.off;
}

// ------------------------------------------------------------------ kernels

// z-score of trajectory rewards inside a group; one wavefront per group, float64 statistics.
__global__ void k_group_norm(const float* __restrict__ R, const int32_t* __restrict__ group_off,
                             const int32_t* __restrict__ members, int n_groups, float eps,
                             float* __restrict__ out) {
  const int lane = threadIdx.x & (kWave - 1);
  const int g = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (g >= n_groups) return;
  const int a = group_off[g], e = group_off[g + 1];
  if (e == a) return;
  double s = 0.0;
  for (int i = a + lane; i < e; i += kWave) s += static_cast<double>(R[members[i]]);
  const double mu = wave_sum(s) / static_cast<double>(e - a);
  double q = 0.0;
  for (int i = a + lane; i < e; i += kWave) {
    const double t = static_cast<double>(R[members[i]]) - mu;
    q += t * t;
  }
  const double sigma = sqrt(wave_sum(q) / static_cast<double>(e - a));
  for (int i = a + lane; i < e; i += kWave) {
    const int b = members[i];
    out[b] = static_cast<float>((static_cast<double>(R[b]) - mu) / (sigma + static_cast<double>(eps)));
  }
}

// ------------------------------------------------------------------ the plan: everything per turn
struct PlanArgs {
  int n_traj, n_turns, n_roles, n_models, n_chunks;
  int64_t n_tokens, n_count;          // n_count: words of tok_count to clear
  const int32_t* __restrict__ traj_turn_off;
  const int32_t* __restrict__ turn_role;
  const int32_t* __restrict__ role_to_model;
  const int64_t* __restrict__ turn_tok_off;
  const float* __restrict__ role_reward;   // NULL level = 0
  const float* __restrict__ turn_reward;
  const float* __restrict__ traj_reward;   // already normalised when groups are given
  const float* __restrict__ w_role;        // NULL weight = 1
  const float* __restrict__ w_turn;
  const float* __restrict__ w_traj;
  unsigned long long* __restrict__ plan_part;
  SegMeta* __restrict__ seg_meta;
  int32_t* __restrict__ blk_first;
  unsigned long long* __restrict__ tok_count;
  // outputs
  int64_t* __restrict__ model_tok_off;
  int32_t* __restrict__ model_turn_off;
  int32_t* __restrict__ model_trajrun_off;
  int64_t* __restrict__ model_rowsel_off;
  int64_t* __restrict__ turn_seg_off;
  int32_t* __restrict__ seg_turn;
  int64_t* __restrict__ traj_seg_off;
  float* __restrict__ turn_scalar;
  int32_t* __restrict__ turn_step;
};

// v[k] of a small per-model array with a run-time k, without indexing registers dynamically
template <typename T, int KM>
__device__ __forceinline__ T pick(const T (&v)[KM], int k) {
  T r = v[0];
#pragma unroll
  for (int i = 1; i < KM; ++i) r = k == i ? v[i] : r;
  return r;
}
template <typename T, int KM>
__device__ __forceinline__ void bump(T (&v)[KM], int k, T by) {
#pragma unroll
  for (int i = 0; i < KM; ++i) v[i] += k == i ? by : T(0);
}

// Per-model counts of one trajectory: turns, tokens, and whether the model has a run in it.
template <int KM>
struct TrajCounts {
  int64_t cnt[KM], tok[KM];
  uint32_t seen;
};
template <int KM>
__device__ __forceinline__ void traj_counts(const PlanArgs& A, const uint8_t* s_phi, int b, TrajCounts<KM>& c) {
#pragma unroll
  for (int k = 0; k < KM; ++k) { c.cnt[k] = 0; c.tok[k] = 0; }
  c.seen = 0;
  if (b >= A.n_traj) return;
  const int t0 = A.traj_turn_off[b], t1 = A.traj_turn_off[b + 1];
  int64_t g0 = A.turn_tok_off[t0];
  for (int u = t0; u < t1; ++u) {
    const int m = s_phi[A.turn_role[u]];
    const int64_t g1 = A.turn_tok_off[u + 1];
    bump(c.cnt, m, int64_t{1});
    bump(c.tok, m, g1 - g0);
    c.seen |= 1u << m;
    g0 = g1;
  }
}

// KM: the smallest of 1, 2, 4, 8 that is at least the number of models (per-model state lives in registers).
template <int KM>
__global__ void __launch_bounds__(kPlanThreads, 2)
k_turn_plan(PlanArgs A) {
  __shared__ int64_t smem[32];
  __shared__ long long s_res[2][kPlanWords];         // [total | before this chunk][model, counter]
  __shared__ uint8_t s_phi[UMAS_MAX_ROLES];          // role -> model
  const int tid = threadIdx.x;
  const int K = A.n_models;
  if (tid < A.n_roles) s_phi[tid] = static_cast<uint8_t>(A.role_to_model[tid]);
  __syncthreads();

  // 1. every chunk of this workgroup: per-model totals of its 256 trajectories, published at once.  The counts of the
  // workgroup's first chunk (its only one unless there are more chunks than workgroups) stay in registers for step 2.
  TrajCounts<KM> first;
  for (int c = blockIdx.x; c < A.n_chunks; c += gridDim.x) {
    TrajCounts<KM> tc;
    traj_counts(A, s_phi, c * kPlanThreads + tid, tc);
    if (c == static_cast<int>(blockIdx.x)) first = tc;
    for (int k = 0; k < K; ++k) {
      const int64_t v[kCnt] = {pick(tc.cnt, k), pick(tc.tok, k), static_cast<int64_t>((tc.seen >> k) & 1u)};
#pragma unroll
      for (int j = 0; j < kCnt; ++j) {
        const int64_t total = block_sum<int64_t>(v[j], smem);
        if (tid == 0)
          __hip_atomic_store(A.plan_part + static_cast<size_t>(c) * kPlanWords + k * kCnt + j,
                             kMark | static_cast<unsigned long long>(total), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }

  // housekeeping that waits for nobody: the token kernel's counts start at zero; with no tokens or no turns it does not run
  {
    const int64_t gtid = static_cast<int64_t>(blockIdx.x) * kPlanThreads + tid, gsize = static_cast<int64_t>(gridDim.x) * kPlanThreads;
    for (int64_t i = gtid; i < A.n_count; i += gsize) A.tok_count[i] = 0ull;
    if (gtid <= K) A.model_rowsel_off[gtid] = 0;
  }

  // 2. every chunk again: where its trajectories' turns go
  for (int c = blockIdx.x; c < A.n_chunks; c += gridDim.x) {
    // totals over all chunks and over the chunks before this one, for every (model, counter): thread t takes the
    // chunks t, t + 256, ..., all words of a chunk in flight together; a word is taken when its ready mark is set
    if (tid < 2 * kPlanWords) (&s_res[0][0])[tid] = 0;
    __syncthreads();
    {
      constexpr int kW = KM * kCnt;
      long long all[kW], before[kW];
#pragma unroll
      for (int j = 0; j < kW; ++j) { all[j] = 0; before[j] = 0; }
      for (int cc = tid; cc < A.n_chunks; cc += kPlanThreads) {
        unsigned long long* const src = A.plan_part + static_cast<size_t>(cc) * kPlanWords;
        unsigned long long w[kW];
#pragma unroll
        for (int j = 0; j < kW; ++j) w[j] = j < K * kCnt ? __hip_atomic_load(src + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : kMark;
#pragma unroll
        for (int j = 0; j < kW; ++j) {
          while (!(w[j] & kMark)) {
            __builtin_amdgcn_s_sleep(2);
            w[j] = __hip_atomic_load(src + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
          const long long v = static_cast<long long>(w[j] & ~kMark);
          all[j] += v;
          before[j] += cc < c ? v : 0;
        }
      }
#pragma unroll
      for (int j = 0; j < kW; ++j) {
        const long long ta = wave_sum(all[j]), tb = wave_sum(before[j]);
        if ((tid & (kWave - 1)) == 0) {
          atomicAdd(reinterpret_cast<unsigned long long*>(&s_res[0][j]), static_cast<unsigned long long>(ta));
          atomicAdd(reinterpret_cast<unsigned long long*>(&s_res[1][j]), static_cast<unsigned long long>(tb));
        }
      }
    }
    __syncthreads();
    // first slot, token offset and run of every stream: streams lie one after the other
    int64_t slot_at[KM], tok_at[KM], run_at[KM];
    {
      int64_t bs = 0, bt = 0, br = 0;
#pragma unroll
      for (int k = 0; k < KM; ++k) {
        slot_at[k] = bs; tok_at[k] = bt; run_at[k] = br;
        if (k < K) { bs += s_res[0][k * kCnt + 0]; bt += s_res[0][k * kCnt + 1]; br += s_res[0][k * kCnt + 2]; }
      }
      if (c == 0 && tid == 0) {
        for (int k = 0; k <= K; ++k) {
          A.model_turn_off[k] = static_cast<int32_t>(k < K ? pick(slot_at, k) : bs);
          A.model_tok_off[k] = k < K ? pick(tok_at, k) : bt;
          A.model_trajrun_off[k] = static_cast<int32_t>(k < K ? pick(run_at, k) : br);
        }
        A.turn_seg_off[A.n_turns] = A.n_tokens;
      }
      // entries of traj_seg_off past the runs read n_tokens
      const int64_t gtid = static_cast<int64_t>(c) * kPlanThreads + tid, gsize = static_cast<int64_t>(A.n_chunks) * kPlanThreads;
      for (int64_t i = br + gtid; i <= A.n_turns; i += gsize) A.traj_seg_off[i] = A.n_tokens;
#pragma unroll
      for (int k = 0; k < KM; ++k)
        if (k < K) { slot_at[k] += s_res[1][k * kCnt + 0]; tok_at[k] += s_res[1][k * kCnt + 1]; run_at[k] += s_res[1][k * kCnt + 2]; }
    }
    // ... plus what the trajectories before this thread's one inside the chunk hold
    const int b = c * kPlanThreads + tid;
    {
      TrajCounts<KM> tc;
      if (c == static_cast<int>(blockIdx.x)) tc = first;
      else traj_counts(A, s_phi, b, tc);
      for (int k = 0; k < K; ++k) {
        int64_t total;
        const int64_t e0 = block_excl_scan<int64_t>(pick(tc.cnt, k), smem, &total);
        const int64_t e1 = block_excl_scan<int64_t>(pick(tc.tok, k), smem, &total);
        const int64_t e2 = block_excl_scan<int64_t>(static_cast<int64_t>((tc.seen >> k) & 1u), smem, &total);
        bump(slot_at, k, e0);
        bump(tok_at, k, e1);
        bump(run_at, k, e2);
      }
    }
    if (b < A.n_traj) {
      const int t0 = A.traj_turn_off[b], t1 = A.traj_turn_off[b + 1];
      const float rj = A.traj_reward ? A.traj_reward[b] : 0.0f;
      // One walk over the trajectory's turns: slots, offsets, runs, composed rewards, the first segment of every token
      // block, the record of every segment.  What a segment's last token says about its end - bit 1: last token of its
      // turn; bit 2: also the last token of the trajectory's run (no later turn of the trajectory with tokens in this
      // stream); bits 3-7: else the number of steps to the run's next turn with tokens (31 = more than 30: look it
      // up) - is known only when that next turn comes by: the record is written as a run's end and its flags are
      // written again then.
      uint32_t seen = 0;
      int last_slot[KM], last_step[KM];   // the model's latest turn with tokens in this trajectory
#pragma unroll
      for (int k = 0; k < KM; ++k) { last_slot[k] = -1; last_step[k] = 0; }
      int64_t g0 = A.turn_tok_off[t0];
      for (int u = t0; u < t1; ++u) {
        const int v = A.turn_role[u];
        const int m = s_phi[v];
        const int64_t g1 = A.turn_tok_off[u + 1], len = g1 - g0;
        const int64_t slot = pick(slot_at, m), off = pick(tok_at, m);
        const int step = u - t0 + 1;
        bump(slot_at, m, int64_t{1});
        bump(tok_at, m, len);
        A.seg_turn[slot] = u;
        A.turn_seg_off[slot] = off;
        if (!((seen >> m) & 1u)) {                   // the trajectory's one run in stream m starts here
          A.traj_seg_off[pick(run_at, m)] = off;
          seen |= 1u << m;
        }
        const float rr = A.role_reward ? A.role_reward[static_cast<size_t>(b) * A.n_roles + v] : 0.0f;
        const float rt = A.turn_reward ? A.turn_reward[u] : 0.0f;
        const float wr = A.w_role ? A.w_role[v] : 1.0f;
        const float wt = A.w_turn ? A.w_turn[v] : 1.0f;
        const float wj = A.w_traj ? A.w_traj[v] : 1.0f;
        // (node + turn) + traj with every product and sum rounded on its own: contraction into fused
        // multiply-adds is switched off for this expression so that the result is reproducible bit for bit
        float rho;
        {
#pragma clang fp contract(off)
          const float pr = wr * rr, pt = wt * rt, pj = wj * rj;
          const float s1 = pr + pt;
          rho = s1 + pj;
        }
        A.turn_scalar[u] = rho;
        A.turn_step[u] = step;
        for (int64_t blk = (off + kTokBlock - 1) / kTokBlock; blk * kTokBlock < off + len; ++blk) A.blk_first[blk] = static_cast<int32_t>(slot);
        SegMeta M;
        M.src = g0;
        M.turn = u;
        M.role = v;
        M.rho = rho;
        M.end_flags = 2 | 4;
        M.pad = 0;
        A.seg_meta[slot] = M;
        if (len > 0) {
          const int prev = pick(last_slot, m);
          if (prev >= 0) {
            const int ds = step - pick(last_step, m);
            A.seg_meta[prev].end_flags = 2 | ((ds < 31 ? ds : 31) << 3);
          }
#pragma unroll
          for (int k = 0; k < KM; ++k) {
            last_slot[k] = m == k ? static_cast<int>(slot) : last_slot[k];
            last_step[k] = m == k ? step : last_step[k];
          }
        }
        g0 = g1;
      }
    }
    __syncthreads();                                 // s_res is the next chunk's
  }
}

// ------------------------------------------------------------------ the tokens: everything per token
// Per token in model-local order: source index, turn, role, mask, flags, placed reward.  A block of 4096 tokens keeps
// the offsets and records of the segments that hold its tokens in LDS (up to kSegWin of them; a block of more and
// therefore very short segments takes a plain per-token path).  What a block cannot know from its own tokens is
// whether its last segment, if it goes on past the block, has another scored token further on, which decides if the
// segment's last scored token so far carries the reward: one wavefront reads ahead in the mask until it finds one or
// the segment ends.  The block also leaves its number of scored tokens for the compaction kernel, and adds it to the
// total of its group of blocks (about the square root of the number of blocks to a group).
constexpr int kSegWin = 256;
constexpr int kCompact = kTokBlock / kTokThreads;   // consecutive tokens of one thread when the scored positions are compacted
static_assert(kCompact == 16, "one 16-byte LDS read per thread");

struct TokArgs {
  int64_t n_tokens;
  int n_turns, n_models, place_mode, grp_shift;
  const int64_t* turn_seg_off;
  const SegMeta* seg_meta;
  const int32_t* blk_first;
  const uint8_t* mask_global;
  unsigned long long* blk_count;   // [blocks] scored tokens of the block
  unsigned long long* grp_count;   // [groups of 2^grp_shift blocks] scored tokens of the group, zero at the start
  int64_t* perm;
  int32_t* tok_turn;
  int32_t* tok_role;
  uint8_t* tok_mask;
  uint8_t* tok_flags;
  float* tok_reward;
};

// every non-zero byte becomes 1: (b | 0x80) - 1 keeps bit 7 exactly when b > 0, or-ed with b's own bit 7
__device__ __forceinline__ uint32_t bytes_to_01(uint32_t m4) {
  return ((((m4 | 0x80808080u) - 0x01010101u) | m4) >> 7) & 0x01010101u;
}
// mask bytes of four consecutive global tokens as one word (one load when the address allows it)
__device__ __forceinline__ uint32_t load_mask4(const uint8_t* __restrict__ mask, int64_t g0, bool base_aligned) {
  if (base_aligned && (g0 & 3) == 0) return *reinterpret_cast<const uint32_t*>(mask + g0);
  return static_cast<uint32_t>(mask[g0]) | (static_cast<uint32_t>(mask[g0 + 1]) << 8) |
         (static_cast<uint32_t>(mask[g0 + 2]) << 16) | (static_cast<uint32_t>(mask[g0 + 3]) << 24);
}
// One wavefront: does segment s, which goes on past position `from`, hold a scored token at or after it?
__device__ __forceinline__ bool scored_token_ahead(const TokArgs& A, int s, int64_t from) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t seg_e = A.turn_seg_off[s + 1];
  const int64_t g = A.seg_meta[s].src + (from - A.turn_seg_off[s]), n = seg_e - from;
  bool found = false;
  for (int64_t i0 = 0; i0 < n && !found; i0 += 8 * kWave) {   // eight bytes per lane, all in flight together
    uint32_t any = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int64_t i = i0 + lane * 8 + k;
      any |= i < n ? A.mask_global[g + i] : 0u;
    }
    found = __any(any != 0);
  }
  return found;
}

// The plain path of a block with more than kSegWin segments: one token at a time, the segment found by a search in
// global memory.  First the masks (into s_mk) ...
__device__ __forceinline__ void many_segments_masks(const TokArgs& A, int64_t blk0, int ntok, int s_first, int s_last, uint8_t* s_mk) {
  for (int pl = threadIdx.x; pl < ntok; pl += kTokThreads) {
    const int64_t p = blk0 + pl;
    const int s = s_first + last_le(A.turn_seg_off + s_first, s_last - s_first, p);
    s_mk[pl] = A.mask_global[A.seg_meta[s].src + (p - A.turn_seg_off[s])] ? 1 : 0;
  }
}
// ... then the outputs.  A scored token carries the reward of its segment if no scored token follows it there: the
// gaps between scored tokens are disjoint, so all these searches together read the block's masks once.
__device__ __forceinline__ void many_segments_outputs(const TokArgs& A, int64_t blk0, int ntok, int s_first, int s_last, const uint8_t* s_mk,
                                                   bool ahead) {
  for (int pl = threadIdx.x; pl < ntok; pl += kTokThreads) {
    const int64_t p = blk0 + pl;
    const int s = s_first + last_le(A.turn_seg_off + s_first, s_last - s_first, p);
    const SegMeta M = A.seg_meta[s];
    const int64_t seg_a = A.turn_seg_off[s], seg_e = A.turn_seg_off[s + 1];
    const uint8_t m = s_mk[pl];
    float rw = 0.f;
    if (m) {
      bool carries = A.place_mode == UMAS_PLACE_ALL;
      if (!carries) {
        const int stop = seg_e - blk0 < ntok ? static_cast<int>(seg_e - blk0) : ntok;
        int q = pl + 1;
        while (q < stop && !s_mk[q]) ++q;
        carries = q == stop && (seg_e - blk0 <= ntok || !ahead);
      }
      rw = carries ? M.rho : 0.f;
    }
    A.perm[p] = M.src + (p - seg_a);
    A.tok_turn[p] = M.turn;
    A.tok_role[p] = M.role;
    A.tok_mask[p] = m;
    A.tok_flags[p] = static_cast<uint8_t>(m | (p == seg_e - 1 ? M.end_flags : 0));
    A.tok_reward[p] = rw;
  }
}

__global__ void __launch_bounds__(kTokThreads)
k_tokens(TokArgs A) {
  __shared__ int64_t smem[32];
  __shared__ int64_t s_off[kSegWin + 1];
  __shared__ int32_t s_loc[kSegWin + 1];            // the same offsets relative to the block's first token, clamped
  __shared__ SegMeta s_meta[kSegWin];
  __shared__ int32_t s_lastv[kSegWin];              // block-relative position of the segment's last scored token in this block, -1
  __shared__ __attribute__((aligned(16))) uint8_t s_mk[kTokBlock];   // the block's masks, 0 or 1 (plain path)
  __shared__ int s_ahead;
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int64_t blk0 = static_cast<int64_t>(blockIdx.x) * kTokBlock;
  const int64_t blk_end = blk0 + kTokBlock < A.n_tokens ? blk0 + kTokBlock : A.n_tokens;
  const int ntok = static_cast<int>(blk_end - blk0);
  const int s_first = A.blk_first[blockIdx.x];
  // segments s_first .. s_last hold the block's tokens (s_last = the segment of the next block's first token)
  const int s_last = blk_end < A.n_tokens ? A.blk_first[blockIdx.x + 1] : A.n_turns - 1;
  const int n_seg = s_last - s_first + 1;
  const bool windowed = n_seg <= kSegWin;
  const bool mask_aligned = (reinterpret_cast<uintptr_t>(A.mask_global) & 3) == 0;
  if (tid == 0) s_ahead = 0;
  *reinterpret_cast<uint4*>(s_mk + tid * kCompact) = make_uint4(0u, 0u, 0u, 0u);
  if (windowed) {
    for (int i = tid; i <= n_seg; i += kTokThreads) {
      const int64_t off = A.turn_seg_off[s_first + i];
      const int64_t rel = off - blk0;
      s_off[i] = off;
      s_loc[i] = static_cast<int32_t>(rel < -(1 << 30) ? -(1 << 30) : rel > (1 << 30) ? (1 << 30) : rel);
      if (i < n_seg) { s_meta[i] = A.seg_meta[s_first + i]; s_lastv[i] = -1; }
    }
  }
  __syncthreads();

  // ---- masks: into registers (windowed path) and LDS, the last scored token of every segment
  uint32_t mk_r[kTokRounds];                        // 0/1 bytes of this thread's four tokens in each round
  int lo_r[kTokRounds];                             // their first token's segment in the window; bit 30: all four lie in it
#pragma unroll
  for (int rd = 0; rd < kTokRounds; ++rd) { mk_r[rd] = 0; lo_r[rd] = 0; }
  if (windowed) {
    uint32_t m4_r[kTokRounds];
#pragma unroll
    for (int rd = 0; rd < kTokRounds; ++rd) {       // every load of the block goes out before anything waits for one
      const int pl0 = rd * kTokRound + tid * kTokPerThread;
      m4_r[rd] = 0;
      if (pl0 >= ntok) continue;
      int lo = 0, hi = n_seg;                       // largest j with s_loc[j] <= pl0: the segment that holds the token
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (s_loc[mid] <= pl0) lo = mid; else hi = mid - 1;
      }
      const bool fast = pl0 + kTokPerThread <= s_loc[lo + 1];
      lo_r[rd] = lo | (fast ? 1 << 30 : 0);
      if (fast) m4_r[rd] = load_mask4(A.mask_global, s_meta[lo].src + (blk0 + pl0 - s_off[lo]), mask_aligned);
    }
#pragma unroll
    for (int rd = 0; rd < kTokRounds; ++rd) {
      const int pl0 = rd * kTokRound + tid * kTokPerThread;
      const bool in = pl0 < ntok, fast = (lo_r[rd] >> 30) != 0;
      const int lo = lo_r[rd] & ((1 << 30) - 1);
      uint32_t mk4 = 0;
      int cand = -1;                                // this thread's last scored token of segment lo
      if (fast) {
        mk4 = bytes_to_01(m4_r[rd]);
        cand = mk4 ? pl0 + (31 - __clz(mk4)) / 8 : -1;
      }
      // when the whole wavefront sits in one segment, one update of the segment's last scored token does
      const int lo0 = __shfl(lo, 0, kWave);
      if (__all(fast && lo == lo0)) {
        const int best = wave_max(cand);
        if (lane == 0 && best >= 0) atomicMax(&s_lastv[lo], best);
      } else if (cand >= 0) {
        atomicMax(&s_lastv[lo], cand);
      }
      if (in && !fast) {                            // a segment boundary or the stream's end inside the four tokens
        int s = lo;
        for (int k = 0; k < kTokPerThread; ++k) {
          const int pl = pl0 + k;
          if (pl >= ntok) break;
          while (s_loc[s + 1] <= pl) ++s;           // also steps over empty segments
          const uint32_t m = A.mask_global[s_meta[s].src + (blk0 + pl - s_off[s])] ? 1u : 0u;
          mk4 |= m << (8 * k);
          if (m) atomicMax(&s_lastv[s], pl);
        }
      }
      mk_r[rd] = mk4;
    }
  } else {
    many_segments_masks(A, blk0, ntok, s_first, s_last, s_mk);
  }
  // the block's last segment, if it goes on past the block: is there a scored token further on?
  if (wave == 1 && A.place_mode == UMAS_PLACE_LAST && A.turn_seg_off[s_last + 1] > blk_end) {
    const bool found = scored_token_ahead(A, s_last, blk_end);
    if (lane == 0) s_ahead = found ? 1 : 0;
  }
  __syncthreads();
  const bool ahead = s_ahead != 0;

  // ---- the block's count of scored tokens, for the compaction kernel: its own word and its group's total
  {
    int32_t c = 0;
    if (windowed) {
#pragma unroll
      for (int rd = 0; rd < kTokRounds; ++rd) c += __popc(mk_r[rd]);
    } else {
      const uint4 w = *reinterpret_cast<const uint4*>(s_mk + tid * kCompact);
      c = __popc(w.x) + __popc(w.y) + __popc(w.z) + __popc(w.w);
    }
    const int32_t total = block_sum<int32_t>(c, reinterpret_cast<int32_t*>(smem));
    if (tid == 0) {
      A.blk_count[blockIdx.x] = static_cast<unsigned long long>(total);
      (void)__hip_atomic_fetch_add(A.grp_count + (blockIdx.x >> A.grp_shift), static_cast<unsigned long long>(total), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
    }
  }

  // ---- outputs per token
  if (windowed) {
#pragma unroll
    for (int rd = 0; rd < kTokRounds; ++rd) {
      const int pl0 = rd * kTokRound + tid * kTokPerThread;
      const int64_t p0 = blk0 + pl0;
      if (pl0 >= ntok) continue;
      int s = lo_r[rd] & ((1 << 30) - 1);
      const uint32_t mk4 = mk_r[rd];
      if ((lo_r[rd] >> 30) != 0) {                  // four tokens of one segment: no per-token bookkeeping
        const SegMeta M = s_meta[s];
        const int64_t g0 = M.src + (p0 - s_off[s]);
        uint32_t fg4 = mk4;
        if (pl0 + kTokPerThread == s_loc[s + 1]) fg4 |= static_cast<uint32_t>(M.end_flags) << 24;
        // the segment's last scored token carries the reward, unless the segment goes on past the block and has another
        const int lastv = s_loc[s + 1] <= kTokBlock || !ahead ? s_lastv[s] : -1;
        float rw[kTokPerThread];
#pragma unroll
        for (int k = 0; k < kTokPerThread; ++k)
          rw[k] = ((mk4 >> (8 * k)) & 1u) && (A.place_mode == UMAS_PLACE_ALL || pl0 + k == lastv) ? M.rho : 0.f;
        *reinterpret_cast<longlong2*>(A.perm + p0) = make_longlong2(g0, g0 + 1);
        *reinterpret_cast<longlong2*>(A.perm + p0 + 2) = make_longlong2(g0 + 2, g0 + 3);
        *reinterpret_cast<int4*>(A.tok_turn + p0) = make_int4(M.turn, M.turn, M.turn, M.turn);
        *reinterpret_cast<int4*>(A.tok_role + p0) = make_int4(M.role, M.role, M.role, M.role);
        *reinterpret_cast<uint32_t*>(A.tok_mask + p0) = mk4;
        *reinterpret_cast<uint32_t*>(A.tok_flags + p0) = fg4;
        *reinterpret_cast<float4*>(A.tok_reward + p0) = make_float4(rw[0], rw[1], rw[2], rw[3]);
        continue;
      }
      for (int k = 0; k < kTokPerThread; ++k) {
        const int pl = pl0 + k;
        if (pl >= ntok) break;
        while (s_loc[s + 1] <= pl) ++s;
        const SegMeta M = s_meta[s];
        const uint32_t m = (mk4 >> (8 * k)) & 1u;
        const bool seg_done = s_loc[s + 1] <= kTokBlock || !ahead;
        A.perm[p0 + k] = M.src + (p0 + k - s_off[s]);
        A.tok_turn[p0 + k] = M.turn;
        A.tok_role[p0 + k] = M.role;
        A.tok_mask[p0 + k] = static_cast<uint8_t>(m);
        A.tok_flags[p0 + k] = static_cast<uint8_t>(m | (pl + 1 == s_loc[s + 1] ? M.end_flags : 0));
        A.tok_reward[p0 + k] = m && (A.place_mode == UMAS_PLACE_ALL || (seg_done && pl == s_lastv[s])) ? M.rho : 0.f;
      }
    }
  } else {
    many_segments_outputs(A, blk0, ntok, s_first, s_last, s_mk, ahead);
  }

}

// The compacted list of scored positions, per stream and stream-relative, from the masks in model-local order.  A
// block of 4096 tokens finds the number of scored tokens in front of it as the totals of the groups of blocks before
// its group plus the counts of the blocks before it in its group, all written by the token kernel.
struct SelArgs {
  int64_t n_tokens;
  int n_models, grp_shift;
  const uint8_t* tok_mask;
  const int64_t* model_tok_off;
  const unsigned long long* blk_count;
  const unsigned long long* grp_count;
  int32_t* rowsel;
  int64_t* model_rowsel_off;
};

constexpr int kSelMul = 2;                          // blocks of the token kernel to one block of the compaction kernel
constexpr int kSelBlock = kTokBlock * kSelMul;
constexpr int kSelPerThread = kSelBlock / kTokThreads;
constexpr int kSelWords = kSelPerThread / 4;

__global__ void __launch_bounds__(kTokThreads)
k_rowsel(SelArgs A) {
  __shared__ int64_t smem[32];
  __shared__ __attribute__((aligned(8))) uint16_t s_out[kSelBlock + 4];   // the block's scored positions, block-relative, compacted
  __shared__ int64_t moff[UMAS_MAX_MODELS + 1];
  __shared__ int32_t s_mro[UMAS_MAX_MODELS + 1];    // scored tokens of the block in front of a stream that starts in it, -1
  const int tid = threadIdx.x;
  const int64_t blk0 = static_cast<int64_t>(blockIdx.x) * kSelBlock;
  const int64_t blk_end = blk0 + kSelBlock < A.n_tokens ? blk0 + kSelBlock : A.n_tokens;
  if (tid <= A.n_models) { moff[tid] = A.model_tok_off[tid]; s_mro[tid] = -1; }
  // what lies in front of the block
  int64_t part = 0;
  {
    const int64_t first = static_cast<int64_t>(blockIdx.x) * kSelMul;   // in blocks of the token kernel
    const int64_t grp = first >> A.grp_shift;
    for (int64_t g = tid; g < grp; g += kTokThreads) part += static_cast<int64_t>(A.grp_count[g]);
    for (int64_t k = (grp << A.grp_shift) + tid; k < first; k += kTokThreads) part += static_cast<int64_t>(A.blk_count[k]);
  }
  const int64_t p0 = blk0 + tid * kSelPerThread;
  uint32_t w4[kSelWords];
#pragma unroll
  for (int k = 0; k < kSelWords; ++k) w4[k] = 0u;
  if (p0 + kSelPerThread <= A.n_tokens) {
#pragma unroll
    for (int q = 0; q < kSelWords / 4; ++q) {
      const uint4 w = *reinterpret_cast<const uint4*>(A.tok_mask + p0 + 16 * q);
      w4[4 * q] = w.x; w4[4 * q + 1] = w.y; w4[4 * q + 2] = w.z; w4[4 * q + 3] = w.w;
    }
  } else {
    for (int k = 0; k < kSelPerThread; ++k)
      if (p0 + k < A.n_tokens) w4[k >> 2] |= static_cast<uint32_t>(A.tok_mask[p0 + k]) << (8 * (k & 3));
  }
  const int64_t prefix = block_sum<int64_t>(part, smem);
  int32_t c = 0;                                    // mask bytes are 0 or 1
#pragma unroll
  for (int k = 0; k < kSelWords; ++k) c += __popc(w4[k]);
  int32_t block_count;
  int o = block_excl_scan<int32_t>(c, reinterpret_cast<int32_t*>(smem), &block_count);
  // The entries leave single up to the first 16-byte boundary of rowsel, four to a store from there; they are staged
  // `pad` places further on so that every such group of four starts at an 8-byte boundary of s_out.
  int32_t* const dst = A.rowsel + prefix;
  const int to_boundary = static_cast<int>((4 - ((reinterpret_cast<uintptr_t>(dst) >> 2) & 3)) & 3);
  const int pad = (4 - to_boundary) & 3;
  // a stream may start inside the block: the scored tokens in front of its first token give its place in rowsel
  const int e = o;
#pragma unroll
  for (int k = 0; k < kSelPerThread; ++k)
    if ((w4[k >> 2] >> (8 * (k & 3))) & 1u) s_out[pad + o++] = static_cast<uint16_t>(tid * kSelPerThread + k);
  for (int j = 0; j <= A.n_models; ++j) {
    const int64_t q = moff[j] - p0;
    if (q >= 0 && q < kSelPerThread && moff[j] < A.n_tokens) {
      int before = 0;
#pragma unroll
      for (int k = 0; k < kSelPerThread; ++k) before += k < q ? static_cast<int>((w4[k >> 2] >> (8 * (k & 3))) & 1u) : 0;
      s_mro[j] = e + before;
    }
  }
  __syncthreads();
  for (int j = tid; j <= A.n_models; j += kTokThreads)
    if (s_mro[j] >= 0) A.model_rowsel_off[j] = prefix + s_mro[j];
  int m0 = 0;                                        // the stream of the block's first token
  while (m0 < A.n_models && moff[m0 + 1] <= blk0) ++m0;
  auto entry = [&](int i) -> int32_t {               // compacted entry i of the block, stream-relative
    const int64_t p = blk0 + s_out[pad + i];
    int m = m0;
    while (m < A.n_models && moff[m + 1] <= p) ++m;
    return static_cast<int32_t>(p - moff[m]);
  };
  const bool one_stream = moff[m0 + 1] >= blk_end;   // the usual case: every entry is relative to the same start
  const int32_t rel0 = static_cast<int32_t>(blk0 - moff[m0]);
  const int head = to_boundary < block_count ? to_boundary : block_count;
  const int n_vec = (block_count - head) / 4;
  if (tid < head) dst[tid] = entry(tid);
  for (int v = tid; v < n_vec; v += kTokThreads) {
    const int i = head + 4 * v;
    if (one_stream) {
      const uint2 q = *reinterpret_cast<const uint2*>(s_out + pad + i);
      *reinterpret_cast<int4*>(dst + i) = make_int4(rel0 + static_cast<int32_t>(q.x & 0xffffu), rel0 + static_cast<int32_t>(q.x >> 16),
                                                   rel0 + static_cast<int32_t>(q.y & 0xffffu), rel0 + static_cast<int32_t>(q.y >> 16));
    } else {
      *reinterpret_cast<int4*>(dst + i) = make_int4(entry(i), entry(i + 1), entry(i + 2), entry(i + 3));
    }
  }
  {
    const int i = head + 4 * n_vec + tid;
    if (i < block_count) dst[i] = entry(i);
  }
  if (blk_end == A.n_tokens && tid == 0)             // streams that start at the very end hold nothing
    for (int j = 0; j <= A.n_models; ++j)
      if (moff[j] >= A.n_tokens) A.model_rowsel_off[j] = prefix + block_count;
}

// ------------------------------------------------------------------ host side
umas_status validate(const umas_graph* g, const umas_rewards* r, const umas_streams* o) {
  UMAS_REQUIRE(g && r && o, UMAS_EINVAL, "graph, rewards and out must not be NULL");
  UMAS_REQUIRE(g->n_roles >= 1 && g->n_roles <= UMAS_MAX_ROLES, UMAS_ESHAPE, "n_roles=%d outside [1,%d]",
               g->n_roles, UMAS_MAX_ROLES);
  UMAS_REQUIRE(g->n_models >= 1 && g->n_models <= UMAS_MAX_MODELS, UMAS_ESHAPE, "n_models=%d outside [1,%d]",
               g->n_models, UMAS_MAX_MODELS);
  UMAS_REQUIRE(g->n_traj >= 0 && g->n_turns >= 0 && g->n_tokens >= 0, UMAS_EINVAL, "negative size");
  UMAS_REQUIRE(g->role_to_model && g->traj_turn_off && g->turn_tok_off && (g->turn_role || g->n_turns == 0),
               UMAS_EINVAL, "role_to_model, traj_turn_off, turn_role, turn_tok_off must not be NULL");
  for (int v = 0; v < g->n_roles; ++v)
    UMAS_REQUIRE(g->role_to_model[v] >= 0 && g->role_to_model[v] < g->n_models, UMAS_EINVAL,
                 "role_to_model[%d]=%d is not a model in [0,%d)", v, g->role_to_model[v], g->n_models);
  UMAS_REQUIRE(g->traj_turn_off[0] == 0 && g->traj_turn_off[g->n_traj] == g->n_turns, UMAS_EINVAL,
               "traj_turn_off must run from 0 to n_turns");
  for (int b = 0; b < g->n_traj; ++b)
    UMAS_REQUIRE(g->traj_turn_off[b] <= g->traj_turn_off[b + 1], UMAS_EINVAL, "traj_turn_off decreases at %d", b);
  UMAS_REQUIRE(g->turn_tok_off[0] == 0 && g->turn_tok_off[g->n_turns] == g->n_tokens, UMAS_EINVAL,
               "turn_tok_off must run from 0 to n_tokens");
  int64_t stream_tokens[UMAS_MAX_MODELS] = {};
  for (int u = 0; u < g->n_turns; ++u) {
    UMAS_REQUIRE(g->turn_tok_off[u] <= g->turn_tok_off[u + 1], UMAS_EINVAL, "turn_tok_off decreases at %d", u);
    UMAS_REQUIRE(g->turn_role[u] >= 0 && g->turn_role[u] < g->n_roles, UMAS_EINVAL,
                 "turn_role[%d]=%d is not a role in [0,%d)", u, g->turn_role[u], g->n_roles);
    stream_tokens[g->role_to_model[g->turn_role[u]]] += g->turn_tok_off[u + 1] - g->turn_tok_off[u];
  }
  // rowsel holds positions relative to the stream's start as int32
  for (int m = 0; m < g->n_models; ++m)
    UMAS_REQUIRE(stream_tokens[m] <= INT32_MAX, UMAS_ESHAPE, "the stream of model %d would hold %lld tokens, more than 2^31 - 1", m,
                 static_cast<long long>(stream_tokens[m]));
  if (g->turn_pred_off) {
    UMAS_REQUIRE(g->turn_pred || g->turn_pred_off[g->n_turns] == 0, UMAS_EINVAL, "turn_pred is NULL");
    UMAS_REQUIRE(g->turn_pred_off[0] == 0, UMAS_EINVAL, "turn_pred_off must start at 0");
    int b = 0;
    for (int u = 0; u < g->n_turns; ++u) {
      while (g->traj_turn_off[b + 1] <= u) ++b;
      UMAS_REQUIRE(g->turn_pred_off[u] <= g->turn_pred_off[u + 1], UMAS_EINVAL, "turn_pred_off decreases at %d", u);
      for (int e = g->turn_pred_off[u]; e < g->turn_pred_off[u + 1]; ++e)
        UMAS_REQUIRE(g->turn_pred[e] >= g->traj_turn_off[b] && g->turn_pred[e] < u, UMAS_EINVAL,
                     "predecessor %d of turn %d is not an earlier turn of the same trajectory", g->turn_pred[e], u);
    }
  }
  if (g->traj_group)
    for (int b = 0; b < g->n_traj; ++b)
      UMAS_REQUIRE(g->traj_group[b] >= 0, UMAS_EINVAL, "traj_group[%d] is negative", b);
  UMAS_REQUIRE(r->place_mode == UMAS_PLACE_LAST || r->place_mode == UMAS_PLACE_ALL, UMAS_EINVAL,
               "place_mode=%d is neither LAST nor ALL", r->place_mode);
  UMAS_REQUIRE(r->norm_eps > 0.0f, UMAS_EINVAL, "norm_eps must be positive");
  UMAS_REQUIRE(o->model_tok_off && o->perm && o->tok_turn && o->tok_role && o->tok_mask && o->tok_reward &&
                   o->turn_seg_off && o->seg_turn && o->model_turn_off && o->traj_seg_off &&
                   o->model_trajrun_off && o->rowsel && o->model_rowsel_off && o->turn_scalar && o->turn_step &&
                   o->tok_flags,
               UMAS_EINVAL, "every pointer of the output streams must be set");
  // the token kernel writes four tokens of every per-token array in one store
  auto aligned16 = [](const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
  UMAS_REQUIRE(aligned16(o->perm) && aligned16(o->tok_turn) && aligned16(o->tok_role) && aligned16(o->tok_mask) &&
                   aligned16(o->tok_flags) && aligned16(o->tok_reward),
               UMAS_EINVAL, "perm, tok_turn, tok_role, tok_mask, tok_flags and tok_reward must be 16-byte aligned");
  return UMAS_OK;
}


}  // namespace
}  // namespace umas

using namespace umas;

extern "C" size_t umas_assign_workspace_bytes(const umas_graph* g) {
  if (!g || g->n_roles < 0 || g->n_traj < 0 || g->n_turns < 0 || g->n_tokens < 0) return 0;
  Carver c(nullptr);
  RouteWs w;
  return carve(c, w, g->n_roles, g->n_traj, g->n_turns, g->n_tokens);
}

extern "C" umas_status umas_assign_token_rewards(const umas_graph* g, const umas_rewards* r,
                                                 const uint8_t* tok_mask_global, const umas_streams* o,
                                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  umas_status vs = validate(g, r, o);
  if (vs != UMAS_OK) return vs;
  UMAS_REQUIRE(tok_mask_global || g->n_tokens == 0, UMAS_EINVAL, "tok_mask_global is NULL");
  const size_t need = umas_assign_workspace_bytes(g);
  UMAS_REQUIRE(workspace && reinterpret_cast<uintptr_t>(workspace) % kAlign == 0 && workspace_bytes >= need,
               UMAS_EWORKSPACE, "workspace must be 256-byte aligned and hold %zu bytes (got %zu)", need,
               workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  const int R = g->n_roles, K = g->n_models, B = g->n_traj, U = g->n_turns;
  const int64_t N = g->n_tokens;
  Carver c(workspace);
  RouteWs w;
  carve(c, w, R, B, U, N);

  // members of each normalisation group, as a CSR over the groups that occur
  int n_groups = 0;
  std::vector<int32_t> goff, gmem;
  if (g->traj_group && r->traj_reward && B > 0) {
    gmem.resize(B);
    for (int b = 0; b < B; ++b) gmem[b] = b;
    std::stable_sort(gmem.begin(), gmem.end(),
                     [&](int32_t x, int32_t y) { return g->traj_group[x] < g->traj_group[y]; });
    goff.push_back(0);
    for (int i = 1; i < B; ++i)
      if (g->traj_group[gmem[i]] != g->traj_group[gmem[i - 1]]) goff.push_back(i);
    goff.push_back(B);
    n_groups = static_cast<int>(goff.size()) - 1;
  }

  // The thin arrays are the first arrays of the workspace, up to traj_norm: they are gathered at the same offsets in a
  // block of pinned host memory and go to the device in one asynchronous copy, together with the zeros that the plan
  // kernel's per-chunk totals start from.  The host arrays have been read when the call returns; the host does not
  // wait for the stream.
  char* const ws_base = static_cast<char*>(workspace);
  const size_t staged_bytes = static_cast<size_t>(reinterpret_cast<char*>(w.traj_norm) - ws_base);
  const int n_chunks = plan_chunks(B);
  ThinStage stage;
  vs = stage.begin(staged_bytes);
  if (vs != UMAS_OK) return vs;
  auto put = [&](const void* dst, const void* src, size_t bytes) {
    stage.put(static_cast<size_t>(static_cast<const char*>(dst) - ws_base), src, bytes);
  };
  put(w.role_to_model, g->role_to_model, sizeof(int32_t) * R);
  put(w.traj_turn_off, g->traj_turn_off, sizeof(int32_t) * (static_cast<size_t>(B) + 1));
  put(w.turn_role, g->turn_role, sizeof(int32_t) * U);
  put(w.turn_tok_off, g->turn_tok_off, sizeof(int64_t) * (static_cast<size_t>(U) + 1));
  put(w.role_reward, r->role_reward, sizeof(float) * static_cast<size_t>(B) * R);
  put(w.turn_reward, r->turn_reward, sizeof(float) * U);
  put(w.traj_reward, r->traj_reward, sizeof(float) * B);
  put(w.weights, r->w_role, sizeof(float) * R);
  put(w.weights + R, r->w_turn, sizeof(float) * R);
  put(w.weights + 2 * R, r->w_traj, sizeof(float) * R);
  if (n_groups > 0) {
    put(w.group_off, goff.data(), sizeof(int32_t) * goff.size());
    put(w.group_members, gmem.data(), sizeof(int32_t) * gmem.size());
  }
  stage.zero(static_cast<size_t>(reinterpret_cast<char*>(w.plan_part) - ws_base),
             sizeof(unsigned long long) * static_cast<size_t>(n_chunks) * kPlanWords);
  vs = stage.flush(workspace, staged_bytes, st);
  if (vs != UMAS_OK) return vs;
  prof_mark(st);

  const float* traj_r = r->traj_reward ? w.traj_reward : nullptr;
  if (n_groups > 0) {
    hipLaunchKernelGGL(k_group_norm, dim3(cdiv(n_groups, 4)), dim3(256), 0, st, w.traj_reward, w.group_off,
                       w.group_members, n_groups, r->norm_eps, w.traj_norm);
    UMAS_LAUNCHED("k_group_norm");
    traj_r = w.traj_norm;
  }
  const int64_t nbk = cdiv(N > 0 ? N : 1, kTokBlock);
  PlanArgs P;
  P.n_traj = B; P.n_turns = U; P.n_roles = R; P.n_models = K; P.n_chunks = n_chunks;
  const int gsh = group_shift(nbk);
  P.n_tokens = N; P.n_count = nbk + (nbk >> gsh) + 1;
  P.traj_turn_off = w.traj_turn_off; P.turn_role = w.turn_role; P.role_to_model = w.role_to_model;
  P.turn_tok_off = w.turn_tok_off;
  P.role_reward = r->role_reward ? w.role_reward : nullptr;
  P.turn_reward = r->turn_reward ? w.turn_reward : nullptr;
  P.traj_reward = traj_r;
  P.w_role = r->w_role ? w.weights : nullptr;
  P.w_turn = r->w_turn ? w.weights + R : nullptr;
  P.w_traj = r->w_traj ? w.weights + 2 * R : nullptr;
  P.plan_part = w.plan_part; P.seg_meta = w.seg_meta; P.blk_first = w.blk_first;
  P.tok_count = w.tok_count;
  P.model_tok_off = o->model_tok_off; P.model_turn_off = o->model_turn_off; P.model_trajrun_off = o->model_trajrun_off;
  P.model_rowsel_off = o->model_rowsel_off; P.turn_seg_off = o->turn_seg_off; P.seg_turn = o->seg_turn;
  P.traj_seg_off = o->traj_seg_off; P.turn_scalar = o->turn_scalar; P.turn_step = o->turn_step;
  // workgroups of the plan kernel wait for one another's totals: no more of them than the device holds at once
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    n_cu = 64;
  const dim3 plan_grid(std::min(n_chunks, (K <= 2 ? kPlanPerCu : 1) * n_cu));
  if (K <= 1) hipLaunchKernelGGL(k_turn_plan<1>, plan_grid, dim3(kPlanThreads), 0, st, P);
  else if (K <= 2) hipLaunchKernelGGL(k_turn_plan<2>, plan_grid, dim3(kPlanThreads), 0, st, P);
  else if (K <= 4) hipLaunchKernelGGL(k_turn_plan<4>, plan_grid, dim3(kPlanThreads), 0, st, P);
  else hipLaunchKernelGGL(k_turn_plan<UMAS_MAX_MODELS>, plan_grid, dim3(kPlanThreads), 0, st, P);
  UMAS_LAUNCHED("k_turn_plan");
  if (U > 0 && N > 0) {
    TokArgs T;
    T.n_tokens = N; T.n_turns = U; T.n_models = K; T.place_mode = r->place_mode; T.grp_shift = gsh;
    T.turn_seg_off = o->turn_seg_off; T.seg_meta = w.seg_meta; T.blk_first = w.blk_first; T.mask_global = tok_mask_global;
    T.blk_count = w.tok_count; T.grp_count = w.tok_count + nbk;
    T.perm = o->perm; T.tok_turn = o->tok_turn; T.tok_role = o->tok_role; T.tok_mask = o->tok_mask;
    T.tok_flags = o->tok_flags; T.tok_reward = o->tok_reward;
    hipLaunchKernelGGL(k_tokens, dim3(static_cast<unsigned>(nbk)), dim3(kTokThreads), 0, st, T);
    UMAS_LAUNCHED("k_tokens");
    SelArgs S;
    S.n_tokens = N; S.n_models = K; S.grp_shift = gsh;
    S.tok_mask = o->tok_mask; S.model_tok_off = o->model_tok_off; S.blk_count = w.tok_count; S.grp_count = w.tok_count + nbk;
    S.rowsel = o->rowsel; S.model_rowsel_off = o->model_rowsel_off;
    hipLaunchKernelGGL(k_rowsel, dim3(cdiv(N, kSelBlock)), dim3(kTokThreads), 0, st, S);
    UMAS_LAUNCHED("k_rowsel");
  }
  return UMAS_OK;
}
