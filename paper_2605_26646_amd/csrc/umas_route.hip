// Reward composition, group normalisation, routing through phi and reward placement.
//
// The thin graph arrives as host arrays (the controller's view: role ids, routing ids,
// reward metadata); it is validated on the host, staged to the device and every step after
// that runs in kernels: per-turn reward r_v = lam_node r_node + lam_turn r_turn + lam_traj
// r_traj (Section "Agent-Specific Reward Interface"), the stable partition of turns by
// phi(role) into model-local streams (Sections "Agent--LLM Mapping", "Model-Local Buffers")
// and the alignment of each turn's reward with its token sequence (paragraph "Batch
// construction").
#include <algorithm>
#include <vector>

#include "umas_common.h"

namespace umas {
namespace {

constexpr int kTurnBlock = 256;   // turns per block in the turn-level kernels
constexpr int kTokThreads = 256;
constexpr int kTokPerThread = 4;   // consecutive tokens of one thread in one round
constexpr int kTokRounds = 4;      // rounds of a block, kTokThreads * kTokPerThread tokens apart
constexpr int kTokRound = kTokThreads * kTokPerThread;
constexpr int kTokBlock = kTokRound * kTokRounds;
constexpr int kCntTokens = 4096;   // mask=1 tokens are counted per this many tokens (one compaction block)
constexpr int kCntRounds = kCntTokens / kTokRound;
static_assert(kTokBlock % kCntTokens == 0 && kCntTokens % kTokRound == 0, "a token block is a whole number of count groups");

// What the token kernel needs to know about one turn segment of a model-local stream.
struct __attribute__((aligned(16))) SegMeta {
  int64_t src;         // global index of the segment's first token
  int64_t last_valid;  // model-local position of its last mask=1 token, or -1
  int32_t turn;
  int32_t role;
  float rho;           // composed reward of the turn
  int32_t end_flags;   // flag bits of the segment's last token besides the mask bit
};
static_assert(sizeof(SegMeta) == 32, "two 16-byte loads");

struct RouteWs {
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
  float* traj_norm;     // [n_traj]
  int32_t* turn_traj;   // [n_turns]
  int32_t* turn_model;  // [n_turns]
  SegMeta* seg_meta;    // [n_turns] per segment slot
  int32_t* blk_first;   // [nblk_tok] segment that holds the first token of each token block
  int64_t* part;        // [2*K][nblk_turn] per-model (turn count, token count) per block, scanned in place
  int64_t* part_total;  // [2*K]
  int64_t* run_blk;     // [nblk_turn]
  int64_t* run_total;   // [1]
  int64_t* tok_blk;     // [nblk_tok]
  int64_t* tok_total;   // [1]
};

size_t carve(Carver& c, RouteWs& w, int n_roles, int n_traj, int n_turns, int64_t n_tokens) {
  const size_t nbt = cdiv(n_turns > 0 ? n_turns : 1, kTurnBlock);
  const size_t nbk = cdiv(n_tokens > 0 ? n_tokens : 1, kCntTokens);   // count groups (>= token blocks)
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
  w.traj_norm = c.take<float>(n_traj);
  w.turn_traj = c.take<int32_t>(n_turns);
  w.turn_model = c.take<int32_t>(n_turns);
  w.seg_meta = c.take<SegMeta>(n_turns);
  w.blk_first = c.take<int32_t>(nbk);
  w.part = c.take<int64_t>(2 * UMAS_MAX_MODELS * nbt);
  w.part_total = c.take<int64_t>(2 * UMAS_MAX_MODELS);
  w.run_blk = c.take<int64_t>(nbt);
  w.run_total = c.take<int64_t>(1);
  w.tok_blk = c.take<int64_t>(nbk);
  w.tok_total = c.take<int64_t>(1);
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

// Per turn: owning trajectory, step inside it, model phi(role), composed reward.
__global__ void k_turn_meta(int n_traj, int n_turns, int n_roles, const int32_t* __restrict__ traj_turn_off,
                            const int32_t* __restrict__ turn_role, const int32_t* __restrict__ role_to_model,
                            const float* __restrict__ role_reward, const float* __restrict__ turn_reward,
                            const float* __restrict__ traj_reward, const float* __restrict__ w_role,
                            const float* __restrict__ w_turn, const float* __restrict__ w_traj,
                            int32_t* __restrict__ turn_traj, int32_t* __restrict__ turn_model,
                            int32_t* __restrict__ turn_step, float* __restrict__ turn_scalar) {
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= n_turns) return;
  // last b with traj_turn_off[b] <= u, skipping empty trajectories that start at the same turn
  int b = last_le(traj_turn_off, n_traj, u);
  const int v = turn_role[u];
  turn_traj[u] = b;
  turn_step[u] = u - traj_turn_off[b] + 1;
  turn_model[u] = role_to_model[v];
  const float rr = role_reward ? role_reward[static_cast<size_t>(b) * n_roles + v] : 0.0f;
  const float rt = turn_reward ? turn_reward[u] : 0.0f;
  const float rj = traj_reward ? traj_reward[b] : 0.0f;
  const float wr = w_role ? w_role[v] : 1.0f;
  const float wt = w_turn ? w_turn[v] : 1.0f;
  const float wj = w_traj ? w_traj[v] : 1.0f;
  // (node + turn) + traj with every product and sum rounded on its own: contraction into fused
  // multiply-adds is switched off for this expression so that the result is reproducible bit for bit
  {
#pragma clang fp contract(off)
    const float pr = wr * rr, pt = wt * rt, pj = wj * rj;
    const float s1 = pr + pt;
    turn_scalar[u] = s1 + pj;
  }
}

// Per block of turns and per model: number of turns and of tokens routed to that model.
__global__ void k_part_reduce(int n_turns, int n_models, int nblk, const int32_t* __restrict__ turn_model,
                              const int64_t* __restrict__ turn_tok_off, int64_t* __restrict__ part) {
  __shared__ int64_t smem[32];
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  const int m = u < n_turns ? turn_model[u] : -1;
  const int64_t len = u < n_turns ? turn_tok_off[u + 1] - turn_tok_off[u] : 0;
  for (int k = 0; k < n_models; ++k) {
    const int64_t c = block_sum<int64_t>(m == k ? 1 : 0, smem);
    const int64_t t = block_sum<int64_t>(m == k ? len : 0, smem);
    if (threadIdx.x == 0) {
      part[static_cast<size_t>(2 * k) * nblk + blockIdx.x] = c;
      part[static_cast<size_t>(2 * k + 1) * nblk + blockIdx.x] = t;
    }
  }
}

// In-place exclusive prefix sum of each row of data[nrows][n]; one block per row, 8 items per thread per round.
__global__ void k_excl_scan_rows(int64_t* __restrict__ data, int n, int64_t* __restrict__ totals) {
  constexpr int kItems = 8;
  __shared__ int64_t smem[32];
  int64_t* row = data + static_cast<size_t>(blockIdx.x) * n;
  int64_t carry = 0;
  for (int i0 = 0; i0 < n; i0 += blockDim.x * kItems) {
    const int base = i0 + threadIdx.x * kItems;
    int64_t v[kItems];
    int64_t sum = 0;
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
      v[k] = base + k < n ? row[base + k] : 0;
      sum += v[k];
    }
    int64_t total;
    int64_t run = carry + block_excl_scan<int64_t>(sum, smem, &total);
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
      if (base + k < n) row[base + k] = run;
      run += v[k];
    }
    carry += total;
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}

// Stream offsets from the per-model totals, then each turn's segment slot and token offset.
__global__ void k_part_apply(int n_turns, int n_models, int nblk, int64_t n_tokens,
                             const int32_t* __restrict__ turn_model, const int64_t* __restrict__ turn_tok_off,
                             const int64_t* __restrict__ part, const int64_t* __restrict__ part_total,
                             int64_t* __restrict__ model_tok_off, int32_t* __restrict__ model_turn_off,
                             int64_t* __restrict__ turn_seg_off, int32_t* __restrict__ seg_turn) {
  __shared__ int64_t smem[32];
  __shared__ int64_t base_turn[UMAS_MAX_MODELS + 1], base_tok[UMAS_MAX_MODELS + 1];
  if (threadIdx.x == 0) {
    int64_t ct = 0, tk = 0;
    for (int k = 0; k < n_models; ++k) {
      base_turn[k] = ct;
      base_tok[k] = tk;
      ct += part_total[2 * k];
      tk += part_total[2 * k + 1];
    }
    base_turn[n_models] = ct;
    base_tok[n_models] = tk;
    if (blockIdx.x == 0) {
      for (int k = 0; k <= n_models; ++k) {
        model_turn_off[k] = static_cast<int32_t>(base_turn[k]);
        model_tok_off[k] = base_tok[k];
      }
      turn_seg_off[n_turns] = n_tokens;
    }
  }
  __syncthreads();
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  const int m = u < n_turns ? turn_model[u] : -1;
  const int64_t len = u < n_turns ? turn_tok_off[u + 1] - turn_tok_off[u] : 0;
  for (int k = 0; k < n_models; ++k) {
    int64_t tot;
    const int64_t c = block_excl_scan<int64_t>(m == k ? 1 : 0, smem, &tot);
    const int64_t t = block_excl_scan<int64_t>(m == k ? len : 0, smem, &tot);
    if (m == k) {
      const int64_t slot = base_turn[k] + part[static_cast<size_t>(2 * k) * nblk + blockIdx.x] + c;
      seg_turn[slot] = u;
      turn_seg_off[slot] = base_tok[k] + part[static_cast<size_t>(2 * k + 1) * nblk + blockIdx.x] + t;
    }
  }
}

// A trajectory run starts at a segment slot whose stream or trajectory differs from the slot before.
__device__ __forceinline__ int run_start(int s, const int32_t* seg_turn, const int32_t* turn_traj,
                                         const int32_t* turn_model) {
  if (s == 0) return 1;
  const int u = seg_turn[s], up = seg_turn[s - 1];
  return (turn_model[u] != turn_model[up] || turn_traj[u] != turn_traj[up]) ? 1 : 0;
}

__global__ void k_run_reduce(int n_turns, const int32_t* __restrict__ seg_turn,
                             const int32_t* __restrict__ turn_traj, const int32_t* __restrict__ turn_model,
                             int64_t* __restrict__ run_blk) {
  __shared__ int64_t smem[32];
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t f = s < n_turns ? run_start(s, seg_turn, turn_traj, turn_model) : 0;
  const int64_t c = block_sum<int64_t>(f, smem);
  if (threadIdx.x == 0) run_blk[blockIdx.x] = c;
}

__global__ void k_run_apply(int n_turns, int n_models, const int32_t* __restrict__ seg_turn,
                            const int32_t* __restrict__ turn_traj, const int32_t* __restrict__ turn_model,
                            const int64_t* __restrict__ run_blk, const int64_t* __restrict__ run_total,
                            const int64_t* __restrict__ turn_seg_off, const int32_t* __restrict__ model_turn_off,
                            int64_t* __restrict__ traj_seg_off, int32_t* __restrict__ model_trajrun_off) {
  __shared__ int64_t smem[32];
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t f = s < n_turns ? run_start(s, seg_turn, turn_traj, turn_model) : 0;
  int64_t tot;
  const int64_t r = run_blk[blockIdx.x] + block_excl_scan<int64_t>(f, smem, &tot);
  if (s < n_turns) {
    if (f) traj_seg_off[r] = turn_seg_off[s];
    for (int k = 0; k <= n_models; ++k)
      if (model_turn_off[k] == s) model_trajrun_off[k] = static_cast<int32_t>(r);
  }
  if (s == 0)
    for (int k = 0; k <= n_models; ++k)
      if (model_turn_off[k] == n_turns) model_trajrun_off[k] = static_cast<int32_t>(*run_total);
}

__global__ void k_fill_i64(int64_t* __restrict__ p, int64_t n, int64_t v) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Per turn segment, sixteen lanes each (four segments per wavefront, so that four chains of dependent loads are in
// flight per wavefront): the highest model-local position of a mask=1 token, the turn's source offset, role and
// reward gathered into one record, the flag bits of its last token (segment end; also trajectory-run end when a run
// starts at the segment's end offset or the stream ends there), and for every token block whose first token lies in
// the segment, the segment's index.
constexpr int kSegLanes = 16;
__global__ void k_seg_meta(int n_turns, int64_t n_tokens, const int32_t* __restrict__ seg_turn,
                           const int64_t* __restrict__ turn_tok_off, const int64_t* __restrict__ turn_seg_off,
                           const int32_t* __restrict__ turn_role, const float* __restrict__ turn_scalar,
                           const int32_t* __restrict__ turn_traj, const int32_t* __restrict__ turn_model,
                           const uint8_t* __restrict__ mask, SegMeta* __restrict__ seg_meta,
                           int32_t* __restrict__ blk_first) {
  const int sub = threadIdx.x & (kSegLanes - 1);
  const int s = (blockIdx.x * blockDim.x + threadIdx.x) / kSegLanes;
  const bool live = s < n_turns;                          // whole groups of sixteen lanes; everybody stays for the shuffles
  const int sc = live ? s : n_turns - 1;
  const bool has_next = sc + 1 < n_turns;
  const int u = seg_turn[sc];
  const int un = has_next ? seg_turn[sc + 1] : u;
  const int64_t g0 = turn_tok_off[u], len = live ? turn_tok_off[u + 1] - g0 : 0;
  const int64_t a = turn_seg_off[sc], e = a + len;
  const int64_t e_next = has_next ? turn_seg_off[sc + 2] : e;     // end of the next segment
  const int role = turn_role[u];
  const float rho = turn_scalar[u];
  const bool next_starts_run = turn_model[u] != turn_model[un] || turn_traj[u] != turn_traj[un];
  int64_t best = -1;
  // walk from the end, 64 tokens (four per lane) at a time; stop at the first step that holds a valid token
  for (int64_t hi = len; __any(hi > 0 && best < 0); hi -= 4 * kSegLanes) {
    int64_t cand = -1;
    if (hi > 0 && best < 0) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {                       // the highest index first
        const int64_t i = hi - 1 - (4 * sub + k);
        if (cand < 0 && i >= 0 && mask[g0 + i]) cand = i;
      }
    }
    // tokens 4 sub .. 4 sub + 3 counted from the end: a lower lane holds higher positions, the maximum is wanted
#pragma unroll
    for (int o = kSegLanes / 2; o > 0; o >>= 1) {
      const int64_t other = __shfl_xor(cand, o, kSegLanes);
      cand = other > cand ? other : cand;
    }
    if (hi > 0 && best < 0) best = cand;
  }
  if (live && sub == 0) {
    // a run ends at e when the stream ends there or a run starts at one of the segments that begin at e:
    // the next one, and if that one is empty the ones after it up to the first non-empty one
    bool run_end = e == n_tokens || (has_next && next_starts_run);
    if (!run_end && has_next && e_next <= e)
      for (int t = s + 2; t < n_turns && !run_end; ++t) {
        run_end = run_start(t, seg_turn, turn_traj, turn_model) != 0;
        if (turn_seg_off[t + 1] > e) break;
      }
    SegMeta m;
    m.src = g0;
    m.last_valid = best < 0 ? -1 : a + best;
    m.turn = u;
    m.role = role;
    m.rho = rho;
    m.end_flags = 2 | (run_end ? 4 : 0);
    seg_meta[s] = m;
  }
  if (live)
    for (int64_t b = (a + kTokBlock - 1) / kTokBlock + sub; b * kTokBlock < e; b += kSegLanes) blk_first[b] = s;
}

// Per token in model-local order: source index, turn, role, mask, flags, placed reward; per block the
// number of mask=1 tokens.  A block keeps the offsets and records of the kSegWin segments from the
// one that holds its first token in LDS; its threads search there (streams whose segments are so
// short that the window does not cover the block read global memory instead).
constexpr int kSegWin = 256;
__global__ void __launch_bounds__(kTokThreads)
k_tokens(int64_t n_tokens, int n_turns, int place_mode, const int64_t* __restrict__ turn_seg_off,
         const SegMeta* __restrict__ seg_meta, const int32_t* __restrict__ blk_first,
         const uint8_t* __restrict__ mask_global, int64_t* __restrict__ perm, int32_t* __restrict__ tok_turn,
         int32_t* __restrict__ tok_role, uint8_t* __restrict__ tok_mask, uint8_t* __restrict__ tok_flags,
         float* __restrict__ tok_reward, int64_t* __restrict__ tok_blk) {
  __shared__ int64_t smem[32];
  __shared__ int64_t s_off[kSegWin + 1];
  __shared__ int32_t s_loc[kSegWin + 1];            // the same offsets relative to the block's first token, clamped
  __shared__ SegMeta s_meta[kSegWin];
  const int64_t blk0 = static_cast<int64_t>(blockIdx.x) * kTokBlock;
  const int s_base = blk_first[blockIdx.x];
  // segments s_base .. s_end hold the block's tokens (s_end = the segment of the next block's first token)
  const int s_end = blk0 + kTokBlock < n_tokens ? blk_first[blockIdx.x + 1] : n_turns - 1;
  const int need = s_end - s_base + 1;
  const int win = need < kSegWin ? need : kSegWin;                           // s_off[0..win], s_meta[0..win) are valid
  for (int i = threadIdx.x; i <= win; i += kTokThreads) {
    const int64_t off = turn_seg_off[s_base + i];
    const int64_t rel = off - blk0;
    s_off[i] = off;
    s_loc[i] = static_cast<int32_t>(rel < -(1 << 30) ? -(1 << 30) : rel > (1 << 30) ? (1 << 30) : rel);
    if (i < win) s_meta[i] = seg_meta[s_base + i];
  }
  __syncthreads();
  const bool in_window = need <= kSegWin;           // every token of the block lies in a windowed segment
  const bool mask_aligned = (reinterpret_cast<uintptr_t>(mask_global) & 3) == 0;
  int64_t cnt[kTokRounds / kCntRounds] = {};
  // Phase A: every round's segment search and mask load.  All loads are in flight before the first
  // store is issued, so no round waits behind the stores of the round before it.
  int lo_r[kTokRounds];
  uint32_t m4_r[kTokRounds];
  bool fast_r[kTokRounds];
#pragma unroll
  for (int rd = 0; rd < kTokRounds; ++rd) {
    const int pl0 = rd * kTokRound + static_cast<int>(threadIdx.x) * kTokPerThread;   // block-relative
    const int64_t p0 = blk0 + pl0;
    lo_r[rd] = 0; m4_r[rd] = 0; fast_r[rd] = false;
    if (!in_window || p0 >= n_tokens) continue;
    int lo = 0, hi = win;                           // largest j with s_loc[j] <= pl0: the segment that holds p0
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (s_loc[mid] <= pl0) lo = mid; else hi = mid - 1;
    }
    lo_r[rd] = lo;
    // fast when the four tokens lie in one segment: no per-token bookkeeping
    fast_r[rd] = pl0 + kTokPerThread <= s_loc[lo + 1] && p0 + kTokPerThread <= n_tokens;
    if (fast_r[rd]) {
      const int64_t g0 = s_meta[lo].src + (p0 - s_off[lo]);
      if (mask_aligned && (g0 & 3) == 0) {
        m4_r[rd] = *reinterpret_cast<const uint32_t*>(mask_global + g0);
      } else {
        m4_r[rd] = static_cast<uint32_t>(mask_global[g0]) | (static_cast<uint32_t>(mask_global[g0 + 1]) << 8) |
                   (static_cast<uint32_t>(mask_global[g0 + 2]) << 16) | (static_cast<uint32_t>(mask_global[g0 + 3]) << 24);
      }
    }
  }
  // Phase B: outputs
#pragma unroll
  for (int rd = 0; rd < kTokRounds; ++rd) {
    const int pl0 = rd * kTokRound + static_cast<int>(threadIdx.x) * kTokPerThread;
    const int64_t p0 = blk0 + pl0;
    if (p0 >= n_tokens) continue;
    int s;
    if (in_window) {
      const int lo = lo_r[rd];
      s = s_base + lo;
      if (fast_r[rd]) {
        const SegMeta M = s_meta[lo];
        const int64_t g0 = M.src + (p0 - s_off[lo]);
        const uint32_t m4 = m4_r[rd];
        // every non-zero byte becomes 1: (b | 0x80) - 1 keeps bit 7 exactly when b > 0 or-ed with b's own bit 7
        const uint32_t mk4 = ((((m4 | 0x80808080u) - 0x01010101u) | m4) >> 7) & 0x01010101u;
        uint32_t fg4 = mk4;
        if (pl0 + kTokPerThread == s_loc[lo + 1]) fg4 |= static_cast<uint32_t>(M.end_flags) << 24;
        float rw4[kTokPerThread] = {0.f, 0.f, 0.f, 0.f};
        if (place_mode == UMAS_PLACE_ALL) {
#pragma unroll
          for (int k = 0; k < kTokPerThread; ++k) rw4[k] = ((mk4 >> (8 * k)) & 1u) ? M.rho : 0.f;
        } else {
          const int64_t idx = M.last_valid - p0;
#pragma unroll
          for (int k = 0; k < kTokPerThread; ++k) rw4[k] = idx == k ? M.rho : 0.f;
        }
        cnt[rd / kCntRounds] += __popc(mk4);
        *reinterpret_cast<longlong2*>(perm + p0) = make_longlong2(g0, g0 + 1);
        *reinterpret_cast<longlong2*>(perm + p0 + 2) = make_longlong2(g0 + 2, g0 + 3);
        *reinterpret_cast<int4*>(tok_turn + p0) = make_int4(M.turn, M.turn, M.turn, M.turn);
        *reinterpret_cast<int4*>(tok_role + p0) = make_int4(M.role, M.role, M.role, M.role);
        *reinterpret_cast<uint32_t*>(tok_mask + p0) = mk4;
        *reinterpret_cast<uint32_t*>(tok_flags + p0) = fg4;
        *reinterpret_cast<float4*>(tok_reward + p0) = make_float4(rw4[0], rw4[1], rw4[2], rw4[3]);
        continue;
      }
    } else {
      s = last_le(turn_seg_off, n_turns, p0);
    }
    int64_t pm[kTokPerThread];
    int32_t tt[kTokPerThread], tr[kTokPerThread];
    uint8_t mk[kTokPerThread], fg[kTokPerThread];
    float rw[kTokPerThread];
    int cur = -1;
    int64_t seg_a = 0, seg_e = 0;
    SegMeta M{};
    uint32_t m4 = 0;
    bool have_m4 = false;
#pragma unroll
    for (int k = 0; k < kTokPerThread; ++k) {
      const int64_t p = p0 + k;
      pm[k] = 0; tt[k] = 0; tr[k] = 0; mk[k] = 0; fg[k] = 0; rw[k] = 0.0f;
      if (p < n_tokens) {
        if (cur < 0 || p >= seg_e) {                // first token, or the segment changed
          if (in_window) { while (s_off[s - s_base + 1] <= p) ++s; }   // also steps over empty segments
          else { while (turn_seg_off[s + 1] <= p) ++s; }
          cur = s;
          seg_a = in_window ? s_off[s - s_base] : turn_seg_off[s];
          seg_e = in_window ? s_off[s - s_base + 1] : turn_seg_off[s + 1];
          M = in_window ? s_meta[s - s_base] : seg_meta[s];
          if (k == 0) {                             // all four tokens in one segment and a 4-byte aligned source: one load
            const int64_t g0 = M.src + (p0 - seg_a);
            have_m4 = mask_aligned && (g0 & 3) == 0 && p0 + kTokPerThread <= seg_e;
            if (have_m4) m4 = *reinterpret_cast<const uint32_t*>(mask_global + g0);
          }
        }
        const int64_t g = M.src + (p - seg_a);
        const uint8_t m = have_m4 ? (((m4 >> (8 * k)) & 0xFFu) ? 1 : 0) : (mask_global[g] ? 1 : 0);
        pm[k] = g; tt[k] = M.turn; tr[k] = M.role; mk[k] = m;
        fg[k] = static_cast<uint8_t>(m | (p == seg_e - 1 ? M.end_flags : 0));
        if (m && (place_mode == UMAS_PLACE_ALL || M.last_valid == p)) rw[k] = M.rho;
        cnt[rd / kCntRounds] += m;
      }
    }
    if (p0 + kTokPerThread <= n_tokens) {
      *reinterpret_cast<longlong2*>(perm + p0) = make_longlong2(pm[0], pm[1]);
      *reinterpret_cast<longlong2*>(perm + p0 + 2) = make_longlong2(pm[2], pm[3]);
      *reinterpret_cast<int4*>(tok_turn + p0) = make_int4(tt[0], tt[1], tt[2], tt[3]);
      *reinterpret_cast<int4*>(tok_role + p0) = make_int4(tr[0], tr[1], tr[2], tr[3]);
      *reinterpret_cast<uchar4*>(tok_mask + p0) = make_uchar4(mk[0], mk[1], mk[2], mk[3]);
      *reinterpret_cast<uchar4*>(tok_flags + p0) = make_uchar4(fg[0], fg[1], fg[2], fg[3]);
      *reinterpret_cast<float4*>(tok_reward + p0) = make_float4(rw[0], rw[1], rw[2], rw[3]);
    } else {
      for (int k = 0; k < kTokPerThread && p0 + k < n_tokens; ++k) {
        perm[p0 + k] = pm[k]; tok_turn[p0 + k] = tt[k]; tok_role[p0 + k] = tr[k];
        tok_mask[p0 + k] = mk[k]; tok_flags[p0 + k] = fg[k]; tok_reward[p0 + k] = rw[k];
      }
    }
  }
#pragma unroll
  for (int gi = 0; gi < kTokRounds / kCntRounds; ++gi) {
    const int64_t total = block_sum<int64_t>(cnt[gi], smem);
    const int64_t slot = static_cast<int64_t>(blockIdx.x) * (kTokRounds / kCntRounds) + gi;
    if (threadIdx.x == 0 && slot * kCntTokens < n_tokens) tok_blk[slot] = total;
    __syncthreads();                                // smem is reused by the next group's sum
  }
}

// Compaction of mask=1 positions into rowsel (stream-relative), plus the per-model offsets.  A block
// covers kSelBlock tokens = one count group of k_tokens, whose scanned counts give its base.
constexpr int kSelPerThread = 16;
constexpr int kSelBlock = kTokThreads * kSelPerThread;
static_assert(kSelBlock == kCntTokens, "a compaction block is one count group");
__global__ void __launch_bounds__(kTokThreads)
k_rowsel(int64_t n_tokens, int n_models, const uint8_t* __restrict__ tok_mask,
         const int64_t* __restrict__ model_tok_off, const int64_t* __restrict__ tok_blk,
         const int64_t* __restrict__ tok_total, int32_t* __restrict__ rowsel,
         int64_t* __restrict__ model_rowsel_off) {
  __shared__ int32_t smem[32];
  __shared__ int32_t s_out[kSelBlock];
  __shared__ int64_t moff[UMAS_MAX_MODELS + 1];
  if (static_cast<int>(threadIdx.x) <= n_models) moff[threadIdx.x] = model_tok_off[threadIdx.x];
  __syncthreads();
  const int64_t p0 = (static_cast<int64_t>(blockIdx.x) * kTokThreads + threadIdx.x) * kSelPerThread;
  uint32_t w[4] = {0u, 0u, 0u, 0u};
  if (p0 + kSelPerThread <= n_tokens) {
    const uint4 m4 = *reinterpret_cast<const uint4*>(tok_mask + p0);
    w[0] = m4.x; w[1] = m4.y; w[2] = m4.z; w[3] = m4.w;
  } else {
    for (int k = 0; k < kSelPerThread; ++k)
      if (p0 + k < n_tokens) w[k >> 2] |= static_cast<uint32_t>(tok_mask[p0 + k]) << (8 * (k & 3));
  }
  const int32_t cnt = __popc(w[0]) + __popc(w[1]) + __popc(w[2]) + __popc(w[3]);   // mask bytes are 0 or 1
  int32_t tot;
  const int64_t base = tok_blk[blockIdx.x];
  int32_t lpos = block_excl_scan<int32_t>(cnt, smem, &tot);
  // a model's stream may start inside this block: only then do tokens need the per-token boundary checks
  const int64_t sel0 = static_cast<int64_t>(blockIdx.x) * kSelBlock;
  bool boundary = false;
  for (int j = 0; j <= n_models; ++j) boundary |= moff[j] > sel0 && moff[j] < sel0 + kSelBlock;
  if (p0 < n_tokens) {
    int m = 0;
    while (m < n_models && moff[m + 1] <= p0) ++m;
    if (!boundary) {
      for (int j = 0; j <= n_models; ++j)
        if (moff[j] == p0) model_rowsel_off[j] = base + lpos;      // only a block's first token can start a stream here
      const int32_t rel = static_cast<int32_t>(p0 - moff[m]);
#pragma unroll
      for (int k = 0; k < kSelPerThread; ++k)
        if ((w[k >> 2] >> (8 * (k & 3))) & 1u) s_out[lpos++] = rel + k;   // bytes past n_tokens are 0
    } else {
#pragma unroll
      for (int k = 0; k < kSelPerThread; ++k) {
        const int64_t p = p0 + k;
        if (p < n_tokens) {
          while (m < n_models && moff[m + 1] <= p) ++m;
          for (int j = 0; j <= n_models; ++j)
            if (moff[j] == p) model_rowsel_off[j] = base + lpos;
          if ((w[k >> 2] >> (8 * (k & 3))) & 1u) s_out[lpos++] = static_cast<int32_t>(p - moff[m]);
        }
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < tot; i += kTokThreads) rowsel[base + i] = s_out[i];   // compacted, coalesced
  if (blockIdx.x == 0 && threadIdx.x == 0)
    for (int j = 0; j <= n_models; ++j)
      if (moff[j] >= n_tokens) model_rowsel_off[j] = *tok_total;
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
  for (int u = 0; u < g->n_turns; ++u) {
    UMAS_REQUIRE(g->turn_tok_off[u] <= g->turn_tok_off[u + 1], UMAS_EINVAL, "turn_tok_off decreases at %d", u);
    UMAS_REQUIRE(g->turn_role[u] >= 0 && g->turn_role[u] < g->n_roles, UMAS_EINVAL,
                 "turn_role[%d]=%d is not a role in [0,%d)", u, g->turn_role[u], g->n_roles);
  }
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
  // block of pinned host memory and go to the device in one asynchronous copy.  The host arrays have been read when
  // the call returns; the host does not wait for the stream.
  char* const ws_base = static_cast<char*>(workspace);
  const size_t staged_bytes = static_cast<size_t>(reinterpret_cast<char*>(w.traj_norm) - ws_base);
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
  const int nbt = cdiv(U > 0 ? U : 1, kTurnBlock);
  hipLaunchKernelGGL(k_fill_i64, dim3(cdiv(U + 1, 256)), dim3(256), 0, st, o->traj_seg_off,
                     static_cast<int64_t>(U) + 1, N);
  UMAS_LAUNCHED("k_fill_i64");
  hipLaunchKernelGGL(k_fill_i64, dim3(1), dim3(256), 0, st, o->model_rowsel_off, static_cast<int64_t>(K) + 1,
                     static_cast<int64_t>(0));
  UMAS_LAUNCHED("k_fill_i64");
  if (U > 0) {
    hipLaunchKernelGGL(k_turn_meta, dim3(nbt), dim3(kTurnBlock), 0, st, B, U, R, w.traj_turn_off, w.turn_role,
                       w.role_to_model, r->role_reward ? w.role_reward : nullptr,
                       r->turn_reward ? w.turn_reward : nullptr, traj_r, r->w_role ? w.weights : nullptr,
                       r->w_turn ? w.weights + R : nullptr, r->w_traj ? w.weights + 2 * R : nullptr,
                       w.turn_traj, w.turn_model, o->turn_step, o->turn_scalar);
    UMAS_LAUNCHED("k_turn_meta");
  }
  hipLaunchKernelGGL(k_part_reduce, dim3(nbt), dim3(kTurnBlock), 0, st, U, K, nbt, w.turn_model, w.turn_tok_off,
                     w.part);
  UMAS_LAUNCHED("k_part_reduce");
  hipLaunchKernelGGL(k_excl_scan_rows, dim3(2 * K), dim3(1024), 0, st, w.part, nbt, w.part_total);
  UMAS_LAUNCHED("k_excl_scan_rows");
  hipLaunchKernelGGL(k_part_apply, dim3(nbt), dim3(kTurnBlock), 0, st, U, K, nbt, N, w.turn_model, w.turn_tok_off,
                     w.part, w.part_total, o->model_tok_off, o->model_turn_off, o->turn_seg_off, o->seg_turn);
  UMAS_LAUNCHED("k_part_apply");
  hipLaunchKernelGGL(k_run_reduce, dim3(nbt), dim3(kTurnBlock), 0, st, U, o->seg_turn, w.turn_traj, w.turn_model,
                     w.run_blk);
  UMAS_LAUNCHED("k_run_reduce");
  hipLaunchKernelGGL(k_excl_scan_rows, dim3(1), dim3(1024), 0, st, w.run_blk, nbt, w.run_total);
  UMAS_LAUNCHED("k_excl_scan_rows");
  hipLaunchKernelGGL(k_run_apply, dim3(nbt), dim3(kTurnBlock), 0, st, U, K, o->seg_turn, w.turn_traj, w.turn_model,
                     w.run_blk, w.run_total, o->turn_seg_off, o->model_turn_off, o->traj_seg_off,
                     o->model_trajrun_off);
  UMAS_LAUNCHED("k_run_apply");
  if (U > 0 && N > 0) {
    hipLaunchKernelGGL(k_seg_meta, dim3(cdiv(U, 256 / kSegLanes)), dim3(256), 0, st, U, N, o->seg_turn, w.turn_tok_off,
                       o->turn_seg_off, w.turn_role, o->turn_scalar, w.turn_traj, w.turn_model, tok_mask_global,
                       w.seg_meta, w.blk_first);
    UMAS_LAUNCHED("k_seg_meta");
    const int nbk = cdiv(N, kTokBlock);
    hipLaunchKernelGGL(k_tokens, dim3(nbk), dim3(kTokThreads), 0, st, N, U, r->place_mode, o->turn_seg_off, w.seg_meta,
                       w.blk_first, tok_mask_global, o->perm, o->tok_turn, o->tok_role, o->tok_mask, o->tok_flags,
                       o->tok_reward, w.tok_blk);
    UMAS_LAUNCHED("k_tokens");
    hipLaunchKernelGGL(k_excl_scan_rows, dim3(1), dim3(1024), 0, st, w.tok_blk, cdiv(N, kCntTokens), w.tok_total);
    UMAS_LAUNCHED("k_excl_scan_rows");
    hipLaunchKernelGGL(k_rowsel, dim3(cdiv(N, kSelBlock)), dim3(kTokThreads), 0, st, N, K, o->tok_mask, o->model_tok_off,
                       w.tok_blk, w.tok_total, o->rowsel, o->model_rowsel_off);
    UMAS_LAUNCHED("k_rowsel");
  }
  return UMAS_OK;
}
