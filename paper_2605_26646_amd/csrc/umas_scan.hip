// Generalised advantage estimation as a masked, segmented reverse scan.
//
// A_t = sum_l (gamma lam)^l delta_{t+l}, delta_t = r_t + gamma V(s_{t+1}) - V(s_t) (paragraph
// "Advantage computation and policy evaluation") is evaluated by its backward recurrence.
// Walking a segment from its last token to its first with the carried state (G, NV) =
// (advantage of the next valid token, value of the next valid token):
//   valid token   G' = gamma*lam*G + gamma*NV + (r - V),  NV' = V
//   masked token  state unchanged, outputs 0
//   segment end   state reset to (0, 0) before the segment's last token
//   turn boundary inside a trajectory segment: state scaled by gamma_turn^(step difference)
// Every one of these is an affine map of (G, NV) of the form
//   G' = a G + b NV + c,  NV' = e NV + f
// and such maps compose associatively, so the recurrence is a parallel scan over maps:
// threads fold their own tokens, wavefronts and blocks combine the folds, and a second pass
// replays each thread's tokens from its incoming state.
#include "umas_common.h"

namespace umas {
namespace {

constexpr int kThreads = 256;
constexpr int kIpt = 16;                   // tokens per thread
constexpr int kTile = kThreads * kIpt;     // tokens per block
constexpr int kPad = kIpt + 1;             // LDS row pitch in words: conflict-free per-thread runs

struct Aff {
  float a, b, c, e, f;
};
__device__ __forceinline__ Aff aff_identity() { return Aff{1.f, 0.f, 0.f, 1.f, 0.f}; }
// the map "first, then second"
__device__ __forceinline__ Aff then(const Aff& first, const Aff& second) {
  Aff r;
  r.a = second.a * first.a;
  r.b = second.a * first.b + second.b * first.e;
  r.c = second.a * first.c + second.b * first.f + second.c;
  r.e = second.e * first.e;
  r.f = second.e * first.f + second.f;
  return r;
}
__device__ __forceinline__ Aff aff_shfl_down(const Aff& m, int o) {
  return Aff{__shfl_down(m.a, o, kWave), __shfl_down(m.b, o, kWave), __shfl_down(m.c, o, kWave),
             __shfl_down(m.e, o, kWave), __shfl_down(m.f, o, kWave)};
}

struct ScanParams {
  int64_t n_tokens;
  int n_seg_entries;           // seg_off has n_seg_entries + 1 entries
  const int64_t* seg_off;      // segment offsets (turn segments or trajectory runs), ascending
  int n_turns;
  const int64_t* turn_seg_off; // only read when decay is on
  const int32_t* tok_turn;     // only read when decay is on
  const int32_t* turn_step;    // only read when decay is on
  int decay;                   // 1: scale the state by gamma_turn^dstep at turn boundaries
  float gamma, lam, gamma_turn;
  const float* reward;
  const float* value;          // may be NULL
  const uint8_t* mask;
};

// Cursor over an ascending offsets array that answers, for tokens visited in descending order,
// whether position p+1 is a boundary.
struct BoundaryCursor {
  const int64_t* off;
  int j;
  __device__ __forceinline__ void init(const int64_t* o, int n, int64_t p_hi_plus1) {
    off = o;
    j = last_le(o, n, p_hi_plus1);
  }
  __device__ __forceinline__ bool at(int64_t p_plus1) {
    while (j > 0 && off[j] > p_plus1) --j;
    return off[j] == p_plus1;
  }
};

// Loads the block's tile of rewards, values and masks into LDS (coalesced), so that each thread
// can then walk its own kIpt consecutive tokens.
__device__ __forceinline__ void load_tile(const ScanParams& P, int64_t t0, float* s_r, float* s_v, uint8_t* s_m) {
  for (int i = threadIdx.x; i < kTile; i += kThreads) {
    const int64_t p = t0 + i;
    const bool in = p < P.n_tokens;
    const int q = i + i / kIpt;
    s_r[q] = in ? P.reward[p] : 0.f;
    s_v[q] = (in && P.value) ? P.value[p] : 0.f;
    s_m[i] = in ? P.mask[p] : 0;
  }
}

// Map of one token (applied after the boundary effects that sit between it and its right neighbour).
__device__ __forceinline__ Aff token_map(const ScanParams& P, int64_t p, float r, float v, uint8_t m,
                                         BoundaryCursor& seg, BoundaryCursor& turn) {
  Aff t = m ? Aff{P.gamma * P.lam, P.gamma, r - v, 0.f, v} : aff_identity();
  if (seg.at(p + 1)) {
    return then(Aff{0.f, 0.f, 0.f, 0.f, 0.f}, t);
  }
  if (P.decay && turn.at(p + 1)) {
    const int ds = P.turn_step[P.tok_turn[p + 1]] - P.turn_step[P.tok_turn[p]];
    const float k = powf(P.gamma_turn, static_cast<float>(ds));
    return then(Aff{k, 0.f, 0.f, k, 0.f}, t);
  }
  return t;
}

// Fold of the thread's tokens, from its last token to its first.
__device__ __forceinline__ Aff thread_fold(const ScanParams& P, int64_t p0, const float* s_r, const float* s_v,
                                           const uint8_t* s_m) {
  Aff acc = aff_identity();
  if (p0 >= P.n_tokens) return acc;
  const int64_t hi = (p0 + kIpt < P.n_tokens ? p0 + kIpt : P.n_tokens);
  BoundaryCursor seg, turn;
  seg.init(P.seg_off, P.n_seg_entries, hi);
  if (P.decay) turn.init(P.turn_seg_off, P.n_turns, hi);
  const int base = threadIdx.x * kPad;
  for (int k = static_cast<int>(hi - p0) - 1; k >= 0; --k) {
    const Aff t = token_map(P, p0 + k, s_r[base + k], s_v[base + k], s_m[threadIdx.x * kIpt + k], seg, turn);
    acc = then(acc, t);
  }
  return acc;
}

// For every thread, the composition of the folds of all threads to its right inside the block
// (exclusive, in application order right to left); *block_fold gets the fold of the whole block.
__device__ __forceinline__ Aff block_suffix_excl(Aff mine, Aff* s_w, Aff* block_fold) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int nwave = blockDim.x / kWave;
  // inclusive suffix inside the wavefront: incl(lane) = fold(63) then ... then fold(lane)
  Aff incl = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const Aff right = aff_shfl_down(incl, o);
    if (lane + o < kWave) incl = then(right, incl);
  }
  Aff excl = aff_shfl_down(incl, 1);
  if (lane == kWave - 1) excl = aff_identity();
  __syncthreads();
  if (lane == 0) s_w[wave] = incl;
  __syncthreads();
  Aff right_waves = aff_identity();
  for (int w = nwave - 1; w > wave; --w) right_waves = then(right_waves, s_w[w]);
  Aff all = aff_identity();
  for (int w = nwave - 1; w >= 0; --w) all = then(all, s_w[w]);
  *block_fold = all;
  return then(right_waves, excl);
}

__global__ void __launch_bounds__(kThreads) k_scan_fold(ScanParams P, Aff* __restrict__ blk_fold) {
  __shared__ float s_r[kThreads * kPad], s_v[kThreads * kPad];
  __shared__ uint8_t s_m[kTile];
  __shared__ Aff s_w[kThreads / kWave];
  const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kTile;
  load_tile(P, t0, s_r, s_v, s_m);
  __syncthreads();
  const Aff mine = thread_fold(P, t0 + static_cast<int64_t>(threadIdx.x) * kIpt, s_r, s_v, s_m);
  Aff all;
  block_suffix_excl(mine, s_w, &all);
  if (threadIdx.x == 0) blk_fold[blockIdx.x] = all;
}

// State entering each block from its right: a reverse exclusive scan over the block folds applied
// to the empty state.  One block; each thread owns a contiguous range of blocks.
__global__ void __launch_bounds__(1024) k_scan_carry(int nblk, const Aff* __restrict__ blk_fold,
                                                     float2* __restrict__ blk_state) {
  __shared__ Aff s_w[1024 / kWave];
  const int per = (nblk + blockDim.x - 1) / blockDim.x;
  const int lo = threadIdx.x * per;
  const int hi = lo + per < nblk ? lo + per : nblk;
  Aff mine = aff_identity();
  for (int b = hi - 1; b >= lo; --b) mine = then(mine, blk_fold[b]);
  Aff all;
  const Aff from_right = block_suffix_excl(mine, s_w, &all);
  float G = from_right.c, NV = from_right.f;   // the map applied to (0, 0)
  for (int b = hi - 1; b >= lo; --b) {
    blk_state[b] = make_float2(G, NV);
    const Aff m = blk_fold[b];
    const float g2 = m.a * G + m.b * NV + m.c;
    NV = m.e * NV + m.f;
    G = g2;
  }
}

__global__ void __launch_bounds__(kThreads)
k_scan_apply(ScanParams P, const float2* __restrict__ blk_state, float* __restrict__ adv,
             float* __restrict__ ret) {
  __shared__ float s_r[kThreads * kPad], s_v[kThreads * kPad];
  __shared__ uint8_t s_m[kTile];
  __shared__ Aff s_w[kThreads / kWave];
  const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kTile;
  load_tile(P, t0, s_r, s_v, s_m);
  __syncthreads();
  const int64_t p0 = t0 + static_cast<int64_t>(threadIdx.x) * kIpt;
  const Aff mine = thread_fold(P, p0, s_r, s_v, s_m);
  Aff all;
  const Aff from_right = block_suffix_excl(mine, s_w, &all);
  const float2 st = blk_state[blockIdx.x];
  float G = from_right.a * st.x + from_right.b * st.y + from_right.c;
  float NV = from_right.e * st.y + from_right.f;
  // replay this thread's tokens; outputs overwrite the staged inputs in LDS
  if (p0 < P.n_tokens) {
    const int64_t hi = (p0 + kIpt < P.n_tokens ? p0 + kIpt : P.n_tokens);
    BoundaryCursor seg, turn;
    seg.init(P.seg_off, P.n_seg_entries, hi);
    if (P.decay) turn.init(P.turn_seg_off, P.n_turns, hi);
    const int base = threadIdx.x * kPad;
    for (int k = static_cast<int>(hi - p0) - 1; k >= 0; --k) {
      const float r = s_r[base + k], v = s_v[base + k];
      const uint8_t m = s_m[threadIdx.x * kIpt + k];
      const Aff t = token_map(P, p0 + k, r, v, m, seg, turn);
      const float g2 = t.a * G + t.b * NV + t.c;
      NV = t.e * NV + t.f;
      G = g2;
      s_r[base + k] = m ? G : 0.f;
      s_v[base + k] = m ? G + v : 0.f;
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kTile; i += kThreads) {
    const int64_t p = t0 + i;
    if (p < P.n_tokens) {
      const int q = i + i / kIpt;
      adv[p] = s_r[q];
      ret[p] = s_v[q];
    }
  }
}

}  // namespace
}  // namespace umas

using namespace umas;

extern "C" size_t umas_advantages_workspace_bytes(int64_t n_tokens) {
  if (n_tokens < 0) return 0;
  const size_t nblk = cdiv(n_tokens > 0 ? n_tokens : 1, kTile);
  Carver c(nullptr);
  c.take<Aff>(nblk);
  c.take<float2>(nblk);
  return c.off;
}

extern "C" umas_status umas_advantages(const umas_streams* s, int64_t n_tokens, int32_t n_turns,
                                       const float* value, float gamma, float lam, float gamma_turn,
                                       int32_t seg_mode, float* adv, float* ret, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
  UMAS_REQUIRE(s, UMAS_EINVAL, "streams is NULL");
  UMAS_REQUIRE(n_tokens >= 0 && n_turns >= 0, UMAS_EINVAL, "negative size");
  UMAS_REQUIRE(seg_mode == UMAS_SEG_TURN || seg_mode == UMAS_SEG_TRAJ, UMAS_EINVAL, "seg_mode=%d is neither TURN nor TRAJ",
               seg_mode);
  UMAS_REQUIRE(s->tok_reward && s->tok_mask && s->turn_seg_off && s->traj_seg_off && s->tok_turn && s->turn_step,
               UMAS_EINVAL, "streams lacks tok_reward, tok_mask, turn_seg_off, traj_seg_off, tok_turn or turn_step");
  UMAS_REQUIRE((adv && ret) || n_tokens == 0, UMAS_EINVAL, "adv and ret must not be NULL");
  UMAS_REQUIRE(gamma == gamma && lam == lam && gamma_turn == gamma_turn, UMAS_EINVAL, "gamma, lam, gamma_turn must be numbers");
  const size_t need = umas_advantages_workspace_bytes(n_tokens);
  UMAS_REQUIRE(workspace && reinterpret_cast<uintptr_t>(workspace) % kAlign == 0 && workspace_bytes >= need,
               UMAS_EWORKSPACE, "workspace must be 256-byte aligned and hold %zu bytes (got %zu)", need,
               workspace_bytes);
  if (n_tokens == 0) return UMAS_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  const int nblk = cdiv(n_tokens, kTile);
  Carver c(workspace);
  Aff* blk_fold = c.take<Aff>(nblk);
  float2* blk_state = c.take<float2>(nblk);
  ScanParams P;
  P.n_tokens = n_tokens;
  P.n_seg_entries = n_turns;
  P.seg_off = seg_mode == UMAS_SEG_TURN ? s->turn_seg_off : s->traj_seg_off;
  P.n_turns = n_turns;
  P.turn_seg_off = s->turn_seg_off;
  P.tok_turn = s->tok_turn;
  P.turn_step = s->turn_step;
  P.decay = (seg_mode == UMAS_SEG_TRAJ && gamma_turn != 1.0f) ? 1 : 0;
  P.gamma = gamma;
  P.lam = lam;
  P.gamma_turn = gamma_turn;
  P.reward = s->tok_reward;
  P.value = value;
  P.mask = s->tok_mask;
  hipLaunchKernelGGL(k_scan_fold, dim3(nblk), dim3(kThreads), 0, st, P, blk_fold);
  UMAS_LAUNCHED("k_scan_fold");
  hipLaunchKernelGGL(k_scan_carry, dim3(1), dim3(1024), 0, st, nblk, blk_fold, blk_state);
  UMAS_LAUNCHED("k_scan_carry");
  hipLaunchKernelGGL(k_scan_apply, dim3(nblk), dim3(kThreads), 0, st, P, blk_state, adv, ret);
  UMAS_LAUNCHED("k_scan_apply");
  return UMAS_OK;
}
