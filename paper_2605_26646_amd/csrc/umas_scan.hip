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
// and such maps compose associatively, so inside a tile of a few thousand tokens the recurrence is a parallel
// scan over maps: threads fold their own few tokens, wavefronts and the block combine the folds, and
// each thread replays its tokens from its incoming state.
//
// One pass over memory (17 bytes per token): segments are independent, so the stream is cut at
// segment boundaries into ranges of about `chunk` tokens; a block walks the tiles of its range from
// right to left and carries the state from tile to tile itself.  No block waits for another.
#include "umas_common.h"

namespace umas {
namespace {

constexpr int kThreads = 256;
constexpr int kIpt = 8;                          // tokens per thread (8 or 16)
constexpr int kTile = kThreads * kIpt;           // tokens per tile
constexpr int kRow = kIpt + 4;                   // LDS words per thread row: its values + 4 words of padding
constexpr int kLdsWords = kThreads * kRow;

enum : uint8_t { kFlagMask = 1, kFlagTurnEnd = 2, kFlagRunEnd = 4 };

struct Aff {
  float a, b, c, e, f;
};
__device__ __forceinline__ Aff aff_identity() { return Aff{1.f, 0.f, 0.f, 1.f, 0.f}; }
// the map "first, then second".  HV = false (no value estimates): NV stays 0, so only G' = a G + c is
// carried and b, e, f are never looked at.
template <bool HV>
__device__ __forceinline__ Aff then(const Aff& first, const Aff& second) {
  Aff r;
  r.a = second.a * first.a;
  if constexpr (HV) {
    r.b = second.a * first.b + second.b * first.e;
    r.c = second.a * first.c + second.b * first.f + second.c;
    r.e = second.e * first.e;
    r.f = second.e * first.f + second.f;
  } else {
    r.b = 0.f;
    r.c = second.a * first.c + second.c;
    r.e = 0.f;
    r.f = 0.f;
  }
  return r;
}
template <bool HV>
__device__ __forceinline__ Aff aff_shfl_down(const Aff& m, int o) {
  if constexpr (HV)
    return Aff{__shfl_down(m.a, o, kWave), __shfl_down(m.b, o, kWave), __shfl_down(m.c, o, kWave),
               __shfl_down(m.e, o, kWave), __shfl_down(m.f, o, kWave)};
  else
    return Aff{__shfl_down(m.a, o, kWave), 0.f, __shfl_down(m.c, o, kWave), 0.f, 0.f};
}

struct ScanParams {
  int64_t n_tokens;
  int64_t chunk;               // tokens per block before snapping to segment boundaries (multiple of kTile)
  int n_seg_entries;           // seg_off has n_seg_entries + 1 entries, ascending, from 0 to n_tokens
  const int64_t* seg_off;
  const uint8_t* flags;        // per token: mask, last-of-turn, last-of-run
  const float* reward;
  const float* value;          // may be NULL
  const int32_t* tok_turn;     // only read when decay is on
  const int32_t* turn_step;    // only read when decay is on
  uint8_t seg_bit;             // kFlagTurnEnd or kFlagRunEnd: which flag ends a segment
  int decay;                   // 1: scale the state by gamma_turn^dstep at turn boundaries inside a segment
  float gamma, lam, gamma_turn;
};

// Smallest boundary (value of off[0..n]) that is >= x; off[0] = 0 and off[n] >= x.  Wavefront-wide:
// every lane of the calling wavefront takes part and gets the same answer.
__device__ __forceinline__ int64_t boundary_at_or_after(const int64_t* __restrict__ off, int n, int64_t x) {
  if (x <= 0) return 0;
  return off[wave_last_le(off, n, x - 1) + 1];
}

// Position of tile element e in the padded LDS arrays.
__device__ __forceinline__ int lds_pos(int e) { return e + 4 * (e / kIpt); }

// For every thread, the composition of the folds of all threads to its right inside the block
// (exclusive, in application order right to left).
template <bool HV>
__device__ __forceinline__ Aff block_suffix_excl(Aff mine, Aff* s_w) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  constexpr int nwave = kThreads / kWave;
  Aff incl = mine;   // inclusive suffix inside the wavefront: fold(63) then ... then fold(lane)
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const Aff right = aff_shfl_down<HV>(incl, o);
    if (lane + o < kWave) incl = then<HV>(right, incl);
  }
  Aff excl = aff_shfl_down<HV>(incl, 1);
  if (lane == kWave - 1) excl = aff_identity();
  if (lane == 0) s_w[wave] = incl;
  __syncthreads();
  Aff right_waves = aff_identity();
  for (int w = nwave - 1; w > wave; --w) right_waves = then<HV>(right_waves, s_w[w]);
  return then<HV>(right_waves, excl);
}

template <bool HV>
__global__ void __launch_bounds__(kThreads)
k_gae_scan(ScanParams P, float* __restrict__ adv, float* __restrict__ ret) {
  __shared__ __attribute__((aligned(16))) float s_r[kLdsWords], s_v[kLdsWords];
  __shared__ Aff s_w[kThreads / kWave];
  __shared__ float s_carry[2];
  __shared__ int64_t s_range[2];
  const int tid = threadIdx.x;
  if (tid < 2 * kWave) {     // wavefront 0 finds the left end of the range, wavefront 1 the right end
    const int which = tid / kWave;
    const int64_t x = (static_cast<int64_t>(blockIdx.x) + which) * P.chunk;
    const int64_t bnd = x >= P.n_tokens ? P.n_tokens : boundary_at_or_after(P.seg_off, P.n_seg_entries, x);
    if ((tid & (kWave - 1)) == 0) {
      s_range[which] = bnd;
      s_carry[which] = 0.f;
    }
  }
  __syncthreads();
  const int64_t start = s_range[0], end = s_range[1];
  if (start >= end) return;
  const float gl = P.gamma * P.lam;

  // raw tile in registers: element e = k*(kThreads*4) + tid*4 of the tile for the values (coalesced 16-byte
  // loads), this thread's own kIpt consecutive tokens for the flags
  struct Raw {
    float4 r4[kIpt / 4], v4[kIpt / 4];
    uint32_t w[kIpt / 4];
  };
  auto load_tile = [&](int64_t t0, Raw& x) {
#pragma unroll
    for (int k = 0; k < kIpt / 4; ++k) {
      const int64_t p = t0 + k * (kThreads * 4) + tid * 4;
      x.r4[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      x.v4[k] = x.r4[k];
      if (p + 3 < P.n_tokens) {
        x.r4[k] = *reinterpret_cast<const float4*>(P.reward + p);
        if constexpr (HV) x.v4[k] = *reinterpret_cast<const float4*>(P.value + p);
      } else {
        float* rp = &x.r4[k].x;
        float* vp = &x.v4[k].x;
        for (int j = 0; j < 4; ++j)
          if (p + j < P.n_tokens) {
            rp[j] = P.reward[p + j];
            if constexpr (HV) vp[j] = P.value[p + j];
          }
      }
    }
    const int64_t p0 = t0 + static_cast<int64_t>(tid) * kIpt;
    if (p0 + kIpt <= P.n_tokens) {
      if constexpr (kIpt == 16) {
        const uint4 f4 = *reinterpret_cast<const uint4*>(P.flags + p0);
        x.w[0] = f4.x; x.w[1] = f4.y; x.w[2] = f4.z; x.w[3] = f4.w;
      } else {
        const uint2 f2 = *reinterpret_cast<const uint2*>(P.flags + p0);
        x.w[0] = f2.x; x.w[1] = f2.y;
      }
    } else {
#pragma unroll
      for (int k = 0; k < kIpt / 4; ++k) x.w[k] = 0;
      for (int k = 0; k < kIpt; ++k)
        if (p0 + k < P.n_tokens) x.w[k >> 2] |= static_cast<uint32_t>(P.flags[p0 + k]) << (8 * (k & 3));
    }
  };

  const int64_t tile_first = start / kTile;
  Raw nxt;
  load_tile(((end - 1) / kTile) * kTile, nxt);
  for (int64_t tile = (end - 1) / kTile; tile >= tile_first; --tile) {
    const int64_t t0 = tile * kTile;
    // transpose through LDS into kIpt consecutive tokens per thread
#pragma unroll
    for (int k = 0; k < kIpt / 4; ++k) {
      const int e = k * (kThreads * 4) + tid * 4;
      *reinterpret_cast<float4*>(s_r + lds_pos(e)) = nxt.r4[k];
      if constexpr (HV) *reinterpret_cast<float4*>(s_v + lds_pos(e)) = nxt.v4[k];
    }
    const int64_t p0 = t0 + static_cast<int64_t>(tid) * kIpt;   // this thread's first token
    uint8_t fl[kIpt];
#pragma unroll
    for (int k = 0; k < kIpt; ++k) fl[k] = static_cast<uint8_t>(nxt.w[k >> 2] >> (8 * (k & 3)));
    if (tile > tile_first) load_tile(t0 - kTile, nxt);           // in flight while this tile is computed
    __syncthreads();
    float r[kIpt], v[kIpt];
#pragma unroll
    for (int k = 0; k < kIpt / 4; ++k) {
      const float4 r4 = *reinterpret_cast<const float4*>(s_r + tid * kRow + 4 * k);
      float4 v4 = make_float4(0.f, 0.f, 0.f, 0.f);
      if constexpr (HV) v4 = *reinterpret_cast<const float4*>(s_v + tid * kRow + 4 * k);
      r[4 * k] = r4.x; r[4 * k + 1] = r4.y; r[4 * k + 2] = r4.z; r[4 * k + 3] = r4.w;
      v[4 * k] = v4.x; v[4 * k + 1] = v4.y; v[4 * k + 2] = v4.z; v[4 * k + 3] = v4.w;
    }
    // tokens outside this block's range belong to a neighbour: identity here, not stored
    float kap[kIpt];   // decay applied before the token (1 = none)
#pragma unroll
    for (int k = 0; k < kIpt; ++k) {
      const int64_t p = p0 + k;
      if (p < start || p >= end) fl[k] = 0xFF;                   // marks "not mine"
      kap[k] = 1.f;
      if (P.decay && fl[k] != 0xFF && (fl[k] & kFlagTurnEnd) && !(fl[k] & P.seg_bit)) {
        const int ds = P.turn_step[P.tok_turn[p + 1]] - P.turn_step[P.tok_turn[p]];
        kap[k] = powf(P.gamma_turn, static_cast<float>(ds));
      }
    }
    // fold of this thread's tokens, right to left
    Aff acc = aff_identity();
#pragma unroll
    for (int k = kIpt - 1; k >= 0; --k) {
      if (fl[k] == 0xFF) continue;
      if (fl[k] & P.seg_bit) acc = Aff{0.f, 0.f, 0.f, 0.f, 0.f};
      else if (P.decay) { acc.a *= kap[k]; acc.b *= kap[k]; acc.c *= kap[k]; acc.e *= kap[k]; acc.f *= kap[k]; }
      if (fl[k] & kFlagMask) {
        const Aff t{gl, P.gamma, r[k] - v[k], 0.f, v[k]};
        acc = then<HV>(acc, t);
      }
    }
    const Aff from_right = block_suffix_excl<HV>(acc, s_w);
    float G = from_right.a * s_carry[0] + from_right.b * s_carry[1] + from_right.c;
    float NV = 0.f;
    if constexpr (HV) NV = from_right.e * s_carry[1] + from_right.f;
    // replay; results overwrite this thread's own LDS rows
#pragma unroll
    for (int k = kIpt - 1; k >= 0; --k) {
      float a = 0.f, b = 0.f;
      if (fl[k] != 0xFF) {
        if (fl[k] & P.seg_bit) { G = 0.f; NV = 0.f; }
        else if (P.decay) { G *= kap[k]; NV *= kap[k]; }
        if (fl[k] & kFlagMask) {
          G = (r[k] - v[k]) + P.gamma * NV + gl * G;
          NV = v[k];
          a = G;
          b = G + v[k];
        }
      }
      r[k] = a;
      v[k] = b;
    }
#pragma unroll
    for (int k = 0; k < kIpt / 4; ++k) {
      *reinterpret_cast<float4*>(s_r + tid * kRow + 4 * k) = make_float4(r[4 * k], r[4 * k + 1], r[4 * k + 2], r[4 * k + 3]);
      if constexpr (HV)     // without values the return equals the advantage
        *reinterpret_cast<float4*>(s_v + tid * kRow + 4 * k) = make_float4(v[4 * k], v[4 * k + 1], v[4 * k + 2], v[4 * k + 3]);
    }
    __syncthreads();                       // everyone has read s_carry and written its results
    if (tid == 0) { s_carry[0] = G; s_carry[1] = NV; }   // state at the tile's left edge
#pragma unroll
    for (int k = 0; k < kIpt / 4; ++k) {
      const int e = k * (kThreads * 4) + tid * 4;
      const int64_t p = t0 + e;
      const float4 a4 = *reinterpret_cast<const float4*>(s_r + lds_pos(e));
      float4 b4 = a4;
      if constexpr (HV) b4 = *reinterpret_cast<const float4*>(s_v + lds_pos(e));
      if (p >= start && p + 3 < end) {
        *reinterpret_cast<float4*>(adv + p) = a4;
        *reinterpret_cast<float4*>(ret + p) = b4;
      } else {
        const float* ap = &a4.x;
        const float* bp = &b4.x;
        for (int j = 0; j < 4; ++j)
          if (p + j >= start && p + j < end) { adv[p + j] = ap[j]; ret[p + j] = bp[j]; }
      }
    }
    __syncthreads();                       // LDS and s_carry are reused by the next tile
  }
}

}  // namespace
}  // namespace umas

using namespace umas;

extern "C" size_t umas_advantages_workspace_bytes(int64_t n_tokens) {
  (void)n_tokens;
  return kAlign;   // the scan keeps its state on chip; the argument is kept for interface stability
}

extern "C" umas_status umas_advantages(const umas_streams* s, int64_t n_tokens, int32_t n_turns,
                                       const float* value, float gamma, float lam, float gamma_turn,
                                       int32_t seg_mode, float* adv, float* ret, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  UMAS_REQUIRE(s, UMAS_EINVAL, "streams is NULL");
  UMAS_REQUIRE(n_tokens >= 0 && n_turns >= 0, UMAS_EINVAL, "negative size");
  UMAS_REQUIRE(seg_mode == UMAS_SEG_TURN || seg_mode == UMAS_SEG_TRAJ, UMAS_EINVAL, "seg_mode=%d is neither TURN nor TRAJ",
               seg_mode);
  UMAS_REQUIRE(s->tok_reward && s->tok_flags && s->turn_seg_off && s->traj_seg_off && s->tok_turn && s->turn_step,
               UMAS_EINVAL, "streams lacks tok_reward, tok_flags, turn_seg_off, traj_seg_off, tok_turn or turn_step");
  UMAS_REQUIRE((adv && ret) || n_tokens == 0, UMAS_EINVAL, "adv and ret must not be NULL");
  UMAS_REQUIRE(gamma == gamma && lam == lam && gamma_turn == gamma_turn, UMAS_EINVAL, "gamma, lam, gamma_turn must be numbers");
  UMAS_REQUIRE(reinterpret_cast<uintptr_t>(s->tok_reward) % 16 == 0 && reinterpret_cast<uintptr_t>(value) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(s->tok_flags) % 16 == 0 && reinterpret_cast<uintptr_t>(adv) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(ret) % 16 == 0,
               UMAS_EINVAL, "tok_reward, tok_flags, value, adv and ret must be 16-byte aligned");
  if (n_tokens == 0) return UMAS_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  ScanParams P;
  P.n_tokens = n_tokens;
  // about 32 ranges per compute unit (several rounds of resident blocks), each a whole number of tiles before it is snapped to segment boundaries
  const int64_t tiles = (n_tokens + kTile - 1) / kTile;
  const int64_t tiles_per_block = (tiles + 8191) / 8192;
  P.chunk = tiles_per_block * kTile;
  P.n_seg_entries = n_turns;
  P.seg_off = seg_mode == UMAS_SEG_TURN ? s->turn_seg_off : s->traj_seg_off;
  P.flags = s->tok_flags;
  P.reward = s->tok_reward;
  P.value = value;
  P.tok_turn = s->tok_turn;
  P.turn_step = s->turn_step;
  P.seg_bit = seg_mode == UMAS_SEG_TURN ? kFlagTurnEnd : kFlagRunEnd;
  P.decay = (seg_mode == UMAS_SEG_TRAJ && gamma_turn != 1.0f) ? 1 : 0;
  P.gamma = gamma;
  P.lam = lam;
  P.gamma_turn = gamma_turn;
  const unsigned nblk = cdiv(n_tokens, P.chunk);
  if (value) hipLaunchKernelGGL(k_gae_scan<true>, dim3(nblk), dim3(kThreads), 0, st, P, adv, ret);
  else hipLaunchKernelGGL(k_gae_scan<false>, dim3(nblk), dim3(kThreads), 0, st, P, adv, ret);
  UMAS_LAUNCHED("k_gae_scan");
  return UMAS_OK;
}
