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
// and such maps compose associatively, so inside a tile of 1024 tokens the recurrence is a parallel scan over maps:
// threads fold their own four tokens, wavefronts and the block combine the folds, and each thread replays its tokens
// from its incoming state.
//
// One pass over memory (17 bytes per token).  Segments are independent, so the stream is cut into ranges of about
// `chunk` tokens at segment boundaries; a workgroup walks the tiles of one range from right to left and carries the
// state from tile to tile itself, the loads of the next tile in flight.  Ranges of ordinary segments need nothing
// from each other: one workgroup per range, in any order (k_gae_scan).
// Only a segment longer than kLongSegment tokens is cut inside.  A range whose right end lies inside such a segment
// is left to a second kernel (k_gae_scan_cut): it first folds all of its tiles into one map and publishes it (a
// second read of that range), composes the published maps of the ranges to its right up to the segment's end into its
// incoming state, and then replays, so a stream that is one giant segment is still spread over the whole device.
// That kernel's workgroups are persistent (range number j G + b from the right in round j of workgroup b) and few
// (one per compute unit at most, a fraction of what the device holds at once, so all of them run together): a range
// only ever waits for maps of ranges to its right, written by the first kernel or by a workgroup that is running,
// and publishing a map waits for nothing, so every wait ends.  When no segment is that long the second kernel finds
// nothing to do and leaves at once.
#include "umas_common.h"

namespace umas {
namespace {

constexpr int kThreads = 256;
constexpr int kIpt = 4;                          // tokens per thread: one 16-byte load per array, no transposition
constexpr int kTile = kThreads * kIpt;           // tokens per tile
constexpr int kChunkTiles = 8;                   // nominal tiles per range
constexpr int64_t kChunk = static_cast<int64_t>(kChunkTiles) * kTile;
constexpr int64_t kLongSegment = 16 * kTile;     // a segment end farther away than this does not move a range's edge
constexpr int kAhead = 1;                        // tiles whose loads are in flight beyond the one in work

enum : uint8_t { kFlagMask = 1, kFlagTurnEnd = 2, kFlagRunEnd = 4 };
constexpr int kFlagStepShift = 3, kFlagStepMany = 31;   // bits 3-7 of a turn end inside a run: steps to the next turn

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

// One range of the stream.  Ranges are numbered from the right end of the stream.
struct __attribute__((aligned(16))) Range {
  int64_t start, end;          // tokens [start, end); empty when start == end
  int32_t cut_right;           // `end` lies inside a long segment: the state entering the range comes from the right
  int32_t cut_left;            // `start` lies inside a long segment: the range to the left will ask for this one's map
  int64_t pad;
};
static_assert(sizeof(Range) == 32, "two 16-byte loads");

constexpr int kStateWords = 5;                     // a, b, c, e, f (without value estimates only a and c are used)
constexpr unsigned long long kReady = 1ull << 32;  // mark in the upper half of a published word

struct ScanParams {
  int64_t n_tokens;
  uint32_t n_ranges;
  Range* ranges;                    // [n_ranges], written by k_gae_scan
  const int64_t* seg_off;           // [n_seg_entries + 1] ascending segment offsets, from 0 to n_tokens
  int n_seg_entries;
  unsigned long long* range_state;  // [n_ranges][kStateWords]: a published map, one float and its ready mark per 64-bit word
  const uint8_t* flags;        // per token: mask, last-of-turn, last-of-run
  const float* reward;
  const float* value;          // may be NULL
  const int32_t* tok_turn;     // only read when the step discount is on
  const int32_t* turn_step;    // only read when the step discount is on
  uint8_t seg_bit;             // kFlagTurnEnd or kFlagRunEnd: which flag ends a segment
  float gamma, lam, gamma_turn;
};

// A record is published word by word; every word carries its own ready mark, so no ordering between the words
// is needed: a reader takes a record when all of its words are marked.  (Device-scope atomics, relaxed.)
__device__ __forceinline__ void publish_word(unsigned long long* p, float x) {
  __hip_atomic_store(p, kReady | static_cast<unsigned long long>(__float_as_uint(x)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool read_word(unsigned long long* p, float* x) {
  const unsigned long long w = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  *x = __uint_as_float(static_cast<uint32_t>(w));
  return (w >> 32) != 0;
}
template <bool HV>
__device__ __forceinline__ void publish(unsigned long long* rec, const Aff& m) {
  publish_word(rec + 0, m.a);
  publish_word(rec + 2, m.c);
  if constexpr (HV) {
    publish_word(rec + 1, m.b);
    publish_word(rec + 3, m.e);
    publish_word(rec + 4, m.f);
  }
}

// ------------------------------------------------------------------ ranges
// Smallest boundary (value of off[0..n]) that is >= x, for ascending off with off[0] = 0 and off[n] >= x.
// Wavefront-wide: every lane of the calling wavefront takes part and gets the same answer.
__device__ __forceinline__ int64_t boundary_at_or_after(const int64_t* __restrict__ off, int n, int64_t x) {
  if (x <= 0) return 0;
  return off[wave_last_le(off, n, x - 1) + 1];
}
// Where the range edge nominally at x really lies: at the next segment boundary unless that is farther than
// kLongSegment away, in which case the edge stays at x, inside the segment (*cut = 1).
__device__ __forceinline__ int64_t range_edge(const int64_t* __restrict__ off, int n, int64_t n_tokens, int64_t x, int* cut) {
  *cut = 0;
  if (x <= 0) return 0;
  if (x >= n_tokens) return n_tokens;
  const int64_t b = boundary_at_or_after(off, n, x);
  if (b - x < kLongSegment) return b;
  *cut = 1;
  return x;
}
// ------------------------------------------------------------------ the scan
// For every thread, the composition of the folds of all threads to its right inside the block (exclusive, in
// application order right to left); *block_total gets the composition of all folds.  s_w holds one map per
// wavefront; the caller alternates between two such arrays so that one barrier per tile is enough.
template <bool HV>
__device__ __forceinline__ Aff block_suffix_excl(Aff mine, Aff* s_w, Aff* block_total) {
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
  Aff total = right_waves;
  for (int w = wave; w >= 0; --w) total = then<HV>(total, s_w[w]);
  *block_total = total;
  return then<HV>(right_waves, excl);
}

// The state that enters range q from the right, found by one wavefront: lane l looks at range q - 1 - l (ranges are
// numbered from the right), and the maps are composed up to the nearest range whose map is a constant, i.e. which
// holds the segment's end.  Only the records up to that range are waited for.
template <bool HV>
__device__ __forceinline__ void look_back(const ScanParams& P, uint32_t q, float* G_in, float* NV_in) {
  const int lane = threadIdx.x & (kWave - 1);
  Aff M = aff_identity();
  for (int64_t base = static_cast<int64_t>(q) - 1;; base -= kWave) {
    const int64_t k = base - lane;
    Aff A{0.f, 0.f, 0.f, 0.f, 0.f};                 // past the right end of the stream: the constant map to (0, 0)
    bool ready = true;
    int first = kWave;
    while (true) {
      if (k >= 0) {
        unsigned long long* rec = P.range_state + static_cast<size_t>(k) * kStateWords;
        ready = read_word(rec + 0, &A.a);
        ready = read_word(rec + 2, &A.c) && ready;
        if constexpr (HV) {
          ready = read_word(rec + 1, &A.b) && ready;
          ready = read_word(rec + 3, &A.e) && ready;
          ready = read_word(rec + 4, &A.f) && ready;
        }
      }
      const bool closed = ready && A.a == 0.f && (!HV || (A.b == 0.f && A.e == 0.f));   // a constant map: nothing further right matters
      const unsigned long long rdy = __ballot(ready), cls = __ballot(closed);
      const int n_ready = rdy == ~0ull ? kWave : __ffsll(static_cast<long long>(~rdy)) - 1;   // ready records in a row from lane 0
      first = cls ? __ffsll(static_cast<long long>(cls)) - 1 : kWave;
      if (first < n_ready || n_ready == kWave) break;
      __builtin_amdgcn_s_sleep(8);
    }
    const int upto = first < kWave ? first : kWave - 1;
    for (int j = 0; j <= upto; ++j) {
      Aff Aj;
      Aj.a = __shfl(A.a, j, kWave);
      Aj.c = __shfl(A.c, j, kWave);
      Aj.b = HV ? __shfl(A.b, j, kWave) : 0.f;
      Aj.e = HV ? __shfl(A.e, j, kWave) : 0.f;
      Aj.f = HV ? __shfl(A.f, j, kWave) : 0.f;
      M = then<HV>(Aj, M);                          // the farther range acts first
    }
    if (first < kWave) break;
  }
  *G_in = M.c;                                      // a constant map: its value
  *NV_in = HV ? M.f : 0.f;
}

// this thread's four consecutive tokens of a tile: 16 bytes per array, 4 bytes of flags; tokens past the end of the
// stream read as masked, without flags
struct Raw {
  float4 r4, v4;
  uint32_t w;
};
template <bool HV>
__device__ __forceinline__ void load_tile(const ScanParams& P, const Range& R, int64_t tile, Raw& x) {
  const int64_t p = tile * kTile + static_cast<int64_t>(threadIdx.x) * kIpt;
  x.r4 = make_float4(0.f, 0.f, 0.f, 0.f);
  x.v4 = x.r4;
  x.w = 0;
  if (p + kIpt <= R.start || p >= R.end) return;    // none of these tokens belongs to the range: a neighbour reads them
  if (p + kIpt <= P.n_tokens) {
    x.r4 = *reinterpret_cast<const float4*>(P.reward + p);
    if constexpr (HV) x.v4 = *reinterpret_cast<const float4*>(P.value + p);
    x.w = *reinterpret_cast<const uint32_t*>(P.flags + p);
  } else {
    float* rp = &x.r4.x;
    float* vp = &x.v4.x;
    for (int j = 0; j < kIpt; ++j)
      if (p + j < P.n_tokens) {
        rp[j] = P.reward[p + j];
        if constexpr (HV) vp[j] = P.value[p + j];
        x.w |= static_cast<uint32_t>(P.flags[p + j]) << (8 * j);
      }
  }
}

// One walk over the tiles of a range, right to left.  REPLAY = false: fold only, returns the range's map in *total.
// REPLAY = true: starts from the state (*G_io, *NV_io), writes advantages and returns, leaves the state at the
// range's left edge in (*G_io, *NV_io) (valid in thread 0).
template <bool HV, bool DECAY, bool REPLAY>
__device__ __forceinline__ void walk_range(const ScanParams& P, const Range& R, float* __restrict__ adv, float* __restrict__ ret,
                                           Aff (*s_w)[kThreads / kWave], float (*s_carry)[2], float* G_io, float* NV_io, Aff* total) {
  const int tid = threadIdx.x;
  const float gl = P.gamma * P.lam;
  const int64_t t_hi = (R.end - 1) / kTile, t_lo = R.start / kTile;
  Raw buf[kAhead + 1];
#pragma unroll
  for (int a = 0; a <= kAhead; ++a)
    if (t_hi - a >= t_lo) load_tile<HV>(P, R, t_hi - a, buf[a]);
  Aff range_map = aff_identity();
  if (REPLAY && tid == 0) { s_carry[0][0] = *G_io; s_carry[0][1] = *NV_io; }
  int par = 0;
  float G = 0.f, NV = 0.f;
  for (int64_t tile = t_hi; tile >= t_lo; --tile) {
    const Raw x = buf[0];
#pragma unroll
    for (int a = 0; a < kAhead; ++a) buf[a] = buf[a + 1];
    if (tile - kAhead - 1 >= t_lo) load_tile<HV>(P, R, tile - kAhead - 1, buf[kAhead]);
    const int64_t p0 = tile * kTile + static_cast<int64_t>(tid) * kIpt;
    const float r[kIpt] = {x.r4.x, x.r4.y, x.r4.z, x.r4.w};
    const float v[kIpt] = {x.v4.x, x.v4.y, x.v4.z, x.v4.w};
    uint32_t fl[kIpt];
    float kap[kIpt];                                // step discount applied before the token (1 = none)
    bool mine[kIpt];                                // tokens outside the range belong to a neighbour
#pragma unroll
    for (int k = 0; k < kIpt; ++k) {
      fl[k] = (x.w >> (8 * k)) & 0xFFu;
      mine[k] = p0 + k >= R.start && p0 + k < R.end;
      kap[k] = 1.f;
      if constexpr (DECAY) {
        if (mine[k] && (fl[k] & kFlagTurnEnd) && !(fl[k] & P.seg_bit)) {   // a later turn of the same run follows: p + 1 exists
          int ds = static_cast<int>(fl[k] >> kFlagStepShift);   // steps to the run's next turn; kFlagStepMany: more than fit
          if (ds == kFlagStepMany) {
            const int64_t p = p0 + k;
            ds = P.turn_step[P.tok_turn[p + 1]] - P.turn_step[P.tok_turn[p]];
          }
          kap[k] = powf(P.gamma_turn, static_cast<float>(ds));
        }
      }
    }
    // fold of this thread's tokens, right to left
    Aff acc = aff_identity();
#pragma unroll
    for (int k = kIpt - 1; k >= 0; --k) {
      if (!mine[k]) continue;
      if (fl[k] & P.seg_bit) acc = Aff{0.f, 0.f, 0.f, 0.f, 0.f};
      else if constexpr (DECAY) { acc.a *= kap[k]; acc.b *= kap[k]; acc.c *= kap[k]; acc.e *= kap[k]; acc.f *= kap[k]; }
      if (fl[k] & kFlagMask) {
        const Aff t{gl, P.gamma, r[k] - v[k], 0.f, v[k]};
        acc = then<HV>(acc, t);
      }
    }
    Aff tile_map;
    const Aff from_right = block_suffix_excl<HV>(acc, s_w[par], &tile_map);   // the one barrier of a tile
    if constexpr (!REPLAY) {
      range_map = then<HV>(range_map, tile_map);    // tiles further right act first
    } else {
      G = from_right.a * s_carry[par][0] + from_right.b * s_carry[par][1] + from_right.c;
      NV = 0.f;
      if constexpr (HV) NV = from_right.e * s_carry[par][1] + from_right.f;
      float a[kIpt], b[kIpt];
#pragma unroll
      for (int k = kIpt - 1; k >= 0; --k) {
        a[k] = 0.f;
        b[k] = 0.f;
        if (!mine[k]) continue;
        if (fl[k] & P.seg_bit) { G = 0.f; NV = 0.f; }
        else if constexpr (DECAY) { G *= kap[k]; NV *= kap[k]; }
        if (fl[k] & kFlagMask) {
          G = (r[k] - v[k]) + P.gamma * NV + gl * G;
          NV = v[k];
          a[k] = G;
          b[k] = G + v[k];
        }
      }
      if (tid == 0) { s_carry[par ^ 1][0] = G; s_carry[par ^ 1][1] = NV; }   // state at the tile's left edge
      if (mine[0] && mine[kIpt - 1]) {
        *reinterpret_cast<float4*>(adv + p0) = make_float4(a[0], a[1], a[2], a[3]);
        *reinterpret_cast<float4*>(ret + p0) = make_float4(b[0], b[1], b[2], b[3]);
      } else {
#pragma unroll
        for (int k = 0; k < kIpt; ++k)
          if (mine[k]) { adv[p0 + k] = a[k]; ret[p0 + k] = b[k]; }
      }
    }
    par ^= 1;
  }
  if constexpr (REPLAY) { *G_io = G; *NV_io = NV; } else { *total = range_map; }
}

// One workgroup per range.  It finds the range's edges (two wavefront-wide searches, one wavefront each), leaves them
// for the second kernel and clears the range's record; then, unless the range is empty or its right end lies inside a
// long segment, it scans the range: nothing comes in from the right.
template <bool HV, bool DECAY>
__global__ void __launch_bounds__(kThreads)
k_gae_scan(ScanParams P, float* __restrict__ adv, float* __restrict__ ret) {
  __shared__ Aff s_w[2][kThreads / kWave];
  __shared__ float s_carry[2][2];
  __shared__ int64_t s_edge[2];
  __shared__ int s_cut[2];
  const int tid = threadIdx.x;
  const uint32_t q = blockIdx.x;                                                   // from the right
  const int64_t i = static_cast<int64_t>(P.n_ranges) - 1 - q;                      // from the left
  if (tid < 2 * kWave) {
    const int which = tid / kWave;                   // wavefront 0: left edge, wavefront 1: right edge
    int cut;
    const int64_t edge = range_edge(P.seg_off, P.n_seg_entries, P.n_tokens, (i + which) * kChunk, &cut);
    if ((tid & (kWave - 1)) == 0) { s_edge[which] = edge; s_cut[which] = cut; }
  }
  __syncthreads();
  Range R;
  R.start = s_edge[0];
  R.end = s_edge[1];
  R.cut_left = s_cut[0];
  R.cut_right = s_cut[1];
  R.pad = 0;
  if (tid == 0) P.ranges[q] = R;
  if (tid < kStateWords) P.range_state[static_cast<size_t>(q) * kStateWords + tid] = 0ull;
  if (R.start >= R.end || R.cut_right) return;      // the same for every thread
  float G = 0.f, NV = 0.f;
  Aff unused;
  walk_range<HV, DECAY, true>(P, R, adv, ret, s_w, s_carry, &G, &NV, &unused);
  // a range that starts inside a long segment: what it hands to the left is a constant
  if (R.cut_left && tid == 0)
    publish<HV>(P.range_state + static_cast<size_t>(q) * kStateWords, Aff{0.f, 0.f, G, 0.f, HV ? NV : 0.f});
}

// The ranges whose right end lies inside a long segment; persistent workgroups.
template <bool HV, bool DECAY>
__global__ void __launch_bounds__(kThreads)
k_gae_scan_cut(ScanParams P, float* __restrict__ adv, float* __restrict__ ret) {
  __shared__ Aff s_w[2][kThreads / kWave];
  __shared__ float s_carry[2][2];
  __shared__ float s_in[2];
  const int tid = threadIdx.x;
  // does any of this workgroup's ranges need it?  every thread looks at some of them, all loads at once
  int mine = 0;
  for (uint64_t q = blockIdx.x + static_cast<uint64_t>(tid) * gridDim.x; q < P.n_ranges; q += static_cast<uint64_t>(kThreads) * gridDim.x)
    mine |= P.ranges[q].cut_right;
  if (!__syncthreads_or(mine)) return;
  for (uint32_t q = blockIdx.x; q < P.n_ranges; q += gridDim.x) {
    const Range R = P.ranges[q];
    if (R.start >= R.end || !R.cut_right) continue; // the same for every thread
    // the range's own map first (published if the left end is cut too), then the state that the ranges to its right
    // hand over, then the replay
    float G = 0.f, NV = 0.f;
    Aff range_map;
    walk_range<HV, DECAY, false>(P, R, adv, ret, s_w, s_carry, &G, &NV, &range_map);
    if (R.cut_left && tid == 0) publish<HV>(P.range_state + static_cast<size_t>(q) * kStateWords, range_map);
    if (tid < kWave) {
      float g_in, nv_in;
      look_back<HV>(P, q, &g_in, &nv_in);
      if (tid == 0) { s_in[0] = g_in; s_in[1] = nv_in; }
    }
    __syncthreads();                                // also: the LDS of the first walk is free
    G = s_in[0];
    NV = s_in[1];
    Aff unused;
    walk_range<HV, DECAY, true>(P, R, adv, ret, s_w, s_carry, &G, &NV, &unused);
    __syncthreads();
  }
}

inline int64_t scan_ranges(int64_t n_tokens) { return (n_tokens + kChunk - 1) / kChunk; }

}  // namespace
}  // namespace umas

using namespace umas;

extern "C" size_t umas_advantages_workspace_bytes(int64_t n_tokens) {
  if (n_tokens < 0) return 0;
  const size_t n = static_cast<size_t>(scan_ranges(n_tokens) > 0 ? scan_ranges(n_tokens) : 1);
  return align_up(n * sizeof(Range)) + align_up(n * kStateWords * sizeof(unsigned long long));   // ranges, records
}

extern "C" umas_status umas_advantages(const umas_streams* s, int64_t n_tokens, int32_t n_turns,
                                       const float* value, float gamma, float lam, float gamma_turn,
                                       int32_t seg_mode, float* adv, float* ret, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
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
  UMAS_REQUIRE(scan_ranges(n_tokens) < (1LL << 31), UMAS_ESHAPE, "at most 2^43 tokens");
  const size_t need = umas_advantages_workspace_bytes(n_tokens);
  UMAS_REQUIRE(workspace && reinterpret_cast<uintptr_t>(workspace) % kAlign == 0 && workspace_bytes >= need, UMAS_EWORKSPACE,
               "workspace must be 256-byte aligned and hold %zu bytes (got %zu)", need, workspace_bytes);
  if (n_tokens == 0) return UMAS_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  const int64_t n_ranges = scan_ranges(n_tokens);
  ScanParams P;
  P.n_tokens = n_tokens;
  P.n_ranges = static_cast<uint32_t>(n_ranges);
  Range* ranges = static_cast<Range*>(workspace);
  P.ranges = ranges;
  P.range_state = reinterpret_cast<unsigned long long*>(static_cast<char*>(workspace) + align_up(static_cast<size_t>(n_ranges) * sizeof(Range)));
  P.seg_off = seg_mode == UMAS_SEG_TURN ? s->turn_seg_off : s->traj_seg_off;
  P.n_seg_entries = n_turns;
  P.flags = s->tok_flags;
  P.reward = s->tok_reward;
  P.value = value;
  P.tok_turn = s->tok_turn;
  P.turn_step = s->turn_step;
  P.seg_bit = seg_mode == UMAS_SEG_TURN ? kFlagTurnEnd : kFlagRunEnd;
  P.gamma = gamma;
  P.lam = lam;
  P.gamma_turn = gamma_turn;
  const bool decay = seg_mode == UMAS_SEG_TRAJ && gamma_turn != 1.0f;
  void (*kernel)(ScanParams, float*, float*) =
      value ? (decay ? k_gae_scan<true, true> : k_gae_scan<true, false>) : (decay ? k_gae_scan<false, true> : k_gae_scan<false, false>);
  hipLaunchKernelGGL(kernel, dim3(P.n_ranges), dim3(kThreads), 0, st, P, adv, ret);
  UMAS_LAUNCHED("k_gae_scan");
  // The ranges cut inside long segments: persistent workgroups that wait for each other's maps.  At most one workgroup
  // per compute unit, far fewer than the device holds at once: whatever else is running, all of them get to run
  // together, so no workgroup waits for one that cannot start.
  void (*kernel_cut)(ScanParams, float*, float*) =
      value ? (decay ? k_gae_scan_cut<true, true> : k_gae_scan_cut<true, false>)
            : (decay ? k_gae_scan_cut<false, true> : k_gae_scan_cut<false, false>);
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    n_cu = 64;
  const unsigned nblk = static_cast<unsigned>(n_ranges < n_cu ? n_ranges : n_cu);
  hipLaunchKernelGGL(kernel_cut, dim3(nblk), dim3(kThreads), 0, st, P, adv, ret);
  UMAS_LAUNCHED("k_gae_scan_cut");
  return UMAS_OK;
}
