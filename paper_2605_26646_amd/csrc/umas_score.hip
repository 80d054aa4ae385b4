// LM-head scoring, the clipped PPO surrogate and the backward through the LM head.
//
// Scoring ("old log probabilities", paragraph "Advantage computation and policy evaluation"):
// for every selected row z = W h, lse = log sum exp z, logp = z[y] - lse, entropy = lse -
// sum softmax(z) z.  The bf16 path computes 256x256 logit tiles with MFMA and reduces each tile
// to per-row (max, sum exp, sum exp*z, taken logit) in registers; logits never leave the chip.
// Update (paragraph "Model-specific updates and synchronization", PPO after Schulman et al.
// 2017): ratio = exp(logp - logp_old), L = max(-A ratio, -A clip(ratio)), g = dL/dlogp, then
// dH = dz W and dW = dz^T H with dz = g (onehot - softmax) run as MFMA GEMMs over a bf16 operand
// [rows, vocabulary] held in a bounded chunk buffer; W and H are read as they lie (operands that are not
// K-contiguous go through transposing LDS reads), the one-hot part (one term per row) is added in float32.
// Without an entropy bonus the dense part of dz is a row factor times the softmax, so the scoring pass of
// the update itself leaves that operand behind: E = bf16(exp(z - z_y)), the softmax numerators relative to
// the taken token's logit, and the row factor -g exp(z_y - lse) is applied where dH is written and folded
// into the copy of H that dW reads; the logits are computed once.  With an entropy bonus (and for blocks
// of rows whose logits spread too far for E) dz is recomputed tile by tile from H, W and lse instead.
// The float32 path is a plain, unblocked implementation for small shapes.
#include <math.h>

#include <mutex>

#include "umas_common.h"
#include "umas_mfma.h"

namespace umas {
namespace {

using Cfg = TileCfg<256, 256, 2, 4>;   // 8 wavefronts, two per SIMD: one issues memory operations while the other feeds the matrix pipe
using Ring = Ring2Cfg<Cfg>;
constexpr int kLogitLds = Ring::LDS_BYTES > Cfg::LDS_BYTES ? Ring::LDS_BYTES : Cfg::LDS_BYTES;   // both main loops fit
constexpr int kGM = 4, kGN = 8;          // tile group resident on one XCD
constexpr int kTilesPerWg = 4;           // logit tiles a workgroup computes one after the other (short K: launch gaps and store drain overlap)
constexpr int kRowBlock = 256;
constexpr float kNegInf = -INFINITY;
constexpr float kMasked = -1e30f;        // stands for a logit that does not exist (vocabulary tail)

__device__ __forceinline__ uint16_t f2bf(float x) {
  return __builtin_bit_cast(uint16_t, static_cast<__bf16>(x));
}
// two floats rounded to bf16 in one word (first in the low half): one conversion instruction
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}
__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

// Online-softmax partial: m = max z, s = sum exp(z - m), t = sum exp(z - m) z.
struct Part {
  float m, s, t;
};
__device__ __forceinline__ Part part_merge(Part x, Part y) {
  if (x.m == kNegInf) return y;
  if (y.m == kNegInf) return x;
  const float M = fmaxf(x.m, y.m);
  const float ex = __expf(x.m - M), ey = __expf(y.m - M);
  return Part{M, x.s * ex + y.s * ey, x.t * ex + y.t * ey};
}

// ------------------------------------------------------------------ small helpers
__global__ void k_fill_u32(uint32_t* __restrict__ p, int64_t n, uint32_t v) {
  int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

hipError_t fill_bytes_zero(void* p, size_t bytes, hipStream_t st) {
  // bytes is a multiple of 4 for every buffer cleared here
  const int64_t n = static_cast<int64_t>(bytes / 4);
  if (n == 0) return hipSuccess;
  const unsigned grid = static_cast<unsigned>(n / 256 + 1 < 65536 ? n / 256 + 1 : 65536);
  hipLaunchKernelGGL(k_fill_u32, dim3(grid), dim3(256), 0, st, static_cast<uint32_t*>(p), n, 0u);
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess && g_prof_on) prof_kernel("k_fill_u32", st);
  return e;
}

// Logit tile Z[v, n] = W[m0 + v, :] . H[row(n0 + n), :] for a 256x256 block of (vocabulary, selected rows),
// row(n) = rowsel[sel0 + n] or sel0 + n.  Rows past V and past n_lim are clamped to valid ones; the
// callers mask what comes out of them.
template <class C>
__device__ __forceinline__ void logit_tile(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H, int d, int V,
                                           const int32_t* __restrict__ rowsel, int64_t sel0, int64_t n_lim, int m0,
                                           int64_t n0, uint16_t* lds, floatx4 (&acc)[C::MI][C::NI]) {
#pragma unroll
  for (int i = 0; i < C::MI; ++i)
#pragma unroll
    for (int j = 0; j < C::NI; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  if (d % C::BK == 0) {
    using R = Ring2Cfg<C>;
    const uint32_t kofs = ring2_kofs();
    uint32_t oa[R::NA], ob[R::NB];
#pragma unroll
    for (int i = 0; i < R::NA; ++i) oa[i] = (static_cast<uint32_t>(min(ring2_row<C>(i), V - 1 - m0)) * d + kofs) * 2u;
#pragma unroll
    for (int i = 0; i < R::NB; ++i) {
      const int64_t n = sel0 + min(n0 + ring2_row<C>(i), n_lim - 1);
      ob[i] = (static_cast<uint32_t>(rowsel ? rowsel[n] : n) * d + kofs) * 2u;   // host checks n_rows*d*2 < 2^32
    }
    mfma_mainloop_ring2<C>(make_rsrc(W + static_cast<int64_t>(m0) * d), oa, make_rsrc(H), ob, d, lds, acc);
  } else {
    const int kofs = slot_kofs();
    const uint16_t* pa[C::NA];
    const uint16_t* pb[C::NB];
#pragma unroll
    for (int i = 0; i < C::NA; ++i) pa[i] = W + static_cast<int64_t>(min(m0 + slot_row<C>(i), V - 1)) * d + kofs;
#pragma unroll
    for (int i = 0; i < C::NB; ++i) {
      const int64_t n = sel0 + min(n0 + slot_row<C>(i), n_lim - 1);
      pb[i] = H + static_cast<int64_t>(rowsel ? rowsel[n] : n) * d + kofs;
    }
    mfma_mainloop<C>(pa, pb, d, lds, acc);
  }
}

// ------------------------------------------------------------------ bf16: logit tiles -> partials
// A = W (vocabulary rows on the M side, so one lane sees many vocabulary entries of one token),
// B = rows c0 .. c0 + mc - 1 of the selection.  partial[tile_m][n] = (m, s, t, taken logit or 0).
//
// The keeping variant serves the backward pass when the dense part of dz is a row factor times the softmax
// (no entropy bonus): it also writes E[n, v] = bf16(exp(z[n, v] - c_n)) to the chunk buffer [mcp, Vp], c_n a
// per-row reference known before the pass (the taken token's logit), so that dz = (a_n exp(c_n - lse_n)) E
// needs no second pass over the logits: the row factor is applied where dH is written and folded into the
// copy of H that dW reads.  A block of 256 rows in which some logit exceeds its reference by more than kKeepMaxGap
// (E could overflow) is flagged and gets its dz from the recomputing kernel instead.
constexpr float kKeepMaxGap = 50.f;
// The [rows, vocabulary] operand of the backward (E, or dz on the recomputing path) lies in blocks of 256 rows x 256
// vocabulary entries, 128 KB each, row-major inside, vocabulary blocks of one block row next to each other: what a
// gradient tile reads per K step is then one run of memory (32 KB of consecutive rows for dW, four steps per block
// for dH) instead of 256 or 64 pieces a row pitch of 300 KB apart.
constexpr int64_t kBlkElems = 256 * 256;
__host__ __device__ __forceinline__ int64_t blk_offset(int64_t row_blk, int64_t voc_blk, int64_t tiles_v) {
  return (row_blk * tiles_v + voc_blk) * kBlkElems;
}
constexpr int kStagePitch = Cfg::WTM * 2 + 16;                                  // one staged row: 128 bf16, 16-byte aligned
constexpr int kStageBytes = Cfg::WM * Cfg::WN * Cfg::WTN * kStagePitch;         // every wavefront stages its block: 64 rows x 128 vocabulary entries
constexpr int kPartBytes = (Cfg::WM * Cfg::BN * 3 + Cfg::BN) * 4;
static_assert(kStageBytes + kPartBytes <= kLogitLds, "staging and the partials fit the tile buffers");
static_assert(kLogitLds <= 160 * 1024, "LDS of one CU");

struct KeepArgs {
  const float* cref;   // [n_pad] reference per selected row, NaN for rows without a valid id
  uint16_t* E;         // [mcp, Vp]
  int64_t Vp;
  int32_t* flags;      // per block of 256 selected rows
  const int32_t* cidx; // per block of 256 selected rows: its place among the chunk's live blocks, -1 for a dead one
};

template <bool KEEP>
__device__ __forceinline__ void score_tiles(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H, int d, int V,
                                            const int32_t* __restrict__ rowsel, int64_t c0, int64_t mc,
                                            const int32_t* __restrict__ ids, int tiles_m, int tiles_n,
                                            float4* __restrict__ partial, int64_t n_pad, const KeepArgs& keep,
                                            uint16_t* lds) {
  using C = Cfg;
  for (int it = 0; it < kTilesPerWg; ++it) {     // a workgroup walks the same place of kTilesPerWg consecutive tile groups
  int tile_m, tile_n;
  if (!tile_coords<kGM, kGN>(tiles_m, tiles_n, &tile_m, &tile_n, it, kTilesPerWg)) continue;
  const int m0 = tile_m * C::BM;
  const int64_t n0 = static_cast<int64_t>(tile_n) * C::BN;   // chunk-relative
  floatx4 acc[C::MI][C::NI];
  logit_tile<C>(W, H, d, V, rowsel, c0, mc, m0, n0, lds, acc);

  // epilogue: the tile buffers are free now.  A lane holds, for each of its NI columns (selected rows), the
  // vocabulary entries vbase + 16 i + r (i < MI, r < 4); the four lanes l, l + 16, l + 32, l + 48 share a column.
  float* s_part = reinterpret_cast<float*>(reinterpret_cast<char*>(lds) + (KEEP ? kStageBytes : 0));   // [WM][BN][3], behind the staging area
  float* s_zy = s_part + C::WM * C::BN * 3;               // [BN]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN;
  char* stage = reinterpret_cast<char*>(lds) + wave * (C::WTN * kStagePitch);
  if (threadIdx.x < C::BN) s_zy[threadIdx.x] = 0.f;
  __syncthreads();                                        // every wavefront has left the main loop's LDS reads
  const int vbase = m0 + wm * C::WTM + (lane >> 4) * 4;   // vocabulary id of element (i = 0, r = 0)
  const bool tail = m0 + C::BM > V;
  if (tail) {   // vocabulary ids past V: a large negative logit whose exponential is 0 and whose products stay finite
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
      for (int j = 0; j < C::NI; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (vbase + i * 16 + r >= V) acc[i][j][r] = kMasked;
  }
  constexpr float kLog2e = 1.44269504088896341f;
  bool over = false;
  // a block of rows none of which has a gradient (all advantages 0) keeps nothing: the backward never looks at it
  const int out_blk = KEEP ? keep.cidx[(c0 >> 8) + tile_n] : -1;
  const bool keeping = KEEP && out_blk >= 0;
#pragma unroll
  for (int j = 0; j < C::NI; ++j) {
    const int col = acc_col<C>(j);
    const int64_t n = n0 + col;
    // exponentials of this lane's entries of column j relative to m (log2 domain), their sum s and sum of e z; the
    // keeping variant stages them as bf16 in this wavefront's LDS region, stored in full lines below
    float m = kMasked, s = 0.f, t = 0.f;
    auto column = [&](float ref, auto premultiplied) {
      const float r2 = ref * kLog2e;
      s = 0.f;
      t = 0.f;
#pragma unroll
      for (int i = 0; i < C::MI; ++i) {
        float e[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float z = acc[i][j][r];
          // without a reference from outside: z - m first, exact 0 where a lane holds nothing but vocabulary tail
          e[r] = decltype(premultiplied)::value ? __builtin_amdgcn_exp2f(fmaf(z, kLog2e, -r2)) : __builtin_amdgcn_exp2f((z - ref) * kLog2e);
          s += e[r];
          t = fmaf(e[r], z, t);
        }
        if (keeping) {
          const uint32_t p01 = pack_bf16x2(e[0], e[1]), p23 = pack_bf16x2(e[2], e[3]);
          *reinterpret_cast<uint2*>(stage + (j * 16 + (lane & 15)) * kStagePitch + (i * 16 + (lane >> 4) * 4) * 2) =
              make_uint2(p01, p23);
        }
      }
    };
    auto lane_max = [&]() {
      float mx = kMasked;
#pragma unroll
      for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) mx = fmaxf(mx, acc[i][j][r]);
      return mx;
    };
    if (keeping) {
      // The keeping variant sums relative to the row's reference c_n instead of the lane's maximum (any reference
      // serves the merge as long as nothing overflows), so the exponentials it sums are the numerators it keeps,
      // and it does not look for the maximum first: a sum beyond 32 e^kKeepMaxGap (or not a number: rows without
      // a valid id have the reference NaN) shows afterwards that some logit may lie more than kKeepMaxGap above
      // c_n.  Only then is the column done again the long way, relative to the lane's maximum: a lane whose maximum
      // does lie that far above c_n flags the block (its dz is recomputed later); rows without a valid id flag
      // nothing, their row factor is 0.
      const float c = n < mc ? keep.cref[c0 + n] : 1e30f;   // rows past the chunk: every exponential is 0, E = 0
      m = c;
      column(c, std::true_type{});
      constexpr float kSumLimit = 1.6e23f;                   // 32 e^50 = 1.66e23
      if (!(s < kSumLimit)) {
        m = lane_max();
        const float gap = m - c;
        over |= gap > kKeepMaxGap;
        if (gap <= kKeepMaxGap) m = c;                       // many large terms, none too large: c serves after all
        else if (m == kMasked) m = 0.f;                     // nothing but vocabulary tail in this lane: exponentials 0 as well
        column(m, std::true_type{});
      }
    } else {
      m = lane_max();
      column(m, std::false_type{});
    }
    Part p{m, s, t};
#pragma unroll
    for (int o = 16; o < kWave; o <<= 1) {
      const Part q{__shfl_xor(p.m, o, kWave), __shfl_xor(p.s, o, kWave), __shfl_xor(p.t, o, kWave)};
      p = part_merge(p, q);
    }
    if (lane < 16) {
      float* dst = s_part + (wm * C::BN + col) * 3;
      dst[0] = p.m; dst[1] = p.s; dst[2] = p.t;
    }
    if (!KEEP && n < mc) {                                  // the keeping variant got the taken logits beforehand
      const int y = ids[rowsel ? rowsel[c0 + n] : c0 + n];
      const int rel = y - vbase;                           // offset from this lane's first element
      if (y >= 0 && y < V && rel >= 0 && rel < C::WTM && (rel & 12) == 0) {
        float zy = 0.f;
#pragma unroll
        for (int i = 0; i < C::MI; ++i)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (i * 16 + r == rel) zy = acc[i][j][r];
        s_zy[col] = zy;
      }
    }
  }
  if (keeping) {
    if (over) keep.flags[(c0 >> 8) + tile_n] = 1;
    // the staged block goes out 16 bytes per lane: one instruction covers 4 rows x 256 contiguous bytes
    const int wn = wave % C::WN;
    uint16_t* out = keep.E + blk_offset(out_blk, tile_m, keep.Vp >> 8) + (wn * C::WTN) * 256 + wm * C::WTM + (lane & 15) * 8;
#pragma unroll 8
    for (int i = 0; i < C::WTN / 4; ++i) {
      const int row = i * 4 + (lane >> 4);
      const uint4 v = *reinterpret_cast<const uint4*>(stage + row * kStagePitch + (lane & 15) * 16);
      typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
      __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4*>(out + row * 256));
    }
  }
  __syncthreads();
  if (threadIdx.x < C::BN) {
    const int col = threadIdx.x;
    Part p{kNegInf, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < C::WM; ++w) {
      const float* src = s_part + (w * C::BN + col) * 3;
      p = part_merge(p, Part{src[0], src[1], src[2]});
    }
    if (c0 + n0 + col < n_pad) partial[static_cast<int64_t>(tile_m) * n_pad + c0 + n0 + col] = make_float4(p.m, p.s, p.t, s_zy[col]);
  }
  __syncthreads();                              // the LDS is the next tile's again
  }
}

// (kernel templates whose bodies use buffer resources do not get their host stubs emitted: plain kernels)
__global__ void __launch_bounds__(Cfg::T)
k_score_tiles(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H, int d, int V,
              const int32_t* __restrict__ rowsel, int64_t n_sel, const int32_t* __restrict__ ids,
              int tiles_m, int tiles_n, float4* __restrict__ partial, int64_t n_pad) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[kLogitLds / 2];
  score_tiles<false>(W, H, d, V, rowsel, 0, n_sel, ids, tiles_m, tiles_n, partial, n_pad, KeepArgs{}, lds);
}
__global__ void __launch_bounds__(Cfg::T)
k_score_keep_tiles(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H, int d, int V,
                   const int32_t* __restrict__ rowsel, int64_t c0, int64_t mc, const int32_t* __restrict__ ids,
                   int tiles_m, int tiles_n, float4* __restrict__ partial, int64_t n_pad,
                   const float* __restrict__ cref, uint16_t* __restrict__ E, int64_t Vp, int32_t* __restrict__ flags,
                   const int32_t* __restrict__ cidx) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[kLogitLds / 2];
  score_tiles<true>(W, H, d, V, rowsel, c0, mc, ids, tiles_m, tiles_n, partial, n_pad, KeepArgs{cref, E, Vp, flags, cidx}, lds);
}

// Merge the per-tile partials of each selected row; compact results and optional scatter.  Eight lanes
// share a row (lane = 8 * part + row within the group of 8 rows, so a load still covers whole 128-byte lines).
constexpr int kFinParts = 8;
__global__ void __launch_bounds__(256)
k_score_finalize(const float4* __restrict__ partial, int tiles_m, int64_t n_pad, int64_t n_begin,
                 int64_t n_end, const float* __restrict__ zy_c, const int32_t* __restrict__ rowsel,
                 const int32_t* __restrict__ ids, int V,
                 float* __restrict__ logp_c, float* __restrict__ lse_c, float* __restrict__ ent_c,
                 float* __restrict__ logp, float* __restrict__ lse, float* __restrict__ entropy) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int part = lane >> 3;
  const int64_t n = n_begin + (static_cast<int64_t>(blockIdx.x) * (blockDim.x / kWave) + wave) * 8 + (lane & 7);
  const bool live = n < n_end;                                // whole groups of lanes; the shuffles below need every lane
  Part p{kNegInf, 0.f, 0.f};
  float zy = 0.f;
  if (live) {
    for (int tm = part; tm < tiles_m; tm += kFinParts) {
      const float4 q = partial[static_cast<int64_t>(tm) * n_pad + n];
      p = part_merge(p, Part{q.x, q.y, q.z});
      zy += q.w;
    }
  }
#pragma unroll
  for (int o = 8; o < kWave; o <<= 1) {
    const Part q{__shfl_xor(p.m, o, kWave), __shfl_xor(p.s, o, kWave), __shfl_xor(p.t, o, kWave)};
    p = part_merge(p, q);
    zy += __shfl_xor(zy, o, kWave);
  }
  if (!live || part != 0) return;
  if (zy_c) zy = zy_c[n];                                   // taken logits computed beforehand
  const int64_t row = rowsel ? rowsel[n] : n;
  const int y = ids[row];
  const bool ok = y >= 0 && y < V;
  const float l = p.m + logf(p.s);
  const float lp = ok ? zy - l : 0.f;
  const float en = ok ? l - p.t / p.s : 0.f;
  if (logp_c) { logp_c[n] = lp; lse_c[n] = l; ent_c[n] = en; }
  if (logp) logp[row] = lp;
  if (lse) lse[row] = l;
  if (entropy) entropy[row] = en;
}

// ------------------------------------------------------------------ float32: plain scoring
// One block per selected row; every thread walks vocabulary entries v = tid, tid + T, ...  The float32 path is the
// plain one for small shapes: its speed does not matter, so dot products and softmax statistics are carried in
// float64 and only the results are rounded to float32 (a float32 dot product of d terms would cost up to
// d 2^-24 of the sum of its terms' magnitudes).
struct PartD {
  double m, s, t;
};
__device__ __forceinline__ PartD partd_merge(PartD x, PartD y) {
  if (x.s == 0.0) return y;
  if (y.s == 0.0) return x;
  const double M = fmax(x.m, y.m);
  const double ex = exp(x.m - M), ey = exp(y.m - M);
  return PartD{M, x.s * ex + y.s * ey, x.t * ex + y.t * ey};
}
__device__ __forceinline__ double dot_f64(const float* __restrict__ a, const float* __restrict__ b, int d) {
  double z = 0.0;
  for (int k = 0; k < d; ++k) z = fma(static_cast<double>(a[k]), static_cast<double>(b[k]), z);
  return z;
}
__global__ void __launch_bounds__(256)
k_score_f32(const float* __restrict__ W, const float* __restrict__ H, int d, int V,
            const int32_t* __restrict__ rowsel, const int32_t* __restrict__ ids,
            float* __restrict__ logp_c, float* __restrict__ lse_c, float* __restrict__ ent_c,
            float* __restrict__ logp, float* __restrict__ lse, float* __restrict__ entropy) {
  extern __shared__ float s_h[];   // [d]
  __shared__ double s_m[4], s_s[4], s_t[4], s_zy;
  const int64_t n = blockIdx.x;
  const int64_t row = rowsel ? rowsel[n] : n;
  for (int k = threadIdx.x; k < d; k += blockDim.x) s_h[k] = H[row * d + k];
  if (threadIdx.x == 0) s_zy = 0.0;
  __syncthreads();
  const int y = ids[row];
  PartD p{0.0, 0.0, 0.0};
  for (int v = threadIdx.x; v < V; v += blockDim.x) {
    const double z = dot_f64(s_h, W + static_cast<int64_t>(v) * d, d);
    if (v == y) s_zy = z;
    p = partd_merge(p, PartD{z, 1.0, z});
  }
  // merge over the block: lanes, then wavefronts
  for (int o = 32; o > 0; o >>= 1) {
    PartD q{__shfl_xor(p.m, o, kWave), __shfl_xor(p.s, o, kWave), __shfl_xor(p.t, o, kWave)};
    p = partd_merge(p, q);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) { s_m[wave] = p.m; s_s[wave] = p.s; s_t[wave] = p.t; }
  __syncthreads();
  if (threadIdx.x == 0) {
    PartD a{0.0, 0.0, 0.0};
    for (int w = 0; w < 4; ++w) a = partd_merge(a, PartD{s_m[w], s_s[w], s_t[w]});
    const bool ok = y >= 0 && y < V;
    const double l = a.m + log(a.s);
    const float lf = static_cast<float>(l);
    const float lp = ok ? static_cast<float>(s_zy - l) : 0.f;
    const float en = ok ? static_cast<float>(l - a.t / a.s) : 0.f;
    if (logp_c) { logp_c[n] = lp; lse_c[n] = lf; ent_c[n] = en; }
    if (logp) logp[row] = lp;
    if (lse) lse[row] = lf;
    if (entropy) entropy[row] = en;
  }
}

// ------------------------------------------------------------------ clipped surrogate
// Per selected row: loss term (single clip, or dual clip when dual_clip > 1) and g = dloss/dlogp of the
// clipped part; per block sums of (L, clipped, entropy,
// logp_old - logp, rows, invalid ids) for the model and for each role, in float64.
constexpr int kStat = 6;
__global__ void __launch_bounds__(kRowBlock)
k_ppo_rows(int64_t norm, int64_t n_begin, int64_t n_end, const int32_t* __restrict__ rowsel, const int32_t* __restrict__ ids, int V,
           const float* __restrict__ logp_c, const float* __restrict__ ent_c, const float* __restrict__ logp_old,
           const float* __restrict__ adv, const int32_t* __restrict__ tok_role, int n_roles, float clip_eps,
           float dual_clip, float k_ent, const float* __restrict__ logp_ref, float kl_coef, int label_apart,
           const float* __restrict__ lse_c, float* __restrict__ g_c,
           float* __restrict__ a_c, float* __restrict__ kz_c, double* __restrict__ blk_stats) {
  extern __shared__ double s_acc[];   // [(1+n_roles) * kStat]
  const int nacc = (1 + n_roles) * kStat;
  for (int i = threadIdx.x; i < nacc; i += blockDim.x) s_acc[i] = 0.0;
  __syncthreads();
  const int64_t n = n_begin + static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;   // n_begin is a multiple of the block size
  if (n < n_end) {
    const int64_t row = rowsel ? rowsel[n] : n;
    const int y = ids[row];
    const bool ok = y >= 0 && y < V;
    float L = 0.f, g = 0.f, clipped = 0.f, en = 0.f, kl = 0.f, lp = 0.f;
    if (ok) {
      lp = logp_c[n];
      const float lo = logp_old ? logp_old[row] : lp, A = adv[row];   // no old log-probs: the update is on-policy, ratio 1
      const float ratio = __expf(lp - lo);
      const float u = -A * ratio;
      const float c = -A * fminf(fmaxf(ratio, 1.f - clip_eps), 1.f + clip_eps);
      bool unclipped = u >= c;
      L = unclipped ? u : c;
      if (dual_clip > 0.f && A < 0.f && -A * dual_clip < L) {   // dual clip: the term of a negative advantage is capped
        L = -A * dual_clip;
        unclipped = false;
      }
      g = unclipped ? u / static_cast<float>(norm) : 0.f;
      clipped = unclipped ? 0.f : 1.f;
      if (kl_coef != 0.f) {   // penalty towards the reference policy: kl_coef (e^x - x - 1), x = logp_ref - logp
        const float x = logp_ref[row] - lp, ex = __expf(x);
        L += kl_coef * (ex - x - 1.f);
        g += kl_coef * (1.f - ex) / static_cast<float>(norm);
      }
      en = ent_c[n];
      kl = lo - lp;
    }
    // With label_apart the taken token's column is left out of the dense (bf16) part of dz and g_c carries all of
    // dz[n, y] = g (1 - p_y) + k_ent p_y (log p_y + entropy) in float32: for a confident token g and g p_y nearly
    // cancel, and the rounding of a bf16 g p_y would be as large as what is left.
    g_c[n] = label_apart && ok ? fmaf(g, -expm1f(lp), k_ent * __expf(lp) * (lp + en)) : g;
    // coefficients of the backward's dense part dz = p (a + kz z): -g from the surrogate, the rest from the
    // entropy bonus k_ent p (log p + entropy); a row with an invalid id has neither
    a_c[n] = ok ? -g + k_ent * (en - lse_c[n]) : 0.f;
    kz_c[n] = ok ? k_ent : 0.f;
    const int role = (tok_role && n_roles > 0) ? tok_role[row] : -1;
    for (int pass = 0; pass < 2; ++pass) {
      if (pass == 1 && (role < 0 || role >= n_roles)) break;
      double* a = s_acc + (pass == 0 ? 0 : (1 + role) * kStat);
      atomicAdd(a + 0, static_cast<double>(L));
      atomicAdd(a + 1, static_cast<double>(clipped));
      atomicAdd(a + 2, static_cast<double>(en));
      atomicAdd(a + 3, static_cast<double>(kl));
      atomicAdd(a + 4, 1.0);
      atomicAdd(a + 5, ok ? 0.0 : 1.0);
    }
  }
  __syncthreads();
  const int64_t blk = n_begin / kRowBlock + blockIdx.x;
  for (int i = threadIdx.x; i < nacc; i += blockDim.x) blk_stats[blk * nacc + i] = s_acc[i];
}

__global__ void __launch_bounds__(256)
k_ppo_stats(int nblk, int n_roles, float entropy_coef, int64_t norm_rows, const double* __restrict__ blk_stats,
            umas_loss_stats* __restrict__ stats) {
  __shared__ double smem[32];
  const int nacc = (1 + n_roles) * kStat;
  for (int k = 0; k <= n_roles; ++k) {
    double sum[kStat];
    for (int j = 0; j < kStat; ++j) {
      double v = 0.0;
      for (int b = threadIdx.x; b < nblk; b += blockDim.x) v += blk_stats[static_cast<int64_t>(b) * nacc + k * kStat + j];
      sum[j] = block_sum<double>(v, smem);
    }
    if (threadIdx.x == 0) {
      const double cnt = sum[4];
      umas_loss_stats s;
      // the model's loss over the caller's normaliser when one is given: micro-batch losses then add up
      const double den = (k == 0 && norm_rows > 0) ? static_cast<double>(norm_rows) : cnt;
      s.loss = cnt > 0 ? static_cast<float>((sum[0] - static_cast<double>(entropy_coef) * sum[2]) / den) : 0.f;
      s.clip_frac = cnt > 0 ? static_cast<float>(sum[1] / cnt) : 0.f;
      s.entropy_mean = cnt > 0 ? static_cast<float>(sum[2] / cnt) : 0.f;
      s.approx_kl = cnt > 0 ? static_cast<float>(sum[3] / cnt) : 0.f;
      s.n_scored = static_cast<int64_t>(cnt);
      s.n_invalid_ids = static_cast<int64_t>(sum[5]);
      stats[k] = s;
    }
  }
}

// ------------------------------------------------------------------ bf16: blocks of rows that have a gradient
// A selected row whose advantage is 0 has g = 0 and (without an entropy bonus or a KL term) no gradient at all; group-normalised
// outcome rewards make whole trajectory groups such rows.  The keeping pass therefore works on the chunk's live blocks
// of 256 selected rows only: E and the scaled copy of H hold them packed, dH has as many row tiles and dW as many K
// steps as there are, and everything that depends on their number is worked out on the device.
struct LiveInfo {
  int32_t n_live;        // live blocks of the chunk
  int32_t k_rows;        // rows of the packed operands that exist (the chunk's last block may be partly filled)
  XcdGroups dw_groups;   // dW tile groups per XCD (see share_dw_groups)
};
__global__ void __launch_bounds__(256)
k_live_flags(int64_t n_sel, const int32_t* __restrict__ rowsel, const float* __restrict__ adv, int32_t* __restrict__ blk_live) {
  const int64_t n = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int live = n < n_sel && adv[rowsel ? rowsel[n] : n] != 0.f;
  const int any = __syncthreads_or(live);
  if (threadIdx.x == 0) blk_live[blockIdx.x] = any;
}
// Shares of the dW tile groups per XCD for k_gemm_dh_dw: every XCD first works through its dH groups (contiguous
// ranges, as tile_coords hands them out; a group costs about Vp K-steps per tile), then dW groups (k_len K-steps per
// tile) go to the XCDs so that all finish as evenly as whole groups allow, at most max_groups to one XCD (the grid has
// no more; 8 max_groups cover all groups).
__device__ void share_dw_groups(int tiles_r, int tiles_v, int tiles_d, int64_t Vp, int64_t k_len, int max_groups, XcdGroups* out) {
  const int64_t groups_dh = static_cast<int64_t>((tiles_r + kGM - 1) / kGM) * ((tiles_d + kGN - 1) / kGN);
  const int64_t per_xcd = (groups_dh + 7) / 8;
  int64_t load[8];
  int cnt[8] = {};
  for (int x = 0; x < 8; ++x) {
    int64_t n = groups_dh - x * per_xcd;
    n = n < 0 ? 0 : (n > per_xcd ? per_xcd : n);
    load[x] = n * Vp;
  }
  const int64_t groups_dw = static_cast<int64_t>((tiles_v + kGM - 1) / kGM) * ((tiles_d + kGN - 1) / kGN);
  if (k_len <= 0) {                                    // nothing to even out
    for (int x = 0; x < 8; ++x) cnt[x] = static_cast<int>(groups_dw / 8 + (x < groups_dw % 8 ? 1 : 0));
  } else {
    // the lowest level T up to which the XCDs can be filled with whole groups so that all groups are placed ...
    auto take = [&](int x, int64_t T) {
      // (a double quotient: the operands stay far below 2^53 and 64-bit integer division is slow here)
      const int64_t n = T > load[x] ? static_cast<int64_t>(static_cast<double>(T - load[x]) / static_cast<double>(k_len)) : 0;
      return static_cast<int>(n < max_groups ? n : max_groups);
    };
    int64_t lo = load[0], hi = load[0];
    for (int x = 1; x < 8; ++x) { lo = load[x] < lo ? load[x] : lo; hi = load[x] > hi ? load[x] : hi; }
    hi += groups_dw * k_len;
    while (lo < hi) {
      const int64_t mid = lo + (hi - lo) / 2;
      int64_t sum = 0;
      for (int x = 0; x < 8; ++x) sum += take(x, mid);
      if (sum >= groups_dw) hi = mid; else lo = mid + 1;
    }
    int64_t total = 0;
    for (int x = 0; x < 8; ++x) { cnt[x] = take(x, lo); total += cnt[x]; }
    // ... and the few groups too many at that level come off the XCDs that would finish last
    for (; total > groups_dw; --total) {
      int worst = -1;
      for (int x = 0; x < 8; ++x)
        if (cnt[x] > 0 && (worst < 0 || load[x] + cnt[x] * k_len > load[worst] + cnt[worst] * k_len)) worst = x;
      --cnt[worst];
    }
  }
  out->first[0] = 0;
  for (int x = 0; x < 8; ++x) out->first[x + 1] = out->first[x] + cnt[x];
}
inline int max_dw_groups_per_xcd(int tiles_v, int tiles_d) {   // 8 x this many cover every group with room to even out
  const int64_t groups_dw = static_cast<int64_t>((tiles_v + kGM - 1) / kGM) * ((tiles_d + kGN - 1) / kGN);
  return static_cast<int>((groups_dw + 7) / 8 + 20);
}
// One workgroup per chunk: packs the live blocks (all of them with all_live), blk0 = first block of the chunk.
__global__ void __launch_bounds__(512)
k_live_scan(int blk0, int nblk, int64_t rows, int all_live, int tiles_v, int tiles_d, int64_t Vp, int max_groups,
            const int32_t* __restrict__ blk_live, int32_t* __restrict__ blk_cidx, int32_t* __restrict__ blk_orig,
            LiveInfo* __restrict__ info) {
  __shared__ int smem[32];
  const int t = threadIdx.x;
  const int live = t < nblk && (all_live || blk_live[blk0 + t]);
  int total;
  const int pos = block_excl_scan<int>(live, smem, &total);
  if (t < nblk) {
    blk_cidx[blk0 + t] = live ? pos : -1;
    if (live) blk_orig[blk0 + pos] = t;
  }
  __shared__ int s_last_live;
  if (t == nblk - 1) s_last_live = live;
  __syncthreads();
  if (t == 0) {
    info->n_live = total;
    const int64_t last_rows = rows - static_cast<int64_t>(nblk - 1) * 256;     // rows of the chunk's last block
    info->k_rows = static_cast<int32_t>(s_last_live ? static_cast<int64_t>(total - 1) * 256 + last_rows : static_cast<int64_t>(total) * 256);
    share_dw_groups(total, tiles_v, tiles_d, Vp, static_cast<int64_t>(total) * 256, max_groups, &info->dw_groups);
  }
}

// ------------------------------------------------------------------ bf16: row references and row factors of the keeping pass
__device__ __forceinline__ void bf16x8_to_f32(const uint4 v, float (&o)[8]) {
  o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
  o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
  o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
  o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
}
// cref[n] = h_n . W[y_n], the taken token's logit (never above the row's logsumexp); NaN for an invalid id.
// One wavefront per selected row.
__global__ void __launch_bounds__(256)
k_label_logit(const uint16_t* __restrict__ H, const uint16_t* __restrict__ W, int d, int V,
              const int32_t* __restrict__ rowsel, int64_t n_sel, const int32_t* __restrict__ ids,
              float* __restrict__ cref) {
  const int lane = threadIdx.x & 63;
  const int64_t n = static_cast<int64_t>(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (n >= n_sel) return;
  const int64_t row = rowsel ? rowsel[n] : n;
  const int y = ids[row];
  if (y < 0 || y >= V) {
    if (lane == 0) cref[n] = NAN;
    return;
  }
  const uint4* h = reinterpret_cast<const uint4*>(H + row * d);
  const uint4* w = reinterpret_cast<const uint4*>(W + static_cast<int64_t>(y) * d);
  float s = 0.f;
  for (int k = lane; k < d / 8; k += kWave) {
    float a[8], b[8];
    bf16x8_to_f32(h[k], a);
    bf16x8_to_f32(w[k], b);
#pragma unroll
    for (int j = 0; j < 8; ++j) s = fmaf(a[j], b[j], s);
  }
  s = wave_sum(s);
  if (lane == 0) cref[n] = s;
}
// Row factor sc[n] = a_n exp(c_n - lse_n) of dz = sc E, and Hs[n - c0, :] = bf16(sc[n] h_n), the operand dW reads, in
// column blocks [d / 256][mcp][256].
// Rows of a flagged block get factor 1: their dz comes complete from the recomputing kernel.  The entry of the
// taken token is cleared in the [rows, V] operand (see k_ppo_rows).
__global__ void __launch_bounds__(256)
k_keep_rows(const uint16_t* __restrict__ H, int d, int V, const int32_t* __restrict__ rowsel, int64_t c0, int64_t rows,
            const int32_t* __restrict__ ids, uint16_t* __restrict__ E, int64_t tiles_v, const float* __restrict__ lse_c,
            const float* __restrict__ a_c,
            const float* __restrict__ cref, const int32_t* __restrict__ flags, const int32_t* __restrict__ cidx,
            float* __restrict__ sc, uint16_t* __restrict__ Hs, int64_t mcp) {
  const int lane = threadIdx.x & 63;
  const int64_t m = static_cast<int64_t>(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (m >= rows) return;
  const int64_t n = c0 + m;
  const int64_t row = rowsel ? rowsel[n] : n;
  const float a = a_c[n];
  const int blk = cidx[n >> 8];                              // place of the row's block among the live ones
  if (blk < 0) {                                             // a dead block: no row of it has a gradient
    if (lane == 0) sc[n] = 0.f;
    return;
  }
  const int64_t mp = static_cast<int64_t>(blk) * 256 + (m & 255);   // row in the packed operands
  const int y = ids[row];
  if (lane == 0 && y >= 0 && y < V)                          // the taken token's column goes through g_c in float32
    E[blk_offset(blk, y >> 8, tiles_v) + (m & 255) * 256 + (y & 255)] = 0;
  float f = 1.f;
  if (!flags[n >> 8]) f = a != 0.f ? a * __expf(cref[n] - lse_c[n]) : 0.f;   // a = 0: invalid id (reference NaN) or no gradient
  if (lane == 0) sc[n] = f;
  const uint4* h = reinterpret_cast<const uint4*>(H + row * d);
  for (int k = lane; k < d / 8; k += kWave) {
    uint4* o = reinterpret_cast<uint4*>(Hs + (static_cast<int64_t>(k >> 5) * mcp + mp) * 256);   // column block k / 32 of the row
    float x[8];
    bf16x8_to_f32(h[k], x);
    uint4 v;
    v.x = pack_bf16x2(x[0] * f, x[1] * f);
    v.y = pack_bf16x2(x[2] * f, x[3] * f);
    v.z = pack_bf16x2(x[4] * f, x[5] * f);
    v.w = pack_bf16x2(x[6] * f, x[7] * f);
    o[k & 31] = v;
  }
}

// ------------------------------------------------------------------ bf16: dz tiles into the chunk buffer
// Same tile product as k_score_tiles; the epilogue forms the dense part of dz = g (onehot - softmax),
// -g exp(z - lse), plus the entropy bonus's term when its coefficient is not 0, and writes it as bf16 to
// dZ [mcp, Vp].  Rows past the chunk and vocabulary ids past V get 0.  The one-hot part g at v = y is a single term per row and is added in
// float32 where dH and dW are written, so that it never meets the bf16 rounding of the dense part.
__device__ __forceinline__ void dz_tile(int tile_m, int tile_n, const uint16_t* __restrict__ W, const uint16_t* __restrict__ H,
                                        int d, int V, const int32_t* __restrict__ rowsel, int64_t c0, int64_t mc,
                                        const float* __restrict__ lse_c, const float* __restrict__ a_c,
                                        const float* __restrict__ kz_c, uint16_t* __restrict__ dZ, int64_t Vp, int out_blk,
                                        uint16_t* lds) {
  using C = Cfg;
  const int m0 = tile_m * C::BM;
  const int64_t n0 = static_cast<int64_t>(tile_n) * C::BN;   // chunk-relative
  floatx4 acc[C::MI][C::NI];
  logit_tile<C>(W, H, d, V, rowsel, c0, mc, m0, n0, lds, acc);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN;
  const int vbase = m0 + wm * C::WTM + (lane >> 4) * 4;
  const bool tail = m0 + C::BM > V;
  // each wavefront stages its 64 (rows) x 128 (vocabulary) block; the 272-byte pitch keeps 16-byte alignment
  char* stage = reinterpret_cast<char*>(lds) + wave * (C::WTN * kStagePitch);
  __syncthreads();                              // every wavefront has left the main loop's LDS reads
  if (tail) {                                   // vocabulary ids past V: the exponential below is 0, the factor next to it finite
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
      for (int j = 0; j < C::NI; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (vbase + i * 16 + r >= V) acc[i][j][r] = kMasked;
  }
#pragma unroll
  for (int j = 0; j < C::NI; ++j) {
    const int64_t n = n0 + acc_col<C>(j);
    // dz = p (a + kz z) with p = exp(z - lse), a = -g + k (entropy - lse), kz = k = entropy_coef / n_sel: the
    // dense part of g (onehot - p) plus the entropy bonus's k p (log p + entropy).  Rows past the chunk: p = 0.
    float l2 = 1e30f, a = 0.f, kz = 0.f;
    if (n < mc) {
      l2 = lse_c[c0 + n] * 1.44269504088896341f;
      a = a_c[c0 + n];
      kz = kz_c[c0 + n];
    }
#pragma unroll
    for (int i = 0; i < C::MI; ++i) {
      float dz[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float z = acc[i][j][r];
        dz[r] = __builtin_amdgcn_exp2f(fmaf(z, 1.44269504088896341f, -l2)) * fmaf(kz, z, a);
      }
      const uint32_t p01 = pack_bf16x2(dz[0], dz[1]), p23 = pack_bf16x2(dz[2], dz[3]);
      // staged in this wavefront's LDS region, stored in full lines below
      *reinterpret_cast<uint2*>(stage + (j * 16 + (lane & 15)) * kStagePitch + (i * 16 + (lane >> 4) * 4) * 2) =
          make_uint2(p01, p23);
    }
  }
  // the staged block goes out 16 bytes per lane: one instruction covers 4 rows x 256 contiguous bytes
  const int wn = wave % C::WN;
  uint16_t* out = dZ + blk_offset(out_blk, tile_m, Vp >> 8) + (wn * C::WTN) * 256 + wm * C::WTM + (lane & 15) * 8;
#pragma unroll 8
  for (int i = 0; i < C::WTN / 4; ++i) {
    const int row = i * 4 + (lane >> 4);
    const uint4 v = *reinterpret_cast<const uint4*>(stage + row * kStagePitch + (lane & 15) * 16);
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4*>(out + row * 256));
  }
  __syncthreads();                              // the LDS is the next tile's again
}
__global__ void __launch_bounds__(Cfg::T)
k_dz_tiles(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H, int d, int V,
           const int32_t* __restrict__ rowsel, int64_t c0, int64_t mc,
           const float* __restrict__ lse_c, const float* __restrict__ a_c, const float* __restrict__ kz_c,
           int tiles_m, int tiles_n, uint16_t* __restrict__ dZ, int64_t Vp) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[kLogitLds / 2];
  for (int it = 0; it < kTilesPerWg; ++it) {     // a workgroup walks the same place of kTilesPerWg consecutive tile groups
    int tile_m, tile_n;
    if (!tile_coords<kGM, kGN>(tiles_m, tiles_n, &tile_m, &tile_n, it, kTilesPerWg)) continue;
    dz_tile(tile_m, tile_n, W, H, d, V, rowsel, c0, mc, lse_c, a_c, kz_c, dZ, Vp, tile_n, lds);
  }
}
// The same tiles for the blocks of 256 rows that the keeping scoring pass has flagged, and only those: a fixed,
// small grid walks (flagged block, vocabulary tile) pairs, so that the usual case of no flag costs next to nothing.
constexpr int kFlaggedGrid = 256;
__global__ void __launch_bounds__(Cfg::T)
k_dz_flagged(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H, int d, int V,
             const int32_t* __restrict__ rowsel, int64_t c0, int64_t mc,
             const float* __restrict__ lse_c, const float* __restrict__ a_c, const float* __restrict__ kz_c,
             int tiles_m, int tiles_n, uint16_t* __restrict__ dZ, int64_t Vp, const int32_t* __restrict__ flags,
             const int32_t* __restrict__ cidx) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[kLogitLds / 2];
  for (int tile_n = 0; tile_n < tiles_n; ++tile_n) {
    const int out_blk = cidx[(c0 >> 8) + tile_n];
    if (!flags[(c0 >> 8) + tile_n] || out_blk < 0) continue;        // the same for every thread of the grid
    for (int tile_m = blockIdx.x; tile_m < tiles_m; tile_m += gridDim.x)
      dz_tile(tile_m, tile_n, W, H, d, V, rowsel, c0, mc, lse_c, a_c, kz_c, dZ, Vp, out_blk, lds);
  }
}

// The taken token's entry of every row of the chunk's blocked dZ is cleared: that column goes through g_c in float32
// (see k_ppo_rows).  One thread per row.
__global__ void __launch_bounds__(256)
k_zero_label(uint16_t* __restrict__ dZ, int64_t tiles_v, int V, const int32_t* __restrict__ rowsel, int64_t c0, int64_t rows,
             const int32_t* __restrict__ ids) {
  const int64_t m = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (m >= rows) return;
  const int y = ids[rowsel ? rowsel[c0 + m] : c0 + m];
  if (y >= 0 && y < V) dZ[blk_offset(m >> 8, y >> 8, tiles_v) + (m & 255) * 256 + (y & 255)] = 0;
}

// ------------------------------------------------------------------ bf16: the two gradient products
// dH = dZ W: A = dZ [mcp, Vp] (or the kept numerators E) is K-contiguous (K = vocabulary), B = W [V, d] is K-major and is read as it lies.
//   dH[rowsel[c0 + m], j] = bf16(sc[m] C[m, j] + g[m] W[y[m], j]) for m < mc (sc: the keeping pass's row factor, else 1)
// dW = dZ^T H: K = rows of the chunk; A = dZ [mcp, Vp] and B = the selected rows of H [*, d] are both K-major.
//   dW[v, j] (+)= C[v, j]
// (kernel templates whose bodies use buffer resources do not get their host stubs emitted: plain kernels)
template <class C>
__device__ __forceinline__ void zero_acc(floatx4 (&acc)[C::MI][C::NI]) {
#pragma unroll
  for (int i = 0; i < C::MI; ++i)
#pragma unroll
    for (int j = 0; j < C::NI; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
}
// K-contiguous operand tile: block row `row_blk` of the blocked [rows, vocabulary] operand; K runs over the vocabulary,
// four steps of 64 per block
template <class C>
__device__ __forceinline__ KContig blocked_rows_tile(const uint16_t* X, int64_t tiles_v, int64_t row_blk) {
  KContig c;
  c.rsrc = make_rsrc(X + blk_offset(row_blk, 0, tiles_v));
  c.hi_bytes = static_cast<uint32_t>(kBlkElems * 2 - 4 * 128);        // from the fourth step of a block to the next block
  const uint32_t kofs = ring2_kofs();
#pragma unroll
  for (int i = 0; i < 4; ++i) c.off[i] = (static_cast<uint32_t>(ring2_row<C>(i)) * 256u + kofs) * 2u;
  return c;
}

// tile_m counts the chunk's live blocks of rows; orig_blk is the block's place in the chunk
__device__ __forceinline__ void dh_tile(int tile_m, int orig_blk, int tile_n, const uint16_t* __restrict__ dZ, int64_t Vp,
                                        const uint16_t* __restrict__ W, int d, int V, uint16_t* __restrict__ dH,
                                        const int32_t* __restrict__ rowsel, int64_t c0, int64_t rows,
                                        const int32_t* __restrict__ ids, const float* __restrict__ g_c,
                                        const float* __restrict__ sc, uint16_t* lds) {
  using C = Cfg;
  const int64_t m0 = static_cast<int64_t>(orig_blk) * C::BM;
  const int n0 = tile_n * C::BN;
  const KContig ca = blocked_rows_tile<C>(dZ, Vp >> 8, tile_m);
  KMajor kb;
  kb.base = reinterpret_cast<const char*>(W + n0);
  kb.ld_bytes = static_cast<int64_t>(d) * 2;
  kb.hi_bytes = 0;
  kb.rowmap = nullptr;
  kb.k_rows = V;                                                     // dz is zero for vocabulary ids past V
  kb.n_units = min(32, (d - n0) / 8);
  floatx4 acc[C::MI][C::NI];
  zero_acc<C>(acc);
  // the third LDS stage goes to W: every group of row tiles streams all of it (twice the bytes of the [rows, V] operand)
  mfma_mainloop_mixed<C, false, true, false, 2>(ca, KMajor{}, KContig{}, kb, static_cast<int>(Vp), lds, acc);
#pragma unroll
  for (int bj = 0; bj < C::NI; ++bj) {
    const int j = n0 + acc_col<C>(bj);
    if (j >= d) continue;
#pragma unroll
    for (int bi = 0; bi < C::MI; ++bi)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t m = m0 + acc_row<C>(bi, r);
        if (m >= rows) continue;
        const int64_t row = rowsel ? rowsel[c0 + m] : c0 + m;
        const float g = g_c[c0 + m];
        float v = sc ? sc[c0 + m] * acc[bi][bj][r] : acc[bi][bj][r];
        if (g != 0.f) v += g * bf2f(W[static_cast<int64_t>(ids[row]) * d + j]);   // g = 0 for invalid ids
        dH[row * d + j] = f2bf(v);
      }
  }
}
// Hx: the rows of H that go with the rows of dZ: H itself (through rowsel, or from row c0 on), or, with hx_blocked, the
// scaled compact copy, which lies in column blocks [d / 256][mcp][256] so that a tile's k-rows are one run of memory
// k_len: rows of the packed [rows, V] operand (a multiple of 256, 0 when no block is live); rows: those that exist
__device__ __forceinline__ void dw_tile(int tile_m, int tile_n, const uint16_t* __restrict__ dZ, int64_t mcp, int64_t Vp,
                                        const uint16_t* __restrict__ Hx, int hx_blocked, int d, int V,
                                        const int32_t* __restrict__ rowmap, int k_len, int rows, float* __restrict__ dW,
                                        int accumulate, uint16_t* lds) {
  using C = Cfg;
  const int64_t m0 = static_cast<int64_t>(tile_m) * C::BM;
  const int n0 = tile_n * C::BN;
  KMajor ka;                                                         // blocked dZ: k = row of the chunk, entries = vocabulary
  ka.base = reinterpret_cast<const char*>(dZ + blk_offset(0, tile_m, Vp >> 8));
  ka.ld_bytes = 512;
  ka.hi_bytes = (Vp >> 8) * kBlkElems * 2 - 256 * 512;               // from the last row of a block to the block below
  ka.rowmap = nullptr;
  ka.k_rows = k_len;
  ka.n_units = 32;
  KMajor kb;                                                         // rows of H: k = row of the chunk, entries = hidden columns
  kb.base = reinterpret_cast<const char*>(hx_blocked ? Hx + static_cast<int64_t>(tile_n) * mcp * 256 : Hx + n0);
  kb.ld_bytes = hx_blocked ? 512 : static_cast<int64_t>(d) * 2;
  kb.hi_bytes = 0;
  kb.rowmap = rowmap;
  kb.k_rows = rows;                                                  // dz is zero for rows past the chunk
  kb.n_units = min(32, (d - n0) / 8);
  floatx4 acc[C::MI][C::NI];
  zero_acc<C>(acc);
  if (k_len > 0) {
    if (rowmap) mfma_mainloop_mixed<C, true, true, true>(KContig{}, ka, KContig{}, kb, k_len, lds, acc);
    else mfma_mainloop_mixed<C, true, true, false>(KContig{}, ka, KContig{}, kb, k_len, lds, acc);
  }
#pragma unroll
  for (int bj = 0; bj < C::NI; ++bj) {
    const int j = n0 + acc_col<C>(bj);
    if (j >= d) continue;
#pragma unroll
    for (int bi = 0; bi < C::MI; ++bi)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t v = m0 + acc_row<C>(bi, r);
        if (v >= V) continue;
        float* dst = dW + v * d + j;
        *dst = accumulate ? *dst + acc[bi][bj][r] : acc[bi][bj][r];
      }
  }
}
// Both products in one launch: the first grid_dh workgroups take the dH tiles, the rest the dW tiles.  dH has few,
// long tiles (K = vocabulary) and on its own leaves a fifth of the last round idle; here an XCD that runs out of dH
// tiles goes on with dW tiles, and the host gives every XCD the share of dW groups that evens out the sum.
__global__ void __launch_bounds__(Cfg::T)
k_gemm_dh_dw(const uint16_t* __restrict__ dZ, int64_t Vp, int64_t mcp, const uint16_t* __restrict__ W,
             const uint16_t* __restrict__ Hx, int hx_blocked, const int32_t* __restrict__ h_rowmap, int d, int V, int tiles_v,
             int tiles_d, unsigned grid_dh, const LiveInfo* __restrict__ info, const int32_t* __restrict__ blk_orig,
             uint16_t* __restrict__ dH, float* __restrict__ dW, int accumulate, const int32_t* __restrict__ rowsel,
             int64_t c0, int64_t rows, const int32_t* __restrict__ ids, const float* __restrict__ g_c,
             const float* __restrict__ sc) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[MixedLdsBytes<Cfg>::value / 2];
  const int n_live = info->n_live;                     // live blocks of rows: dH row tiles, dW K blocks
  int tile_m, tile_n;
  if (blockIdx.x < grid_dh) {
    if (!tile_coords<kGM, kGN>(n_live, tiles_d, &tile_m, &tile_n)) return;
    dh_tile(tile_m, blk_orig[(c0 >> 8) + tile_m], tile_n, dZ, Vp, W, d, V, dH, rowsel, c0, rows, ids, g_c, sc, lds);
  } else {
    if (!tile_coords_shared<kGM, kGN>(tiles_v, tiles_d, blockIdx.x - grid_dh, info->dw_groups, &tile_m, &tile_n)) return;
    dw_tile(tile_m, tile_n, dZ, mcp, Vp, Hx, hx_blocked, d, V, h_rowmap, n_live * 256, info->k_rows, dW, accumulate, lds);
  }
}

// One-hot part of dW: dW[y_n, :] += g_n h_n for every selected row, in float32.  Rows that took the same token add
// into the same dW row, hence atomics - and token frequencies are skewed (a seventh of the rows of a Zipf(1.1) batch
// took the most frequent token), so adding row by row queues thousands of atomics on the same cache lines.  A
// workgroup therefore takes kOneHotRows consecutive selected rows and adds them up by token first: the first row of
// every token in the group is its leader; a wavefront sums the leader and its followers in registers, 2048 columns at
// a time (16-byte loads, a lane owning eight consecutive columns of each of four pieces), turns every piece through
// its corner of LDS so that consecutive lanes hold consecutive columns, and issues one atomic per element of the sum.
constexpr int kOneHotRows = 128;
constexpr int kOneHotPieces = 4;                    // pieces of 512 columns a wavefront holds at a time
__global__ void __launch_bounds__(256)
k_dw_onehot(const uint16_t* __restrict__ H, int d, const int32_t* __restrict__ rowsel, int64_t n_sel,
            const int32_t* __restrict__ ids, const float* __restrict__ g_c, float* __restrict__ dW) {
  __shared__ int32_t s_id[kOneHotRows];             // token of the row, -1 when the row adds nothing
  __shared__ float s_g[kOneHotRows];
  __shared__ int64_t s_row[kOneHotRows];
  __shared__ int32_t s_leader[kOneHotRows];         // the group's leaders, compacted
  __shared__ int32_t s_n_leader;
  __shared__ float s_turn[256 / kWave][8 * kWave];  // one piece per wavefront, in column order
  const int tid = threadIdx.x, lane = tid & 63, wave = tid / kWave;
  if (tid < kOneHotRows) {
    const int64_t n = static_cast<int64_t>(blockIdx.x) * kOneHotRows + tid;
    float g = 0.f;
    int64_t row = 0;
    int32_t id = -1;
    if (n < n_sel) {
      g = g_c[n];                                  // 0: clipped rows, zero advantage, invalid ids
      row = rowsel ? rowsel[n] : n;
      if (g != 0.f) id = ids[row];
    }
    s_id[tid] = id; s_g[tid] = g; s_row[tid] = row;
  }
  if (tid == 0) s_n_leader = 0;
  __syncthreads();
  if (tid < kOneHotRows) {
    const int32_t id = s_id[tid];
    bool leader = id >= 0;
    for (int u = 0; u < tid && leader; ++u) leader = s_id[u] != id;
    if (leader) s_leader[atomicAdd(&s_n_leader, 1)] = tid;
  }
  __syncthreads();
  const int n_leader = s_n_leader;
  float* turn = s_turn[wave];
  for (int li = wave; li < n_leader; li += 256 / kWave) {
    const int32_t id = s_id[s_leader[li]];
    float* dst = dW + static_cast<int64_t>(id) * d;
    unsigned long long same[kOneHotRows / kWave];   // the rows of the group that took this token
#pragma unroll
    for (int k = 0; k < kOneHotRows / kWave; ++k) same[k] = __ballot(s_id[lane + kWave * k] == id);
    for (int c0 = 0; c0 < d; c0 += kOneHotPieces * 8 * kWave) {   // d is a multiple of 8: a lane's eight columns are all inside or all outside
      float acc[kOneHotPieces][8];
#pragma unroll
      for (int q = 0; q < kOneHotPieces; ++q)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[q][k] = 0.f;
#pragma unroll
      for (int k = 0; k < kOneHotRows / kWave; ++k) {
        for (unsigned long long m = same[k]; m; m &= m - 1) {
          const int u = kWave * k + __ffsll(static_cast<long long>(m)) - 1;
          const uint16_t* h = H + s_row[u] * d;
          const float g = s_g[u];
          uint4 hv[kOneHotPieces];
#pragma unroll
          for (int q = 0; q < kOneHotPieces; ++q) {   // the row's pieces are in flight together
            const int c = c0 + (q * kWave + lane) * 8;
            hv[q] = c < d ? *reinterpret_cast<const uint4*>(h + c) : make_uint4(0u, 0u, 0u, 0u);
          }
#pragma unroll
          for (int q = 0; q < kOneHotPieces; ++q) {
            const uint32_t w4[4] = {hv[q].x, hv[q].y, hv[q].z, hv[q].w};
#pragma unroll
            for (int k2 = 0; k2 < 4; ++k2) {
              acc[q][2 * k2] += g * bf2f(static_cast<uint16_t>(w4[k2] & 0xFFFFu));
              acc[q][2 * k2 + 1] += g * bf2f(static_cast<uint16_t>(w4[k2] >> 16));
            }
          }
        }
      }
#pragma unroll
      for (int q = 0; q < kOneHotPieces; ++q) {
        const int cq = c0 + q * 8 * kWave;           // first column of the piece
        if (cq >= d) break;
        // column cq + 8 lane + k sits in this lane's acc[q][k]; after the turn, lane l adds columns cq + 64 k + l
        *reinterpret_cast<float4*>(turn + 8 * lane) = make_float4(acc[q][0], acc[q][1], acc[q][2], acc[q][3]);
        *reinterpret_cast<float4*>(turn + 8 * lane + 4) = make_float4(acc[q][4], acc[q][5], acc[q][6], acc[q][7]);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int c = cq + kWave * k + lane;
          if (c < d) unsafeAtomicAdd(dst + c, turn[kWave * k + lane]);
        }
        __builtin_amdgcn_wave_barrier();
      }
    }
  }
}

// ------------------------------------------------------------------ float32: plain backward
// dz[n, v] = g (onehot - exp(z - lse)) for a chunk of selected rows, z recomputed with the same float64 dot
// product as the forward pass; sums are carried in float64 here too.
__global__ void __launch_bounds__(256)
k_dz_f32(const float* __restrict__ W, const float* __restrict__ H, int d, int V, const int32_t* __restrict__ rowsel,
         int64_t c0, const int32_t* __restrict__ ids, const float* __restrict__ lse_c, const float* __restrict__ g_c,
         const float* __restrict__ ent_c, const float* __restrict__ kz_c, float* __restrict__ dz) {
  extern __shared__ float s_h[];
  const int64_t n = blockIdx.x;
  const int64_t row = rowsel ? rowsel[c0 + n] : c0 + n;
  for (int k = threadIdx.x; k < d; k += blockDim.x) s_h[k] = H[row * d + k];
  __syncthreads();
  __shared__ double s_red[32];
  const int y = ids[row];
  const double l = lse_c[c0 + n], g = g_c[c0 + n], en = ent_c[c0 + n], k_ent = kz_c[c0 + n];
  // The taken token's entry g (1 - p_y): for a confident token (p_y > 1/2) 1 - p_y cancels down to the error of p_y,
  // and the sum of the other probabilities, which carries only their relative error, is taken in its place.
  double rest = 0.0, label_ent = 0.0, p_label = 0.0;
  for (int v = threadIdx.x; v < V; v += blockDim.x) {
    const double z = dot_f64(s_h, W + static_cast<int64_t>(v) * d, d);
    const double p = exp(z - l);
    const double e = k_ent != 0.0 ? k_ent * p * ((z - l) + en) : 0.0;     // entropy bonus: k p (log p + entropy)
    if (v == y) {
      label_ent = e;
      p_label = p;
    } else {
      rest += p;
      dz[n * V + v] = static_cast<float>(-g * p + e);
    }
  }
  rest = block_sum<double>(rest, s_red);
  if (y >= 0 && y < V && threadIdx.x == y % static_cast<int>(blockDim.x))
    dz[n * V + y] = static_cast<float>(g * (p_label > 0.5 ? rest : 1.0 - p_label) + label_ent);
}
// dH[row, j] = sum_v dz[n, v] W[v, j]
__global__ void __launch_bounds__(256)
k_dh_f32(const float* __restrict__ dz, const float* __restrict__ W, int d, int V, const int32_t* __restrict__ rowsel,
         int64_t c0, float* __restrict__ dH) {
  const int64_t n = blockIdx.x;
  const int64_t row = rowsel ? rowsel[c0 + n] : c0 + n;
  for (int j = threadIdx.x; j < d; j += blockDim.x) {
    double s = 0.0;
    for (int v = 0; v < V; ++v) s = fma(static_cast<double>(dz[n * V + v]), static_cast<double>(W[static_cast<int64_t>(v) * d + j]), s);
    dH[row * d + j] = static_cast<float>(s);
  }
}
// dW[v, j] (+)= sum_n dz[n, v] H[row(n), j]
__global__ void __launch_bounds__(256)
k_dw_f32(const float* __restrict__ dz, const float* __restrict__ H, int d, int V, const int32_t* __restrict__ rowsel,
         int64_t c0, int64_t mc, int accumulate, float* __restrict__ dW) {
  const int v = blockIdx.x;
  for (int j = threadIdx.x; j < d; j += blockDim.x) {
    double s = 0.0;
    for (int64_t n = 0; n < mc; ++n) {
      const int64_t row = rowsel ? rowsel[c0 + n] : c0 + n;
      s = fma(static_cast<double>(dz[n * V + v]), static_cast<double>(H[row * d + j]), s);
    }
    float* dst = dW + static_cast<int64_t>(v) * d + j;
    *dst = accumulate ? static_cast<float>(static_cast<double>(*dst) + s) : static_cast<float>(s);
  }
}

// ------------------------------------------------------------------ host side
constexpr int64_t kF32ChunkRows = 4096;
constexpr double kF32MaxWork = 137438953472.0;   // 2^37 multiply-adds per product
constexpr int64_t kMaxChunkRows = 1 << 17;

int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

struct ScoreWs {
  float4* partial;   // [tiles_m][n_pad]
  float* logp_c;
  float* lse_c;
  float* ent_c;
};
size_t carve_score(Carver& c, ScoreWs& w, int64_t n_sel, int V, umas_dtype dt, bool compact) {
  const int64_t n_pad = round_up(n_sel > 0 ? n_sel : 1, Cfg::BN);
  const int64_t tiles_m = (V + Cfg::BM - 1) / Cfg::BM;
  w.partial = dt == UMAS_BF16 ? c.take<float4>(static_cast<size_t>(tiles_m) * n_pad) : nullptr;
  w.logp_c = w.lse_c = w.ent_c = nullptr;
  if (compact) {
    w.logp_c = c.take<float>(n_pad);
    w.lse_c = c.take<float>(n_pad);
    w.ent_c = c.take<float>(n_pad);
  }
  return c.off;
}

struct PpoWs {
  ScoreWs score;
  float* g_c;
  float* a_c;        // per selected row: coefficients of the backward's dense part
  float* kz_c;
  float* cref;       // keeping pass: per selected row, the reference of E and the row factor of dz = sc E
  float* sc;
  int32_t* flags;    // keeping pass: blocks of 256 selected rows whose dz must be recomputed
  int32_t* blk_live; // per block of 256 selected rows: some row has a gradient
  int32_t* blk_cidx; // its place among the live blocks of its chunk, -1 for a dead one
  int32_t* blk_orig; // per chunk: live block -> block of the chunk
  LiveInfo* live;    // of the chunk in work
  double* blk_stats;
  char* chunk;       // rest of the workspace: dZ (or E) [mcp, Vp], then the scaled copy of the chunk's rows of H
  size_t fixed_bytes;
};
// bytes one chunk of mc rows needs
size_t chunk_bytes(int64_t mc, int d, int V, umas_dtype dt) {
  if (dt == UMAS_F32) return align_up(static_cast<size_t>(mc) * V * sizeof(float));
  const int64_t Vp = round_up(V, 256), mcp = round_up(mc, 256);
  return align_up(static_cast<size_t>(mcp) * Vp * 2) + align_up(static_cast<size_t>(mcp) * round_up(d, 256) * 2);
}
size_t carve_ppo(Carver& c, PpoWs& w, int64_t n_sel, int d, int V, umas_dtype dt, int n_roles) {
  (void)d;                                      // the per-chunk buffers depend on d, the fixed part does not
  carve_score(c, w.score, n_sel, V, dt, true);
  const int64_t n_pad = round_up(n_sel > 0 ? n_sel : 1, Cfg::BN);
  w.g_c = c.take<float>(n_pad);
  w.a_c = c.take<float>(n_pad);
  w.kz_c = c.take<float>(n_pad);
  w.cref = c.take<float>(n_pad);
  w.sc = c.take<float>(n_pad);
  w.flags = c.take<int32_t>(static_cast<size_t>(cdiv(n_pad, kRowBlock)));
  w.blk_live = c.take<int32_t>(static_cast<size_t>(cdiv(n_pad, kRowBlock)));
  w.blk_cidx = c.take<int32_t>(static_cast<size_t>(cdiv(n_pad, kRowBlock)));
  w.blk_orig = c.take<int32_t>(static_cast<size_t>(cdiv(n_pad, kRowBlock)));
  w.live = c.take<LiveInfo>(1);
  w.blk_stats = c.take<double>(static_cast<size_t>(cdiv(n_pad, kRowBlock)) * (1 + n_roles) * kStat);
  w.chunk = c.base ? c.base + c.off : nullptr;
  w.fixed_bytes = c.off;
  return c.off;
}

umas_status check_model_args(const void* H, const void* W, umas_dtype dt, int64_t n_rows, int d, int V,
                             const int32_t* ids, const int32_t* rowsel, int64_t n_sel) {
  UMAS_REQUIRE(dt == UMAS_F32 || dt == UMAS_BF16, UMAS_EDTYPE, "dtype=%d is neither F32 nor BF16", static_cast<int>(dt));
  UMAS_REQUIRE(n_rows >= 0 && n_sel >= 0, UMAS_EINVAL, "negative row count");
  UMAS_REQUIRE(d >= 1 && V >= 1, UMAS_ESHAPE, "d=%d and V=%d must be positive", d, V);
  UMAS_REQUIRE(dt != UMAS_BF16 || d % 8 == 0, UMAS_ESHAPE, "bf16 needs d %% 8 == 0 (d=%d)", d);
  UMAS_REQUIRE(dt != UMAS_F32 || d <= 8192, UMAS_ESHAPE, "the float32 path supports d <= 8192 (d=%d)", d);
  // the float32 path is the plain, untiled one (every thread walks whole rows of W): small shapes only
  UMAS_REQUIRE(dt != UMAS_F32 || static_cast<double>(n_sel) * V * d <= kF32MaxWork, UMAS_ESHAPE,
               "the float32 path is for small shapes: n_sel * V * d = %.3g exceeds %.3g; use bf16",
               static_cast<double>(n_sel) * V * d, kF32MaxWork);
  UMAS_REQUIRE(dt != UMAS_BF16 || static_cast<uint64_t>(n_rows) * d * 2 < (1ull << 32), UMAS_ESHAPE,
               "bf16 H must be smaller than 4 GiB (32-bit buffer offsets): n_rows=%lld d=%d",
               static_cast<long long>(n_rows), d);
  UMAS_REQUIRE(rowsel || n_sel == n_rows, UMAS_EINVAL, "rowsel is NULL but n_sel != n_rows");
  UMAS_REQUIRE(n_sel <= n_rows, UMAS_EINVAL, "n_sel=%lld exceeds n_rows=%lld", static_cast<long long>(n_sel),
               static_cast<long long>(n_rows));
  UMAS_REQUIRE((H && ids) || n_rows == 0, UMAS_EINVAL, "H and ids must not be NULL");
  UMAS_REQUIRE(W, UMAS_EINVAL, "W must not be NULL");
  UMAS_REQUIRE(reinterpret_cast<uintptr_t>(H) % 16 == 0 && reinterpret_cast<uintptr_t>(W) % 16 == 0, UMAS_EINVAL,
               "H and W must be 16-byte aligned");
  return UMAS_OK;
}

umas_status check_ws(void* ws, size_t have, size_t need) {
  UMAS_REQUIRE(ws && reinterpret_cast<uintptr_t>(ws) % kAlign == 0 && have >= need, UMAS_EWORKSPACE,
               "workspace must be 256-byte aligned and hold %zu bytes (got %zu)", need, have);
  return UMAS_OK;
}

// Forward scoring of the selected rows into compact arrays and/or scattered outputs.
umas_status run_score(const void* H, const void* W, umas_dtype dt, int d, int V, const int32_t* ids,
                      const int32_t* rowsel, int64_t n_sel, const ScoreWs& w, float* logp, float* lse,
                      float* entropy, hipStream_t st) {
  if (n_sel == 0) return UMAS_OK;
  if (dt == UMAS_BF16) {
    const int tiles_m = (V + Cfg::BM - 1) / Cfg::BM;
    const int tiles_n = static_cast<int>((n_sel + Cfg::BN - 1) / Cfg::BN);
    const int64_t n_pad = round_up(n_sel, Cfg::BN);
    hipLaunchKernelGGL(k_score_tiles, dim3(tile_grid<kGM, kGN>(tiles_m, tiles_n, kTilesPerWg)), dim3(Cfg::T), 0, st,
                       static_cast<const uint16_t*>(W), static_cast<const uint16_t*>(H), d, V, rowsel, n_sel, ids,
                       tiles_m, tiles_n, w.partial, n_pad);
    UMAS_LAUNCHED("k_score_tiles");
    hipLaunchKernelGGL(k_score_finalize, dim3(cdiv(n_sel, 32)), dim3(256), 0, st, w.partial, tiles_m, n_pad,
                       static_cast<int64_t>(0), n_sel, static_cast<const float*>(nullptr), rowsel, ids, V, w.logp_c, w.lse_c,
                       w.ent_c, logp, lse, entropy);
    UMAS_LAUNCHED("k_score_finalize");
  } else {
    hipLaunchKernelGGL(k_score_f32, dim3(static_cast<unsigned>(n_sel)), dim3(256), d * sizeof(float), st,
                       static_cast<const float*>(W), static_cast<const float*>(H), d, V, rowsel, ids, w.logp_c,
                       w.lse_c, w.ent_c, logp, lse, entropy);
    UMAS_LAUNCHED("k_score_f32");
  }
  return UMAS_OK;
}

}  // namespace
}  // namespace umas

using namespace umas;

extern "C" size_t umas_policy_logprobs_workspace_bytes(int64_t n_sel, int32_t d, int32_t V, umas_dtype dtype) {
  (void)d;
  if (n_sel < 0 || V < 1) return 0;
  Carver c(nullptr);
  ScoreWs w;
  const size_t b = carve_score(c, w, n_sel, V, dtype, false);
  return b > 0 ? b : kAlign;
}

extern "C" umas_status umas_policy_logprobs(const void* H, const void* W, umas_dtype dtype, int64_t n_rows, int32_t d,
                                            int32_t V, const int32_t* ids, const int32_t* rowsel, int64_t n_sel,
                                            float* logp, float* lse, float* entropy, void* workspace,
                                            size_t workspace_bytes, void* hip_stream) {
  umas_status s = check_model_args(H, W, dtype, n_rows, d, V, ids, rowsel, n_sel);
  if (s != UMAS_OK) return s;
  UMAS_REQUIRE((logp && lse) || n_rows == 0, UMAS_EINVAL, "logp and lse must not be NULL");
  UMAS_REQUIRE(n_sel < (1LL << 31), UMAS_ESHAPE, "at most 2^31-1 selected rows");
  s = check_ws(workspace, workspace_bytes, umas_policy_logprobs_workspace_bytes(n_sel, d, V, dtype));
  if (s != UMAS_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  if (rowsel && n_rows > 0) {
    UMAS_HIP(fill_bytes_zero(logp, n_rows * sizeof(float), st));
    UMAS_HIP(fill_bytes_zero(lse, n_rows * sizeof(float), st));
    if (entropy) UMAS_HIP(fill_bytes_zero(entropy, n_rows * sizeof(float), st));
  }
  Carver c(workspace);
  ScoreWs w;
  carve_score(c, w, n_sel, V, dtype, false);
  return run_score(H, W, dtype, d, V, ids, rowsel, n_sel, w, logp, lse, entropy, st);
}

// ------------------------------------------------------------------ scoring without any allocation
// The per-tile partials of the scoring pass live in a file-scope device array in place of a caller's workspace.
// Every GPU holds its own copy of the array at its own address, resolved once per device; host code only ever
// uses that resolved address.  Nothing in it has to start at zero: the tile kernel writes every partial that the
// merge kernel reads.
static __device__ __align__(256) unsigned char scratch[UMAS_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // per device: address of `scratch` there, NULL until first used

umas_status static_scratch(void** out) {
  int dev = -1;
  UMAS_HIP(hipGetDevice(&dev));
  UMAS_REQUIRE(dev >= 0 && dev < kMaxDevices, UMAS_ESHAPE, "device %d outside [0,%d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    UMAS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    UMAS_REQUIRE(p, UMAS_EHIP, "hipGetSymbolAddress returned no address for the static scratch");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return UMAS_OK;
}
}  // namespace

extern "C" umas_status umas_policy_logprobs_static(const void* H, const void* W, umas_dtype dtype, int64_t n_rows,
                                                   int32_t d, int32_t V, const int32_t* ids, const int32_t* rowsel,
                                                   int64_t n_sel, float* logp, float* lse, float* entropy,
                                                   void* hip_stream) {
  umas_status s = check_model_args(H, W, dtype, n_rows, d, V, ids, rowsel, n_sel);
  if (s != UMAS_OK) return s;
  UMAS_REQUIRE((logp && lse) || n_rows == 0, UMAS_EINVAL, "logp and lse must not be NULL");
  UMAS_REQUIRE(n_sel < (1LL << 31), UMAS_ESHAPE, "at most 2^31-1 selected rows");
  const size_t need = umas_policy_logprobs_workspace_bytes(n_sel, d, V, dtype);
  UMAS_REQUIRE(need <= static_cast<size_t>(UMAS_STATIC_SCRATCH_BYTES), UMAS_EWORKSPACE,
               "%lld selected rows against a vocabulary of %d need %zu bytes of scratch, the static scratch holds %zu: "
               "score fewer rows per call or use umas_policy_logprobs with a workspace",
               static_cast<long long>(n_sel), V, need, static_cast<size_t>(UMAS_STATIC_SCRATCH_BYTES));
  void* ws = nullptr;
  s = static_scratch(&ws);
  if (s != UMAS_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  if (rowsel && n_rows > 0) {
    UMAS_HIP(fill_bytes_zero(logp, n_rows * sizeof(float), st));
    UMAS_HIP(fill_bytes_zero(lse, n_rows * sizeof(float), st));
    if (entropy) UMAS_HIP(fill_bytes_zero(entropy, n_rows * sizeof(float), st));
  }
  Carver c(ws);
  ScoreWs w;
  carve_score(c, w, n_sel, V, dtype, false);
  return run_score(H, W, dtype, d, V, ids, rowsel, n_sel, w, logp, lse, entropy, st);
}

extern "C" size_t umas_ppo_loss_workspace_bytes_min(int64_t n_sel, int32_t d, int32_t V, umas_dtype dtype,
                                                    int32_t n_roles) {
  if (n_sel < 0 || d < 1 || V < 1 || n_roles < 0) return 0;
  Carver c(nullptr);
  PpoWs w;
  carve_ppo(c, w, n_sel, d, V, dtype, n_roles);
  const int64_t mc = n_sel < 256 ? (n_sel > 0 ? n_sel : 1) : 256;
  return c.off + chunk_bytes(mc, d, V, dtype);
}

extern "C" size_t umas_ppo_loss_workspace_bytes(int64_t n_sel, int32_t d, int32_t V, umas_dtype dtype,
                                                int32_t n_roles) {
  if (n_sel < 0 || d < 1 || V < 1 || n_roles < 0) return 0;
  Carver c(nullptr);
  PpoWs w;
  carve_ppo(c, w, n_sel, d, V, dtype, n_roles);
  int64_t mc = n_sel > 0 ? n_sel : 1;
  const int64_t cap = dtype == UMAS_F32 ? kF32ChunkRows : kMaxChunkRows;
  if (mc > cap) {
    const int64_t nchunk = (mc + cap - 1) / cap;
    mc = round_up((mc + nchunk - 1) / nchunk, 256);
  }
  return c.off + chunk_bytes(mc, d, V, dtype);
}

extern "C" umas_status umas_ppo_loss_fwd_bwd(const void* H, const void* W, umas_dtype dtype, int64_t n_rows, int32_t d,
                                             int32_t V, const int32_t* ids, const int32_t* rowsel, int64_t n_sel,
                                             const float* logp_old, const float* adv, const int32_t* tok_role,
                                             int32_t n_roles, float clip_eps, float entropy_coef, float dual_clip,
                                             int32_t accumulate_dW, int64_t norm_rows, const float* logp_ref,
                                             float kl_coef, umas_loss_stats* stats, float* logp_new, void* dH,
                                             float* dW, void* workspace, size_t workspace_bytes, void* hip_stream) {
  umas_status s = check_model_args(H, W, dtype, n_rows, d, V, ids, rowsel, n_sel);
  if (s != UMAS_OK) return s;
  UMAS_REQUIRE((adv && dH) || n_rows == 0, UMAS_EINVAL, "adv and dH must not be NULL");
  UMAS_REQUIRE(stats && dW, UMAS_EINVAL, "stats and dW must not be NULL");
  UMAS_REQUIRE(n_roles >= 0 && n_roles <= UMAS_MAX_ROLES, UMAS_ESHAPE, "n_roles=%d outside [0,%d]", n_roles, UMAS_MAX_ROLES);
  UMAS_REQUIRE(tok_role || n_roles == 0, UMAS_EINVAL, "tok_role is NULL but n_roles > 0");
  UMAS_REQUIRE(clip_eps > 0.f && clip_eps < 1.f, UMAS_EINVAL, "clip_eps=%g outside (0,1)", static_cast<double>(clip_eps));
  UMAS_REQUIRE(entropy_coef >= 0.f, UMAS_EINVAL, "entropy_coef=%g must not be negative", static_cast<double>(entropy_coef));
  UMAS_REQUIRE(dual_clip == 0.f || dual_clip > 1.f, UMAS_EINVAL, "dual_clip=%g must be 0 (off) or larger than 1",
               static_cast<double>(dual_clip));
  UMAS_REQUIRE(n_sel < (1LL << 31), UMAS_ESHAPE, "at most 2^31-1 selected rows");
  UMAS_REQUIRE(norm_rows == 0 || norm_rows >= n_sel, UMAS_EINVAL, "norm_rows=%lld must be 0 or at least n_sel=%lld",
               static_cast<long long>(norm_rows), static_cast<long long>(n_sel));
  UMAS_REQUIRE(kl_coef >= 0.f, UMAS_EINVAL, "kl_coef=%g must not be negative", static_cast<double>(kl_coef));
  UMAS_REQUIRE(kl_coef == 0.f || logp_ref || n_rows == 0, UMAS_EINVAL, "kl_coef > 0 needs logp_ref");
  s = check_ws(workspace, workspace_bytes, umas_ppo_loss_workspace_bytes_min(n_sel, d, V, dtype, n_roles));
  if (s != UMAS_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  const size_t esz = dtype == UMAS_BF16 ? 2 : 4;
  Carver c(workspace);
  PpoWs w;
  carve_ppo(c, w, n_sel, d, V, dtype, n_roles);

  // rows that are not selected, and (bf16 without an entropy bonus) selected rows in blocks without any gradient,
  // are not visited by the backward
  const bool skips_dead_blocks = dtype == UMAS_BF16 && entropy_coef == 0.f;
  if (rowsel && n_rows > 0 && logp_new) UMAS_HIP(fill_bytes_zero(logp_new, n_rows * sizeof(float), st));
  if ((rowsel || skips_dead_blocks) && n_rows > 0) UMAS_HIP(fill_bytes_zero(dH, static_cast<size_t>(n_rows) * d * esz, st));
  if (!accumulate_dW && n_sel == 0) UMAS_HIP(fill_bytes_zero(dW, static_cast<size_t>(V) * d * sizeof(float), st));

  // chunks of selected rows sized to the workspace
  const size_t room = workspace_bytes - w.fixed_bytes;
  int64_t mc = n_sel > 0 ? n_sel : 1;
  const int64_t cap = dtype == UMAS_F32 ? kF32ChunkRows : kMaxChunkRows;
  if (mc > cap) mc = cap;
  while (mc > 256 && chunk_bytes(mc, d, V, dtype) > room) mc = round_up(mc / 2, 256);
  if (mc > 256) {   // balance the chunks
    const int64_t nchunk = (n_sel + mc - 1) / mc;
    const int64_t even = round_up((n_sel + nchunk - 1) / nchunk, 256);
    if (even < mc) mc = even;
  }
  UMAS_REQUIRE(chunk_bytes(mc < n_sel ? mc : (n_sel > 0 ? n_sel : 1), d, V, dtype) <= room, UMAS_EWORKSPACE,
               "workspace cannot hold one chunk of %lld rows", static_cast<long long>(mc));

  const int nblk = cdiv(n_sel > 0 ? n_sel : 1, kRowBlock);
  const int64_t norm = norm_rows > 0 ? norm_rows : n_sel;   // rows the token mean is taken over
  const float k_ent = norm > 0 ? entropy_coef / static_cast<float>(norm) : 0.f;
  // Without an entropy bonus dz is a row factor times the softmax: the scoring pass keeps the numerators
  // and the logits are not computed a second time.
  const bool keep = dtype == UMAS_BF16 && entropy_coef == 0.f && n_sel > 0;
  const int64_t Vp = round_up(V, 256);
  const uint16_t* Wb = static_cast<const uint16_t*>(W);
  const uint16_t* Hb = static_cast<const uint16_t*>(H);

  if (!keep) {
    // forward scoring and the surrogate
    s = run_score(H, W, dtype, d, V, ids, rowsel, n_sel, w.score, logp_new, nullptr, nullptr, st);
    if (s != UMAS_OK) return s;
    hipLaunchKernelGGL(k_ppo_rows, dim3(nblk), dim3(kRowBlock), (1 + n_roles) * kStat * sizeof(double), st, norm,
                       static_cast<int64_t>(0), n_sel, rowsel, ids, V, w.score.logp_c, w.score.ent_c, logp_old, adv,
                       tok_role, n_roles, clip_eps, dual_clip, k_ent, logp_ref, kl_coef, dtype == UMAS_BF16 ? 1 : 0, w.score.lse_c,
                       w.g_c, w.a_c, w.kz_c,
                       w.blk_stats);
    UMAS_LAUNCHED("k_ppo_rows");
  } else {
    hipLaunchKernelGGL(k_label_logit, dim3(cdiv(n_sel, 4)), dim3(256), 0, st, Hb, Wb, d, V, rowsel, n_sel, ids, w.cref);
    UMAS_LAUNCHED("k_label_logit");
    UMAS_HIP(fill_bytes_zero(w.flags, static_cast<size_t>(nblk) * sizeof(int32_t), st));
    hipLaunchKernelGGL(k_live_flags, dim3(nblk), dim3(256), 0, st, n_sel, rowsel, adv, w.blk_live);
    UMAS_LAUNCHED("k_live_flags");
    const int64_t n_pad = round_up(n_sel, Cfg::BN);
    const int tiles_v = static_cast<int>(Vp / 256), tiles_d = (d + 255) / 256;
    const int max_groups = max_dw_groups_per_xcd(tiles_v, tiles_d);
    for (int64_t c0 = 0; c0 < n_sel; c0 += mc) {
      const int64_t rows = n_sel - c0 < mc ? n_sel - c0 : mc;
      const int64_t mcp = round_up(rows, 256);
      const int tiles_r = static_cast<int>(mcp / 256);
      uint16_t* E = reinterpret_cast<uint16_t*>(w.chunk);
      uint16_t* Hs = reinterpret_cast<uint16_t*>(w.chunk + align_up(static_cast<size_t>(mcp) * Vp * 2));
      hipLaunchKernelGGL(k_live_scan, dim3(1), dim3(512), 0, st, static_cast<int>(c0 >> 8), tiles_r, rows, kl_coef != 0.f ? 1 : 0, tiles_v,
                         tiles_d, Vp, max_groups, w.blk_live, w.blk_cidx, w.blk_orig, w.live);   // a KL term gives every row a gradient
      UMAS_LAUNCHED("k_live_scan");
      hipLaunchKernelGGL(k_score_keep_tiles, dim3(tile_grid<kGM, kGN>(tiles_v, tiles_r, kTilesPerWg)), dim3(Cfg::T), 0, st,
                         Wb, Hb, d, V, rowsel, c0, rows, ids, tiles_v, tiles_r, w.score.partial, n_pad, w.cref, E, Vp, w.flags,
                         w.blk_cidx);
      UMAS_LAUNCHED("k_score_keep_tiles");
      hipLaunchKernelGGL(k_score_finalize, dim3(cdiv(rows, 32)), dim3(256), 0, st, w.score.partial, tiles_v, n_pad, c0,
                         c0 + rows, w.cref, rowsel, ids, V, w.score.logp_c, w.score.lse_c, w.score.ent_c, logp_new,
                         static_cast<float*>(nullptr), static_cast<float*>(nullptr));
      UMAS_LAUNCHED("k_score_finalize");
      hipLaunchKernelGGL(k_ppo_rows, dim3(cdiv(rows, kRowBlock)), dim3(kRowBlock), (1 + n_roles) * kStat * sizeof(double),
                         st, norm, c0, c0 + rows, rowsel, ids, V, w.score.logp_c, w.score.ent_c, logp_old, adv, tok_role,
                         n_roles, clip_eps, dual_clip, k_ent, logp_ref, kl_coef, 1, w.score.lse_c, w.g_c, w.a_c, w.kz_c,
                         w.blk_stats);
      UMAS_LAUNCHED("k_ppo_rows");
      // blocks of rows the scoring pass flagged (a logit far above the row's reference) get dz the long way
      hipLaunchKernelGGL(k_dz_flagged, dim3(kFlaggedGrid), dim3(Cfg::T), 0, st, Wb, Hb, d, V, rowsel, c0, rows,
                         w.score.lse_c, w.a_c, w.kz_c, tiles_v, tiles_r, E, Vp, w.flags, w.blk_cidx);
      UMAS_LAUNCHED("k_dz_flagged");
      hipLaunchKernelGGL(k_keep_rows, dim3(cdiv(rows, 4)), dim3(256), 0, st, Hb, d, V, rowsel, c0, rows, ids, E,
                         static_cast<int64_t>(tiles_v), w.score.lse_c, w.a_c, w.cref, w.flags, w.blk_cidx, w.sc, Hs, mcp);
      UMAS_LAUNCHED("k_keep_rows");
      const unsigned grid_dh = tile_grid<kGM, kGN>(tiles_r, tiles_d);
      hipLaunchKernelGGL(k_gemm_dh_dw, dim3(grid_dh + static_cast<unsigned>(max_groups) * kGM * kGN * 8), dim3(Cfg::T), 0, st,
                         E, Vp, mcp, Wb, Hs, 1, static_cast<const int32_t*>(nullptr), d, V, tiles_v, tiles_d, grid_dh,
                         w.live, w.blk_orig, static_cast<uint16_t*>(dH), dW, (accumulate_dW || c0 > 0) ? 1 : 0, rowsel, c0,
                         rows, ids, w.g_c, w.sc);
      UMAS_LAUNCHED("k_gemm_dh_dw");
    }
  }
  hipLaunchKernelGGL(k_ppo_stats, dim3(1), dim3(256), 0, st, nblk, n_roles, entropy_coef, norm_rows, w.blk_stats, stats);
  UMAS_LAUNCHED("k_ppo_stats");
  if (n_sel == 0) return UMAS_OK;
  if (keep) {
    hipLaunchKernelGGL(k_dw_onehot, dim3(cdiv(n_sel, kOneHotRows)), dim3(256), 0, st, Hb, d, rowsel, n_sel, ids, w.g_c, dW);
    UMAS_LAUNCHED("k_dw_onehot");
    return UMAS_OK;
  }

  if (dtype == UMAS_F32) {
    float* dz = reinterpret_cast<float*>(w.chunk);
    for (int64_t c0 = 0; c0 < n_sel; c0 += mc) {
      const int64_t rows = n_sel - c0 < mc ? n_sel - c0 : mc;
      hipLaunchKernelGGL(k_dz_f32, dim3(static_cast<unsigned>(rows)), dim3(256), d * sizeof(float), st,
                         static_cast<const float*>(W), static_cast<const float*>(H), d, V, rowsel, c0, ids,
                         w.score.lse_c, w.g_c, w.score.ent_c, w.kz_c, dz);
      UMAS_LAUNCHED("k_dz_f32");
      hipLaunchKernelGGL(k_dh_f32, dim3(static_cast<unsigned>(rows)), dim3(256), 0, st, dz,
                         static_cast<const float*>(W), d, V, rowsel, c0, static_cast<float*>(dH));
      UMAS_LAUNCHED("k_dh_f32");
      hipLaunchKernelGGL(k_dw_f32, dim3(static_cast<unsigned>(V)), dim3(256), 0, st, dz, static_cast<const float*>(H),
                         d, V, rowsel, c0, rows, (accumulate_dW || c0 > 0) ? 1 : 0, dW);
      UMAS_LAUNCHED("k_dw_f32");
    }
    return UMAS_OK;
  }

  for (int64_t c0 = 0; c0 < n_sel; c0 += mc) {
    const int64_t rows = n_sel - c0 < mc ? n_sel - c0 : mc;
    const int64_t mcp = round_up(rows, 256);
    uint16_t* dZ = reinterpret_cast<uint16_t*>(w.chunk);
    const int tiles_v = static_cast<int>(Vp / 256), tiles_r = static_cast<int>(mcp / 256), tiles_d = (d + 255) / 256;
    hipLaunchKernelGGL(k_dz_tiles, dim3(tile_grid<kGM, kGN>(tiles_v, tiles_r, kTilesPerWg)), dim3(Cfg::T), 0, st, Wb, Hb, d, V, rowsel,
                       c0, rows, w.score.lse_c, w.a_c, w.kz_c, tiles_v, tiles_r, dZ, Vp);
    UMAS_LAUNCHED("k_dz_tiles");
    hipLaunchKernelGGL(k_zero_label, dim3(cdiv(rows, 256)), dim3(256), 0, st, dZ, static_cast<int64_t>(tiles_v), V, rowsel, c0, rows,
                       ids);
    UMAS_LAUNCHED("k_zero_label");
    // with an entropy bonus every row has a gradient: all blocks are live
    const int max_groups = max_dw_groups_per_xcd(tiles_v, tiles_d);
    hipLaunchKernelGGL(k_live_scan, dim3(1), dim3(512), 0, st, static_cast<int>(c0 >> 8), tiles_r, rows, 1, tiles_v, tiles_d, Vp,
                       max_groups, w.blk_live, w.blk_cidx, w.blk_orig, w.live);
    UMAS_LAUNCHED("k_live_scan");
    const unsigned grid_dh = tile_grid<kGM, kGN>(tiles_r, tiles_d);
    hipLaunchKernelGGL(k_gemm_dh_dw, dim3(grid_dh + static_cast<unsigned>(max_groups) * kGM * kGN * 8), dim3(Cfg::T), 0, st,
                       dZ, Vp, mcp, Wb, rowsel ? Hb : Hb + c0 * d, 0, rowsel ? rowsel + c0 : static_cast<const int32_t*>(nullptr), d,
                       V, tiles_v, tiles_d, grid_dh, w.live, w.blk_orig, static_cast<uint16_t*>(dH), dW,
                       (accumulate_dW || c0 > 0) ? 1 : 0, rowsel, c0, rows, ids, w.g_c, static_cast<const float*>(nullptr));
    UMAS_LAUNCHED("k_gemm_dh_dw");
  }
  hipLaunchKernelGGL(k_dw_onehot, dim3(cdiv(n_sel, kOneHotRows)), dim3(256), 0, st, Hb, d, rowsel, n_sel, ids, w.g_c, dW);
  UMAS_LAUNCHED("k_dw_onehot");
  return UMAS_OK;
}
