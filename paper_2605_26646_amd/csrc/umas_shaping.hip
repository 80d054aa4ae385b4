// Token-level shaping around the advantage step: the reference-policy KL folded into the rewards and
// advantage whitening per model or per (model, role).
//
// The worker groups compute "reference-policy log probabilities" next to the old log-probs (Section
// "PPO-Style Training Loop"); the paper prints no penalty, so the per-token estimate
// logp - logp_ref, scaled by beta and subtracted from the token reward, is taken.  Whitening keeps
// role identity (Section "Parameter Sharing in the System": roles stay distinct under sharing), so
// the statistics can be per role inside a model's stream.
// Both are streaming kernels: 16-byte loads and stores, block sums in float64, a fixed-order final
// reduction so that results do not depend on scheduling.
#include "umas_common.h"

namespace umas {
namespace {

constexpr int kST = 256;            // threads per workgroup
constexpr int kSIpt = 8;            // tokens per thread per step
constexpr int kSMaxGrid = 2048;

struct ModelOffsets {
  int64_t off[UMAS_MAX_MODELS + 1];
};

// r_out = r - beta (logp - logp_ref) on mask=1 tokens; per block (sum of logp - logp_ref, count).
__global__ void __launch_bounds__(kST)
k_kl_rewards(int64_t n, const float* r, const float* __restrict__ logp, const float* __restrict__ logp_ref,
             const uint8_t* __restrict__ mask, float beta, float* r_out, double* __restrict__ blk) {   // r_out may be r
  __shared__ double smem[32];
  double ksum = 0.0, cnt = 0.0;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kST * kSIpt;
  for (int64_t p0 = (static_cast<int64_t>(blockIdx.x) * kST + threadIdx.x) * kSIpt; p0 < n; p0 += stride) {
    float rr[kSIpt], a[kSIpt], b[kSIpt];
    uint8_t m[kSIpt];
    if (p0 + kSIpt <= n) {
#pragma unroll
      for (int k = 0; k < kSIpt / 4; ++k) {
        const float4 r4 = *reinterpret_cast<const float4*>(r + p0 + 4 * k);
        const float4 a4 = *reinterpret_cast<const float4*>(logp + p0 + 4 * k);
        const float4 b4 = *reinterpret_cast<const float4*>(logp_ref + p0 + 4 * k);
        rr[4 * k] = r4.x; rr[4 * k + 1] = r4.y; rr[4 * k + 2] = r4.z; rr[4 * k + 3] = r4.w;
        a[4 * k] = a4.x; a[4 * k + 1] = a4.y; a[4 * k + 2] = a4.z; a[4 * k + 3] = a4.w;
        b[4 * k] = b4.x; b[4 * k + 1] = b4.y; b[4 * k + 2] = b4.z; b[4 * k + 3] = b4.w;
      }
      const uint2 m2 = *reinterpret_cast<const uint2*>(mask + p0);
#pragma unroll
      for (int k = 0; k < kSIpt; ++k) m[k] = static_cast<uint8_t>((k < 4 ? m2.x : m2.y) >> (8 * (k & 3)));
    } else {
#pragma unroll
      for (int k = 0; k < kSIpt; ++k) {
        const bool in = p0 + k < n;
        rr[k] = in ? r[p0 + k] : 0.f; a[k] = in ? logp[p0 + k] : 0.f; b[k] = in ? logp_ref[p0 + k] : 0.f;
        m[k] = in ? mask[p0 + k] : 0;
      }
    }
#pragma unroll
    for (int k = 0; k < kSIpt; ++k) {
      const float kl = a[k] - b[k];
      if (m[k]) {
        rr[k] -= beta * kl;
        ksum += static_cast<double>(kl);
        cnt += 1.0;
      }
    }
    if (p0 + kSIpt <= n) {
#pragma unroll
      for (int k = 0; k < kSIpt / 4; ++k)
        *reinterpret_cast<float4*>(r_out + p0 + 4 * k) = make_float4(rr[4 * k], rr[4 * k + 1], rr[4 * k + 2], rr[4 * k + 3]);
    } else {
      for (int k = 0; k < kSIpt && p0 + k < n; ++k) r_out[p0 + k] = rr[k];
    }
  }
  const double s0 = block_sum<double>(ksum, smem);
  __syncthreads();
  const double s1 = block_sum<double>(cnt, smem);
  if (threadIdx.x == 0) {
    blk[2 * blockIdx.x] = s0;
    blk[2 * blockIdx.x + 1] = s1;
  }
}
__global__ void __launch_bounds__(256)
k_kl_mean(const double* __restrict__ blk, int nblk, float* __restrict__ kl_mean) {
  __shared__ double smem[32];
  double a = 0.0, c = 0.0;
  for (int b = threadIdx.x; b < nblk; b += blockDim.x) { a += blk[2 * b]; c += blk[2 * b + 1]; }
  const double s0 = block_sum<double>(a, smem);
  __syncthreads();
  const double s1 = block_sum<double>(c, smem);
  if (threadIdx.x == 0) *kl_mean = s1 > 0 ? static_cast<float>(s0 / s1) : 0.f;
}

// Group of a token: its model (scope MODEL) or model * n_roles + role (scope MODEL_ROLE).
__device__ __forceinline__ int model_of(const ModelOffsets& mo, int n_models, int64_t p) {
  int m = 0;
  while (m + 1 < n_models && mo.off[m + 1] <= p) ++m;
  return m;
}

// Pass 1: per block and group (sum A, sum A^2, count) over the mask=1 tokens, float64.
__global__ void __launch_bounds__(kST)
k_whiten_sums(int64_t n, const float* __restrict__ adv, const uint8_t* __restrict__ mask, const int32_t* __restrict__ role,
              ModelOffsets mo, int n_models, int n_roles, int by_role, double* __restrict__ blk) {
  extern __shared__ double s_acc[];             // [groups][3]
  const int groups = by_role ? n_models * n_roles : n_models;
  for (int i = threadIdx.x; i < groups * 3; i += kST) s_acc[i] = 0.0;
  __syncthreads();
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kST * 4;
  for (int64_t p0 = (static_cast<int64_t>(blockIdx.x) * kST + threadIdx.x) * 4; p0 < n; p0 += stride) {
    float a[4];
    uint8_t m[4];
    int rl[4] = {0, 0, 0, 0};
    if (p0 + 4 <= n) {
      const float4 a4 = *reinterpret_cast<const float4*>(adv + p0);
      const uint32_t m4 = *reinterpret_cast<const uint32_t*>(mask + p0);
      a[0] = a4.x; a[1] = a4.y; a[2] = a4.z; a[3] = a4.w;
#pragma unroll
      for (int k = 0; k < 4; ++k) m[k] = static_cast<uint8_t>(m4 >> (8 * k));
      if (by_role) {
        const int4 r4 = *reinterpret_cast<const int4*>(role + p0);
        rl[0] = r4.x; rl[1] = r4.y; rl[2] = r4.z; rl[3] = r4.w;
      }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const bool in = p0 + k < n;
        a[k] = in ? adv[p0 + k] : 0.f;
        m[k] = in ? mask[p0 + k] : 0;
        rl[k] = (in && by_role) ? role[p0 + k] : 0;
      }
    }
    // group of each of the four tokens (-1 = not counted)
    int gk[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      gk[k] = -1;
      if (!m[k] || (by_role && (rl[k] < 0 || rl[k] >= n_roles))) continue;   // a role outside [0, n_roles) joins no group
      gk[k] = by_role ? model_of(mo, n_models, p0 + k) * n_roles + rl[k] : model_of(mo, n_models, p0 + k);
    }
    // Usual case: every counted token of the wavefront's 256 belongs to one group.  Their sums are formed in
    // float32 across the lanes (256 values: rounding far below the float32 inputs' own) and one lane adds them
    // to the float64 accumulators; otherwise every lane adds its own tokens.
    int g0 = -1;
#pragma unroll
    for (int k = 0; k < 4; ++k) if (gk[k] >= 0 && g0 < 0) g0 = gk[k];
    const unsigned long long have = __ballot(g0 >= 0);
    const int gref = have ? __shfl(g0, __ffsll(static_cast<long long>(have)) - 1, kWave) : -1;
    bool same = true;
#pragma unroll
    for (int k = 0; k < 4; ++k) same = same && (gk[k] < 0 || gk[k] == gref);
    if (__all(same)) {
      if (have) {
        float sa = 0.f, sq = 0.f, sc = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (gk[k] >= 0) { sa += a[k]; sq = fmaf(a[k], a[k], sq); sc += 1.f; }
        sa = wave_sum(sa); sq = wave_sum(sq); sc = wave_sum(sc);
        if ((threadIdx.x & (kWave - 1)) == 0) {
          atomicAdd(s_acc + 3 * gref, static_cast<double>(sa));
          atomicAdd(s_acc + 3 * gref + 1, static_cast<double>(sq));
          atomicAdd(s_acc + 3 * gref + 2, static_cast<double>(sc));
        }
      }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (gk[k] >= 0) {
          const double x = static_cast<double>(a[k]);
          atomicAdd(s_acc + 3 * gk[k], x); atomicAdd(s_acc + 3 * gk[k] + 1, x * x); atomicAdd(s_acc + 3 * gk[k] + 2, 1.0);
        }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < groups * 3; i += kST) blk[static_cast<size_t>(blockIdx.x) * groups * 3 + i] = s_acc[i];
}
// Per group (one workgroup each): mean and 1/sqrt(var + eps) from the block sums, added in a fixed order.
__global__ void __launch_bounds__(256)
k_whiten_stats(const double* __restrict__ blk, int nblk, int groups, float eps, double2* __restrict__ mu_rstd) {
  __shared__ double smem[32];
  const int g = blockIdx.x;
  double v[3] = {0.0, 0.0, 0.0};
  for (int b = threadIdx.x; b < nblk; b += blockDim.x) {
    const double* p = blk + (static_cast<size_t>(b) * groups + g) * 3;
    v[0] += p[0]; v[1] += p[1]; v[2] += p[2];
  }
  double t[3];
  for (int j = 0; j < 3; ++j) {
    t[j] = block_sum<double>(v[j], smem);
    __syncthreads();
  }
  if (threadIdx.x != 0) return;
  double2 o = make_double2(0.0, 1.0);
  if (t[2] > 0) {
    const double mu = t[0] / t[2];
    double var = t[1] / t[2] - mu * mu;
    if (var < 0) var = 0;
    o = make_double2(mu, 1.0 / sqrt(var + static_cast<double>(eps)));
  }
  mu_rstd[g] = o;
}
// Pass 2: A' = (A - mu_g) rstd_g on mask=1 tokens, 0 elsewhere.
__global__ void __launch_bounds__(kST)
k_whiten_apply(int64_t n, const float* adv, const uint8_t* __restrict__ mask, const int32_t* __restrict__ role,
               ModelOffsets mo, int n_models, int n_roles, int by_role, const double2* __restrict__ mu_rstd,
               float* out) {   // out may be adv
  extern __shared__ double2 s_ms[];
  const int groups = by_role ? n_models * n_roles : n_models;
  for (int i = threadIdx.x; i < groups; i += kST) s_ms[i] = mu_rstd[i];
  __syncthreads();
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kST * 4;
  for (int64_t p0 = (static_cast<int64_t>(blockIdx.x) * kST + threadIdx.x) * 4; p0 < n; p0 += stride) {
    float a[4], o[4];
    uint8_t m[4];
    int rl[4] = {0, 0, 0, 0};
    const bool full = p0 + 4 <= n;
    if (full) {
      const float4 a4 = *reinterpret_cast<const float4*>(adv + p0);
      const uint32_t m4 = *reinterpret_cast<const uint32_t*>(mask + p0);
      a[0] = a4.x; a[1] = a4.y; a[2] = a4.z; a[3] = a4.w;
#pragma unroll
      for (int k = 0; k < 4; ++k) m[k] = static_cast<uint8_t>(m4 >> (8 * k));
      if (by_role) {
        const int4 r4 = *reinterpret_cast<const int4*>(role + p0);
        rl[0] = r4.x; rl[1] = r4.y; rl[2] = r4.z; rl[3] = r4.w;
      }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const bool in = p0 + k < n;
        a[k] = in ? adv[p0 + k] : 0.f;
        m[k] = in ? mask[p0 + k] : 0;
        rl[k] = (in && by_role) ? role[p0 + k] : 0;
      }
    }
    const int m0 = model_of(mo, n_models, p0);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      o[k] = 0.f;
      if (m[k] && !(by_role && (rl[k] < 0 || rl[k] >= n_roles))) {
        const int md = (p0 + k < mo.off[m0 + 1] || m0 + 1 >= n_models) ? m0 : model_of(mo, n_models, p0 + k);
        const double2 ms = s_ms[by_role ? md * n_roles + rl[k] : md];
        o[k] = static_cast<float>((static_cast<double>(a[k]) - ms.x) * ms.y);   // the mean in full precision: groups of nearly equal values
      }
    }
    if (full) *reinterpret_cast<float4*>(out + p0) = make_float4(o[0], o[1], o[2], o[3]);
    else
      for (int k = 0; k < 4 && p0 + k < n; ++k) out[p0 + k] = o[k];
  }
}

unsigned stream_grid(int64_t n, int per_block) {
  const int64_t b = (n + per_block - 1) / per_block;
  return static_cast<unsigned>(b < 1 ? 1 : b > kSMaxGrid ? kSMaxGrid : b);
}

}  // namespace
}  // namespace umas

using namespace umas;

extern "C" size_t umas_kl_rewards_workspace_bytes(int64_t n_tokens) {
  if (n_tokens < 0) return 0;
  Carver c(nullptr);
  c.take<double>(2 * static_cast<size_t>(stream_grid(n_tokens, kST * kSIpt)));
  return c.off;
}

extern "C" umas_status umas_kl_rewards(const float* tok_reward, const float* logp, const float* logp_ref,
                                       const uint8_t* tok_mask, int64_t n_tokens, float beta, float* tok_reward_out,
                                       float* kl_mean, void* workspace, size_t workspace_bytes, void* hip_stream) {
  UMAS_REQUIRE(n_tokens >= 0, UMAS_EINVAL, "negative size");
  UMAS_REQUIRE((tok_reward && logp && logp_ref && tok_mask && tok_reward_out) || n_tokens == 0, UMAS_EINVAL,
               "tok_reward, logp, logp_ref, tok_mask and tok_reward_out must not be NULL");
  UMAS_REQUIRE(kl_mean, UMAS_EINVAL, "kl_mean must not be NULL");
  UMAS_REQUIRE(beta == beta, UMAS_EINVAL, "beta must be a number");
  UMAS_REQUIRE(reinterpret_cast<uintptr_t>(tok_reward) % 16 == 0 && reinterpret_cast<uintptr_t>(logp) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(logp_ref) % 16 == 0 && reinterpret_cast<uintptr_t>(tok_mask) % 8 == 0 &&
                   reinterpret_cast<uintptr_t>(tok_reward_out) % 16 == 0,
               UMAS_EINVAL, "token arrays must be 16-byte aligned (the mask 8-byte)");
  const size_t need = umas_kl_rewards_workspace_bytes(n_tokens);
  UMAS_REQUIRE(workspace && reinterpret_cast<uintptr_t>(workspace) % kAlign == 0 && workspace_bytes >= need, UMAS_EWORKSPACE,
               "workspace must be 256-byte aligned and hold %zu bytes (got %zu)", need, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  const unsigned grid = stream_grid(n_tokens, kST * kSIpt);
  double* blk = static_cast<double*>(workspace);
  hipLaunchKernelGGL(k_kl_rewards, dim3(grid), dim3(kST), 0, st, n_tokens, tok_reward, logp, logp_ref, tok_mask, beta,
                     tok_reward_out, blk);
  UMAS_LAUNCHED("k_kl_rewards");
  hipLaunchKernelGGL(k_kl_mean, dim3(1), dim3(256), 0, st, blk, static_cast<int>(grid), kl_mean);
  UMAS_LAUNCHED("k_kl_mean");
  return UMAS_OK;
}

extern "C" size_t umas_whiten_workspace_bytes(int64_t n_tokens, int32_t n_models, int32_t n_roles) {
  if (n_tokens < 0 || n_models < 1 || n_roles < 1) return 0;
  Carver c(nullptr);
  const size_t groups = static_cast<size_t>(n_models) * n_roles;
  c.take<double>(static_cast<size_t>(stream_grid(n_tokens, kST * 4)) * groups * 3);
  c.take<double2>(groups);
  return c.off;
}

extern "C" umas_status umas_whiten_advantages(const float* adv, const uint8_t* tok_mask, const int32_t* tok_role,
                                              const int64_t* model_tok_off, int32_t n_models, int32_t n_roles,
                                              int64_t n_tokens, int32_t scope, float eps, float* adv_out,
                                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  UMAS_REQUIRE(n_tokens >= 0, UMAS_EINVAL, "negative size");
  UMAS_REQUIRE(n_models >= 1 && n_models <= UMAS_MAX_MODELS, UMAS_ESHAPE, "n_models=%d outside [1,%d]", n_models, UMAS_MAX_MODELS);
  UMAS_REQUIRE(n_roles >= 1 && n_roles <= UMAS_MAX_ROLES, UMAS_ESHAPE, "n_roles=%d outside [1,%d]", n_roles, UMAS_MAX_ROLES);
  UMAS_REQUIRE(scope == UMAS_WHITEN_MODEL || scope == UMAS_WHITEN_MODEL_ROLE, UMAS_EINVAL, "scope=%d is neither MODEL nor MODEL_ROLE", scope);
  UMAS_REQUIRE(eps > 0.f, UMAS_EINVAL, "eps must be positive");
  UMAS_REQUIRE(model_tok_off, UMAS_EINVAL, "model_tok_off must not be NULL");
  UMAS_REQUIRE(model_tok_off[0] == 0 && model_tok_off[n_models] == n_tokens, UMAS_EINVAL, "model_tok_off must run from 0 to n_tokens");
  for (int m = 0; m < n_models; ++m)
    UMAS_REQUIRE(model_tok_off[m] <= model_tok_off[m + 1], UMAS_EINVAL, "model_tok_off decreases at %d", m);
  const int by_role = scope == UMAS_WHITEN_MODEL_ROLE ? 1 : 0;
  UMAS_REQUIRE((adv && tok_mask && adv_out && (tok_role || !by_role)) || n_tokens == 0, UMAS_EINVAL,
               "adv, tok_mask, adv_out (and tok_role for the per-role scope) must not be NULL");
  UMAS_REQUIRE(reinterpret_cast<uintptr_t>(adv) % 16 == 0 && reinterpret_cast<uintptr_t>(adv_out) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(tok_mask) % 4 == 0 && reinterpret_cast<uintptr_t>(tok_role) % 16 == 0,
               UMAS_EINVAL, "token arrays must be 16-byte aligned (the mask 4-byte)");
  const size_t need = umas_whiten_workspace_bytes(n_tokens, n_models, n_roles);
  UMAS_REQUIRE(workspace && reinterpret_cast<uintptr_t>(workspace) % kAlign == 0 && workspace_bytes >= need, UMAS_EWORKSPACE,
               "workspace must be 256-byte aligned and hold %zu bytes (got %zu)", need, workspace_bytes);
  if (n_tokens == 0) return UMAS_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  ModelOffsets mo;
  for (int m = 0; m <= UMAS_MAX_MODELS; ++m) mo.off[m] = m <= n_models ? model_tok_off[m] : n_tokens;
  const int groups = by_role ? n_models * n_roles : n_models;
  const unsigned grid = stream_grid(n_tokens, kST * 4);
  Carver c(workspace);
  double* blk = c.take<double>(static_cast<size_t>(grid) * n_models * n_roles * 3);
  double2* ms = c.take<double2>(static_cast<size_t>(n_models) * n_roles);
  hipLaunchKernelGGL(k_whiten_sums, dim3(grid), dim3(kST), groups * 3 * sizeof(double), st, n_tokens, adv, tok_mask, tok_role,
                     mo, n_models, n_roles, by_role, blk);
  UMAS_LAUNCHED("k_whiten_sums");
  hipLaunchKernelGGL(k_whiten_stats, dim3(groups), dim3(256), 0, st, blk, static_cast<int>(grid), groups, eps, ms);
  UMAS_LAUNCHED("k_whiten_stats");
  hipLaunchKernelGGL(k_whiten_apply, dim3(grid), dim3(kST), groups * sizeof(double2), st, n_tokens, adv, tok_mask, tok_role, mo,
                     n_models, n_roles, by_role, ms, adv_out);
  UMAS_LAUNCHED("k_whiten_apply");
  return UMAS_OK;
}
