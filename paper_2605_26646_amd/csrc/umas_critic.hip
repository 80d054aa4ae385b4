// Critic: value head V = w . h + b on the selected rows, clipped value loss and its backward.
//
// The worker groups of Section "PPO-Style Training Loop" compute value estimates next to the
// log-probs and update "actor and critic" from the ready batch.  The paper prints no value loss; the
// clipped form used with PPO is taken:
//   Vc = clip(V, V_old - eps, V_old + eps);  L = 1/2 max((V - R)^2, (Vc - R)^2);  loss = mean L
//   g = dloss/dV = (V - R) / S where the unclipped term is the larger one (ties included), else 0
//   dH_i = g_i w,  dw = sum_i g_i h_i,  db = sum_i g_i
// The whole step is one pass over H: one wavefront per row keeps the row in registers, forms the dot
// product and the row's g, writes dH and adds g h to its dw accumulators; the next row is already in
// flight.  Per-wavefront partial sums are reduced by small kernels in a fixed order, so results do not
// depend on scheduling.
#include <type_traits>

#include <algorithm>

#include "umas_common.h"

namespace umas {
namespace {

constexpr int kVT = 256;                 // threads per workgroup
constexpr int kVWaves = kVT / kWave;
constexpr int kMaxKV = 16;               // 16-byte column vectors per lane: d <= 64 * 16 * (8 bf16 | 4 float)
constexpr int kMaxGrid = 1024;           // workgroups of the row kernel at most (the launch takes no more than are resident at once)
constexpr int kVStat = 4;                // (sum L, clipped rows, sum V, rows)

__device__ __forceinline__ uint16_t f2bf(float x) { return __builtin_bit_cast(uint16_t, static_cast<__bf16>(x)); }

// Sums over a row and over rows: float for bf16 inputs (every product is exact in float), float64 for float32
// inputs, whose bar is 1e-5 and whose speed does not matter (a float sum of d float32 products loses up to
// d 2^-24 of the sum of their magnitudes, which the difference V - R then magnifies).
template <typename T> using AccT = std::conditional_t<std::is_same<T, float>::value, double, float>;

// 16 bytes of a row as floats: 8 bf16 or 4 float
template <typename T> struct Vec;
template <> struct Vec<uint16_t> {
  static constexpr int N = 8;
  __device__ static void load(const uint16_t* p, float (&x)[8]) { unpack(*reinterpret_cast<const uint4*>(p), x); }
  __device__ static void unpack(const uint4& v, float (&x)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(w[i] << 16);
      x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  __device__ static void store(uint16_t* p, const float (&x)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = static_cast<uint32_t>(f2bf(x[2 * i])) | (static_cast<uint32_t>(f2bf(x[2 * i + 1])) << 16);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};
template <> struct Vec<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float (&x)[4]) { unpack(*reinterpret_cast<const uint4*>(p), x); }
  __device__ static void unpack(const uint4& v, float (&x)[4]) {
    x[0] = __uint_as_float(v.x); x[1] = __uint_as_float(v.y); x[2] = __uint_as_float(v.z); x[3] = __uint_as_float(v.w);
  }
  __device__ static void store(float* p, const float (&x)[4]) { *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]); }
};

__global__ void k_zero_u32(uint32_t* __restrict__ p, int64_t n) {
  int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (; i < n; i += stride) p[i] = 0u;
}

// Forward only: one wavefront per selected row.
template <typename T>
__global__ void __launch_bounds__(kVT)
k_value_fwd(const T* __restrict__ H, const T* __restrict__ w, float bias, int d, const int32_t* __restrict__ rowsel,
            int64_t n_sel, float* __restrict__ value) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t n = static_cast<int64_t>(blockIdx.x) * kVWaves + threadIdx.x / kWave;
  if (n >= n_sel) return;
  const int64_t row = rowsel ? rowsel[n] : n;
  const T* h = H + row * d;
  AccT<T> acc = 0;
  for (int c = lane * Vec<T>::N; c < d; c += kWave * Vec<T>::N) {
    float x[Vec<T>::N], y[Vec<T>::N];
    Vec<T>::load(h + c, x);
    Vec<T>::load(w + c, y);
#pragma unroll
    for (int i = 0; i < Vec<T>::N; ++i) acc = fma(static_cast<AccT<T>>(x[i]), static_cast<AccT<T>>(y[i]), acc);
  }
  acc = wave_sum(acc);
  if (lane == 0) value[row] = static_cast<float>(acc + static_cast<AccT<T>>(bias));
}

// Loss and backward, one wavefront per row.  Lane l owns the 16-byte column vectors l, l + 64, ... (KV of them):
// it keeps its part of w, of the current row and of the next row (prefetched) in registers, and its part of
// dw in float accumulators over all rows of the wavefront.  No barrier in the row loop.
template <typename T, int KV>
__global__ void __launch_bounds__(kVT)
k_value_rows(const T* __restrict__ H, const T* __restrict__ w, float bias, int d, const int32_t* __restrict__ rowsel,
             int64_t n_sel, int64_t norm, int64_t rows_per_block, const float* __restrict__ value_old, const float* __restrict__ ret,
             const int32_t* __restrict__ tok_role, int n_roles, float clip_eps, float* __restrict__ value_new,
             T* __restrict__ dH, int accumulate_dH, float* __restrict__ part_dw, double* __restrict__ blk_stats) {
  __shared__ double s_acc[(1 + UMAS_MAX_ROLES) * kVStat];
  constexpr int N = Vec<T>::N;
  const int nvec = d / N;
  const int nacc = (1 + n_roles) * kVStat;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  for (int i = threadIdx.x; i < nacc; i += kVT) s_acc[i] = 0.0;
  __syncthreads();
  // w and the rows stay packed as loaded (16 bytes per vector) and are unpacked where they are used
  using A = AccT<T>;
  uint4 wp[KV];
  A acc[KV][N];
#pragma unroll
  for (int k = 0; k < KV; ++k) {
    const int cv = lane + k * kWave;
#pragma unroll
    for (int i = 0; i < N; ++i) acc[k][i] = 0;
    wp[k] = make_uint4(0u, 0u, 0u, 0u);
    if (cv < nvec) wp[k] = *reinterpret_cast<const uint4*>(w + cv * N);
  }
  float gsum = 0.f;
  const float inv_s = 1.f / static_cast<float>(norm);
  const int64_t r_begin = static_cast<int64_t>(blockIdx.x) * rows_per_block;
  const int64_t r_end = r_begin + rows_per_block < n_sel ? r_begin + rows_per_block : n_sel;

  uint4 cur[KV], nxt[KV];
  float vo_next = 0.f, ret_next = 0.f;               // the next row's old value and return come with the row
  auto fetch = [&](int64_t n) {
    const int64_t row = rowsel ? rowsel[n] : n;
#pragma unroll
    for (int k = 0; k < KV; ++k) {
      const int cv = lane + k * kWave;
      nxt[k] = make_uint4(0u, 0u, 0u, 0u);
      if (cv < nvec) nxt[k] = *reinterpret_cast<const uint4*>(H + row * d + cv * N);
    }
    vo_next = value_old[row];
    ret_next = ret[row];
    return row;
  };
  int64_t n = r_begin + wave;
  int64_t row_next = n < r_end ? fetch(n) : 0;
  for (; n < r_end; n += kVWaves) {
    const int64_t row = row_next;
    const float vo = vo_next, R = ret_next;
    A dot = 0;
#pragma unroll
    for (int k = 0; k < KV; ++k) {
      cur[k] = nxt[k];
      float x[N], y[N];
      Vec<T>::unpack(cur[k], x);
      Vec<T>::unpack(wp[k], y);
#pragma unroll
      for (int i = 0; i < N; ++i) dot = fma(static_cast<A>(x[i]), static_cast<A>(y[i]), dot);
    }
    if (n + kVWaves < r_end) row_next = fetch(n + kVWaves);     // in flight while this row is finished
    dot = wave_sum(dot);
    // the value is a float32 result; loss and gradient are formed from that rounded value
    const float V = static_cast<float>(dot + static_cast<A>(bias));
    const float vc = fminf(fmaxf(V, vo - clip_eps), vo + clip_eps);   // V itself inside the range: an exact tie
    const float lu = (V - R) * (V - R), lc = (vc - R) * (vc - R);
    const bool unclipped = lu >= lc;
    const float g = unclipped ? (V - R) * inv_s : 0.f;
    gsum += g;
    if (lane == 0) {
      if (value_new) value_new[row] = V;
      const int role = (tok_role && n_roles > 0) ? tok_role[row] : -1;
      for (int pass = 0; pass < 2; ++pass) {
        if (pass == 1 && (role < 0 || role >= n_roles)) break;
        double* a = s_acc + (pass == 0 ? 0 : (1 + role) * kVStat);
        atomicAdd(a + 0, static_cast<double>(0.5f * (unclipped ? lu : lc)));
        atomicAdd(a + 1, unclipped ? 0.0 : 1.0);
        atomicAdd(a + 2, static_cast<double>(V));
        atomicAdd(a + 3, 1.0);
      }
    }
#pragma unroll
    for (int k = 0; k < KV; ++k) {
      const int cv = lane + k * kWave;
      if (cv < nvec) {
        float x[N], y[N], o[N];
        Vec<T>::unpack(cur[k], x);
        Vec<T>::unpack(wp[k], y);
        if (accumulate_dH) Vec<T>::load(dH + row * d + cv * N, o);
#pragma unroll
        for (int i = 0; i < N; ++i) {
          acc[k][i] = fma(static_cast<A>(g), static_cast<A>(x[i]), acc[k][i]);
          o[i] = accumulate_dH ? o[i] + g * y[i] : g * y[i];
        }
        Vec<T>::store(dH + row * d + cv * N, o);
      }
    }
  }
  // every wavefront leaves its own partial row: [blocks * waves][d + 1]
  float* pd = part_dw + (static_cast<size_t>(blockIdx.x) * kVWaves + wave) * (d + 1);
#pragma unroll
  for (int k = 0; k < KV; ++k) {
    const int cv = lane + k * kWave;
    if (cv < nvec)
#pragma unroll
      for (int i = 0; i < N; ++i) pd[cv * N + i] = static_cast<float>(acc[k][i]);
  }
  if (lane == 0) pd[d] = gsum;
  __syncthreads();
  for (int i = threadIdx.x; i < nacc; i += kVT) blk_stats[static_cast<size_t>(blockIdx.x) * nacc + i] = s_acc[i];
}

// out[o][j] = sum of the rows o*group .. o*group + group - 1 of in[n_in][ld] (fixed order); the last stage adds
// into or overwrites dw (columns < d) and db (column d).
__global__ void __launch_bounds__(256)
k_value_reduce(const float* __restrict__ in, int n_in, int ld, int group, float* __restrict__ out, int d, int final_stage,
               int accumulate, float* __restrict__ dw, float* __restrict__ db) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int o = blockIdx.y;
  if (j >= ld) return;
  const int b0 = o * group, b1 = b0 + group < n_in ? b0 + group : n_in;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  int b = b0;
  for (; b + 4 <= b1; b += 4) {
    s0 += in[static_cast<size_t>(b) * ld + j];
    s1 += in[static_cast<size_t>(b + 1) * ld + j];
    s2 += in[static_cast<size_t>(b + 2) * ld + j];
    s3 += in[static_cast<size_t>(b + 3) * ld + j];
  }
  for (; b < b1; ++b) s0 += in[static_cast<size_t>(b) * ld + j];
  const float s = (s0 + s1) + (s2 + s3);
  if (!final_stage) {
    out[static_cast<size_t>(o) * ld + j] = s;
  } else {
    float* dst = j < d ? dw + j : db;
    if (dst) *dst = accumulate ? *dst + s : s;
  }
}
__global__ void __launch_bounds__(256)
k_value_stats(int nblk, int n_roles, int64_t norm_rows, const double* __restrict__ blk_stats, umas_value_stats* __restrict__ stats) {
  __shared__ double smem[32];
  const int nacc = (1 + n_roles) * kVStat;
  for (int k = 0; k <= n_roles; ++k) {
    double sum[kVStat];
    for (int j = 0; j < kVStat; ++j) {
      double v = 0.0;
      for (int b = threadIdx.x; b < nblk; b += blockDim.x) v += blk_stats[static_cast<size_t>(b) * nacc + k * kVStat + j];
      sum[j] = block_sum<double>(v, smem);
    }
    if (threadIdx.x == 0) {
      const double cnt = sum[3];
      umas_value_stats s;
      const double den = (k == 0 && norm_rows > 0) ? static_cast<double>(norm_rows) : cnt;   // the caller's normaliser
      s.loss = cnt > 0 ? static_cast<float>(sum[0] / den) : 0.f;
      s.clip_frac = cnt > 0 ? static_cast<float>(sum[1] / cnt) : 0.f;
      s.value_mean = cnt > 0 ? static_cast<float>(sum[2] / cnt) : 0.f;
      s.reserved = 0.f;
      s.n_scored = static_cast<int64_t>(cnt);
      stats[k] = s;
    }
  }
}

constexpr int kReduceGroup = 64;
unsigned value_grid(int64_t n_sel) {
  const int64_t b = (n_sel + kVWaves - 1) / kVWaves;
  return static_cast<unsigned>(b < 1 ? 1 : b > kMaxGrid ? kMaxGrid : b);
}
int max_d(umas_dtype dt) { return dt == UMAS_BF16 ? kWave * kMaxKV * 8 : kWave * kMaxKV * 4; }

// Workgroups of the row kernel that the device holds at once (the kernel's register use differs with KV): its grid is
// one resident round, so that no second, partly filled round follows.  Looked up once per instance.
template <typename T, int K>
unsigned resident_value_blocks() {
  static unsigned cached = 0;
  if (cached) return cached;
  int dev = 0, n_cu = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    n_cu = 64;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_value_rows<T, K>, kVT, 0) != hipSuccess || per_cu < 1) per_cu = 1;
  cached = static_cast<unsigned>(per_cu) * static_cast<unsigned>(n_cu);
  return cached;
}

template <typename T>
unsigned resident_value_blocks_kv(int kv) {
  if (kv <= 1) return resident_value_blocks<T, 1>();
  if (kv <= 2) return resident_value_blocks<T, 2>();
  if (kv <= 4) return resident_value_blocks<T, 4>();
  if (kv <= 8) return resident_value_blocks<T, 8>();
  return resident_value_blocks<T, 16>();
}

template <typename T>
void launch_value_rows(int kv, unsigned grid, hipStream_t st, const void* H, const void* w, float bias, int d,
                       const int32_t* rowsel, int64_t n_sel, int64_t norm, int64_t rpb, const float* value_old, const float* ret,
                       const int32_t* tok_role, int n_roles, float clip_eps, float* value_new, void* dH, int acc_dH,
                       float* part_dw, double* blk_stats) {
#define UMAS_VALUE_CASE(K)                                                                                              \
  hipLaunchKernelGGL((k_value_rows<T, K>), dim3(grid), dim3(kVT), 0, st, static_cast<const T*>(H), static_cast<const T*>(w), \
                     bias, d, rowsel, n_sel, norm, rpb, value_old, ret, tok_role, n_roles, clip_eps, value_new,         \
                     static_cast<T*>(dH), acc_dH, part_dw, blk_stats)
  if (kv <= 1) UMAS_VALUE_CASE(1);
  else if (kv <= 2) UMAS_VALUE_CASE(2);
  else if (kv <= 4) UMAS_VALUE_CASE(4);
  else if (kv <= 8) UMAS_VALUE_CASE(8);
  else UMAS_VALUE_CASE(16);
#undef UMAS_VALUE_CASE
}

umas_status check_value_args(const void* H, const void* w, umas_dtype dt, int64_t n_rows, int d, const int32_t* rowsel,
                             int64_t n_sel) {
  UMAS_REQUIRE(dt == UMAS_F32 || dt == UMAS_BF16, UMAS_EDTYPE, "dtype=%d is neither F32 nor BF16", static_cast<int>(dt));
  UMAS_REQUIRE(n_rows >= 0 && n_sel >= 0 && n_sel <= n_rows, UMAS_EINVAL, "row counts must satisfy 0 <= n_sel <= n_rows");
  UMAS_REQUIRE(rowsel || n_sel == n_rows, UMAS_EINVAL, "rowsel is NULL but n_sel != n_rows");
  const int n = dt == UMAS_BF16 ? 8 : 4;
  UMAS_REQUIRE(d >= n && d % n == 0 && d <= max_d(dt), UMAS_ESHAPE, "d=%d must be a multiple of %d and at most %d", d, n, max_d(dt));
  UMAS_REQUIRE((H || n_rows == 0) && w, UMAS_EINVAL, "H and w must not be NULL");
  UMAS_REQUIRE(reinterpret_cast<uintptr_t>(H) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0, UMAS_EINVAL,
               "H and w must be 16-byte aligned");
  return UMAS_OK;
}

}  // namespace
}  // namespace umas

using namespace umas;

extern "C" size_t umas_value_workspace_bytes(int64_t n_sel, int32_t d, umas_dtype dtype, int32_t n_roles) {
  if (n_sel < 0 || d < 1 || n_roles < 0) return 0;
  (void)dtype;
  const unsigned grid = value_grid(n_sel);
  Carver c(nullptr);
  c.take<float>(static_cast<size_t>(grid) * kVWaves * (d + 1));                                  // one partial row per wavefront
  c.take<float>(static_cast<size_t>(cdiv(grid * kVWaves, kReduceGroup)) * (d + 1));             // first reduction stage
  c.take<double>(static_cast<size_t>(grid) * (1 + n_roles) * kVStat);
  return c.off;
}

extern "C" umas_status umas_values(const void* H, const void* w, float bias, umas_dtype dtype, int64_t n_rows, int32_t d,
                                   const int32_t* rowsel, int64_t n_sel, float* value, void* hip_stream) {
  umas_status s = check_value_args(H, w, dtype, n_rows, d, rowsel, n_sel);
  if (s != UMAS_OK) return s;
  UMAS_REQUIRE(value || n_rows == 0, UMAS_EINVAL, "value must not be NULL");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  if (rowsel && n_rows > 0) {
    hipLaunchKernelGGL(k_zero_u32, dim3(cdiv(n_rows, 1024) < 4096 ? cdiv(n_rows, 1024) : 4096), dim3(256), 0, st,
                       reinterpret_cast<uint32_t*>(value), n_rows);
    UMAS_LAUNCHED("k_zero_u32");
  }
  if (n_sel == 0) return UMAS_OK;
  if (dtype == UMAS_BF16)
    hipLaunchKernelGGL(k_value_fwd<uint16_t>, dim3(cdiv(n_sel, kVWaves)), dim3(kVT), 0, st, static_cast<const uint16_t*>(H),
                       static_cast<const uint16_t*>(w), bias, d, rowsel, n_sel, value);
  else
    hipLaunchKernelGGL(k_value_fwd<float>, dim3(cdiv(n_sel, kVWaves)), dim3(kVT), 0, st, static_cast<const float*>(H),
                       static_cast<const float*>(w), bias, d, rowsel, n_sel, value);
  UMAS_LAUNCHED("k_value_fwd");
  return UMAS_OK;
}

extern "C" umas_status umas_value_loss_fwd_bwd(const void* H, const void* w, float bias, umas_dtype dtype, int64_t n_rows,
                                               int32_t d, const int32_t* rowsel, int64_t n_sel, const float* value_old,
                                               const float* ret, const int32_t* tok_role, int32_t n_roles,
                                               float clip_eps_v, int32_t accumulate_dH, int32_t accumulate_dw,
                                               int64_t norm_rows, umas_value_stats* stats, float* value_new, void* dH, float* dw, float* db,
                                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  umas_status s = check_value_args(H, w, dtype, n_rows, d, rowsel, n_sel);
  if (s != UMAS_OK) return s;
  UMAS_REQUIRE(n_roles >= 0 && n_roles <= UMAS_MAX_ROLES, UMAS_ESHAPE, "n_roles=%d outside [0,%d]", n_roles, UMAS_MAX_ROLES);
  UMAS_REQUIRE(clip_eps_v > 0.f, UMAS_EINVAL, "clip_eps_v must be positive");
  UMAS_REQUIRE(stats && dw && (dH || n_rows == 0), UMAS_EINVAL, "stats, dw and dH must not be NULL");
  UMAS_REQUIRE((value_old && ret) || n_sel == 0, UMAS_EINVAL, "value_old and ret must not be NULL");
  UMAS_REQUIRE(reinterpret_cast<uintptr_t>(dH) % 16 == 0, UMAS_EINVAL, "dH must be 16-byte aligned");
  UMAS_REQUIRE(norm_rows == 0 || norm_rows >= n_sel, UMAS_EINVAL, "norm_rows=%lld must be 0 or at least n_sel=%lld",
               static_cast<long long>(norm_rows), static_cast<long long>(n_sel));
  const int64_t norm = norm_rows > 0 ? norm_rows : n_sel;   // rows the mean is taken over
  const size_t need = umas_value_workspace_bytes(n_sel, d, dtype, n_roles);
  UMAS_REQUIRE(workspace && reinterpret_cast<uintptr_t>(workspace) % kAlign == 0 && workspace_bytes >= need, UMAS_EWORKSPACE,
               "workspace must be 256-byte aligned and hold %zu bytes (got %zu)", need, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  const size_t esz = dtype == UMAS_BF16 ? 2 : 4;
  const int nvec = d / (dtype == UMAS_BF16 ? 8 : 4);
  const int kv = (nvec + kWave - 1) / kWave;
  // at most value_grid(n_sel) workgroups (what the workspace is sized for), and no more than are resident at once
  const unsigned resident = dtype == UMAS_BF16 ? resident_value_blocks_kv<uint16_t>(kv) : resident_value_blocks_kv<float>(kv);
  const unsigned grid = std::min(value_grid(n_sel), resident);
  const int n_part = static_cast<int>(grid) * kVWaves, n_part2 = static_cast<int>(cdiv(n_part, kReduceGroup));
  Carver c(workspace);
  float* part_dw = c.take<float>(static_cast<size_t>(n_part) * (d + 1));
  float* part2 = c.take<float>(static_cast<size_t>(n_part2) * (d + 1));
  double* blk_stats = c.take<double>(static_cast<size_t>(grid) * (1 + n_roles) * kVStat);

  auto zero = [&](void* p, size_t bytes) -> hipError_t {
    const int64_t n = static_cast<int64_t>(bytes / 4);
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_zero_u32, dim3(cdiv(n, 1024) < 8192 ? cdiv(n, 1024) : 8192), dim3(256), 0, st,
                       static_cast<uint32_t*>(p), n);
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess && g_prof_on) prof_kernel("k_zero_u32", st);
    return e;
  };
  if (rowsel && n_rows > 0) {
    if (value_new) UMAS_HIP(zero(value_new, n_rows * sizeof(float)));
    if (!accumulate_dH) UMAS_HIP(zero(dH, static_cast<size_t>(n_rows) * d * esz));
  }
  if (n_sel > 0) {
    const int64_t rpb = (n_sel + grid - 1) / grid;                 // rows per workgroup; every wavefront writes its partial row
    if (dtype == UMAS_BF16)
      launch_value_rows<uint16_t>(kv, grid, st, H, w, bias, d, rowsel, n_sel, norm, rpb, value_old, ret, tok_role, n_roles,
                                  clip_eps_v, value_new, dH, accumulate_dH, part_dw, blk_stats);
    else
      launch_value_rows<float>(kv, grid, st, H, w, bias, d, rowsel, n_sel, norm, rpb, value_old, ret, tok_role, n_roles,
                               clip_eps_v, value_new, dH, accumulate_dH, part_dw, blk_stats);
    UMAS_LAUNCHED("k_value_rows");
  } else {
    // an empty selection still defines the outputs: zero partials give zero statistics and gradients
    UMAS_HIP(zero(part_dw, static_cast<size_t>(n_part) * (d + 1) * sizeof(float)));
    UMAS_HIP(zero(blk_stats, static_cast<size_t>(grid) * (1 + n_roles) * kVStat * sizeof(double)));
  }
  hipLaunchKernelGGL(k_value_reduce, dim3(cdiv(d + 1, 256), n_part2), dim3(256), 0, st, part_dw, n_part, d + 1, kReduceGroup,
                     part2, d, 0, 0, static_cast<float*>(nullptr), static_cast<float*>(nullptr));
  UMAS_LAUNCHED("k_value_reduce");
  hipLaunchKernelGGL(k_value_reduce, dim3(cdiv(d + 1, 256), 1), dim3(256), 0, st, part2, n_part2, d + 1, n_part2,
                     static_cast<float*>(nullptr), d, 1, accumulate_dw, dw, db);
  UMAS_LAUNCHED("k_value_reduce");
  hipLaunchKernelGGL(k_value_stats, dim3(1), dim3(256), 0, st, static_cast<int>(grid), n_roles, norm_rows, blk_stats, stats);
  UMAS_LAUNCHED("k_value_stats");
  return UMAS_OK;
}
