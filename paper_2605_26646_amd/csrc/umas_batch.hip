// Ready-batch construction: a model-local buffer becomes a batch ready for the update by dropping
// incomplete trajectories, shuffling, and cutting what is left into minibatches that match the worker
// group's configuration (Section "Model-Local Buffers", B_i -> D_i^ready).
//
// The shuffle is an input (a permutation of the trajectories).  The kept trajectories, in shuffled
// order, are cut into n_minibatch contiguous parts whose sizes differ by at most one; for every model
// and minibatch the scored rows of its trajectories are listed trajectory by trajectory in shuffled
// order, rows of one trajectory in stream order.  All of it is index work on the streams that
// umas_assign_token_rewards wrote: a trajectory's turns are contiguous inside a stream (one "trajectory
// run"), so a run's rows are one slice of rowsel, and minibatches are built by moving slices.
#include <vector>

#include "umas_common.h"

namespace umas {
namespace {

constexpr int kScanItems = 8;
constexpr int kScanTile = 256 * kScanItems;       // entries one workgroup scans

// flag[q] = 1 when the q-th trajectory of the shuffle is kept.
__global__ void k_kept_flags(int n_traj, const int32_t* __restrict__ order, const uint8_t* __restrict__ keep,
                             int64_t* __restrict__ flag) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= n_traj) return;
  const int b = order ? order[q] : q;
  flag[q] = (!keep || keep[b]) ? 1 : 0;
}
// rank[b] = position of trajectory b among the kept trajectories in shuffled order (pos = scanned flags), or -1.
__global__ void k_kept_rank(int n_traj, const int32_t* __restrict__ order, const uint8_t* __restrict__ keep,
                            const int64_t* __restrict__ pos, int32_t* __restrict__ rank) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= n_traj) return;
  const int b = order ? order[q] : q;
  rank[b] = (!keep || keep[b]) ? static_cast<int32_t>(pos[q]) : -1;
}

// Exclusive prefix sums of the rows of data[nrows][n] in three steps: every workgroup scans its tile of a row in
// place and leaves the tile's total, the totals of a row are scanned by one workgroup, the tiles add their offset.
__global__ void __launch_bounds__(256)
k_scan_tiles(int64_t* __restrict__ data, int n, int ntile, int64_t* __restrict__ tile_sum) {
  __shared__ int64_t smem[32];
  int64_t* row = data + static_cast<size_t>(blockIdx.y) * n;
  const int base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
  int64_t v[kScanItems];
  int64_t sum = 0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    v[k] = base + k < n ? row[base + k] : 0;
    sum += v[k];
  }
  int64_t total;
  int64_t r = block_excl_scan<int64_t>(sum, smem, &total);
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    if (base + k < n) row[base + k] = r;
    r += v[k];
  }
  if (threadIdx.x == 0) tile_sum[static_cast<size_t>(blockIdx.y) * ntile + blockIdx.x] = total;
}
__global__ void __launch_bounds__(256)
k_scan_add(int64_t* __restrict__ data, int n, int ntile, const int64_t* __restrict__ tile_off) {
  int64_t* row = data + static_cast<size_t>(blockIdx.y) * n;
  const int64_t off = tile_off[static_cast<size_t>(blockIdx.y) * ntile + blockIdx.x];
  const int base = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k)
    if (base + k < n) row[base + k] += off;
}

// First index i in [0, n) with a[i] >= x (n if none).
__device__ __forceinline__ int64_t lower_bound_i32(const int32_t* __restrict__ a, int64_t n, int64_t x) {
  int64_t lo = 0, hi = n;
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (a[mid] < x) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// Per trajectory run: its model, trajectory and the slice of rowsel that holds its scored rows; written
// at (model, rank of the trajectory) when the trajectory is kept.
__global__ void k_run_slices(int n_turns, int n_traj, int n_models, const int64_t* __restrict__ traj_seg_off,
                             const int32_t* __restrict__ model_trajrun_off, const int64_t* __restrict__ model_tok_off,
                             const int64_t* __restrict__ model_rowsel_off, const int32_t* __restrict__ rowsel,
                             const int32_t* __restrict__ tok_turn, const int32_t* __restrict__ traj_turn_off,
                             const int32_t* __restrict__ rank, int64_t* __restrict__ cnt_mq, int64_t* __restrict__ src_mq) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n_turns || j >= model_trajrun_off[n_models]) return;
  const int64_t start = traj_seg_off[j], end = traj_seg_off[j + 1];
  if (end <= start) return;
  int m = 0;
  while (m + 1 < n_models && model_trajrun_off[m + 1] <= j) ++m;
  const int u = tok_turn[start];
  int lo = 0, hi = n_traj;                         // trajectory of turn u: last b with traj_turn_off[b] <= u
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (traj_turn_off[mid] <= u) lo = mid; else hi = mid - 1;
  }
  const int q = rank[lo];
  if (q < 0) return;
  const int64_t ra = model_rowsel_off[m], n_m = model_rowsel_off[m + 1] - ra, t0 = model_tok_off[m];
  const int64_t i0 = lower_bound_i32(rowsel + ra, n_m, start - t0), i1 = lower_bound_i32(rowsel + ra, n_m, end - t0);
  cnt_mq[static_cast<size_t>(m) * n_traj + q] = i1 - i0;
  src_mq[static_cast<size_t>(m) * n_traj + q] = ra + i0;
}

// In-place exclusive prefix sum of each row of data[nrows][n]; one block per row, 8 entries per thread per round.
__global__ void __launch_bounds__(1024)
k_scan_rows(int64_t* __restrict__ data, int n, int64_t* __restrict__ totals) {
  __shared__ int64_t smem[32];
  int64_t* row = data + static_cast<size_t>(blockIdx.x) * n;
  int64_t carry = 0;
  for (int i0 = 0; i0 < n; i0 += blockDim.x * kScanItems) {
    const int base = i0 + threadIdx.x * kScanItems;
    int64_t v[kScanItems];
    int64_t sum = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
      v[k] = base + k < n ? row[base + k] : 0;
      sum += v[k];
    }
    int64_t total;
    int64_t r = carry + block_excl_scan<int64_t>(sum, smem, &total);
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
      if (base + k < n) row[base + k] = r;
      r += v[k];
    }
    carry += total;
    __syncthreads();
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}

// mb_off[m][k] = rows before minibatch k of model m; minibatch k starts at the first kept trajectory q
// with q * n_minibatch / n_kept >= k, i.e. q = ceil(k n_kept / n_minibatch).
__global__ void k_mb_offsets(int n_models, int n_minibatch, int n_traj, const int64_t* __restrict__ n_kept_p,
                             const int64_t* __restrict__ scan_mq, const int64_t* __restrict__ totals,
                             int64_t* __restrict__ mb_off) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_models * (n_minibatch + 1)) return;
  const int m = i / (n_minibatch + 1), k = i % (n_minibatch + 1);
  int64_t base = 0;
  for (int mm = 0; mm < m; ++mm) base += totals[mm];
  const int64_t n_kept = *n_kept_p;
  const int64_t q = (static_cast<int64_t>(k) * n_kept + n_minibatch - 1) / n_minibatch;
  mb_off[i] = base + ((k == n_minibatch || q >= n_kept) ? totals[m] : scan_mq[static_cast<size_t>(m) * n_traj + q]);
}

// One wavefront per (model, kept trajectory): its rowsel slice goes to its place in mb_rowsel.
__global__ void __launch_bounds__(256)
k_mb_copy(int n_models, int n_traj, const int64_t* __restrict__ n_kept_p, const int64_t* __restrict__ scan_mq,
          const int64_t* __restrict__ src_mq, const int64_t* __restrict__ totals, const int32_t* __restrict__ rowsel,
          int32_t* __restrict__ mb_rowsel) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t w = static_cast<int64_t>(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t n_kept = *n_kept_p;
  if (w >= static_cast<int64_t>(n_models) * n_traj) return;
  const int m = static_cast<int>(w / n_traj);
  const int64_t q = w % n_traj;
  if (q >= n_kept) return;
  int64_t base = 0;
  for (int mm = 0; mm < m; ++mm) base += totals[mm];
  const size_t at = static_cast<size_t>(m) * n_traj + q;
  const int64_t dst = base + scan_mq[at];
  const int64_t len = (q + 1 < n_traj ? scan_mq[at + 1] : totals[m]) - scan_mq[at];
  const int64_t src = src_mq[at];
  for (int64_t i0 = lane; i0 < len; i0 += 4 * kWave) {       // four loads in flight per lane
    int32_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = i0 + k * kWave < len ? rowsel[src + i0 + k * kWave] : 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (i0 + k * kWave < len) mb_rowsel[dst + i0 + k * kWave] = v[k];
  }
}

__global__ void k_zero_i64(int64_t* __restrict__ p, int64_t n) {
  int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (; i < n; i += stride) p[i] = 0;
}

struct BatchWs {
  int32_t* traj_turn_off;
  int32_t* order;
  uint8_t* keep;
  int32_t* rank;
  int64_t* flag;     // [n_traj] kept flags in shuffled order, scanned in place
  int64_t* n_kept;
  int64_t* tile_sum; // [n_models][tiles] totals of the scan tiles, scanned in place
  int64_t* cnt_mq;   // [n_models][n_traj], scanned in place
  int64_t* src_mq;   // [n_models][n_traj]
  int64_t* totals;   // [n_models]
};
size_t carve_batch(Carver& c, BatchWs& w, int n_traj, int n_models) {
  w.traj_turn_off = c.take<int32_t>(static_cast<size_t>(n_traj) + 1);
  w.order = c.take<int32_t>(n_traj);
  w.keep = c.take<uint8_t>(n_traj);
  w.rank = c.take<int32_t>(n_traj);
  w.flag = c.take<int64_t>(n_traj);
  w.n_kept = c.take<int64_t>(1);
  w.tile_sum = c.take<int64_t>(static_cast<size_t>(n_models) * cdiv(n_traj > 0 ? n_traj : 1, kScanTile));
  w.cnt_mq = c.take<int64_t>(static_cast<size_t>(n_models) * n_traj);
  w.src_mq = c.take<int64_t>(static_cast<size_t>(n_models) * n_traj);
  w.totals = c.take<int64_t>(n_models);
  return c.off;
}

}  // namespace
}  // namespace umas

using namespace umas;

extern "C" size_t umas_ready_batch_workspace_bytes(int32_t n_traj, int32_t n_models) {
  if (n_traj < 0 || n_models < 1) return 0;
  Carver c(nullptr);
  BatchWs w;
  return carve_batch(c, w, n_traj, n_models);
}

extern "C" umas_status umas_ready_batch(const umas_streams* s, int32_t n_models, int32_t n_turns,
                                        const int32_t* traj_turn_off, int32_t n_traj, const uint8_t* traj_keep,
                                        const int32_t* traj_order, int32_t n_minibatch, int32_t* mb_rowsel,
                                        int64_t* mb_off, void* workspace, size_t workspace_bytes, void* hip_stream) {
  UMAS_REQUIRE(s && s->traj_seg_off && s->model_trajrun_off && s->model_tok_off && s->model_rowsel_off && s->rowsel && s->tok_turn,
               UMAS_EINVAL, "streams lacks traj_seg_off, model_trajrun_off, model_tok_off, model_rowsel_off, rowsel or tok_turn");
  UMAS_REQUIRE(n_models >= 1 && n_models <= UMAS_MAX_MODELS, UMAS_ESHAPE, "n_models=%d outside [1,%d]", n_models, UMAS_MAX_MODELS);
  UMAS_REQUIRE(n_traj >= 0 && n_turns >= 0, UMAS_EINVAL, "negative size");
  UMAS_REQUIRE(n_minibatch >= 1, UMAS_EINVAL, "n_minibatch=%d must be at least 1", n_minibatch);
  UMAS_REQUIRE(traj_turn_off && mb_off && (mb_rowsel || n_turns == 0), UMAS_EINVAL, "traj_turn_off, mb_rowsel and mb_off must not be NULL");
  UMAS_REQUIRE(traj_turn_off[0] == 0 && traj_turn_off[n_traj] == n_turns, UMAS_EINVAL, "traj_turn_off must run from 0 to n_turns");
  for (int b = 0; b < n_traj; ++b)
    UMAS_REQUIRE(traj_turn_off[b] <= traj_turn_off[b + 1], UMAS_EINVAL, "traj_turn_off decreases at %d", b);
  if (traj_order) {                                  // a permutation of the trajectories
    std::vector<uint8_t> seen(static_cast<size_t>(n_traj), 0);
    for (int q = 0; q < n_traj; ++q) {
      const int b = traj_order[q];
      UMAS_REQUIRE(b >= 0 && b < n_traj && !seen[b], UMAS_EINVAL, "traj_order is not a permutation (entry %d = %d)", q, b);
      seen[b] = 1;
    }
  }
  const size_t need = umas_ready_batch_workspace_bytes(n_traj, n_models);
  UMAS_REQUIRE(workspace && reinterpret_cast<uintptr_t>(workspace) % kAlign == 0 && workspace_bytes >= need, UMAS_EWORKSPACE,
               "workspace must be 256-byte aligned and hold %zu bytes (got %zu)", need, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  prof_mark(st);
  Carver c(workspace);
  BatchWs w;
  carve_batch(c, w, n_traj, n_models);
  // the thin arrays (the first arrays of the workspace, up to rank) go through pinned staging memory in one
  // asynchronous copy: they have been read when the call returns, and the host does not wait for the stream
  char* const ws_base = static_cast<char*>(workspace);
  const size_t staged_bytes = static_cast<size_t>(reinterpret_cast<char*>(w.rank) - ws_base);
  ThinStage stage;
  umas_status vs = stage.begin(staged_bytes);
  if (vs != UMAS_OK) return vs;
  stage.put(static_cast<size_t>(reinterpret_cast<char*>(w.traj_turn_off) - ws_base), traj_turn_off, (static_cast<size_t>(n_traj) + 1) * sizeof(int32_t));
  stage.put(static_cast<size_t>(reinterpret_cast<char*>(w.order) - ws_base), traj_order, static_cast<size_t>(n_traj) * sizeof(int32_t));
  stage.put(static_cast<size_t>(reinterpret_cast<char*>(w.keep) - ws_base), traj_keep, static_cast<size_t>(n_traj));
  vs = stage.flush(workspace, staged_bytes, st);
  if (vs != UMAS_OK) return vs;
  prof_mark(st);

  const int64_t n_mq = static_cast<int64_t>(n_models) * n_traj;
  hipLaunchKernelGGL(k_zero_i64, dim3(cdiv(n_mq > 0 ? n_mq : 1, 256) < 4096 ? cdiv(n_mq > 0 ? n_mq : 1, 256) : 4096), dim3(256), 0,
                     st, w.cnt_mq, n_mq);
  UMAS_LAUNCHED("k_zero_i64");
  const int ntile = static_cast<int>(cdiv(n_traj > 0 ? n_traj : 1, kScanTile));
  // exclusive scan of data[rows][n_traj]; totals[r] receives the sum of row r
  auto scan = [&](int64_t* data, int rows, int64_t* totals) -> umas_status {
    hipLaunchKernelGGL(k_scan_tiles, dim3(ntile, rows), dim3(256), 0, st, data, n_traj, ntile, w.tile_sum);
    UMAS_LAUNCHED("k_scan_tiles");
    hipLaunchKernelGGL(k_scan_rows, dim3(rows), dim3(1024), 0, st, w.tile_sum, ntile, totals);
    UMAS_LAUNCHED("k_scan_rows");
    hipLaunchKernelGGL(k_scan_add, dim3(ntile, rows), dim3(256), 0, st, data, n_traj, ntile, w.tile_sum);
    UMAS_LAUNCHED("k_scan_add");
    return UMAS_OK;
  };
  const int32_t* d_order = traj_order ? w.order : nullptr;
  const uint8_t* d_keep = traj_keep ? w.keep : nullptr;
  if (n_traj > 0) {
    hipLaunchKernelGGL(k_kept_flags, dim3(cdiv(n_traj, 256)), dim3(256), 0, st, n_traj, d_order, d_keep, w.flag);
    UMAS_LAUNCHED("k_kept_flags");
  }
  umas_status ss = scan(w.flag, 1, w.n_kept);
  if (ss != UMAS_OK) return ss;
  if (n_traj > 0) {
    hipLaunchKernelGGL(k_kept_rank, dim3(cdiv(n_traj, 256)), dim3(256), 0, st, n_traj, d_order, d_keep, w.flag, w.rank);
    UMAS_LAUNCHED("k_kept_rank");
  }
  if (n_turns > 0 && n_traj > 0) {
    hipLaunchKernelGGL(k_run_slices, dim3(cdiv(n_turns, 256)), dim3(256), 0, st, n_turns, n_traj, n_models, s->traj_seg_off,
                       s->model_trajrun_off, s->model_tok_off, s->model_rowsel_off, s->rowsel, s->tok_turn, w.traj_turn_off,
                       w.rank, w.cnt_mq, w.src_mq);
    UMAS_LAUNCHED("k_run_slices");
  }
  ss = scan(w.cnt_mq, n_models, w.totals);
  if (ss != UMAS_OK) return ss;
  hipLaunchKernelGGL(k_mb_offsets, dim3(cdiv(static_cast<size_t>(n_models) * (n_minibatch + 1), 256)), dim3(256), 0, st,
                     n_models, n_minibatch, n_traj, w.n_kept, w.cnt_mq, w.totals, mb_off);
  UMAS_LAUNCHED("k_mb_offsets");
  if (n_mq > 0) {
    hipLaunchKernelGGL(k_mb_copy, dim3(cdiv(n_mq, 4)), dim3(256), 0, st, n_models, n_traj, w.n_kept, w.cnt_mq, w.src_mq,
                       w.totals, s->rowsel, mb_rowsel);
    UMAS_LAUNCHED("k_mb_copy");
  }
  return UMAS_OK;
}
