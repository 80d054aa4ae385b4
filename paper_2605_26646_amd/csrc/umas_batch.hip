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
#include <algorithm>
#include <vector>

#include "umas_common.h"

namespace umas {
namespace {

constexpr int kScanItems = 8;
constexpr int kScanTile = 256 * kScanItems;       // entries one workgroup scans at a time
constexpr int kPerCu = 2;                         // workgroups per compute unit of the kernels that wait for one another
constexpr unsigned long long kMark = 1ull << 63;  // ready mark of a published sum

// Sum of the published words part[0 .. n): every thread takes some, a word is taken when its ready mark is set;
// also returns, in *before, the sum of the words part[0 .. upto).  Result in every thread.  Waiting is safe because
// every workgroup publishes all of its words before it reads any, and all workgroups of the grid are resident.
__device__ __forceinline__ int64_t sum_published(unsigned long long* part, int n, int upto, int64_t* smem, int64_t* before) {
  int64_t all = 0, bef = 0;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    unsigned long long w;
    while (!((w = __hip_atomic_load(part + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) & kMark)) __builtin_amdgcn_s_sleep(2);
    const int64_t v = static_cast<int64_t>(w & ~kMark);
    all += v;
    bef += i < upto ? v : 0;
  }
  *before = block_sum<int64_t>(bef, smem);
  return block_sum<int64_t>(all, smem);
}

// rank[b] = position of trajectory b among the kept trajectories in shuffled order, or -1; *n_kept = their number.
// Tiles of kScanTile positions of the shuffle; a workgroup publishes the kept count of each of its tiles, then places
// each of them behind the tiles before it.  Also clears what the later kernels add to or wait for: zero_a, zero_b.
__global__ void __launch_bounds__(256)
k_kept_ranks(int n_traj, int ntile, const int32_t* __restrict__ order, const uint8_t* __restrict__ keep,
             unsigned long long* part, int32_t* __restrict__ rank, int64_t* __restrict__ n_kept,
             int64_t* __restrict__ zero_a, int64_t n_zero_a, unsigned long long* __restrict__ zero_b, int64_t n_zero_b) {
  __shared__ int64_t smem[32];
  const int tid = threadIdx.x;
  auto flags_of = [&](int t, int32_t (&b)[kScanItems], int (&f)[kScanItems]) {
    int sum = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
      const int q = t * kScanTile + tid * kScanItems + k;
      b[k] = q < n_traj ? (order ? order[q] : q) : -1;
    }
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
      f[k] = b[k] >= 0 && (!keep || keep[b[k]]) ? 1 : 0;
      sum += f[k];
    }
    return sum;
  };
  for (int t = blockIdx.x; t < ntile; t += gridDim.x) {
    int32_t b[kScanItems];
    int f[kScanItems];
    const int64_t total = block_sum<int64_t>(flags_of(t, b, f), smem);
    if (tid == 0) __hip_atomic_store(part + t, kMark | static_cast<unsigned long long>(total), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  {
    const int64_t gtid = static_cast<int64_t>(blockIdx.x) * blockDim.x + tid, gsize = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = gtid; i < n_zero_a; i += gsize) zero_a[i] = 0;
    for (int64_t i = gtid; i < n_zero_b; i += gsize) zero_b[i] = 0ull;
  }
  for (int t = blockIdx.x; t < ntile; t += gridDim.x) {
    int64_t before;
    const int64_t all = sum_published(part, ntile, t, smem, &before);
    if (t == 0 && tid == 0) *n_kept = all;
    int32_t b[kScanItems];
    int f[kScanItems];
    const int mine = flags_of(t, b, f);
    int32_t total;
    int32_t pos = static_cast<int32_t>(before) + block_excl_scan<int32_t>(mine, reinterpret_cast<int32_t*>(smem), &total);
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
      if (b[k] >= 0) rank[b[k]] = f[k] ? pos : -1;
      pos += f[k];
    }
  }
}

// Per trajectory run: its model, trajectory and the slice of rowsel that holds its scored rows; written
// at (model, rank of the trajectory) when the trajectory is kept.  Three binary searches per run (the first row at
// or behind its start, the same for its end, its trajectory) advance in one loop, their loads in flight together.
// (Wider searches were slower here: the kernel is bound by the number of scattered loads, not by their latency.)
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
  const int64_t ra = model_rowsel_off[m], n_m = model_rowsel_off[m + 1] - ra, t0 = model_tok_off[m];
  const int32_t* __restrict__ rs = rowsel + ra;
  int lo = 0, hi = n_traj;                         // trajectory of turn u: last b with traj_turn_off[b] <= u
  int64_t lo0 = 0, hi0 = n_m, lo1 = 0, hi1 = n_m;  // first rows at or behind the run's start and its end
  const int64_t x0 = start - t0, x1 = end - t0;
  while (lo < hi || lo0 < hi0 || lo1 < hi1) {
    const int mid = (lo + hi + 1) >> 1;
    const int64_t mid0 = (lo0 + hi0) >> 1, mid1 = (lo1 + hi1) >> 1;
    const int32_t a = lo < hi ? traj_turn_off[mid] : 0;
    const int32_t r0 = lo0 < hi0 ? rs[mid0] : 0;
    const int32_t r1 = lo1 < hi1 ? rs[mid1] : 0;
    if (lo < hi) { if (a <= u) lo = mid; else hi = mid - 1; }
    if (lo0 < hi0) { if (r0 < x0) lo0 = mid0 + 1; else hi0 = mid0; }
    if (lo1 < hi1) { if (r1 < x1) lo1 = mid1 + 1; else hi1 = mid1; }
  }
  const int q = rank[lo];
  if (q < 0) return;
  cnt_mq[static_cast<size_t>(m) * n_traj + q] = lo1 - lo0;
  src_mq[static_cast<size_t>(m) * n_traj + q] = ra + lo0;
}

// In-place exclusive prefix sums of the rows of data[n_models][n_traj] (the rows of every model by kept rank), the
// rows' totals, and mb_off[m][k] = rows before minibatch k of model m: minibatch k starts at the first kept
// trajectory q with q * n_minibatch / n_kept >= k, i.e. q = ceil(k n_kept / n_minibatch).  Tiles of kScanTile
// entries of a row; a workgroup publishes the sum of each of its tiles, then places each of them behind the tiles
// before it in its row and the rows before that.
__global__ void __launch_bounds__(256)
k_mb_scan(int n_models, int n_traj, int ntile, int n_minibatch, int balance_rows, const int64_t* __restrict__ n_kept_p,
          int64_t* __restrict__ data, unsigned long long* part, int64_t* __restrict__ totals, int64_t* __restrict__ mb_off) {
  __shared__ int64_t smem[32];
  __shared__ int64_t s_scan[kScanTile];
  const int tid = threadIdx.x;
  const int n_all = n_models * ntile;
  for (int t = blockIdx.x; t < n_all; t += gridDim.x) {
    const int64_t* row = data + static_cast<size_t>(t / ntile) * n_traj;
    const int base = (t % ntile) * kScanTile + tid * kScanItems;
    int64_t sum = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) sum += base + k < n_traj ? row[base + k] : 0;
    const int64_t total = block_sum<int64_t>(sum, smem);
    if (tid == 0) __hip_atomic_store(part + t, kMark | static_cast<unsigned long long>(total), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  const int64_t n_kept = *n_kept_p;
  for (int t = blockIdx.x; t < n_all; t += gridDim.x) {
    const int m = t / ntile, tile0 = (t % ntile) * kScanTile;
    int64_t before_row, in_row_before;
    const int64_t row_total = sum_published(part + static_cast<size_t>(m) * ntile, ntile, t % ntile, smem, &in_row_before);
    (void)sum_published(part, m * ntile, m * ntile, smem, &before_row);   // the rows of the models before m
    int64_t* row = data + static_cast<size_t>(m) * n_traj;
    const int base = tile0 + tid * kScanItems;
    int64_t v[kScanItems];
    int64_t sum = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
      v[k] = base + k < n_traj ? row[base + k] : 0;
      sum += v[k];
    }
    int64_t total;
    int64_t r = in_row_before + block_excl_scan<int64_t>(sum, smem, &total);
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
      if (base + k < n_traj) row[base + k] = r;
      s_scan[tid * kScanItems + k] = r;
      r += v[k];
    }
    __syncthreads();
    if (t % ntile == 0 && tid == 0) totals[m] = row_total;
    for (int k = tid; k <= n_minibatch; k += blockDim.x) {
      int64_t* out = mb_off + static_cast<size_t>(m) * (n_minibatch + 1) + k;
      if (balance_rows) {
        // cut by rows: part k starts at the first trajectory whose first row is at or behind ceil(k T / M); the tile
        // whose prefix sums first reach the threshold writes it (the first tile when the threshold is 0)
        const int64_t thr = (static_cast<int64_t>(k) * row_total + n_minibatch - 1) / n_minibatch;
        const int len = n_traj - tile0 < kScanTile ? n_traj - tile0 : kScanTile;   // entries of the tile that exist
        if (thr <= in_row_before ? tile0 == 0 : thr <= in_row_before + total) {
          int lo = 0, hi = len;                          // first entry of the tile at or above the threshold, len if none
          while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_scan[mid] < thr) lo = mid + 1; else hi = mid;
          }
          *out = before_row + (lo < len ? s_scan[lo] : in_row_before + total);
        }
        continue;
      }
      const int64_t q = (static_cast<int64_t>(k) * n_kept + n_minibatch - 1) / n_minibatch;
      if (k == n_minibatch || q >= n_kept) {
        if (t % ntile == 0) *out = before_row + row_total;
      } else if (q >= tile0 && q < tile0 + kScanTile) {
        *out = before_row + s_scan[q - tile0];
      }
    }
    __syncthreads();                                // s_scan and smem are the next tile's
  }
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

// Parts under a budget of scored rows, one wavefront per model: starting from the model's first row, a part ends at
// the last trajectory boundary within max_rows rows of its start, or, when not even the first trajectory fits, behind
// that trajectory.  scan_mq holds the model's rows before each kept trajectory (kept rank order), so a boundary is found
// by one wavefront-wide search per part (one trip to memory when the part spans fewer than 256 trajectories); every part holds at least one row, so the walk ends after at most as many
// steps as the model has rows.  Entries of the offsets past the last part repeat the model's end.
constexpr int kPackThreads = 1024;
__global__ void __launch_bounds__(kPackThreads)
k_mb_pack(int n_traj, int64_t max_rows, const int64_t* __restrict__ n_kept_p, const int64_t* __restrict__ scan_mq,
          const int64_t* __restrict__ totals, int64_t* __restrict__ mb_off, int32_t* __restrict__ n_parts) {
  __shared__ int s_parts;
  const int m = blockIdx.x, tid = threadIdx.x;
  const int n_kept = static_cast<int>(*n_kept_p);
  const int64_t* row = scan_mq + static_cast<size_t>(m) * n_traj;
  const int64_t total = totals[m];
  int64_t base = 0;
  for (int mm = 0; mm < m; ++mm) base += totals[mm];
  int64_t* out = mb_off + static_cast<size_t>(m) * (static_cast<size_t>(n_traj) + 1);
  if (tid < kWave) {                                 // the walk is one wavefront's; the others help with the tail afterwards
    if (tid == 0) out[0] = base;
    int k = 0;
    int64_t at = 0;                                  // first row of the open part, relative to the model's first
    int j0 = 0;                                      // a kept trajectory with row[j0] == at
    // parts that span fewer than about 200 trajectories on average are looked for among the next 256 entries first
    const bool near = static_cast<double>(max_rows) * n_kept < 200.0 * static_cast<double>(total);
    while (at < total) {                             // n_kept >= 1 here
      const int64_t limit = at + max_rows;
      int64_t end = total;
      if (total > limit) {
        // largest j with row[j] <= limit: with short parts first among the 256 entries from j0 on (one trip;
        // row[j0] = at <= limit), and only if all of those hold, by the general search behind them
        const int avail = n_kept - 1 - j0;           // entries j0 .. j0 + avail exist
        int64_t v[4] = {0, 0, 0, 0};
        int c = 4 * kWave;
        if (near) {
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = tid + q * kWave <= avail ? row[j0 + tid + q * kWave] : INT64_MAX;
          c = 0;
#pragma unroll
          for (int q = 0; q < 4; ++q) c += __popcll(__ballot(v[q] <= limit));
        }
        int j;
        if (c < 4 * kWave) {
          j = j0 + c - 1;
          const int64_t mine = (c - 1) >> 6 == 0 ? v[0] : (c - 1) >> 6 == 1 ? v[1] : (c - 1) >> 6 == 2 ? v[2] : v[3];
          end = __shfl(mine, (c - 1) & (kWave - 1), kWave);
        } else {
          const int from = near ? 4 * kWave - 1 : 0;   // row[j0 + from] <= limit either way
          j = j0 + from + wave_last_le(row + j0 + from, avail - from, limit);
          end = row[j];
        }
        if (end == at) {                             // the trajectory at the part's start is over the budget by itself
          ++j;
          end = j < n_kept ? row[j] : total;
        }
        j0 = j;
      }
      ++k;
      if (tid == 0) out[k] = base + end;
      at = end;
    }
    if (tid == 0) { n_parts[m] = k; s_parts = k; }
  }
  __syncthreads();
  for (int64_t i = s_parts + 1 + tid; i <= n_traj; i += kPackThreads) out[i] = base + total;
}

struct BatchWs {
  int32_t* traj_turn_off;
  int32_t* order;
  uint8_t* keep;
  unsigned long long* part_q;   // [tiles] kept counts of the tiles of the shuffle; zeros come with the staged copy
  int32_t* rank;
  int64_t* n_kept;
  unsigned long long* part_mq;  // [n_models][tiles] sums of the tiles of cnt_mq
  int64_t* cnt_mq;   // [n_models][n_traj], scanned in place
  int64_t* src_mq;   // [n_models][n_traj]
  int64_t* totals;   // [n_models]
  int64_t* one_off;  // [n_models][2] the scan kernel's offsets when the parts are cut by k_mb_pack
};
inline int scan_tiles(int n_traj) { return static_cast<int>(cdiv(n_traj > 0 ? n_traj : 1, kScanTile)); }
size_t carve_batch(Carver& c, BatchWs& w, int n_traj, int n_models) {
  w.traj_turn_off = c.take<int32_t>(static_cast<size_t>(n_traj) + 1);
  w.order = c.take<int32_t>(n_traj);
  w.keep = c.take<uint8_t>(n_traj);
  w.part_q = c.take<unsigned long long>(scan_tiles(n_traj));
  w.rank = c.take<int32_t>(n_traj);
  w.n_kept = c.take<int64_t>(1);
  w.part_mq = c.take<unsigned long long>(static_cast<size_t>(n_models) * scan_tiles(n_traj));
  w.cnt_mq = c.take<int64_t>(static_cast<size_t>(n_models) * n_traj);
  w.src_mq = c.take<int64_t>(static_cast<size_t>(n_models) * n_traj);
  w.totals = c.take<int64_t>(n_models);
  w.one_off = c.take<int64_t>(2 * static_cast<size_t>(n_models));
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

namespace {
umas_status ready_batch(const umas_streams* s, int32_t n_models, int32_t n_turns, const int32_t* traj_turn_off, int32_t n_traj,
                        const uint8_t* traj_keep, const int32_t* traj_order, int32_t n_minibatch, int balance_rows,
                        int64_t max_rows, int32_t* n_parts, int32_t* mb_rowsel, int64_t* mb_off, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  const bool packed = n_parts != nullptr;           // parts under a row budget instead of n_minibatch parts
  UMAS_REQUIRE(!packed || max_rows >= 1, UMAS_EINVAL, "max_rows=%lld must be at least 1", static_cast<long long>(max_rows));
  if (max_rows > (int64_t{1} << 62)) max_rows = int64_t{1} << 62;   // more than any batch holds; keeps start + budget inside int64
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
  // asynchronous copy, together with the zeros that the first kernel's tile counts start from: they have been read
  // when the call returns, and the host does not wait for the stream
  char* const ws_base = static_cast<char*>(workspace);
  const size_t staged_bytes = static_cast<size_t>(reinterpret_cast<char*>(w.rank) - ws_base);
  const int ntile = scan_tiles(n_traj);
  ThinStage stage;
  umas_status vs = stage.begin(staged_bytes);
  if (vs != UMAS_OK) return vs;
  stage.put(static_cast<size_t>(reinterpret_cast<char*>(w.traj_turn_off) - ws_base), traj_turn_off, (static_cast<size_t>(n_traj) + 1) * sizeof(int32_t));
  stage.put(static_cast<size_t>(reinterpret_cast<char*>(w.order) - ws_base), traj_order, static_cast<size_t>(n_traj) * sizeof(int32_t));
  stage.put(static_cast<size_t>(reinterpret_cast<char*>(w.keep) - ws_base), traj_keep, static_cast<size_t>(n_traj));
  stage.zero(static_cast<size_t>(reinterpret_cast<char*>(w.part_q) - ws_base), static_cast<size_t>(ntile) * sizeof(unsigned long long));
  vs = stage.flush(workspace, staged_bytes, st);
  if (vs != UMAS_OK) return vs;
  prof_mark(st);

  // workgroups of the two scanning kernels wait for one another's sums: no more of them than the device holds at once
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    n_cu = 64;
  const int64_t n_mq = static_cast<int64_t>(n_models) * n_traj;
  const int32_t* d_order = traj_order ? w.order : nullptr;
  const uint8_t* d_keep = traj_keep ? w.keep : nullptr;
  hipLaunchKernelGGL(k_kept_ranks, dim3(std::min(ntile, kPerCu * n_cu)), dim3(256), 0, st, n_traj, ntile, d_order, d_keep, w.part_q,
                     w.rank, w.n_kept, w.cnt_mq, n_mq, w.part_mq, static_cast<int64_t>(n_models) * ntile);
  UMAS_LAUNCHED("k_kept_ranks");
  if (n_turns > 0 && n_traj > 0) {
    hipLaunchKernelGGL(k_run_slices, dim3(cdiv(n_turns, 256)), dim3(256), 0, st, n_turns, n_traj, n_models, s->traj_seg_off,
                       s->model_trajrun_off, s->model_tok_off, s->model_rowsel_off, s->rowsel, s->tok_turn, w.traj_turn_off,
                       w.rank, w.cnt_mq, w.src_mq);
    UMAS_LAUNCHED("k_run_slices");
  }
  hipLaunchKernelGGL(k_mb_scan, dim3(std::min(n_models * ntile, kPerCu * n_cu)), dim3(256), 0, st, n_models, n_traj, ntile,
                     packed ? 1 : n_minibatch, balance_rows, w.n_kept, w.cnt_mq, w.part_mq, w.totals, packed ? w.one_off : mb_off);
  UMAS_LAUNCHED("k_mb_scan");
  if (packed) {
    hipLaunchKernelGGL(k_mb_pack, dim3(n_models), dim3(kPackThreads), 0, st, n_traj, max_rows, w.n_kept, w.cnt_mq, w.totals, mb_off, n_parts);
    UMAS_LAUNCHED("k_mb_pack");
  }
  if (n_mq > 0) {
    hipLaunchKernelGGL(k_mb_copy, dim3(cdiv(n_mq, 4)), dim3(256), 0, st, n_models, n_traj, w.n_kept, w.cnt_mq, w.src_mq,
                       w.totals, s->rowsel, mb_rowsel);
    UMAS_LAUNCHED("k_mb_copy");
  }
  return UMAS_OK;
}
}  // namespace

extern "C" umas_status umas_ready_batch(const umas_streams* s, int32_t n_models, int32_t n_turns,
                                        const int32_t* traj_turn_off, int32_t n_traj, const uint8_t* traj_keep,
                                        const int32_t* traj_order, int32_t n_minibatch, int32_t* mb_rowsel,
                                        int64_t* mb_off, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return ready_batch(s, n_models, n_turns, traj_turn_off, n_traj, traj_keep, traj_order, n_minibatch, 0, 0, nullptr, mb_rowsel, mb_off,
                     workspace, workspace_bytes, hip_stream);
}

extern "C" umas_status umas_ready_batch_balanced(const umas_streams* s, int32_t n_models, int32_t n_turns,
                                                 const int32_t* traj_turn_off, int32_t n_traj, const uint8_t* traj_keep,
                                                 const int32_t* traj_order, int32_t n_minibatch, int32_t* mb_rowsel,
                                                 int64_t* mb_off, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return ready_batch(s, n_models, n_turns, traj_turn_off, n_traj, traj_keep, traj_order, n_minibatch, 1, 0, nullptr, mb_rowsel, mb_off,
                     workspace, workspace_bytes, hip_stream);
}

extern "C" umas_status umas_ready_batch_packed(const umas_streams* s, int32_t n_models, int32_t n_turns,
                                               const int32_t* traj_turn_off, int32_t n_traj, const uint8_t* traj_keep,
                                               const int32_t* traj_order, int64_t max_rows, int32_t* mb_rowsel,
                                               int64_t* mb_off, int32_t* n_parts, void* workspace, size_t workspace_bytes,
                                               void* hip_stream) {
  UMAS_REQUIRE(n_parts, UMAS_EINVAL, "n_parts must not be NULL");
  return ready_batch(s, n_models, n_turns, traj_turn_off, n_traj, traj_keep, traj_order, 1, 0, max_rows, n_parts, mb_rowsel, mb_off,
                     workspace, workspace_bytes, hip_stream);
}
