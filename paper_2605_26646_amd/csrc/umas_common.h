// Shared host/device helpers of libumas: error reporting, workspace carving, wave and
// block primitives for 64-wide wavefronts.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/umas.h"

namespace umas {

umas_status fail(umas_status code, const char* fmt, ...);

// Kernel timing aid (umas_profile_enable / umas_profile_read).
extern bool g_prof_on;
void prof_mark(hipStream_t st);                     // opens an interval at the start of an API call
void prof_kernel(const char* name, hipStream_t st); // closes the interval of the kernel just launched

// Staging of thin host arrays.  The calls that take host arrays copy them into a block of pinned host memory that
// the library keeps (a ring of kSlots blocks, each grown to the largest request it has seen) and enqueue ONE
// asynchronous copy of the block to the device: the caller's arrays have been read when the call returns, and the
// host never waits for the stream.  A block is reused kSlots calls later; only then does the host wait, and only
// until the copy that was issued from that block has run.
class ThinStage {
 public:
  static constexpr int kSlots = 4;
  // Takes the next block of the ring with room for `bytes`; 256-byte aligned.  Holds the ring's lock until flush().
  umas_status begin(size_t bytes);
  // Copies n bytes to offset `off` of the block (nothing for src == nullptr or n == 0).
  void put(size_t off, const void* src, size_t n);
  void zero(size_t off, size_t n);
  // Enqueues the copy of the first `bytes` bytes of the block to `dst` on `st` and releases the ring.
  umas_status flush(void* dst, size_t bytes, hipStream_t st);
  // Releases the ring without copying (an error between begin and flush).
  void abandon();

 private:
  char* cur_ = nullptr;
  int slot_ = -1;
};

#define UMAS_HIP(expr)                                                                 \
  do {                                                                                 \
    hipError_t e__ = (expr);                                                           \
    if (e__ != hipSuccess)                                                             \
      return ::umas::fail(UMAS_EHIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

// After every kernel launch: check the launch and, when kernel timing is on, close the kernel's
// interval with an event on its stream `st` (intervals open at prof_mark or at the previous launch).
#define UMAS_LAUNCHED(name)                                                                  \
  do {                                                                                       \
    hipError_t e__ = hipGetLastError();                                                      \
    if (e__ != hipSuccess)                                                                   \
      return ::umas::fail(UMAS_EHIP, "launch of %s failed: %s", name, hipGetErrorString(e__)); \
    if (::umas::g_prof_on) ::umas::prof_kernel(name, st);                                    \
  } while (0)

#define UMAS_REQUIRE(cond, code, ...) \
  do {                                \
    if (!(cond)) return ::umas::fail(code, __VA_ARGS__); \
  } while (0)

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }

// Carves 256-byte aligned arrays out of a caller-provided workspace; with base == nullptr it
// only measures.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base(static_cast<char*>(b)) {}
  template <typename T>
  T* take(size_t n) {
    size_t bytes = align_up(n * sizeof(T));
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += bytes;
    return p;
  }
};

inline unsigned cdiv(size_t a, size_t b) { return static_cast<unsigned>((a + b - 1) / b); }

// ------------------------------------------------------------------ device primitives
constexpr int kWave = 64;

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
template <typename T>
__device__ __forceinline__ T wave_max(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    T t = __shfl_xor(v, o, kWave);
    v = t > v ? t : v;
  }
  return v;
}
template <typename T>
__device__ __forceinline__ T wave_incl_scan(T v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    T t = __shfl_up(v, o, kWave);
    if (lane >= o) v += t;
  }
  return v;
}

// Exclusive prefix sum over the threads of a block (blockDim.x a multiple of 64, at most 1024).
// `smem` holds at least 17 values of T.  Returns the exclusive prefix; *total gets the block sum.
template <typename T>
__device__ __forceinline__ T block_excl_scan(T v, T* smem, T* total) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int nwave = blockDim.x / kWave;
  T incl = wave_incl_scan(v);
  __syncthreads();  // smem may still be read from a previous use
  if (lane == kWave - 1) smem[wave] = incl;
  __syncthreads();
  if (threadIdx.x == 0) {
    T run = 0;
    for (int w = 0; w < nwave; ++w) {
      T t = smem[w];
      smem[w] = run;
      run += t;
    }
    smem[16] = run;
  }
  __syncthreads();
  *total = smem[16];
  return incl - v + smem[wave];
}

template <typename T>
__device__ __forceinline__ T block_sum(T v, T* smem) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int nwave = blockDim.x / kWave;
  v = wave_sum(v);
  __syncthreads();
  if (lane == 0) smem[wave] = v;
  __syncthreads();
  T r = 0;
  for (int w = 0; w < nwave; ++w) r += smem[w];
  return r;
}

// Largest j in [0, n] with off[j] <= x, for ascending off[0..n] and off[0] <= x.
template <typename T>
__device__ __forceinline__ int last_le(const T* __restrict__ off, int n, T x) {
  int lo = 0, hi = n;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (off[mid] <= x) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Largest j in [0, n] with off[j] <= x (ascending off, off[0] <= x), found by one wavefront probing
// 256 positions per round (four per lane, all four loads in flight together: a round costs one trip to
// memory); every lane of the wavefront must call it and gets the same answer.
__device__ __forceinline__ int wave_last_le(const int64_t* __restrict__ off, int n, int64_t x) {
  const int lane = threadIdx.x & (kWave - 1);
  constexpr int kProbes = 4 * kWave;
  int lo = 0, hi = n;
  while (hi - lo >= kProbes) {
    const int step = (hi - lo) / kProbes;
    // probe i = 1 .. 256 sits at lo + i * step; lane l takes probes l + 1, l + 65, l + 129, l + 193
    bool ok[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) ok[k] = off[lo + (lane + 1 + k * kWave) * step] <= x;
    int c = 0;                                     // probes 1..c hold (the predicate is monotone)
#pragma unroll
    for (int k = 0; k < 4; ++k) c += __popcll(__ballot(ok[k]));
    const int nhi = c == kProbes ? hi : lo + (c + 1) * step - 1;
    lo += c * step;
    hi = nhi;
  }
  int c = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int j = lo + lane + k * kWave;
    c += __popcll(__ballot(j <= hi && off[j] <= x));
  }
  return lo + c - 1;
}

}  // namespace umas
