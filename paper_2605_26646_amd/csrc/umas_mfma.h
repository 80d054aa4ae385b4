// bf16 MFMA tile engine for gfx950: C[M,N] += A[M,K] * B[N,K]^T with both operands K-contiguous.
//
// A workgroup owns a BM x BN tile of C and walks K in steps of 64.  Global memory is read in
// 16-byte vectors into registers one K-step ahead, written to one of two LDS stages (row pitch
// 72 bf16 so that the 16-byte fragment reads of 16 consecutive rows fall on distinct banks) and
// consumed by v_mfma_f32_32x32x16_bf16.  Each wavefront owns a (BM/WM) x (BN/WN) sub-tile as a
// grid of 32x32 MFMA blocks with float accumulators.
//
// Accumulator layout of one 32x32 block (register r of lane l):
//   row (A side, "M")  = 8*(r/4) + 4*(l/32) + r%4
//   col (B side, "N")  = l%32
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace umas {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int BM_, int BN_, int WM_, int WN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int BK = 64;
  static constexpr int LDP = 72;                       // LDS row pitch in bf16 elements
  static constexpr int T = 64 * WM * WN;               // threads per workgroup
  static constexpr int WTM = BM / WM, WTN = BN / WN;   // wavefront sub-tile
  static constexpr int TM = WTM / 32, TN = WTN / 32;   // 32x32 blocks per wavefront
  static constexpr int NA = BM * 8 / T, NB = BN * 8 / T;   // 16-byte vectors per thread per K-step
  static constexpr int ROWS_PER_PASS = T / 8;          // rows covered by one vector slot of all threads
  static constexpr int STAGE = (BM + BN) * LDP;        // bf16 elements per LDS stage
  static constexpr int LDS_BYTES = 2 * STAGE * 2;
  static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "sub-tiles are grids of 32x32 blocks");
  static_assert((BM * 8) % T == 0 && (BN * 8) % T == 0, "vector slots divide evenly");
};

// Row of the tile that vector slot i of this thread loads, and the thread's 8-element K offset.
template <class C>
__device__ __forceinline__ int slot_row(int i) { return (threadIdx.x >> 3) + i * C::ROWS_PER_PASS; }
__device__ __forceinline__ int slot_kofs() { return (threadIdx.x & 7) * 8; }

// pa[i] / pb[i]: address of (row of slot i, k = slot_kofs()); always a readable row: callers clamp rows
// outside the matrix to a valid one and ignore the results that come from them.  Only the K tail
// (K not a multiple of 64) is zero-filled, because every output depends on it.
template <class C>
__device__ __forceinline__ void mfma_mainloop(const uint16_t* const (&pa)[C::NA], const uint16_t* const (&pb)[C::NB],
                                              int K, uint16_t* lds, floatx16 (&acc)[C::TM][C::TN]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int kofs = slot_kofs();
  uint4 ra[C::NA], rb[C::NB];
  const int nk = (K + C::BK - 1) / C::BK;
  const bool ktail = (K % C::BK) != 0;

  auto gload = [&](int kt) {
    const int k = kt * C::BK;
    if (ktail && kt == nk - 1) {
      // clamp the address into the row and drop what lies past K
      const bool kin = k + kofs < K;
      const int kk = kin ? k : 0;
#pragma unroll
      for (int i = 0; i < C::NA; ++i) {
        uint4 v = *reinterpret_cast<const uint4*>(pa[i] + kk);
        ra[i] = make_uint4(kin ? v.x : 0u, kin ? v.y : 0u, kin ? v.z : 0u, kin ? v.w : 0u);
      }
#pragma unroll
      for (int i = 0; i < C::NB; ++i) {
        uint4 v = *reinterpret_cast<const uint4*>(pb[i] + kk);
        rb[i] = make_uint4(kin ? v.x : 0u, kin ? v.y : 0u, kin ? v.z : 0u, kin ? v.w : 0u);
      }
    } else {
#pragma unroll
      for (int i = 0; i < C::NA; ++i) ra[i] = *reinterpret_cast<const uint4*>(pa[i] + k);
#pragma unroll
      for (int i = 0; i < C::NB; ++i) rb[i] = *reinterpret_cast<const uint4*>(pb[i] + k);
    }
  };
  auto swrite = [&](int stage) {
    uint16_t* sa = lds + stage * C::STAGE;
    uint16_t* sb = sa + C::BM * C::LDP;
#pragma unroll
    for (int i = 0; i < C::NA; ++i) *reinterpret_cast<uint4*>(sa + slot_row<C>(i) * C::LDP + kofs) = ra[i];
#pragma unroll
    for (int i = 0; i < C::NB; ++i) *reinterpret_cast<uint4*>(sb + slot_row<C>(i) * C::LDP + kofs) = rb[i];
  };
  auto compute = [&](int stage) {
    const uint16_t* sa = lds + stage * C::STAGE + (wm * C::WTM + (lane & 31)) * C::LDP + (lane >> 5) * 8;
    const uint16_t* sb = lds + stage * C::STAGE + (C::BM + wn * C::WTN + (lane & 31)) * C::LDP + (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < C::BK / 16; ++kk) {
      bf16x8 af[C::TM], bfr[C::TN];
#pragma unroll
      for (int tm = 0; tm < C::TM; ++tm) af[tm] = *reinterpret_cast<const bf16x8*>(sa + tm * 32 * C::LDP + kk * 16);
#pragma unroll
      for (int tn = 0; tn < C::TN; ++tn) bfr[tn] = *reinterpret_cast<const bf16x8*>(sb + tn * 32 * C::LDP + kk * 16);
#pragma unroll
      for (int tm = 0; tm < C::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < C::TN; ++tn)
          acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[tm], bfr[tn], acc[tm][tn], 0, 0, 0);
    }
  };

  gload(0);
  swrite(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) gload(kt + 1);
    compute(cur);
    if (kt + 1 < nk) swrite(cur ^ 1);
    __syncthreads();
  }
}

// Position of accumulator element (tm, tn, r) inside the workgroup tile.
template <class C>
__device__ __forceinline__ int acc_row(int tm, int r) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  return (wave / C::WN) * C::WTM + tm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
}
template <class C>
__device__ __forceinline__ int acc_col(int tn) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  return (wave % C::WN) * C::WTN + tn * 32 + (lane & 31);
}

// Workgroups are handed to the 8 XCDs round-robin; give every XCD a contiguous range of the
// logical tile order, and order tiles in groups of GM x GN so that the workgroups resident on
// one XCD share operand rows through its L2.  Returns false for a padding workgroup.
template <int GM, int GN>
__device__ __forceinline__ bool tile_coords(int tiles_m, int tiles_n, int* tm, int* tn) {
  const int total_groups_n = (tiles_n + GN - 1) / GN;
  const int total_groups_m = (tiles_m + GM - 1) / GM;
  const long long slots = static_cast<long long>(total_groups_m) * total_groups_n * (GM * GN);
  const long long per_xcd = (slots + 7) / 8;
  const long long bid = blockIdx.x;
  const long long logical = (bid & 7) * per_xcd + (bid >> 3);
  if ((bid >> 3) >= per_xcd || logical >= slots) return false;
  const long long grp = logical / (GM * GN);
  const int within = static_cast<int>(logical % (GM * GN));
  const int gm = static_cast<int>(grp / total_groups_n), gn = static_cast<int>(grp % total_groups_n);
  *tm = gm * GM + within % GM;
  *tn = gn * GN + within / GM;
  return *tm < tiles_m && *tn < tiles_n;
}
template <int GM, int GN>
inline unsigned tile_grid(int tiles_m, int tiles_n) {
  const long long slots = static_cast<long long>((tiles_m + GM - 1) / GM) * ((tiles_n + GN - 1) / GN) * (GM * GN);
  return static_cast<unsigned>(((slots + 7) / 8) * 8);
}

}  // namespace umas
