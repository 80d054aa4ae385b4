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

// ---------------------------------------------------------------------------------------------
// Fast main loop for K % 64 == 0: tiles go from global memory straight into LDS
// (buffer_load_dwordx4 ... lds: no staging registers, no ds_write), fragments are read one 16-wide
// K-slice ahead of the MFMAs that consume them.
//
// LDS layout: rows of 128 bytes without padding; the 16-byte chunk c of row r sits in slot
// c ^ ((r >> 1) & 7), which spreads the fragment reads of 16 consecutive rows over all banks.
// One wavefront-wide load instruction fills 8 consecutive rows (1 KB); lane l of it fills slot l & 7
// of row l >> 3, so it fetches chunk (l & 7) ^ ((row >> 1) & 7) of that row from global memory.
//
// Operands are addressed as raw buffers: a wave-uniform base (the caller picks it so that every
// byte offset of the tile fits 32 bits) plus one 32-bit byte offset per load slot.
#ifndef UMAS_LOAD_PARTS
#define UMAS_LOAD_PARTS 2
#endif
template <class C>
struct DirectCfg {
  static constexpr int ROWB = 128;                                 // bytes per LDS row
  static constexpr int STAGEB = (C::BM + C::BN) * ROWB;            // bytes per stage
  static constexpr int LDS_BYTES = 2 * STAGEB;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0xFFFFFFFF, 0x00020000);
}

// K offset (in elements) of the chunk this thread fetches for all of its slots.
__device__ __forceinline__ int direct_kofs() {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  return 8 * ((lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7));
}

// oa[i] / ob[i]: byte offset from the operand's base of (row of slot i, k = direct_kofs()); rows outside
// the matrix are clamped to a valid row by the caller, which ignores what comes out of them.
template <class C>
__device__ __forceinline__ void mfma_mainloop_direct(__amdgpu_buffer_rsrc_t ra, const uint32_t (&oa)[C::NA],
                                                     __amdgpu_buffer_rsrc_t rb, const uint32_t (&ob)[C::NB], int K,
                                                     uint16_t* lds, floatx16 (&acc)[C::TM][C::TN]) {
  using D = DirectCfg<C>;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / C::WN, wn = wave % C::WN;
  char* base = reinterpret_cast<char*>(lds);
  const int nk = K / C::BK;

  // slot i of this wavefront fills rows [i*ROWS_PER_PASS + wave*8, +8) of the A (or B) area; the
  // loads of one K-step are issued in BK/16 parts, one part under each K-slice's MFMAs
  constexpr int kParts = C::BK / 16;
  constexpr int kLoadParts = UMAS_LOAD_PARTS;   // the loads are issued under the first kLoadParts K-slices
  static_assert(C::NA % kParts == 0 && C::NB % kParts == 0, "load slots split evenly over the K-slices");
  auto gload_part = [&](int kt, int stage, int part) {
    const int kbytes = kt * C::BK * 2;
    char* sa = base + stage * D::STAGEB + wave * 8 * D::ROWB;
    char* sb = sa + C::BM * D::ROWB;
#pragma unroll
    for (int i = part * (C::NA / kParts); i < (part + 1) * (C::NA / kParts); ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, reinterpret_cast<uint32_t*>(sa + i * C::ROWS_PER_PASS * D::ROWB), 16,
                                               oa[i], kbytes, 0, 0);
#pragma unroll
    for (int i = part * (C::NB / kParts); i < (part + 1) * (C::NB / kParts); ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, reinterpret_cast<uint32_t*>(sb + i * C::ROWS_PER_PASS * D::ROWB), 16,
                                               ob[i], kbytes, 0, 0);
  };

  // byte offsets of this lane's fragment chunk for the four K-slices of a stage
  const int sw = (lane >> 1) & 7;
  int coff[C::BK / 16];
#pragma unroll
  for (int kk = 0; kk < C::BK / 16; ++kk) coff[kk] = ((kk * 2 + (lane >> 5)) ^ sw) * 16;
  const int arow = (wm * C::WTM + (lane & 31)) * D::ROWB;
  const int brow = (C::BM + wn * C::WTN + (lane & 31)) * D::ROWB;

  bf16x8 af[2][C::TM], bfr[2][C::TN];
  auto fload = [&](int buf, int stage, int kk) {
    const char* sa = base + stage * D::STAGEB + arow + coff[kk];
    const char* sb = base + stage * D::STAGEB + brow + coff[kk];
#pragma unroll
    for (int tm = 0; tm < C::TM; ++tm) af[buf][tm] = *reinterpret_cast<const bf16x8*>(sa + tm * 32 * D::ROWB);
#pragma unroll
    for (int tn = 0; tn < C::TN; ++tn) bfr[buf][tn] = *reinterpret_cast<const bf16x8*>(sb + tn * 32 * D::ROWB);
  };

#pragma unroll
  for (int part = 0; part < kParts; ++part) gload_part(0, 0, part);
  __syncthreads();
  fload(0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    // The other stage was last read before the barrier that ended the previous step.  In the last
    // step the loads repeat the final tile, which nobody uses, to keep the loop branch-free.
    const int kn = kt + 1 < nk ? kt + 1 : kt;
#pragma unroll
    for (int kk = 0; kk < kParts; ++kk) {
      // Memory phase: a quarter of the next tile's global->LDS loads and the fragment reads of the
      // next K-slice.  Compute phase: the MFMAs of this slice, whose fragments were requested one
      // phase earlier.  The fences keep the two phases in this order so that every read has a whole
      // compute phase to land.
      if (kk < kLoadParts) {
#pragma unroll
        for (int part = kk * (kParts / kLoadParts); part < (kk + 1) * (kParts / kLoadParts); ++part)
          gload_part(kn, cur ^ 1, part);
      }
      if (kk + 1 < kParts) fload((kk + 1) & 1, cur, kk + 1);
#pragma unroll
      for (int tm = 0; tm < C::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < C::TN; ++tn)
          acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][tm], bfr[kk & 1][tn], acc[tm][tn], 0, 0, 0);
      // inside the slice: one memory instruction after each MFMA, so that their issue hides under the
      // matrix pipe (the reads and loads here feed later slices, never this one)
#pragma unroll
      for (int i = 0; i < C::TM * C::TN; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (kk + 1 < kParts && i < C::TM + C::TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        else if (kk < kLoadParts) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    fload(0, cur ^ 1, 0);
    __builtin_amdgcn_sched_barrier(0);
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
