// bf16 MFMA tile engine for gfx950: C[M,N] += A[M,K] * B[N,K]^T with both operands K-contiguous.
//
// A workgroup owns a BM x BN tile of C and walks K in steps of 64; each wavefront owns a
// (BM/WM) x (BN/WN) sub-tile as a grid of 32x32 blocks of v_mfma_f32_32x32x16_bf16 with float
// accumulators.  Two main loops: a general one (any K that is a multiple of 8: global memory is read
// in 16-byte vectors into registers one K-step ahead and written to one of two LDS stages of row
// pitch 72 bf16) and a fast one for K % 64 == 0 that fills the LDS straight from global memory.
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

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0xFFFFFFFF, 0x00020000);
}

// ---------------------------------------------------------------------------------------------
// Fast main loop for K % 64 == 0.
//
// K is walked in steps of 64: 128 bytes per row, the line size of the vector caches, so every line is
// fetched once.  Tiles go from global memory straight into one of two LDS stages of (BM + BN) x 128 bytes
// (buffer_load_dwordx4 ... lds: no staging registers, no ds_write); one wavefront-wide load fills 8
// consecutive rows (1 KB).  Operands are addressed as raw buffers: a wave-uniform base (the caller picks it
// so that every byte offset of the tile fits 32 bits) plus one 32-bit byte offset per load slot.  The 16-byte chunk c of row r sits in slot
// c ^ ((r >> 1) & 7), which keeps the fragment reads of 16 consecutive rows on distinct banks.
// Per step j (stage j & 1): loads of step j+1 go to the other stage right away (everybody left it before the
// barrier of the previous step); slices 0..2 run; then the wavefront waits for its own loads and LDS reads,
// the workgroup meets at the barrier, and slice 3 runs while the first fragments of the next stage are read.
template <class C>
struct Ring2Cfg {
  static constexpr int BK = 64;
  static constexpr int ROWB = 128;
  static constexpr int STAGEB = (C::BM + C::BN) * ROWB;
  static constexpr int LDS_BYTES = 2 * STAGEB;
  static constexpr int NA = C::BM * 8 / C::T, NB = C::BN * 8 / C::T;   // 16-byte loads per thread per step
  static constexpr int ROWS_PER_PASS = C::T / 8;
  static_assert(C::T % 64 == 0 && (C::BM * 8) % C::T == 0 && (C::BN * 8) % C::T == 0, "load slots divide evenly");
};
template <class C>
__device__ __forceinline__ int ring2_row(int i) { return i * (C::T / 8) + (threadIdx.x >> 3); }
// K offset (elements) of the chunk this lane fetches: slot (tid & 7) of row ring2_row holds chunk slot ^ ((row >> 1) & 7);
// rows per pass and wavefront row offsets are multiples of 8, so (row >> 1) & 7 = ((tid >> 3) >> 1) & 7 with tid >> 3 < 64
__device__ __forceinline__ int ring2_kofs() {
  const int t = threadIdx.x;
  return 8 * ((t & 7) ^ (((t >> 3) >> 1) & 7));
}

template <class C>
__device__ __forceinline__ void mfma_mainloop_ring2(__amdgpu_buffer_rsrc_t ra, const uint32_t (&oa)[Ring2Cfg<C>::NA],
                                                    __amdgpu_buffer_rsrc_t rb, const uint32_t (&ob)[Ring2Cfg<C>::NB],
                                                    int K, uint16_t* lds, floatx16 (&acc)[C::TM][C::TN]) {
  using R = Ring2Cfg<C>;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / C::WN, wn = wave % C::WN;
  char* base = reinterpret_cast<char*>(lds);
  const int nsub = K / R::BK;

  auto gload = [&](int sub, int stage) {
    const int kbytes = sub * R::BK * 2;
    char* sa = base + stage * R::STAGEB + wave * 8 * R::ROWB;
    char* sb = sa + C::BM * R::ROWB;
#pragma unroll
    for (int i = 0; i < R::NA; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, reinterpret_cast<uint32_t*>(sa + i * R::ROWS_PER_PASS * R::ROWB), 16,
                                               oa[i], kbytes, 0, 0);
#pragma unroll
    for (int i = 0; i < R::NB; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, reinterpret_cast<uint32_t*>(sb + i * R::ROWS_PER_PASS * R::ROWB), 16,
                                               ob[i], kbytes, 0, 0);
  };
  const int sw = (lane >> 1) & 7;                    // (row >> 1) & 7 of this lane's fragment rows
  const int arow = (wm * C::WTM + (lane & 31)) * R::ROWB;
  const int brow = (C::BM + wn * C::WTN + (lane & 31)) * R::ROWB;
  bf16x8 af[2][C::TM], bfr[2][C::TN];
  auto fload = [&](int buf, int stage, int kk) {
    const int coff = ((2 * kk + (lane >> 5)) ^ sw) * 16;
    const char* sa = base + stage * R::STAGEB + arow + coff;
    const char* sb = base + stage * R::STAGEB + brow + coff;
#pragma unroll
    for (int tm = 0; tm < C::TM; ++tm) af[buf][tm] = *reinterpret_cast<const bf16x8*>(sa + tm * 32 * R::ROWB);
#pragma unroll
    for (int tn = 0; tn < C::TN; ++tn) bfr[buf][tn] = *reinterpret_cast<const bf16x8*>(sb + tn * 32 * R::ROWB);
  };
  auto mfmas = [&](int buf) {
#pragma unroll
    for (int tm = 0; tm < C::TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < C::TN; ++tn)
        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][tm], bfr[buf][tn], acc[tm][tn], 0, 0, 0);
  };
  auto interleave = [&](int n_ds, int n_vm) {
#pragma unroll
    for (int i = 0; i < C::TM * C::TN; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < n_ds) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if (i < n_vm) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
  };

  gload(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
  fload(0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  for (int j = 0; j < nsub; ++j) {
    const int st = j & 1;
    // past the end of K the loads repeat the last step (nobody reads them)
    gload(j + 1 < nsub ? j + 1 : nsub - 1, st ^ 1);
    fload(1, st, 1);
    mfmas(0);
    interleave(C::TM + C::TN, R::NA + R::NB);
    __builtin_amdgcn_sched_barrier(0);
    fload(0, st, 2);
    mfmas(1);
    interleave(C::TM + C::TN, 0);
    __builtin_amdgcn_sched_barrier(0);
    fload(1, st, 3);
    mfmas(0);
    interleave(C::TM + C::TN, 0);
    __builtin_amdgcn_sched_barrier(0);
    // own loads of the next stage landed, own reads of this stage done; then everybody's
    __builtin_amdgcn_s_waitcnt(0x0070);              // vmcnt(0) and lgkmcnt(0), expcnt untouched (gfx9 encoding)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    fload(0, st ^ 1, 0);
    mfmas(1);
    interleave(C::TM + C::TN, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
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
