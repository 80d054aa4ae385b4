// bf16 MFMA tile engine for gfx950: C[M,N] += A[M,K] * B[N,K]^T with both operands K-contiguous.
//
// A workgroup owns a BM x BN tile of C and walks K in steps of 64; each wavefront owns a
// (BM/WM) x (BN/WN) sub-tile as a grid of 16x16 blocks of v_mfma_f32_16x16x32_bf16 with float
// accumulators (on random operands a register-only loop of this instruction sustains 2.0 PFLOP/s on this
// part, one of the 32x32x16 form 1.77: the chip runs into its power limit later).  Two main loops: a
// general one (any K that is a multiple of 8: global memory is read in 16-byte vectors into registers one
// K-step ahead and written to one of two LDS stages of row pitch 72 bf16) and a fast one for K % 64 == 0
// that fills the LDS straight from global memory.
//
// Operand layout of one block (lane l): row (or column) l % 16, k = 8 (l / 16) .. 8 (l / 16) + 7.
// Accumulator layout of one 16x16 block (register r of lane l):
//   row (A side, "M")  = 4*(l/16) + r
//   col (B side, "N")  = l%16
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace umas {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

template <int BM_, int BN_, int WM_, int WN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int BK = 64;
  static constexpr int LDP = 72;                       // LDS row pitch in bf16 elements
  static constexpr int T = 64 * WM * WN;               // threads per workgroup
  static constexpr int WTM = BM / WM, WTN = BN / WN;   // wavefront sub-tile
  static constexpr int MI = WTM / 16, NI = WTN / 16;   // 16x16 blocks per wavefront
  static constexpr int NA = BM * 8 / T, NB = BN * 8 / T;   // 16-byte vectors per thread per K-step
  static constexpr int ROWS_PER_PASS = T / 8;          // rows covered by one vector slot of all threads
  static constexpr int STAGE = (BM + BN) * LDP;        // bf16 elements per LDS stage
  static constexpr int LDS_BYTES = 2 * STAGE * 2;
  static_assert(BM % (32 * WM) == 0 && BN % (16 * WN) == 0, "sub-tiles are grids of 16x16 blocks, an even number along M");
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
                                              int K, uint16_t* lds, floatx4 (&acc)[C::MI][C::NI]) {
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
    // operand of a 16x16x32 block: lane l holds row l % 16, k = 8 (l / 16) .. + 7 of the 32-wide slice
    const uint16_t* sa = lds + stage * C::STAGE + (wm * C::WTM + (lane & 15)) * C::LDP + (lane >> 4) * 8;
    const uint16_t* sb = lds + stage * C::STAGE + (C::BM + wn * C::WTN + (lane & 15)) * C::LDP + (lane >> 4) * 8;
#pragma unroll
    for (int kk = 0; kk < C::BK / 32; ++kk) {
      bf16x8 af[C::MI], bfr[C::NI];
#pragma unroll
      for (int i = 0; i < C::MI; ++i) af[i] = *reinterpret_cast<const bf16x8*>(sa + i * 16 * C::LDP + kk * 32);
#pragma unroll
      for (int j = 0; j < C::NI; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(sb + j * 16 * C::LDP + kk * 32);
#pragma unroll
      for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
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
// fetched once.  Tiles go from global memory straight into LDS stages of 256 rows x 128 bytes per operand
// (buffer_load_dwordx4 ... lds: no staging registers, no ds_write); one wavefront-wide load fills 8
// consecutive rows (1 KB).  Operands are addressed as raw buffers: a wave-uniform base (the caller picks it
// so that every byte offset of the tile fits 32 bits) plus one 32-bit byte offset per load slot.  The 16-byte chunk c of row r sits in slot
// c ^ ((r >> 1) & 7), which keeps the fragment reads of 16 consecutive rows on distinct banks.
// Operand A has three stages and is loaded two steps ahead, operand B two stages, one step ahead (the callers
// put the operand that comes from farther away in A).  Per step j: the loads of B for step j+1 and of A for step
// j+2 go out right away (everybody left those stages before the barrier of the previous step); phases 0..2 run;
// then the wavefront waits for its LDS reads and for all loads but the youngest ones (A of step j+2: loads into
// LDS return in the order they were issued), the workgroup meets at the barrier, and phase 3 runs while the first
// fragments of the next step are read.
template <class C>
struct Ring2Cfg {
  static constexpr int BK = 64;
  static constexpr int ROWB = 128;
  static constexpr int ASTAGE = C::BM * ROWB, BSTAGE = C::BN * ROWB;   // bytes of one stage of an operand
  static constexpr int BBASE = 3 * ASTAGE;                             // three stages of A, then two of B
  static constexpr int LDS_BYTES = BBASE + 2 * BSTAGE;
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
                                                    int K, uint16_t* lds, floatx4 (&acc)[C::MI][C::NI]) {
  using R = Ring2Cfg<C>;
  constexpr int HA = C::MI / 2;                      // A blocks of one half of the wavefront's sub-tile
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / C::WN, wn = wave % C::WN;
  char* base = reinterpret_cast<char*>(lds);
  const int nsub = K / R::BK;

  static_assert(R::NA == 4, "the wait before the barrier leaves four loads outstanding");
  auto gload_a = [&](int sub, int ia) {
    const int kbytes = sub * R::BK * 2;
    char* sa = base + ia * R::ASTAGE + wave * 8 * R::ROWB;
#pragma unroll
    for (int i = 0; i < R::NA; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, reinterpret_cast<uint32_t*>(sa + i * R::ROWS_PER_PASS * R::ROWB), 16,
                                               oa[i], kbytes, 0, 0);
  };
  auto gload_b = [&](int sub, int ib) {
    const int kbytes = sub * R::BK * 2;
    char* sb = base + R::BBASE + ib * R::BSTAGE + wave * 8 * R::ROWB;
#pragma unroll
    for (int i = 0; i < R::NB; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, reinterpret_cast<uint32_t*>(sb + i * R::ROWS_PER_PASS * R::ROWB), 16,
                                               ob[i], kbytes, 0, 0);
  };
  // Operand of a 16x16x32 block: lane l holds row l % 16, k = 8 (l / 16) .. + 7 of the 32-wide slice, i.e. chunk
  // 4 s + l / 16 of the row.  A step is four phases of 16 MFMAs: (slice 0, upper half of the A rows), (slice 0,
  // lower half), (slice 1, upper), (slice 1, lower); the B fragments of a slice serve both of its phases.
  const int sw = (lane >> 1) & 7;                    // (row >> 1) & 7 of this lane's fragment rows
  const int arow = (wm * C::WTM + (lane & 15)) * R::ROWB;
  const int brow = R::BBASE + (wn * C::WTN + (lane & 15)) * R::ROWB;
  bf16x8 af[2][HA], bfr[2][C::NI];
  auto fload_a = [&](int buf, int ia, int s, int h) {
    const int coff = ((4 * s + (lane >> 4)) ^ sw) * 16;
    const char* sa = base + ia * R::ASTAGE + arow + coff + h * HA * 16 * R::ROWB;
#pragma unroll
    for (int i = 0; i < HA; ++i) af[buf][i] = *reinterpret_cast<const bf16x8*>(sa + i * 16 * R::ROWB);
  };
  auto fload_b = [&](int buf, int ib, int s) {
    const int coff = ((4 * s + (lane >> 4)) ^ sw) * 16;
    const char* sb = base + ib * R::BSTAGE + brow + coff;
#pragma unroll
    for (int j = 0; j < C::NI; ++j) bfr[buf][j] = *reinterpret_cast<const bf16x8*>(sb + j * 16 * R::ROWB);
  };
  auto mfmas = [&](int abuf, int bbuf, int h) {
#pragma unroll
    for (int i = 0; i < HA; ++i)
#pragma unroll
      for (int j = 0; j < C::NI; ++j)
        acc[h * HA + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[abuf][i], bfr[bbuf][j], acc[h * HA + i][j], 0, 0, 0);
  };
  auto interleave = [&](int n_ds, int n_vm) {
#pragma unroll
    for (int i = 0; i < HA * C::NI; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < n_ds) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if (i < n_vm) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
  };

  auto clamp_sub = [&](int sub) { return sub < nsub ? sub : nsub - 1; };   // past the end of K the loads repeat the last step (nobody reads them)
  gload_a(0, 0);
  gload_b(0, 0);
  gload_a(clamp_sub(1), 1);
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
  fload_b(0, 0, 0);
  fload_a(0, 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  int ia = 0;                                        // A stage of the current step
  for (int j = 0; j < nsub; ++j) {
    const int ib = j & 1;
    const int ia1 = ia == 2 ? 0 : ia + 1, ia2 = ia1 == 2 ? 0 : ia1 + 1;
    gload_b(clamp_sub(j + 1), ib ^ 1);
    gload_a(clamp_sub(j + 2), ia2);
    fload_a(1, ia, 0, 1);
    mfmas(0, 0, 0);
    interleave(HA, R::NA + R::NB);
    __builtin_amdgcn_sched_barrier(0);
    fload_b(1, ib, 1);
    fload_a(0, ia, 1, 0);
    mfmas(1, 0, 1);
    interleave(HA + C::NI, 0);
    __builtin_amdgcn_sched_barrier(0);
    fload_a(1, ia, 1, 1);
    mfmas(0, 1, 0);
    interleave(HA, 0);
    __builtin_amdgcn_sched_barrier(0);
    // own reads of this step done, own loads for the next step landed (the four youngest, A of the step after
    // next, may still be on their way); then everybody's
    __builtin_amdgcn_s_waitcnt(0x0074);              // vmcnt(4) and lgkmcnt(0), expcnt untouched (gfx9 encoding)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    fload_b(0, ib ^ 1, 0);
    fload_a(0, ia1, 0, 0);
    mfmas(1, 1, 1);
    interleave(HA + C::NI, 0);
    __builtin_amdgcn_sched_barrier(0);
    ia = ia1;
  }
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
}

// ---------------------------------------------------------------------------------------------
// The same loop for operands that are not K-contiguous in memory.
//
// An operand stored K-major (row k holds the 256 tile entries of that k next to each other, 512 bytes) is
// brought into LDS as it lies: a stage holds 64 k-rows of 512 bytes, one wavefront-wide load fills two of
// them.  Fragments come out through ds_read_b64_tr_b16, which transposes on the way: in a group of 16
// lanes, lane l receives element l % 4 of the 8-byte chunks addressed by lanes l / 4, l / 4 + 4, l / 4 + 8
// and l / 4 + 12.  Lane i = q + 4 j of a group therefore points at k-row kbase + j, entries 4 q .. 4 q + 3
// of the block's 16, and lane l ends up with entry l of the 16 for the four k of the read; two reads give
// the eight k of a 16x16x32 operand, group g of the wavefront taking k-rows 8 g .. 8 g + 7 of the slice.
// The 16-byte unit u of k-row k sits in slot u ^ (4 (k & 3)) ^ (2 ((k >> 3) & 1)), which keeps the 32 lanes
// served in one cycle (two groups, four k-rows each) on distinct banks.
typedef short short4v __attribute__((ext_vector_type(4)));

template <class C>
struct MixedLdsBytes {          // LDS of mfma_mainloop_mixed: three A stages and two B stages of 32 KB, like the ring's
  static constexpr int value = Ring2Cfg<C>::LDS_BYTES;
};
struct KMajor {                 // an operand tile stored K-major
  const char* base;             // byte address of (k-row 0, first entry of the tile)
  int64_t ld_bytes;             // bytes between consecutive k-rows
  int64_t hi_bytes;             // added once more per 256 k-rows (an operand stored in blocks of 256 rows), else 0
  const int32_t* rowmap;        // with BMAP: k-row k lives in row rowmap[k] of the matrix (ld_bytes apart, from base)
  int k_rows;                   // k-rows that exist; later ones read the last one (the other operand is zero there)
  int n_units;                  // 16-byte units of a k-row that exist from base on (<= 32); later ones read the last one
};
struct KContig {                // an operand tile stored K-contiguous: per-slot byte offsets from a base
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t off[4];
  uint32_t hi_bytes;            // added once more per 256 k (an operand stored in blocks of 256 columns), else 0
};

template <class C, bool ATR, bool BTR, bool BMAP = false, int AHEAD = (BMAP ? 0 : 1)>
__device__ __forceinline__ void mfma_mainloop_mixed(const KContig& ca, const KMajor& ka, const KContig& cb, const KMajor& kb,
                                                    int K, uint16_t* lds, floatx4 (&acc)[C::MI][C::NI]) {
  using R = Ring2Cfg<C>;
  static_assert(C::BM == 256 && C::BN == 256 && C::T == 512 && R::NA == 4 && R::NB == 4, "written for 256x256 tiles, 8 wavefronts");
  constexpr int HA = C::MI / 2;                      // A blocks of one half of the wavefront's sub-tile
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / C::WN, wn = wave % C::WN;
  char* base = reinterpret_cast<char*>(lds);
  const int nsub = K / R::BK;
  // LDS: five stages of 32 KB.  One operand (AHEAD = 1: A, AHEAD = 2: B) has three of them and is loaded two steps
  // ahead, the other two, one step ahead; the callers give the third stage to the operand that comes from farther
  // away.  With a row map on B (loads of two kinds in flight, which do not return in one order) AHEAD is 0 and both
  // stay one step ahead.
  static_assert(AHEAD >= 0 && AHEAD <= 2 && !(BMAP && AHEAD != 0), "which operand is loaded two steps ahead");
  constexpr int kAStage = C::BM * R::ROWB, kBStage = C::BN * R::ROWB;
  constexpr int kABase = AHEAD == 2 ? 3 * kBStage : 0, kBBase = AHEAD == 2 ? 0 : 3 * kAStage;
  static_assert(3 * kAStage + 2 * kBStage <= MixedLdsBytes<C>::value && kAStage == kBStage, "LDS of the mixed loop");

  // K-major loads: pass p covers k-rows 16 p .. 16 p + 15, this wavefront rows 16 p + 2 wave, + 1; lane l fills slot
  // l & 31 of row k = 16 p + 2 wave + (l >> 5) and fetches unit slot ^ 4 (k & 3) ^ 2 ((k >> 3) & 1)
  const int tr_krow = 2 * wave + (lane >> 5);        // + 16 p
  const int tr_slot_unit = (lane & 31) ^ (4 * (tr_krow & 3)) ^ (2 * ((tr_krow >> 3) & 1));
  int32_t rows_a[4] = {0, 0, 0, 0}, rows_b[4] = {0, 0, 0, 0};   // rows of the step after next when a rowmap is set
  auto map_rows = [&](const KMajor& k, int sub, int32_t (&rows)[4]) {
#pragma unroll
    for (int p = 0; p < 4; ++p) rows[p] = k.rowmap[min(sub * R::BK + 16 * p + tr_krow, k.k_rows - 1)];
  };
  auto gload_kmajor = [&](const KMajor& k, const int32_t (&rows)[4], int sub, char* region, auto mapped) {
    const uint32_t ubytes = static_cast<uint32_t>(min(tr_slot_unit, k.n_units - 1)) * 16u;
    if constexpr (decltype(mapped)::value) {
      const __amdgpu_buffer_rsrc_t r = make_rsrc(k.base);
#pragma unroll
      for (int p = 0; p < 4; ++p)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r, reinterpret_cast<uint32_t*>(region + (16 * p + 2 * wave) * 512), 16,
                                                 static_cast<uint32_t>(rows[p]) * static_cast<uint32_t>(k.ld_bytes) + ubytes, 0, 0, 0);
    } else {
      const int k0 = min(sub * R::BK, ((k.k_rows - 1) / R::BK) * R::BK);          // first k-row of the (clamped) step
      const __amdgpu_buffer_rsrc_t r = make_rsrc(k.base + static_cast<int64_t>(k0) * k.ld_bytes + (k0 >> 8) * k.hi_bytes);
#pragma unroll
      for (int p = 0; p < 4; ++p)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r, reinterpret_cast<uint32_t*>(region + (16 * p + 2 * wave) * 512), 16,
                                                 static_cast<uint32_t>(min(16 * p + tr_krow, k.k_rows - 1 - k0)) * static_cast<uint32_t>(k.ld_bytes) + ubytes,
                                                 0, 0, 0);
    }
  };
  auto gload_kcontig = [&](const KContig& c, int sub, char* region) {
    const int kbytes = sub * R::BK * 2 + (sub >> 2) * static_cast<int>(c.hi_bytes);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(c.rsrc, reinterpret_cast<uint32_t*>(region + (i * R::ROWS_PER_PASS + wave * 8) * R::ROWB), 16,
                                               c.off[i], kbytes, 0, 0);
  };
  auto gload_a = [&](int sub, int ia) {
    char* sa = base + kABase + ia * kAStage;
    if (ATR) gload_kmajor(ka, rows_a, sub, sa, std::false_type{}); else gload_kcontig(ca, sub, sa);
  };
  auto gload_b = [&](int sub, int ib) {
    char* sb = base + kBBase + ib * kBStage;
    if (BTR) gload_kmajor(kb, rows_b, sub, sb, std::integral_constant<bool, BMAP>{}); else gload_kcontig(cb, sub, sb);
  };

  // fragment addresses (K-contiguous operands as in mfma_mainloop_ring2)
  const int sw = (lane >> 1) & 7;
  const int arow = (wm * C::WTM + (lane & 15)) * R::ROWB;
  const int brow = (wn * C::WTN + (lane & 15)) * R::ROWB;
  const int tq = lane & 3, tj = (lane >> 2) & 3;     // position q + 4 j inside the group of 16 lanes
  const int tg = lane >> 4;                          // the group: k-rows 8 g .. 8 g + 7 of a slice
  // The transposing reads are issued as inline assembly: the compiler cannot tell that they do not touch the stage
  // the LDS-filling loads are writing and would wait for those loads before every one of them.  Their results are
  // therefore handed over by an explicit wait (tr_wait_*) that also names the registers, so that no use moves above it.
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (__attribute__((address_space(3))) char*)(base)));
  // LDS byte address of this lane's chunk for block t (16 entries = two units) of an operand whose sub-tile starts at
  // unit u0: k-row 8 g + j, 8-byte half of the unit, unit slot; stage, region, slice and the + 4 k-rows of the second
  // read are added as offsets
  auto tr_addr = [&](int u0, int t) -> uint32_t {
    const int unit = u0 + t * 2 + (tq >> 1);
    return lds0 + (tg * 8 + tj) * 512 + (tq & 1) * 8 + ((unit ^ (4 * tj) ^ (2 * (tg & 1))) * 16);
  };
  uint32_t tra[C::MI], trb[C::NI];
#pragma unroll
  for (int i = 0; i < C::MI; ++i) tra[i] = tr_addr(wm * (C::WTM / 8), i);
#pragma unroll
  for (int j = 0; j < C::NI; ++j) trb[j] = tr_addr(wn * (C::WTN / 8), j);
  typedef short short8v __attribute__((ext_vector_type(8)));
  bf16x8 af[2][HA], bfr[2][C::NI];
  auto fload_a = [&](int buf, int ia, auto s_c, auto h_c) {
    constexpr int s = decltype(s_c)::value, h = decltype(h_c)::value;
    const uint32_t stoff = kABase + static_cast<uint32_t>(ia) * kAStage;
#pragma unroll
    for (int i = 0; i < HA; ++i) {
      if (ATR) {
        short4v lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(tra[h * HA + i] + stoff), "n"(s * 32 * 512));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(tra[h * HA + i] + stoff), "n"(s * 32 * 512 + 4 * 512));
        const short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        af[buf][i] = __builtin_bit_cast(bf16x8, v);
      } else {
        const int coff = ((4 * s + (lane >> 4)) ^ sw) * 16;
        af[buf][i] = *reinterpret_cast<const bf16x8*>(base + stoff + arow + coff + (h * HA + i) * 16 * R::ROWB);
      }
    }
  };
  auto fload_b = [&](int buf, int ib, auto s_c) {
    constexpr int s = decltype(s_c)::value;
    const uint32_t stoff = kBBase + static_cast<uint32_t>(ib) * kBStage;
#pragma unroll
    for (int j = 0; j < C::NI; ++j) {
      if (BTR) {
        short4v lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(trb[j] + stoff), "n"(s * 32 * 512));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(trb[j] + stoff), "n"(s * 32 * 512 + 4 * 512));
        const short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        bfr[buf][j] = __builtin_bit_cast(bf16x8, v);
      } else {
        const int coff = ((4 * s + (lane >> 4)) ^ sw) * 16;
        bfr[buf][j] = *reinterpret_cast<const bf16x8*>(base + stoff + brow + coff + j * 16 * R::ROWB);
      }
    }
  };
  // every LDS read issued so far has returned; the named fragments may be used from here on
  auto tr_wait_a = [&](int buf) {
    if (ATR) {
#pragma unroll
      for (int i = 0; i < HA; ++i) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(af[buf][i]));
    }
  };
  auto tr_wait_b = [&](int buf) {
    if (BTR) {
#pragma unroll
      for (int j = 0; j < C::NI; ++j) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bfr[buf][j]));
    }
  };
  auto mfmas = [&](int abuf, int bbuf, int h) {
#pragma unroll
    for (int i = 0; i < HA; ++i)
#pragma unroll
      for (int j = 0; j < C::NI; ++j)
        acc[h * HA + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[abuf][i], bfr[bbuf][j], acc[h * HA + i][j], 0, 0, 0);
  };

  constexpr int kDsA = (ATR ? 2 : 1) * HA, kDsB = (BTR ? 2 : 1) * C::NI;   // LDS reads of an A half, of a slice of B
  auto interleave = [&](int n_ds, int n_vm) {
#pragma unroll
    for (int i = 0; i < HA * C::NI; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < n_ds) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if (i < n_vm) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  auto clamp_sub = [&](int sub) { return sub < nsub ? sub : nsub - 1; };   // past the end the last step is loaded again (nobody reads it)
  if (BTR && BMAP) map_rows(kb, 0, rows_b);
  gload_a(0, 0);
  gload_b(0, 0);
  if (AHEAD == 1) gload_a(clamp_sub(1), 1);
  if (AHEAD == 2) gload_b(clamp_sub(1), 1);
  if (BTR && BMAP) map_rows(kb, clamp_sub(1), rows_b);
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
  fload_b(0, 0, I0{});
  fload_a(0, 0, I0{}, I0{});
  auto next3 = [](int i) { return i == 2 ? 0 : i + 1; };
  int ia = 0, ib = 0;                                // stages of the current step
  for (int j = 0; j < nsub; ++j) {
    const int ia1 = AHEAD == 1 ? next3(ia) : (ia ^ 1);              // stages of the next step
    const int ib1 = AHEAD == 2 ? next3(ib) : (ib ^ 1);
    tr_wait_a(0);
    tr_wait_b(0);
    if (AHEAD == 1) {                                // the loads that may stay outstanding go out last
      gload_b(clamp_sub(j + 1), ib1);
      gload_a(clamp_sub(j + 2), next3(ia1));
    } else if (AHEAD == 2) {
      gload_a(clamp_sub(j + 1), ia1);
      gload_b(clamp_sub(j + 2), next3(ib1));
    } else {
      gload_a(clamp_sub(j + 1), ia1);
      gload_b(clamp_sub(j + 1), ib1);
    }
    if (BTR && BMAP) map_rows(kb, clamp_sub(j + 2), rows_b);
    fload_a(1, ia, I0{}, I1{});
    mfmas(0, 0, 0);
    interleave(kDsA, 8);
    __builtin_amdgcn_sched_barrier(0);
    tr_wait_a(1);
    fload_b(1, ib, I1{});
    fload_a(0, ia, I1{}, I0{});
    mfmas(1, 0, 1);
    interleave(kDsA + kDsB, 0);
    __builtin_amdgcn_sched_barrier(0);
    tr_wait_a(0);
    tr_wait_b(1);
    fload_a(1, ia, I1{}, I1{});
    mfmas(0, 1, 0);
    interleave(kDsA, 0);
    __builtin_amdgcn_sched_barrier(0);
    // own LDS reads of this step done and own loads for the next step landed: with three A stages the four
    // youngest loads (A of the step after next) may still be on their way; then everybody's
    if (AHEAD != 0) __builtin_amdgcn_s_waitcnt(0x0074);   // vmcnt(4), lgkmcnt(0)
    else __builtin_amdgcn_s_waitcnt(0x0070);         // vmcnt(0), lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    tr_wait_a(1);
    fload_b(0, ib1, I0{});
    fload_a(0, ia1, I0{}, I0{});
    mfmas(1, 1, 1);
    interleave(kDsA + kDsB, 0);
    __builtin_amdgcn_sched_barrier(0);
    ia = ia1;
    ib = ib1;
  }
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
}

// Position of accumulator element r of block (i, j) inside the workgroup tile: row 4 (l / 16) + r, column l % 16 of the block.
template <class C>
__device__ __forceinline__ int acc_row(int i, int r) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  return (wave / C::WN) * C::WTM + i * 16 + (lane >> 4) * 4 + r;
}
template <class C>
__device__ __forceinline__ int acc_col(int j) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  return (wave % C::WN) * C::WTN + j * 16 + (lane & 15);
}

// Workgroups are handed to the 8 XCDs round-robin; give every XCD a contiguous range of the
// logical tile order, and order tiles in groups of GM x GN so that the workgroups resident on
// one XCD share operand rows through its L2.  A workgroup handles `per_wg` tiles one after the other:
// the tile with the same place in `per_wg` consecutive groups, so that the workgroups of an XCD keep
// working on one group at a time.  Returns false when iteration `it` of this workgroup has no tile.
template <int GM, int GN>
__device__ __forceinline__ bool tile_coords(int tiles_m, int tiles_n, int* tm, int* tn, int it = 0, int per_wg = 1) {
  const int total_groups_n = (tiles_n + GN - 1) / GN;
  const int total_groups_m = (tiles_m + GM - 1) / GM;
  const long long groups = static_cast<long long>(total_groups_m) * total_groups_n;
  const long long groups_per_xcd = (groups + 7) / 8;                       // contiguous range of groups per XCD
  const long long bid = blockIdx.x;
  const long long w = bid >> 3;                                            // workgroup number inside its XCD
  const long long grp_in_xcd = (w / (GM * GN)) * per_wg + it;
  const int within = static_cast<int>(w % (GM * GN));
  if (grp_in_xcd >= groups_per_xcd) return false;
  const long long grp = (bid & 7) * groups_per_xcd + grp_in_xcd;
  if (grp >= groups) return false;
  const int gm = static_cast<int>(grp / total_groups_n), gn = static_cast<int>(grp % total_groups_n);
  *tm = gm * GM + within % GM;
  *tn = gn * GN + within / GM;
  return *tm < tiles_m && *tn < tiles_n;
}
// The same order with an explicit share of the groups per XCD: XCD x owns groups first[x] .. first[x + 1] - 1.
// `bid` is the workgroup's number among the workgroups that use this table (a multiple of 8 lies before it in
// the grid, so bid % 8 is still its XCD).
struct XcdGroups {
  int first[9];
};
template <int GM, int GN>
__device__ __forceinline__ bool tile_coords_shared(int tiles_m, int tiles_n, long long bid, const XcdGroups& g, int* tm, int* tn) {
  const int total_groups_n = (tiles_n + GN - 1) / GN;
  const int xcd = static_cast<int>(bid & 7);
  const long long w = bid >> 3;
  const long long grp = g.first[xcd] + w / (GM * GN);
  const int within = static_cast<int>(w % (GM * GN));
  if (grp >= g.first[xcd + 1]) return false;
  const int gm = static_cast<int>(grp / total_groups_n), gn = static_cast<int>(grp % total_groups_n);
  *tm = gm * GM + within % GM;
  *tn = gn * GN + within / GM;
  return *tm < tiles_m && *tn < tiles_n;
}
template <int GM, int GN>
inline unsigned tile_grid(int tiles_m, int tiles_n, int per_wg = 1) {
  const long long groups = static_cast<long long>((tiles_m + GM - 1) / GM) * ((tiles_n + GN - 1) / GN);
  const long long groups_per_xcd = (groups + 7) / 8;
  const long long wg_groups = (groups_per_xcd + per_wg - 1) / per_wg;       // groups of workgroups per XCD
  return static_cast<unsigned>(wg_groups * (GM * GN) * 8);
}

}  // namespace umas
