// Grouped bf16 GEMM core for gfx950 matrix cores, shared by every dense contraction of the layer:
//
//   C[m, n] = sum_k A(m, k) * B(k, n)          fp32 accumulation, v_mfma_f32_32x32x16_bf16
//
// Each operand is contiguous either along the contraction index or along its own index:
//   A k-contiguous (rows indexed by m) / B k-contiguous (rows indexed by n): router and key scores (Eq. 5, Eq. 6)
//     and dOut . V^T in the backward;
//   B n-contiguous (rows indexed by k): where the contraction runs over neurons or tokens while the rows of V, K,
//     dOut, h are contiguous in d: the value sum of Eq. 4, dh, dK, dV;
//   A m-contiguous (rows indexed by k): dK, dV, whose A operand is the slot-major activation matrix, read as it is.
//
// Tile TM (m) x 256 (n) x 64 (k), a policy's kTM.  Two shapes of workgroup:
//   kTM = 128 (or 192): 4 compute waves as 2 x 2, each wave TM/2 x 128 = (TM/64) x 4 MFMA tiles, plus two or four
//     loader waves that own the whole global -> LDS traffic (16 B per lane).  Ring depths kSA, kSB up to three.
//     Used by the router, the token-major problems and (as an option) the neuron-major ones.
//   kTM = 256: 8 compute waves as 4 x 2, each wave 64 x 128, and no loader waves (kLoaders = 0): the accumulators of
//     8 waves leave no registers for further waves on their SIMDs, so every compute wave requests an eighth of the
//     operands itself, right after each barrier.  Two slots per ring (128 KB).  Used by the neuron-major problems
//     (dV, dK), whose output has no ragged edge: a third fewer operand bytes per flop through L2 -> LDS, and half as
//     many store phases.  Measured at the LLaMA-7B-shaped configuration: dV 0.355 -> 0.340 ms, dK 0.345 -> 0.339 ms.
// The operands have a ring each in LDS: kSA slots of TM x 64 for A, kSB slots of 256 x 64 for B.  (A 192-row tile
// for the token-major problems moves 22 % fewer operand bytes per flop than the 128-row one and was measured 15 %
// faster per flop, but their groups then fill a whole number of tiles worse and the step as a whole did not gain.)
// LDS layouts are XOR-swizzled so that both the linear DMA writes and the fragment reads are free of bank conflicts:
//   k-contiguous operand: rows of 64 k = 8 chunks of 16 B; logical chunk c of row r sits at chunk
//     c ^ ((r >> 1) & 7); fragments are read with ds_read_b128.
//   n-contiguous B, and m-contiguous A of 256 rows: rows of 256 = 32 chunks; logical chunk c of row k sits at chunk
//     c ^ (2 * (k & 7));
//   m-contiguous A of 128 rows: 16 chunks per row; logical chunk c of row k sits at chunk c ^ (4 * (k & 3));
//     these are read with the transposing ds_read_b64_tr_b16, which hands lane i of a 16-lane group the four
//     k-consecutive values of column i of a 4 x 16 block.
//
// The k tiles of all the tiles a workgroup works through form ONE stream through the rings: right after the barrier
// that hands position s to the compute waves, A of position s + kSA - 1 and B of position s + kSB - 1 are requested
// (the operand with the shorter lead first), whether or not those belong to the next output tile, so the operand
// pipeline never drains at a tile boundary.  There is exactly one workgroup barrier per k tile of the stream,
// executed by all the waves.  (An extra barrier at the end of every tile, releasing its last stage before the stores
// so that the loaders request a third k tile during the epilogue, was measured and did not pay.)
//
// With loader waves, a compute wave keeps two register sets of fragments: the LDS reads of k16 step s + 1 are issued
// before the matrix instructions of step s, and the barrier of the next k tile sits in front of the last matrix
// instructions of the current one.
//
// The epilogue needs neither LDS nor barriers: neighbouring lanes exchange one accumulator value through a DPP
// move, so that every lane holds two adjacent columns of one row, and hands them to the policy, which stores them
// (4 bytes of bf16, converted before the exchange, or 8 bytes of fp32 per lane; a half wave writes 64 or 128
// contiguous bytes of each of two rows per instruction).  While the compute waves store, the loaders are already
// up to two k tiles into the next tile.
//
// Workgroups are mapped to tiles XCD-aware: consecutive workgroup ids go round-robin to the 8 XCDs,
// so workgroup id w works for XCD w % 8, and all tiles of one group (block of neurons) are given to
// one XCD, consecutively, so that the group's operand panels are fetched from HBM once and shared in
// that XCD's L2.
#pragma once
#include <type_traits>

#include "common.h"

namespace meft {

constexpr int kTN = 256, kTK = 64;
#ifndef MEFT_TOK_TM
#define MEFT_TOK_TM 128
#define MEFT_TOK_SA 3
#define MEFT_TOK_SB 3
#endif
#ifndef MEFT_NEU_TM
#define MEFT_NEU_TM 256
#endif
constexpr int kTMTok = MEFT_TOK_TM;    // tile rows of the token-major problems (groups of tokens against a block's rows)
constexpr int kTMNeu = 128;            // tile rows of the router
constexpr int kTMNeuW = MEFT_NEU_TM;   // largest tile rows of the neuron-major problems (dV, dK): 256; 128 rules the larger tile out
constexpr int kBSlotElems = kTN * kTK;                         // one B slot: 32 KB
constexpr int kIdRingSlots = 4;                                // k tiles of gathered-row numbers kept per loader
constexpr int kXcd = 8;
// waves that request operands: the policy's loader waves, or (kLoaders == 0) its compute waves themselves
template <class P>
constexpr int loading_waves() { return P::kLoaders ? P::kLoaders : P::kCW; }
// LDS of a launch: the two operand rings and, where the numbers of gathered B rows travel through LDS, 1 KB per
// loading wave
template <class P>
constexpr int operand_lds_bytes() { return (P::kSA * P::kTM + P::kSB * kTN) * kTK * 2; }
template <class P>
constexpr int gemm_lds_bytes() {
  return operand_lds_bytes<P>() + (P::kRowIdsInMemory ? loading_waves<P>() * kIdRingSlots * 64 * 4 : 0);
}
// threads of a launch: the policy's compute waves plus its loader waves
template <class P>
constexpr int gemm_threads() { return 64 * (P::kCW + P::kLoaders); }

#define MEFT_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define MEFT_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// Read-only index arrays are read through the constant address space where the index is wave-uniform: that
// makes the load a scalar load, which is counted apart from the vector loads that pace the operand pipeline
// (a vector load would make the compiler wait for every outstanding operand load before using its result).
template <typename T>
__device__ __forceinline__ const __attribute__((address_space(4))) T* as_const(const T* p) {
  return reinterpret_cast<const __attribute__((address_space(4))) T*>(reinterpret_cast<uintptr_t>(p));
}

struct TileCoord {
  int g;       // group (block of neurons); 0 for an ungrouped problem
  int m0, n0;  // first row / column of the tile inside the group's problem
  int Mrows;   // rows of the group's problem
  int Ncols;   // columns of the group's problem
  int nk;      // k tiles
  int slot0;   // first slot of the group in the slot-ordered arrays (token-grouped problems)
  int aux;     // policy-defined
};

// A problem policy P provides:
//   static constexpr int kTM, kSA, kSB;                 tile rows (128 or 192) and the slots of the A and B rings
//   static constexpr int kLoaders;                      loader waves, 2 or 4
//   __device__ bool locate(int wg, TileCoord&) const;   false: no tile with id wg, nor with any larger id on
//                                                       the same XCD (ids wg + 8, wg + 16, ...)
//   static constexpr bool kAMC;                         A contiguous along m (rows indexed by k)?
//       false: __device__ const uint16_t* a_row(const TileCoord&, int m) const;    start of row m (clamped)
//       true:  __device__ const uint16_t* a_mat() const;                 row 0 of the matrix that holds A,
//              __device__ int a_cols(const TileCoord&) const;            its row length (a multiple of 8), and
//              __device__ int a_krow(const TileCoord&, int k) const;     the number of the row that holds contraction
//              index k (possibly negative; a row of zeros beyond the contraction length)
//   static constexpr bool kBNC;                         B contiguous along n (rows indexed by k)?
//       false: __device__ const uint16_t* b_row(const TileCoord&, int n) const;    start of B row n (clamped)
//       true:  __device__ const uint16_t* b_row_ptr(int row) const;   start of B row `row`; rows are
//              TileCoord::Ncols elements apart;  and, with static constexpr bool kRowIdsInMemory (false where B
//              is k-contiguous),
//         false: __device__ int b_row_ids(const TileCoord&, int k) const;  number of the B row that holds k (plain
//                arithmetic, no memory access), any valid row for k beyond the contraction length;
//         true:  __device__ const int32_t* b_row_id_src(const TileCoord&, int k0) const;  where the numbers of the B
//                rows of k0 .. k0 + 63 are stored (valid rows also beyond the contraction length: those products are
//                zero); called for k0 = 0, 64, ... below 64 * nk.  The numbers travel like the operands: a
//                4-byte-per-lane global -> LDS load puts the 64 numbers of a k tile into a small ring in LDS one
//                position ahead of the operand request that uses them;
//   __device__ const uint16_t* a_base() const, b_base() const;   lowest address any load of the operand reads;
//   uint32_t a_bytes, b_bytes;  bool buf;               bytes readable from there, and whether both operands are small
//                                                       enough (< 4 GB) for buffer loads (set by set_gemm_extents)
//   __device__ int out_cols(const TileCoord&) const;    columns of the group's output that are stored
//   __device__ int row_tag(const TileCoord&, int m) const;   0: row m of the group's output is not stored (also for
//                m beyond the group's rows); anything else is handed back to row_off.  May read memory: it is asked
//                before the k loop.
//   __device__ size_t row_off(const TileCoord&, int tag, int m) const;   element offset of (row m, column 0) in
//                the output array
//   static constexpr bool kRowsLinear;   true: row_off does not depend on the tag and is linear in m with the step
//                __device__ int out_ld(const TileCoord&) const;   (the kernel then multiplies once per tile)
//   static constexpr bool kOutBf16;   the output is bf16 (the kernel converts, two columns to a word) or fp32
//       false: __device__ void store2(size_t at, int n, float v0, float v1, uint32_t aux) const;   store C[m][n] = v0
//                and C[m][n + 1] = v1 at element offset `at` (= row_off + n; n even, n < round-up of out_cols to 32;
//                the policy checks n and n + 1 against out_cols where that is not a multiple of 32)
//       true:  __device__ void store_pk(size_t at, int n, uint32_t pk, uint32_t aux) const;   the same with
//                pk = bf16(C[m][n]) | bf16(C[m][n + 1]) << 16
//   static constexpr bool kAux;  true: __device__ uint32_t load_aux(const TileCoord&, int m, int n) const;   a word
//                the policy wants next to the two values of (m, n), e.g. a mask; called for every position of the
//                tile, stored or not, so the policy clamps m and n to valid ones

// Twelve transposing LDS reads of one k16 step (the two m-contiguous A fragments and the four n-contiguous B
// fragments, low and high k half each) followed by the wait for them.  xa = {A0 low, A0 high, A1 low, A1 high}.
// Written as one asm block for the compute waves that also request operands: issued through the builtin, the
// compiler would order these reads after every outstanding global->LDS load (it cannot tell the slots apart),
// which would drain the operand pipeline at every k tile.  The barrier that hands a position over already
// guarantees that the slots read here have landed.
template <int OFFA, int OFFB>
__device__ __forceinline__ void tr_read12(u32x2 (&oa)[4], u32x2 (&ob)[8], const uint32_t (&xa)[4],
                                          const uint32_t (&blo)[4], const uint32_t (&bhi)[4]) {
  asm volatile(
      "ds_read_b64_tr_b16 %0, %12 offset:%24\n\t"
      "ds_read_b64_tr_b16 %1, %13 offset:%24\n\t"
      "ds_read_b64_tr_b16 %2, %14 offset:%24\n\t"
      "ds_read_b64_tr_b16 %3, %15 offset:%24\n\t"
      "ds_read_b64_tr_b16 %4, %16 offset:%25\n\t"
      "ds_read_b64_tr_b16 %5, %17 offset:%25\n\t"
      "ds_read_b64_tr_b16 %6, %18 offset:%25\n\t"
      "ds_read_b64_tr_b16 %7, %19 offset:%25\n\t"
      "ds_read_b64_tr_b16 %8, %20 offset:%25\n\t"
      "ds_read_b64_tr_b16 %9, %21 offset:%25\n\t"
      "ds_read_b64_tr_b16 %10, %22 offset:%25\n\t"
      "ds_read_b64_tr_b16 %11, %23 offset:%25\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(oa[0]), "=&v"(oa[1]), "=&v"(oa[2]), "=&v"(oa[3]), "=&v"(ob[0]), "=&v"(ob[1]), "=&v"(ob[2]),
        "=&v"(ob[3]), "=&v"(ob[4]), "=&v"(ob[5]), "=&v"(ob[6]), "=&v"(ob[7])
      : "v"(xa[0]), "v"(xa[1]), "v"(xa[2]), "v"(xa[3]), "v"(blo[0]), "v"(bhi[0]), "v"(blo[1]), "v"(bhi[1]),
        "v"(blo[2]), "v"(bhi[2]), "v"(blo[3]), "v"(bhi[3]), "n"(OFFA), "n"(OFFB)
      : "memory");
}

// Workgroup barrier of a compute wave: it first waits for its own LDS traffic.  (A loader wave waits for the
// operand loads that have to have landed instead.)
#define MEFT_BARRIER_LDS() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

// P::kCW compute waves (the first waves of the workgroup) and P::kLoaders loader waves (two, or four where the
// loaders' own instruction stream paces the loads: row numbers to look up, an address to form per load; none where
// the compute waves load).  Measured on gfx950 the operand path, not the matrix cores or LDS latency, bounds these
// contractions (a compute unit keeps about a hundred 128-byte read requests in flight on average), and with four
// compute waves a wave that both requests operands and issues MFMAs keeps neither queue full.  The workgroup is persistent: it works through tiles wg, wg + gridDim.x, ...
// (gridDim.x is a multiple of 8, so it stays on one XCD's list).
// kBuf: the operand loads are buffer loads (both operand matrices smaller than 4 GB) instead of global loads
__device__ __forceinline__ uint32_t byte_off(const uint16_t* ptr, const uint16_t* base) {
  return (uint32_t)(reinterpret_cast<uintptr_t>(ptr) - reinterpret_cast<uintptr_t>(base));
}

template <class P, bool kBuf>
__global__ __launch_bounds__(gemm_threads<P>(), 1) void gemm_mfma_kernel(P p, int n_tiles_bound) {
  constexpr int kCW = P::kCW;                       // compute waves: 4 (2 x 2) or 8 (4 x 2)
  constexpr bool kSelf = P::kLoaders == 0;          // the compute waves request the operands themselves
  constexpr int kLoaders = loading_waves<P>();      // waves that request operands
  constexpr int TM = P::kTM, SA = P::kSA, SB = P::kSB;
  constexpr int WM = TM / (kCW / 2);                // rows of a compute wave: 64 or 96
  constexpr int MI = WM / 32;                       // 32-row MFMA tiles per compute wave: 2 or 3
  constexpr int kASlotElems = TM * kTK;
  constexpr int kBRing = SA * kASlotElems;          // element offset of the B ring
  static_assert(kLoaders == 2 || kLoaders == 4 || kLoaders == 8, "waves that load: 2, 4 or 8");
  static_assert((kCW == 4 && (TM == 128 || TM == 192)) || (kCW == 8 && TM == 256), "tile rows: 128, 192 or 256");
  static_assert(SA >= 2 && SA <= 3 && SB >= 2 && SB <= 3, "ring depths: 2 or 3");
  static_assert(!P::kAMC || TM == 128 || TM == 256, "the m-contiguous A layouts are written for 128 and 256 rows");
  static_assert(!kSelf || (P::kAMC && P::kBNC && SA == 2 && SB == 2 && kCW == 8),
                "compute waves that load: written for the neuron-major problems with two slots per ring");
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // locate() answers false only when the workgroup's XCD has no tile with this or any larger id
  auto next_tile = [&](int wg, TileCoord& t) -> bool { return wg < n_tiles_bound && p.locate(wg, t); };
  const int step = gridDim.x;

  TileCoord tc;
  if (!next_tile(blockIdx.x, tc)) return;   // the same answer in every wave

  // ---------------------------------------------------------------------- operand requests
  // (state and steps of a wave that loads: a loader wave, or with kSelf every compute wave; dead code in the compute
  // waves of a launch with loader waves)
    const int lw = kSelf ? wave : wave - kCW;
    constexpr int LA = TM / 8 / kLoaders;    // A wave-loads (1 KB each) per loader and slot: 12, 8, 6 or 4
    constexpr int LB = kTN / 8 / kLoaders;   // B wave-loads (1 KB each) per loader and slot: 16 or 8
    constexpr int DA = SA - 1, DB = SB - 1;  // positions ahead of the barrier at which A and B are requested
    constexpr int kAhead = (DA - 1) * LA + (DB - 1) * LB;   // loads that may still be in flight at a barrier
    static_assert(kAhead <= 63, "partial vmcnt wait out of range");
    const int lr8 = lane >> 3;
    int* idring = reinterpret_cast<int*>(smem + operand_lds_bytes<P>() / 2) + lw * kIdRingSlots * 64;

    // Cursors over one and the same sequence of (tile, k tile) positions: the operand A, the operand B, and (where
    // they sit in memory) the row numbers of gathered B rows, which run one position ahead of B.
    struct Cursor {
      int wg, k, n, slot;
      bool ok;
      TileCoord t;
    };
    Cursor ca{(int)blockIdx.x, 0, 0, 0, true, tc}, cb = ca, cd = ca;
    cd.ok = P::kBNC && P::kRowIdsInMemory;
    //   consume: position handed to the compute waves at the next barrier
    int wg_c = blockIdx.x, nk_c = tc.nk;

    // A, k-contiguous: a wave-load covers 8 rows (m) x 128 bytes; fixed row pointers per tile, advanced by k.
    // A, m-contiguous, 128 rows: a wave-load covers 4 rows (k) x 256 bytes; lane l fetches the 16-byte chunk
    //   (l & 15) ^ (4 * (row & 3)) of its row (the LDS swizzle; row & 3 == (l >> 4) & 3 for every load), so one
    //   column offset per tile serves all the loads.  With 256 rows the slot has the shape of an n-contiguous B slot
    //   and is filled the same way.
    // B, k-contiguous: like A, 8 rows (n) x 128 bytes.
    // B, n-contiguous: a wave-load covers two k rows (lanes 0..31 the even one, lanes 32..63 the odd one), 512 bytes
    //   of each; lane l fetches the chunk (l & 31) ^ (2 * (row & 7)); row & 7 only depends on i & 3, so four
    //   column offsets per tile cover all the loads.
    //
    // Every wave-load fills 1 KB of LDS, and the loads of a loader fill consecutive kilobytes.  The instruction's
    // immediate offset is added to the global AND the LDS address (checked on the device), so four consecutive loads
    // share one LDS base (one write of M0 instead of four) with offsets 0, 1, 2, 3 KB, and the global pointers are
    // set up that many bytes lower.
    const uint16_t* pa[P::kAMC ? 4 : LA];   // m-contiguous: row 0 at this lane's column, one per offset 0..3 KB
    const uint16_t* pb[P::kBNC ? 4 : LB];
    // Buffer loads (kBuf): the same addresses as 32-bit byte offsets from the operand's lowest address, without the
    // kilobyte shifts (every load writes M0, a scalar instruction).  Whatever is the same in all lanes goes into the
    // instruction's scalar offset: the k offset of k-contiguous operands, the row offset of consecutive B rows.
    [[maybe_unused]] uint32_t oa[P::kAMC ? 4 : LA], ob[P::kBNC ? 4 : LB];
    const int half = lane >> 5;
    auto setup_a = [&]() {
      const TileCoord& t = ca.t;
      if constexpr (kBuf) {
        if constexpr (P::kAMC && TM == 256) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int chunk = (lane & 31) ^ (2 * ((2 * q + half) & 7));
            const int col = t.m0 + chunk * 8, last = p.a_cols(t) - 8;
            oa[q] = byte_off(p.a_mat() + (col > last ? last : col), p.a_base());
          }
        } else if constexpr (P::kAMC) {
          const int chunk = (lane & 15) ^ (4 * ((lane >> 4) & 3));
          const int col = t.m0 + chunk * 8, last = p.a_cols(t) - 8;
          const uint32_t o = byte_off(p.a_mat() + (col > last ? last : col), p.a_base());
#pragma unroll
          for (int q = 0; q < 4; ++q) oa[q] = o;
        } else {
#pragma unroll
          for (int i = 0; i < LA; ++i) {
            const int row = (lw * LA + i) * 8 + lr8;
            oa[i] = byte_off(p.a_row(t, t.m0 + row) + (((lane & 7) ^ ((row >> 1) & 7)) << 3), p.a_base());
          }
        }
      } else {
        if constexpr (P::kAMC && TM == 256) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int chunk = (lane & 31) ^ (2 * ((2 * q + half) & 7));
            const int col = t.m0 + chunk * 8, last = p.a_cols(t) - 8;
            pa[q] = p.a_mat() + ((col > last ? last : col) - q * 512);   // clamp (rows beyond Mrows are never stored)
          }
        } else if constexpr (P::kAMC) {
          const int chunk = (lane & 15) ^ (4 * ((lane >> 4) & 3));
          const int col = t.m0 + chunk * 8, last = p.a_cols(t) - 8;
          const int acol = col > last ? last : col;                       // clamp (rows beyond Mrows are never stored)
#pragma unroll
          for (int q = 0; q < 4; ++q) pa[q] = p.a_mat() + (acol - q * 512);
        } else {
#pragma unroll
          for (int i = 0; i < LA; ++i) {
            const int row = (lw * LA + i) * 8 + lr8;
            pa[i] = p.a_row(t, t.m0 + row) + (((lane & 7) ^ ((row >> 1) & 7)) << 3) - (i & 3) * 512;
          }
        }
      }
    };
    auto setup_b = [&]() {
      const TileCoord& t = cb.t;
      if constexpr (kBuf) {
        if constexpr (P::kBNC) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int chunk = (lane & 31) ^ (2 * ((2 * q + half) & 7));
            int col = t.n0 + chunk * 8;
            col = col > t.Ncols - 8 ? t.Ncols - 8 : col;
            ob[q] = byte_off(p.b_row_ptr(0) + col, p.b_base());
          }
        } else {
#pragma unroll
          for (int i = 0; i < LB; ++i) {
            const int row = (lw * LB + i) * 8 + lr8;
            ob[i] = byte_off(p.b_row(t, t.n0 + row) + (((lane & 7) ^ ((row >> 1) & 7)) << 3), p.b_base());
          }
        }
      } else {
        if constexpr (P::kBNC) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int chunk = (lane & 31) ^ (2 * ((2 * q + half) & 7));
            int col = t.n0 + chunk * 8;
            col = col > t.Ncols - 8 ? t.Ncols - 8 : col;              // clamp (columns beyond Ncols are never stored)
            pb[q] = p.b_row_ptr(0) + col - q * 512;
          }
        } else {
#pragma unroll
          for (int i = 0; i < LB; ++i) {
            const int row = (lw * LB + i) * 8 + lr8;
            pb[i] = p.b_row(t, t.n0 + row) + (((lane & 7) ^ ((row >> 1) & 7)) << 3) - (i & 3) * 512;
          }
        }
      }
    };
    // Where every operand matrix is smaller than 4 GB the loads are buffer loads (a wave-uniform resource descriptor,
    // a 32-bit offset per lane and a scalar offset instead of a 64-bit address per lane): the vector-memory path
    // takes them faster (score GEMM 0.331 -> 0.314 ms), and a load of the k-contiguous problems then costs the
    // loader a write of M0 and nothing else.
    __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.a_base()), 0, (int)p.a_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.b_base()), 0, (int)p.b_bytes, 0x00020000);
    // load number i of a loader into the 1 KB slot i of its part of an operand region (see above)
    // (the offset has to be a literal: the switch folds away once the loop over i is unrolled)
#define MEFT_LOAD_1K(src, region, i)                                                    \
  do {                                                                                  \
    const auto* g_ = MEFT_GPTR(src);                                                    \
    auto* l_ = MEFT_LPTR((region) + ((i) & ~3) * 512);                                  \
    switch ((i) & 3) {                                                                  \
      case 0: __builtin_amdgcn_global_load_lds(g_, l_, 16, 0, 0); break;                \
      case 1: __builtin_amdgcn_global_load_lds(g_, l_, 16, 1024, 0); break;             \
      case 2: __builtin_amdgcn_global_load_lds(g_, l_, 16, 2048, 0); break;             \
      default: __builtin_amdgcn_global_load_lds(g_, l_, 16, 3072, 0); break;            \
    }                                                                                   \
  } while (0)
    // buffer load number i: lane offset `voff`, wave-uniform offset `soff` (bytes).  The casts are needed: handed an
    // unsigned offset, this toolchain's host pass drops the kernel's launch stub without any diagnostic and the
    // library then fails to load with an undefined symbol.
#define MEFT_LOAD_1K_BUF(rsrc, voff, soff, region, i) \
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, MEFT_LPTR((region) + (i) * 512), 16, (int)(voff), (int)(soff), 0, 0)

    auto request_ids = [&]() {
      if constexpr (P::kBNC && P::kRowIdsInMemory) {
        if (!cd.ok) return;
        __builtin_amdgcn_global_load_lds(MEFT_GPTR(p.b_row_id_src(cd.t, cd.k * kTK) + lane),
                                         MEFT_LPTR(idring + (cd.n & (kIdRingSlots - 1)) * 64), 4, 0, 0);
        ++cd.n;
        if (++cd.k == cd.t.nk) { cd.wg += step; cd.k = 0; cd.ok = next_tile(cd.wg, cd.t); }
      }
    };
    // one k tile of A into the next slot of the A ring; false: the stream has ended, nothing was requested
    auto request_a = [&]() -> bool {
      if (!ca.ok) return false;
      const TileCoord& t = ca.t;
      uint16_t* my_a = smem + ca.slot * kASlotElems + lw * LA * 512;   // 512 elements = 1 KB per load
      [[maybe_unused]] int a_row_bytes = 0;
      if constexpr (P::kAMC) a_row_bytes = p.a_cols(t) * 2;
      if constexpr (kBuf) {
        const int k_bytes = ca.k * kTK * 2;
#pragma unroll
        for (int i = 0; i < LA; ++i) {
          if constexpr (P::kAMC) {
            const int row = p.a_krow(t, ca.k * kTK + (TM == 256 ? 2 * (lw * LA + i) + half : 4 * (lw * LA + i) + (lane >> 4)));
            MEFT_LOAD_1K_BUF(rsrc_a, oa[i & 3] + (uint32_t)row * (uint32_t)a_row_bytes, 0, my_a, i);
          } else {
            MEFT_LOAD_1K_BUF(rsrc_a, oa[i], k_bytes, my_a, i);
          }
        }
      } else {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
          if constexpr (P::kAMC) {
            const int row = p.a_krow(t, ca.k * kTK + (TM == 256 ? 2 * (lw * LA + i) + half : 4 * (lw * LA + i) + (lane >> 4)));
            MEFT_LOAD_1K(reinterpret_cast<const char*>(pa[i & 3]) + (int64_t)row * a_row_bytes, my_a, i);
          } else {
            MEFT_LOAD_1K(pa[i] + ca.k * kTK, my_a, i);
          }
        }
      }
      ++ca.n;
      ca.slot = ca.slot + 1 == SA ? 0 : ca.slot + 1;
      if (++ca.k == t.nk) {
        ca.wg += step; ca.k = 0; ca.ok = next_tile(ca.wg, ca.t);
        if (ca.ok) setup_a();
      }
      return true;
    };
    // one k tile of B into the next slot of the B ring
    auto request_b = [&]() -> bool {
      if (!cb.ok) return false;
      const TileCoord& t = cb.t;
      // n-contiguous B: ids[i] = number of the B row this lane fetches in its i-th load,
      // k = 64 * cb.k + 2 * (lw * LB + i) + half
      int ids[LB];
      if constexpr (P::kBNC && P::kRowIdsInMemory) {
        // out of the ring; one asm block with its own wait (through plain loads the compiler would first drain every
        // outstanding operand load)
        const uint32_t a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(
            idring + (cb.n & (kIdRingSlots - 1)) * 64 + 2 * lw * LB + half);
        if constexpr (LB == 16) {
        asm volatile(
            "ds_read_b32 %0, %16\n\tds_read_b32 %1, %16 offset:8\n\tds_read_b32 %2, %16 offset:16\n\t"
            "ds_read_b32 %3, %16 offset:24\n\tds_read_b32 %4, %16 offset:32\n\tds_read_b32 %5, %16 offset:40\n\t"
            "ds_read_b32 %6, %16 offset:48\n\tds_read_b32 %7, %16 offset:56\n\tds_read_b32 %8, %16 offset:64\n\t"
            "ds_read_b32 %9, %16 offset:72\n\tds_read_b32 %10, %16 offset:80\n\tds_read_b32 %11, %16 offset:88\n\t"
            "ds_read_b32 %12, %16 offset:96\n\tds_read_b32 %13, %16 offset:104\n\tds_read_b32 %14, %16 offset:112\n\t"
            "ds_read_b32 %15, %16 offset:120\n\ts_waitcnt lgkmcnt(0)"
            : "=&v"(ids[0]), "=&v"(ids[1]), "=&v"(ids[2]), "=&v"(ids[3]), "=&v"(ids[4]), "=&v"(ids[5]), "=&v"(ids[6]),
              "=&v"(ids[7]), "=&v"(ids[8]), "=&v"(ids[9]), "=&v"(ids[10]), "=&v"(ids[11]), "=&v"(ids[12]),
              "=&v"(ids[13]), "=&v"(ids[14]), "=&v"(ids[15])
            : "v"(a)
            : "memory");
        } else if constexpr (LB == 4) {
        asm volatile(
            "ds_read_b32 %0, %4\n\tds_read_b32 %1, %4 offset:8\n\tds_read_b32 %2, %4 offset:16\n\t"
            "ds_read_b32 %3, %4 offset:24\n\ts_waitcnt lgkmcnt(0)"
            : "=&v"(ids[0]), "=&v"(ids[1]), "=&v"(ids[2]), "=&v"(ids[3])
            : "v"(a)
            : "memory");
        } else {
        static_assert(LB == 16 || LB == 8 || LB == 4, "row-number reads are written out for 16, 8 and 4 loads");
        asm volatile(
            "ds_read_b32 %0, %8\n\tds_read_b32 %1, %8 offset:8\n\tds_read_b32 %2, %8 offset:16\n\t"
            "ds_read_b32 %3, %8 offset:24\n\tds_read_b32 %4, %8 offset:32\n\tds_read_b32 %5, %8 offset:40\n\t"
            "ds_read_b32 %6, %8 offset:48\n\tds_read_b32 %7, %8 offset:56\n\ts_waitcnt lgkmcnt(0)"
            : "=&v"(ids[0]), "=&v"(ids[1]), "=&v"(ids[2]), "=&v"(ids[3]), "=&v"(ids[4]), "=&v"(ids[5]), "=&v"(ids[6]),
              "=&v"(ids[7])
            : "v"(a)
            : "memory");
        }
      } else if constexpr (P::kBNC) {
#pragma unroll
        for (int i = 0; i < LB; ++i) ids[i] = p.b_row_ids(t, cb.k * kTK + 2 * (lw * LB + i) + half);
      }
      uint16_t* my_b = smem + kBRing + cb.slot * kBSlotElems + lw * LB * 512;
      if constexpr (kBuf) {
        const int k_bytes = cb.k * kTK * 2;
        if constexpr (P::kBNC) {
          const uint32_t row_bytes = (uint32_t)t.Ncols * 2u;
          bool linear = false;
          if constexpr (!P::kRowIdsInMemory) {
            linear = p.b_rows_linear(t, cb.k * kTK);
            if (linear) {
              // 64 consecutive rows: this lane's row is first + 2 * (lw * LB + i) + half
              const uint32_t first = (uint32_t)p.b_row_ids(t, cb.k * kTK) * row_bytes, hoff = half * row_bytes;
#pragma unroll
              for (int i = 0; i < LB; ++i)
                MEFT_LOAD_1K_BUF(rsrc_b, ob[i & 3] + hoff, (int)(first + 2u * (lw * LB + i) * row_bytes), my_b, i);
            }
          }
          if (!linear) {
#pragma unroll
            for (int i = 0; i < LB; ++i)
              MEFT_LOAD_1K_BUF(rsrc_b, ob[i & 3] + (uint32_t)ids[i] * row_bytes, 0, my_b, i);
          }
        } else {
#pragma unroll
          for (int i = 0; i < LB; ++i) MEFT_LOAD_1K_BUF(rsrc_b, ob[i], k_bytes, my_b, i);
        }
      } else {
        if constexpr (P::kBNC) {
          const uint32_t row_bytes = (uint32_t)t.Ncols * 2u;
#pragma unroll
          for (int i = 0; i < LB; ++i)
            MEFT_LOAD_1K(reinterpret_cast<const char*>(pb[i & 3]) + (uint64_t)(uint32_t)ids[i] * row_bytes, my_b, i);
        } else {
#pragma unroll
          for (int i = 0; i < LB; ++i) MEFT_LOAD_1K(pb[i] + cb.k * kTK, my_b, i);
        }
      }
      ++cb.n;
      cb.slot = cb.slot + 1 == SB ? 0 : cb.slot + 1;
      if (++cb.k == t.nk) {
        cb.wg += step; cb.k = 0; cb.ok = next_tile(cb.wg, cb.t);
        if (cb.ok) setup_b();
      }
      return true;
    };
    // the requests that follow a barrier: one k tile of each operand, the one with the shorter lead first, so that
    // the loads which may still be in flight at the next barrier are the most recent ones.  true: both were made.
    auto request_batch = [&]() -> bool {
      request_ids();
      bool a, b;
      if constexpr (DA <= DB) { a = request_a(); b = request_b(); }
      else { b = request_b(); a = request_a(); }
      return a && b;
    };

  if (kSelf || wave >= kCW) {
    setup_a();
    setup_b();
    if constexpr (P::kBNC && P::kRowIdsInMemory) {
#pragma unroll
      for (int s = 0; s < DB + 1; ++s) request_ids();
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    // before the first barrier: position 0 of both operands first, then the positions the leads reach
    bool full = request_a();
    full = request_b() && full;
#pragma unroll
    for (int s = 1; s < DA; ++s) full = request_a() && full;
#pragma unroll
    for (int s = 1; s < DB; ++s) full = request_b() && full;
    // compute waves that load: position 0 has to have landed at the first barrier (later positions are awaited
    // before the barrier that hands them over)
    if constexpr (kSelf) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ------------------------------------------------------------------ loader waves
    for (; !kSelf;) {
      for (int kt = 0; kt < nk_c; ++kt) {
        // The position handed over now has landed once at most the kAhead most recent loads are outstanding (the
        // counter retires in issue order), provided the last batch of requests was complete; near the end of the
        // stream everything is awaited.
        if (full) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(kAhead) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        // every compute wave is past the previous position: its slots are free
        full = request_batch();
      }
      wg_c += step;
      TileCoord t;
      if (!next_tile(wg_c, t)) return;
      nk_c = t.nk;
    }
  }

  // -------------------------------------------------------------------- compute waves
  const int wm = (wave >> 1) * WM, wn = (wave & 1) * 128;
  const int fr = lane & 31, fc = lane >> 5;
  // k-contiguous operands: element offsets of this lane's fragment rows inside a slot, and their swizzle keys
  int offA[MI], keyA[MI], offB[4], keyB[4];
#pragma unroll
  for (int i = 0; i < MI; ++i) { const int r = wm + i * 32 + fr; offA[i] = r * kTK; keyA[i] = (r >> 1) & 7; }
#pragma unroll
  for (int j = 0; j < 4; ++j) { const int r = wn + j * 32 + fr; offB[j] = r * kTK; keyB[j] = (r >> 1) & 7; }
  // m- / n-contiguous operands: LDS byte offsets (inside a slot) of this lane's transposing reads.  Lane s of a
  // 16-lane group points at row (k base + s/4), columns 4*(s%4)..+3 of a 4 x 16 block and receives column s of that
  // block, four consecutive k.  Low half: k = 8*(lane/32) + 0..3, high half +4.
  uint32_t tra_lo[2], tra_hi[2], tr_lo[4], tr_hi[4];
  {
    const int gq = lane >> 4, s = lane & 15;
    const int k_lo = 8 * (gq >> 1) + (s >> 2), k_hi = k_lo + 4;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int m = wm + i * 32 + 16 * (gq & 1) + 4 * (s & 3);
      const int x_lo = TM == 256 ? 2 * (k_lo & 7) : 4 * (k_lo & 3), x_hi = TM == 256 ? 2 * (k_hi & 7) : 4 * (k_hi & 3);
      tra_lo[i] = (uint32_t)(k_lo * TM + (((m >> 3) ^ x_lo) << 3) + (m & 7)) * 2u;
      tra_hi[i] = (uint32_t)(k_hi * TM + (((m >> 3) ^ x_hi) << 3) + (m & 7)) * 2u;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = wn + j * 32 + 16 * (gq & 1) + 4 * (s & 3);
      tr_lo[j] = (uint32_t)(k_lo * kTN + (((n >> 3) ^ (2 * (k_lo & 7))) << 3) + (n & 7)) * 2u;
      tr_hi[j] = (uint32_t)(k_hi * kTN + (((n >> 3) ^ (2 * (k_hi & 7))) << 3) + (n & 7)) * 2u;
    }
  }

  int wg = blockIdx.x;
  int slot_a = 0, slot_b = 0;   // run on across tiles, like the loaders' slots
  for (;;) {
    // lane l: the tag of row wm + l of this tile (and, with 96 rows per wave, lane l < 32: of row wm + 64 + l).
    // Asked before the k loop, so that a policy's memory read has long returned when the answer is needed.
    const int my_tag = p.row_tag(tc, tc.m0 + wm + lane);
    [[maybe_unused]] int my_tag_hi = 0;
    if constexpr (WM > 64) my_tag_hi = lane < WM - 64 ? p.row_tag(tc, tc.m0 + wm + 64 + lane) : 0;

    f32x16 acc[MI][4];
    const int nk = tc.nk;
    bool more = false;
    TileCoord tn;
    // The fragments of one k16 step.  Two sets alternate: the LDS reads of step s + 1 are issued before the matrix
    // instructions of step s, so that their latency passes under those 8 (12) instructions instead of in front of
    // the next ones.  (Left to itself the compiler reads each step's fragments into the same registers right before
    // their use, and the matrix pipe idles for an LDS round trip four times per k tile.)
    struct Frags { bf16x8 a[MI], b[4]; };
    Frags f0, f1;
    constexpr uint32_t kStepA = 16 * TM * 2;   // bytes of 16 k rows of an m-contiguous A slot
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    // transposing read of this lane's 8 values of one operand fragment: low and high k half, 8 bytes each
    auto tr_pair = [&](const uint16_t* slot, uint32_t lo_off, uint32_t hi_off) -> bf16x8 {
      const auto* base = (const __attribute__((address_space(3))) char*)(slot);
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(base + lo_off));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(base + hi_off));
      return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // issue the LDS reads of k16 step KS of the current slots
    auto load_frags = [&](auto ks_tag, Frags& f) {
      constexpr int ks = decltype(ks_tag)::value;
      const uint16_t* sta = smem + slot_a * kASlotElems;
      const uint16_t* stb = smem + kBRing + slot_b * kBSlotElems;
      const int c = ks * 2 + fc;   // k-contiguous operands: this lane's 16-byte chunk of the k16 step
      // k16 step ks starts 16 rows further (B: 8192 bytes, m-contiguous A: 4096 or 8192 bytes); that changes neither
      // (k & 7) nor (k & 3), so the swizzles hold
      if constexpr (!P::kAMC) {
#pragma unroll
        for (int i = 0; i < MI; ++i) f.a[i] = *reinterpret_cast<const bf16x8*>(&sta[offA[i] + ((c ^ keyA[i]) << 3)]);
      } else {
        static_assert(!P::kAMC || P::kBNC, "an m-contiguous A comes with an n-contiguous B");
#pragma unroll
        for (int i = 0; i < 2; ++i) f.a[i] = tr_pair(sta, tra_lo[i] + ks * kStepA, tra_hi[i] + ks * kStepA);
      }
      if constexpr (!P::kBNC) {
#pragma unroll
        for (int j = 0; j < 4; ++j) f.b[j] = *reinterpret_cast<const bf16x8*>(&stb[offB[j] + ((c ^ keyB[j]) << 3)]);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) f.b[j] = tr_pair(stb, tr_lo[j] + ks * 8192u, tr_hi[j] + ks * 8192u);
      }
    };
    // kZero: the step starts from zero instead of from acc (the matrix instruction takes the constant as its addend,
    // so the accumulators are never cleared by hand)
    auto mma = [&](auto zero_tag, const Frags& f) {
      constexpr bool kZero = decltype(zero_tag)::value;
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if constexpr (kZero) {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], zero, 0, 0, 0);
          } else {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
          }
        }
    };
    // nothing moves across: the order of reads and matrix instructions below is the schedule
#define MEFT_FENCE() __builtin_amdgcn_sched_barrier(0)
    // Steps 0..2 of a k tile whose first fragments (f0) are on their way; its step 3 (f1) is left to the caller.
    auto k_steps = [&](auto first_tag) {
      load_frags(std::integral_constant<int, 1>{}, f1);
      MEFT_FENCE();
      mma(first_tag, f0);
      MEFT_FENCE();
      load_frags(std::integral_constant<int, 2>{}, f0);
      MEFT_FENCE();
      mma(std::false_type{}, f1);
      MEFT_FENCE();
      load_frags(std::integral_constant<int, 3>{}, f1);
      MEFT_FENCE();
      mma(std::false_type{}, f0);
      MEFT_FENCE();
      slot_a = slot_a + 1 == SA ? 0 : slot_a + 1;
      slot_b = slot_b + 1 == SB ? 0 : slot_b + 1;
    };
    if constexpr (kSelf) {
      // Compute waves that load.  The compiler orders every LDS read it knows of behind all outstanding global -> LDS
      // loads (it cannot tell the slots apart), which would undo the prefetch, so here the fragments are read by asm
      // blocks that wait for themselves; with two compute waves per SIMD the other wave's matrix instructions cover
      // that wait.  A position's operands are requested right after the barrier that hands over the position before
      // it, and awaited (vmcnt) right before the barrier that hands it over; the first position of a tile is awaited
      // before the previous tile's stores, so that no barrier waits for stores.
      auto k_tile_self = [&](auto first_tag) {
        const uint16_t* sta = smem + slot_a * kASlotElems;
        const uint16_t* stb = smem + kBRing + slot_b * kBSlotElems;
        const uint32_t abase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(sta);
        const uint32_t sbase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(stb);
        const uint32_t xa[4] = {abase + tra_lo[0], abase + tra_hi[0], abase + tra_lo[1], abase + tra_hi[1]};
        uint32_t alo[4], ahi[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { alo[j] = sbase + tr_lo[j]; ahi[j] = sbase + tr_hi[j]; }
        auto step16 = [&](auto ks_tag, auto zero_tag) {
          constexpr int ks = decltype(ks_tag)::value;
          u32x2 oa[4], o[8];
          tr_read12<ks * (int)kStepA, ks * 8192>(oa, o, xa, alo, ahi);
          Frags f;
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const u32x4 w = {oa[2 * i].x, oa[2 * i].y, oa[2 * i + 1].x, oa[2 * i + 1].y};
            f.a[i] = __builtin_bit_cast(bf16x8, w);
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const u32x4 w = {o[2 * j].x, o[2 * j].y, o[2 * j + 1].x, o[2 * j + 1].y};
            f.b[j] = __builtin_bit_cast(bf16x8, w);
          }
          mma(zero_tag, f);
        };
        step16(std::integral_constant<int, 0>{}, first_tag);
        step16(std::integral_constant<int, 1>{}, std::false_type{});
        step16(std::integral_constant<int, 2>{}, std::false_type{});
        step16(std::integral_constant<int, 3>{}, std::false_type{});
        slot_a = slot_a + 1 == SA ? 0 : slot_a + 1;
        slot_b = slot_b + 1 == SB ? 0 : slot_b + 1;
      };
      MEFT_BARRIER_LDS();   // (the tile's first position was awaited before: see above)
      request_batch();
      wg += step;
      more = next_tile(wg, tn);
      k_tile_self(std::true_type{});
      for (int kt = 1; kt < nk; ++kt) {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        request_batch();
        k_tile_self(std::false_type{});
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
    MEFT_BARRIER_LDS();   // the loaders have seen the tile's first k tile land
    wg += step;
    more = next_tile(wg, tn);
    load_frags(std::integral_constant<int, 0>{}, f0);
    MEFT_FENCE();
    k_steps(std::true_type{});
    for (int kt = 1; kt < nk; ++kt) {
      // The barrier for k tile kt sits in front of the last matrix instructions of k tile kt - 1: every LDS read of
      // that position has returned (the barrier macro waits for them), so the loaders may have its slots, and the
      // first reads of the new position pass under those instructions.
      MEFT_BARRIER_LDS();
      load_frags(std::integral_constant<int, 0>{}, f0);
      MEFT_FENCE();
      mma(std::false_type{}, f1);
      MEFT_FENCE();
      k_steps(std::false_type{});
    }
    mma(std::false_type{}, f1);
    }
#undef MEFT_FENCE

    // ---- epilogue, out of the registers.  acc[i][j][r] is C[m][n] with m = wm + i*32 + (r/4)*8 + (lane/32)*4 + r%4
    // and n = wn + j*32 + lane%32.  For a register pair (r, r+1), r even, an even lane (column c) keeps its value of
    // row m and takes its right neighbour's value of that row; the odd lane (column c+1) keeps its value of row m+1
    // and takes its left neighbour's (DPP quad_perm [1,0,3,2] swaps neighbours).  Both then hold columns (c, c+1) of
    // one row.  Per 32 rows of the accumulators (i), four register pairs at a time, the rows' tags and whatever the
    // policy reads per element (load_aux: unconditional loads, all in flight together) are fetched first, then the
    // values are exchanged and stored.
    {
      const bool odd = (lane & 1) != 0;
      const int nj = (p.out_cols(tc) - (tc.n0 + wn) + 31) / 32;   // 32-column fragments of this wave with stored columns
      const int ncol = tc.n0 + wn + (fr & ~1);
      // row of this lane inside the wave's rows = lane_row + a constant of the register pair
      const int lane_row = fc * 4 + (lane & 1);
      [[maybe_unused]] size_t lane_at = 0;
      [[maybe_unused]] int ld = 0;
      if constexpr (P::kRowsLinear) {
        ld = p.out_ld(tc);
        lane_at = p.row_off(tc, 1, tc.m0 + wm + lane_row) + ncol;   // one multiplication per tile
      }
      [[maybe_unused]] const unsigned long long ok_mask = __ballot(my_tag != 0);
      [[maybe_unused]] const unsigned long long ok_mask_hi = __ballot(my_tag_hi != 0);
      auto epilogue = [&](auto full_tag) {
        constexpr bool kFull = decltype(full_tag)::value;   // all four fragments of the wave lie inside the output
#pragma unroll
        for (int i = 0; i < MI; ++i) {
#pragma unroll
          for (int qh = 0; qh < 2; ++qh) {
            int tag[4];
            uint32_t aux[4][4];
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
              const int r = 2 * (qh * 4 + qq);
              const int rl = i * 32 + (r >> 2) * 8 + (r & 3) + lane_row;
              // the row's tag: a bit of the wave's ballot where it only says "stored or not" (no trip through the LDS
              // pipeline, which the loaders keep busy), a lane permute where it carries a number
              if constexpr (P::kRowsLinear) {
                tag[qq] = i < 2 ? (int)((ok_mask >> rl) & 1ull) : (int)((ok_mask_hi >> (rl - 64)) & 1ull);
              } else {
                tag[qq] = i < 2 ? __builtin_amdgcn_ds_bpermute(rl << 2, my_tag)
                                : __builtin_amdgcn_ds_bpermute((rl - 64) << 2, my_tag_hi);
              }
              if constexpr (P::kAux) {
#pragma unroll
                for (int j = 0; j < 4; ++j) aux[qq][j] = p.load_aux(tc, tc.m0 + wm + rl, ncol + 32 * j);
              } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) aux[qq][j] = 0u;
              }
            }
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
              const int r = 2 * (qh * 4 + qq);
              const int rc = i * 32 + (r >> 2) * 8 + (r & 3);   // the register pair's constant part of the row
              [[maybe_unused]] uint32_t pk[4];
              [[maybe_unused]] float lo[4], hi[4];
              if constexpr (P::kOutBf16) {
                // bf16 output: both rows' values of this lane's column are packed first, (row m | row m+1 << 16); one
                // neighbour swap of the packed word and one byte permute give (column c | column c+1 << 16) of the
                // lane's row (even lanes: row m from the low halves, odd lanes: row m+1 from the high halves)
                const uint32_t sel = odd ? 0x03020706u : 0x05040100u;   // bytes 0-3: own word, 4-7: the neighbour's
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                  const uint32_t own = pack_bf16x2(acc[i][j][r], acc[i][j][r + 1]);
                  const uint32_t nb = (uint32_t)__builtin_amdgcn_update_dpp((int)own, (int)own, 0xB1, 0xF, 0xF, true);
                  pk[j] = __builtin_amdgcn_perm(nb, own, sel);
                }
              } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                  const float a = acc[i][j][r], b = acc[i][j][r + 1];   // plain copies: the values go to the builtin as floats
                  const float an = __builtin_amdgcn_update_dpp(a, a, 0xB1, 0xF, 0xF, true);   // the neighbour's a
                  const float bn = __builtin_amdgcn_update_dpp(b, b, 0xB1, 0xF, 0xF, true);   // the neighbour's b
                  lo[j] = odd ? bn : a;
                  hi[j] = odd ? b : an;
                }
              }
              if (tag[qq] != 0) {
                size_t at;
                if constexpr (P::kRowsLinear) at = lane_at + (size_t)(rc * ld);   // rc * ld: scalar arithmetic
                else at = p.row_off(tc, tag[qq], tc.m0 + wm + rc + lane_row) + ncol;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                  if (kFull || j < nj) {
                    if constexpr (P::kOutBf16) p.store_pk(at + 32 * j, ncol + 32 * j, pk[j], aux[qq][j]);
                    else p.store2(at + 32 * j, ncol + 32 * j, lo[j], hi[j], aux[qq][j]);
                  }
                }
              }
            }
          }
        }
      };
      if (nj >= 4) epilogue(std::true_type{});
      else epilogue(std::false_type{});
    }
    if (!more) break;
    tc = tn;
  }
}

// ---- tile schedule shared by the grouped problems ----------------------------------------------
// Every non-empty group (block of neurons with its tokens) is given to one XCD; XCD x works through its list
// in order.  grp[x][i] = (group, number of m tiles -- of tile_m rows -- of the groups before it in this list); an end entry
// (-1, total m tiles) closes the list.  Inside a group the m tiles vary fastest, so that the tiles that share a
// B panel (one n tile of the group's block) run at the same time and the panel is read from HBM once.
//
// Groups differ in size (the router does not balance them), so they are dealt out longest first, each to the
// XCD with the least work so far (ties to the lower XCD); the work of a group is counted in 64-row units plus
// a constant for the per-tile overhead, which balances both the token-major tile counts and the contraction
// lengths of the neuron-major problems.  Which XCD computes a group has no influence on any result.
//
// Groups of at most `small_rows` tokens come last in every list (the deal runs from the longest group down), and a
// second set of list lengths counts only the larger groups in front of them: a problem that leaves the small groups
// to the per-pair kernels (small_groups.h) walks that prefix of the same lists.
struct TokenSched {
  const int2* grp;       // [kXcd][cap]
  const int* len;        // [kXcd] number of groups in the list; [kXcd]: 1 = every list holds every group (split);
                         // [kXcd + 1 + x]: groups of more than small_rows tokens in XCD x's list (a prefix of it)
  int cap;               // entries per XCD (n_groups + 1)
  int max_tiles;         // upper bound of m tiles of one XCD (for the tile-id bound of a launch)
};
constexpr int kSchedLenInts = 2 * kXcd + 1;

constexpr int kSchedSortMax = 1024;   // up to this many groups are dealt out longest first; more: round-robin

// Executed by one whole workgroup of 1024 threads.
__device__ __forceinline__ void build_sched_body(const int32_t* __restrict__ group_off, int n_groups, int cap,
                                                 int2* __restrict__ grp, int* __restrict__ len, int tile_m,
                                                 int small_rows) {
  __shared__ int s_rows[kSchedSortMax];
  __shared__ int s_order[kSchedSortMax];
  __shared__ int s_sorted[kSchedSortMax];
  const int tid = threadIdx.x;
  if (n_groups <= kSchedSortMax) {
    int rows = 0;
    if (tid < n_groups) { rows = group_off[tid + 1] - group_off[tid]; s_rows[tid] = rows; }
    const int n_full = __syncthreads_count(rows > 0);   // non-empty groups; also orders the writes above
    if (tid < n_groups) {
      int rank = 0;   // position in the order (rows descending, group id ascending): a permutation
      for (int g = 0; g < n_groups; ++g) {
        const int r = s_rows[g];
        rank += (r > rows || (r == rows && g < tid)) ? 1 : 0;
      }
      s_order[rank] = tid;
      s_sorted[rank] = rows;
    }
    __syncthreads();
    // Fewer non-empty groups than XCDs: a deal of whole groups would leave XCDs idle.  Then every list holds every
    // group, len[kXcd] says so, and XCD x takes the tiles x, x + 8, ... of each group (locate_token_tile).
    const bool split = n_full < kXcd;
    if (tid == 0) len[kXcd] = split ? 1 : 0;
    if (tid < 64) {
      // the deal itself is sequential; lanes 0..7 of the first wave each keep one XCD's work, list length and tile
      // count, and a three-step DPP butterfly finds the least loaded XCD (ties to the lower one)
      const int lane = tid;
      int load = 0, n = 0, tiles = 0, n_big = 0;
      for (int i = 0; i < n_full; ++i) {   // descending order: the non-empty groups come first
        const int g = s_order[i], r = s_sorted[i];
        if (split) {
          if (lane < kXcd) {
            grp[(size_t)lane * cap + n] = make_int2(g, tiles);
            n += 1;
            n_big += r > small_rows ? 1 : 0;
            tiles += (r + tile_m - 1) / tile_m;
          }
          continue;
        }
        int key = lane < kXcd ? ((load << 3) | lane) : 0x7FFFFFFF;
        key = min(key, __builtin_amdgcn_update_dpp(key, key, 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
        key = min(key, __builtin_amdgcn_update_dpp(key, key, 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
        key = min(key, __builtin_amdgcn_update_dpp(key, key, 0x141, 0xF, 0xF, false));   // row_half_mirror
        if (lane == (key & (kXcd - 1))) {   // true in one of the lanes 0..7 only: the higher lanes hold 0x7FFFFFFF
          grp[(size_t)lane * cap + n] = make_int2(g, tiles);
          n += 1;
          n_big += r > small_rows ? 1 : 0;
          tiles += (r + tile_m - 1) / tile_m;
          load += (r + 63) / 64 + 2;
        }
      }
      if (lane < kXcd) {
        grp[(size_t)lane * cap + n] = make_int2(-1, tiles);
        len[lane] = n;
        len[kXcd + 1 + lane] = n_big;
      }
    }
  } else if (tid < kXcd) {
    const int x = tid;
    if (x == 0) len[kXcd] = 0;
    int n = 0, tiles = 0;
    for (int g = x; g < n_groups; g += kXcd) {
      const int rows = group_off[g + 1] - group_off[g];
      if (rows == 0) continue;
      grp[(size_t)x * cap + n++] = make_int2(g, tiles);
      tiles += (rows + tile_m - 1) / tile_m;
    }
    grp[(size_t)x * cap + n] = make_int2(-1, tiles);
    len[x] = n;
    len[kXcd + 1 + x] = n;   // unsorted lists: no group counts as small (the host passes small_rows = 0 here)
  }
}

__global__ __launch_bounds__(1024) void build_sched_kernel(const int32_t* __restrict__ group_off, int n_groups,
                                                           int cap, int2* __restrict__ grp, int* __restrict__ len,
                                                           int tile_m, int small_rows) {
  build_sched_body(group_off, n_groups, cap, grp, len, tile_m, small_rows);
}

// big_only: walk only the groups of more than small_rows tokens (the prefix of every list that the second set of
// lengths describes)
__device__ __forceinline__ bool locate_token_tile(const TokenSched& s, const int32_t* group_off, int wg, int tn,
                                                   bool big_only, int& g, int& mt, int& nt, int& slot0, int& rows) {
  const int x = wg & (kXcd - 1), local = wg >> 3;
  const int n = as_const(s.len)[big_only ? kXcd + 1 + x : x];
  const auto* list = as_const(s.grp) + (size_t)x * s.cap;
  if (as_const(s.len)[kXcd] != 0) {
    // split lists (fewer than 8 entries): XCD x takes the tiles x, x + 8, ... of every group, m tiles fastest
    int rest = local;
    for (int i = 0; i < n; ++i) {
      const int tm = list[i + 1].y - list[i].y, all = tm * tn;
      const int mine = all > x ? (all - x + kXcd - 1) / kXcd : 0;
      if (rest < mine) {
        const int w = x + kXcd * rest;
        g = list[i].x;
        nt = w / tm;
        mt = w - nt * tm;
        slot0 = as_const(group_off)[g];
        rows = as_const(group_off)[g + 1] - slot0;
        return true;
      }
      rest -= mine;
    }
    return false;
  }
  if (n == 0 || local >= list[n].y * tn) return false;
  int lo = 0, hi = n;  // list[lo].y * tn <= local < list[hi].y * tn
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (list[mid].y * tn <= local) lo = mid; else hi = mid;
  }
  g = list[lo].x;
  const int tm = list[lo + 1].y - list[lo].y;
  const int w = local - list[lo].y * tn;
  nt = w / tm;
  mt = w - nt * tm;
  slot0 = as_const(group_off)[g];
  rows = as_const(group_off)[g + 1] - slot0;
  return true;
}

}  // namespace meft
