// Grouped bf16 GEMM core for gfx950 matrix cores, shared by every dense contraction of the layer:
//
//   C[m, n] = sum_k A[m, k] * B(k, n)          fp32 accumulation, v_mfma_f32_32x32x16_bf16
//
// A is always contiguous along k.  B is either contiguous along k ("KC": rows indexed by n, used for
// the router and key scores, Eq. 5 / Eq. 6, and for dOut.V^T in the backward) or contiguous along n
// ("NC": rows indexed by k, used where the contraction runs over neurons or tokens: the value sum of
// Eq. 4, dh, dK, dV).  This file holds what both layouts share and the kernel of the KC problems, whose
// outputs need a pass through LDS (fp32 scores scattered by entry, masked activations in two layouts);
// gemm_stream.h holds the kernel of the NC problems.
//
// Tile 128 (m) x 256 (n) x 64 (k), 4 compute waves as 2 x 2, each wave 64 x 128 = 2 x 4 MFMA tiles, plus
// loader waves.  Operands go global -> LDS directly (global_load_lds, 16 B per lane), three stages of
// 48 KB in a ring with one barrier per k tile; the wait for a stage is a partial vmcnt so that the next
// stage's loads stay in flight.  LDS layouts are XOR-swizzled so that both the linear DMA writes
// and the fragment reads are free of bank conflicts:
//   k-contiguous operand: rows of 64 k = 8 chunks of 16 B; logical chunk c of row r sits at chunk
//     c ^ ((r >> 1) & 7); fragments are read with ds_read_b128.
//   n-contiguous operand: rows of 256 n = 32 chunks of 16 B; logical chunk c of row k sits at chunk
//     c ^ (2 * (k & 7)); fragments are read with the transposing ds_read_b64_tr_b16, which hands
//     lane i of a 16-lane group the four k-consecutive values of column i of a 4 x 16 block.
//
// Workgroups are mapped to tiles XCD-aware: consecutive workgroup ids go round-robin to the 8 XCDs,
// so workgroup id w works for XCD w % 8, and all tiles of one group (block of neurons) are given to
// one XCD, consecutively, so that the group's operand panels are fetched from HBM once and shared in
// that XCD's L2.
#pragma once
#include "common.h"

namespace meft {

constexpr int kTM = 128, kTN = 256, kTK = 64, kStages = 3;
constexpr int kStageElems = (kTM + kTN) * kTK;                 // 24576 bf16 = 48 KB
constexpr int kOperandLdsBytes = kStages * kStageElems * 2;    // 144 KB
constexpr int kIdRingSlots = 4;                                // k tiles of gathered-row numbers kept per loader
constexpr int kGemmLdsBytes = kOperandLdsBytes + 2 * kIdRingSlots * 64 * 4;   // + 2 KB
constexpr int kXcd = 8;

#define MEFT_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define MEFT_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;

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
//   static constexpr bool kBNC;                         B contiguous along n?
//   __device__ bool locate(int wg, TileCoord&) const;   false: no tile with id wg, nor with any larger id on
//                                                       the same XCD (ids wg + 8, wg + 16, ...)
//   __device__ const uint16_t* a_row(const TileCoord&, int m) const;   start of row m (clamped by the policy)
// and, for the kernel in this file (KC):
//   __device__ const uint16_t* b_row(const TileCoord&, int n) const;   start of B row n (clamped)
//   __device__ void store_rows(const TileCoord&, int r0, float* rows, int tid) const;   write tile rows r0..r0+31;
//       executed by the 256 compute threads (tid 0..255); any workgroup barrier inside must be MEFT_BARRIER_LDS()
//   static constexpr int kStoreBarriers;                number of such barriers in one store_rows call
// (gemm_stream.h lists what an NC policy provides instead.)
//
// acc[i][j][r] of a wave holds C[m][n] with m = wm + i*32 + (r/4)*8 + (lane/32)*4 + r%4,
// n = wn + j*32 + lane%32 (tile-local); the kernel lays 32 rows at a time out row-major in LDS (tile_index with
// the row counted from the pass start) and hands them to store_rows, which all 256 threads execute.  Global
// loads inside store_rows make the compiler wait for every outstanding vector-memory operation, including
// the next tile's operand loads; policies therefore read per-row indices with scalar loads where they can.

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// index of element (m, n) of an epilogue pass in LDS, m counted from the first row of the pass
__device__ __forceinline__ int tile_index(int m, int n) { return m * kTN + (n ^ (((m >> 2) & 1) << 7)); }

// Eight transposing LDS reads (the four n-contiguous B fragments of one k16 step, low and high k half)
// followed by the wait for them.  Written as one asm block: issued through the builtin, the compiler
// would order these reads after every outstanding global->LDS load (it cannot tell the stages apart),
// which would drain the operand pipeline at every k tile.  The barrier that hands a stage over already
// guarantees that the stage read here has landed.
template <int OFF>
__device__ __forceinline__ void tr_read8(u32x2 (&o)[8], const uint32_t (&alo)[4], const uint32_t (&ahi)[4]) {
  asm volatile(
      "ds_read_b64_tr_b16 %0, %8 offset:%16\n\t"
      "ds_read_b64_tr_b16 %1, %9 offset:%16\n\t"
      "ds_read_b64_tr_b16 %2, %10 offset:%16\n\t"
      "ds_read_b64_tr_b16 %3, %11 offset:%16\n\t"
      "ds_read_b64_tr_b16 %4, %12 offset:%16\n\t"
      "ds_read_b64_tr_b16 %5, %13 offset:%16\n\t"
      "ds_read_b64_tr_b16 %6, %14 offset:%16\n\t"
      "ds_read_b64_tr_b16 %7, %15 offset:%16\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]), "=&v"(o[4]), "=&v"(o[5]), "=&v"(o[6]), "=&v"(o[7])
      : "v"(alo[0]), "v"(ahi[0]), "v"(alo[1]), "v"(ahi[1]), "v"(alo[2]), "v"(ahi[2]), "v"(alo[3]), "v"(ahi[3]),
        "n"(OFF)
      : "memory");
}

constexpr int kEpiRows = 32;   // rows of the output tile staged through LDS per epilogue pass
constexpr int kLoaders = 2;    // waves that only request operands (the other four only compute)
constexpr int kGemmThreads = 256 + 64 * kLoaders;

// Workgroup barrier for the kernel below.  All six waves execute the same sequence of barriers; a compute wave
// first waits for its own LDS traffic, a loader wave for the operand loads that have to have landed.
#define MEFT_BARRIER_LDS() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

// Four compute waves (tid 0..255) and kLoaders loader waves.  The loaders own the whole global -> LDS traffic:
// measured on gfx950 the operand path, not the matrix cores or LDS, bounds these contractions (a compute unit keeps
// about a hundred 128-byte read requests in flight, no more), and a wave that both requests operands and issues
// MFMAs keeps neither queue full.  The workgroup is persistent: it works through tiles wg, wg + gridDim.x, ...
// (gridDim.x is a multiple of 8, so it stays on one XCD's list); the first two operand stages of the next tile are
// requested before the epilogue of the current one.
template <class P>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_mfma_kernel(P p, int n_tiles_bound) {
  static_assert(!P::kBNC, "n-contiguous B operands go through gemm_stream_kernel");
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // locate() answers false only when the workgroup's XCD has no tile with this or any larger id
  auto next_tile = [&](int& wg, TileCoord& t) -> bool { return wg < n_tiles_bound && p.locate(wg, t); };
  constexpr int kPasses = kTM / kEpiRows;

  int wg = blockIdx.x;
  TileCoord tc;
  if (!next_tile(wg, tc)) return;   // the same answer in every wave

  if (wave >= 4) {
    // ------------------------------------------------------------------ loader waves
    const int lw = wave - 4;
    constexpr int LA = kTM / 8 / kLoaders;   // A wave-loads (8 rows x 128 B) per loader and stage: 8
    constexpr int LB = kTN / 8 / kLoaders;   // B wave-loads (8 rows x 128 B) per loader and stage: 16
    static_assert(LA + LB <= 63, "partial vmcnt wait out of range");
    struct Loads {
      const uint16_t* pa[LA];
      const uint16_t* pb[LB];
    };
    const int lr8 = lane >> 3;
    auto setup = [&](Loads& L, const TileCoord& t) {
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        const int row = (lw * LA + i) * 8 + lr8;
        L.pa[i] = p.a_row(t, t.m0 + row) + (((lane & 7) ^ ((row >> 1) & 7)) << 3);
      }
#pragma unroll
      for (int i = 0; i < LB; ++i) {
        const int row = (lw * LB + i) * 8 + lr8;
        L.pb[i] = p.b_row(t, t.n0 + row) + (((lane & 7) ^ ((row >> 1) & 7)) << 3);
      }
    };
    auto issue = [&](const Loads& L, int kt, int stage) {
      uint16_t* sa = smem + stage * kStageElems;
      uint16_t* sb = sa + kTM * kTK;
#pragma unroll
      for (int i = 0; i < LA; ++i)
        __builtin_amdgcn_global_load_lds(MEFT_GPTR(L.pa[i] + kt * kTK), MEFT_LPTR(sa + (lw * LA + i) * 8 * kTK), 16, 0, 0);
#pragma unroll
      for (int i = 0; i < LB; ++i)
        __builtin_amdgcn_global_load_lds(MEFT_GPTR(L.pb[i] + kt * kTK), MEFT_LPTR(sb + (lw * LB + i) * 8 * kTK), 16, 0, 0);
    };

    // requests the first kStages - 1 k tiles of a tile
    auto prologue = [&](const Loads& L, const TileCoord& t) {
#pragma unroll
      for (int s = 0; s < kStages - 1; ++s)
        if (s < t.nk) issue(L, s, s);
    };
    Loads cur;
    setup(cur, tc);
    prologue(cur, tc);
    for (;;) {
      const int nk = tc.nk;
      int stage = 0;
      bool more = false;
      TileCoord tn;
      Loads nxt;
      for (int kt = 0; kt < nk; ++kt) {
        // k tile kt has landed once at most LA + LB younger loads of this wave are outstanding (the counter retires
        // in issue order); with no younger k tile requested, everything is awaited
        if (kt + 1 < nk) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(LA + LB) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        if (kt + kStages - 1 < nk) {
          int ps = stage - 1;
          if (ps < 0) ps += kStages;
          issue(cur, kt + kStages - 1, ps);                // the buffer of k tile kt-1: every compute wave is past it
        }
        if (kt == 0) { wg += gridDim.x; more = next_tile(wg, tn); }
        if (kt == nk - 1 && more) setup(nxt, tn);
        stage = stage + 1 == kStages ? 0 : stage + 1;
      }
      MEFT_BARRIER_LDS();   // every compute wave is done reading operand stages
      if (more) prologue(nxt, tn);
      // the epilogue's barriers (two per pass plus those inside the policy's store_rows)
#pragma unroll
      for (int b = 0; b < kPasses * (2 + P::kStoreBarriers); ++b) MEFT_BARRIER_LDS();
      if (!more) return;
      tc = tn;
      cur = nxt;
    }
  }

  // -------------------------------------------------------------------- compute waves
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 128;
  const int fr = lane & 31, fc = lane >> 5;
  int offA[2], keyA[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) { const int r = wm + i * 32 + fr; offA[i] = r * kTK; keyA[i] = (r >> 1) & 7; }
  int offB[4], keyB[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) { const int r = wn + j * 32 + fr; offB[j] = kTM * kTK + r * kTK; keyB[j] = (r >> 1) & 7; }

  for (;;) {
    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = tc.nk;
    int stage = 0;
    bool more = false;
    TileCoord tn;
    for (int kt = 0; kt < nk; ++kt) {
      MEFT_BARRIER_LDS();   // the loaders have seen k tile kt land
      if (kt == 0) { wg += gridDim.x; more = next_tile(wg, tn); }
      const uint16_t* st = smem + stage * kStageElems;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        bf16x8 fa[2], fb[4];
        const int c = ks * 2 + fc;
#pragma unroll
        for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(&st[offA[i] + ((c ^ keyA[i]) << 3)]);
#pragma unroll
        for (int j = 0; j < 4; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(&st[offB[j] + ((c ^ keyB[j]) << 3)]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
      stage = stage + 1 == kStages ? 0 : stage + 1;
    }

    MEFT_BARRIER_LDS();   // every compute wave is done reading operand stages; the loaders go on with the next tile

    // ---- epilogue: the fp32 tile goes through the LDS region of stage 2, kEpiRows rows at a time, so that the
    // policy can store whole rows with 16-byte accesses.  Layout of a pass: row-major, 256 floats per row, the
    // two 128-float halves of a row swapped when (row >> 2) is odd (keeps the half-waves of one accumulator
    // write in different banks).  Rows 32*pass .. +31 belong to the waves with wm == 64*(pass/2), fragment pass%2.
    float* tile = reinterpret_cast<float*>(smem + (kStages - 1) * kStageElems);
#pragma unroll
    for (int pass = 0; pass < kPasses; ++pass) {
      if ((wave >> 1) == (pass >> 1)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int n = wn + j * 32 + fr;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int ml = (r >> 2) * 8 + fc * 4 + (r & 3);
            tile[tile_index(ml, n)] = acc[pass & 1][j][r];
          }
        }
      }
      MEFT_BARRIER_LDS();
      p.store_rows(tc, pass * kEpiRows, tile, tid);   // contains P::kStoreBarriers workgroup barriers
      MEFT_BARRIER_LDS();
    }
    if (!more) break;
    tc = tn;
  }
}

// ---- tile schedule shared by the grouped problems ----------------------------------------------
// Every non-empty group (block of neurons with its tokens) is given to one XCD; XCD x works through its list
// in order.  grp[x][i] = (group, number of m tiles of the groups before it in this list); an end entry
// (-1, total m tiles) closes the list.  Inside a group the m tiles vary fastest, so that the tiles that share a
// B panel (one n tile of the group's block) run at the same time and the panel is read from HBM once.
//
// Groups differ in size (the router does not balance them), so they are dealt out longest first, each to the
// XCD with the least work so far (ties to the lower XCD); the work of a group is counted in 64-row units plus
// a constant for the per-tile overhead, which balances both the token-major tile counts and the contraction
// lengths of the neuron-major problems.  Which XCD computes a group has no influence on any result.
struct TokenSched {
  const int2* grp;       // [kXcd][cap]
  const int* len;        // [kXcd] number of groups in the list
  int cap;               // entries per XCD (n_groups + 1)
  int max_tiles;         // upper bound of m tiles of one XCD (for the tile-id bound of a launch)
};

constexpr int kSchedSortMax = 1024;   // up to this many groups are dealt out longest first; more: round-robin

// One workgroup of 1024 threads.
__global__ __launch_bounds__(1024) void build_sched_kernel(const int32_t* __restrict__ group_off, int n_groups,
                                                           int cap, int2* __restrict__ grp, int* __restrict__ len) {
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
    if (tid < 64) {
      // the deal itself is sequential; lanes 0..7 of the first wave each keep one XCD's work, list length and tile
      // count, and a three-step DPP butterfly finds the least loaded XCD (ties to the lower one)
      const int lane = tid;
      int load = 0, n = 0, tiles = 0;
      for (int i = 0; i < n_full; ++i) {   // descending order: the non-empty groups come first
        const int g = s_order[i], r = s_sorted[i];
        int key = lane < kXcd ? ((load << 3) | lane) : 0x7FFFFFFF;
        key = min(key, __builtin_amdgcn_update_dpp(key, key, 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
        key = min(key, __builtin_amdgcn_update_dpp(key, key, 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
        key = min(key, __builtin_amdgcn_update_dpp(key, key, 0x141, 0xF, 0xF, false));   // row_half_mirror
        if (lane == (key & (kXcd - 1))) {   // true in one of the lanes 0..7 only: the higher lanes hold 0x7FFFFFFF
          grp[(size_t)lane * cap + n] = make_int2(g, tiles);
          n += 1;
          tiles += (r + kTM - 1) / kTM;
          load += (r + 63) / 64 + 2;
        }
      }
      if (lane < kXcd) {
        grp[(size_t)lane * cap + n] = make_int2(-1, tiles);
        len[lane] = n;
      }
    }
  } else if (tid < kXcd) {
    const int x = tid;
    int n = 0, tiles = 0;
    for (int g = x; g < n_groups; g += kXcd) {
      const int rows = group_off[g + 1] - group_off[g];
      if (rows == 0) continue;
      grp[(size_t)x * cap + n++] = make_int2(g, tiles);
      tiles += (rows + kTM - 1) / kTM;
    }
    grp[(size_t)x * cap + n] = make_int2(-1, tiles);
    len[x] = n;
  }
}

__device__ __forceinline__ bool locate_token_tile(const TokenSched& s, const int32_t* group_off, int wg, int tn,
                                                   int& g, int& mt, int& nt, int& slot0, int& rows) {
  const int x = wg & (kXcd - 1), local = wg >> 3;
  const int n = as_const(s.len)[x];
  const auto* list = as_const(s.grp) + (size_t)x * s.cap;
  if (local >= list[n].y * tn) return false;
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
