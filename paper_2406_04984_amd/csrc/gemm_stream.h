// Streaming variant of the grouped bf16 GEMM core for the contractions whose B operand is contiguous along n
// (value sum of Eq. 4, dh, dK, dV) and whose output is a bf16 matrix with contiguous rows.
//
// Same tile (128 x 256 x 64), LDS layouts, fragment reads and wave roles as gemm_mfma_kernel.  Two things differ:
//
//  * The k tiles of all the tiles a workgroup works through form ONE stream through the three-stage ring: the
//    loaders request stream position s + 2 right after the barrier that hands position s to the compute waves,
//    whether or not s + 2 belongs to the next output tile.  The operand pipeline therefore never drains at a tile
//    boundary (measured, draining and refilling it cost about as much as five k tiles per output tile).
//
//  * The epilogue needs neither LDS nor barriers: neighbouring lanes exchange one accumulator value through a DPP
//    move, so that every lane holds two adjacent columns of one row, packs them to bf16 and stores 4 bytes.  A half
//    wave thus writes 64 contiguous bytes of each of two rows per instruction.  While the compute waves store, the
//    loaders are already two k tiles into the next tile.
//
// There is exactly one workgroup barrier per k tile of the stream, executed by all six waves.  (An extra barrier at
// the end of every tile, releasing its last stage before the stores so that the loaders request a third k tile
// during the epilogue, was measured and did not pay.)
//
// A policy P of this kernel provides locate and a_row (see gemm_mfma.h) and
//   static constexpr bool kRowIdsInMemory;
//       false: __device__ int b_row_ids(const TileCoord&, int k) const;  number of the B row that holds k (plain
//              arithmetic, no memory access), any valid row for k beyond the contraction length;
//       true:  __device__ const int32_t* b_row_id_src(const TileCoord&, int k0) const;  where the numbers of the B rows
//              of k0 .. k0 + 63 are stored (valid rows also beyond the contraction length: those products are zero);
//              called for k0 = 0, 64, ... below 64 * nk.  The numbers travel like the operands: a 4-byte-per-lane
//              global -> LDS load puts the 64 numbers of a k tile into a small ring in LDS one position ahead of
//              the operand request that uses them;
//   __device__ const uint16_t* b_row_ptr(int row) const;          start of B row `row`; rows are TileCoord::Ncols
//                                                                 elements apart
//   __device__ uint16_t* out_base(const TileCoord&) const;        row 0, column 0 of the group's output; the leading
//                                                                 dimension is TileCoord::Ncols (a multiple of 32)
//   __device__ bool out_row_ok(const TileCoord&, int m) const;    is row m of the group's output stored?  (false for
//                                                                 m beyond the group's rows); may read memory
#pragma once
#include <type_traits>

#include "gemm_mfma.h"

namespace meft {

// Twelve transposing LDS reads of one k16 step (the two m-contiguous A fragments and the four n-contiguous B
// fragments, low and high k half each) followed by the wait for them; one asm block for the reason given at
// tr_read8.  xa = {A0 low, A0 high, A1 low, A1 high}.
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

template <class P>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_stream_kernel(P p, int n_tiles_bound) {
  static_assert(P::kBNC, "the streaming kernel covers the n-contiguous B layouts");
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // locate() answers false only when the workgroup's XCD has no tile with this or any larger id
  auto next_tile = [&](int wg, TileCoord& t) -> bool { return wg < n_tiles_bound && p.locate(wg, t); };
  const int step = gridDim.x;

  TileCoord tc;
  if (!next_tile(blockIdx.x, tc)) return;   // the same answer in every wave

  if (wave >= 4) {
    // ------------------------------------------------------------------ loader waves
    const int lw = wave - 4;
    constexpr int LA = kTM / 8 / kLoaders;   // A wave-loads (8 rows x 128 B) per loader and stage
    constexpr int LB = 32 / kLoaders;        // B wave-loads (2 rows x 512 B) per loader and stage
    static_assert(LA + LB <= 63, "partial vmcnt wait out of range");
    const int lr8 = lane >> 3;
    int* idring = reinterpret_cast<int*>(smem + kOperandLdsBytes / 2) + lw * kIdRingSlots * 64;

    // Three cursors walk the same sequence of (tile, k tile) pairs: the row numbers of the gathered B rows are
    // requested three positions ahead of the barrier, the operands two positions ahead.
    //   consume: position handed to the compute waves at the next barrier
    int wg_c = blockIdx.x, nk_c = tc.nk;
    //   operands
    int wg_o = blockIdx.x, k_o = 0, n_o = 0, stage_o = 0;
    bool ok_o = true;
    TileCoord t_o = tc;
    // A, k-contiguous: a wave-load covers 8 rows (m) x 128 bytes; fixed row pointers per tile, advanced by k.
    // A, m-contiguous (P::kAMC): a wave-load covers 4 rows (k) x 256 bytes; lane l fetches the 16-byte chunk
    // (l & 15) ^ (4 * (row & 3)) of its row (the LDS swizzle; row & 3 == (l >> 4) & 3 for every load), so one column
    // offset per tile serves all the loads.
    const uint16_t* pa[LA];
    int acol = 0;
    auto setup = [&]() {
      if constexpr (P::kAMC) {
        const int chunk = (lane & 15) ^ (4 * ((lane >> 4) & 3));
        const int col = t_o.m0 + chunk * 8, last = p.a_cols(t_o) - 8;
        acol = col > last ? last : col;                                 // clamp (rows beyond Mrows are never stored)
      } else {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
          const int row = (lw * LA + i) * 8 + lr8;
          pa[i] = p.a_row(t_o, t_o.m0 + row) + (((lane & 7) ^ ((row >> 1) & 7)) << 3);
        }
      }
    };
    //   row numbers (only where they sit in memory)
    int wg_d = blockIdx.x, k_d = 0, n_d = 0;
    bool ok_d = P::kRowIdsInMemory;
    TileCoord t_d = tc;

    auto request_ids = [&]() {
      if constexpr (P::kRowIdsInMemory) {
        if (!ok_d) return;
        __builtin_amdgcn_global_load_lds(MEFT_GPTR(p.b_row_id_src(t_d, k_d * kTK) + lane),
                                         MEFT_LPTR(idring + (n_d & (kIdRingSlots - 1)) * 64), 4, 0, 0);
        ++n_d;
        if (++k_d == t_d.nk) { wg_d += step; k_d = 0; ok_d = next_tile(wg_d, t_d); }
      }
    };
    // B: a wave-load covers two k rows (lanes 0..31 the even one, lanes 32..63 the odd one), 512 bytes of each.
    // Lane l fetches the 16-byte chunk (l & 31) ^ (2 * (row & 7)) of its row (the LDS swizzle); row & 7 only
    // depends on i & 3, so four column offsets per tile cover all the loads.
    const int half = lane >> 5;
    const uint16_t* bcol[4];
    auto setup_b = [&]() {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int chunk = (lane & 31) ^ (2 * ((2 * q + half) & 7));
        int col = t_o.n0 + chunk * 8;
        col = col > t_o.Ncols - 8 ? t_o.Ncols - 8 : col;              // clamp (columns beyond Ncols are never stored)
        bcol[q] = p.b_row_ptr(0) + col;
      }
    };
    auto request_operands = [&]() {
      if (!ok_o) return;
      // ids[i]: number of the B row this lane fetches in its i-th load, k = 64 * k_o + 2 * (lw * LB + i) + half
      int ids[LB];
      if constexpr (P::kRowIdsInMemory) {
        // out of the ring; one asm block with its own wait (through plain loads the compiler would first drain every
        // outstanding operand load)
        const uint32_t a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(
            idring + (n_o & (kIdRingSlots - 1)) * 64 + 2 * lw * LB + half);
        static_assert(LB == 16, "the block below reads sixteen row numbers");
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
      } else {
#pragma unroll
        for (int i = 0; i < LB; ++i) ids[i] = p.b_row_ids(t_o, k_o * kTK + 2 * (lw * LB + i) + half);
      }
      uint16_t* sa = smem + stage_o * kStageElems;
      uint16_t* sb = sa + kTM * kTK;
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        if constexpr (P::kAMC) {
          const uint16_t* src = p.a_krow(t_o, k_o * kTK + 4 * (lw * LA + i) + (lane >> 4)) + acol;
          __builtin_amdgcn_global_load_lds(MEFT_GPTR(src), MEFT_LPTR(sa + (lw * LA + i) * 4 * kTM), 16, 0, 0);
        } else {
          __builtin_amdgcn_global_load_lds(MEFT_GPTR(pa[i] + k_o * kTK), MEFT_LPTR(sa + (lw * LA + i) * 8 * kTK), 16, 0, 0);
        }
      }
      const uint32_t row_bytes = (uint32_t)t_o.Ncols * 2u;
#pragma unroll
      for (int i = 0; i < LB; ++i) {
        const char* src = reinterpret_cast<const char*>(bcol[i & 3]) + (uint64_t)(uint32_t)ids[i] * row_bytes;
        __builtin_amdgcn_global_load_lds(MEFT_GPTR(src), MEFT_LPTR(sb + (lw * LB + i) * 512), 16, 0, 0);
      }
      ++n_o;
      stage_o = stage_o + 1 == kStages ? 0 : stage_o + 1;
      if (++k_o == t_o.nk) {
        wg_o += step; k_o = 0; ok_o = next_tile(wg_o, t_o);
        if (ok_o) { setup(); setup_b(); }
      }
    };

    setup();
    setup_b();
    if constexpr (P::kRowIdsInMemory) {
#pragma unroll
      for (int s = 0; s < kStages; ++s) request_ids();
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
#pragma unroll
    for (int s = 0; s < kStages - 1; ++s) request_operands();

    int n_c = 0;   // positions handed over so far
    for (;;) {
      for (int kt = 0; kt < nk_c; ++kt) {
        // position n_c has landed once at most the LA + LB loads of position n_c + 1 are outstanding (the counter
        // retires in issue order, and the row numbers of a later position are requested before those loads); with
        // nothing requested beyond n_c, everything is awaited
        if (n_o > n_c + 1) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(LA + LB) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        // every compute wave is past position n_c - 1: its stage takes position n_c + 2
        request_ids();
        request_operands();
        ++n_c;
      }
      wg_c += step;
      TileCoord t;
      if (!next_tile(wg_c, t)) return;
      nk_c = t.nk;
    }
  }

  // -------------------------------------------------------------------- compute waves
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 128;
  const int fr = lane & 31, fc = lane >> 5;
  int offA[2], keyA[2];            // k-contiguous A
  uint32_t tra_lo[2], tra_hi[2];   // m-contiguous A: LDS byte offsets (inside a stage) of the transposing reads
#pragma unroll
  for (int i = 0; i < 2; ++i) { const int r = wm + i * 32 + fr; offA[i] = r * kTK; keyA[i] = (r >> 1) & 7; }
  {
    // rows of 128 m = 16 chunks of 16 B; logical chunk c of row k sits at chunk c ^ (4 * (k & 3))
    const int gq = lane >> 4, s = lane & 15;
    const int k_lo = 8 * (gq >> 1) + (s >> 2), k_hi = k_lo + 4;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int m = wm + i * 32 + 16 * (gq & 1) + 4 * (s & 3);
      tra_lo[i] = (uint32_t)(k_lo * kTM + (((m >> 3) ^ (4 * (k_lo & 3))) << 3) + (m & 7)) * 2u;
      tra_hi[i] = (uint32_t)(k_hi * kTM + (((m >> 3) ^ (4 * (k_hi & 3))) << 3) + (m & 7)) * 2u;
    }
  }
  uint32_t tr_lo[4], tr_hi[4];  // LDS byte offsets (inside a stage's B region) of this lane's transposing reads
  {
    // lane s of a 16-lane group points at row (k base + s/4), columns 4*(s%4)..+3 of a 4 x 16 block and
    // receives column s of that block, four consecutive k.  Low half: k = 8*(lane/32) + 0..3, high half +4.
    const int gq = lane >> 4, s = lane & 15;
    const int k_lo = 8 * (gq >> 1) + (s >> 2), k_hi = k_lo + 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = wn + j * 32 + 16 * (gq & 1) + 4 * (s & 3);
      tr_lo[j] = (uint32_t)(k_lo * 256 + (((n >> 3) ^ (2 * (k_lo & 7))) << 3) + (n & 7)) * 2u;
      tr_hi[j] = (uint32_t)(k_hi * 256 + (((n >> 3) ^ (2 * (k_hi & 7))) << 3) + (n & 7)) * 2u;
    }
  }

  int wg = blockIdx.x;
  int stage = 0;   // runs on across tiles, like the loaders' stage_o
  for (;;) {
    // lane l: is row wm + l of this tile stored?  Asked before the k loop, so that a policy's memory read has
    // long returned when the answer is needed.
    const int row_ok = p.out_row_ok(tc, tc.m0 + wm + lane) ? 1 : 0;

    f32x16 acc[2][4];
    const int nk = tc.nk;
    bool more = false;
    TileCoord tn;
    // one k tile out of stage `stage`; kFirst: the first k16 step starts from zero instead of from acc (the matrix
    // instruction takes the constant as its addend, so the accumulators are never cleared by hand)
    auto k_tile = [&](auto first_tag) {
      constexpr bool kFirst = decltype(first_tag)::value;
      const uint16_t* st = smem + stage * kStageElems;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        bf16x8 fa[2], fb[4];
        // k16 step ks starts 16 rows further (B: 8192 bytes, m-contiguous A: 4096 bytes); that changes neither
        // (k & 7) nor (k & 3), so the swizzles hold
        const uint32_t sbase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(st + kTM * kTK);
        uint32_t alo[4], ahi[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { alo[j] = sbase + tr_lo[j]; ahi[j] = sbase + tr_hi[j]; }
        u32x2 o[8];
        if constexpr (P::kAMC) {
          const uint32_t abase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(st);
          const uint32_t xa[4] = {abase + tra_lo[0], abase + tra_hi[0], abase + tra_lo[1], abase + tra_hi[1]};
          u32x2 oa[4];
          if (ks == 0) tr_read12<0, 0>(oa, o, xa, alo, ahi);
          else if (ks == 1) tr_read12<4096, 8192>(oa, o, xa, alo, ahi);
          else if (ks == 2) tr_read12<8192, 16384>(oa, o, xa, alo, ahi);
          else tr_read12<12288, 24576>(oa, o, xa, alo, ahi);
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const u32x4 w = {oa[2 * i].x, oa[2 * i].y, oa[2 * i + 1].x, oa[2 * i + 1].y};
            fa[i] = __builtin_bit_cast(bf16x8, w);
          }
        } else {
          const int c = ks * 2 + fc;
#pragma unroll
          for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(&st[offA[i] + ((c ^ keyA[i]) << 3)]);
          if (ks == 0) tr_read8<0>(o, alo, ahi);
          else if (ks == 1) tr_read8<8192>(o, alo, ahi);
          else if (ks == 2) tr_read8<16384>(o, alo, ahi);
          else tr_read8<24576>(o, alo, ahi);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const u32x4 w = {o[2 * j].x, o[2 * j].y, o[2 * j + 1].x, o[2 * j + 1].y};
          fb[j] = __builtin_bit_cast(bf16x8, w);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (kFirst && ks == 0) {
              const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], zero, 0, 0, 0);
            } else {
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
          }
      }
      stage = stage + 1 == kStages ? 0 : stage + 1;
    };
    MEFT_BARRIER_LDS();   // the loaders have seen the tile's first k tile land
    wg += step;
    more = next_tile(wg, tn);
    k_tile(std::true_type{});
    for (int kt = 1; kt < nk; ++kt) {
      MEFT_BARRIER_LDS();
      k_tile(std::false_type{});
    }

    // ---- epilogue, out of the registers.  acc[i][j][r] is C[m][n] with m = wm + i*32 + (r/4)*8 + (lane/32)*4 + r%4
    // and n = wn + j*32 + lane%32.  For a register pair (r, r+1), r even, an even lane (column c) keeps its value of
    // row m and takes its right neighbour's value of that row; the odd lane (column c+1) keeps its value of row m+1
    // and takes its left neighbour's (DPP quad_perm [1,0,3,2] swaps neighbours).  Both then hold columns (c, c+1) of
    // one row.
    {
      const bool odd = (lane & 1) != 0;
      const int ld = tc.Ncols;
      const int nj = (ld - (tc.n0 + wn)) / 32;   // 32-column fragments of this wave that lie inside the matrix
      uint16_t* base = p.out_base(tc) + (size_t)(tc.m0 + wm) * ld + (tc.n0 + wn + (fr & ~1));
#pragma unroll
      for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const int rl = i * 32 + (r >> 2) * 8 + fc * 4 + (r & 3) + (lane & 1);    // row inside the wave's 64
          const bool ok = __builtin_amdgcn_ds_bpermute(rl << 2, row_ok) != 0;
          uint32_t pk[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float a = acc[i][j][r], b = acc[i][j][r + 1];   // plain copies: the values go to the builtin as floats
            const float an = __builtin_amdgcn_update_dpp(a, a, 0xB1, 0xF, 0xF, true);   // the neighbour's a
            const float bn = __builtin_amdgcn_update_dpp(b, b, 0xB1, 0xF, 0xF, true);   // the neighbour's b
            pk[j] = odd ? pack_bf16x2(bn, b) : pack_bf16x2(a, an);
          }
          if (ok) {
            uint32_t* rowp = reinterpret_cast<uint32_t*>(base + (size_t)rl * ld);
            if (nj > 0) rowp[0] = pk[0];
            if (nj > 1) rowp[16] = pk[1];
            if (nj > 2) rowp[32] = pk[2];
            if (nj > 3) rowp[48] = pk[3];
          }
        }
      }
    }
    if (!more) break;
    tc = tn;
  }
}

}  // namespace meft
