// (token, block) dispatch in three passes over the entries, for up to 1024 blocks and 2^20 entries: the grouping of
// the T * top_e entries by block that the grouped GEMMs work from.  Entry i = t * top_e + q holds block sblk[i] (or
// -1); slots are the entries sorted by block, entries of one block in ascending entry (= token) order:
//   perm[slot] = entry, group_off[b] = first slot of block b, cnt[b] = its entries, tile_off = prefix of
//   ceil(cnt / BM), and on the matrix-core path tok_of_slot, slot_of_ent and the per-XCD tile schedule.
// A chunk is 1024 consecutive entries, one per thread.  Pass 1 counts the entries of every block per chunk, pass 2
// (one workgroup) turns the counts into offsets and deals the groups to the XCDs, pass 3 places the entries.  The
// rank of an entry inside its wave comes from ballots over the distinct blocks of the wave, the rest from prefix
// sums, so the order is the entry order and nothing depends on the timing of atomics.
// (Shapes beyond these limits use count_blocks / fill_groups / slot_maps / build_sched, which scan the entries
// once per block.)
#pragma once
#include "gemm_mfma.h"
#include "select.h"
#include "small_groups.h"

namespace meft {

constexpr int kDispMaxBlocks = 1024;    // LDS: 16 waves x n_blocks counters
constexpr int kDispMaxChunks = 1024;

// Rank of this lane's entry among the entries of the same block in its wave, in lane (= entry) order; lane
// `leader of the block` also writes the block's count in the wave to row[block] (row zeroed by the caller).
__device__ __forceinline__ int wave_block_ranks(int b, int* row) {
  const int lane = threadIdx.x & 63;
  int rank = 0;
  unsigned long long todo = __ballot(b >= 0);
  while (todo) {   // wave-uniform: one round per distinct block of the wave
    const int leader = __ffsll(todo) - 1;
    const int b0 = __shfl(b, leader, 64);
    const unsigned long long m = __ballot(b == b0);
    if (b == b0) rank = __popcll(m & ((1ull << lane) - 1ull));
    if (lane == leader) row[b0] = __popcll(m);
    todo &= ~m;
  }
  return rank;
}

__device__ __forceinline__ int dispatch_block_of(const int32_t* __restrict__ sblk, int i, int n_ent, int n_blocks) {
  const int b = i < n_ent ? sblk[i] : -1;
  return (unsigned)b < (unsigned)n_blocks ? b : -1;
}

// pass 1: H[chunk][b] = entries of block b in the chunk.  Dynamic LDS: 16 * n_blocks ints.
__global__ __launch_bounds__(1024) void dispatch_count_kernel(const int32_t* __restrict__ sblk, int n_ent,
                                                              int n_blocks, int32_t* __restrict__ H) {
  extern __shared__ int s_cnt[];   // [16 waves][n_blocks]
  const int tid = threadIdx.x, w = tid >> 6, c = blockIdx.x;
  for (int i = tid; i < 16 * n_blocks; i += 1024) s_cnt[i] = 0;
  __syncthreads();
  wave_block_ranks(dispatch_block_of(sblk, c * 1024 + tid, n_ent, n_blocks), s_cnt + w * n_blocks);
  __syncthreads();
  for (int b = tid; b < n_blocks; b += 1024) {
    int run = 0;
#pragma unroll
    for (int ww = 0; ww < 16; ++ww) run += s_cnt[ww * n_blocks + b];
    H[(size_t)c * n_blocks + b] = run;
  }
}

// pass 2, one workgroup: H[chunk][b] becomes the number of entries of block b in the chunks before; cnt, group_off,
// tile_off; with grp != nullptr also the tile schedule; with small_ent != nullptr the lists of the small groups.
__global__ __launch_bounds__(1024) void dispatch_scan_kernel(int32_t* __restrict__ H, int n_chunks, int n_blocks,
                                                             int BM, int32_t* __restrict__ cnt,
                                                             int32_t* __restrict__ group_off,
                                                             int32_t* __restrict__ tile_off, int cap,
                                                             int2* __restrict__ grp, int* __restrict__ len,
                                                             int sched_tile_m, int small_rows,
                                                             int2* __restrict__ small_ent,
                                                             int32_t* __restrict__ small_grp,
                                                             int32_t* __restrict__ small_cnt) {
  __shared__ int s_w[16];
  const int tid = threadIdx.x;   // = block, n_blocks <= 1024
  int tot = 0;
  if (tid < n_blocks) {
    // sixteen independent loads at a time: the serial part is the additions, not the memory latency
    for (int c0 = 0; c0 < n_chunks; c0 += 16) {
      int t[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) t[j] = c0 + j < n_chunks ? H[(size_t)(c0 + j) * n_blocks + tid] : 0;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        if (c0 + j < n_chunks) H[(size_t)(c0 + j) * n_blocks + tid] = tot;
        tot += t[j];
      }
    }
    cnt[tid] = tot;
  }
  int all_g, all_t;
  const int go = block_excl_scan_1024(tot, s_w, all_g);
  const int to = block_excl_scan_1024((tot + BM - 1) / BM, s_w, all_t);
  if (tid < n_blocks) { group_off[tid] = go; tile_off[tid] = to; }
  if (tid == 0) { group_off[n_blocks] = all_g; tile_off[n_blocks] = all_t; }
  if (grp != nullptr) {
    __syncthreads();   // group_off is read back below
    build_sched_body(group_off, n_blocks, cap, grp, len, sched_tile_m, small_rows);
  }
  if (small_ent != nullptr) {
    __syncthreads();   // group_off is read back; s_w is free again
    small_lists_body(group_off, n_blocks, small_rows, small_ent, small_grp, small_cnt, s_w);
  }
}

// pass 3: perm, and with tok_of_slot != nullptr the slot maps (tok_of_slot padded by `pad` valid entries).
// Dynamic LDS: 16 * n_blocks ints.
__global__ __launch_bounds__(1024) void dispatch_place_kernel(const int32_t* __restrict__ sblk, int n_ent,
                                                              int n_blocks, int e, const int32_t* __restrict__ H,
                                                              const int32_t* __restrict__ group_off,
                                                              int32_t* __restrict__ perm,
                                                              int32_t* __restrict__ tok_of_slot,
                                                              int32_t* __restrict__ slot_of_ent, int pad) {
  extern __shared__ int s_cnt[];   // [16 waves][n_blocks]
  const int tid = threadIdx.x, w = tid >> 6, c = blockIdx.x;
  for (int i = tid; i < 16 * n_blocks; i += 1024) s_cnt[i] = 0;
  __syncthreads();
  const int i = c * 1024 + tid;
  const int b = dispatch_block_of(sblk, i, n_ent, n_blocks);
  const int rank = wave_block_ranks(b, s_cnt + w * n_blocks);
  __syncthreads();
  // per block: first slot of wave 0's entries, then the exclusive prefix over the waves
  for (int bb = tid; bb < n_blocks; bb += 1024) {
    int run = group_off[bb] + H[(size_t)c * n_blocks + bb];
#pragma unroll
    for (int ww = 0; ww < 16; ++ww) {
      const int t = s_cnt[ww * n_blocks + bb];
      s_cnt[ww * n_blocks + bb] = run;
      run += t;
    }
  }
  __syncthreads();
  if (b >= 0) {
    const int slot = s_cnt[w * n_blocks + b] + rank;
    perm[slot] = i;
    if (tok_of_slot != nullptr) {
      tok_of_slot[slot] = i / e;
      slot_of_ent[i] = slot;
    }
  }
  if (tok_of_slot != nullptr && c == 0 && tid < pad) tok_of_slot[group_off[n_blocks] + tid] = 0;
}

}  // namespace meft
