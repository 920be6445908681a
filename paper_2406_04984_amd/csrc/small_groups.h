// Small token groups on the block-dense path.  The router does not balance its blocks (the paper uses no balancing
// loss; its experts simply run one after another), so a batch may send a handful of tokens to many blocks.  For such
// a group the matrix-core contractions after the selection would read the block's rows of V or K to use the few
// dozen that the group's tokens selected, and run whole tiles for a few rows.  Groups of at most `small_rows` tokens
// are therefore left out of those contractions (the tile schedule lists them last; see TokenSched) and handled here
// pair by pair, through the same intermediate arrays, so that everything downstream is unchanged:
//   forward   part[slot, :]   = sum over the token's selected neurons j of the block of act * V[j, :]        (Eq. 4)
//   backward  ds[t, i]        = act > 0 ? dOut[t, :] . V[j, :] : 0;   dhpart[slot, :] = sum ds * K[j, :]
//             dV[j, :], dK[j, :] of the block's touched neurons, the group's tokens summed in ascending order
// (Section 3.1, last paragraph).  The key scores of a small group still come from the score contraction: every
// neuron of a routed block has to be scored whatever the group's size (Eq. 6).
// A pair moves one row of d elements, so these kernels are bound by latency rather than by arithmetic: the work of
// one entry is spread over many waves (column chunks of 512 elements across workgroups, pairs across the waves of a
// workgroup), every sum in an order that the launch alone fixes.
// The entries of the small groups are listed once per dispatch (small_lists_body); workgroup x of a launch takes the
// entries x, x + gridDim.x, ... of that list, so consecutive workgroups, which go to the XCDs in turn, hold
// consecutive entries and every XCD gets its share of the memory traffic.
#pragma once
#include "common.h"
#include "select.h"

#ifndef MEFT_SMALL_ROWS
#define MEFT_SMALL_ROWS 16
#endif

namespace meft {

constexpr int kSmallRowChunk = 16;  // neurons per workgroup of the dV / dK kernel
constexpr int kSmallRowsMax = 16;   // upper limit of small_rows (size of that kernel's tables)
constexpr int kSmallRows = MEFT_SMALL_ROWS;   // a group of at most this many tokens is small; 0 switches the path off
constexpr int kSmallCols = 512;     // elements of a row that one wave covers in one step: 64 lanes x 8
constexpr int kSmallPairSplit = 8;  // workgroups that share the pairs of one entry in small_ds_kernel
static_assert(kSmallRows >= 0 && kSmallRows <= kSmallRowsMax, "the tables of small_dvdk_kernel hold kSmallRowsMax tokens");

// Positions p (ascending) of the pairs of one token whose neuron lies in block g, into s_list; returns their number.
// `it` = the token's idx row (any order), k entries.  s_w: 4 ints of scratch.  Called by all 256 threads.
__device__ __forceinline__ int collect_block_pairs(const int32_t* __restrict__ it, int k, int N, int bs, int g,
                                                   int* s_list, int* s_w) {
  int n = 0;
  for (int p0 = 0; p0 < k; p0 += 256) {
    const int p = p0 + (int)threadIdx.x;
    const int hit = (p < k && clampi(it[p], 0, N - 1) / bs == g) ? 1 : 0;
    int tot;
    const int pos = block_excl_scan_256(hit, s_w, tot);
    if (hit) s_list[n + pos] = p;
    n += tot;
  }
  __syncthreads();
  return n;
}

// The small groups of a dispatch and their entries, in group order: small_grp[0 .. small_cnt[1]) = groups of 1 to
// small_rows tokens, small_ent[0 .. small_cnt[0]) = (group, slot) of their entries.  The kernels below walk these
// lists, so that their launches need not cover every (group, token) position.  n_groups <= 1024; executed by one
// whole workgroup of 1024 threads (s_w: 16 ints of scratch).
__device__ __forceinline__ void small_lists_body(const int32_t* __restrict__ group_off, int n_groups, int small_rows,
                                                 int2* __restrict__ small_ent, int32_t* __restrict__ small_grp,
                                                 int32_t* __restrict__ small_cnt, int* s_w) {
  const int tid = threadIdx.x;
  int s0 = 0, rows = 0;
  if (tid < n_groups) { s0 = group_off[tid]; rows = group_off[tid + 1] - s0; }
  const bool sm = rows > 0 && rows <= small_rows;
  int tot_e, tot_g;
  const int eo = block_excl_scan_1024(sm ? rows : 0, s_w, tot_e);
  const int go = block_excl_scan_1024(sm ? 1 : 0, s_w, tot_g);
  if (sm) {
    small_grp[go] = tid;
    for (int i = 0; i < rows; ++i) small_ent[eo + i] = make_int2(tid, s0 + i);
  }
  if (tid == 0) { small_cnt[0] = tot_e; small_cnt[1] = tot_g; }
}

__global__ __launch_bounds__(1024) void small_lists_kernel(const int32_t* __restrict__ group_off, int n_groups,
                                                           int small_rows, int2* __restrict__ small_ent,
                                                           int32_t* __restrict__ small_grp,
                                                           int32_t* __restrict__ small_cnt) {
  __shared__ int s_w[16];
  small_lists_body(group_off, n_groups, small_rows, small_ent, small_grp, small_cnt, s_w);
}

// part[slot, c0 : c0 + 512] = sum over the entry's pairs of coef[t, p] * W[j, c0 : c0 + 512], c0 = 512 * blockIdx.y
// (W = V, coef = act: the forward's partial output row; W = K, coef = ds: the partial dh row).  Wave w takes the pairs
// w, w + 4, ... of the list; the four partial sums are added in wave order.  Dynamic LDS: k ints.
__global__ __launch_bounds__(256) void small_rowsum_kernel(const bf16_t* __restrict__ W,
                                                           const int32_t* __restrict__ idx,
                                                           const float* __restrict__ coef,
                                                           const int2* __restrict__ small_ent,
                                                           const int32_t* __restrict__ small_cnt,
                                                           const int32_t* __restrict__ tok_of_slot, int d, int k,
                                                           int N, int bs, bf16_t* __restrict__ part) {
  extern __shared__ int s_list[];
  __shared__ int s_w[4];
  __shared__ float s_red[3][kSmallCols];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = blockIdx.y * kSmallCols + lane * 8;
  const bool live = col < d;
  const int n_ent = small_cnt[0];
  for (int e = blockIdx.x; e < n_ent; e += gridDim.x) {
    const int g = small_ent[e].x, slot = small_ent[e].y, t = tok_of_slot[slot];
    const int32_t* it = idx + (size_t)t * k;
    const float* ct = coef + (size_t)t * k;
    const int n = collect_block_pairs(it, k, N, bs, g, s_list, s_w);
    float acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = 0.f;
    constexpr int U = 4;
    int q = wave;
    for (; q + 4 * (U - 1) < n; q += 4 * U) {
      float x[U][8], a[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int p = s_list[q + 4 * u];
        a[u] = ct[p];
        if (live) Vec8<bf16_t>::load(W + (size_t)clampi(it[p], 0, N - 1) * d + col, x[u]);
      }
      if (live) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[c] = fmaf(a[u], x[u][c], acc[c]);
      }
    }
    for (; q < n; q += 4) {
      const int p = s_list[q];
      const float a = ct[p];
      if (live) {
        float x[8];
        Vec8<bf16_t>::load(W + (size_t)clampi(it[p], 0, N - 1) * d + col, x);
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] = fmaf(a, x[c], acc[c]);
      }
    }
    if (wave > 0) {
#pragma unroll
      for (int c = 0; c < 8; ++c) s_red[wave - 1][lane * 8 + c] = acc[c];
    }
    __syncthreads();
    if (wave == 0 && live) {
#pragma unroll
      for (int w = 0; w < 3; ++w)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] += s_red[w][lane * 8 + c];
      Vec8<bf16_t>::store(part + (size_t)slot * d + col, acc);
    }
    __syncthreads();   // s_list and s_red are reused by the next entry
  }
}

// backward: ds32[t * k + p] = act > 0 ? dOut[t, :] . V[j, :] : 0 for the pairs of the entry; one wave per pair, the
// entry's pairs dealt to the 4 * kSmallPairSplit waves of the workgroups blockIdx.y = 0 .. kSmallPairSplit - 1.
// Dynamic LDS: k ints.
__global__ __launch_bounds__(256) void small_ds_kernel(const bf16_t* __restrict__ V, const bf16_t* __restrict__ dOut,
                                                       const int32_t* __restrict__ idx, const float* __restrict__ act,
                                                       const int2* __restrict__ small_ent,
                                                       const int32_t* __restrict__ small_cnt,
                                                       const int32_t* __restrict__ tok_of_slot, int d, int k, int N,
                                                       int bs, float* __restrict__ ds32) {
  extern __shared__ int s_list[];
  __shared__ int s_w[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_ent = small_cnt[0];
  for (int e = blockIdx.x; e < n_ent; e += gridDim.x) {
    const int g = small_ent[e].x, t = tok_of_slot[small_ent[e].y];
    const int32_t* it = idx + (size_t)t * k;
    const float* at = act + (size_t)t * k;
    const int n = collect_block_pairs(it, k, N, bs, g, s_list, s_w);
    const bf16_t* grow = dOut + (size_t)t * d;
    for (int q = blockIdx.y * 4 + wave; q < n; q += 4 * kSmallPairSplit) {
      const int p = s_list[q];
      const bf16_t* vrow = V + (size_t)clampi(it[p], 0, N - 1) * d;
      float dot = 0.f;
#pragma unroll 4
      for (int col = lane * 8; col < d; col += kSmallCols) {
        float x[8], y[8];
        Vec8<bf16_t>::load(vrow + col, x);
        Vec8<bf16_t>::load(grow + col, y);
#pragma unroll
        for (int c = 0; c < 8; ++c) dot = fmaf(x[c], y[c], dot);
      }
      dot = wave_sum(dot);
      if (lane == 0) ds32[(size_t)t * k + p] = at[p] > 0.f ? dot : 0.f;
    }
    __syncthreads();   // s_list is reused by the next entry
  }
}

// backward: dV and dK rows of a small group's block.  Only this group's tokens select neurons of its block, so the
// touched rows of the block are exactly the rows some token of the group selected.  The chunk of kSmallRowChunk
// neurons is the fast launch index (blockIdx.x), so that the chunks of one group, whose work is alike, go to the
// XCDs in turn whatever the sizes of the groups.  Per (group, chunk): tables in LDS say which tokens of the group
// select each neuron of the chunk, with which activation and activation gradient; the (selected neuron, 512 columns)
// pieces are dealt to the four waves, and a neuron's rows are summed over the group's tokens in ascending slot
// (= token) order.
__device__ __forceinline__ void small_dvdk_piece(const bf16_t* __restrict__ h, const bf16_t* __restrict__ dOut,
                                                 const int* tok, const float* a, const float* s, int rows, int d,
                                                 int col, float (&aK)[8], float (&aV)[8]) {
#pragma unroll
  for (int c = 0; c < 8; ++c) { aK[c] = 0.f; aV[c] = 0.f; }
  for (int i = 0; i < rows; ++i) {
    const int t = tok[i];
    if (t < 0) continue;
    float xg[8], xh[8];
    Vec8<bf16_t>::load(dOut + (size_t)t * d + col, xg);
    Vec8<bf16_t>::load(h + (size_t)t * d + col, xh);
    const float av = a[i], sv = s[i];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      aV[c] = fmaf(av, xg[c], aV[c]);
      aK[c] = fmaf(sv, xh[c], aK[c]);
    }
  }
}

__global__ __launch_bounds__(256) void small_dvdk_kernel(const bf16_t* __restrict__ h, const bf16_t* __restrict__ dOut,
                                                         const int32_t* __restrict__ idx, const float* __restrict__ act,
                                                         const float* __restrict__ ds32,
                                                         const int32_t* __restrict__ small_grp,
                                                         const int32_t* __restrict__ small_cnt,
                                                         const int32_t* __restrict__ group_off,
                                                         const int32_t* __restrict__ tok_of_slot, int d, int k, int N,
                                                         int bs, bf16_t* __restrict__ dK, bf16_t* __restrict__ dV) {
  __shared__ int s_tok[kSmallRowChunk][kSmallRowsMax];     // token that selects the neuron, or -1
  __shared__ float s_a[kSmallRowChunk][kSmallRowsMax];     // its activation
  __shared__ float s_s[kSmallRowChunk][kSmallRowsMax];     // its activation gradient
  __shared__ int s_rows[kSmallRowChunk];                   // the selected neurons of the chunk, ascending
  __shared__ int s_nrows;
  static_assert(kSmallRowChunk <= 64, "one lane of the first wave per neuron of the chunk");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r0 = blockIdx.x * kSmallRowChunk;   // first neuron of the chunk, inside the block
  const int n_grp = small_cnt[1];
  for (int e = blockIdx.y; e < n_grp; e += gridDim.y) {
    const int g = small_grp[e];
    const int slot0 = group_off[g], rows = min(group_off[g + 1] - slot0, kSmallRowsMax);   // (at most small_rows)
    for (int z = tid; z < kSmallRowChunk * kSmallRowsMax; z += 256) (&s_tok[0][0])[z] = -1;
    __syncthreads();
    // the group's rows * k pairs, four per thread and step, loads first
    const int n_pairs = rows * k;
    for (int z0 = 0; z0 < n_pairs; z0 += 4 * 256) {
      int ii[4], pp[4], tt[4], jj[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int z = z0 + u * 256 + tid;
        ii[u] = z < n_pairs ? z / k : -1;
        pp[u] = z - ii[u] * k;
        tt[u] = ii[u] >= 0 ? tok_of_slot[slot0 + ii[u]] : 0;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) jj[u] = ii[u] >= 0 ? clampi(idx[(size_t)tt[u] * k + pp[u]], 0, N - 1) : -1;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int r = jj[u] - g * bs - r0;
        if (jj[u] >= 0 && jj[u] / bs == g && r >= 0 && r < kSmallRowChunk) {   // ids are distinct inside a token: one writer per cell
          s_tok[r][ii[u]] = tt[u];
          s_a[r][ii[u]] = act[(size_t)tt[u] * k + pp[u]];
          s_s[r][ii[u]] = ds32[(size_t)tt[u] * k + pp[u]];
        }
      }
    }
    __syncthreads();
    if (wave == 0) {
      bool any = false;
      if (lane < kSmallRowChunk)
        for (int i = 0; i < rows; ++i) any |= s_tok[lane][i] >= 0;
      const unsigned long long m = __ballot(any);
      if (any) s_rows[__popcll(m & ((1ull << lane) - 1ull))] = lane;
      if (lane == 0) s_nrows = __popcll(m);
    }
    __syncthreads();
    const int cpr = (d + kSmallCols - 1) / kSmallCols;   // column pieces per row
    const int n_items = s_nrows * cpr;
    int it = wave;
    for (; it + 4 < n_items; it += 8) {   // two pieces at a time
      const int z0 = it / cpr, z1 = (it + 4) / cpr;
      const int r_0 = s_rows[z0], r_1 = s_rows[z1];
      const int c_0 = (it - z0 * cpr) * kSmallCols + lane * 8, c_1 = (it + 4 - z1 * cpr) * kSmallCols + lane * 8;
      float k0[8], v0[8], k1[8], v1[8];
      if (c_0 < d) small_dvdk_piece(h, dOut, s_tok[r_0], s_a[r_0], s_s[r_0], rows, d, c_0, k0, v0);
      if (c_1 < d) small_dvdk_piece(h, dOut, s_tok[r_1], s_a[r_1], s_s[r_1], rows, d, c_1, k1, v1);
      const size_t j0 = (size_t)g * bs + r0 + r_0, j1 = (size_t)g * bs + r0 + r_1;
      if (c_0 < d) { Vec8<bf16_t>::store(dV + j0 * d + c_0, v0); Vec8<bf16_t>::store(dK + j0 * d + c_0, k0); }
      if (c_1 < d) { Vec8<bf16_t>::store(dV + j1 * d + c_1, v1); Vec8<bf16_t>::store(dK + j1 * d + c_1, k1); }
    }
    for (; it < n_items; it += 4) {
      const int z0 = it / cpr, r_0 = s_rows[z0];
      const int c_0 = (it - z0 * cpr) * kSmallCols + lane * 8;
      if (c_0 >= d) continue;
      float k0[8], v0[8];
      small_dvdk_piece(h, dOut, s_tok[r_0], s_a[r_0], s_s[r_0], rows, d, c_0, k0, v0);
      const size_t j0 = (size_t)g * bs + r0 + r_0;
      Vec8<bf16_t>::store(dV + j0 * d + c_0, v0);
      Vec8<bf16_t>::store(dK + j0 * d + c_0, k0);
    }
    __syncthreads();   // the tables are reused by the next group
  }
}

}  // namespace meft
