// Batch-union evaluation of the adapter (Algorithm 1 as printed): S = the union of all tokens' selections,
// K[S] and V[S] are compacted, and every token is evaluated densely over S:
//     out = ReLU(h K[S]^T) V[S],   with the matching backward.
// The compacted rows are cut into virtual blocks of `vbs` rows, and every token is given an entry for every
// virtual block; with that index structure the contractions are the same grouped matrix-core GEMMs as in the
// per-token block-dense path (group = one virtual block with all T tokens), the ReLU being applied in the score
// GEMM's epilogue instead of a top-k selection.
#pragma once
#include "dense_path.h"

namespace meft {

// flag[j] = 1 for every selected neuron id (flags cleared before); ids outside [0, N) are ignored
__global__ __launch_bounds__(256) void mark_idx_kernel(const int32_t* __restrict__ idx, int P, int N,
                                                       int32_t* __restrict__ flag) {
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= P) return;
  const int j = idx[p];
  if ((unsigned)j < (unsigned)N) flag[j] = 1;
}

// Index structure of the virtual blocks, from the union size U = *n_S (device):
//   n_real = ceil(U / vbs) blocks hold rows; block g < n_real has all T tokens as its group, slot g*T + t.
//   entry of token t for block g: t*nvb + g.  Blocks g >= n_real are empty (sblk = -1).
// One thread per (block, token) slot of the full nvb x T grid; the small tables are written by workgroup 0.
__global__ __launch_bounds__(256) void union_maps_kernel(const int32_t* __restrict__ n_S, int cap, int T, int vbs,
                                                         int nvb,
                                                         int32_t* __restrict__ sblk, int32_t* __restrict__ perm,
                                                         int32_t* __restrict__ tok_of_slot,
                                                         int32_t* __restrict__ slot_of_ent,
                                                         int32_t* __restrict__ group_off,
                                                         int32_t* __restrict__ rowflag) {
  const int U = max(0, min(*n_S, cap));   // cap <= nvb * vbs is the capacity of S
  const int n_real = (U + vbs - 1) / vbs;
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < (long long)nvb * T) {
    const int g = (int)(i / T), t = (int)(i - (long long)g * T);
    const int ent = t * nvb + g;
    if (g < n_real) {
      perm[i] = ent;
      tok_of_slot[i] = t;
      slot_of_ent[ent] = (int)i;
      sblk[ent] = g;
    } else {
      sblk[ent] = -1;
    }
  }
  // kSlotPad valid entries behind the last real slot (the GEMMs look row numbers up a little beyond a group)
  if (i >= (long long)n_real * T && i < (long long)n_real * T + kSlotPad) tok_of_slot[i] = 0;
  if (i < (long long)nvb * vbs) rowflag[i] = i < U ? 1 : 0;   // which compacted rows exist
  if (blockIdx.x == 0) {
    for (int g = threadIdx.x; g <= nvb; g += 256) {
      const int r = g < n_real ? g : n_real;
      group_off[g] = r * T;
    }
  }
}

// dst[i, :] = src[S[i], :] for i < U, zero for U <= i < n_real*vbs (the tail of the last virtual block).
// One workgroup per compacted row at a time; 16-byte accesses (bf16 rows, d % 8 == 0).
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint16_t* __restrict__ src,
                                                          const int32_t* __restrict__ S,
                                                          const int32_t* __restrict__ n_S, int cap, int N, int d,
                                                          int vbs, uint16_t* __restrict__ dst) {
  const int U = max(0, min(*n_S, cap));
  const int rows = ((U + vbs - 1) / vbs) * vbs;
  for (int i = blockIdx.x; i < rows; i += gridDim.x) {
    int j = -1;
    if (i < U) { j = S[i]; if ((unsigned)j >= (unsigned)N) j = -1; }
    u32x4* o = reinterpret_cast<u32x4*>(dst + (size_t)i * d);
    const u32x4* in = j >= 0 ? reinterpret_cast<const u32x4*>(src + (size_t)j * d) : nullptr;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int c = threadIdx.x; c < d / 8; c += 256) o[c] = in ? in[c] : zero;
  }
}

// dst[S[i], :] = src[i, :] for i < U: the compacted gradient rows go to their neurons' rows.
__global__ __launch_bounds__(256) void scatter_rows_kernel(const uint16_t* __restrict__ src,
                                                           const int32_t* __restrict__ S,
                                                           const int32_t* __restrict__ n_S, int N, int d, int cap,
                                                           uint16_t* __restrict__ dst) {
  const int U = max(0, min(*n_S, cap));
  for (int i = blockIdx.x; i < U; i += gridDim.x) {
    const int j = S[i];
    if ((unsigned)j >= (unsigned)N) continue;
    const u32x4* in = reinterpret_cast<const u32x4*>(src + (size_t)i * d);
    u32x4* o = reinterpret_cast<u32x4*>(dst + (size_t)j * d);
    for (int c = threadIdx.x; c < d / 8; c += 256) o[c] = in[c];
  }
}

}  // namespace meft
