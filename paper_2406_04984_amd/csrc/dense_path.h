// The block-dense formulation of the layer for bf16: because every token's selected neurons lie
// in its top_e blocks, each stage is a contraction between the tokens routed to a block and that
// block's rows, with the activations of unselected (token, neuron) pairs set to zero.  With
// top_k / (top_e * block_size) around 1/16 the matrix cores do this faster than per-pair row
// gathers can move their bytes, and every operand panel is read from HBM once.
//
// Per block b with its token group G_b (slots, ascending token order), block_size neurons, hidden d:
//   scores   S [G_b, bs] = h[G_b, :] . K_b^T                     (Eq. 6)            KC GEMM
//   forward  part[G_b, d] = A'[G_b, bs] . V_b  (stored bf16)     (Eq. 4, one block) NC GEMM
//            out[t, :] = sum over the token's blocks of part      (row reduce)
//   backward G [G_b, bs] = dOut[G_b, :] . V_b^T, DS' = G * [A' > 0]                 KC GEMM
//            dhpart[G_b, d] = DS'[G_b, bs] . K_b ; dh = row reduce                 NC GEMM
//            dV_b[bs, d] = A'^T[bs, G_b] . dOut[G_b, :]                            NC GEMM
//            dK_b[bs, d] = DS'^T[bs, G_b] . h[G_b, :]                              NC GEMM
// A'[slot, r] = bf16(act) where neuron r of the block is selected by the slot's token, else 0.
#pragma once
#include "gemm_mfma.h"
#include "select.h"

namespace meft {

__device__ __forceinline__ int round_up64(int v) { return (v + 63) & ~63; }

// entries (all 0, a valid token) behind the last slot of tok_of_slot, so that look-ups for the padded tail of a
// group's contraction and the one-k-tile-ahead prefetch of row numbers stay inside the array
constexpr int kSlotPad = 192;

// ---- problem policies for gemm_mfma_kernel ----------------------------------------------------

// Router scores (Eq. 5): p[T, n_blocks] = h . Wg^T, one group.  The problem is skinny (n_blocks columns), so
// the contraction is split `ksplit` ways over workgroups to fill the chip; split s writes its partial
// scores to p + s*T*n_blocks and the top-e kernel adds the partials in a fixed order.
struct ProbRouter {
  static constexpr int kTM = kTMNeu, kSA = 3, kSB = 3, kCW = 4;   // 128-row tiles: twice as many workgroups for a small problem
  static constexpr int kLoaders = 2;
  static constexpr bool kAMC = false;
  static constexpr bool kBNC = false;
  static constexpr bool kRowIdsInMemory = false;
  const uint16_t* h; const uint16_t* Wg; float* p;
  int T, d, B, ksplit;
  uint32_t a_bytes, b_bytes; bool buf;
  __device__ const uint16_t* a_base() const { return h; }
  __device__ const uint16_t* b_base() const { return Wg; }
  __device__ bool locate(int wg, TileCoord& tc) const {
    const int tn = (B + kTN - 1) / kTN;
    const int ks = wg % ksplit, w = wg / ksplit, mt = w / tn;
    tc.g = 0; tc.m0 = mt * kTM; tc.n0 = (w - mt * tn) * kTN; tc.Mrows = T; tc.Ncols = B;
    tc.nk = d / kTK / ksplit; tc.slot0 = 0; tc.aux = ks;
    return tc.m0 < T;
  }
  __device__ const uint16_t* a_row(const TileCoord& tc, int m) const {
    return h + (size_t)(m < T ? m : T - 1) * d + (size_t)tc.aux * tc.nk * kTK;
  }
  __device__ const uint16_t* b_row(const TileCoord& tc, int n) const {
    return Wg + (size_t)(n < B ? n : B - 1) * d + (size_t)tc.aux * tc.nk * kTK;
  }
  __device__ int out_cols(const TileCoord&) const { return B; }
  static constexpr bool kAux = false;
  static constexpr bool kOutBf16 = false;
  __device__ int row_tag(const TileCoord&, int m) const { return m < T ? 1 : 0; }
  static constexpr bool kRowsLinear = true;
  __device__ int out_ld(const TileCoord&) const { return B; }
  __device__ size_t row_off(const TileCoord& tc, int, int m) const { return ((size_t)tc.aux * T + m) * B; }
  __device__ void store2(size_t at, int n, float v0, float v1, uint32_t) const {
    if (n < B) p[at] = v0;
    if (n + 1 < B) p[at + 1] = v1;
  }
};

// Token-major, B contiguous along k: rows = tokens of the group (gathered through perm), columns =
// the block's neurons.  What is written depends on MODE:
//   kTokScores: key scores, fp32, by entry.
//   kTokMasked: the activation gradient, masked by A' > 0, bf16, slot-major (DS').
//   kTokRelu:   ReLU of the scores (Eq. 2 without a selection: the batch-union evaluation of Algorithm 1), bf16,
//               written through the same pointer.
constexpr int kTokScores = 0, kTokMasked = 1, kTokRelu = 2;

template <int MODE>
struct ProbTokKC {
  static constexpr int kTM = kTMTok, kSA = MEFT_TOK_SA, kSB = MEFT_TOK_SB, kCW = 4;
  static constexpr int kLoaders = 2;
  static constexpr bool kAMC = false;
  static constexpr bool kBNC = false;
  static constexpr bool kRowIdsInMemory = false;
  const uint16_t* X;          // h (scores) or dOut (activation gradient), [T, d]
  const uint16_t* W;          // K or V, [N, d]
  const int32_t* perm; const int32_t* group_off;
  TokenSched sched;
  int big_only;               // 1: the groups of at most small_rows tokens are left to the per-pair kernels
  int e, bs, bsp, d;
  float* sc;                  // kTokScores: [T*e, bs]
  const uint16_t* Ap;         // kTokMasked: A' [slots, bsp]
  uint16_t* DS;               // kTokMasked / kTokRelu: [slots, bsp]; columns bs..bsp are written as zeros
  uint32_t a_bytes, b_bytes; bool buf;
  __device__ const uint16_t* a_base() const { return X; }
  __device__ const uint16_t* b_base() const { return W; }
  __device__ bool locate(int wg, TileCoord& tc) const {
    int mt, nt, rows;
    if (!locate_token_tile(sched, group_off, wg, (bs + kTN - 1) / kTN, big_only != 0, tc.g, mt, nt, tc.slot0, rows))
      return false;
    tc.m0 = mt * kTM; tc.n0 = nt * kTN; tc.Mrows = rows; tc.Ncols = bs; tc.nk = d / kTK;
    return true;
  }
  __device__ const uint16_t* a_row(const TileCoord& tc, int m) const {
    const int ent = perm[tc.slot0 + (m < tc.Mrows ? m : tc.Mrows - 1)];
    return X + (size_t)(ent / e) * d;
  }
  __device__ const uint16_t* b_row(const TileCoord& tc, int n) const {
    return W + ((size_t)tc.g * bs + (n < bs ? n : bs - 1)) * d;
  }
  __device__ int out_cols(const TileCoord&) const { return MODE == kTokScores ? bs : bsp; }
  // scores: the row's entry number + 1; otherwise 1 for a row of the group
  __device__ int row_tag(const TileCoord& tc, int m) const {
    if (m >= tc.Mrows) return 0;
    return MODE == kTokScores ? perm[tc.slot0 + m] + 1 : 1;
  }
  static constexpr bool kRowsLinear = MODE != kTokScores;   // the score rows go by entry
  __device__ int out_ld(const TileCoord&) const { return bsp; }
  __device__ size_t row_off(const TileCoord& tc, int tag, int m) const {
    return MODE == kTokScores ? (size_t)(tag - 1) * bs : (size_t)(tc.slot0 + m) * bsp;
  }
  // kTokMasked: the two activations of A' that decide whether the two gradient values are kept
  static constexpr bool kAux = MODE == kTokMasked;
  __device__ uint32_t load_aux(const TileCoord& tc, int m, int n) const {
    const int mm = m < tc.Mrows ? m : tc.Mrows - 1, nn = n < bsp ? n : bsp - 2;
    return *reinterpret_cast<const uint32_t*>(Ap + (size_t)(tc.slot0 + mm) * bsp + nn);
  }
  static constexpr bool kOutBf16 = MODE != kTokScores;
  __device__ void store2(size_t at, int n, float v0, float v1, uint32_t) const {   // kTokScores
    if ((bs & 1) == 0) {   // rows are 8-byte aligned and n + 1 < bs whenever n < bs
      if (n < bs) *reinterpret_cast<f32x2_hw*>(sc + at) = f32x2_hw{v0, v1};
    } else {
      if (n < bs) sc[at] = v0;
      if (n + 1 < bs) sc[at + 1] = v1;
    }
  }
  __device__ void store_pk(size_t at, int n, uint32_t pk, uint32_t mk) const {   // kTokMasked, kTokRelu
    if (n >= bsp) return;   // bsp is even: n + 1 < bsp
    // a half is kept where the deciding value is positive: sign bit clear and not zero
    uint32_t keep = 0u;
    if constexpr (MODE == kTokMasked) {
      // decided by the activations (A' holds zeros in the columns bs..bsp)
      if ((mk & 0x7FFFu) != 0u && (mk & 0x8000u) == 0u) keep |= 0xFFFFu;
      if ((mk & 0x7FFF0000u) != 0u && (mk & 0x80000000u) == 0u) keep |= 0xFFFF0000u;
    } else {
      // ReLU of the value itself; columns beyond the block (computed from clamped operand rows) are zero
      if (n < bs && (pk & 0x7FFFu) != 0u && (pk & 0x8000u) == 0u) keep |= 0xFFFFu;
      if (n + 1 < bs && (pk & 0x7FFF0000u) != 0u && (pk & 0x80000000u) == 0u) keep |= 0xFFFF0000u;
    }
    *reinterpret_cast<uint32_t*>(DS + at) = pk & keep;
  }
};

// Token-major, B contiguous along n: part[slot, :] = A[slot, 0:bs] . W_b   (W = V: forward value sum;
// W = K: dh).  A is slot-major [slots, bsp] with zero padding in columns bs..bsp.
struct ProbTokNC {
  static constexpr int kTM = kTMTok, kSA = MEFT_TOK_SA, kSB = MEFT_TOK_SB, kCW = 4;
  static constexpr int kLoaders = 4;   // measured: 0.375 -> 0.339 ms (value sum) against two
  static constexpr bool kAMC = false;
  static constexpr bool kBNC = true;
  static constexpr bool kRowIdsInMemory = false;
  const uint16_t* A;          // A' or DS'
  const uint16_t* W;          // V or K, [N, d]
  const int32_t* group_off;
  TokenSched sched;
  int big_only;               // 1: the groups of at most small_rows tokens are left to the per-pair kernels
  int bs, bsp, d;
  uint16_t* part;             // [slots, d] bf16: one block's contribution to a token's row
  uint32_t a_bytes, b_bytes; bool buf;
  __device__ const uint16_t* a_base() const { return A; }
  __device__ const uint16_t* b_base() const { return W; }
  __device__ bool locate(int wg, TileCoord& tc) const {
    int mt, nt, rows;
    if (!locate_token_tile(sched, group_off, wg, (d + kTN - 1) / kTN, big_only != 0, tc.g, mt, nt, tc.slot0, rows))
      return false;
    tc.m0 = mt * kTM; tc.n0 = nt * kTN; tc.Mrows = rows; tc.Ncols = d; tc.nk = bsp / kTK;
    return true;
  }
  __device__ const uint16_t* a_row(const TileCoord& tc, int m) const {
    return A + (size_t)(tc.slot0 + (m < tc.Mrows ? m : tc.Mrows - 1)) * bsp;
  }
  __device__ int b_row_ids(const TileCoord& tc, int k) const { return tc.g * bs + (k < bs ? k : bs - 1); }
  // the 64 rows from k0 on are consecutive rows of W (no clamping inside the k tile)
  __device__ bool b_rows_linear(const TileCoord&, int k0) const { return k0 + kTK <= bs; }
  __device__ const uint16_t* b_row_ptr(int row) const { return W + (size_t)row * d; }
  __device__ int out_cols(const TileCoord&) const { return d; }   // d % 64 == 0
  static constexpr bool kAux = false;
  __device__ int row_tag(const TileCoord& tc, int m) const { return m < tc.Mrows ? 1 : 0; }
  static constexpr bool kRowsLinear = true;
  __device__ int out_ld(const TileCoord&) const { return d; }
  __device__ size_t row_off(const TileCoord& tc, int, int m) const { return (size_t)(tc.slot0 + m) * d; }
  static constexpr bool kOutBf16 = true;
  __device__ void store_pk(size_t at, int, uint32_t pk, uint32_t) const { *reinterpret_cast<uint32_t*>(part + at) = pk; }
};

// Neuron-major, both operands indexed by the contraction index (slot) in their rows:
//   G_b[bs, d] = sum over the slots of group b of A[slot, 0:bs]^T . X[token(slot), :]
// (A = A', X = dOut: dV;  A = DS', X = h: dK).  A is the slot-major matrix the token-major kernels write and read,
// so no transposed copy of the activations exists.  The contraction length is padded to 64: the padding rows of A
// come from a row of zeros that the workspace keeps in front of the activation matrices, those of X are any valid
// rows.  Only rows whose neuron is touched are written.
// TM = 256: 256 x 256 tiles, eight compute waves that request their operands themselves, two slots per ring; TM = 128:
// 128 x 256 with four compute and four loader waves (measured: 0.425 -> 0.388 ms (dV) against two).  The host takes
// the larger tile where it does not add rows beyond the block (neu_tile_rows).
template <int TM>
struct ProbNeuTN {
  static constexpr int kTM = TM, kSA = TM == 256 ? 2 : 3, kSB = kSA, kCW = TM == 256 ? 8 : 4;
  static constexpr int kLoaders = TM == 256 ? 0 : 4;
  static constexpr bool kAMC = true;
  static constexpr bool kBNC = true;
  static constexpr bool kRowIdsInMemory = true;
  const uint16_t* A;          // [slots, bsp]
  int zrow;                   // number of a row of bsp zeros, counted from A's row 0 (it lies before A: negative)
  const uint16_t* X;          // [T, d]
  const int32_t* group_off; const int32_t* tok_of_slot;
  const int32_t* flag;        // [N] > 0 where some token selected the neuron
  TokenSched sched;           // only the group lists are used: every group has the same number of tiles
  int big_only;               // 1: the groups of at most small_rows tokens are left to the per-pair kernels
  int bs, bsp, d;
  uint16_t* G;                // dV or dK [N, d]
  uint32_t a_bytes, b_bytes; bool buf;
  __device__ const uint16_t* a_base() const { return A + (int64_t)zrow * bsp; }   // the row of zeros lies lowest
  __device__ const uint16_t* b_base() const { return X; }
  __device__ bool locate(int wg, TileCoord& tc) const {
    const int tm = (bs + kTM - 1) / kTM, tn = (d + kTN - 1) / kTN;
    const int x = wg & (kXcd - 1), local = wg >> 3;
    int gi, w;
    if (as_const(sched.len)[kXcd] != 0) {   // split lists: this XCD takes the tiles x, x + 8, ... of every group
      const int mine = tm * tn > x ? (tm * tn - x + kXcd - 1) / kXcd : 0;
      if (mine == 0) return false;
      gi = local / mine;
      w = x + kXcd * (local - gi * mine);
    } else {
      gi = local / (tm * tn);
      w = local - gi * (tm * tn);
    }
    if (gi >= as_const(sched.len)[big_only ? kXcd + 1 + x : x]) return false;
    tc.g = as_const(sched.grp)[(size_t)x * sched.cap + gi].x;
    tc.slot0 = as_const(group_off)[tc.g];
    const int rows = as_const(group_off)[tc.g + 1] - tc.slot0;   // > 0: the lists hold non-empty groups only
    // m tiles vary fastest: the tiles that share the gathered rows of one n tile run together
    tc.m0 = (w % tm) * kTM; tc.n0 = (w / tm) * kTN; tc.Mrows = bs; tc.Ncols = d; tc.nk = round_up64(rows) / kTK;
    tc.aux = rows;
    return true;
  }
  __device__ const uint16_t* a_mat() const { return A; }
  __device__ int a_cols(const TileCoord&) const { return bsp; }
  __device__ int a_krow(const TileCoord& tc, int k) const { return k < tc.aux ? tc.slot0 + k : zrow; }
  // tok_of_slot is padded by kSlotPad valid entries, which covers the padded contraction length
  __device__ const int32_t* b_row_id_src(const TileCoord& tc, int k0) const { return tok_of_slot + tc.slot0 + k0; }
  __device__ const uint16_t* b_row_ptr(int row) const { return X + (size_t)row * d; }
  __device__ int out_cols(const TileCoord&) const { return d; }   // d % 64 == 0
  __device__ int row_tag(const TileCoord& tc, int m) const {
    return (m < bs && flag[(size_t)tc.g * bs + m] > 0) ? 1 : 0;
  }
  static constexpr bool kAux = false;
  static constexpr bool kRowsLinear = true;
  __device__ int out_ld(const TileCoord&) const { return d; }
  __device__ size_t row_off(const TileCoord& tc, int, int m) const { return ((size_t)tc.g * bs + m) * d; }
  static constexpr bool kOutBf16 = true;
  __device__ void store_pk(size_t at, int, uint32_t pk, uint32_t) const { *reinterpret_cast<uint32_t*>(G + at) = pk; }
};

// ---- helper kernels ----------------------------------------------------------------------------

// Backward: the distinct blocks of a token's selected neurons, ascending, padded with -1 to top_e
// entries.  One wave per token; block ids go through an LDS bitmap.  More than top_e distinct blocks
// is a caller error: the extra blocks are dropped (their pairs then contribute nothing).
__global__ __launch_bounds__(64) void blocks_from_idx_kernel(const int32_t* __restrict__ idx, int k, int N, int bs,
                                                             int n_blocks, int e, int32_t* __restrict__ sblk) {
  extern __shared__ uint32_t s_bits[];  // [ceil(n_blocks/32)]
  const int t = blockIdx.x, lane = threadIdx.x;
  const int words = (n_blocks + 31) / 32;
  for (int w = lane; w < words; w += 64) s_bits[w] = 0u;
  __syncthreads();
  for (int i = lane; i < k; i += 64) {
    const int b = clampi(idx[(size_t)t * k + i], 0, N - 1) / bs;
    atomicOr(&s_bits[b >> 5], 1u << (b & 31));
  }
  __syncthreads();
  int base = 0;
  for (int w0 = 0; w0 < words; w0 += 64) {
    const int w = w0 + lane;
    uint32_t bits = w < words ? s_bits[w] : 0u;
    const int c = __popc(bits);
    const int incl = wave_incl_scan(c);
    int pos = base + incl - c;
    while (bits) {
      const int b = __ffs(bits) - 1;
      bits &= bits - 1;
      if (pos < e) sblk[(size_t)t * e + pos] = w * 32 + b;
      ++pos;
    }
    base += __shfl(incl, 63, 64);
  }
  for (int q = base + lane; q < e; q += 64) sblk[(size_t)t * e + q] = -1;
}

// After fill_groups: slot -> token (padded by kSlotPad valid entries) and entry -> slot.
__global__ __launch_bounds__(256) void slot_maps_kernel(const int32_t* __restrict__ perm,
                                                        const int32_t* __restrict__ group_off, int n_groups, int e,
                                                        int32_t* __restrict__ tok_of_slot,
                                                        int32_t* __restrict__ slot_of_ent) {
  const int n_slots = group_off[n_groups];
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n_slots) {
    const int ent = perm[i];
    tok_of_slot[i] = ent / e;
    slot_of_ent[ent] = i;
  } else if (i < n_slots + kSlotPad) {
    tok_of_slot[i] = 0;
  }
}

// Backward: the token's dense activation rows A'[slot, 0:bsp] (one per block it uses, slot-major, bf16(act) where
// a neuron was selected, else 0) from the saved (idx, act), and the touched flags (zero before).  One workgroup
// per token: the rows are put together in LDS and written whole, 16 bytes per thread and step.
// Dynamic LDS: e * bsp * 2 bytes.
__global__ __launch_bounds__(256) void act_rows_kernel(const int32_t* __restrict__ idx, const float* __restrict__ act,
                                                       int k, int N, int bs, int bsp, int e,
                                                       const int32_t* __restrict__ sblk,
                                                       const int32_t* __restrict__ slot_of_ent,
                                                       uint16_t* __restrict__ Ap, int32_t* __restrict__ flag) {
  extern __shared__ __attribute__((aligned(16))) uint16_t s_rows[];   // [e][bsp]
  const int t = blockIdx.x, tid = threadIdx.x;
  const int words = e * bsp / 8;   // 16-byte words
  u32x4* s4 = reinterpret_cast<u32x4*>(s_rows);
  for (int w = tid; w < words; w += 256) s4[w] = u32x4{0u, 0u, 0u, 0u};
  __syncthreads();
  for (int p = tid; p < k; p += 256) {
    const int j = clampi(idx[(size_t)t * k + p], 0, N - 1);
    const int b = j / bs, r = j - b * bs;
    flag[j] = 1;
    int q = -1;
    for (int z = 0; z < e; ++z)
      if (sblk[(size_t)t * e + z] == b) { q = z; break; }
    if (q >= 0) s_rows[q * bsp + r] = (uint16_t)f32_to_bf16_bits(act[(size_t)t * k + p]);
  }
  __syncthreads();
  const int wpr = bsp / 8;   // words per row
  for (int w = tid; w < words; w += 256) {
    const int q = w / wpr, c = w - q * wpr;
    if (sblk[(size_t)t * e + q] < 0) continue;   // fewer than e blocks in use: no slot
    reinterpret_cast<u32x4*>(Ap + (size_t)slot_of_ent[t * e + q] * bsp)[c] = s4[w];
  }
}

// out[t, :] = sum over the token's entries of part[slot(entry), :] (bf16 partials, fp32 sum), rounded to bf16.
template <int NV>
__global__ __launch_bounds__(256) void reduce_parts_kernel(const uint16_t* __restrict__ part,
                                                           const int32_t* __restrict__ sblk,
                                                           const int32_t* __restrict__ slot_of_ent, int d, int e,
                                                           uint16_t* __restrict__ out) {
  const int t = blockIdx.x, tid = threadIdx.x, nthr = blockDim.x;
  float acc[NV][8];
#pragma unroll
  for (int v = 0; v < NV; ++v)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[v][c] = 0.f;
  for (int q = 0; q < e; ++q) {
    if (sblk[(size_t)t * e + q] < 0) continue;
    const bf16_t* row = reinterpret_cast<const bf16_t*>(part) + (size_t)slot_of_ent[t * e + q] * d;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col = (tid + v * nthr) * 8;
      if (col < d) {
        float x[8];
        Vec8<bf16_t>::load(row + col, x);
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[v][c] += x[c];
      }
    }
  }
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int col = (tid + v * nthr) * 8;
    if (col < d) Vec8<bf16_t>::store(reinterpret_cast<bf16_t*>(out) + (size_t)t * d + col, acc[v]);
  }
}

// touched = ascending ids with flag > 0, in two launches over chunks of kFlagChunk flags:
// per-chunk counts, then every chunk sums the counts before it and writes its ids in order.
constexpr int kFlagChunk = 2048;

__global__ __launch_bounds__(256) void count_flags_kernel(const int32_t* __restrict__ flag, int N,
                                                          int32_t* __restrict__ chunk_cnt) {
  __shared__ int s_w[4];
  const int j0 = blockIdx.x * kFlagChunk + threadIdx.x * (kFlagChunk / 256);
  int f = 0;
#pragma unroll
  for (int z = 0; z < kFlagChunk / 256; ++z)
    if (j0 + z < N) f += flag[j0 + z] > 0;
  int tot;
  block_excl_scan_256(f, s_w, tot);
  if (threadIdx.x == 0) chunk_cnt[blockIdx.x] = tot;
}

__global__ __launch_bounds__(256) void compact_flags_kernel(const int32_t* __restrict__ flag, int N,
                                                            const int32_t* __restrict__ chunk_cnt,
                                                            int32_t* __restrict__ touched,
                                                            int32_t* __restrict__ n_touched) {
  __shared__ int s_w[4];
  int before = 0;
  for (int c = threadIdx.x; c < (int)blockIdx.x; c += 256) before += chunk_cnt[c];
  int base;
  block_excl_scan_256(before, s_w, base);   // base = number of touched ids in earlier chunks
  const int j0 = blockIdx.x * kFlagChunk + threadIdx.x * (kFlagChunk / 256);
  int f = 0;
#pragma unroll
  for (int z = 0; z < kFlagChunk / 256; ++z)
    if (j0 + z < N) f += flag[j0 + z] > 0;
  int tot;
  int pos = base + block_excl_scan_256(f, s_w, tot);
#pragma unroll
  for (int z = 0; z < kFlagChunk / 256; ++z)
    if (j0 + z < N && flag[j0 + z] > 0) touched[pos++] = j0 + z;
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 255) *n_touched = base + tot;
}

}  // namespace meft
