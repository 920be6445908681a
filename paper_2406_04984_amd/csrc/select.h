// Selection kernels: top-e blocks per token from router scores, dispatch of (token, block)
// entries to per-block groups, and top-k neurons per token from the candidate scores.
// Ties go to the lower index in both selections; +0 and -0 tie.
#pragma once
#include "common.h"

namespace meft {

// ---------------------------------------------------------------------------------------------
// Top-e blocks (Algorithm 1: tau <- TopK(p, number of experts)).  One wave per token.  The row of
// B scores sits in LDS as ordered keys; e rounds of a wave-wide arg-max, the winner is retired
// by zeroing its key (a live key is never 0 for finite scores).  Output order: score descending,
// block id ascending.  The scores may arrive as n_part partial sums, part_stride floats apart.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void route_topk_kernel(const float* __restrict__ p, int n_part, size_t part_stride,
                                                        const float* __restrict__ bias, int B, int e,
                                                        int32_t* __restrict__ block_idx,
                                                        float* __restrict__ block_score) {
  extern __shared__ uint32_t s_key[];
  const int t = blockIdx.x, lane = threadIdx.x;
  const float* row = p + (size_t)t * B;
  for (int b = lane; b < B; b += kWave) {
    float v = row[b];
    for (int s = 1; s < n_part; ++s) v += row[s * part_stride + b];   // partial scores of a split contraction
    if (bias) v += bias[b];
    s_key[b] = order_key(v);
  }
  __syncthreads();
  for (int q = 0; q < e; ++q) {
    unsigned long long best = 0ull;
    for (int b = lane; b < B; b += kWave) {
      const uint32_t k = s_key[b];
      const unsigned long long c = ((unsigned long long)k << 32) | (uint32_t)(0x7FFFFFFF - b);
      if (k != 0u && c > best) best = c;
    }
    best = wave_max_u64(best);
    const int bsel = 0x7FFFFFFF - (int)(uint32_t)(best & 0xFFFFFFFFull);
    if (lane == 0) {
      block_idx[(size_t)t * e + q] = bsel;
      if (block_score) block_score[(size_t)t * e + q] = key_to_float((uint32_t)(best >> 32));
      s_key[bsel] = 0u;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// Dispatch.  (1) per token, the e block ids sorted ascending (so that the concatenated candidate
// order of a token is its ascending neuron-id order); ids are clamped into [0, B).
// ---------------------------------------------------------------------------------------------
__global__ void sort_blocks_kernel(const int32_t* __restrict__ block_idx, int T, int e, int B,
                                   int32_t* __restrict__ sblk) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const int32_t* src = block_idx + (size_t)t * e;
  int32_t* dst = sblk + (size_t)t * e;
  for (int i = 0; i < e; ++i) {  // insertion sort; e is small
    const int v = clampi(src[i], 0, B - 1);
    int z = i - 1;
    while (z >= 0 && dst[z] > v) { dst[z + 1] = dst[z]; --z; }
    dst[z + 1] = v;
  }
}

// exclusive scan of one int per thread over a 256-thread workgroup; returns the total in `total`
__device__ __forceinline__ int block_excl_scan_256(int v, int* s_wave /*[4]*/, int& total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int incl = wave_incl_scan(v);
  if (lane == 63) s_wave[w] = incl;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) base += (i < w) ? s_wave[i] : 0;
  total = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
  __syncthreads();
  return base + incl - v;
}

// exclusive scan of one int per thread over a 1024-thread workgroup
__device__ __forceinline__ int block_excl_scan_1024(int v, int* s_wave /*[16]*/, int& total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int incl = wave_incl_scan(v);
  if (lane == 63) s_wave[w] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) { const int x = s_wave[i]; base += (i < w) ? x : 0; tot += x; }
  total = tot;
  __syncthreads();
  return base + incl - v;
}

// number of entries equal to b among sblk[i0, i1); 16-byte loads where the range allows
__device__ __forceinline__ int count_eq(const int32_t* __restrict__ sblk, int i0, int i1, int b) {
  int c = 0, i = i0;
  for (; i < i1 && (i & 3); ++i) c += (sblk[i] == b);
  for (; i + 4 <= i1; i += 4) {
    const int4 v = *reinterpret_cast<const int4*>(sblk + i);
    c += (v.x == b) + (v.y == b) + (v.z == b) + (v.w == b);
  }
  for (; i < i1; ++i) c += (sblk[i] == b);
  return c;
}

// (2) cnt[b] = number of entries of block b.  One workgroup of 1024 threads per block; every thread counts
// a contiguous chunk.
__global__ __launch_bounds__(1024) void count_blocks_kernel(const int32_t* __restrict__ sblk, int n_ent,
                                                            int32_t* __restrict__ cnt) {
  __shared__ int s_w[16];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int chunk = (n_ent + 1023) / 1024;
  const int i0 = min(n_ent, tid * chunk), i1 = min(n_ent, i0 + chunk);
  int tot;
  block_excl_scan_1024(count_eq(sblk, i0, i1, b), s_w, tot);
  if (tid == 0) cnt[b] = tot;
}

// (3) group_off / tile_off (prefix sums over blocks of cnt and of ceil(cnt/BM)) and the stable
// fill perm[group_off[b] + rank] = entry, entries of a block in ascending entry order.
__global__ __launch_bounds__(1024) void fill_groups_kernel(const int32_t* __restrict__ sblk, int n_ent,
                                                           const int32_t* __restrict__ cnt, int B, int BM,
                                                           int32_t* __restrict__ group_off,
                                                           int32_t* __restrict__ tile_off,
                                                           int32_t* __restrict__ perm) {
  __shared__ int s_w[16];
  const int b = blockIdx.x, tid = threadIdx.x;
  int go = 0, to = 0;
  for (int i = tid; i < b; i += 1024) { const int c = cnt[i]; go += c; to += (c + BM - 1) / BM; }
  int tot_g, tot_t;
  block_excl_scan_1024(go, s_w, tot_g);
  block_excl_scan_1024(to, s_w, tot_t);
  if (tid == 0) {
    group_off[b] = tot_g;
    tile_off[b] = tot_t;
    if (b == B - 1) {
      group_off[B] = tot_g + cnt[b];
      tile_off[B] = tot_t + (cnt[b] + BM - 1) / BM;
    }
  }
  const int chunk = (n_ent + 1023) / 1024;
  const int i0 = min(n_ent, tid * chunk), i1 = min(n_ent, i0 + chunk);
  int tot;
  int rank = block_excl_scan_1024(count_eq(sblk, i0, i1, b), s_w, tot);
  for (int i = i0; i < i1; ++i)
    if (sblk[i] == b) perm[tot_g + rank++] = i;
}

// ---------------------------------------------------------------------------------------------
// Top-k neurons of one token (Eq. 1 applied to the candidates of the chosen blocks).  One workgroup per token.
// The C candidate scores (fp32, candidate position = ascending neuron id) are turned into ordered 32-bit keys; a
// most-significant-digit radix select (4 passes of 8 bits) finds the key of the k-th largest and how many of its
// equals still belong; then one ordered sweep emits the selected positions in ascending order: all keys above
// the threshold, and the first `need` positions that equal it.  With Ap != nullptr it also writes the token's
// dense activation rows (one per chosen block, slot-major, zero where not selected).
//
// The token's keys live in registers: thread `tid` owns the KPT consecutive candidate
// positions tid*KPT .. tid*KPT + KPT - 1 (256 * KPT >= C), reads them once from global memory and keeps their
// ordered keys for all histogram passes, the ordered sweep and the dense activation rows.  LDS holds the 256-bin
// histogram (a thread adds runs of equal digits with one atomic, which takes most of the same-address conflicts out
// of the first pass: sign and exponent bits, a handful of distinct digits) and the staging arrays of the outputs.
// The passes stop as soon as a whole bucket is selected (usually after three).  The kernel is bound by its
// instruction count, not by memory: nested branches, per-position integer divisions and nearly empty global stores
// were what it spent its time on.
// ---------------------------------------------------------------------------------------------
constexpr int kTopkEmitLds = 1024;   // selections per token that go through LDS in one round

// Waves per SIMD that the register allocation aims at.  Up to 16 keys per thread seven (72 registers): measured
// best at 16 keys (0.095 ms against 0.102 with the 86 registers the compiler takes unasked, 0.118 at six waves, 0.123
// at eight); with more keys per thread as many as hold them without spilling.
constexpr int topk_waves(int kpt) { return kpt <= 16 ? 7 : (kpt <= 32 ? 4 : 2); }

template <int KPT, bool kFull>   // kFull: C == 256 * KPT, every position holds a candidate
__global__ __launch_bounds__(256, topk_waves(KPT)) void topk_select_reg_kernel(const float* __restrict__ sc,
                                                              const int32_t* __restrict__ sblk, int C, int bs,
                                                              int e, int k, int32_t* __restrict__ idx,
                                                              float* __restrict__ act,
                                                              const int32_t* __restrict__ slot_of_ent, int bsp,
                                                              uint16_t* __restrict__ Ap) {
  __shared__ int s_hist[256];
  __shared__ int s_w[4];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need;
  __shared__ int s_done;
  // staging for the outputs: the sweep reaches a selected position in a few lanes at a time, and that many nearly
  // empty global stores would cost more than everything before them
  __shared__ int s_idx[kTopkEmitLds];
  __shared__ float s_act[kTopkEmitLds];
  const int t = blockIdx.x, tid = threadIdx.x;
  const float* row = sc + (size_t)t * C;
  const int p0 = tid * KPT;
  uint32_t key[KPT];   // 0 for positions beyond C: below every real key, never selected
  if ((C & 3) == 0 && (KPT & 3) == 0) {
#pragma unroll
    for (int z = 0; z < KPT; z += 4) {
      if (p0 + z < C) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(row + p0 + z);
        key[z] = order_key(v.x); key[z + 1] = order_key(v.y); key[z + 2] = order_key(v.z); key[z + 3] = order_key(v.w);
      } else {
        key[z] = key[z + 1] = key[z + 2] = key[z + 3] = 0u;
      }
    }
  } else {
#pragma unroll
    for (int z = 0; z < KPT; ++z) key[z] = p0 + z < C ? order_key(row[p0 + z]) : 0u;
  }
  if (tid == 0) { s_prefix = 0u; s_need = k; s_done = 0; }
  __syncthreads();

  for (int shift = 24; shift >= 0; shift -= 8) {
    s_hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = s_prefix;
    const uint32_t himask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
    // A thread adds a run of equal digits with one atomic (that takes most of the same-address conflicts out of the
    // first pass).  Written without nested branches: a run ends where a matching key has another digit; the first
    // "run" is an empty one of digit 0, whose add of zero is harmless.
    uint32_t cur = 0u;
    int cnt = 0;
#pragma unroll
    for (int z = 0; z < KPT; ++z) {
      const bool m = (kFull || p0 + z < C) && (key[z] & himask) == prefix;
      const uint32_t dgt = (key[z] >> shift) & 255u;
      const bool start = m && dgt != cur;
      if (start) atomicAdd(&s_hist[cur], cnt);
      cnt = (start ? 0 : cnt) + (m ? 1 : 0);
      cur = start ? dgt : cur;
    }
    atomicAdd(&s_hist[cur], cnt);
    __syncthreads();
    // thread `tid` owns digit 255 - tid, so that an exclusive scan counts the larger digits
    const int digit = 255 - tid;
    const int h = s_hist[digit];
    int tot;
    const int above = block_excl_scan_256(h, s_w, tot);
    const int need = s_need;
    __syncthreads();
    if (above < need && need <= above + h) {
      const uint32_t found = prefix | ((uint32_t)digit << shift);
      if (h == need - above && shift > 0 && found != 0u) {
        // every key with these leading digits is selected: "greater than found - 1" says the same as a threshold
        // with all digits known, and the remaining passes are not needed (the usual case after three passes)
        s_prefix = found - 1u;
        s_need = 0;
        s_done = 1;
      } else {
        s_prefix = found;
        s_need = need - above;
      }
    }
    __syncthreads();
    if (s_done) break;
  }
  const uint32_t thr = s_prefix;
  const int need = s_need;  // how many keys equal to thr are selected

  int ngt = 0, neq = 0;
#pragma unroll
  for (int z = 0; z < KPT; ++z) {
    ngt += key[z] > thr;               // padding keys are 0 <= thr's lower bound: never greater
    neq += (kFull || p0 + z < C) && key[z] == thr;
  }
  int tot;
  const int packed = block_excl_scan_256(ngt | (neq << 16), s_w, tot);  // C <= 12288 < 2^15
  int gt_before = packed & 0xFFFF, eq_before = packed >> 16;
  uint32_t sel = 0u;   // bit z: position p0 + z is selected (KPT <= 32 bits used per word)
  uint32_t sel_hi = 0u;
  const int q0 = p0 / bs, r0 = p0 - q0 * bs;   // block entry and row of the thread's first position
  // The selected (position, key) pairs go to their output slots through LDS, kTopkEmitLds slots at a time (one round
  // unless top_k is larger than that); the write-out turns a position into a neuron number and a key into max(score, 0).
  for (int base = 0; base < k; base += kTopkEmitLds) {
    int gt_run = gt_before, eq_run = eq_before;
#pragma unroll
    for (int z = 0; z < KPT; ++z) {
      const bool in = kFull || p0 + z < C;
      const bool gt = key[z] > thr, eq = in && key[z] == thr;
      if (gt || (eq && eq_run < need)) {
        const int slot = gt_run + min(eq_run, need) - base;  // selected positions before this one
        if ((unsigned)slot < (unsigned)kTopkEmitLds) {
          s_idx[slot] = p0 + z;
          s_act[slot] = __uint_as_float(key[z]);
        }
        if (z < 32) sel |= 1u << z; else sel_hi |= 1u << (z - 32);
      }
      gt_run += gt;
      eq_run += eq;
    }
    __syncthreads();
    const int n_out = min(k - base, kTopkEmitLds);
    for (int j = tid; j < n_out; j += 256) {
      const int i = s_idx[j], q = i / bs;
      const float v = key_to_float(__float_as_uint(s_act[j]));
      idx[(size_t)t * k + base + j] = sblk[(size_t)t * e + q] * bs + (i - q * bs);
      act[(size_t)t * k + base + j] = v > 0.f ? v : 0.f;
    }
    if (base + kTopkEmitLds < k) __syncthreads();   // the next round overwrites the staging arrays
  }
  if (Ap == nullptr) return;
  // dense activation rows A'[slot, 0:bsp] for the matrix-core path: bf16(act) where selected, else 0
  // a selected key of a positive score has its top bit set and the score's bits below it; everything else gives 0
  float a32[KPT];
#pragma unroll
  for (int z = 0; z < KPT; ++z) {
    const uint32_t on = z < 32 ? (uint32_t)__builtin_amdgcn_sbfe((int)sel, z, 1)
                               : (uint32_t)__builtin_amdgcn_sbfe((int)sel_hi, z - 32, 1);
    const uint32_t pos = (uint32_t)((int)key[z] >> 31);
    a32[z] = __uint_as_float(key[z] & 0x7FFFFFFFu & on & pos);
  }
  if (bs % KPT == 0 && (KPT & 7) == 0) {
    // the thread's positions lie in one block's row, 16-byte aligned
    if (p0 < C) {
      uint16_t* dst = Ap + (size_t)slot_of_ent[(size_t)t * e + q0] * bsp + r0;
#pragma unroll
      for (int z = 0; z < KPT; z += 8) {
        u32x4 w;
        w.x = pack_bf16x2(a32[z], a32[z + 1]); w.y = pack_bf16x2(a32[z + 2], a32[z + 3]);
        w.z = pack_bf16x2(a32[z + 4], a32[z + 5]); w.w = pack_bf16x2(a32[z + 6], a32[z + 7]);
        *reinterpret_cast<u32x4*>(dst + z) = w;
      }
    }
  } else {
#pragma unroll
    for (int z = 0; z < KPT; ++z) {
      const int i = p0 + z;
      if (i < C) {
        const int qz = i / bs, rz = i - qz * bs;
        Ap[(size_t)slot_of_ent[t * e + qz] * bsp + rz] = (uint16_t)f32_to_bf16_bits(a32[z]);
      }
    }
  }
  // the padding columns bs .. bsp - 1 of the token's rows are zero
  const int pad = bsp - bs;
  for (int j = tid; j < e * pad; j += 256) {
    const int qz = j / pad, rz = bs + (j - qz * pad);
    Ap[(size_t)slot_of_ent[t * e + qz] * bsp + rz] = 0;
  }
}

// ---------------------------------------------------------------------------------------------
// The register-resident selection for 12288 < C <= 65536 candidates: 1024 threads per token, thread `tid` owns
// the KPT consecutive positions from tid*KPT (1024 * KPT >= C).  Same passes as above; no dense activation rows
// (shapes this large do not take the matrix-core path).
// ---------------------------------------------------------------------------------------------
template <int KPT>
__global__ __launch_bounds__(1024) void topk_select_reg1024_kernel(const float* __restrict__ sc,
                                                                   const int32_t* __restrict__ sblk, int C, int bs,
                                                                   int e, int k, int32_t* __restrict__ idx,
                                                                   float* __restrict__ act) {
  __shared__ int s_hist[256];
  __shared__ int s_w[16];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need;
  const int t = blockIdx.x, tid = threadIdx.x;
  const float* row = sc + (size_t)t * C;
  const int p0 = tid * KPT;
  // 0 for positions beyond C: below every key of a finite score (whose top byte is never 0), so it is never
  // selected, never equals the threshold, and is only ever counted in digit 0 of the first pass, which the search
  // for the k-th largest (k <= C) does not reach
  uint32_t key[KPT];
  if ((C & 3) == 0) {
#pragma unroll
    for (int z = 0; z < KPT; z += 4) {
      if (p0 + z < C) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(row + p0 + z);
        key[z] = order_key(v.x); key[z + 1] = order_key(v.y); key[z + 2] = order_key(v.z); key[z + 3] = order_key(v.w);
      } else {
        key[z] = key[z + 1] = key[z + 2] = key[z + 3] = 0u;
      }
    }
  } else {
#pragma unroll
    for (int z = 0; z < KPT; ++z) key[z] = p0 + z < C ? order_key(row[p0 + z]) : 0u;
  }
  if (tid == 0) { s_prefix = 0u; s_need = k; }
  __syncthreads();

  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) s_hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = s_prefix;
    const uint32_t himask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
    int cur = -1, cnt = 0;
#pragma unroll
    for (int z = 0; z < KPT; ++z) {
      if ((key[z] & himask) == prefix) {   // padding keys (0) only ever land in digit 0 of the first pass
        const int dgt = (int)((key[z] >> shift) & 255u);
        if (dgt == cur) {
          ++cnt;
        } else {
          if (cnt) atomicAdd(&s_hist[cur], cnt);
          cur = dgt;
          cnt = 1;
        }
      }
    }
    if (cnt) atomicAdd(&s_hist[cur], cnt);
    __syncthreads();
    // thread `tid` < 256 owns digit 255 - tid, so that an exclusive scan counts the larger digits
    const int digit = 255 - tid;
    const int h = tid < 256 ? s_hist[digit] : 0;
    int tot;
    const int above = block_excl_scan_1024(h, s_w, tot);
    const int need = s_need;
    __syncthreads();
    if (tid < 256 && above < need && need <= above + h) {
      s_prefix = prefix | ((uint32_t)digit << shift);
      s_need = need - above;
    }
    __syncthreads();
  }
  const uint32_t thr = s_prefix;
  const int need = s_need;  // how many keys equal to thr are selected (>= 1)

  int ngt = 0, neq = 0;
#pragma unroll
  for (int z = 0; z < KPT; ++z) {
    ngt += key[z] > thr;
    neq += key[z] == thr;
  }
  int tot;
  int gt_before = block_excl_scan_1024(ngt, s_w, tot);
  int eq_before = block_excl_scan_1024(neq, s_w, tot);
#pragma unroll
  for (int z = 0; z < KPT; ++z) {
    const bool gt = key[z] > thr, eq = key[z] == thr;
    if (gt || (eq && eq_before < need)) {
      const int slot = gt_before + min(eq_before, need);  // selected positions before this one
      const int i = p0 + z;
      const int q = i / bs, r = i - q * bs;
      const float v = key_to_float(key[z]);
      idx[(size_t)t * k + slot] = sblk[(size_t)t * e + q] * bs + r;
      act[(size_t)t * k + slot] = v > 0.f ? v : 0.f;
    }
    gt_before += gt;
    eq_before += eq;
  }
}

// ---------------------------------------------------------------------------------------------
// The same selection for candidate sets that do not fit in LDS (the paper's ablation without key experts
// is one block holding every neuron: Section 4.3 "MEFT w/o KE", Eq. 1-4 over all r neurons).  The scores
// stay in global memory and are read once per pass: four histogram passes (8 bits each) for the k-th
// largest key and the number of its equals that belong, then one ordered sweep in tiles of 4096 candidates
// (thread order = position order inside a tile, a running base across tiles) that emits the selected
// positions in ascending order.  One workgroup of 1024 threads per token; C % 4 == 0 is not required.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void topk_select_big_kernel(const float* __restrict__ sc,
                                                               const int32_t* __restrict__ sblk, int C, int bs,
                                                               int e, int k, int32_t* __restrict__ idx,
                                                               float* __restrict__ act) {
  __shared__ int s_hist[256];
  __shared__ int s_w[16];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need;
  const int t = blockIdx.x, tid = threadIdx.x;
  const float* row = sc + (size_t)t * C;
  if (tid == 0) { s_prefix = 0u; s_need = k; }
  __syncthreads();

  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) s_hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = s_prefix;
    const uint32_t himask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (int i = tid; i < C; i += 1024) {
      const uint32_t key = order_key(row[i]);
      if ((key & himask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    // thread `tid` < 256 owns digit 255 - tid, so that an exclusive scan counts the larger digits
    const int digit = 255 - tid;
    const int h = tid < 256 ? s_hist[digit] : 0;
    int tot;
    const int above = block_excl_scan_1024(h, s_w, tot);
    const int need = s_need;
    __syncthreads();
    if (tid < 256 && above < need && need <= above + h) {
      s_prefix = prefix | ((uint32_t)digit << shift);
      s_need = need - above;
    }
    __syncthreads();
  }
  const uint32_t thr = s_prefix;
  const int need = s_need;  // how many keys equal to thr are selected (>= 1)

  int gt_base = 0, eq_base = 0;   // selected-or-equal counts in the tiles before this one (same in every thread)
  for (int base = 0; base < C; base += 4096) {
    const int i0 = base + tid * 4;
    uint32_t key[4];
    int ngt = 0, neq = 0;
#pragma unroll
    for (int z = 0; z < 4; ++z) {
      key[z] = i0 + z < C ? order_key(row[i0 + z]) : 0u;   // key 0 is below every real key (thr >= a real key)
      const bool in = i0 + z < C;
      ngt += in && key[z] > thr;
      neq += in && key[z] == thr;
    }
    int tot_gt, tot_eq;
    int gt_before = gt_base + block_excl_scan_1024(ngt, s_w, tot_gt);
    int eq_before = eq_base + block_excl_scan_1024(neq, s_w, tot_eq);
#pragma unroll
    for (int z = 0; z < 4; ++z) {
      if (i0 + z >= C) break;
      const bool gt = key[z] > thr, eq = key[z] == thr;
      if (gt || (eq && eq_before < need)) {
        const int slot = gt_before + min(eq_before, need);  // selected positions before this one
        const int i = i0 + z;
        const int q = i / bs, r = i - q * bs;
        const float v = key_to_float(key[z]);
        idx[(size_t)t * k + slot] = sblk[(size_t)t * e + q] * bs + r;
        act[(size_t)t * k + slot] = v > 0.f ? v : 0.f;
      }
      gt_before += gt;
      eq_before += eq;
    }
    gt_base += tot_gt;
    eq_base += tot_eq;
  }
}

}  // namespace meft
