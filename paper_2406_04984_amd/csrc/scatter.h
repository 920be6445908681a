// Backward weight gradients without floating-point atomics: the (token, neuron) pairs are grouped
// by neuron (counting sort; integer atomics only decide positions, and every group is then put in
// ascending pair order, i.e. ascending token), and the group is summed in that fixed order, in chunks of
// kSegChunk pairs (one workgroup each; the chunk sums of a long group are added in chunk order):
//   dV[j,:] = sum act * dOut[t,:],  dK[j,:] = sum ds * h[t,:].
// Only touched rows are written.
#pragma once
#include "common.h"

namespace meft {

__global__ void fill_i32_kernel(int32_t* __restrict__ p, size_t n, int32_t v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// plain streaming copy of n 16-byte words (grid-stride); calibrates bandwidth counters
__global__ __launch_bounds__(256) void probe_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                         size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// A loop of nothing but matrix instructions: every wave keeps eight independent 32 x 32 accumulators busy with
// v_mfma_f32_32x32x16_bf16 on operands of pseudo-random bits (finite bf16 values; what a matrix core draws depends on
// how many bits toggle).  Gives the rate the matrix cores sustain on this machine: the published peak assumes a
// clock that a chip under this load does not hold.  Each thread stores one float so that the loop is not removed.
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ out, int iters) {
  const uint32_t tid = blockIdx.x * 256u + threadIdx.x;
  uint32_t x = tid * 2654435761u + 12345u;
  auto next = [&]() {   // two bf16 values with exponents 0x3F/0x40: magnitudes between 0.5 and 4, random signs
    x = x * 1664525u + 1013904223u;
    return (x & 0x80FF80FFu) | 0x3F003F00u;
  };
  bf16x8 a[2], b[4];
#pragma unroll
  for (int i = 0; i < 2; ++i) a[i] = __builtin_bit_cast(bf16x8, u32x4{next(), next(), next(), next()});
#pragma unroll
  for (int j = 0; j < 4; ++j) b[j] = __builtin_bit_cast(bf16x8, u32x4{next(), next(), next(), next()});
  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += acc[i][j][r];
  out[tid] = sum;
}

// block id of every (token, neuron) pair (ids clamped into range)
__global__ void blocks_of_pairs_kernel(const int32_t* __restrict__ idx, int P, int N, int bs,
                                       int32_t* __restrict__ blk) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p < P) blk[p] = clampi(idx[p], 0, N - 1) / bs;
}

// copies the rows listed in touched[0 .. *n_touched) from a device matrix to the same rows of a matrix in
// pinned host memory (the device writes over the host link); one workgroup per listed row, `vec` 16-byte
// words per row
__global__ __launch_bounds__(256) void rows_to_host_kernel(const int32_t* __restrict__ touched,
                                                           const int32_t* __restrict__ n_touched,
                                                           const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                           int vec) {
  const int u = blockIdx.x;
  if (u >= *n_touched) return;
  const size_t row = (size_t)touched[u] * vec;
  for (int i = threadIdx.x; i < vec; i += 256) dst[row + i] = src[row + i];
}

// cnt[j] += 1 for every pair
__global__ void pair_count_kernel(const int32_t* __restrict__ idx, int P, int N, int32_t* __restrict__ cnt) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p < P) atomicAdd(&cnt[clampi(idx[p], 0, N - 1)], 1);
}

// A neuron's pairs are summed in chunks of kSegChunk consecutive pairs, one workgroup per chunk, so that a neuron that
// very many tokens selected does not leave one workgroup with all of its pairs.
constexpr int kSegChunk = 256;

// seg_off = exclusive scan of cnt; touched = ascending ids with cnt > 0; and per touched neuron u (in that order)
// work_off[u] = chunks of the touched neurons before it, multi_off[u] = the same counting only neurons of more than
// one chunk (their chunks leave partial sums in a buffer); entry [*n_touched] of both holds the total.  One workgroup
// of 1024; thread t owns a run of consecutive counters (a multiple of 4, so that its 16-byte loads and stores are
// aligned) and reads them sixteen at a time with independent loads: read one by one, each counter costs a trip to memory.
__global__ __launch_bounds__(1024) void pair_scan_kernel(const int32_t* __restrict__ cnt, int N,
                                                         int32_t* __restrict__ seg_off,
                                                         int32_t* __restrict__ touched,
                                                         int32_t* __restrict__ n_touched,
                                                         int32_t* __restrict__ work_off,
                                                         int32_t* __restrict__ multi_off) {
  __shared__ int s_c[16], s_f[16], s_w[16], s_m[16];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int chunk = ((N + 1023) / 1024 + 3) & ~3;
  const int j0 = min(N, tid * chunk), j1 = min(N, j0 + chunk);
  auto load16 = [&](int j, int (&v)[16]) {
    if (j + 16 <= j1) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const i32x4 x = *reinterpret_cast<const i32x4*>(cnt + j + 4 * q);
        v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
      }
    } else {
#pragma unroll
      for (int q = 0; q < 16; ++q) v[q] = j + q < j1 ? cnt[j + q] : 0;
    }
  };
  auto chunks_of = [](int v) { return (v + kSegChunk - 1) / kSegChunk; };
  int c = 0, f = 0, wk = 0, mu = 0;
  for (int j = j0; j < j1; j += 16) {
    int v[16];
    load16(j, v);
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int ch = chunks_of(v[q]);
      c += v[q]; f += v[q] > 0; wk += ch; mu += ch > 1 ? ch : 0;
    }
  }
  const int ci = wave_incl_scan(c), fi = wave_incl_scan(f), wi = wave_incl_scan(wk), mi = wave_incl_scan(mu);
  if (lane == 63) { s_c[w] = ci; s_f[w] = fi; s_w[w] = wi; s_m[w] = mi; }
  __syncthreads();
  int cb = 0, fb = 0, wb = 0, mb = 0;
  for (int i = 0; i < w; ++i) { cb += s_c[i]; fb += s_f[i]; wb += s_w[i]; mb += s_m[i]; }
  int off = cb + ci - c, nt = fb + fi - f, wo = wb + wi - wk, mo = mb + mi - mu;
  for (int j = j0; j < j1; j += 16) {
    int v[16], o[16];
    load16(j, v);
#pragma unroll
    for (int q = 0; q < 16; ++q) { o[q] = off; off += v[q]; }
    if (j + 16 <= j1) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<i32x4*>(seg_off + j + 4 * q) = i32x4{o[4 * q], o[4 * q + 1], o[4 * q + 2], o[4 * q + 3]};
    } else {
#pragma unroll
      for (int q = 0; q < 16; ++q)
        if (j + q < j1) seg_off[j + q] = o[q];
    }
#pragma unroll
    for (int q = 0; q < 16; ++q)
      if (v[q] > 0) {   // (v[q] is 0 beyond the run)
        const int ch = chunks_of(v[q]);
        touched[nt] = j + q;
        work_off[nt] = wo;
        multi_off[nt] = mo;
        ++nt; wo += ch; mo += ch > 1 ? ch : 0;
      }
  }
  if (tid == 1023) { seg_off[N] = off; *n_touched = nt; work_off[nt] = wo; multi_off[nt] = mo; }
}

// unordered placement of the pairs into their neuron's segment
__global__ void pair_fill_kernel(const int32_t* __restrict__ idx, int P, int N,
                                 const int32_t* __restrict__ seg_off, int32_t* __restrict__ cursor,
                                 int32_t* __restrict__ pair_list) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= P) return;
  const int j = clampi(idx[p], 0, N - 1);
  const int pos = atomicAdd(&cursor[j], 1);
  pair_list[seg_off[j] + pos] = p;
}

// puts every segment in ascending pair order (pair ids are distinct).  One workgroup per touched neuron.  Up to
// kRankMax entries: rank of an entry = number of smaller entries of the segment.  Up to kBitonicMax: a bitonic sort
// in LDS (a neuron that thousands of tokens selected would cost L^2 comparisons otherwise).  Beyond that (more tokens
// than kBitonicMax selected one neuron): ranks counted against global memory, slow but never wrong.
__global__ __launch_bounds__(256) void seg_sort_kernel(const int32_t* __restrict__ touched,
                                                       const int32_t* __restrict__ n_touched,
                                                       const int32_t* __restrict__ seg_off,
                                                       const int32_t* __restrict__ pair_list,
                                                       int32_t* __restrict__ pair_sorted) {
  constexpr int kRankMax = 256, kBitonicMax = 8192;
  __shared__ int32_t s_p[kBitonicMax];
  const int u = blockIdx.x;
  if (u >= *n_touched) return;
  const int j = touched[u];
  const int o = seg_off[j], L = seg_off[j + 1] - o;
  const int32_t* src = pair_list + o;
  if (L <= kRankMax) {
    for (int i = threadIdx.x; i < L; i += 256) s_p[i] = src[i];
    __syncthreads();
    for (int i = threadIdx.x; i < L; i += 256) {
      const int v = s_p[i];
      int r = 0;
      for (int z = 0; z < L; ++z) r += s_p[z] < v;
      pair_sorted[o + r] = v;
    }
  } else if (L <= kBitonicMax) {
    int n = 512;
    while (n < L) n <<= 1;
    for (int i = threadIdx.x; i < n; i += 256) s_p[i] = i < L ? src[i] : 0x7FFFFFFF;   // padding sorts to the end
    __syncthreads();
    for (int size = 2; size <= n; size <<= 1)
      for (int stride = size >> 1; stride > 0; stride >>= 1) {
        for (int i = threadIdx.x; i < n / 2; i += 256) {
          const int lo = ((i / stride) * stride * 2) + (i % stride), hi = lo + stride;
          const bool up = (lo & size) == 0;   // ascending half of this merge
          const int a = s_p[lo], b = s_p[hi];
          if ((a > b) == up) { s_p[lo] = b; s_p[hi] = a; }
        }
        __syncthreads();
      }
    for (int i = threadIdx.x; i < L; i += 256) pair_sorted[o + i] = s_p[i];
  } else {
    for (int i = threadIdx.x; i < L; i += 256) {
      const int v = src[i];
      int r = 0;
      for (int z = 0; z < L; ++z) r += src[z] < v;
      pair_sorted[o + r] = v;
    }
  }
}

// One chunk of a touched neuron's pairs (kSegChunk consecutive pairs of its segment, summed in ascending pair order):
// workgroup w takes chunk number w of the list that work_off describes.  A neuron of one chunk gets its rows dV[j,:],
// dK[j,:] written here; the chunks of a longer segment leave their fp32 sums in `part` ([chunk][dV | dK][d], chunks
// numbered by multi_off), which seg_finish_kernel adds in chunk order.
template <typename T, int NV>
__global__ __launch_bounds__(256) void seg_reduce_kernel(const int32_t* __restrict__ touched,
                                                         const int32_t* __restrict__ n_touched,
                                                         const int32_t* __restrict__ seg_off,
                                                         const int32_t* __restrict__ work_off,
                                                         const int32_t* __restrict__ multi_off,
                                                         const int32_t* __restrict__ pair_sorted,
                                                         const float* __restrict__ act,
                                                         const float* __restrict__ ds,
                                                         const T* __restrict__ h, const T* __restrict__ dOut,
                                                         int d, int k, T* __restrict__ dK,
                                                         T* __restrict__ dV, float* __restrict__ part) {
  const int nt = *n_touched;
  const int wk = blockIdx.x;
  if (wk >= work_off[nt]) return;
  int lo = 0, hi = nt;   // work_off[lo] <= wk < work_off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (work_off[mid] <= wk) lo = mid; else hi = mid;
  }
  const int u = lo, c = wk - work_off[u], nch = work_off[u + 1] - work_off[u];
  const int j = touched[u];
  const int o = seg_off[j] + c * kSegChunk;
  const int L = min(seg_off[j + 1] - o, kSegChunk);
  const int tid = threadIdx.x, nthr = blockDim.x;
  float aK[NV][8], aV[NV][8];
#pragma unroll
  for (int v = 0; v < NV; ++v)
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) { aK[v][cc] = 0.f; aV[v][cc] = 0.f; }
  constexpr int U = 2;
  int q = 0;
  for (; q + U <= L; q += U) {
    float xh[U][NV][8], xg[U][NV][8], a[U], s[U];
#pragma unroll
    for (int z = 0; z < U; ++z) {
      const int p = pair_sorted[o + q + z];
      const int t = p / k;
      a[z] = act[p];
      s[z] = ds[p];
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int col = (tid + v * nthr) * 8;
        if (col < d) {
          Vec8<T>::load(dOut + (size_t)t * d + col, xg[z][v]);
          Vec8<T>::load(h + (size_t)t * d + col, xh[z][v]);
        }
      }
    }
#pragma unroll
    for (int z = 0; z < U; ++z)
#pragma unroll
      for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) {
          aV[v][cc] = fmaf(a[z], xg[z][v][cc], aV[v][cc]);
          aK[v][cc] = fmaf(s[z], xh[z][v][cc], aK[v][cc]);
        }
  }
  for (; q < L; ++q) {
    const int p = pair_sorted[o + q];
    const int t = p / k;
    const float a = act[p], s = ds[p];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col = (tid + v * nthr) * 8;
      if (col < d) {
        float xg[8], xh[8];
        Vec8<T>::load(dOut + (size_t)t * d + col, xg);
        Vec8<T>::load(h + (size_t)t * d + col, xh);
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) {
          aV[v][cc] = fmaf(a, xg[cc], aV[v][cc]);
          aK[v][cc] = fmaf(s, xh[cc], aK[v][cc]);
        }
      }
    }
  }
  if (nch == 1) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col = (tid + v * nthr) * 8;
      if (col < d) {
        Vec8<T>::store(dV + (size_t)j * d + col, aV[v]);
        Vec8<T>::store(dK + (size_t)j * d + col, aK[v]);
      }
    }
  } else {
    float* pv = part + (size_t)(multi_off[u] + c) * 2 * d;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col = (tid + v * nthr) * 8;
      if (col < d) {
        Vec8<float>::store(pv + col, aV[v]);
        Vec8<float>::store(pv + d + col, aK[v]);
      }
    }
  }
}

// The rows of the touched neurons of more than one chunk: their chunks' partial sums added in chunk order.
template <typename T, int NV>
__global__ __launch_bounds__(256) void seg_finish_kernel(const int32_t* __restrict__ touched,
                                                         const int32_t* __restrict__ n_touched,
                                                         const int32_t* __restrict__ work_off,
                                                         const int32_t* __restrict__ multi_off,
                                                         const float* __restrict__ part, int d,
                                                         T* __restrict__ dK, T* __restrict__ dV) {
  const int nt = *n_touched;
  for (int u = blockIdx.x; u < nt; u += gridDim.x) {
    const int nch = work_off[u + 1] - work_off[u];
    if (nch <= 1) continue;
    const int j = touched[u];
    const float* pv = part + (size_t)multi_off[u] * 2 * d;
    const int tid = threadIdx.x, nthr = blockDim.x;
    float aK[NV][8], aV[NV][8];
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
      for (int cc = 0; cc < 8; ++cc) { aK[v][cc] = 0.f; aV[v][cc] = 0.f; }
    for (int c = 0; c < nch; ++c) {
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int col = (tid + v * nthr) * 8;
        if (col < d) {
          float xv[8], xk[8];
          Vec8<float>::load(pv + (size_t)c * 2 * d + col, xv);
          Vec8<float>::load(pv + (size_t)c * 2 * d + d + col, xk);
#pragma unroll
          for (int cc = 0; cc < 8; ++cc) { aV[v][cc] += xv[cc]; aK[v][cc] += xk[cc]; }
        }
      }
    }
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col = (tid + v * nthr) * 8;
      if (col < d) {
        Vec8<T>::store(dV + (size_t)j * d + col, aV[v]);
        Vec8<T>::store(dK + (size_t)j * d + col, aK[v]);
      }
    }
  }
}

}  // namespace meft
