// Per-token gather kernels: the activation-weighted value sum of the forward (Eq. 4) and, for
// the backward, the activation gradient ds = (dOut . V_j) * [act > 0] together with
// dh = sum_j ds_j K_j.  One workgroup per token; every thread owns NV groups of 8 consecutive
// columns, so a row is read with full 16-byte (bf16) or 32-byte (fp32) vectors, coalesced over
// the workgroup.
#pragma once
#include "common.h"

namespace meft {

// out[t,:] = sum_i act[t,i] * V[idx[t,i],:]
template <typename T, int NV>
__global__ __launch_bounds__(256) void gather_fwd_kernel(const T* __restrict__ V,
                                                         const int32_t* __restrict__ idx,
                                                         const float* __restrict__ act, int d, int k,
                                                         int N, T* __restrict__ out) {
  const int t = blockIdx.x, tid = threadIdx.x, nthr = blockDim.x;
  float acc[NV][8];
#pragma unroll
  for (int v = 0; v < NV; ++v)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[v][c] = 0.f;
  const int32_t* it = idx + (size_t)t * k;
  const float* at = act + (size_t)t * k;
  constexpr int U = 4;
  int i = 0;
  for (; i + U <= k; i += U) {
    float x[U][NV][8];
    float a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = clampi(it[i + u], 0, N - 1);
      a[u] = at[i + u];
      const T* row = V + (size_t)j * d;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int col = (tid + v * nthr) * 8;
        if (col < d) Vec8<T>::load(row + col, x[u][v]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[v][c] = fmaf(a[u], x[u][v][c], acc[v][c]);
  }
  for (; i < k; ++i) {
    const int j = clampi(it[i], 0, N - 1);
    const float a = at[i];
    const T* row = V + (size_t)j * d;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col = (tid + v * nthr) * 8;
      if (col < d) {
        float x[8];
        Vec8<T>::load(row + col, x);
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[v][c] = fmaf(a, x[c], acc[v][c]);
      }
    }
  }
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int col = (tid + v * nthr) * 8;
    if (col < d) Vec8<T>::store(out + (size_t)t * d + col, acc[v]);
  }
}

// ds[t,i] = act[t,i] > 0 ? dOut[t,:] . V[idx[t,i],:] : 0 ;  dh[t,:] = sum_i ds[t,i] * K[idx[t,i],:]
// Picks are handled in batches of PB: every thread forms PB partial dots over its columns, the
// partials are summed over the workgroup (wave shuffle, then LDS across waves), then the K rows
// are accumulated with the finished ds.  dh may be null.
template <typename T, int NV, int PB>
__global__ __launch_bounds__(256) void gather_bwd_kernel(const T* __restrict__ K, const T* __restrict__ V,
                                                         const T* __restrict__ dOut,
                                                         const int32_t* __restrict__ idx,
                                                         const float* __restrict__ act, int d, int k,
                                                         int N, float* __restrict__ ds,
                                                         T* __restrict__ dh) {
  __shared__ float s_part[4][PB];
  const int t = blockIdx.x, tid = threadIdx.x, nthr = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nthr >> 6;
  float g[NV][8], acc[NV][8];
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int col = (tid + v * nthr) * 8;
#pragma unroll
    for (int c = 0; c < 8; ++c) { g[v][c] = 0.f; acc[v][c] = 0.f; }
    if (col < d) Vec8<T>::load(dOut + (size_t)t * d + col, g[v]);
  }
  const int32_t* it = idx + (size_t)t * k;
  const float* at = act + (size_t)t * k;
  for (int i0 = 0; i0 < k; i0 += PB) {
    float part[PB];
    int jj[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      part[u] = 0.f;
      const int i = i0 + u;
      jj[u] = i < k ? clampi(it[i], 0, N - 1) : -1;
      if (jj[u] >= 0) {
        const T* row = V + (size_t)jj[u] * d;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          const int col = (tid + v * nthr) * 8;
          if (col < d) {
            float x[8];
            Vec8<T>::load(row + col, x);
#pragma unroll
            for (int c = 0; c < 8; ++c) part[u] = fmaf(g[v][c], x[c], part[u]);
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < PB; ++u) part[u] = wave_sum(part[u]);
    if (lane == 0) {
#pragma unroll
      for (int u = 0; u < PB; ++u) s_part[wave][u] = part[u];
    }
    __syncthreads();
    float dsv[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      float s = 0.f;
      for (int w = 0; w < nw; ++w) s += s_part[w][u];
      const int i = i0 + u;
      dsv[u] = (i < k && at[i] > 0.f) ? s : 0.f;
    }
    if (tid < PB && i0 + tid < k) {
      float s = 0.f;
      for (int w = 0; w < nw; ++w) s += s_part[w][tid];
      ds[(size_t)t * k + i0 + tid] = at[i0 + tid] > 0.f ? s : 0.f;
    }
    __syncthreads();
    if (dh) {
#pragma unroll
      for (int u = 0; u < PB; ++u) {
        if (jj[u] >= 0 && dsv[u] != 0.f) {
          const T* row = K + (size_t)jj[u] * d;
#pragma unroll
          for (int v = 0; v < NV; ++v) {
            const int col = (tid + v * nthr) * 8;
            if (col < d) {
              float x[8];
              Vec8<T>::load(row + col, x);
#pragma unroll
              for (int c = 0; c < 8; ++c) acc[v][c] = fmaf(dsv[u], x[c], acc[v][c]);
            }
          }
        }
      }
    }
  }
  if (dh) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col = (tid + v * nthr) * 8;
      if (col < d) Vec8<T>::store(dh + (size_t)t * d + col, acc[v]);
    }
  }
}

}  // namespace meft
