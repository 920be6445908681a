// Score GEMMs: C[m, n] = sum_c A[row(m), c] * Bm[n, c]  ("NT": both operands are contiguous
// along the contraction).  Used for the router scores (Eq. 5: one problem, A = h, Bm = Wg) and
// for the in-block key scores (Eq. 6: one problem per block, rows = the tokens routed to the
// block, Bm = that block's keys).  fp32 accumulation.
#pragma once
#include "common.h"

namespace meft {

struct GemmNTArgs {
  const void* A;         // rows of length Kdim, leading dimension lda
  const void* Bm;        // [n_groups*Ng, ldb]; group g owns rows [g*Ng, (g+1)*Ng)
  float* C;              // output rows, leading dimension ldc
  const int* perm;       // entries grouped by problem ([group_off[n_groups]]), or nullptr
  const int* group_off;  // [n_groups+1] first slot of each group in perm, or nullptr
  const int* tile_off;   // [n_groups+1] prefix sum of ceil(rows_g / BM), or nullptr
  int n_groups;          // 1 when perm == nullptr
  int M;                 // rows when perm == nullptr
  int Ng;                // columns per group
  int Kdim;
  int lda, ldb, ldc;
  int e;                 // with perm: A row = entry / e, C row = entry
};

// Finds the group and the first row of m-tile `mt`; returns false if the tile does not exist.
template <int BM>
__device__ __forceinline__ bool locate_tile(const GemmNTArgs& a, int mt, int& g, int& m0, int& Mg,
                                            int& slot0) {
  if (a.perm == nullptr) {
    g = 0; m0 = mt * BM; Mg = a.M; slot0 = 0;
    return m0 < Mg;
  }
  if (mt >= a.tile_off[a.n_groups]) return false;
  int lo = 0, hi = a.n_groups;  // tile_off[lo] <= mt < tile_off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.tile_off[mid] <= mt) lo = mid; else hi = mid;
  }
  g = lo;
  m0 = (mt - a.tile_off[g]) * BM;
  slot0 = a.group_off[g];
  Mg = a.group_off[g + 1] - slot0;
  return true;
}

// ---------------------------------------------------------------------------------------------
// bf16 inputs, MFMA 32x32x16, 128x128 tile, 4 waves (2x2), each wave 64x64 = 2x2 MFMA tiles.
// LDS rows are padded by 8 elements (16 B) so that the 32 rows an operand read touches start in
// different banks.
// ---------------------------------------------------------------------------------------------
constexpr int kGemmBM = 128, kGemmBN = 128, kGemmBK = 64, kGemmPad = 8;

__global__ __launch_bounds__(256) void gemm_nt_bf16_kernel(GemmNTArgs a) {
  constexpr int BM = kGemmBM, BN = kGemmBN, BK = kGemmBK, LD = kGemmBK + kGemmPad;
  __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LD];
  __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LD];
  __shared__ int sRowA[BM];
  __shared__ int sRowC[BM];

  int g, m0, Mg, slot0;
  if (!locate_tile<BM>(a, blockIdx.x, g, m0, Mg, slot0)) return;
  const int n0 = blockIdx.y * BN;
  const int tid = threadIdx.x;

  if (tid < BM) {
    const int m = m0 + tid;
    int ra = -1, rc = -1;
    if (m < Mg) {
      if (a.perm) { rc = a.perm[slot0 + m]; ra = rc / a.e; } else { ra = m; rc = m; }
    }
    sRowA[tid] = ra;
    sRowC[tid] = rc;
  }
  __syncthreads();

  const uint16_t* A = static_cast<const uint16_t*>(a.A);
  const uint16_t* Bm = static_cast<const uint16_t*>(a.Bm) + (size_t)g * a.Ng * a.ldb;

  // global -> register staging: 4 vectors of 8 elements per thread and operand
  const int vrow = tid >> 3;        // 0..31 (+32 per step)
  const int vk = (tid & 7) * 8;     // element offset inside the k tile
  const uint16_t* pa[4];
  const uint16_t* pb[4];
  bool va[4], vb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = vrow + i * 32;
    const int ra = sRowA[r];
    va[i] = ra >= 0;
    pa[i] = A + (size_t)(va[i] ? ra : 0) * a.lda + vk;
    const int n = n0 + r;
    vb[i] = n < a.Ng;
    pb[i] = Bm + (size_t)(vb[i] ? n : 0) * a.ldb + vk;
  }
  u32x4 ra4[4], rb4[4];
  const u32x4 zero = {0u, 0u, 0u, 0u};
  auto gload = [&](int k0) {
    const bool kin = (k0 + vk) < a.Kdim;  // Kdim % 8 == 0: a vector is fully in or out
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ra4[i] = (va[i] && kin) ? *reinterpret_cast<const u32x4*>(pa[i] + k0) : zero;
      rb4[i] = (vb[i] && kin) ? *reinterpret_cast<const u32x4*>(pb[i] + k0) : zero;
    }
  };

  const int wave = tid >> 6, lane = tid & 63;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  gload(0);
  for (int k0 = 0; k0 < a.Kdim; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *reinterpret_cast<u32x4*>(&sA[(vrow + i * 32) * LD + vk]) = ra4[i];
      *reinterpret_cast<u32x4*>(&sB[(vrow + i * 32) * LD + vk]) = rb4[i];
    }
    __syncthreads();
    if (k0 + BK < a.Kdim) gload(k0 + BK);
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = *reinterpret_cast<const bf16x8*>(&sA[(wm + i * 32 + fr) * LD + ks + fk]);
        fb[i] = *reinterpret_cast<const bf16x8*>(&sB[(wn + i * 32 + fr) * LD + ks + fk]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // accumulator element r of a 32x32 tile: row (r/4)*8 + (lane/32)*4 + r%4, column lane%32
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + wn + j * 32 + fr;
      if (n >= a.Ng) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ml = wm + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const int rc = sRowC[ml];
        if (rc >= 0) a.C[(size_t)rc * a.ldc + n] = acc[i][j][r];
      }
    }
}

// ---------------------------------------------------------------------------------------------
// fp32 inputs: LDS-tiled FMA GEMM, 64x64 tile, 256 threads, 4x4 outputs per thread.
// ---------------------------------------------------------------------------------------------
constexpr int kGemmF32BM = 64, kGemmF32BN = 64, kGemmF32BK = 16;

__global__ __launch_bounds__(256) void gemm_nt_f32_kernel(GemmNTArgs a) {
  constexpr int BM = kGemmF32BM, BN = kGemmF32BN, BK = kGemmF32BK;
  __shared__ float sA[BK][BM + 4];
  __shared__ float sB[BK][BN + 4];
  __shared__ int sRowA[BM];
  __shared__ int sRowC[BM];

  int g, m0, Mg, slot0;
  if (!locate_tile<BM>(a, blockIdx.x, g, m0, Mg, slot0)) return;
  const int n0 = blockIdx.y * BN;
  const int tid = threadIdx.x;
  if (tid < BM) {
    const int m = m0 + tid;
    int ra = -1, rc = -1;
    if (m < Mg) {
      if (a.perm) { rc = a.perm[slot0 + m]; ra = rc / a.e; } else { ra = m; rc = m; }
    }
    sRowA[tid] = ra;
    sRowC[tid] = rc;
  }
  __syncthreads();

  const float* A = static_cast<const float*>(a.A);
  const float* Bm = static_cast<const float*>(a.Bm) + (size_t)g * a.Ng * a.ldb;
  // one float4 per thread and operand: row = tid/4, k = (tid%4)*4
  const int lr = tid >> 2, lk = (tid & 3) * 4;
  const int ra = sRowA[lr];
  const int nb = n0 + lr;
  const float* pa = A + (size_t)(ra >= 0 ? ra : 0) * a.lda + lk;
  const float* pb = Bm + (size_t)(nb < a.Ng ? nb : 0) * a.ldb + lk;
  const int tm = (tid >> 4) * 4, tn = (tid & 15) * 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < a.Kdim; k0 += BK) {
    f32x4 xa = {0.f, 0.f, 0.f, 0.f}, xb = {0.f, 0.f, 0.f, 0.f};
    if (k0 + lk < a.Kdim) {  // Kdim % 4 == 0
      if (ra >= 0) xa = *reinterpret_cast<const f32x4*>(pa + k0);
      if (nb < a.Ng) xb = *reinterpret_cast<const f32x4*>(pb + k0);
    }
    sA[lk + 0][lr] = xa.x; sA[lk + 1][lr] = xa.y; sA[lk + 2][lr] = xa.z; sA[lk + 3][lr] = xa.w;
    sB[lk + 0][lr] = xb.x; sB[lk + 1][lr] = xb.y; sB[lk + 2][lr] = xb.z; sB[lk + 3][lr] = xb.w;
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      const f32x4 av = *reinterpret_cast<const f32x4*>(&sA[kk][tm]);
      const f32x4 bv = *reinterpret_cast<const f32x4*>(&sB[kk][tn]);
      const float am[4] = {av.x, av.y, av.z, av.w};
      const float bn[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(am[i], bn[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int rc = sRowC[tm + i];
    if (rc < 0) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tn + j;
      if (n < a.Ng) a.C[(size_t)rc * a.ldc + n] = acc[i][j];
    }
  }
}

}  // namespace meft
