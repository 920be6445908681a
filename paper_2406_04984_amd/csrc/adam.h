// Row-sparse Adam: the optimizer step for the rows of K or V that received a gradient in this step
// (Section 3.1, last paragraph: only activated parameters have gradients; Section 4.3: Adam).
// One workgroup per touched row at a time; each thread owns groups of 8 consecutive columns, so every
// access is a 16- or 32-byte vector access and a row is streamed once.  The work is pure HBM traffic:
// per element the gradient and the weight are read, both moments are read and written, the weight is written.
#pragma once
#include "common.h"

namespace meft {

struct AdamScalars {
  float lr, b1, b2, omb1, omb2, eps, inv_c1, inv_c2;   // omb = 1 - beta, inv_c = 1 / (1 - beta^step)
};

template <typename T>
__global__ __launch_bounds__(256) void adam_rows_kernel(T* __restrict__ W, const T* __restrict__ G,
                                                        float* __restrict__ m, float* __restrict__ v,
                                                        float* __restrict__ master,
                                                        const int32_t* __restrict__ touched,
                                                        const int32_t* __restrict__ n_touched, int N, int d,
                                                        AdamScalars a) {
  const int n = min(*n_touched, N);
  for (int i = blockIdx.x; i < n; i += gridDim.x) {
    const int j = touched[i];
    if ((unsigned)j >= (unsigned)N) continue;   // not an id of this matrix: leave everything as it is
    const size_t row = (size_t)j * d;
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
      float g[8], w[8], mm[8], vv[8];
      Vec8<T>::load(G + row + c, g);
      if (master) Vec8<float>::load(master + row + c, w);
      else Vec8<T>::load(W + row + c, w);
      Vec8<float>::load(m + row + c, mm);
      Vec8<float>::load(v + row + c, vv);
#pragma unroll
      for (int z = 0; z < 8; ++z) {
        mm[z] = a.b1 * mm[z] + a.omb1 * g[z];
        vv[z] = a.b2 * vv[z] + a.omb2 * g[z] * g[z];
        w[z] -= a.lr * (mm[z] * a.inv_c1) / (sqrtf(vv[z] * a.inv_c2) + a.eps);
      }
      Vec8<float>::store(m + row + c, mm);
      Vec8<float>::store(v + row + c, vv);
      if (master) Vec8<float>::store(master + row + c, w);
      Vec8<T>::store(W + row + c, w);
    }
  }
}

}  // namespace meft
