// Portable LDS-tiled GEMM used for fp32 storage and for shapes the MFMA kernels do not cover.
// Y[m][n] (+)= sum_k X[m][k] * W[n][k]; fp32 accumulation in a fixed order (deterministic).
#include "kernels.h"

namespace mdz {

template <typename T>
__global__ void __launch_bounds__(256) gemm_generic_kernel(const T* __restrict__ X, const T* __restrict__ Wp,
                                                           float* __restrict__ Y, int M, int N, int K, int64_t kp,
                                                           int64_t ldy, bool accumulate) {
  __shared__ float xs[16][64 + 4];
  __shared__ float wsm[16][64 + 4];
  const int bm = blockIdx.y * 64, bn = blockIdx.x * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      int idx = threadIdx.x + e * 256;
      int r = idx >> 4, kk = idx & 15;
      int m = bm + r, n = bn + r, k = k0 + kk;
      xs[kk][r] = (m < M && k < K) ? to_float(X[(int64_t)m * K + k]) : 0.f;
      wsm[kk][r] = (n < N && k < K) ? to_float(Wp[Packed<T>::index(n, k, kp)]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = xs[kk][ty * 4 + i];
        b[i] = wsm[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = bm + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = bn + tx * 4 + j;
      if (n >= N) continue;
      float* y = Y + (int64_t)m * ldy + n;
      *y = accumulate ? *y + acc[i][j] : acc[i][j];
    }
  }
}

int launch_gemm_generic(int dtype, const void* X, const void* Wp, float* Y, int M, int N, int K, int64_t ldy,
                        bool accumulate, hipStream_t st) {
  ProfScope prof_(PROF_GEMM, st);
  if (M == 0 || N == 0) return MDZ_OK;
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  MDZ_WITH_ELEM(dtype, (gemm_generic_kernel<E><<<grid, 256, 0, st>>>((const E*)X, (const E*)Wp, Y, M, N, K,
                                                                     Packed<E>::padded_k(K), ldy, accumulate)));
  MDZ_LAUNCH_CHECK();
  return MDZ_OK;
}

}  // namespace mdz
