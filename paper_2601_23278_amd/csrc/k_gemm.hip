// Dense projections  C[M, N] = A[M, K] * W[N, K]^T  (activations times [out, in] weights), fp32 accumulate.
//
// Two kernels:
//   k_gemm_valu  any element type, any shape: LDS-tiled 64x64x16, 4x4 outputs per lane on the vector ALU.
//                Used for fp32 models (the tiny oracle-check configuration) and for shapes the MFMA kernel
//                does not take.
//   k_gemm_mfma  bf16 on the matrix cores (see below).
// M is read from device memory when the row count is only known on the device (packed batch after eviction).
#include "focus_internal.h"

namespace fk {

template <typename T> __device__ __forceinline__ float to_f(T v) { return (float)v; }

template <typename T, int EPI>
__device__ __forceinline__ void store_out(void *out, size_t idx, float acc) {
  if (EPI == EPI_STORE) ((T *)out)[idx] = (T)acc;
  else if (EPI == EPI_ADD_F32) ((float *)out)[idx] += acc;
  else ((float *)out)[idx] = acc;
}

template <typename T, int EPI>
__global__ __launch_bounds__(256) void k_gemm_valu(const T *__restrict__ A, const T *__restrict__ W, int N, int K, Rows rows,
                                                   void *out, int ldo) {
  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  if (m0 >= M) return;
  __shared__ float As[16][65], Ws[16][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = threadIdx.x; i < 1024; i += 256) {
      int rr = i >> 4, kk = i & 15;
      int gm = m0 + rr, gn = n0 + rr, gk = k0 + kk;
      As[kk][rr] = (gm < M && gk < K) ? to_f(A[(size_t)gm * K + gk]) : 0.f;
      Ws[kk][rr] = (gn < N && gk < K) ? to_f(W[(size_t)gn * K + gk]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i], w[i] = Ws[kk][tx * 4 + i];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * w[j];
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i) {
    int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
    for (int j = 0; j < 4; ++j) {
      int gn = n0 + tx * 4 + j;
      if (gn < N) store_out<T, EPI>(out, (size_t)gm * ldo + gn, acc[i][j]);
    }
  }
}

template <typename T>
static void launch_valu(hipStream_t s, const void *A, const void *W, int N, int K, Rows rows, int epi, void *out, int ldo) {
  dim3 grid((N + 63) / 64, (rows.cap + 63) / 64);
  if (epi == EPI_STORE)
    k_gemm_valu<T, EPI_STORE><<<grid, 256, 0, s>>>((const T *)A, (const T *)W, N, K, rows, out, ldo);
  else if (epi == EPI_ADD_F32)
    k_gemm_valu<T, EPI_ADD_F32><<<grid, 256, 0, s>>>((const T *)A, (const T *)W, N, K, rows, out, ldo);
  else
    k_gemm_valu<T, EPI_STORE_F32><<<grid, 256, 0, s>>>((const T *)A, (const T *)W, N, K, rows, out, ldo);
}

void gemm(hipStream_t s, int dtype, const void *A, const void *W, int N, int K, Rows rows, int epilogue,
          void *out, int ldo) {
  if (rows.cap <= 0) return;
  if (dtype == FOCUS_F32) launch_valu<float>(s, A, W, N, K, rows, epilogue, out, ldo);
  else launch_valu<bf16_t>(s, A, W, N, K, rows, epilogue, out, ldo);
}

}  // namespace fk
