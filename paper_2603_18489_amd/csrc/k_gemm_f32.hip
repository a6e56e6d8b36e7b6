// fp32 GEMM for the float32 model path: C[M,N] = scale * A[M,K] W[N,K]^T (or C += ...).
// Both operands are K-contiguous.  64x64 output tile per 256-thread block, K step 16, operands
// staged through LDS transposed so that each thread reads its 4+4 values as float4.  Any
// M, N, K: edge tiles are guarded.  This path serves small float32 models; the bf16 path has
// its own MFMA kernels.
#include "ec_internal.h"

namespace ec {

constexpr int GF_BM = 64, GF_BN = 64, GF_BK = 16;

__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A,
                                                       const float* __restrict__ W,
                                                       float* __restrict__ C, int ldc, int M,
                                                       int N, int K, int accumulate,
                                                       float scale) {
  __shared__ float As[GF_BK][GF_BM + 4];
  __shared__ float Ws[GF_BK][GF_BN + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * GF_BM, n0 = blockIdx.x * GF_BN;
  const int tx = tid & 15, ty = tid >> 4;  // thread computes rows ty*4.., cols tx*4..
  const int lrow = tid >> 2, lk = (tid & 3) * 4;  // loader: row 0..63, k offset 0,4,8,12
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += GF_BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int k = k0 + lk + i;
      int am = m0 + lrow, wn = n0 + lrow;
      As[lk + i][lrow] = (am < M && k < K) ? A[(size_t)am * K + k] : 0.f;
      Ws[lk + i][lrow] = (wn < N && k < K) ? W[(size_t)wn * K + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GF_BK; ++kk) {
      float4 a = *(const float4*)&As[kk][ty * 4];
      float4 w = *(const float4*)&Ws[kk][tx * 4];
      float av[4] = {a.x, a.y, a.z, a.w}, wv[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], wv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float* c = C + (size_t)m * ldc + n;
      float v = acc[i][j] * scale;
      *c = accumulate ? (*c + v) : v;
    }
  }
}

void launch_gemm_f32(const float* A, const float* W, float* C, int ldc, int M, int N, int K,
                     int accumulate, float scale, hipStream_t s) {
  if (M <= 0 || N <= 0) return;
  dim3 grid((N + GF_BN - 1) / GF_BN, (M + GF_BM - 1) / GF_BM);
  gemm_f32_kernel<<<grid, 256, 0, s>>>(A, W, C, ldc, M, N, K, accumulate, scale);
}

}  // namespace ec
