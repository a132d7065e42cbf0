// Batched-over-time GEMMs of the training step (the paper's LinearLayer forward / backward /
// calculateGradient, Fig. "Codes of Performing Actual Computation"), all in the single
// "A * B^T, both k-contiguous" form, plus the tiled transpose that brings the backward and
// weight-gradient operands into that form.
#include "gemm_core.h"
#include "kernels.h"

namespace cmt {

template <typename T>
__global__ __launch_bounds__(256) void gemm_nt_kernel(const T* __restrict__ A, int lda, const T* __restrict__ B, int ldb,
                                                      int M, int N, int K, float* __restrict__ Cf, T* __restrict__ Ct,
                                                      int ldc, const float* __restrict__ bias, int accumulate) {
  __shared__ __align__(16) char smem[GEMM_SMEM_BYTES];
  const int m0 = blockIdx.y * GEMM_BM, n0 = blockIdx.x * GEMM_BN;
  v16f acc[2][2];
  gemm_mainloop<T>(A, lda, B, ldb, M, N, K, m0, n0, acc, smem);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wm = w >> 1, wn = w & 1;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int col = n0 + wn * 64 + nt * 32 + (lane & 31);
    if (col >= N) continue;
    const float bv = bias ? bias[col] : 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = m0 + wm * 64 + mt * 32 + acc32_row(lane, i);
        if (row >= M) continue;
        const size_t o = (size_t)row * ldc + col;
        float v = acc[mt][nt][i] + bv;
        if (accumulate) v += Cf[o];
        if (Cf) Cf[o] = v;
        if (Ct) Ct[o] = from_f<T>(v);
      }
    }
  }
}

void launch_gemm_nt(int prec, const void* A, int lda, const void* B, int ldb, int M, int N, int K,
                    float* Cf, void* Ct, int ldc, const float* bias, int accumulate, hipStream_t st) {
  if (M <= 0 || N <= 0) return;
  dim3 grid((N + GEMM_BN - 1) / GEMM_BN, (M + GEMM_BM - 1) / GEMM_BM);
  if (prec)
    hipLaunchKernelGGL(gemm_nt_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)A, lda,
                       (const bf16_t*)B, ldb, M, N, K, Cf, (bf16_t*)Ct, ldc, bias, accumulate);
  else
    hipLaunchKernelGGL(gemm_nt_kernel<float>, grid, dim3(256), 0, st, (const float*)A, lda,
                       (const float*)B, ldb, M, N, K, Cf, (float*)Ct, ldc, bias, accumulate);
}

// 64x64 tiles through LDS; reads and writes are both row-contiguous.
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, int ldin, T* __restrict__ out, int ldout,
                                                        int R, int C) {
  __shared__ T tile[64][65];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int r = r0 + ty + 4 * i, c = c0 + tx;
    if (r < R && c < C) tile[ty + 4 * i][tx] = in[(size_t)r * ldin + c];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = c0 + ty + 4 * i, r = r0 + tx;
    if (r < R && c < C) out[(size_t)c * ldout + r] = tile[tx][ty + 4 * i];
  }
}

void launch_transpose(int prec, const void* in, int ldin, void* out, int ldout, int R, int C, hipStream_t st) {
  if (R <= 0 || C <= 0) return;
  dim3 grid((C + 63) / 64, (R + 63) / 64);
  if (prec)
    hipLaunchKernelGGL(transpose_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)in, ldin, (bf16_t*)out, ldout, R, C);
  else
    hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, st, (const float*)in, ldin, (float*)out, ldout, R, C);
}

}  // namespace cmt
