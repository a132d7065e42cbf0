// LDS-tiled 128x128 matrix-core main loop for C = A * B^T with both operands k-contiguous
// (the paper's LinearLayer forward GEMM form; every batched-over-time contraction of the step is
// brought to this form).  256 threads = 4 wavefronts in a 2x2 grid, each owning a 64x64 block as
// 2x2 MFMA 32x32 tiles.  Tiles of 128 rows x 128 bytes of k are double-buffered in LDS; the next
// tile's global loads are in flight while the current one feeds the matrix cores.
#pragma once
#include "common.h"

namespace cmt {

constexpr int GEMM_BM = 128, GEMM_BN = 128;
constexpr int GEMM_ROWB = 128 + 16;                       // LDS row pitch in bytes (padding against bank conflicts)
constexpr int GEMM_TILE_BYTES = GEMM_BM * GEMM_ROWB;      // one operand tile
constexpr int GEMM_SMEM_BYTES = 4 * GEMM_TILE_BYTES;      // 2 buffers x (A, B)

template <typename T>
__device__ __forceinline__ void gemm_load_tile(const T* __restrict__ P, int ld, int rows, int K, int r0, int k0,
                                               uint4 (&regs)[4]) {
  constexpr int EPC = 16 / sizeof(T);                     // elements per 16-byte chunk
  const int t = threadIdx.x;
  const int chunk = t & 7;
  const int kc = k0 + chunk * EPC;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    int r = r0 + (t >> 3) + 32 * p;
    r = r < rows ? r : rows - 1;                          // clamped rows are never stored
    if (kc < K) regs[p] = *reinterpret_cast<const uint4*>(P + (size_t)r * ld + kc);
    else regs[p] = make_uint4(0, 0, 0, 0);
  }
}
__device__ __forceinline__ void gemm_store_tile(char* tile, const uint4 (&regs)[4]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int p = 0; p < 4; ++p)
    *reinterpret_cast<uint4*>(tile + ((t >> 3) + 32 * p) * GEMM_ROWB + (t & 7) * 16) = regs[p];
}

// acc[mt][nt]: rows m0 + wm*64 + mt*32 + acc32_row(lane,i), cols n0 + wn*64 + nt*32 + lane%32
template <typename T>
__device__ __forceinline__ void gemm_mainloop(const T* __restrict__ A, int lda, const T* __restrict__ B, int ldb,
                                              int M, int N, int K, int m0, int n0, v16f (&acc)[2][2], char* smem) {
  constexpr int BK = 128 / sizeof(T);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wm = w >> 1, wn = w & 1;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  uint4 ra[4], rb[4];
  gemm_load_tile<T>(A, lda, M, K, m0, 0, ra);
  gemm_load_tile<T>(B, ldb, N, K, n0, 0, rb);
  gemm_store_tile(smem, ra);
  gemm_store_tile(smem + GEMM_TILE_BYTES, rb);
  __syncthreads();
  const int nk = (K + BK - 1) / BK;
  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt & 1) * 2 * GEMM_TILE_BYTES;
    char* nxt = smem + ((kt + 1) & 1) * 2 * GEMM_TILE_BYTES;
    const bool more = kt + 1 < nk;
    if (more) {
      gemm_load_tile<T>(A, lda, M, K, m0, (kt + 1) * BK, ra);
      gemm_load_tile<T>(B, ldb, N, K, n0, (kt + 1) * BK, rb);
    }
    const char* ta = cur + (wm * 64 + (lane & 31)) * GEMM_ROWB + (lane >> 5) * 8 * sizeof(T);
    const char* tb = cur + GEMM_TILE_BYTES + (wn * 64 + (lane & 31)) * GEMM_ROWB + (lane >> 5) * 8 * sizeof(T);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      Frag<T> fa[2], fb[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        fa[x].load(reinterpret_cast<const T*>(ta + x * 32 * GEMM_ROWB + ks * 16 * sizeof(T)));
        fb[x].load(reinterpret_cast<const T*>(tb + x * 32 * GEMM_ROWB + ks * 16 * sizeof(T)));
      }
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) mma32(acc[a][b], fa[a], fb[b]);
    }
    if (more) {
      gemm_store_tile(nxt, ra);
      gemm_store_tile(nxt + GEMM_TILE_BYTES, rb);
    }
    __syncthreads();
  }
}

}  // namespace cmt
