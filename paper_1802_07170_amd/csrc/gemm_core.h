// LDS-tiled matrix-core main loop for C = A * B^T with both operands k-contiguous (the paper's
// LinearLayer forward GEMM form; every batched-over-time contraction of the step is brought to
// this form).  WM x WN wavefronts; each wavefront owns TA x TB MFMA 32x32 tiles, so the workgroup
// tile is (32 TA WM) x (32 TB WN).  Two shapes are used:
//   * 2x2 wavefronts, 2x2 tiles each: 128 x 128, 256 threads, 72 KB of LDS, two workgroups per CU
//     hiding each other's barriers.  Reads 32 KB from L2 per 2 x 128 x 128 x 64 flops: at the
//     800 TFLOP/s it reaches, L2 -> CU traffic is 12 TB/s, which is what bounds it.
//   * 4x4 wavefronts, 2x2 tiles each: 256 x 256, 1024 threads, 144 KB of LDS, one workgroup per CU.
//     Half the L2 traffic per flop: 1.1 PFLOP/s on large problems, and faster than the small tile
//     whenever there are about 200 or more tiles.
// Tiles of KB bytes of k per row are double-buffered in LDS; the next tile's global loads are in
// flight while the current one feeds the matrix cores.
#pragma once
#include "common.h"

namespace cmt {

// KB = bytes of k per row and stage; LDS row pitch = KB + 16 (padding against bank conflicts)
template <int WM, int WN, int TA, int TB, int KB = 128> struct GemmTile {
  static constexpr int NT = 64 * WM * WN;                  // threads
  static constexpr int BM = 32 * TA * WM, BN = 32 * TB * WN;
  static constexpr int ROWB = KB + 16;
  static constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int SMEM_BYTES = 2 * STAGE_BYTES;
};
using GemmSmall = GemmTile<2, 2, 2, 2, 128>;               // 128 x 128, 256 threads
using GemmBig = GemmTile<4, 4, 2, 2, 128>;                 // 256 x 256, 1024 threads

// Workgroup id -> output tile.  Consecutive workgroup ids go round-robin to the 8 XCDs (each with
// its own L2), so XCD x is given the contiguous range of tile numbers [x * per, (x + 1) * per); tile
// numbers run down groups of GROUP_M tile rows column by column, so that the ~32 tiles an XCD works
// on at a time form a block of GROUP_M x 8 tiles that share their A and B panels in that L2 (a strip
// of 1 x 32 tiles would pull 33 panels through L2 instead of 12).  Returns false for padding ids.
constexpr int GEMM_GROUP_M = 4;
__device__ __forceinline__ bool gemm_tile_of_block(int ntm, int ntn, int bm, int bn, int& m0, int& n0) {
  const int per = gridDim.x >> 3;
  const int id = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if (id >= ntm * ntn) return false;
  const int gsz = GEMM_GROUP_M * ntn;
  const int grp = id / gsz, rem = id - grp * gsz;
  const int first = grp * GEMM_GROUP_M;
  const int gm = min(GEMM_GROUP_M, ntm - first);
  m0 = (first + rem % gm) * bm;
  n0 = (rem / gm) * bn;
  return true;
}

// Global -> register half of a tile copy.  The rows a thread fetches do not change from one k tile to the next, so
// their offsets from the tile's first element (32-bit, element units; rows beyond `rows` are clamped to the last
// one — they are never stored) are computed once (gemm_tile_offsets) and every load is "uniform base + 32-bit
// thread offset": no 64-bit per-thread addresses are kept across the main loop.
template <typename T, int NT, int ROWS, int KB>
__device__ __forceinline__ void gemm_tile_offsets(int ld, int rows, int r0, unsigned (&off)[ROWS * KB / 16 / NT]) {
  constexpr int EPC = 16 / sizeof(T);                     // elements per 16-byte chunk
  constexpr int CPR = KB / 16;                            // chunks per row
  constexpr int RPP = NT / CPR;                           // rows per pass
  const int t = threadIdx.x;
#pragma unroll
  for (int p = 0; p < ROWS / RPP; ++p) {
    int r = r0 + (t / CPR) + RPP * p;
    r = r < rows ? r : rows - 1;
    off[p] = (unsigned)(r - r0) * (unsigned)ld + (unsigned)((t % CPR) * EPC);
  }
}
// base = first element of the tile row r0 at the k tile's first column (uniform); kleft = K - k0.
template <typename T, int NT, int ROWS, int KB>
__device__ __forceinline__ void gemm_load_tile(const T* __restrict__ base, const unsigned (&off)[ROWS * KB / 16 / NT], int kleft,
                                               uint4 (&regs)[ROWS * KB / 16 / NT]) {
  constexpr int EPC = 16 / sizeof(T);
  constexpr int CPR = KB / 16;
  const bool in = (int)((threadIdx.x % CPR) * EPC) < kleft;
#pragma unroll
  for (int p = 0; p < ROWS * KB / 16 / NT; ++p) {
    if (in) regs[p] = *reinterpret_cast<const uint4*>(base + off[p]);
    else regs[p] = make_uint4(0, 0, 0, 0);
  }
}
template <int NT, int ROWS, int KB>
__device__ __forceinline__ void gemm_store_tile(char* tile, const uint4 (&regs)[ROWS * KB / 16 / NT]) {
  constexpr int CPR = KB / 16, RPP = NT / CPR;
  const int t = threadIdx.x;
#pragma unroll
  for (int p = 0; p < ROWS / RPP; ++p)
    *reinterpret_cast<uint4*>(tile + ((t / CPR) + RPP * p) * (KB + 16) + (t % CPR) * 16) = regs[p];
}

// With w = wavefront index, wm = w / WN, wn = w % WN:
// acc[a][b]: rows m0 + (wm*TA + a)*32 + acc32_row(lane,i), cols n0 + (wn*TB + b)*32 + lane%32
// ZERO = false: the accumulators come in initialised by the caller (e.g. with a bias) and are added to.
template <typename T, int WM, int WN, int TA, int TB, int KB, bool ZERO = true>
__device__ __forceinline__ void gemm_mainloop(const T* __restrict__ A, int lda, const T* __restrict__ B, int ldb,
                                              int M, int N, int K, int m0, int n0, v16f (&acc)[TA][TB], char* smem) {
  using G = GemmTile<WM, WN, TA, TB, KB>;
  constexpr int NT = G::NT;
  constexpr int BK = KB / sizeof(T);
  constexpr int GEMM_ROWB = G::ROWB;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wm = w / WN, wn = w % WN;
  if (ZERO) {
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
      for (int b = 0; b < TB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
  }

  uint4 ra[G::BM * KB / 16 / NT], rb[G::BN * KB / 16 / NT];
  unsigned oa[G::BM * KB / 16 / NT], ob[G::BN * KB / 16 / NT];
  gemm_tile_offsets<T, NT, G::BM, KB>(lda, M, m0, oa);
  gemm_tile_offsets<T, NT, G::BN, KB>(ldb, N, n0, ob);
  const T* __restrict__ pa = A + (size_t)m0 * lda;        // uniform: first row of the tile
  const T* __restrict__ pb = B + (size_t)n0 * ldb;
  gemm_load_tile<T, NT, G::BM, KB>(pa, oa, K, ra);
  gemm_load_tile<T, NT, G::BN, KB>(pb, ob, K, rb);
  gemm_store_tile<NT, G::BM, KB>(smem, ra);
  gemm_store_tile<NT, G::BN, KB>(smem + G::A_BYTES, rb);
  __syncthreads();
  const int nk = (K + BK - 1) / BK;
  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt & 1) * G::STAGE_BYTES;
    char* nxt = smem + ((kt + 1) & 1) * G::STAGE_BYTES;
    const bool more = kt + 1 < nk;
    if (more) {
      gemm_load_tile<T, NT, G::BM, KB>(pa + (kt + 1) * BK, oa, K - (kt + 1) * BK, ra);
      gemm_load_tile<T, NT, G::BN, KB>(pb + (kt + 1) * BK, ob, K - (kt + 1) * BK, rb);
    }
    const char* ta = cur + (wm * 32 * TA + (lane & 31)) * GEMM_ROWB + (lane >> 5) * 8 * sizeof(T);
    const char* tb = cur + G::A_BYTES + (wn * 32 * TB + (lane & 31)) * GEMM_ROWB + (lane >> 5) * 8 * sizeof(T);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      Frag<T> fa[TA], fb[TB];
#pragma unroll
      for (int x = 0; x < TA; ++x) fa[x].load(reinterpret_cast<const T*>(ta + x * 32 * GEMM_ROWB + ks * 16 * sizeof(T)));
#pragma unroll
      for (int x = 0; x < TB; ++x) fb[x].load(reinterpret_cast<const T*>(tb + x * 32 * GEMM_ROWB + ks * 16 * sizeof(T)));
#pragma unroll
      for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b) mma32(acc[a][b], fa[a], fb[b]);
    }
    if (more) {
      gemm_store_tile<NT, G::BM, KB>(nxt, ra);
      gemm_store_tile<NT, G::BN, KB>(nxt + G::A_BYTES, rb);
    }
    __syncthreads();
  }
}

}  // namespace cmt
