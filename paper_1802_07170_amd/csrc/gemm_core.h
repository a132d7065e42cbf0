// LDS-tiled matrix-core main loop for C = A * B^T with both operands k-contiguous (the paper's
// LinearLayer forward GEMM form; every batched-over-time contraction of the step is brought to
// this form).  WM x WN wavefronts; each wavefront owns TA x TB MFMA 32x32 tiles, so the workgroup
// tile is (32 TA WM) x (32 TB WN).  Two shapes are used:
//   * 2x2 wavefronts, 2x2 tiles each: 128 x 128, 256 threads, 72 KB of LDS, two workgroups per CU
//     hiding each other's barriers.  Needs 32 KB from L2 per 2 x 128 x 128 x 64 flops.
//   * 4x4 wavefronts, 2x2 tiles each: 256 x 256, 1024 threads, 144 KB of LDS, one workgroup per CU.
//     Half the L2 traffic per flop (64 KB per k tile): 1.3 PFLOP/s on large problems, and faster than the
//     small tile whenever there are about 200 or more tiles.
// What bounds both is the rate at which a CU takes data from L2: about 49 GB/s per CU measured with the main
// loop's loads alone (12.6 TB/s over the chip), i.e. at most 1.6 PFLOP/s for the big tile and 0.8 for the small.
// Tiles of KB bytes of k per row are double-buffered in LDS; the next tile's global loads are in
// flight while the current one feeds the matrix cores.  16-bit operands go from global memory straight
// into LDS (global_load_lds_dwordx4, no staging registers): rows of 128 bytes without padding, the
// 16-byte chunks of a row XOR-swizzled by the row number so that fragment reads stay free of bank
// conflicts (gemm_swz).  32-bit operands are staged through registers into rows padded by 16 bytes.
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
// of 1 x 32 tiles would pull 33 panels through L2 instead of 12).  Returns false for padding ids.  The
// launched grid must hold at least 8 * ceil(ntm * ntn / 8) workgroups.
constexpr int GEMM_GROUP_M = 4;
// tile number (in the grouped order described above) -> first row and column of the tile
__device__ __forceinline__ void gemm_tile_from_index(int id, int ntm, int ntn, int bm, int bn, int& m0, int& n0) {
  const int gsz = GEMM_GROUP_M * ntn;
  const int grp = id / gsz, rem = id - grp * gsz;
  const int first = grp * GEMM_GROUP_M;
  const int gm = min(GEMM_GROUP_M, ntm - first);
  m0 = (first + rem % gm) * bm;
  n0 = (rem / gm) * bn;
}
// workgroup id -> tile number for a launch of at least 8 * ceil(nt / 8) workgroups over nt tiles; -1 for padding ids.
// `per` comes from the tiles that exist, not from the launched grid: a launch sized for more rows than the
// device-side count leaves (ids beyond the last tile exit) still spreads its tiles evenly over the XCDs.
// `vb` = the (virtual) workgroup id: blockIdx.x, or blockIdx.x + a multiple of the grid for a workgroup that walks
// several tiles (the grid is a multiple of 8, so it stays with the tile range of its XCD).
__device__ __forceinline__ int gemm_tile_index(int nt, int vb) {
  const int per = (nt + 7) >> 3, j = vb >> 3;
  const int id = (vb & 7) * per + j;
  return (j >= per || id >= nt) ? -1 : id;
}
__device__ __forceinline__ int gemm_tile_index(int nt) { return gemm_tile_index(nt, (int)blockIdx.x); }
__device__ __forceinline__ bool gemm_tile_of_block(int ntm, int ntn, int bm, int bn, int& m0, int& n0, int vb = -1) {
  const int id = gemm_tile_index(ntm * ntn, vb < 0 ? (int)blockIdx.x : vb);
  if (id < 0) return false;
  gemm_tile_from_index(id, ntm, ntn, bm, bn, m0, n0);
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

// ---- 16-bit operands: global -> LDS without staging registers ----
// LDS image of a tile: row r (128 bytes = 64 elements of k) at r * 128; the 16-byte chunk c of the row sits at
// position c ^ gemm_swz(r).  A load instruction of wavefront w writes 64 consecutive 16-byte slots (the hardware
// adds lane * 16 to the base in M0), so slot (p * NT + thread) holds row slot / 8, position slot % 8, and the
// thread fetches the chunk that belongs there.
__device__ __forceinline__ int gemm_swz(int r) { return (r ^ (r >> 3)) & 7; }

// byte offsets from the tile's first row at the k tile's first column; rows beyond `rows` clamped (never stored)
template <int NT, int ROWS>
__device__ __forceinline__ void gemm_dl_offsets(int ld, int rows, int r0, unsigned (&off)[ROWS * 8 / NT]) {
  static_assert((ROWS * 8) % NT == 0, "tile rows must fill whole passes of the workgroup");
#pragma unroll
  for (int p = 0; p < ROWS * 8 / NT; ++p) {
    const int slot = p * NT + threadIdx.x, r = slot >> 3, c = (slot & 7) ^ gemm_swz(r);
    const int row = min(r0 + r, rows - 1) - r0;
    off[p] = ((unsigned)row * (unsigned)ld + (unsigned)(c * 8)) * 2u;
  }
}
__device__ __forceinline__ unsigned gemm_lds_address(const char* p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const char*)p;
}
// Asynchronous: completion is awaited with gemm_dl_wait() before the barrier that publishes the stage.
// The instruction is written out because the compiler, when it knows a load writes LDS, waits for every
// outstanding one before the next LDS read of any address — which would serialise the two stages.  M0 (the LDS
// base of the transfer) is a register the compiler reserves and loads directly before each use of its own, so
// setting it here disturbs nothing (it cannot be named as a clobber).
template <int NT, int ROWS>
__device__ __forceinline__ void gemm_dl_issue(const bf16_t* __restrict__ base, const unsigned (&off)[ROWS * 8 / NT], char* tile, int w) {
#pragma unroll
  for (int p = 0; p < ROWS * 8 / NT; ++p) {
    const unsigned dst = gemm_lds_address(tile) + (unsigned)((p * NT + w * 64) * 16);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(off[p]), "s"(base) : "memory");
  }
}
__device__ __forceinline__ void gemm_dl_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// A k tile with fewer than 64 valid columns (the last one of a K that is no multiple of 64): through registers,
// chunks beyond K as zeros, into the same LDS image.
template <int NT, int ROWS>
__device__ __forceinline__ void gemm_dl_fill_tail(const bf16_t* __restrict__ base, const unsigned (&off)[ROWS * 8 / NT], int kleft, char* tile) {
#pragma unroll
  for (int p = 0; p < ROWS * 8 / NT; ++p) {
    const int slot = p * NT + threadIdx.x, r = slot >> 3, c = (slot & 7) ^ gemm_swz(r);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (c * 8 < kleft) v = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(base) + off[p]);
    *reinterpret_cast<uint4*>(tile + slot * 16) = v;
  }
}

template <int WM, int WN, int TA, int TB, bool ZERO>
__device__ __forceinline__ void gemm_mainloop_dl(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ B, int ldb,
                                                 int M, int N, int K, int m0, int n0, v16f (&acc)[TA][TB], char* smem) {
  constexpr int NT = 64 * WM * WN, BM = 32 * TA * WM, BN = 32 * TB * WN;
  constexpr int A_BYTES = BM * 128, STAGE = (BM + BN) * 128;
  static_assert(2 * STAGE <= GemmTile<WM, WN, TA, TB, 128>::SMEM_BYTES, "LDS image larger than the tile's allocation");
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = w / WN, wn = w % WN;
  if (ZERO) {
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
      for (int b = 0; b < TB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
  }
  unsigned oa[BM * 8 / NT], ob[BN * 8 / NT];
  gemm_dl_offsets<NT, BM>(lda, M, m0, oa);
  gemm_dl_offsets<NT, BN>(ldb, N, n0, ob);
  const bf16_t* __restrict__ pa = A + (size_t)m0 * lda;    // uniform: first row of the tile
  const bf16_t* __restrict__ pb = B + (size_t)n0 * ldb;
  auto fill = [&](char* stage, int k0) {
    if (K - k0 >= 64) {
      gemm_dl_issue<NT, BM>(pa + k0, oa, stage, w);
      gemm_dl_issue<NT, BN>(pb + k0, ob, stage + A_BYTES, w);
    } else {
      gemm_dl_fill_tail<NT, BM>(pa + k0, oa, K - k0, stage);
      gemm_dl_fill_tail<NT, BN>(pb + k0, ob, K - k0, stage + A_BYTES);
    }
  };
  fill(smem, 0);
  gemm_dl_wait();
  __syncthreads();
  // fragment of row r at k step ks: chunk 2 ks + lane / 32, at position chunk ^ gemm_swz(r)
  int fa_row[TA], fa_s[TA], fb_row[TB], fb_s[TB];
#pragma unroll
  for (int x = 0; x < TA; ++x) { const int r = (wm * TA + x) * 32 + (lane & 31); fa_row[x] = r * 128; fa_s[x] = gemm_swz(r) ^ (lane >> 5); }
#pragma unroll
  for (int x = 0; x < TB; ++x) { const int r = (wn * TB + x) * 32 + (lane & 31); fb_row[x] = A_BYTES + r * 128; fb_s[x] = gemm_swz(r) ^ (lane >> 5); }
  const int nk = (K + 63) / 64;
  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt & 1) * STAGE;
    char* nxt = smem + ((kt + 1) & 1) * STAGE;
    if (kt + 1 < nk) fill(nxt, (kt + 1) * 64);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      Frag<bf16_t> fa[TA], fb[TB];
#pragma unroll
      for (int x = 0; x < TA; ++x) fa[x].load(reinterpret_cast<const bf16_t*>(cur + fa_row[x] + ((fa_s[x] ^ (2 * ks)) << 4)));
#pragma unroll
      for (int x = 0; x < TB; ++x) fb[x].load(reinterpret_cast<const bf16_t*>(cur + fb_row[x] + ((fb_s[x] ^ (2 * ks)) << 4)));
#pragma unroll
      for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b) mma32(acc[a][b], fa[a], fb[b]);
    }
    gemm_dl_wait();
    __syncthreads();
  }
}

// With w = wavefront index, wm = w / WN, wn = w % WN:
// acc[a][b]: rows m0 + (wm*TA + a)*32 + acc32_row(lane,i), cols n0 + (wn*TB + b)*32 + lane%32
// ZERO = false: the accumulators come in initialised by the caller (e.g. with a bias) and are added to.
template <typename T, int WM, int WN, int TA, int TB, int KB, bool ZERO = true>
__device__ __forceinline__ void gemm_mainloop(const T* __restrict__ A, int lda, const T* __restrict__ B, int ldb,
                                              int M, int N, int K, int m0, int n0, v16f (&acc)[TA][TB], char* smem) {
  if constexpr (sizeof(T) == 2 && KB == 128) {
    gemm_mainloop_dl<WM, WN, TA, TB, ZERO>(A, lda, B, ldb, M, N, K, m0, n0, acc, smem);
    return;
  }
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
