// Batched-over-time GEMMs of the training step (the paper's LinearLayer forward / backward /
// calculateGradient, Fig. "Codes of Performing Actual Computation"), all in the single
// "A * B^T, both k-contiguous" form, plus the tiled transpose that brings the backward and
// weight-gradient operands into that form.
#include "gemm_core.h"
#include "kernels.h"
#include <algorithm>
#include <cstdlib>
#include <vector>

namespace cmt {

// Dispatch thresholds, from measurements on MI355X (bf16, k = 1024 .. 4096): with 208 tiles of
// 256 x 256 the big tile already wins (628 against 546 TFLOP/s), with 128 it loses.
static int env_int(const char* name, int dflt) {
  const char* e = getenv(name);
  return e && *e ? atoi(e) : dflt;
}
static const int GEMM_BIG_MIN_TILES = env_int("CMT_GEMM_BIG_MIN_TILES", 192);
static const int GEMM_SPLIT_BELOW = env_int("CMT_GEMM_SPLIT_BELOW", 129);
static const int GEMM_SPLIT_TARGET = env_int("CMT_GEMM_SPLIT_TARGET", 512);
static const int GEMM_SPLIT_MAX = env_int("CMT_GEMM_SPLIT_MAX", 16);
static const int GEMM_BIGSPLIT_MIN_K = env_int("CMT_GEMM_BIGSPLIT_MIN_K", 8192);
// beyond this many big tiles (by the host's row count) the small tile without a split measured faster (large
// workload: 160 tiles, 3.15 against 3.57 ms for the output layer)
static const int GEMM_BIGSPLIT_MAX_TILES = env_int("CMT_GEMM_BIGSPLIT_MAX_TILES", 96);


// Number of k splits when the row count is known to the device alone: as many as make one round of workgroups
// over the chip's 256 CUs out of the tiles that exist, at most the launched number.  The kernel and the plane
// sum both derive it from the same count.
__host__ __device__ inline int gemm_dyn_splits(int tiles, int launched) {
  const int ns = 256 / (tiles > 0 ? tiles : 1);
  return ns < 1 ? 1 : (ns > launched ? launched : ns);
}

// One output tile (the one of virtual workgroup id vb) of C (+)= A B^T (+ bias): main loop and store.
template <typename T, int WM, int WN, int TA, int TB, int KB>
__device__ __forceinline__ void gemm_nt_tile(const T* __restrict__ A, int lda, const T* __restrict__ B, int ldb, int M, int N, int K,
                                             float* __restrict__ Cf0, T* __restrict__ Ct, int ldc, const float* __restrict__ bias,
                                             int accumulate, int ntn, int kchunk, size_t plane_stride, int dyn_split, int vb,
                                             char* smem) {
  using G = GemmTile<WM, WN, TA, TB, KB>;
  int m0, n0;
  if (!gemm_tile_of_block((M + G::BM - 1) / G::BM, ntn, G::BM, G::BN, m0, n0, vb)) return;
  if (dyn_split) {                                 // the number of k splits follows the tiles that exist: one round of workgroups
    const int ns = gemm_dyn_splits((M + G::BM - 1) / G::BM * ntn, gridDim.y);
    if ((int)blockIdx.y >= ns) return;
    kchunk = ((K + ns - 1) / ns + 63) / 64 * 64;
  }
  const int k0 = blockIdx.y * kchunk;
  const int klen = min(kchunk, K - k0);
  if (klen <= 0 && gridDim.y == 1) return;
  v16f acc[TA][TB];
  gemm_mainloop<T, WM, WN, TA, TB, KB>(A + k0, lda, B + k0, ldb, M, N, klen, m0, n0, acc, smem);
  float* const Cf = gridDim.y > 1 ? Cf0 + blockIdx.y * plane_stride : Cf0;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wm = w / WN, wn = w % WN;
#pragma unroll
  for (int nt = 0; nt < TB; ++nt) {
    const int col = n0 + wn * 32 * TB + nt * 32 + (lane & 31);
    if (col >= N) continue;
    const float bv = bias ? bias[col] : 0.f;
#pragma unroll
    for (int mt = 0; mt < TA; ++mt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = m0 + wm * 32 * TA + mt * 32 + acc32_row(lane, i);
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

// blockIdx.y = k split index: each split contracts kchunk elements of k and, when there is more
// than one, writes its own fp32 plane Cf + split * plane_stride (summed afterwards, fixed order).
// WALK: the launch has fewer workgroups than tiles (it is to leave part of the chip to other streams) and every
// workgroup walks the tiles of the virtual ids blockIdx.x, blockIdx.x + grid, ...  It is a variant of its own because
// the loop costs the one-tile-per-workgroup kernel a spilled register.
template <typename T, int WM, int WN, int TA, int TB, int KB, bool WALK = false>
__global__ __launch_bounds__(64 * WM * WN) void gemm_nt_kernel(const T* __restrict__ A, int lda, const T* __restrict__ B, int ldb,
                                                               int M, int N, int K, float* __restrict__ Cf0, T* __restrict__ Ct,
                                                               int ldc, const float* __restrict__ bias, int accumulate, int ntn,
                                                               int kchunk, size_t plane_stride, RowLimit lim, int lim_kind,
                                                               int dyn_split) {
  using G = GemmTile<WM, WN, TA, TB, KB>;
  __shared__ __align__(16) char smem[G::SMEM_BYTES];
  if (lim.n) {                                     // a bound that only the device knows (uniform over the grid)
    const int e = max(*lim.n - lim.base, 0);
    if (lim_kind == 1) M = min(M, e);
    else K = min(K, (e + 63) / 64 * 64);
    if (M <= 0 || K <= 0) return;
  }
  if constexpr (WALK) {
    const int ntiles8 = (((M + G::BM - 1) / G::BM * ntn + 7) >> 3) << 3;
    for (int vb = blockIdx.x; vb < ntiles8; vb += gridDim.x) {
      gemm_nt_tile<T, WM, WN, TA, TB, KB>(A, lda, B, ldb, M, N, K, Cf0, Ct, ldc, bias, accumulate, ntn, kchunk, plane_stride, dyn_split,
                                          vb, smem);
      __syncthreads();                             // (the next tile refills the LDS)
    }
  } else {
    gemm_nt_tile<T, WM, WN, TA, TB, KB>(A, lda, B, ldb, M, N, K, Cf0, Ct, ldc, bias, accumulate, ntn, kchunk, plane_stride, dyn_split,
                                        (int)blockIdx.x, smem);
  }
}

// out = sum of planes (+ bias per column) (+ previous out).  VEC = 4: four consecutive columns per thread as one
// 16-byte access per plane (N, ldc and the plane stride multiples of 4, all bases 16-byte aligned).
template <int VEC>
__global__ __launch_bounds__(256) void gemm_planes_sum_kernel(const float* __restrict__ planes, int np, size_t stride,
                                                              float* __restrict__ out, int M, int N, int ldc,
                                                              const float* __restrict__ bias, int accumulate, RowLimit lim,
                                                              int dyn_bm, int dyn_ntn) {
  if (lim.n) M = min(M, max(*lim.n - lim.base, 0));
  if (dyn_bm) np = gemm_dyn_splits((M + dyn_bm - 1) / dyn_bm * dyn_ntn, np);   // the planes the GEMM wrote
  const unsigned nq = (unsigned)N / VEC;                  // column groups per row
  const size_t n = (size_t)M * nq;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const unsigned r = (unsigned)(i / nq), c = ((unsigned)i - r * nq) * VEC;
    const float* src = planes + (size_t)r * N + c;
    float* o = out + (size_t)r * ldc + c;
    if (VEC == 4) {
      float4 v = bias ? *reinterpret_cast<const float4*>(bias + c) : make_float4(0.f, 0.f, 0.f, 0.f);
      for (int p = 0; p < np; ++p) {
        const float4 a = *reinterpret_cast<const float4*>(src + (size_t)p * stride);
        v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
      }
      if (accumulate) {
        const float4 a = *reinterpret_cast<const float4*>(o);
        v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
      }
      *reinterpret_cast<float4*>(o) = v;
    } else {
      float v = bias ? bias[c] : 0.f;
      for (int p = 0; p < np; ++p) v += src[(size_t)p * stride];
      *o = accumulate ? *o + v : v;
    }
  }
}

static void launch_planes_sum(const float* planes, int nks, size_t pstride, float* Cf, int M, int N, int ldc, const float* bias,
                              int accumulate, RowLimit rl, hipStream_t st, int dyn_bm = 0, int dyn_ntn = 0) {
  const bool vec = N % 4 == 0 && ldc % 4 == 0 && pstride % 4 == 0 && ((size_t)Cf | (size_t)planes | (size_t)bias) % 16 == 0;
  size_t g = (pstride / (vec ? 4 : 1) + 255) / 256;
  if (g > 4096) g = 4096;
  if (vec)
    hipLaunchKernelGGL(gemm_planes_sum_kernel<4>, dim3((unsigned)g), dim3(256), 0, st, planes, nks, pstride, Cf, M, N, ldc, bias,
                       accumulate, rl, dyn_bm, dyn_ntn);
  else
    hipLaunchKernelGGL(gemm_planes_sum_kernel<1>, dim3((unsigned)g), dim3(256), 0, st, planes, nks, pstride, Cf, M, N, ldc, bias,
                       accumulate, rl, dyn_bm, dyn_ntn);
}

template <typename T, int WM, int WN, int TA, int TB>
static void gemm_go(dim3 grid, hipStream_t st, const void* A, int lda, const void* B, int ldb, int M, int N, int K, float* out,
                    void* Ct, int ldc, const float* bias, int acc, int ntn, int kchunk, size_t pstride, RowLimit lim, int lim_kind,
                    int dyn_split = 0, int wg_cap = 0) {
  if (wg_cap > 0 && (int)grid.x > (wg_cap + 7) / 8 * 8) {
    grid.x = (wg_cap + 7) / 8 * 8;
    hipLaunchKernelGGL((gemm_nt_kernel<T, WM, WN, TA, TB, 128, true>), grid, dim3(64 * WM * WN), 0, st, (const T*)A, lda, (const T*)B, ldb,
                       M, N, K, out, (T*)Ct, ldc, bias, acc, ntn, kchunk, pstride, lim, lim_kind, dyn_split);
    return;
  }
  hipLaunchKernelGGL((gemm_nt_kernel<T, WM, WN, TA, TB, 128>), grid, dim3(64 * WM * WN), 0, st, (const T*)A, lda, (const T*)B, ldb,
                     M, N, K, out, (T*)Ct, ldc, bias, acc, ntn, kchunk, pstride, lim, lim_kind, dyn_split);
}

void launch_gemm_nt(int prec, const void* A, int lda, const void* B, int ldb, int M, int N, int K,
                    float* Cf, void* Ct, int ldc, const float* bias, int accumulate, hipStream_t st,
                    float* split_scratch, size_t split_scratch_floats, RowLimit lim, int lim_kind, int wg_cap) {
  if (M <= 0 || N <= 0) return;
  // enough 256 x 256 tiles to fill the chip: the big tile (half the L2 traffic per flop)
  const int ntm_b = (M + GemmBig::BM - 1) / GemmBig::BM, ntn_b = (N + GemmBig::BN - 1) / GemmBig::BN;
  if (ntm_b * ntn_b >= GEMM_BIG_MIN_TILES) {
    const int grid = ((ntm_b * ntn_b + 7) / 8) * 8;
    if (prec) gemm_go<bf16_t, 4, 4, 2, 2>(dim3(grid, 1), st, A, lda, B, ldb, M, N, K, Cf, Ct, ldc, bias, accumulate, ntn_b, K, 0, lim, lim_kind, 0, wg_cap);
    else gemm_go<float, 4, 4, 2, 2>(dim3(grid, 1), st, A, lda, B, ldb, M, N, K, Cf, Ct, ldc, bias, accumulate, ntn_b, K, 0, lim, lim_kind, 0, wg_cap);
    return;
  }
  // a long contraction over few output tiles (dH_o = dz W_o: k = the vocabulary): big tiles with k split into
  // planes.  With a device-side row limit the kernel picks the number of splits itself (gemm_dyn_splits) out of
  // the launched maximum; otherwise the host aims at about one and a half rounds of workgroups.
  if (split_scratch && Cf && !Ct && K >= GEMM_BIGSPLIT_MIN_K && ntm_b * ntn_b <= GEMM_BIGSPLIT_MAX_TILES) {
    const bool dyn = lim.n && lim_kind == 1;
    int ks = dyn ? GEMM_SPLIT_MAX : (384 + ntm_b * ntn_b - 1) / (ntm_b * ntn_b);
    if (ks > GEMM_SPLIT_MAX) ks = GEMM_SPLIT_MAX;
    while (ks > 1 && ((size_t)ks * M * N > split_scratch_floats || K / ks < 2048)) --ks;
    if (ks > 1 && (dyn || ks * ntm_b * ntn_b >= GEMM_BIG_MIN_TILES)) {     // else the small tile fills the chip better
      const int kchunk = ((K + ks - 1) / ks + 63) / 64 * 64;
      const int nks = dyn ? ks : (K + kchunk - 1) / kchunk;
      const size_t pstride = (size_t)M * N;
      const int grid = ((ntm_b * ntn_b + 7) / 8) * 8;
      if (prec) gemm_go<bf16_t, 4, 4, 2, 2>(dim3(grid, nks), st, A, lda, B, ldb, M, N, K, split_scratch, nullptr, N, nullptr, 0, ntn_b, kchunk, pstride, lim, lim_kind, dyn, wg_cap);
      else gemm_go<float, 4, 4, 2, 2>(dim3(grid, nks), st, A, lda, B, ldb, M, N, K, split_scratch, nullptr, N, nullptr, 0, ntn_b, kchunk, pstride, lim, lim_kind, dyn, wg_cap);
      launch_planes_sum(split_scratch, nks, pstride, Cf, M, N, ldc, bias, accumulate, lim_kind == 1 ? lim : RowLimit{}, st,
                        dyn ? GemmBig::BM : 0, ntn_b);
      return;
    }
  }
  using G = GemmSmall;
  const int ntm = (M + G::BM - 1) / G::BM, ntn = (N + G::BN - 1) / G::BN;
  const int nb = ntm * ntn;
  const int grid = ((nb + 7) / 8) * 8;
  const int esz = prec ? 2 : 4;
  const int bk = 128 / esz;
  // few output tiles but a long contraction: split k over workgroups (two workgroups per CU wanted)
  int ks = 1;
  if (split_scratch && Cf && !Ct && nb < GEMM_SPLIT_BELOW && K >= 16 * bk) {
    ks = (GEMM_SPLIT_TARGET + nb - 1) / nb;
    if (ks > GEMM_SPLIT_MAX) ks = GEMM_SPLIT_MAX;
    while (ks > 1 && ((size_t)ks * M * N > split_scratch_floats || K / ks < 4 * bk)) --ks;
  }
  int kchunk = K;
  if (ks > 1) kchunk = ((K + ks - 1) / ks + bk - 1) / bk * bk;
  const int nks = (K + kchunk - 1) / kchunk;
  const size_t pstride = (size_t)M * N;
  float* out = nks > 1 ? split_scratch : Cf;
  const int oldc = nks > 1 ? N : ldc;
  const float* obias = nks > 1 ? nullptr : bias;
  const int oacc = nks > 1 ? 0 : accumulate;
  if (prec) gemm_go<bf16_t, 2, 2, 2, 2>(dim3(grid, nks), st, A, lda, B, ldb, M, N, K, out, Ct, oldc, obias, oacc, ntn, kchunk, pstride, lim, lim_kind, 0, wg_cap);
  else gemm_go<float, 2, 2, 2, 2>(dim3(grid, nks), st, A, lda, B, ldb, M, N, K, out, Ct, oldc, obias, oacc, ntn, kchunk, pstride, lim, lim_kind, 0, wg_cap);
  if (nks > 1) launch_planes_sum(split_scratch, nks, pstride, Cf, M, N, ldc, bias, accumulate, lim_kind == 1 ? lim : RowLimit{}, st);
}

constexpr int GEMM_GROUP_MAX = 16;
struct GemmGroupArgs { int n; int tile_start[GEMM_GROUP_MAX + 1]; GemmProb p[GEMM_GROUP_MAX]; };

template <typename T, int WM, int WN, int TA, int TB>
__global__ __launch_bounds__(64 * WM * WN) void gemm_nt_group_kernel(GemmGroupArgs g) {
  using G = GemmTile<WM, WN, TA, TB, 128>;
  __shared__ __align__(16) char smem[G::SMEM_BYTES];
  // the workgroups walk the tile queue: workgroup v takes the tiles of the virtual ids v, v + grid, v + 2 grid, ...
  // (the grid is a multiple of 8, so a workgroup stays with the tile range of its XCD); a grid as large as the
  // queue is the plain one-tile-per-workgroup launch
  const int nt_all = g.tile_start[g.n], per = (nt_all + 7) >> 3;
  for (int vb = blockIdx.x; (vb >> 3) < per; vb += gridDim.x) {
  const int id = (vb & 7) * per + (vb >> 3);
  if (id >= nt_all) continue;
  int q = 0;
  while (q + 1 < g.n && id >= g.tile_start[q + 1]) ++q;   // uniform over the workgroup
  const GemmProb& pr = g.p[q];
  const int M = pr.M, N = pr.N, ldc = pr.ldc;
  int m0, n0;
  gemm_tile_from_index(id - g.tile_start[q], (M + G::BM - 1) / G::BM, (N + G::BN - 1) / G::BN, G::BM, G::BN, m0, n0);
  v16f acc[TA][TB];
  gemm_mainloop<T, WM, WN, TA, TB, 128>((const T*)pr.A, pr.lda, (const T*)pr.B, pr.ldb, M, N, pr.K, m0, n0, acc, smem);
  __syncthreads();                                        // (the next tile of a walking workgroup refills the LDS)
  float* __restrict__ C = pr.C;
  const int accumulate = pr.accumulate;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wm = w / WN, wn = w % WN;
#pragma unroll
  for (int nt = 0; nt < TB; ++nt) {
    const int col = n0 + wn * 32 * TB + nt * 32 + (lane & 31);
    if (col >= N) continue;
#pragma unroll
    for (int mt = 0; mt < TA; ++mt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = m0 + wm * 32 * TA + mt * 32 + acc32_row(lane, i);
        if (row >= M) continue;
        const size_t o = (size_t)row * ldc + col;
        C[o] = accumulate ? C[o] + acc[mt][nt][i] : acc[mt][nt][i];
      }
    }
  }
  }
}

template <typename T, int WM, int WN, int TA, int TB>
static void gemm_group_go(const GemmProb* probs, int n, hipStream_t st, int wg_cap) {
  using G = GemmTile<WM, WN, TA, TB, 128>;
  for (int c0 = 0; c0 < n; c0 += GEMM_GROUP_MAX) {
    GemmGroupArgs g{};
    g.n = std::min(GEMM_GROUP_MAX, n - c0);
    int nt = 0;
    for (int i = 0; i < g.n; ++i) {
      g.p[i] = probs[c0 + i];
      g.tile_start[i] = nt;
      nt += ((g.p[i].M + G::BM - 1) / G::BM) * ((g.p[i].N + G::BN - 1) / G::BN);
    }
    g.tile_start[g.n] = nt;
    if (nt == 0) continue;
    int grid = ((nt + 7) / 8) * 8;
    if (wg_cap > 0 && grid > (wg_cap + 7) / 8 * 8) grid = (wg_cap + 7) / 8 * 8;
    hipLaunchKernelGGL((gemm_nt_group_kernel<T, WM, WN, TA, TB>), dim3(grid), dim3(64 * WM * WN), 0, st, g);
  }
}

void launch_gemm_nt_group(int prec, const GemmProb* probs, int n, hipStream_t st, float* split_scratch, size_t split_scratch_floats,
                          int wg_cap) {
  if (!prec) {
    // fp32 operands: one launch per problem, k split over workgroups where there are few tiles.  These GEMMs are
    // matrix-core bound either way, and the shorter workgroups of the split form leave the CUs sooner to the
    // recurrences' kernels running beside them (small workload: 11.2 against 11.4 ms per step).
    for (int i = 0; i < n; ++i)
      launch_gemm_nt(prec, probs[i].A, probs[i].lda, probs[i].B, probs[i].ldb, probs[i].M, probs[i].N, probs[i].K, probs[i].C, nullptr,
                     probs[i].ldc, nullptr, probs[i].accumulate, st, split_scratch, split_scratch_floats, RowLimit{}, 0, wg_cap);
    return;
  }
  std::vector<GemmProb> live;
  long big = 0;
  for (int i = 0; i < n; ++i) {
    if (probs[i].M <= 0 || probs[i].N <= 0) continue;
    live.push_back(probs[i]);
    big += (long)((probs[i].M + GemmBig::BM - 1) / GemmBig::BM) * ((probs[i].N + GemmBig::BN - 1) / GemmBig::BN);
  }
  if (live.empty()) return;
  // enough 256 x 256 tiles over the whole group to fill the chip: the big tile, else the small one
  if (big >= GEMM_BIG_MIN_TILES) gemm_group_go<bf16_t, 4, 4, 2, 2>(live.data(), (int)live.size(), st, wg_cap);
  else gemm_group_go<bf16_t, 2, 2, 2, 2>(live.data(), (int)live.size(), st, wg_cap);
}

// Measurement aid: nothing but matrix-core instructions (4 independent 32x32x16 bf16 accumulator chains per
// wavefront, operands in registers), to read the rate the matrix cores reach on this chip beside the
// nominal peak.  out receives one value per lane so that the loop cannot be dropped.
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* __restrict__ out, int iters) {
  Frag<bf16_t> a, b;
  a.v = make_uint4(0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);
  b.v = make_uint4(0x3f803f80u, 0x3f803f80u + blockIdx.x, 0x3f803f80u, 0x3f803f80u);
  v16f acc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[q][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int q = 0; q < 4; ++q) mma32(acc[q], a, b);
  }
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[q][i];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}
double launch_mfma_rate(float* out, int blocks, int iters, hipStream_t st) {
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(256), 0, st, out, iters);
  return (double)blocks * 4 /*wavefronts*/ * iters * 4.0 * (2.0 * 32 * 32 * 16);
}

// 64x64 tiles through LDS; reads and writes are both row-contiguous.
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, int ldin, T* __restrict__ out, int ldout,
                                                        int R, int C) {
  __shared__ T tile[64][64 + 4 / sizeof(T)];             // row pitch of an odd number of 32-bit words: no bank conflicts in either pass
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
