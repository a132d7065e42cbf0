// Vocabulary projection + log-softmax + cross-entropy (Eq. 1), forward and backward, one slab of target
// positions at a time (the whole batch up to CE_SLAB_MAX_ROWS positions, larger batches in several slabs,
// so the slab buffers stop growing with the batch); the logits are contracted exactly once:
//   ce_fwd_kernel : logits of a 256 x 256 tile on the matrix cores; per target position and group of
//                   64 vocabulary entries the maximum m, the sum of e = exp(z - m) and the label's
//                   logit are kept, and e itself is stored (transposed, [V, slab rows]) in the
//                   operand type (a multiplicative quantity, so bf16 keeps its relative precision
//                   whatever the logit's magnitude);
//   ce_row_kernel : row log-sum-exp from the partials, masked negative log-likelihood;
//   ce_scale_kernel: dz^T = (e^T * exp(m - lse) - q) * mask / n_tok with q the target distribution
//                   (onehot, or smoothed: (1 - eps) onehot + eps / V), elementwise, in place, plus
//                   dz (through LDS), so that dH_o = dz W_o and dW_o += dz^T H_o are plain
//                   k-contiguous GEMMs.
#include "gemm_core.h"
#include "kernels.h"

namespace cmt {

using CeG = GemmBig;                                      // 256 x 256 logit tile, 16 wavefronts of 64 x 64
int ce_num_partials(int V) { return 4 * ((V + CeG::BN - 1) / CeG::BN); }

// The tile is computed transposed — vocabulary rows on the matrix cores' row side, target positions
// on the column side — so that in the accumulator layout a lane holds 32 vocabulary entries of ONE
// target position (two 32x32 tiles x 16 registers) and the other 32 of the wavefront's 64 sit in the
// lane 32 away: the row statistics need one cross-lane exchange instead of a 32-lane butterfly.
template <typename T>
__global__ __launch_bounds__(CeG::NT) void ce_fwd_kernel(const T* __restrict__ Ho, int ldho, const T* __restrict__ Wo,
                                                         const float* __restrict__ Bo, const int32_t* __restrict__ labels,
                                                         int M, int V, int H, T* __restrict__ ET, int ldet,
                                                         float* __restrict__ pmax, float* __restrict__ psum,
                                                         float* __restrict__ psz, float* __restrict__ zy, int np, RowLimit lim) {
  __shared__ __align__(16) char smem[CeG::SMEM_BYTES];    // main-loop stages; afterwards the staged e tile
  if (lim.n) M = min(M, max(*lim.n - lim.base, 0));       // rows that exist (uniform over the grid)
  if (M <= 0) return;
  int v0, r0;                                             // tile: vocabulary rows v0.., target positions r0..
  if (!gemm_tile_of_block((V + CeG::BM - 1) / CeG::BM, (M + CeG::BN - 1) / CeG::BN, CeG::BM, CeG::BN, v0, r0)) return;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wm = w >> 2, wn = w & 3;
  // the accumulators start from the bias of their vocabulary entries, so the main loop leaves the logits
  v16f acc[2][2];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int v = v0 + wm * 64 + mt * 32 + acc32_row(lane, i);
      const float bv = v < V ? Bo[v] : 0.f;
      acc[mt][0][i] = bv; acc[mt][1][i] = bv;
    }
  gemm_mainloop<T, 4, 4, 2, 2, 128, false>(Wo, H, Ho, ldho, V, M, H, v0, r0, acc, smem);   // ends with a barrier: LDS is free
  const int pidx = (v0 >> 6) + wm;                        // this wavefront's group of 64 vocabulary entries
  // e leaves through LDS: every wavefront stages its 64 vocabulary entries x 64 (fp32: 32) target positions
  // and writes them out as whole rows of E^T — 128 contiguous bytes per row instead of the 64-byte pieces of
  // the accumulator layout
  constexpr int NTS = sizeof(T) == 2 ? 2 : 1;             // 32-position halves staged together
  constexpr int SROW = 32 * NTS * (int)sizeof(T) + 16;    // staged row pitch in bytes (padded against bank conflicts)
  char* stage = smem + w * (64 * SROW);
  static_assert(16 * 64 * SROW <= CeG::SMEM_BYTES, "staging area exceeds the kernel's LDS");
  // The epilogue handles 64 logits per lane with a handful of vector instructions each (it is bound by their
  // count, not by memory): the vocabulary bound is tested only in the tile that contains it, the label's logit is
  // picked outside the loops, and the 16-bit path uses the hardware exponential and the packed bf16 conversion.
  const bool ragged = v0 + CeG::BM > V;                   // uniform: the tile reaches past the vocabulary
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int r = r0 + wn * 64 + nt * 32 + (lane & 31);
    const int y = r < M ? labels[r] : -1;
    float mx = -INFINITY, sz = 0.f;
    if (ragged) {                                         // entries past the vocabulary: logit -inf, e = 0
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (v0 + wm * 64 + mt * 32 + acc32_row(lane, i) >= V) acc[mt][nt][i] = -INFINITY;
    }
    if (psz) {                                            // label smoothing needs the mean logit of the row
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) sz += acc[mt][nt][i] > -INFINITY ? acc[mt][nt][i] : 0.f;
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc[mt][nt][i]);
    // the label's logit: entry yl of this wavefront's 64 sits in register (yl / 32, 4 (yl % 32 / 8) + yl % 4) of the
    // one of the two lanes sharing position r whose half (lane / 32) equals (yl / 4) % 2
    const int yl = y - v0 - wm * 64;
    if (y >= 0 && yl >= 0 && yl < 64 && ((yl >> 2) & 1) == (lane >> 5)) {
      const int want = (yl >> 5) * 16 + ((yl & 31) >> 3) * 4 + (yl & 3);
      float zlab = 0.f;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) zlab = (mt * 16 + i == want) ? acc[mt][nt][i] : zlab;
      zy[r] = zlab;
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float ms = mx > -INFINITY ? mx : 0.f;           // a group wholly past the vocabulary: exp(-inf - 0) = 0
    float e = 0.f;
    char* srow = stage + ((nt % NTS) * 32 + (lane & 31)) * sizeof(T);
    if constexpr (sizeof(T) == 2) {
      typedef float f32x2 __attribute__((ext_vector_type(2)));
      typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const f32x2 ev = {__expf(acc[mt][nt][i] - ms), __expf(acc[mt][nt][i + 1] - ms)};
          e += ev[0] + ev[1];
          const bf16x2 eb = __builtin_convertvector(ev, bf16x2);   // round to nearest even, one instruction per pair
          const int vl = mt * 32 + acc32_row(lane, i);             // i even: entries i and i + 1 are rows vl and vl + 1
          *reinterpret_cast<__bf16*>(srow + vl * SROW) = eb[0];
          *reinterpret_cast<__bf16*>(srow + (vl + 1) * SROW) = eb[1];
        }
    } else {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float ev = expf(acc[mt][nt][i] - ms);
          e += ev;
          *reinterpret_cast<float*>(srow + (mt * 32 + acc32_row(lane, i)) * SROW) = ev;
        }
    }
    if (nt % NTS == NTS - 1) {                            // a staged block is complete: 64 rows of 32 * NTS positions
      __syncthreads();
      constexpr int CPR = 32 * NTS * (int)sizeof(T) / 16; // 16-byte chunks per staged row
      constexpr int RPP = 64 / CPR;                       // rows per pass
      const int rbase = r0 + wn * 64 + (nt / NTS) * 32 * NTS;
#pragma unroll 2
      for (int ps = 0; ps < 64 / RPP; ++ps) {
        const int vl = ps * RPP + lane / CPR, ch = lane % CPR;
        const int v = v0 + wm * 64 + vl;
        // rows past M (inside the slab buffer, pitch ldet >= the tile's extent) hold values nobody reads
        if (v < V)
          *reinterpret_cast<uint4*>(ET + (size_t)v * ldet + rbase + ch * (16 / (int)sizeof(T))) =
              *reinterpret_cast<const uint4*>(stage + vl * SROW + ch * 16);
      }
      if (nt + 1 < 2) __syncthreads();                    // the staging area is reused by the next half
    }
    e += __shfl_xor(e, 32, 64);
    if (psz) sz += __shfl_xor(sz, 32, 64);
    if (lane < 32 && r < M) {                             // partials are kept [group][position]: 32 lanes, 128 bytes
      pmax[(size_t)pidx * ldet + r] = mx;
      psum[(size_t)pidx * ldet + r] = e;
      if (psz) psz[(size_t)pidx * ldet + r] = sz;
    }
  }
}

void launch_ce_fwd(int prec, const void* Ho, int ldho, const void* Wo, const float* Bo, const int32_t* labels,
                   int M, int V, int H, void* ET, int pitch, float* pmax, float* psum, float* psz, float* zy, hipStream_t st,
                   RowLimit lim) {
  const int ntv = (V + CeG::BM - 1) / CeG::BM, ntr = (M + CeG::BN - 1) / CeG::BN;
  const int grid = ((ntv * ntr + 7) / 8) * 8;
  const int np = ce_num_partials(V);
  if (prec)
    hipLaunchKernelGGL(ce_fwd_kernel<bf16_t>, dim3(grid), dim3(CeG::NT), 0, st, (const bf16_t*)Ho, ldho, (const bf16_t*)Wo, Bo,
                       labels, M, V, H, (bf16_t*)ET, pitch, pmax, psum, psz, zy, np, lim);
  else
    hipLaunchKernelGGL(ce_fwd_kernel<float>, dim3(grid), dim3(CeG::NT), 0, st, (const float*)Ho, ldho, (const float*)Wo, Bo,
                       labels, M, V, H, (float*)ET, pitch, pmax, psum, psz, zy, np, lim);
}

// Combines the partials (kept [group][position], row pitch `pitch`) of 32 target positions per workgroup: thread
// t takes position t % 32 and every 32nd group from t / 32 on, so that a half-wavefront reads 32 consecutive
// positions of one group; the 32 group strands of a position meet in LDS, in a fixed order.  Row loss
// against the smoothed target distribution (1 - eps) onehot(y) + eps / V:
// (1 - eps) (lse - z_y) + eps (lse - mean_v z_v); eps = 0: plain nll.
constexpr int CE_ROW_STRANDS = 32, CE_ROW_ROWS = 32;
__device__ __forceinline__ float ce_row_meet(float (&red)[CE_ROW_STRANDS][CE_ROW_ROWS], int pg, int rl, float v, bool take_max) {
  red[pg][rl] = v;
  __syncthreads();
  float r = red[0][rl];
#pragma unroll
  for (int k = 1; k < CE_ROW_STRANDS; ++k) r = take_max ? fmaxf(r, red[k][rl]) : r + red[k][rl];
  __syncthreads();
  return r;
}
__global__ __launch_bounds__(CE_ROW_ROWS * CE_ROW_STRANDS) void ce_row_kernel(const float* __restrict__ pmax, const float* __restrict__ psum,
                                                                    const float* __restrict__ psz, const float* __restrict__ zy,
                                                                    const float* __restrict__ mask, int M, int np, int pitch, float eps, int V,
                                                                    float* __restrict__ lse, float* __restrict__ nll, RowLimit lim) {
  __shared__ float red[CE_ROW_STRANDS][CE_ROW_ROWS];
  const int rl = threadIdx.x % CE_ROW_ROWS, pg = threadIdx.x / CE_ROW_ROWS;
  const int row = blockIdx.x * CE_ROW_ROWS + rl;
  if (lim.n) M = min(M, max(*lim.n - lim.base, 0));
  if (blockIdx.x * CE_ROW_ROWS >= M) return;
  const bool ok = row < M;
  float mx = -INFINITY;
  if (ok) {
#pragma unroll 4
    for (int p = pg; p < np; p += CE_ROW_STRANDS) mx = fmaxf(mx, pmax[(size_t)p * pitch + row]);
  }
  mx = ce_row_meet(red, pg, rl, mx, true);
  float s = 0.f, sz = 0.f;
  if (ok) {
#pragma unroll 4
    for (int p = pg; p < np; p += CE_ROW_STRANDS) {
      const float pm = pmax[(size_t)p * pitch + row];
      const float ps = psum[(size_t)p * pitch + row];
      if (pm > -INFINITY) s += ps * expf(pm - mx);
      if (eps > 0.f) sz += psz[(size_t)p * pitch + row];
    }
  }
  s = ce_row_meet(red, pg, rl, s, false);
  if (eps > 0.f) sz = ce_row_meet(red, pg, rl, sz, false);
  if (pg == 0 && ok) {
    const float l = mx + logf(s);
    lse[row] = l;
    float r = l - zy[row];
    if (eps > 0.f) r = (1.f - eps) * r + eps * (l - sz / (float)V);
    nll[row] = !mask || mask[row] > 0.f ? r : 0.f;
  }
}

// single block: the valid target positions (mask > 0), taken in time-major order, get consecutive
// indices, so that the output layer works on a dense row set: pos[r] = index of row r or -1,
// row[c] = the row behind index c, labels_c / rowscale_c = label and 1 / n_tok per index,
// *n_valid = loss[1] = n_tok.  Needs only the lengths, so it runs before the encoder.
__global__ __launch_bounds__(1024) void ce_compact_kernel(const float* __restrict__ mask, const int32_t* __restrict__ labels, int M,
                                                          int32_t* __restrict__ pos, int32_t* __restrict__ row,
                                                          int32_t* __restrict__ labels_c, float* __restrict__ rowscale_c,
                                                          int32_t* __restrict__ n_valid, float* __restrict__ loss) {
  __shared__ int s_scan[2][1024];
  const int t = threadIdx.x;
  const int per = (M + 1023) / 1024;
  const int r0 = min(M, t * per), r1 = min(M, r0 + per);
  int c = 0;
  for (int r = r0; r < r1; ++r) c += mask[r] > 0.f;
  s_scan[0][t] = c;
  __syncthreads();
  int cur = 0;
  for (int o = 1; o < 1024; o <<= 1) {                    // inclusive scan of the per-thread counts
    s_scan[cur ^ 1][t] = s_scan[cur][t] + (t >= o ? s_scan[cur][t - o] : 0);
    cur ^= 1;
    __syncthreads();
  }
  const int total = s_scan[cur][1023];
  const float inv = total > 0 ? 1.0f / (float)total : 0.f;
  int idx = s_scan[cur][t] - c;
  for (int r = r0; r < r1; ++r) {
    if (mask[r] > 0.f) {
      pos[r] = idx; row[idx] = r; labels_c[idx] = labels[r]; rowscale_c[idx] = inv;
      ++idx;
    } else {
      pos[r] = -1;
    }
  }
  if (t == 0) { *n_valid = total; loss[1] = (float)total; }
}

// dst[c, :] = src[row[c], :] for c < *n_valid (cols * sizeof(T) and the pitches are multiples of 16 bytes).
// Rows from *n_valid up to the next multiple of 64 are zero-filled: the weight-gradient contraction
// dW_o = dz^T H_o runs over whole blocks of 64 rows, and its other operand is zero there, so these
// rows must hold numbers, whatever the workspace held before.
template <typename T>
__global__ __launch_bounds__(128) void ce_gather_rows_kernel(const T* __restrict__ src, int lds, const int32_t* __restrict__ row,
                                                             const int32_t* __restrict__ n_valid, T* __restrict__ dst, int ldd,
                                                             int cols) {
  const int c = blockIdx.x;
  const int n = *n_valid;
  if (c >= (n + 63) / 64 * 64) return;
  constexpr int VE = 16 / sizeof(T);
  T* d = dst + (size_t)c * ldd;
  if (c >= n) {
    for (int k = threadIdx.x * VE; k < cols; k += 128 * VE) *reinterpret_cast<uint4*>(d + k) = make_uint4(0, 0, 0, 0);
    return;
  }
  const T* s = src + (size_t)row[c] * lds;
  for (int k = threadIdx.x * VE; k < cols; k += 128 * VE) *reinterpret_cast<uint4*>(d + k) = *reinterpret_cast<const uint4*>(s + k);
}
void launch_ce_gather_rows(int prec, const void* src, int lds, const int32_t* row, const int32_t* n_valid, int max_rows, void* dst,
                           int ldd, int cols, hipStream_t st) {
  if (max_rows <= 0) return;
  if (prec) hipLaunchKernelGGL(ce_gather_rows_kernel<bf16_t>, dim3(max_rows), dim3(128), 0, st, (const bf16_t*)src, lds, row, n_valid,
                               (bf16_t*)dst, ldd, cols);
  else hipLaunchKernelGGL(ce_gather_rows_kernel<float>, dim3(max_rows), dim3(128), 0, st, (const float*)src, lds, row, n_valid,
                          (float*)dst, ldd, cols);
}

// single block: loss = sum nll / n_tok, summed in a fixed order
__global__ __launch_bounds__(1024) void ce_loss_kernel(const float* __restrict__ nll, int M, float* __restrict__ loss,
                                                       int* __restrict__ flags, RowLimit lim) {
  __shared__ float s_sum[1024];
  const int t = threadIdx.x;
  if (lim.n) M = min(M, max(*lim.n - lim.base, 0));
  float a = 0.f;
  for (int r = t; r < M; r += 1024) a += nll[r];
  s_sum[t] = a;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (t < o) s_sum[t] += s_sum[t + o];
    __syncthreads();
  }
  if (t == 0) {
    const float ntok = loss[1];
    const float l = ntok > 0.f ? s_sum[0] / ntok : 0.f;
    loss[0] = l;
    if (!isfinite(l)) atomicOr(flags, 4);
  }
}

void launch_ce_compact(const float* mask, const int32_t* labels, int M, int32_t* pos, int32_t* row, int32_t* labels_c,
                       float* rowscale_c, int32_t* n_valid, float* loss, hipStream_t st) {
  hipLaunchKernelGGL(ce_compact_kernel, dim3(1), dim3(1024), 0, st, mask, labels, M, pos, row, labels_c, rowscale_c, n_valid, loss);
}
void launch_ce_rows(const float* pmax, const float* psum, const float* psz, const float* zy, const float* mask, int M, int np,
                    int pitch, float eps, int V, float* lse, float* nll, hipStream_t st, RowLimit lim) {
  hipLaunchKernelGGL(ce_row_kernel, dim3((M + CE_ROW_ROWS - 1) / CE_ROW_ROWS), dim3(CE_ROW_ROWS * CE_ROW_STRANDS), 0, st, pmax, psum,
                     psz, zy, mask, M, np, pitch, eps, V, lse, nll, lim);
}
void launch_ce_loss(const float* nll, int M, float* loss, int* flags, hipStream_t st, RowLimit lim) {
  hipLaunchKernelGGL(ce_loss_kernel, dim3(1), dim3(1024), 0, st, nll, M, loss, flags, lim);
}

// ------------------------------------------------------------------------------------------------
// e^T -> dz^T in place, dz through an LDS transpose, and per block of 64 target positions the column
// sums of dz (partial dB_o, summed by the caller in a fixed order).  One workgroup per 64 vocabulary
// entries (= one group of partials) x 64 target positions: thread t first takes vocabulary entry
// t / 4 and 16 consecutive positions, then position t / 4 and 16 consecutive vocabulary entries, so
// that both matrices move as 16-byte vectors.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ce_scale_kernel(T* __restrict__ ET, int ldet, int V, int Mc, const float* __restrict__ pmax,
                                                       int np, const float* __restrict__ lse, const int32_t* __restrict__ labels,
                                                       const float* __restrict__ rowscale, float eps, T* __restrict__ dz,
                                                       float* __restrict__ dbo_part, RowLimit lim) {
  constexpr int VE = 16 / sizeof(T);                      // elements per 16-byte vector
  constexpr int NV = 16 / VE;                             // vectors per thread
  __shared__ __align__(16) T tile[64][64 + VE];           // [position][vocabulary entry]
  __shared__ __align__(16) float sf[64], srs[64];
  __shared__ __align__(16) int sy[64];
  const int v0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int t = threadIdx.x;
  if (lim.n) Mc = min(Mc, max(*lim.n - lim.base, 0));
  if (r0 >= Mc) {                                         // a block of rows that does not exist: its share of dB_o is zero
    const int v = v0 + (t >> 2);
    if ((t & 3) == 0 && v < V) dbo_part[(size_t)blockIdx.y * V + v] = 0.f;
    return;
  }
  // dz = (e * f - q) * rs with f = exp(m - lse), q = (1 - eps) onehot + eps / V, rs = mask / n_tok, as one
  // multiply-add per element: dz = e * sa - (sb + [label] * sc), sa = f rs, sb = eps / V rs, sc = (1 - eps) rs
  // (rows that do not exist: all three zero)
  const float epsv = eps / (float)V;
  if (t < 64) {
    const int r = r0 + t;
    float f = 0.f, rs = 0.f;
    int y = -1;
    if (r < Mc) {
      const float pm = pmax[(size_t)blockIdx.x * ldet + r];
      f = pm > -INFINITY ? expf(pm - lse[r]) : 0.f;
      rs = rowscale[r];
      y = labels[r];
    }
    sf[t] = f * rs; srs[t] = rs; sy[t] = y;
  }
  __syncthreads();
  {
    const int vl = t >> 2, v = v0 + vl, rb = (t & 3) * 16;
    const bool edge = r0 + 64 > Mc;                       // uniform: the block holds rows that do not exist
    float cs = 0.f;                                       // this block's share of dB_o[v]: 64 positions in fixed order
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      T x[VE];
      if (v < V) *reinterpret_cast<uint4*>(x) = *reinterpret_cast<const uint4*>(ET + (size_t)v * ldet + r0 + rb + q * VE);
      else *reinterpret_cast<uint4*>(x) = make_uint4(0, 0, 0, 0);
      float a[VE], rs[VE];
      int y[VE];
      *reinterpret_cast<uint4*>(a) = *reinterpret_cast<const uint4*>(&sf[rb + q * VE]);
      *reinterpret_cast<uint4*>(rs) = *reinterpret_cast<const uint4*>(&srs[rb + q * VE]);
      *reinterpret_cast<uint4*>(y) = *reinterpret_cast<const uint4*>(&sy[rb + q * VE]);
      if constexpr (VE == 8) {
        *reinterpret_cast<uint4*>(a + 4) = *reinterpret_cast<const uint4*>(&sf[rb + q * VE + 4]);
        *reinterpret_cast<uint4*>(rs + 4) = *reinterpret_cast<const uint4*>(&srs[rb + q * VE + 4]);
        *reinterpret_cast<uint4*>(y + 4) = *reinterpret_cast<const uint4*>(&sy[rb + q * VE + 4]);
      }
      float d[VE];
#pragma unroll
      for (int j = 0; j < VE; ++j) {
        const float e = edge && r0 + rb + q * VE + j >= Mc ? 0.f : to_f<T>(x[j]);   // (what such rows hold is anything)
        d[j] = v < V ? fmaf(e, a[j], -(epsv * rs[j] + (y[j] == v ? (1.f - eps) * rs[j] : 0.f))) : 0.f;
      }
      if constexpr (sizeof(T) == 2) {
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int j = 0; j < VE; j += 2) {                 // round to nearest even, one instruction per pair
          const f32x2 dv = {d[j], d[j + 1]};
          const bf16x2 db = __builtin_convertvector(dv, bf16x2);
          *reinterpret_cast<bf16x2*>(&x[j]) = db;
        }
      } else {
#pragma unroll
        for (int j = 0; j < VE; ++j) x[j] = from_f<T>(d[j]);
      }
#pragma unroll
      for (int j = 0; j < VE; ++j) {
        cs += to_f<T>(x[j]);
        tile[rb + q * VE + j][vl] = x[j];
      }
      if (v < V) *reinterpret_cast<uint4*>(ET + (size_t)v * ldet + r0 + rb + q * VE) = *reinterpret_cast<const uint4*>(x);
    }
    cs += __shfl_xor(cs, 1, 64);
    cs += __shfl_xor(cs, 2, 64);
    if ((t & 3) == 0 && v < V) dbo_part[(size_t)blockIdx.y * V + v] = cs;
  }
  __syncthreads();
  {
    const int rl = t >> 2, r = r0 + rl, vb = (t & 3) * 16;
    if (r < Mc) {
#pragma unroll
      for (int q = 0; q < NV; ++q)
        if (v0 + vb + q * VE < V)
          *reinterpret_cast<uint4*>(dz + (size_t)r * V + v0 + vb + q * VE) = *reinterpret_cast<const uint4*>(&tile[rl][vb + q * VE]);
    }
  }
}

void launch_ce_scale(int prec, void* ET, int pitch, int V, int Mc, const float* pmax, const float* lse, const int32_t* labels,
                     const float* rowscale, float eps, void* dz, float* dbo_part, hipStream_t st, RowLimit lim) {
  dim3 grid((V + 63) / 64, (Mc + 63) / 64);
  const int np = ce_num_partials(V);
  if (prec)
    hipLaunchKernelGGL(ce_scale_kernel<bf16_t>, grid, dim3(256), 0, st, (bf16_t*)ET, pitch, V, Mc, pmax, np, lse, labels,
                       rowscale, eps, (bf16_t*)dz, dbo_part, lim);
  else
    hipLaunchKernelGGL(ce_scale_kernel<float>, grid, dim3(256), 0, st, (float*)ET, pitch, V, Mc, pmax, np, lse, labels,
                       rowscale, eps, (float*)dz, dbo_part, lim);
}

}  // namespace cmt
