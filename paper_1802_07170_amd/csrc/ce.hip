// Vocabulary projection + log-softmax + cross-entropy (Eq. 1), forward and backward, one slab of at
// most CE_SLAB_ROWS target positions at a time; the full [rows, vocabulary] matrix never exists and
// the logits are contracted exactly once:
//   ce_fwd_kernel : logits of a 256 x 256 tile on the matrix cores; per row and group of 64 columns
//                   the maximum m, the sum of e = exp(z - m) and the label's logit are kept, and e
//                   itself is stored in the operand type (a multiplicative quantity, so bf16 keeps
//                   its relative precision whatever the logit's magnitude);
//   ce_row_kernel : row log-sum-exp from the partials, masked negative log-likelihood;
//   ce_scale_kernel: dz = (e * exp(m - lse) - q) * mask / n_tok with q the target distribution
//                   (onehot, or smoothed: (1 - eps) onehot + eps / V), elementwise, in place, plus
//                   its transpose (through LDS), so that dH_o = dz W_o and dW_o += dz^T H_o are
//                   plain k-contiguous GEMMs.
#include "gemm_core.h"
#include "kernels.h"

namespace cmt {

using CeG = GemmBig;                                      // 256 x 256 logit tile, 16 wavefronts of 64 x 64
int ce_num_partials(int V) { return 4 * ((V + CeG::BN - 1) / CeG::BN); }
size_t ce_slab_elems(int V) { return (size_t)CE_SLAB_ROWS * V; }

template <typename T>
__global__ __launch_bounds__(CeG::NT) void ce_fwd_kernel(const T* __restrict__ Ho, int ldho, const T* __restrict__ Wo,
                                                         const float* __restrict__ Bo, const int32_t* __restrict__ labels,
                                                         int M, int V, int H, T* __restrict__ E, float* __restrict__ pmax,
                                                         float* __restrict__ psum, float* __restrict__ psz,
                                                         float* __restrict__ zy, int np, int ntn) {
  __shared__ __align__(16) char smem[CeG::SMEM_BYTES];
  const int per = gridDim.x >> 3;
  const int id = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  const int m0 = (id / ntn) * CeG::BM, n0 = (id % ntn) * CeG::BN;
  if (m0 >= M) return;
  v16f acc[2][2];
  gemm_mainloop<T, 4, 4, 2, 2, 128>(Ho, ldho, Wo, H, M, V, H, m0, n0, acc, smem);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wm = w >> 2, wn = w & 3;
  int col[2];
  float bo[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    col[b] = n0 + wn * 64 + b * 32 + (lane & 31);
    bo[b] = col[b] < V ? Bo[col[b]] : 0.f;
  }
  const int pidx = (n0 >> 6) + wn;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = m0 + wm * 64 + mt * 32 + acc32_row(lane, i);
      const int y = row < M ? labels[row] : -1;
      float z[2];
      float mx = -INFINITY;
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        z[b] = col[b] < V ? acc[mt][b][i] + bo[b] : -INFINITY;
        if (y == col[b]) zy[row] = z[b];
        mx = fmaxf(mx, z[b]);
      }
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      float e = 0.f, sz = 0.f;
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const float eb = mx > -INFINITY ? expf(z[b] - mx) : 0.f;          // exp(-inf) = 0 for columns past V
        e += eb;
        if (col[b] < V) sz += z[b];
        if (row < M && col[b] < V) E[(size_t)row * V + col[b]] = from_f<T>(eb);
      }
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) e += __shfl_xor(e, o, 64);
      if (psz) {                                            // label smoothing needs the mean logit of the row
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) sz += __shfl_xor(sz, o, 64);
      }
      if ((lane & 31) == 0 && row < M) {
        pmax[(size_t)row * np + pidx] = mx;
        psum[(size_t)row * np + pidx] = e;
        if (psz) psz[(size_t)row * np + pidx] = sz;
      }
    }
  }
}

void launch_ce_fwd(int prec, const void* Ho, int ldho, const void* Wo, const float* Bo, const int32_t* labels,
                   int M, int V, int H, void* E, float* pmax, float* psum, float* psz, float* zy, hipStream_t st) {
  const int ntm = (M + CeG::BM - 1) / CeG::BM, ntn = (V + CeG::BN - 1) / CeG::BN;
  const int grid = ((ntm * ntn + 7) / 8) * 8;
  const int np = ce_num_partials(V);
  if (prec)
    hipLaunchKernelGGL(ce_fwd_kernel<bf16_t>, dim3(grid), dim3(CeG::NT), 0, st, (const bf16_t*)Ho, ldho, (const bf16_t*)Wo, Bo,
                       labels, M, V, H, (bf16_t*)E, pmax, psum, psz, zy, np, ntn);
  else
    hipLaunchKernelGGL(ce_fwd_kernel<float>, dim3(grid), dim3(CeG::NT), 0, st, (const float*)Ho, ldho, (const float*)Wo, Bo,
                       labels, M, V, H, (float*)E, pmax, psum, psz, zy, np, ntn);
}

// one wavefront per row: combine the partials.  Row loss against the smoothed target distribution
// (1 - eps) onehot(y) + eps / V:  (1 - eps) (lse - z_y) + eps (lse - mean_v z_v); eps = 0: plain nll.
__global__ __launch_bounds__(256) void ce_row_kernel(const float* __restrict__ pmax, const float* __restrict__ psum,
                                                     const float* __restrict__ psz, const float* __restrict__ zy,
                                                     const float* __restrict__ mask, int M, int np, float eps, int V,
                                                     float* __restrict__ lse, float* __restrict__ nll) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= M) return;
  float mx = -INFINITY;
  for (int p = lane; p < np; p += 64) mx = fmaxf(mx, pmax[(size_t)row * np + p]);
  mx = wave_max(mx);
  float s = 0.f;
  for (int p = lane; p < np; p += 64) {
    const float pm = pmax[(size_t)row * np + p];
    if (pm > -INFINITY) s += psum[(size_t)row * np + p] * expf(pm - mx);
  }
  s = wave_sum(s);
  float sz = 0.f;
  if (eps > 0.f) {
    for (int p = lane; p < np; p += 64) sz += psz[(size_t)row * np + p];
    sz = wave_sum(sz);
  }
  if (lane == 0) {
    const float l = mx + logf(s);
    lse[row] = l;
    float r = l - zy[row];
    if (eps > 0.f) r = (1.f - eps) * r + eps * (l - sz / (float)V);
    nll[row] = mask[row] > 0.f ? r : 0.f;
  }
}

// single block: n_tok and the per-row scale mask / n_tok.  Needs only the lengths, so it runs before
// the decoder and every slab's backward can follow its forward directly.
__global__ __launch_bounds__(1024) void ce_rowscale_kernel(const float* __restrict__ mask, int M, float* __restrict__ rowscale,
                                                           float* __restrict__ loss) {
  __shared__ float s_cnt[1024];
  const int t = threadIdx.x;
  float c = 0.f;
  for (int r = t; r < M; r += 1024) c += mask[r];
  s_cnt[t] = c;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (t < o) s_cnt[t] += s_cnt[t + o];
    __syncthreads();
  }
  const float ntok = s_cnt[0];
  const float inv = ntok > 0.f ? 1.0f / ntok : 0.f;
  for (int r = t; r < M; r += 1024) rowscale[r] = mask[r] * inv;
  if (t == 0) loss[1] = ntok;
}

// single block: loss = sum nll / n_tok, summed in a fixed order
__global__ __launch_bounds__(1024) void ce_loss_kernel(const float* __restrict__ nll, int M, float* __restrict__ loss,
                                                       int* __restrict__ flags) {
  __shared__ float s_sum[1024];
  const int t = threadIdx.x;
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

void launch_ce_rowscale(const float* mask, int M, float* rowscale, float* loss, hipStream_t st) {
  hipLaunchKernelGGL(ce_rowscale_kernel, dim3(1), dim3(1024), 0, st, mask, M, rowscale, loss);
}
void launch_ce_rows(const float* pmax, const float* psum, const float* psz, const float* zy, const float* mask, int M, int np,
                    float eps, int V, float* lse, float* nll, hipStream_t st) {
  hipLaunchKernelGGL(ce_row_kernel, dim3((M + 3) / 4), dim3(256), 0, st, pmax, psum, psz, zy, mask, M, np, eps, V, lse, nll);
}
void launch_ce_loss(const float* nll, int M, float* loss, int* flags, hipStream_t st) {
  hipLaunchKernelGGL(ce_loss_kernel, dim3(1), dim3(1024), 0, st, nll, M, loss, flags);
}

// ------------------------------------------------------------------------------------------------
// e -> dz, in place, dz^T, and per block of 64 rows the column sums of dz (partial dB_o, summed by
// the caller in a fixed order).  One workgroup per 64 rows x 64 columns (= one group of partials):
// thread t takes row t / 4 and 16 consecutive columns; the transpose goes through LDS so that both
// the dz rows and the dz^T rows leave as 16-byte stores.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ce_scale_kernel(T* __restrict__ E, int V, int Mc, const float* __restrict__ pmax, int np,
                                                       const float* __restrict__ lse, const int32_t* __restrict__ labels,
                                                       const float* __restrict__ rowscale, float eps, T* __restrict__ dzT,
                                                       int ldzt, float* __restrict__ dbo_part) {
  constexpr int VE = 16 / sizeof(T);                      // elements per 16-byte vector
  constexpr int NV = 16 / VE;                             // vectors per thread
  __shared__ __align__(16) T tile[64][64 + VE];
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int t = threadIdx.x;
  {
    const int r = t >> 2, row = r0 + r, cb = (t & 3) * 16;
    float f = 0.f, rs = 0.f;
    const float epsv = eps / (float)V;                      // target distribution (1 - eps) onehot + eps / V
    int y = -1;
    if (row < Mc) {
      const float pm = pmax[(size_t)row * np + blockIdx.x];
      f = pm > -INFINITY ? expf(pm - lse[row]) : 0.f;
      rs = rowscale[row];
      y = labels[row];
    }
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col = c0 + cb + v * VE;
      T x[VE];
      if (row < Mc && col < V) *reinterpret_cast<uint4*>(x) = *reinterpret_cast<const uint4*>(E + (size_t)row * V + col);
      else *reinterpret_cast<uint4*>(x) = make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int j = 0; j < VE; ++j) {
        const float d = row < Mc && col < V ? (to_f<T>(x[j]) * f - (y == col + j ? 1.f - eps : 0.f) - epsv) * rs : 0.f;
        x[j] = from_f<T>(d);
        tile[cb + v * VE + j][r] = x[j];
      }
      if (row < Mc && col < V) *reinterpret_cast<uint4*>(E + (size_t)row * V + col) = *reinterpret_cast<const uint4*>(x);
    }
  }
  __syncthreads();
  {
    const int c = t >> 2, col = c0 + c, rb = (t & 3) * 16;
    float cs = 0.f;                                         // this block's share of dB_o[col]: 64 rows in fixed order
    if (col < V) {
#pragma unroll
      for (int v = 0; v < NV; ++v) {                        // rows past Mc hold zeros; the slab is CE_SLAB_ROWS wide
        const uint4 x = *reinterpret_cast<const uint4*>(&tile[c][rb + v * VE]);
        *reinterpret_cast<uint4*>(dzT + (size_t)col * ldzt + r0 + rb + v * VE) = x;
        const T* xe = reinterpret_cast<const T*>(&x);
#pragma unroll
        for (int j = 0; j < VE; ++j) cs += to_f<T>(xe[j]);
      }
    }
    cs += __shfl_xor(cs, 1, 64);
    cs += __shfl_xor(cs, 2, 64);
    if ((t & 3) == 0 && col < V) dbo_part[(size_t)blockIdx.y * V + col] = cs;
  }
}

void launch_ce_scale(int prec, void* E, int V, int Mc, const float* pmax, const float* lse, const int32_t* labels,
                     const float* rowscale, float eps, void* dzT, float* dbo_part, hipStream_t st) {
  dim3 grid((V + 63) / 64, (Mc + 63) / 64);
  const int np = ce_num_partials(V);
  if (prec)
    hipLaunchKernelGGL(ce_scale_kernel<bf16_t>, grid, dim3(256), 0, st, (bf16_t*)E, V, Mc, pmax, np, lse, labels, rowscale,
                       eps, (bf16_t*)dzT, CE_SLAB_ROWS, dbo_part);
  else
    hipLaunchKernelGGL(ce_scale_kernel<float>, grid, dim3(256), 0, st, (float*)E, V, Mc, pmax, np, lse, labels, rowscale,
                       eps, (float*)dzT, CE_SLAB_ROWS, dbo_part);
}

}  // namespace cmt
