// Vocabulary projection + log-softmax + cross-entropy (Eq. 1), forward and backward, without ever
// writing the [rows, vocab] logit or probability matrix:
//   forward : logits are produced 128x128 tile at a time by the matrix cores and immediately
//             reduced to per-row (max, sum exp) partials over 64 columns, plus the label's logit;
//   backward: dz = (softmax(z) - onehot) * mask / n_tok is rebuilt per 64x128 tile from the row
//             log-sum-exp, rounded to the operand type into LDS and consumed there as the operand
//             of the second contraction (dH_o = dz W_o, or dW_o = dz^T H_o), whose 64 x H output
//             stays in registers for the whole kernel.
#include "gemm_core.h"
#include "kernels.h"

namespace cmt {

constexpr int CE_TA = 2, CE_TB = 2;                       // 128 x 128 logit tile per workgroup
using CeTile = GemmTile<CE_TA, CE_TB>;
int ce_num_partials(int V) { return 2 * ((V + CeTile::BN - 1) / CeTile::BN); }

template <typename T>
__global__ __launch_bounds__(256) void ce_fwd_kernel(const T* __restrict__ Ho, int ldho, const T* __restrict__ Wo,
                                                     const float* __restrict__ Bo, const int32_t* __restrict__ labels,
                                                     int M, int V, int H, float* __restrict__ pmax,
                                                     float* __restrict__ psum, float* __restrict__ zy, int np) {
  __shared__ __align__(16) char smem[CeTile::SMEM_BYTES];
  const int m0 = blockIdx.y * CeTile::BM, n0 = blockIdx.x * CeTile::BN;
  v16f acc[CE_TA][CE_TB];
  gemm_mainloop<T, CE_TA, CE_TB>(Ho, ldho, Wo, H, M, V, H, m0, n0, acc, smem);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wm = w >> 1, wn = w & 1;
  int col[CE_TB];
  float bo[CE_TB];
#pragma unroll
  for (int b = 0; b < CE_TB; ++b) {
    col[b] = n0 + wn * 32 * CE_TB + b * 32 + (lane & 31);
    bo[b] = col[b] < V ? Bo[col[b]] : 0.f;
  }
  const int pidx = blockIdx.x * 2 + wn;
#pragma unroll
  for (int mt = 0; mt < CE_TA; ++mt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = m0 + wm * 32 * CE_TA + mt * 32 + acc32_row(lane, i);
      const int y = row < M ? labels[row] : -1;
      float z[CE_TB];
      float mx = -INFINITY;
#pragma unroll
      for (int b = 0; b < CE_TB; ++b) {
        z[b] = col[b] < V ? acc[mt][b][i] + bo[b] : -INFINITY;
        if (y == col[b]) zy[row] = z[b];
        mx = fmaxf(mx, z[b]);
      }
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      float e = 0.f;
      if (mx > -INFINITY) {
#pragma unroll
        for (int b = 0; b < CE_TB; ++b) e += expf(z[b] - mx);              // exp(-inf) = 0 for columns past V
      }
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) e += __shfl_xor(e, o, 64);
      if ((lane & 31) == 0 && row < M) {
        pmax[(size_t)row * np + pidx] = mx;
        psum[(size_t)row * np + pidx] = e;
      }
    }
  }
}

void launch_ce_fwd(int prec, const void* Ho, int ldho, const void* Wo, const float* Bo, const int32_t* labels,
                   int M, int V, int H, float* pmax, float* psum, float* zy, hipStream_t st) {
  dim3 grid((V + CeTile::BN - 1) / CeTile::BN, (M + CeTile::BM - 1) / CeTile::BM);
  const int np = ce_num_partials(V);
  if (prec)
    hipLaunchKernelGGL(ce_fwd_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)Ho, ldho, (const bf16_t*)Wo, Bo, labels,
                       M, V, H, pmax, psum, zy, np);
  else
    hipLaunchKernelGGL(ce_fwd_kernel<float>, grid, dim3(256), 0, st, (const float*)Ho, ldho, (const float*)Wo, Bo, labels,
                       M, V, H, pmax, psum, zy, np);
}

// one wavefront per row: combine the partials
__global__ __launch_bounds__(256) void ce_row_kernel(const float* __restrict__ pmax, const float* __restrict__ psum,
                                                     const float* __restrict__ zy, const float* __restrict__ mask,
                                                     int M, int np, float* __restrict__ lse, float* __restrict__ nll) {
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
  if (lane == 0) {
    const float l = mx + logf(s);
    lse[row] = l;
    nll[row] = mask[row] > 0.f ? l - zy[row] : 0.f;
  }
}

// single block: n_tok, loss and the per-row scale, summed in a fixed order
__global__ __launch_bounds__(1024) void ce_loss_kernel(const float* __restrict__ nll, const float* __restrict__ mask, int M,
                                                       float* __restrict__ rowscale, float* __restrict__ loss,
                                                       int* __restrict__ flags) {
  __shared__ float s_sum[1024], s_cnt[1024];
  const int t = threadIdx.x;
  float a = 0.f, c = 0.f;
  for (int r = t; r < M; r += 1024) { a += nll[r]; c += mask[r]; }
  s_sum[t] = a; s_cnt[t] = c;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (t < o) { s_sum[t] += s_sum[t + o]; s_cnt[t] += s_cnt[t + o]; }
    __syncthreads();
  }
  const float ntok = s_cnt[0];
  const float inv = ntok > 0.f ? 1.0f / ntok : 0.f;
  for (int r = t; r < M; r += 1024) rowscale[r] = mask[r] * inv;
  if (t == 0) {
    const float l = s_sum[0] * inv;
    loss[0] = l;
    loss[1] = ntok;
    if (!isfinite(l)) atomicOr(flags, 4);
  }
}

void launch_ce_reduce(const float* pmax, const float* psum, const float* zy, const float* mask, int M, int np,
                      float* lse, float* nll, float* rowscale, float* loss, int* flags, hipStream_t st) {
  hipLaunchKernelGGL(ce_row_kernel, dim3((M + 3) / 4), dim3(256), 0, st, pmax, psum, zy, mask, M, np, lse, nll);
  hipLaunchKernelGGL(ce_loss_kernel, dim3(1), dim3(1024), 0, st, nll, mask, M, rowscale, loss, flags);
}

// ------------------------------------------------------------------------------------------------
// backward.  P = 64 stationary rows, Q = streamed rows in tiles of 128.
//   MODE 0 (dH_o): P = H_o rows (m), Q = W_o rows (v), QT = W_o^T;  out[split, m, :] = sum_v dz[m,v] W_o[v,:]
//   MODE 1 (dW_o): P = W_o rows (v), Q = H_o rows (m), QT = H_o^T;  dWo[v, :] = sum_m dz[m,v] H_o[m,:]
// 8 wavefronts: the score tile S[64,128] is 2x4 MFMA 32x32 tiles, one per wavefront (operands
// straight from global memory / L2, each element is used once per block); the output [64, H] is
// split by columns, 32*HT per wavefront.
// ------------------------------------------------------------------------------------------------
template <typename T, int HT, int MODE>
__global__ __launch_bounds__(512) void ce_bwd_kernel(const T* __restrict__ P, int ldp, int nP, const T* __restrict__ Q, int ldq, int nQ,
                                                     const T* __restrict__ QT, int ldqt, const float* __restrict__ Bo,
                                                     const int32_t* __restrict__ labels, const float* __restrict__ lse,
                                                     const float* __restrict__ rowscale, int H, int tiles_per_split,
                                                     float* __restrict__ out, float* __restrict__ dBo) {
  constexpr int DZ_ROWB = 128 * sizeof(T) + 16;
  __shared__ __align__(16) char dzs[64 * DZ_ROWB];
  __shared__ float s_a[64], s_b[64];       // MODE 0: lse, rowscale of the 64 rows; MODE 1: Bo of the 64 vocab rows
  __shared__ int s_lab[64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int p0 = blockIdx.x * 64;
  const int M = MODE == 0 ? nP : nQ, V = MODE == 0 ? nQ : nP;
  if (threadIdx.x < 64) {
    const int p = p0 + threadIdx.x;
    if (MODE == 0) {
      s_a[threadIdx.x] = p < nP ? lse[p] : 0.f;
      s_b[threadIdx.x] = p < nP ? rowscale[p] : 0.f;
      s_lab[threadIdx.x] = p < nP ? labels[p] : -1;
    } else {
      s_a[threadIdx.x] = p < nP ? Bo[p] : 0.f;
    }
  }
  __syncthreads();
  const int ntiles = (nQ + 127) / 128;
  const int t_begin = blockIdx.y * tiles_per_split;
  const int t_end = min(ntiles, t_begin + tiles_per_split);

  v16f acc2[2][HT];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < HT; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc2[a][b][i] = 0.f;
  float dbo = 0.f;

  const int mt1 = w & 1, nt1 = w >> 1;                      // this wavefront's score tile
  const int prow = min(p0 + 32 * mt1 + (lane & 31), nP - 1);
  const T* pa = P + (size_t)prow * ldp + 8 * (lane >> 5);
  const int hbase = w * 32 * HT;

  for (int qt = t_begin; qt < t_end; ++qt) {
    const int q0 = qt * 128;
    // ---- scores: S = P Q^T over k = H ----------------------------------------------------------
    v16f s;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
    const int qrow = min(q0 + 32 * nt1 + (lane & 31), nQ - 1);
    const T* pb = Q + (size_t)qrow * ldq + 8 * (lane >> 5);
    for (int k = 0; k < H; k += 64) {
      Frag<T> fa[4], fb[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (k + 16 * u < H) { fa[u].load(pa + k + 16 * u); fb[u].load(pb + k + 16 * u); }
        else { fa[u].zero(); fb[u].zero(); }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) mma32(s, fa[u], fb[u]);
    }
    // ---- dz tile -> LDS --------------------------------------------------------------------------
    {
      const int ql = 32 * nt1 + (lane & 31), q = q0 + ql;
      float qa = 0.f, qb = 0.f; int qlab = -1;
      if (q < nQ) {
        if (MODE == 0) qa = Bo[q];
        else { qa = lse[q]; qb = rowscale[q]; qlab = labels[q]; }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int pl = 32 * mt1 + acc32_row(lane, i);
        float dz = 0.f;
        if (q < nQ && p0 + pl < nP) {
          if (MODE == 0) dz = (expf(s[i] + qa - s_a[pl]) - (s_lab[pl] == q ? 1.f : 0.f)) * s_b[pl];
          else dz = (expf(s[i] + s_a[pl] - qa) - (qlab == p0 + pl ? 1.f : 0.f)) * qb;
        }
        *reinterpret_cast<T*>(dzs + pl * DZ_ROWB + ql * sizeof(T)) = from_f<T>(dz);
      }
    }
    __syncthreads();
    if (MODE == 1 && threadIdx.x < 64) {
      const T* r = reinterpret_cast<const T*>(dzs + threadIdx.x * DZ_ROWB);
      float a = 0.f;
      for (int j = 0; j < 128; ++j) a += to_f<T>(r[j]);
      dbo += a;
    }
    // ---- second contraction: out[64, H] += dz[64,128] * Qmat[128, H] -----------------------------
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      Frag<T> fa[2], fb[HT];
      const int kq = q0 + ks * 16 + 8 * (lane >> 5);
#pragma unroll
      for (int a = 0; a < 2; ++a)
        fa[a].load(reinterpret_cast<const T*>(dzs + (32 * a + (lane & 31)) * DZ_ROWB + (ks * 16 + 8 * (lane >> 5)) * sizeof(T)));
#pragma unroll
      for (int b = 0; b < HT; ++b) {
        const int hr = min(hbase + 32 * b + (lane & 31), H - 1);
        if (kq < nQ) fb[b].load(QT + (size_t)hr * ldqt + kq);
        else fb[b].zero();
      }
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < HT; ++b) mma32(acc2[a][b], fa[a], fb[b]);
    }
    __syncthreads();
  }
  // ---- write the 64 x H block --------------------------------------------------------------------
  float* o = out + (MODE == 0 ? (size_t)blockIdx.y * nP * H : 0);
#pragma unroll
  for (int b = 0; b < HT; ++b) {
    const int h = hbase + 32 * b + (lane & 31);
    if (h >= H) continue;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int p = p0 + 32 * a + acc32_row(lane, i);
        if (p < nP) o[(size_t)p * H + h] = acc2[a][b][i];
      }
  }
  if (MODE == 1 && threadIdx.x < 64 && p0 + threadIdx.x < nP) dBo[p0 + threadIdx.x] = dbo;
  (void)M; (void)V;
}

int ce_bwd_nsplit(int M, int V) {
  const int mt = (M + 63) / 64, vt = (V + 127) / 128;
  int ns = (512 + mt - 1) / mt;
  if (ns > vt) ns = vt;
  if (ns > 16) ns = 16;
  if (ns < 1) ns = 1;
  return ns;
}

template <typename T, int MODE>
static void ce_bwd_dispatch(const T* P, int ldp, int nP, const T* Q, int ldq, int nQ, const T* QT, int ldqt, const float* Bo,
                            const int32_t* labels, const float* lse, const float* rowscale, int H, int nsplit,
                            float* out, float* dBo, hipStream_t st) {
  const int ntiles = (nQ + 127) / 128;
  const int tps = (ntiles + nsplit - 1) / nsplit;
  dim3 grid((nP + 63) / 64, nsplit);
#define CE_BWD_GO(HT)                                                                                          \
  hipLaunchKernelGGL((ce_bwd_kernel<T, HT, MODE>), grid, dim3(512), 0, st, P, ldp, nP, Q, ldq, nQ, QT, ldqt, Bo, labels, \
                     lse, rowscale, H, tps, out, dBo)
  if (H <= 256) CE_BWD_GO(1);
  else if (H <= 512) CE_BWD_GO(2);
  else CE_BWD_GO(4);
#undef CE_BWD_GO
}

void launch_ce_bwd_dh(int prec, const void* Ho, int ldho, const void* Wo, const void* WoT, const float* Bo,
                      const int32_t* labels, const float* lse, const float* rowscale,
                      int M, int V, int H, int nsplit, float* dHo_part, hipStream_t st) {
  if (prec)
    ce_bwd_dispatch<bf16_t, 0>((const bf16_t*)Ho, ldho, M, (const bf16_t*)Wo, H, V, (const bf16_t*)WoT, V, Bo, labels, lse,
                               rowscale, H, nsplit, dHo_part, nullptr, st);
  else
    ce_bwd_dispatch<float, 0>((const float*)Ho, ldho, M, (const float*)Wo, H, V, (const float*)WoT, V, Bo, labels, lse,
                              rowscale, H, nsplit, dHo_part, nullptr, st);
}

void launch_ce_bwd_dw(int prec, const void* Ho, int ldho, const void* HoT, int ldhot, const void* Wo, const float* Bo,
                      const int32_t* labels, const float* lse, const float* rowscale,
                      int M, int V, int H, float* dWo, float* dBo, hipStream_t st) {
  if (prec)
    ce_bwd_dispatch<bf16_t, 1>((const bf16_t*)Wo, H, V, (const bf16_t*)Ho, ldho, M, (const bf16_t*)HoT, ldhot, Bo, labels, lse,
                               rowscale, H, 1, dWo, dBo, st);
  else
    ce_bwd_dispatch<float, 1>((const float*)Wo, H, V, (const float*)Ho, ldho, M, (const float*)HoT, ldhot, Bo, labels, lse,
                              rowscale, H, 1, dWo, dBo, st);
}

// ------------------------------------------------------------------------------------------------
// backward, slab variant.  For a slab of at most CE_SLAB_ROWS rows the logits are rebuilt tile by
// tile (same main loop as the forward kernel) and dz = (softmax(z) - onehot) * mask / n_tok is
// written, in the operand type, as dz[rows, V] and dz^T[V, rows]; two plain GEMMs then give
// dH_o = dz W_o and dW_o += dz^T H_o at full matrix-core tiles.  Recomputing a dz element costs
// 2H flops against 6 bytes of slab traffic, so on this machine staging a bounded slab beats
// rebuilding dz a second time; the slab is reused for every group of rows, its size does not grow
// with the batch, and the full [rows, vocabulary] matrix never exists.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ce_dz_kernel(const T* __restrict__ Ho, int ldho, const T* __restrict__ Wo,
                                                    const float* __restrict__ Bo, const int32_t* __restrict__ labels,
                                                    const float* __restrict__ lse, const float* __restrict__ rowscale,
                                                    int Mc, int V, int H, T* __restrict__ dz, int ldz,
                                                    T* __restrict__ dzT, int ldzt, int ntn) {
  using G = GemmTile<2, 2, 128>;
  __shared__ __align__(16) char smem[G::SMEM_BYTES];
  const int per = gridDim.x >> 3;
  const int id = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  const int m0 = (id / ntn) * G::BM, n0 = (id % ntn) * G::BN;
  if (m0 >= Mc) return;
  v16f acc[2][2];
  gemm_mainloop<T, 2, 2, 128>(Ho, ldho, Wo, H, Mc, V, H, m0, n0, acc, smem);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wm = w >> 1, wn = w & 1;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int col = n0 + wn * 64 + nt * 32 + (lane & 31);
    if (col >= V) continue;
    const float bo = Bo[col];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {                       // 4 groups of 4 consecutive rows
        const int row0 = m0 + wm * 64 + mt * 32 + acc32_row(lane, 4 * q);
        T v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = row0 + i;
          float d = 0.f;
          if (row < Mc)
            d = (expf(acc[mt][nt][4 * q + i] + bo - lse[row]) - (labels[row] == col ? 1.f : 0.f)) * rowscale[row];
          v[i] = from_f<T>(d);
          if (row < Mc) dz[(size_t)row * ldz + col] = v[i];
        }
        if (row0 < Mc) {                                  // ldzt and row0 are multiples of 4: one aligned store
          T* o = dzT + (size_t)col * ldzt + row0;
          if (sizeof(T) == 2) *reinterpret_cast<uint2*>(o) = *reinterpret_cast<const uint2*>(v);
          else *reinterpret_cast<uint4*>(o) = *reinterpret_cast<const uint4*>(v);
        }
      }
    }
  }
}

size_t ce_slab_elems(int V) { return (size_t)CE_SLAB_ROWS * V; }

void launch_ce_dz(int prec, const void* Ho, int ldho, const void* Wo, const float* Bo, const int32_t* labels, const float* lse,
                  const float* rowscale, int Mc, int V, int H, void* dz, void* dzT, hipStream_t st) {
  using G = GemmTile<2, 2, 128>;
  const int ntm = (Mc + G::BM - 1) / G::BM, ntn = (V + G::BN - 1) / G::BN;
  const int grid = ((ntm * ntn + 7) / 8) * 8;
  if (prec)
    hipLaunchKernelGGL(ce_dz_kernel<bf16_t>, dim3(grid), dim3(256), 0, st, (const bf16_t*)Ho, ldho, (const bf16_t*)Wo, Bo, labels,
                       lse, rowscale, Mc, V, H, (bf16_t*)dz, V, (bf16_t*)dzT, CE_SLAB_ROWS, ntn);
  else
    hipLaunchKernelGGL(ce_dz_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)Ho, ldho, (const float*)Wo, Bo, labels, lse,
                       rowscale, Mc, V, H, (float*)dz, V, (float*)dzT, CE_SLAB_ROWS, ntn);
}

}  // namespace cmt
