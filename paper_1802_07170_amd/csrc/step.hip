// Kernels of the two time loops (encoder / decoder recurrences and their backward passes).
// Per step the batch is tiny (M = B <= 128) and the work is bound by streaming the layer's
// weights, so these kernels put the WEIGHT rows on the matrix cores' row side (16 rows per
// workgroup, read exactly once per step straight from global memory into MFMA fragments, no LDS
// staging) and the batch on the column side; the wavefronts of a workgroup split the k range and
// combine their partial tiles through LDS.  For the LSTM the 16 rows of a workgroup are the four
// gates of four hidden units, so that after the reduction every lane holds i, f, g, o of one
// (unit, sentence) pair and the cell update is fused in-register.
#include "common.h"
#include "kernels.h"

namespace cmt {

constexpr int STEP_MAXBT = 4;          // batch tiles (of 16 sentences) per workgroup pass

// Fragment of the concatenated k axis [a0 (K0) ; a1 (K1)], 8 elements at chunk index `chunk`.
template <typename T>
__device__ __forceinline__ void load_seg_frags(Frag<T>& fw, Frag<T> (&fx)[STEP_MAXBT], int chunk, int nc0, int nc,
                                               const T* wrow, int w0_off, int w1_off,
                                               const T* a0, int lda0, const T* a1, int lda1,
                                               int brow_base, int Bp, int nbt) {
  if (chunk >= nc) {
    fw.zero();
#pragma unroll
    for (int b = 0; b < STEP_MAXBT; ++b) fx[b].zero();
    return;
  }
  const bool first = chunk < nc0;
  const int kk = first ? chunk * 8 : (chunk - nc0) * 8;
  fw.load(wrow + (first ? w0_off : w1_off) + kk);
  const T* a = first ? a0 : a1;
  const int lda = first ? lda0 : lda1;
#pragma unroll
  for (int b = 0; b < STEP_MAXBT; ++b) {
    if (b < nbt) {
      int r = brow_base + 16 * b;
      r = r < Bp ? r : Bp - 1;
      fx[b].load(a + (size_t)r * lda + kk);
    } else {
      fx[b].zero();
    }
  }
}

// Runs the split-k contraction for one 16-row weight tile and reduces across wavefronts.
// On return, wavefronts w < nbt hold in `res` the full sums of batch tile w:
// res[i] = row (4 * (lane / 16) + i) of the weight tile, sentence 16 * (bt0 + w) + lane % 16.
template <typename T, int KS>
__device__ __forceinline__ bool step_contract(const T* wrow, int w0_off, int w1_off, const T* a0, int lda0, int K0,
                                              const T* a1, int lda1, int K1, int Bp, int bt0, int nbt, v4f& res,
                                              float* red /* [KS][STEP_MAXBT][64][4] */) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int nc0 = K0 >> 3, nc = (K0 + K1) >> 3;
  const int nsteps = (nc + 3) >> 2;
  const int brow_base = 16 * bt0 + (lane & 15);
  v4f acc[STEP_MAXBT];
#pragma unroll
  for (int b = 0; b < STEP_MAXBT; ++b) acc[b] = v4f{0.f, 0.f, 0.f, 0.f};
  // interleaved k-steps: wavefront w takes steps w, w + KS, ...; two steps in flight
  for (int s = w; s < nsteps; s += 2 * KS) {
    Frag<T> fw0, fw1, fx0[STEP_MAXBT], fx1[STEP_MAXBT];
    load_seg_frags<T>(fw0, fx0, 4 * s + (lane >> 4), nc0, nc, wrow, w0_off, w1_off, a0, lda0, a1, lda1, brow_base, Bp, nbt);
    const int s1 = s + KS;
    load_seg_frags<T>(fw1, fx1, s1 < nsteps ? 4 * s1 + (lane >> 4) : nc, nc0, nc, wrow, w0_off, w1_off, a0, lda0, a1, lda1,
                      brow_base, Bp, nbt);
#pragma unroll
    for (int b = 0; b < STEP_MAXBT; ++b) mma16(acc[b], fw0, fx0[b]);
#pragma unroll
    for (int b = 0; b < STEP_MAXBT; ++b) mma16(acc[b], fw1, fx1[b]);
  }
#pragma unroll
  for (int b = 0; b < STEP_MAXBT; ++b)
    *reinterpret_cast<v4f*>(red + ((w * STEP_MAXBT + b) * 64 + lane) * 4) = acc[b];
  __syncthreads();
  if (w >= nbt) return false;
  v4f r = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < KS; ++k) r += *reinterpret_cast<const v4f*>(red + ((k * STEP_MAXBT + w) * 64 + lane) * 4);
  res = r;
  return true;
}

// ------------------------------------------------------------------------------------------------
// LSTM forward step
// ------------------------------------------------------------------------------------------------
struct LstmFwdArgs { LstmFwdDir d[2]; };

template <typename T, int KS>
__global__ __launch_bounds__(64 * KS) void lstm_fwd_kernel(LstmFwdArgs args, int Bp, int Hh) {
  __shared__ __align__(16) float red[KS * STEP_MAXBT * 64 * 4];
  const LstmFwdDir& d = args.d[blockIdx.z];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int u0 = blockIdx.x * 4;
  const int bt0 = blockIdx.y * STEP_MAXBT;
  const int nbt = min(STEP_MAXBT, (Bp + 15) / 16 - bt0);
  // weight-tile row m = lane % 16: gate m % 4 of unit u0 + m / 4
  const int m = lane & 15;
  const int unit_ld = min(u0 + (m >> 2), Hh - 1);
  const T* wrow = (const T*)d.W + (size_t)((m & 3) * Hh + unit_ld) * d.ldw;
  v4f pre;
  if (!step_contract<T, KS>(wrow, d.wx_off, d.wh_off, (const T*)d.x, d.ldx, d.Kx, (const T*)d.hprev, d.ldh, Hh, Bp, bt0,
                            nbt, pre, red))
    return;
  const int u = u0 + (lane >> 4);
  const int b = 16 * (bt0 + w) + (lane & 15);
  if (u >= Hh || b >= Bp) return;
  float p[4];
#pragma unroll
  for (int g = 0; g < 4; ++g)
    p[g] = pre[g] + (d.gx ? d.gx[(size_t)b * d.ldgx + g * Hh + u] : d.bias[g * Hh + u]);
  const float ig = sigm(p[0]), fg = sigm(p[1]), gg = tanhf(p[2]), og = sigm(p[3]);
  const float cp = d.cprev[(size_t)b * Hh + u];
  const float cn = fg * cp + ig * gg;
  const float hn = og * tanhf(cn);
  const bool valid = d.mask[b] > 0.f;
  const T hp = ((const T*)d.hprev)[(size_t)b * d.ldh + u];
  const T hout = valid ? from_f<T>(hn) : hp;
  ((T*)d.hnext)[(size_t)b * Hh + u] = hout;
  d.cnext[(size_t)b * Hh + u] = valid ? cn : cp;
  float* gs = d.gsave + (size_t)b * 4 * Hh + u;
  gs[0] = ig; gs[Hh] = fg; gs[2 * Hh] = gg; gs[3 * Hh] = og;
  if (d.ycat) ((T*)d.ycat)[(size_t)b * d.ldy + u] = hout;
}

void launch_lstm_fwd(int prec, const LstmFwdDir* dirs, int ndir, int Bp, int Hh, hipStream_t st) {
  LstmFwdArgs a;
  a.d[0] = dirs[0];
  a.d[1] = dirs[ndir > 1 ? 1 : 0];
  const int nbt = (Bp + 15) / 16;
  dim3 grid((Hh + 3) / 4, (nbt + STEP_MAXBT - 1) / STEP_MAXBT, ndir);
  const int K = dirs[0].Kx + Hh;
  if (K >= 1024) {
    if (prec) hipLaunchKernelGGL((lstm_fwd_kernel<bf16_t, 8>), grid, dim3(512), 0, st, a, Bp, Hh);
    else hipLaunchKernelGGL((lstm_fwd_kernel<float, 8>), grid, dim3(512), 0, st, a, Bp, Hh);
  } else {
    if (prec) hipLaunchKernelGGL((lstm_fwd_kernel<bf16_t, 4>), grid, dim3(256), 0, st, a, Bp, Hh);
    else hipLaunchKernelGGL((lstm_fwd_kernel<float, 4>), grid, dim3(256), 0, st, a, Bp, Hh);
  }
}

// ------------------------------------------------------------------------------------------------
// generic step GEMM with epilogue
// ------------------------------------------------------------------------------------------------
template <typename T, int KS>
__global__ __launch_bounds__(64 * KS) void step_gemm_kernel(StepGemm g, int Bp) {
  __shared__ __align__(16) float red[KS * STEP_MAXBT * 64 * 4];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int n0 = blockIdx.x * 16;
  const int bt0 = blockIdx.y * STEP_MAXBT;
  const int nbt = min(STEP_MAXBT, (Bp + 15) / 16 - bt0);
  const int nrow = min(n0 + (lane & 15), g.N - 1);
  const T* wrow = (const T*)g.W + (size_t)nrow * g.ldw;
  v4f r;
  if (!step_contract<T, KS>(wrow, g.w0_off, g.w1_off, (const T*)g.a0, g.lda0, g.K0, (const T*)g.a1, g.lda1, g.K1, Bp, bt0,
                            nbt, r, red))
    return;
  const int b = 16 * (bt0 + w) + (lane & 15);
  if (b >= Bp) return;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int n = n0 + 4 * (lane >> 4) + i;
    if (n >= g.N) continue;
    if (g.mode == 0) {
      ((T*)g.outT)[(size_t)b * g.ldo + n] = from_f<T>(tanhf(r[i]));
    } else if (n < g.nsplit) {
      float* o = g.out0 + (size_t)b * g.ld0 + n;
      *o = g.acc0 ? *o + r[i] : r[i];
    } else {
      float* o = g.out1 + (size_t)b * g.ld1 + (n - g.nsplit);
      *o = g.acc1 ? *o + r[i] : r[i];
    }
  }
}

void launch_step_gemm(int prec, const StepGemm& g, int Bp, hipStream_t st) {
  const int nbt = (Bp + 15) / 16;
  dim3 grid((g.N + 15) / 16, (nbt + STEP_MAXBT - 1) / STEP_MAXBT);
  const int K = g.K0 + g.K1;
  if (K >= 2048) {
    if (prec) hipLaunchKernelGGL((step_gemm_kernel<bf16_t, 16>), grid, dim3(1024), 0, st, g, Bp);
    else hipLaunchKernelGGL((step_gemm_kernel<float, 16>), grid, dim3(1024), 0, st, g, Bp);
  } else if (K >= 1024) {
    if (prec) hipLaunchKernelGGL((step_gemm_kernel<bf16_t, 8>), grid, dim3(512), 0, st, g, Bp);
    else hipLaunchKernelGGL((step_gemm_kernel<float, 8>), grid, dim3(512), 0, st, g, Bp);
  } else {
    if (prec) hipLaunchKernelGGL((step_gemm_kernel<bf16_t, 4>), grid, dim3(256), 0, st, g, Bp);
    else hipLaunchKernelGGL((step_gemm_kernel<float, 4>), grid, dim3(256), 0, st, g, Bp);
  }
}

// ------------------------------------------------------------------------------------------------
// LSTM cell backward (pointwise), one thread per (sentence, unit)
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void lstm_bwd_point_kernel(LstmBwdPoint p, int Bp, int Hh) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= Bp * Hh) return;
  const int b = idx / Hh, u = idx - b * Hh;
  const float dh_state = p.dh[idx];
  const float dc_state = p.dc[idx];
  const float dy = p.dy ? p.dy[(size_t)b * p.lddy + u] : 0.f;
  T* dg = (T*)p.dg + (size_t)b * 4 * Hh + u;
  if (!(p.mask[b] > 0.f)) {                       // masked step: state passes through, no gate gradient
    const T z = from_f<T>(0.f);
    dg[0] = z; dg[Hh] = z; dg[2 * Hh] = z; dg[3 * Hh] = z;
    p.dh[idx] = dh_state;                          // (an output of a masked step is the constant 0: dy is dropped)
    return;
  }
  const float* gs = p.gsave + (size_t)b * 4 * Hh + u;
  const float ig = gs[0], fg = gs[Hh], gg = gs[2 * Hh], og = gs[3 * Hh];
  const float cp = p.cprev[idx], cn = p.cnext[idx];
  const float tc = tanhf(cn);
  const float dh = dh_state + dy;
  const float dog = dh * tc;
  const float dc = dc_state + dh * og * (1.f - tc * tc);
  dg[0] = from_f<T>(dc * gg * ig * (1.f - ig));
  dg[Hh] = from_f<T>(dc * cp * fg * (1.f - fg));
  dg[2 * Hh] = from_f<T>(dc * ig * (1.f - gg * gg));
  dg[3 * Hh] = from_f<T>(dog * og * (1.f - og));
  p.dc[idx] = dc * fg;
  p.dh[idx] = 0.f;                                 // the recurrent GEMM adds dgates * W_h onto this
}

void launch_lstm_bwd_point(int prec, const LstmBwdPoint& p, int Bp, int Hh, hipStream_t st) {
  const int n = Bp * Hh;
  if (prec) hipLaunchKernelGGL(lstm_bwd_point_kernel<bf16_t>, dim3((n + 255) / 256), dim3(256), 0, st, p, Bp, Hh);
  else hipLaunchKernelGGL(lstm_bwd_point_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, st, p, Bp, Hh);
}

// ------------------------------------------------------------------------------------------------
// attention, one workgroup per sentence
// ------------------------------------------------------------------------------------------------
// dots[i] = vec . Mat[i, b, :] for i < n (vec fp32 in LDS); one wavefront per source position.
template <typename T>
__device__ __forceinline__ void att_dots(const T* __restrict__ Mat, size_t pitch /*elements between i*/, int n, int H,
                                         const float* vec, float* dots) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  for (int i = w; i < n; i += nw) {
    const T* row = Mat + (size_t)i * pitch;
    float a = 0.f;
    for (int c = lane; c < (H >> 3); c += 64) {
      Frag<T> f;
      f.load(row + 8 * c);
#pragma unroll
      for (int e = 0; e < 8; ++e) a += f.get(e) * vec[8 * c + e];
    }
    a = wave_sum(a);
    if (lane == 0) dots[i] = a;
  }
}
// out[h] = sum_{i<n} coef[i] * Mat[i, b, h]; the thread block splits i into groups and reduces in LDS.
// Returns the value for column-chunk owners (threads with group 0) in res[8].
template <typename T>
__device__ __forceinline__ bool att_wsum(const T* __restrict__ Mat, size_t pitch, int n, int H, const float* coef,
                                         float* part /* [ng][H] */, float (&res)[8], int& chunk_out) {
  const int nch = H >> 3;                                   // chunks of 8 columns
  const int ng = max(1, (int)blockDim.x / nch);
  const int t = threadIdx.x;
  const int g = t / nch, c = t - g * nch;
  float a[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] = 0.f;
  if (g < ng) {
    for (int i = g; i < n; i += ng) {
      Frag<T> f;
      f.load(Mat + (size_t)i * pitch + 8 * c);
      const float w = coef[i];
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] += w * f.get(e);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[(size_t)g * H + 8 * c + e] = a[e];
  }
  __syncthreads();
  if (g != 0) return false;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float s = 0.f;
    for (int k = 0; k < ng; ++k) s += part[(size_t)k * H + 8 * c + e];
    res[e] = s;
  }
  chunk_out = c;
  return true;
}

constexpr int ATT_MAXH = 1024, ATT_MAXS = 512;

template <typename T>
__global__ __launch_bounds__(256) void att_fwd_kernel(const T* __restrict__ Kmat, const T* __restrict__ Hs,
                                                      const T* __restrict__ Ht, const int32_t* __restrict__ src_len,
                                                      int S, int Bp, int H, float* __restrict__ a_out, T* __restrict__ Cs) {
  __shared__ float vec[ATT_MAXH];
  __shared__ float sc[ATT_MAXS];
  __shared__ float part[2048];
  const int b = blockIdx.x, t = threadIdx.x;
  const int n = min(src_len[b], S);
  for (int h = t; h < H; h += 256) vec[h] = to_f<T>(Ht[(size_t)b * H + h]);
  __syncthreads();
  const size_t pitch = (size_t)Bp * H;
  att_dots<T>(Kmat + (size_t)b * H, pitch, n, H, vec, sc);
  __syncthreads();
  if (t < 64) {                                            // softmax over the valid positions (Eq. 3)
    float mx = -INFINITY;
    for (int i = t; i < n; i += 64) mx = fmaxf(mx, sc[i]);
    mx = wave_max(mx);
    float s = 0.f;
    for (int i = t; i < n; i += 64) { const float e = expf(sc[i] - mx); sc[i] = e; s += e; }
    s = wave_sum(s);
    const float inv = n > 0 ? 1.f / s : 0.f;
    for (int i = t; i < S; i += 64) {
      const float a = i < n ? sc[i] * inv : 0.f;
      if (i < n) sc[i] = a;
      a_out[(size_t)b * S + i] = a;
    }
  }
  __syncthreads();
  float res[8]; int c;
  if (att_wsum<T>(Hs + (size_t)b * H, pitch, n, H, sc, part, res, c)) {
#pragma unroll
    for (int e = 0; e < 8; ++e) Cs[(size_t)b * H + 8 * c + e] = from_f<T>(res[e]);
  }
}

void launch_att_fwd(int prec, const void* Kmat, const void* Hs, const void* Ht, const int32_t* src_len,
                    int S, int Bp, int H, float* a, void* Cs, hipStream_t st) {
  if (prec) hipLaunchKernelGGL(att_fwd_kernel<bf16_t>, dim3(Bp), dim3(256), 0, st, (const bf16_t*)Kmat, (const bf16_t*)Hs,
                               (const bf16_t*)Ht, src_len, S, Bp, H, a, (bf16_t*)Cs);
  else hipLaunchKernelGGL(att_fwd_kernel<float>, dim3(Bp), dim3(256), 0, st, (const float*)Kmat, (const float*)Hs,
                          (const float*)Ht, src_len, S, Bp, H, a, (float*)Cs);
}

template <typename T>
__global__ __launch_bounds__(256) void att_bwd_kernel(const T* __restrict__ Kmat, const T* __restrict__ Hs,
                                                      const float* __restrict__ dCs, const float* __restrict__ a,
                                                      const int32_t* __restrict__ src_len, int S, int Bp, int H,
                                                      float* __restrict__ ds_out, float* __restrict__ dHt) {
  __shared__ float vec[ATT_MAXH];
  __shared__ float sc[ATT_MAXS];
  __shared__ float part[2048];
  const int b = blockIdx.x, t = threadIdx.x;
  const int n = min(src_len[b], S);
  for (int h = t; h < H; h += 256) vec[h] = dCs[(size_t)b * H + h];
  __syncthreads();
  const size_t pitch = (size_t)Bp * H;
  att_dots<T>(Hs + (size_t)b * H, pitch, n, H, vec, sc);          // da_i = dC_s . H_s^i
  __syncthreads();
  if (t < 64) {                                                   // ds = a (da - sum a da)
    float dot = 0.f;
    for (int i = t; i < n; i += 64) dot += a[(size_t)b * S + i] * sc[i];
    dot = wave_sum(dot);
    for (int i = t; i < S; i += 64) {
      const float v = i < n ? a[(size_t)b * S + i] * (sc[i] - dot) : 0.f;
      if (i < n) sc[i] = v;
      ds_out[(size_t)b * S + i] = v;
    }
  }
  __syncthreads();
  float res[8]; int c;
  if (att_wsum<T>(Kmat + (size_t)b * H, pitch, n, H, sc, part, res, c)) {
#pragma unroll
    for (int e = 0; e < 8; ++e) dHt[(size_t)b * H + 8 * c + e] += res[e];
  }
}

void launch_att_bwd(int prec, const void* Kmat, const void* Hs, const float* dCs, const float* a, const int32_t* src_len,
                    int S, int Bp, int H, float* ds, float* dHt, hipStream_t st) {
  if (prec) hipLaunchKernelGGL(att_bwd_kernel<bf16_t>, dim3(Bp), dim3(256), 0, st, (const bf16_t*)Kmat, (const bf16_t*)Hs,
                               dCs, a, src_len, S, Bp, H, ds, dHt);
  else hipLaunchKernelGGL(att_bwd_kernel<float>, dim3(Bp), dim3(256), 0, st, (const float*)Kmat, (const float*)Hs, dCs, a,
                          src_len, S, Bp, H, ds, dHt);
}

// After the decoder loop: for a block (sentence b, 256 hidden columns, 32 source positions):
//   dHs[i,b,h] = sum_j a[j,b,i] dCs[j,b,h]        dK[i,b,h] = sum_j ds[j,b,i] Ht[j,b,h]
template <typename T>
__global__ __launch_bounds__(256) void att_deferred_kernel(const float* __restrict__ a, const float* __restrict__ ds,
                                                           const float* __restrict__ dCs, const T* __restrict__ Ht, int ldht,
                                                           int S, int Tn, int Bp, int H, float* __restrict__ dHs,
                                                           T* __restrict__ dK) {
  __shared__ float sa[32], sd[32];
  const int b = blockIdx.x, h = blockIdx.y * 256 + threadIdx.x, i0 = blockIdx.z * 32;
  float accC[32], accK[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) { accC[i] = 0.f; accK[i] = 0.f; }
  for (int j = 0; j < Tn; ++j) {
    __syncthreads();
    if (threadIdx.x < 32) {
      const int i = i0 + threadIdx.x;
      sa[threadIdx.x] = i < S ? a[((size_t)j * Bp + b) * S + i] : 0.f;
      sd[threadIdx.x] = i < S ? ds[((size_t)j * Bp + b) * S + i] : 0.f;
    }
    __syncthreads();
    if (h < H) {
      const float dc = dCs[((size_t)j * Bp + b) * H + h];
      const float ht = to_f<T>(Ht[(size_t)j * ldht + (size_t)b * H + h]);
#pragma unroll
      for (int i = 0; i < 32; ++i) { accC[i] += sa[i] * dc; accK[i] += sd[i] * ht; }
    }
  }
  if (h >= H) return;
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    if (i0 + i < S) {
      const size_t o = ((size_t)(i0 + i) * Bp + b) * H + h;
      dHs[o] = accC[i];
      dK[o] = from_f<T>(accK[i]);
    }
  }
}

void launch_att_deferred(int prec, const float* a, const float* ds, const float* dCs, const void* Ht, int ldht,
                         int S, int T, int Bp, int H, float* dHs, void* dK, hipStream_t st) {
  dim3 grid(Bp, (H + 255) / 256, (S + 31) / 32);
  if (prec) hipLaunchKernelGGL(att_deferred_kernel<bf16_t>, grid, dim3(256), 0, st, a, ds, dCs, (const bf16_t*)Ht, ldht, S, T,
                               Bp, H, dHs, (bf16_t*)dK);
  else hipLaunchKernelGGL(att_deferred_kernel<float>, grid, dim3(256), 0, st, a, ds, dCs, (const float*)Ht, ldht, S, T, Bp, H,
                          dHs, (float*)dK);
}

template <typename T>
__global__ __launch_bounds__(256) void tanh_bwd_kernel(const float* __restrict__ dce, const float* __restrict__ dfeed,
                                                       const T* __restrict__ Ho, T* __restrict__ dpre, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float ho = to_f<T>(Ho[i]);
  const float d = dce[i] + (dfeed ? dfeed[i] : 0.f);
  dpre[i] = from_f<T>(d * (1.f - ho * ho));
}

void launch_tanh_bwd(int prec, const float* dHo_ce, const float* dHo_feed, const void* Ho, void* dpre, int n, hipStream_t st) {
  if (prec) hipLaunchKernelGGL(tanh_bwd_kernel<bf16_t>, dim3((n + 255) / 256), dim3(256), 0, st, dHo_ce, dHo_feed,
                               (const bf16_t*)Ho, (bf16_t*)dpre, n);
  else hipLaunchKernelGGL(tanh_bwd_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, st, dHo_ce, dHo_feed,
                          (const float*)Ho, (float*)dpre, n);
}

}  // namespace cmt
