// Beam search bookkeeping on the device (hyperparameter table: beam size 10, length penalty 0.6;
// the Settings section names the length normalisation of Wu et al. 2016).  The decoder runs on
// R = B * K rows, row r = b * K + s holding live hypothesis s of sentence b.  Per step:
//   beam_row_topk_kernel one workgroup per live row: log-sum-exp of its logits and its K best tokens;
//   beam_merge_kernel   one workgroup per sentence: the K best one-token extensions over all live
//                       hypotheses (equal scores: the lower (slot, token) pair first), finished
//                       hypotheses split off, history written;
//   beam_reorder_kernel the surviving hypotheses' decoder states and H_o move to their new rows.
// After the last step beam_finish_kernel walks the back-pointers of each sentence's best finished
// hypothesis.  Nothing returns to the host inside the loop.
#include "common.h"
#include "kernels.h"

namespace cmt {

// dst[i, r, 0:cols] = src[i, r / K, 0:cols] for r < R, zero rows for r in [R, Rp); i < n_outer.
// Row pitches in elements; cols * sizeof(T) is a multiple of 16.
template <typename T>
__global__ __launch_bounds__(128) void beam_expand_kernel(const T* __restrict__ src, int ld_src, int rows_src, T* __restrict__ dst,
                                                          int ld_dst, int R, int Rp, int K, int cols) {
  const int r = blockIdx.x, i = blockIdx.y;
  constexpr int VE = 16 / sizeof(T);
  const T* s = r < R ? src + ((size_t)i * rows_src + r / K) * ld_src : nullptr;
  T* d = dst + ((size_t)i * Rp + r) * ld_dst;
  for (int c = threadIdx.x * VE; c < cols; c += 128 * VE)
    *reinterpret_cast<uint4*>(d + c) = s ? *reinterpret_cast<const uint4*>(s + c) : make_uint4(0, 0, 0, 0);
}
void launch_beam_expand(int elem_bytes, const void* src, int ld_src, int rows_src, void* dst, int ld_dst, int n_outer, int R, int Rp,
                        int K, int cols, hipStream_t st) {
  dim3 grid(Rp, n_outer);
  if (elem_bytes == 2)
    hipLaunchKernelGGL(beam_expand_kernel<bf16_t>, grid, dim3(128), 0, st, (const bf16_t*)src, ld_src, rows_src, (bf16_t*)dst, ld_dst,
                       R, Rp, K, cols);
  else
    hipLaunchKernelGGL(beam_expand_kernel<float>, grid, dim3(128), 0, st, (const float*)src, ld_src, rows_src, (float*)dst, ld_dst, R,
                       Rp, K, cols);
}

// start of a search: one live hypothesis per sentence (slot 0, score 0, previous token bos)
__global__ __launch_bounds__(256) void beam_init_kernel(BeamState bs, int B, int Rp, int K, int bos, const int32_t* __restrict__ len_src,
                                                        int32_t* __restrict__ len_exp) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r < Rp) {
    const int b = r / K, s = r - b * K;
    const bool real = b < B;
    bs.cum[r] = real && s == 0 ? 0.f : -INFINITY;
    bs.tok[r] = bos;
    bs.mask[r] = real && s == 0 ? 1.f : 0.f;
    len_exp[r] = real ? len_src[b] : 0;
  }
  if (r < B) { bs.nlive[r] = 1; bs.fin_score[r] = -INFINITY; bs.fin_step[r] = -1; bs.fin_par[r] = 0; bs.fin_tok[r] = 0; }
}
void launch_beam_init(const BeamState& bs, int B, int Rp, int K, int bos, const int32_t* len_src, int32_t* len_exp, hipStream_t st) {
  hipLaunchKernelGGL(beam_init_kernel, dim3((Rp + 255) / 256), dim3(256), 0, st, bs, B, Rp, K, bos, len_src, len_exp);
}

constexpr int BEAM_MAX = 16;
constexpr int BEAM_CAND_CAP = 2048;     // candidates a row's workgroup keeps in LDS

// (value, index) ordering: larger value first, then lower index
__device__ __forceinline__ bool beam_better(float v, int f, float bv, int bf) { return v > bv || (v == bv && f < bf); }

// Wavefront-wide best (value, index) pair; every lane gets the result.
__device__ __forceinline__ void beam_wave_best(float& v, int& f) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(v, o, 64);
    const int of = __shfl_xor(f, o, 64);
    if (beam_better(ov, of, v, f)) { v = ov; f = of; }
  }
}
// Workgroup-wide best (value, index) pair of 256 threads; every thread gets the result.
__device__ __forceinline__ void beam_block_best(float& v, int& f, float* s_v, int* s_f) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(v, o, 64);
    const int of = __shfl_xor(f, o, 64);
    if (beam_better(ov, of, v, f)) { v = ov; f = of; }
  }
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  __syncthreads();                                       // the previous round's readers are done
  if (lane == 0) { s_v[w] = v; s_f[w] = f; }
  __syncthreads();
  v = s_v[0]; f = s_f[0];
#pragma unroll
  for (int q = 1; q < 4; ++q)
    if (beam_better(s_v[q], s_f[q], v, f)) { v = s_v[q]; f = s_f[q]; }
}

// One workgroup per hypothesis row: log-sum-exp of the row's logits and its K best tokens (larger
// logit first, then lower token), written best first; entries beyond the row's candidates are
// (-inf, INT_MAX).  The K best of a row contain every extension of it that can be among the K best
// of its sentence (log-softmax is monotonic within a row).
//   pass 1: every thread's best element; the K-th best of those 256 is a lower bound tau on the
//           row's K-th best logit;
//   pass 2: sum of exp(z - max), and the elements >= tau are appended to a list in LDS;
//   then K rounds of a workgroup-wide arg-max over that list.  A list that overflows (many equal
//   logits) falls back to K rounds over the row itself.
// Both passes keep four 16-byte loads per thread in flight (a row is 128 KB at V = 32000 and the workgroup's 256 threads
// would otherwise wait for one load at a time).  FAST (16-bit path): the hardware exponential in the log-sum-exp.
template <bool FAST>
__global__ __launch_bounds__(256) void beam_row_topk_kernel(const float* __restrict__ z, int V, BeamState bs, int K) {
  __shared__ float s_v[4];
  __shared__ int s_f[4];
  __shared__ float s_sum[4];
  __shared__ float s_cv[BEAM_CAND_CAP];
  __shared__ int s_ci[BEAM_CAND_CAP];
  __shared__ int s_n;
  const int r = blockIdx.x, t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int b = r / K, slot = r - b * K;
  if (slot >= bs.nlive[b]) return;                       // dead row (uniform over the workgroup)
  const float* zr = z + (size_t)r * V;
  const int nv4 = V >> 2;                                // V is a multiple of 8
  // ---- pass 1 ----------------------------------------------------------------------------------------
  float tv = -INFINITY; int ti = 0x7fffffff;
  for (int c0 = t; c0 < nv4; c0 += 4 * 256) {
    float4 q[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int c = c0 + 256 * k;
      q[k] = c < nv4 ? *reinterpret_cast<const float4*>(zr + 4 * c) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {                         // ascending token order, as one load at a time would visit them
      const int c = c0 + 256 * k;
      if (c >= nv4) break;
      if (beam_better(q[k].x, 4 * c, tv, ti)) { tv = q[k].x; ti = 4 * c; }
      if (beam_better(q[k].y, 4 * c + 1, tv, ti)) { tv = q[k].y; ti = 4 * c + 1; }
      if (beam_better(q[k].z, 4 * c + 2, tv, ti)) { tv = q[k].z; ti = 4 * c + 2; }
      if (beam_better(q[k].w, 4 * c + 3, tv, ti)) { tv = q[k].w; ti = 4 * c + 3; }
    }
  }
  // The K-th best of one wavefront's 64 thread-bests is already such a bound (its threads hold bests of disjoint
  // parts of the row): K rounds of shuffles per wavefront, no barriers, then the largest of the four bounds.
  float mx = -INFINITY, tau = -INFINITY;
  {
    bool taken = false;
    for (int round = 0; round < K; ++round) {
      float v = taken ? -INFINITY : tv;
      int f = taken ? 0x7fffffff : ti;
      beam_wave_best(v, f);
      if (round == 0) mx = v;
      tau = v;                                           // -inf when fewer than K of its threads hold an element
      if (!taken && f == ti) taken = true;
    }
  }
  if (lane == 0) { s_v[w] = tau; s_sum[w] = mx; }
  if (t == 0) s_n = 0;
  __syncthreads();
  tau = fmaxf(fmaxf(s_v[0], s_v[1]), fmaxf(s_v[2], s_v[3]));
  mx = fmaxf(fmaxf(s_sum[0], s_sum[1]), fmaxf(s_sum[2], s_sum[3]));
  __syncthreads();                                       // (s_sum is written again below)
  // ---- pass 2 ----------------------------------------------------------------------------------------
  float e = 0.f;
  for (int c0 = t; c0 < nv4; c0 += 4 * 256) {
    float4 q[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int c = c0 + 256 * k;
      q[k] = c < nv4 ? *reinterpret_cast<const float4*>(zr + 4 * c) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int c = c0 + 256 * k;
      if (c >= nv4) break;
      const float x[4] = {q[k].x, q[k].y, q[k].z, q[k].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        e += FAST ? __expf(x[i] - mx) : expf(x[i] - mx);
        if (x[i] >= tau) {
          const int pos = atomicAdd(&s_n, 1);
          if (pos < BEAM_CAND_CAP) { s_cv[pos] = x[i]; s_ci[pos] = 4 * c + i; }
        }
      }
    }
  }
  e = wave_sum(e);
  if (lane == 0) s_sum[w] = e;
  __syncthreads();
  if (t == 0) bs.row_lse[r] = mx + logf((s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]));
  const int n = s_n;
  // ---- K rounds: the best element strictly after the previous winner in the (value, token) order ---------
  float pv = INFINITY; int pi = -1;
  if (n <= 256) {                                        // (the usual case) a short list: one wavefront, shuffles only
    if (w != 0) return;
    for (int round = 0; round < K; ++round) {
      float v = -INFINITY; int f = 0x7fffffff;
      for (int q = lane; q < n; q += 64) {
        const float x = s_cv[q]; const int xi = s_ci[q];
        if ((x < pv || (x == pv && xi > pi)) && beam_better(x, xi, v, f)) { v = x; f = xi; }
      }
      beam_wave_best(v, f);
      if (lane == 0) { bs.cand_z[(size_t)r * BEAM_MAX + round] = v; bs.cand_tok[(size_t)r * BEAM_MAX + round] = f; }
      pv = v; pi = f;
    }
    return;
  }
  for (int round = 0; round < K; ++round) {
    float v = -INFINITY; int f = 0x7fffffff;
    if (n <= BEAM_CAND_CAP) {
      for (int q = t; q < n; q += 256) {
        const float x = s_cv[q]; const int xi = s_ci[q];
        if ((x < pv || (x == pv && xi > pi)) && beam_better(x, xi, v, f)) { v = x; f = xi; }
      }
    } else {
      for (int c = t; c < nv4; c += 256) {
        const float4 q = *reinterpret_cast<const float4*>(zr + 4 * c);
        const float x[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int xi = 4 * c + i;
          if ((x[i] < pv || (x[i] == pv && xi > pi)) && beam_better(x[i], xi, v, f)) { v = x[i]; f = xi; }
        }
      }
    }
    beam_block_best(v, f, s_v, s_f);
    if (t == 0) { bs.cand_z[(size_t)r * BEAM_MAX + round] = v; bs.cand_tok[(size_t)r * BEAM_MAX + round] = f; }
    pv = v; pi = f;
  }
}

// One workgroup per sentence: the K best one-token extensions over the candidates of its live rows
// (equal scores: the lower (slot, token) pair first), finished hypotheses split off, history written.
__global__ __launch_bounds__(256) void beam_merge_kernel(int V, BeamState bs, int K, int j, int max_len, int eos, float alpha) {
  __shared__ float s_v[4];
  __shared__ int s_f[4];
  __shared__ float s_winv[BEAM_MAX];
  __shared__ int s_winf[BEAM_MAX];
  const int b = blockIdx.x, t = threadIdx.x;
  const int nl = bs.nlive[b];
  const int row0 = b * K;
  if (nl == 0) {                                         // the sentence is done (uniform over the workgroup)
    if (t < K) { bs.parent[row0 + t] = -1; bs.new_cum[row0 + t] = -INFINITY; }
    return;
  }
  // thread t holds candidate t % K of live row t / K (K * K <= 256)
  float cv = -INFINITY; int cf = 0x7fffffff;
  {
    const int s = t / K, i = t - s * K;
    if (s < nl) {
      const int r = row0 + s;
      const float zc = bs.cand_z[(size_t)r * BEAM_MAX + i];
      const int tk = bs.cand_tok[(size_t)r * BEAM_MAX + i];
      if (tk != 0x7fffffff) { cv = (bs.cum[r] - bs.row_lse[r]) + zc; cf = s * V + tk; }
    }
  }
  bool taken = false;
  for (int round = 0; round < K; ++round) {
    float v = taken ? -INFINITY : cv;
    int f = taken ? 0x7fffffff : cf;
    beam_block_best(v, f, s_v, s_f);
    if (t == 0) { s_winv[round] = v; s_winf[round] = f; }
    if (!taken && f == cf && cf != 0x7fffffff) taken = true;
  }
  __syncthreads();
  // ---- split the winners into finished and live hypotheses ---------------------------------------------
  if (t == 0) {
    int n_new = 0;
    const bool last = j == max_len - 1;
    for (int q = 0; q < K; ++q) {
      const float v = s_winv[q];
      const int f = s_winf[q];
      if (!(v > -INFINITY)) break;                       // fewer candidates than K
      const int s = f / V, tk = f - s * V;
      if (tk == eos || last) {
        const float norm = v / powf((5.f + (float)(j + 1)) / 6.f, alpha);
        if (norm > bs.fin_score[b]) {                    // strict: the hypothesis finished first keeps a tie
          bs.fin_score[b] = norm; bs.fin_step[b] = j; bs.fin_par[b] = s; bs.fin_tok[b] = tk;
        }
      } else {
        const int r = row0 + n_new;
        bs.new_cum[r] = v;
        bs.parent[r] = row0 + s;
        bs.new_tok[r] = tk;
        bs.hist_tok[(size_t)j * bs.hist_ld + r] = tk;
        bs.hist_par[(size_t)j * bs.hist_ld + r] = s;
        ++n_new;
      }
    }
    bs.nlive[b] = n_new;
    for (int q = n_new; q < K; ++q) { bs.new_cum[row0 + q] = -INFINITY; bs.parent[row0 + q] = -1; }
  }
}
void launch_beam_select(const float* z, int V, const BeamState& bs, int B, int K, int j, int max_len, int eos, float alpha,
                        hipStream_t st, int fast_exp) {
  if (fast_exp) hipLaunchKernelGGL(beam_row_topk_kernel<true>, dim3(B * K), dim3(256), 0, st, z, V, bs, K);
  else hipLaunchKernelGGL(beam_row_topk_kernel<false>, dim3(B * K), dim3(256), 0, st, z, V, bs, K);
  hipLaunchKernelGGL(beam_merge_kernel, dim3(B), dim3(256), 0, st, V, bs, K, j, max_len, eos, alpha);
}

// New row r takes the states of row parent[r] (or stays dead): per layer h (T) and c (fp32), and the
// H_o that becomes its input feed; scores, tokens and masks are switched over.
template <typename T>
__global__ __launch_bounds__(256) void beam_reorder_kernel(BeamReorder ro, BeamState bs, int H, int L) {
  const int r = blockIdx.x, t = threadIdx.x;
  const int pr = bs.parent[r];
  if (t == 0) {
    bs.cum[r] = bs.new_cum[r];
    bs.mask[r] = pr >= 0 ? 1.f : 0.f;
    if (pr >= 0) bs.tok[r] = bs.new_tok[r];
  }
  if (pr < 0) return;
  constexpr int VE = 16 / sizeof(T);
  for (int l = 0; l < L; ++l) {
    const T* hs = (const T*)ro.h_src[l] + (size_t)pr * ro.ldh;
    T* hd = (T*)ro.h_dst[l] + (size_t)r * ro.ldh;
    T* hf = (T*)ro.h_dst_fm[l];
    for (int c = t * VE; c < H; c += 256 * VE) {
      const uint4 v = *reinterpret_cast<const uint4*>(hs + c);
      *reinterpret_cast<uint4*>(hd + c) = v;
      if (sizeof(T) == 2 && hf) *reinterpret_cast<uint4*>(hf + fm_offset(r, c, H >> 5)) = v;   // 8 elements of one k chunk
    }
    const float* cs = ro.c_src[l] + (size_t)pr * H;
    float* cd = ro.c_dst[l] + (size_t)r * H;
    for (int c = t * 4; c < H; c += 256 * 4) *reinterpret_cast<float4*>(cd + c) = *reinterpret_cast<const float4*>(cs + c);
  }
  const T* os = (const T*)ro.ho_src + (size_t)pr * ro.ldho_src;
  T* od = (T*)ro.ho_dst + (size_t)r * ro.ldho_dst;
  T* of = (T*)ro.ho_dst_fm;
  for (int c = t * VE; c < H; c += 256 * VE) {
    const uint4 v = *reinterpret_cast<const uint4*>(os + c);
    *reinterpret_cast<uint4*>(od + c) = v;
    if (sizeof(T) == 2 && of) *reinterpret_cast<uint4*>(of + fm_offset(r, ro.ho_fm_k0 + c, ro.ho_fm_nsteps)) = v;
  }
}
void launch_beam_reorder(int prec, const BeamReorder& ro, const BeamState& bs, int R, int H, int L, hipStream_t st) {
  if (prec) hipLaunchKernelGGL(beam_reorder_kernel<bf16_t>, dim3(R), dim3(256), 0, st, ro, bs, H, L);
  else hipLaunchKernelGGL(beam_reorder_kernel<float>, dim3(R), dim3(256), 0, st, ro, bs, H, L);
}

// one thread per sentence: walk the back-pointers of the best finished hypothesis
__global__ __launch_bounds__(64) void beam_finish_kernel(BeamState bs, int B, int K, int max_len, int pad, int32_t* __restrict__ out_ids,
                                                         int32_t* __restrict__ out_len, float* __restrict__ out_score) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b >= B) return;
  const int j = bs.fin_step[b];
  const int len = j + 1;
  int32_t* o = out_ids + (size_t)b * max_len;
  for (int q = 0; q < max_len; ++q) o[q] = pad;
  out_len[b] = len;
  out_score[b] = bs.fin_score[b];
  if (j < 0) { out_len[b] = 0; return; }
  o[j] = bs.fin_tok[b];
  int s = bs.fin_par[b];
  for (int q = j - 1; q >= 0; --q) {
    const size_t i = (size_t)q * bs.hist_ld + b * K + s;
    o[q] = bs.hist_tok[i];
    s = bs.hist_par[i];
  }
}
void launch_beam_finish(const BeamState& bs, int B, int K, int max_len, int pad, int32_t* out_ids, int32_t* out_len, float* out_score,
                        hipStream_t st) {
  hipLaunchKernelGGL(beam_finish_kernel, dim3((B + 63) / 64), dim3(64), 0, st, bs, B, K, max_len, pad, out_ids, out_len, out_score);
}

}  // namespace cmt
