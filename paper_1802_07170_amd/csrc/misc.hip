// Memory-bound helpers of the training step: embedding gather (the paper's EmbeddingLayer
// forward) with masks and input validation, the deterministic embedding-gradient scatter (the
// paper's `firstOccurs` idea: the first occurrence of a word owns its gradient row), SGD, the
// counter-based initialiser, casts, copies and small reductions.
#include "common.h"
#include "kernels.h"

namespace cmt {

// one workgroup per (position t, sentence b)
template <typename T>
__global__ __launch_bounds__(128) void gather_kernel(const T* __restrict__ table, int vocab, int E,
                                                     const int32_t* __restrict__ ids, const int32_t* __restrict__ len,
                                                     int B, int Bp, int L, int shift, int bos, T* __restrict__ out,
                                                     float* __restrict__ mask, int32_t* __restrict__ tok,
                                                     int32_t* __restrict__ labels, int32_t* __restrict__ len_p,
                                                     int* __restrict__ flags) {
  const int t = blockIdx.x, b = blockIdx.y;
  const size_t row = (size_t)t * Bp + b;
  constexpr int EPC = 16 / sizeof(T);
  uint4* o = reinterpret_cast<uint4*>(out + row * E);
  const int nch = E / EPC;
  if (b >= B) {
    for (int c = threadIdx.x; c < nch; c += 128) o[c] = make_uint4(0, 0, 0, 0);
    if (threadIdx.x == 0) {
      mask[row] = 0.f; tok[row] = -1;
      if (labels) labels[row] = 0;
      if (t == 0) len_p[b] = 0;
    }
    return;
  }
  int n = len[b];
  if (n < 1 || n > L) { if (threadIdx.x == 0) atomicOr(flags, 2); n = n < 1 ? 1 : L; }
  int id = shift ? (t == 0 ? bos : ids[(size_t)b * L + t - 1]) : ids[(size_t)b * L + t];
  const bool valid = t < n;
  if (id < 0 || id >= vocab) { if (valid && threadIdx.x == 0) atomicOr(flags, 1); id = 0; }
  const uint4* src = reinterpret_cast<const uint4*>(table + (size_t)id * E);
  for (int c = threadIdx.x; c < nch; c += 128) o[c] = src[c];
  if (threadIdx.x == 0) {
    mask[row] = valid ? 1.f : 0.f;
    tok[row] = valid ? id : -1;
    if (labels) {
      int y = ids[(size_t)b * L + t];
      if (y < 0 || y >= vocab) { if (valid) atomicOr(flags, 1); y = 0; }
      labels[row] = y;
    }
    if (t == 0) len_p[b] = n;
  }
}

void launch_gather(int prec, const void* table, int vocab, int E, const int32_t* ids, const int32_t* len,
                   int B, int Bp, int L, int shift, int bos, void* out, float* mask, int32_t* tok,
                   int32_t* labels, int32_t* len_p, int* flags, hipStream_t st) {
  dim3 grid(L, Bp);
  if (prec) hipLaunchKernelGGL(gather_kernel<bf16_t>, grid, dim3(128), 0, st, (const bf16_t*)table, vocab, E, ids, len, B, Bp, L,
                               shift, bos, (bf16_t*)out, mask, tok, labels, len_p, flags);
  else hipLaunchKernelGGL(gather_kernel<float>, grid, dim3(128), 0, st, (const float*)table, vocab, E, ids, len, B, Bp, L,
                          shift, bos, (float*)out, mask, tok, labels, len_p, flags);
}

// One workgroup per position p.  If no earlier position holds the same id, this workgroup sums the gradient
// rows of every occurrence q >= p in ascending q and stores the whole row (each thread owns up to two groups of
// four consecutive columns, E <= 2048); otherwise it exits.  The occurrence scan is done once per position, and
// rows are fetched sixteen at a time as 16-byte vectors so their loads overlap.
constexpr int EMBED_SCATTER_MAX_E = 2048;
__global__ __launch_bounds__(256) void embed_scatter_kernel(const float* __restrict__ dX, const int32_t* __restrict__ tok,
                                                            int n, int E, float* __restrict__ dE) {
  __shared__ int s_found;
  __shared__ int s_list[256];
  __shared__ int s_wcnt[4];
  const int p = blockIdx.x, t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int id = tok[p];
  if (id < 0) return;
  if (t == 0) s_found = 0;
  __syncthreads();
  for (int q = t; q < p; q += 256)
    if (tok[q] == id) s_found = 1;
  __syncthreads();
  if (s_found) return;
  const int eq = E >> 2;                                  // float4 groups per row
  float4 acc[2] = {make_float4(0.f, 0.f, 0.f, 0.f), make_float4(0.f, 0.f, 0.f, 0.f)};
  for (int base = p; base < n; base += 256) {
    const int q = base + t;
    const bool match = q < n && tok[q] == id;
    const unsigned long long bal = __ballot(match);
    if (lane == 0) s_wcnt[w] = __popcll(bal);
    __syncthreads();
    int off = 0;
    for (int k = 0; k < w; ++k) off += s_wcnt[k];
    const int total = s_wcnt[0] + s_wcnt[1] + s_wcnt[2] + s_wcnt[3];
    if (match) s_list[off + __popcll(bal & ((1ull << lane) - 1ull))] = q;
    __syncthreads();
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const int c4 = t + 256 * g;
      if (c4 < eq) {
        for (int k = 0; k < total; k += 16) {             // 16 rows in flight: a frequent id's chain is latency-bound
          float4 v[16];
#pragma unroll
          for (int j = 0; j < 16; ++j)
            v[j] = k + j < total ? reinterpret_cast<const float4*>(dX + (size_t)s_list[k + j] * E)[c4] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
          for (int j = 0; j < 16; ++j) { acc[g].x += v[j].x; acc[g].y += v[j].y; acc[g].z += v[j].z; acc[g].w += v[j].w; }
        }
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    const int c4 = t + 256 * g;
    if (c4 < eq) reinterpret_cast<float4*>(dE + (size_t)id * E)[c4] = acc[g];
  }
}

__global__ __launch_bounds__(256) void fill_f32_kernel(float* __restrict__ p, size_t n, float v) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) p[i] = v;
}
static inline int grid_for(size_t n, int per_block = 256) {
  size_t g = (n + per_block - 1) / per_block;
  return (int)(g > 65536 ? 65536 : (g < 1 ? 1 : g));
}
void launch_fill_f32(float* p, size_t n, float v, hipStream_t st) {
  if (n == 0) return;
  hipLaunchKernelGGL(fill_f32_kernel, dim3(grid_for(n)), dim3(256), 0, st, p, n, v);
}
void launch_fill_T(int prec, void* p, size_t n, hipStream_t st) {
  // zero bits are zero in both types; fill as 32-bit words (n even for bf16 by construction of the callers)
  const size_t words = prec ? (n + 1) / 2 : n;
  launch_fill_f32((float*)p, words, 0.f, st);
}

void launch_embed_scatter(const float* dX, const int32_t* tok, int n, int V, int E, float* dE, hipStream_t st, bool zero_first) {
  if (zero_first) launch_fill_f32(dE, (size_t)V * E, 0.f, st);
  hipLaunchKernelGGL(embed_scatter_kernel, dim3(n), dim3(256), 0, st, dX, tok, n, E, dE);   // E <= EMBED_SCATTER_MAX_E (checked with the configuration)
}

template <typename T>
__global__ __launch_bounds__(256) void copy2d_kernel(const T* __restrict__ s, int lds, T* __restrict__ d, int ldd, int rows,
                                                     int cols) {
  const size_t n = (size_t)rows * cols;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) {
    const size_t r = i / cols, c = i - r * cols;
    d[r * ldd + c] = s[r * lds + c];
  }
}
void launch_copy2d_f32(const float* src, int lds, float* dst, int ldd, int rows, int cols, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return;
  hipLaunchKernelGGL(copy2d_kernel<float>, dim3(grid_for((size_t)rows * cols)), dim3(256), 0, st, src, lds, dst, ldd, rows, cols);
}
void launch_copy2d_T(int prec, const void* src, int lds, void* dst, int ldd, int rows, int cols, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return;
  if (prec) hipLaunchKernelGGL(copy2d_kernel<bf16_t>, dim3(grid_for((size_t)rows * cols)), dim3(256), 0, st, (const bf16_t*)src,
                               lds, (bf16_t*)dst, ldd, rows, cols);
  else launch_copy2d_f32((const float*)src, lds, (float*)dst, ldd, rows, cols, st);
}

struct FillJobs { FillJob j[MULTI_MAX_JOBS]; };
struct CopyJobs { CopyJob j[MULTI_MAX_JOBS]; };
__global__ __launch_bounds__(256) void fill_multi_kernel(FillJobs jobs) {
  const FillJob& job = jobs.j[blockIdx.y];
  uint32_t* p = (uint32_t*)job.p;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < job.words; i += stride) p[i] = 0u;
}
__global__ __launch_bounds__(256) void copy2d_multi_kernel(CopyJobs jobs) {
  const CopyJob& job = jobs.j[blockIdx.y];
  const uint32_t* s = (const uint32_t*)job.src;
  uint32_t* d = (uint32_t*)job.dst;
  const size_t n = (size_t)job.rows * job.cols, stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    const size_t r = i / job.cols, c = i - r * job.cols;
    d[r * job.ldd + c] = s[r * job.lds + c];
  }
}
void launch_fill_multi(const FillJob* jobs, int n, hipStream_t st) {
  for (int base = 0; base < n; base += MULTI_MAX_JOBS) {
    const int m = n - base < MULTI_MAX_JOBS ? n - base : MULTI_MAX_JOBS;
    FillJobs a;
    size_t most = 1;
    for (int i = 0; i < MULTI_MAX_JOBS; ++i) {
      a.j[i] = i < m ? jobs[base + i] : FillJob{nullptr, 0};
      if (a.j[i].words > most) most = a.j[i].words;
    }
    hipLaunchKernelGGL(fill_multi_kernel, dim3(grid_for(most), m), dim3(256), 0, st, a);
  }
}
void launch_copy2d_multi(const CopyJob* jobs, int n, hipStream_t st) {
  for (int base = 0; base < n; base += MULTI_MAX_JOBS) {
    const int m = n - base < MULTI_MAX_JOBS ? n - base : MULTI_MAX_JOBS;
    CopyJobs a;
    size_t most = 1;
    for (int i = 0; i < MULTI_MAX_JOBS; ++i) {
      a.j[i] = i < m ? jobs[base + i] : CopyJob{nullptr, 0, nullptr, 0, 0, 0};
      const size_t cnt = (size_t)a.j[i].rows * a.j[i].cols;
      if (cnt > most) most = cnt;
    }
    hipLaunchKernelGGL(copy2d_multi_kernel, dim3(grid_for(most), m), dim3(256), 0, st, a);
  }
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* __restrict__ s, bf16_t* __restrict__ d, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) d[i] = f2bf(s[i]);
}
void launch_cast(int prec, const float* src, void* dst, size_t n, hipStream_t st) {
  if (n == 0) return;
  if (prec) hipLaunchKernelGGL(cast_bf16_kernel, dim3(grid_for(n)), dim3(256), 0, st, src, (bf16_t*)dst, n);
  else hipLaunchKernelGGL(copy2d_kernel<float>, dim3(grid_for(n)), dim3(256), 0, st, src, 0, (float*)dst, 0, 1, (int)n);
}

__global__ __launch_bounds__(256) void add_f32_kernel(float* __restrict__ d, const float* __restrict__ s, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) d[i] += s[i];
}
void launch_add_f32(float* dst, const float* src, size_t n, hipStream_t st) {
  if (n == 0) return;
  hipLaunchKernelGGL(add_f32_kernel, dim3(grid_for(n)), dim3(256), 0, st, dst, src, n);
}

__global__ __launch_bounds__(256) void sum_parts_kernel(const float* __restrict__ parts, int nparts, size_t n,
                                                        float* __restrict__ out) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) {
    float a = 0.f;
    for (int p0 = 0; p0 < nparts; p0 += 8) {       // eight loads in flight, added in ascending order
      float v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = p0 + q < nparts ? parts[(size_t)(p0 + q) * n + i] : 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) a += v[q];
    }
    out[i] = a;
  }
}
void launch_sum_parts(const float* parts, int nparts, size_t n, float* out, hipStream_t st) {
  if (n == 0) return;
  hipLaunchKernelGGL(sum_parts_kernel, dim3(grid_for(n)), dim3(256), 0, st, parts, nparts, n, out);
}

// column sums of a T matrix [M, N]: 64 columns x 4 row groups per block, 16 row splits over grid.y
constexpr int COLSUM_SPLITS = 16;
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ G, int ld, int M, int N, float* __restrict__ parts) {
  __shared__ float red[4][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63), rg = threadIdx.x >> 6;
  const int rows_per = (M + COLSUM_SPLITS - 1) / COLSUM_SPLITS;
  const int r0 = blockIdx.y * rows_per, r1 = min(M, r0 + rows_per);
  float a = 0.f;
  if (c < N)
    for (int r = r0 + rg; r < r1; r += 4) a += to_f<T>(G[(size_t)r * ld + c]);
  red[rg][threadIdx.x & 63] = a;
  __syncthreads();
  if (rg == 0 && c < N) parts[(size_t)blockIdx.y * N + c] = red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] + red[3][threadIdx.x];
}
void launch_colsum(int prec, const void* dG, int ld, int M, int N, float* scratch, float* db, hipStream_t st) {
  dim3 grid((N + 63) / 64, COLSUM_SPLITS);
  if (prec) hipLaunchKernelGGL(colsum_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)dG, ld, M, N, scratch);
  else hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, st, (const float*)dG, ld, M, N, scratch);
  launch_sum_parts(scratch, COLSUM_SPLITS, (size_t)N, db, st);
}

// p <- p - lr g, four elements per thread and pass; with pc the bf16 working copy of the parameters is written in
// the same pass (one read of p less than a separate cast).  Nothing is updated while an error flag of an earlier
// step is pending (its gradients are undefined); the working copy then stays valid as it is.
__global__ __launch_bounds__(256) void sgd_kernel(float* __restrict__ p, const float* __restrict__ g, size_t n, float lr,
                                                  const int* __restrict__ flags, bf16_t* __restrict__ pc) {
  if (flags && *flags) return;
  const size_t n4 = n >> 2;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    float4 a = reinterpret_cast<const float4*>(p)[i];
    const float4 b = reinterpret_cast<const float4*>(g)[i];
    a.x -= lr * b.x; a.y -= lr * b.y; a.z -= lr * b.z; a.w -= lr * b.w;
    reinterpret_cast<float4*>(p)[i] = a;
    if (pc) {
      uint2 o;
      o.x = (uint32_t)f2bf(a.x) | ((uint32_t)f2bf(a.y) << 16);
      o.y = (uint32_t)f2bf(a.z) | ((uint32_t)f2bf(a.w) << 16);
      reinterpret_cast<uint2*>(pc)[i] = o;
    }
  }
  for (size_t i = (n4 << 2) + (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    const float v = p[i] - lr * g[i];
    p[i] = v;
    if (pc) pc[i] = f2bf(v);
  }
}
void launch_sgd(float* p, const float* g, size_t n, float lr, const int* flags, void* bf16_copy, hipStream_t st) {
  if (n == 0) return;
  hipLaunchKernelGGL(sgd_kernel, dim3(grid_for((n + 3) / 4)), dim3(256), 0, st, p, g, n, lr, flags, (bf16_t*)bf16_copy);
}

// SplitMix64 of (seed + element index); top 24 bits -> uniform [-scale, scale)
__global__ __launch_bounds__(256) void init_uniform_kernel(float* __restrict__ p, size_t n, uint64_t seed, float scale) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) {
    uint64_t x = seed + (uint64_t)i + 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    x = x ^ (x >> 31);
    const float u = (float)(uint32_t)(x >> 40);
    p[i] = (u * (2.0f / 16777216.0f) - 1.0f) * scale;
  }
}
void launch_init_uniform(float* p, size_t n, uint64_t seed, float scale, hipStream_t st) {
  if (n == 0) return;
  hipLaunchKernelGGL(init_uniform_kernel, dim3(grid_for(n)), dim3(256), 0, st, p, n, seed, scale);
}

// ------------------------------------------------------------------------------------------------
// Measurement aid: what a chip-wide barrier between resident workgroups costs — the price a persistent,
// weight-stationary recurrence would pay per time step instead of a kernel boundary.  Every workgroup
// arrives with one device-scope atomic increment and polls the counter until all have arrived; with
// `fences` the arrival is preceded and the departure followed by a device-scope fence, as an exchange of
// data between the workgroups needs (each XCD has its own L2).  The wait is bounded: after max_spin polls a
// workgroup gives up, raises *gave_up and leaves, so the kernel ends whatever happens (e.g. when not all
// workgroups are resident at once).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void grid_barrier_probe_kernel(unsigned* __restrict__ counter, int rounds, int fences, int max_spin,
                                                                 int* __restrict__ gave_up) {
  __shared__ int s_stop;
  const unsigned n = gridDim.x;
  for (int r = 0; r < rounds; ++r) {
    __syncthreads();
    if (threadIdx.x == 0) {
      if (fences) __threadfence();
      atomicAdd(counter, 1u);
      const unsigned target = (unsigned)(r + 1) * n;
      int spin = 0;
      while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target && spin < max_spin) ++spin;
      s_stop = spin >= max_spin;
      if (s_stop) atomicOr(gave_up, 1);
      if (fences) __threadfence();
    }
    __syncthreads();
    if (s_stop) break;
  }
}
void launch_grid_barrier_probe(unsigned* counter, int* gave_up, int blocks, int rounds, int fences, int max_spin, hipStream_t st) {
  hipLaunchKernelGGL(grid_barrier_probe_kernel, dim3(blocks), dim3(256), 0, st, counter, rounds, fences, max_spin, gave_up);
}

// ------------------------------------------------------------------------------------------------
// greedy decoding helpers
// ------------------------------------------------------------------------------------------------
// x[b, 0:E] = table[tok[b]] for b < B, zero rows for the batch padding
template <typename T>
__global__ __launch_bounds__(128) void dec_embed_kernel(const T* __restrict__ table, int E, const int32_t* __restrict__ tok, int B,
                                                        T* __restrict__ x, int ldx, T* __restrict__ x_fm, int nsteps_fm) {
  const int b = blockIdx.x;
  const T* src = b < B ? table + (size_t)tok[b] * E : nullptr;
  for (int c = threadIdx.x * 8; c < E; c += 128 * 8) {
    uint4 v[sizeof(T) / 2];                              // 8 elements
    if (src) for (int q = 0; q < (int)(sizeof(T) / 2); ++q) v[q] = reinterpret_cast<const uint4*>(src + c)[q];
    else for (int q = 0; q < (int)(sizeof(T) / 2); ++q) v[q] = make_uint4(0, 0, 0, 0);
    for (int q = 0; q < (int)(sizeof(T) / 2); ++q) reinterpret_cast<uint4*>(x + (size_t)b * ldx + c)[q] = v[q];
    if (sizeof(T) == 2 && x_fm) *reinterpret_cast<uint4*>(x_fm + fm_offset(b, c, nsteps_fm)) = v[0];   // 8 elements of one k chunk
  }
}
void launch_dec_embed(int prec, const void* table, int E, const int32_t* tok, int B, int Bp, void* x, int ldx, hipStream_t st,
                      void* x_fm, int nsteps_fm) {
  if (prec) hipLaunchKernelGGL(dec_embed_kernel<bf16_t>, dim3(Bp), dim3(128), 0, st, (const bf16_t*)table, E, tok, B, (bf16_t*)x, ldx,
                               (bf16_t*)x_fm, nsteps_fm);
  else hipLaunchKernelGGL(dec_embed_kernel<float>, dim3(Bp), dim3(128), 0, st, (const float*)table, E, tok, B, (float*)x, ldx,
                          (float*)nullptr, 0);
}

// One workgroup per sentence: token = argmax_v (z[b, v] + bias[v]), the lowest index winning a tie.
// A sentence that has not ended records the token at out_ids[b, j]; it ends when the token is eos or
// j is the last step.  tok[b] (the next step's input) is always updated.
// With a table the workgroup then copies the token's embedding row into the next step's input x[b, 0:E] (and its
// fragment-major copy): the lookup needs no launch of its own in the chain of dependent kernels.
template <typename T>
__global__ __launch_bounds__(1024) void dec_argmax_kernel(const float* __restrict__ z, int ldz, const float* __restrict__ bias, int V,
                                                          int j, int max_len, int eos, int32_t* __restrict__ tok,
                                                          int32_t* __restrict__ done, int32_t* __restrict__ out_ids,
                                                          int32_t* __restrict__ out_len, const T* __restrict__ table, int E,
                                                          T* __restrict__ x, int ldx, T* __restrict__ x_fm, int nsteps_fm,
                                                          const int32_t* __restrict__ part_idx) {
  __shared__ float smax[16];
  __shared__ int sidx[16];
  __shared__ int s_tok;
  const int b = blockIdx.x, t = threadIdx.x;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  // equal values: the lowest index wins, whatever order the candidates come in
  const float* zr = z + (size_t)b * ldz;
  if (part_idx) {                                        // partial results [k][sentence]: value and token
    for (int k = t; k < V; k += 1024) {
      const float xv = z[(size_t)k * ldz + b];
      const int xi = part_idx[(size_t)k * ldz + b];
      if (xv > best || (xv == best && xi < bi)) { best = xv; bi = xi; }
    }
  } else
  if ((V & 3) == 0 && (ldz & 3) == 0 && (((size_t)z | (size_t)bias) & 15) == 0) {
    for (int v = 4 * t; v < V; v += 4096) {              // 16-byte loads: four candidates per thread and pass
      const float4 a = *reinterpret_cast<const float4*>(zr + v);
      const float4 c = *reinterpret_cast<const float4*>(bias + v);
      const float x[4] = {a.x + c.x, a.y + c.y, a.z + c.z, a.w + c.w};
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (x[q] > best || (x[q] == best && v + q < bi)) { best = x[q]; bi = v + q; }
    }
  } else {
    for (int v = t; v < V; v += 1024) {
      const float x = zr[v] + bias[v];
      if (x > best || (x == best && v < bi)) { best = x; bi = v; }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
  }
  if ((t & 63) == 0) { smax[t >> 6] = best; sidx[t >> 6] = bi; }
  __syncthreads();
  if (t == 0) {
    for (int w = 1; w < 16; ++w)
      if (smax[w] > best || (smax[w] == best && sidx[w] < bi)) { best = smax[w]; bi = sidx[w]; }
    if (bi == 0x7fffffff) bi = 0;                        // a row of NaNs: keep the token in range
    tok[b] = bi;
    s_tok = bi;
    if (!done[b]) {
      out_ids[(size_t)b * max_len + j] = bi;
      if (bi == eos || j == max_len - 1) { done[b] = 1; out_len[b] = j + 1; }
    }
  }
  if (!table) return;
  __syncthreads();
  const T* src = table + (size_t)s_tok * E;
  constexpr int EPC = 16 / sizeof(T);                     // elements per 16-byte chunk
  for (int c = t * EPC; c < E; c += 1024 * EPC) {
    const uint4 v = *reinterpret_cast<const uint4*>(src + c);
    *reinterpret_cast<uint4*>(x + (size_t)b * ldx + c) = v;
    if (sizeof(T) == 2 && x_fm) *reinterpret_cast<uint4*>(x_fm + fm_offset(b, c, nsteps_fm)) = v;
  }
}
void launch_dec_argmax(const float* z, int ldz, const float* bias, int V, int B, int j, int max_len, int eos, int32_t* tok,
                       int32_t* done, int32_t* out_ids, int32_t* out_len, hipStream_t st, int prec, const void* table, int E, void* x,
                       int ldx, void* x_fm, int nsteps_fm, const int32_t* part_idx) {
  if (prec)
    hipLaunchKernelGGL(dec_argmax_kernel<bf16_t>, dim3(B), dim3(1024), 0, st, z, ldz, bias, V, j, max_len, eos, tok, done, out_ids, out_len,
                       (const bf16_t*)table, E, (bf16_t*)x, ldx, (bf16_t*)x_fm, nsteps_fm, part_idx);
  else
    hipLaunchKernelGGL(dec_argmax_kernel<float>, dim3(B), dim3(1024), 0, st, z, ldz, bias, V, j, max_len, eos, tok, done, out_ids, out_len,
                       (const float*)table, E, (float*)x, ldx, (float*)nullptr, 0, part_idx);
}

// start of a decode: tok = bos, done = 0, out_ids = pad, out_len = 0, mask = 1 for b < B else 0
__global__ __launch_bounds__(256) void dec_init_kernel(int B, int Bp, int max_len, int bos, int pad, int32_t* __restrict__ tok,
                                                       int32_t* __restrict__ done, int32_t* __restrict__ out_ids,
                                                       int32_t* __restrict__ out_len, float* __restrict__ mask) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < Bp) { tok[i] = bos; done[i] = 0; mask[i] = i < B ? 1.f : 0.f; }
  if (i < B) out_len[i] = 0;
  if (i < B * max_len) out_ids[i] = pad;
}
void launch_dec_init(int B, int Bp, int max_len, int bos, int pad, int32_t* tok, int32_t* done, int32_t* out_ids, int32_t* out_len,
                     float* mask, hipStream_t st) {
  const int n = B * max_len > Bp ? B * max_len : Bp;
  hipLaunchKernelGGL(dec_init_kernel, dim3((n + 255) / 256), dim3(256), 0, st, B, Bp, max_len, bos, pad, tok, done, out_ids, out_len, mask);
}

}  // namespace cmt
