// Kernels of the two time loops (encoder / decoder recurrences and their backward passes).
// Per step the batch is tiny (M = B <= 128): the layer's weights are streamed from HBM once, and what
// a launch waits for is the traffic from L2 to the CUs — weights once, plus the step's activations once
// per workgroup that needs them.  These kernels therefore put the WEIGHT rows on the matrix cores' row
// side (16-row tiles read straight from global memory into MFMA fragments, no LDS staging) and the
// batch on the column side, and choose how many row tiles and sentence tiles a workgroup owns so that
// the sum of both kinds of traffic is small while the chip stays full.  The wavefronts of a workgroup
// split the k range; every wavefront issues all loads of a round before its first MFMA so that a
// whole workgroup's operand bytes are in flight at once, and the partial tiles are combined through
// LDS.  A k range split over workgroups gives partial "planes" that the consuming kernel sums (no
// atomics, fixed order).
// For the LSTM a 16-row tile is the four gates of four hidden units, so that after the reduction
// every lane holds i, f, g, o of one (unit, sentence) pair and the cell update is fused in-register.
// Workgroup numbering is XCD-aware: the hardware deals consecutive workgroup ids round-robin to
// the 8 XCDs, so the workgroups that share a weight tile (different sentence groups) get ids 8 apart
// and meet in one L2.
#include <stdlib.h>

#include <algorithm>

#include "common.h"
#include "kernels.h"

namespace cmt {

constexpr int STEP_MAXBT = 4;          // batch tiles (of 16 sentences) per workgroup

struct StepGrid { int nx, kb, nz; };
struct StepGemmArgs { StepGemm g[STEP_MAX_INST]; };
struct LstmBwdPointArgs { LstmBwdPoint p[STEP_MAX_INST]; };
__device__ __forceinline__ bool decode_block(const StepGrid& g, int& x, int& kb, int& z) {
  const int L = blockIdx.x;
  const int xcd = L & 7;
  int r = L >> 3;
  // (an integer division costs some twenty instructions at the head of a kernel that lasts microseconds: the
  // common counts, one and powers of two, go without)
  if (g.nz == 1) z = 0;
  else if ((g.nz & (g.nz - 1)) == 0) { z = r & (g.nz - 1); r >>= __builtin_ctz(g.nz); }
  else { z = r % g.nz; r /= g.nz; }
  if (g.kb == 1) kb = 0;
  else if ((g.kb & (g.kb - 1)) == 0) { kb = r & (g.kb - 1); r >>= __builtin_ctz(g.kb); }
  else { kb = r % g.kb; r /= g.kb; }
  x = xcd + 8 * r;
  return x < g.nx;
}
static inline int step_grid_blocks(const StepGrid& g) { return ((g.nx + 7) / 8) * 8 * g.kb * g.nz; }

// Split-k contraction of RT 16-row weight tiles against up to 64 sentences inside one workgroup.
// Wavefront w takes k-steps w + KS * (u + U * round); fragment chunk c of the concatenated k axis
// [a0 (K0); a1 (K1)] covers 8 elements; all loads of a round are issued before its first MFMA.
// The partial tiles go through LDS; afterwards tile t = rt * STEP_MAXBT + bt is summed by wavefront
// t % KS.  red must hold KS * RT * STEP_MAXBT * 256 floats.
template <typename T, int RT, int KS, int U, int BT = STEP_MAXBT>
__device__ __forceinline__ void step_contract(const T* const (&wrow)[RT], int w0_off, int w1_off, const T* a0, int lda0,
                                              int K0, const T* a1, int lda1, int K1, int Bp, int bt0, int nbt, float* red) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int nc0 = K0 >> 3, nc = (K0 + K1) >> 3;
  const int nsteps = (nc + 3) >> 2;
  const int brow = 16 * bt0 + (lane & 15);
  v4f acc[RT][BT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int b = 0; b < BT; ++b) acc[rt][b] = v4f{0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < nsteps; s0 += KS * U) {
    Frag<T> fw[U][RT], fx[U][BT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int chunk = 4 * (s0 + w + KS * u) + (lane >> 4);
      if (chunk < nc) {
        const bool first = chunk < nc0;
        const int kk = first ? chunk * 8 : (chunk - nc0) * 8;
        const int wo = (first ? w0_off : w1_off) + kk;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) fw[u][rt].load(wrow[rt] + wo);
        const T* a = first ? a0 : a1;
        const int lda = first ? lda0 : lda1;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
          if (b < nbt) fx[u][b].load(a + (size_t)min(brow + 16 * b, Bp - 1) * lda + kk);
          else fx[u][b].zero();
        }
      } else {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) fw[u][rt].zero();
#pragma unroll
        for (int b = 0; b < BT; ++b) fx[u][b].zero();
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int b = 0; b < BT; ++b) mma16(acc[rt][b], fw[u][rt], fx[u][b]);
  }
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int b = 0; b < BT; ++b)
      *reinterpret_cast<v4f*>(red + (((w * RT + rt) * BT + b) * 64 + lane) * 4) = acc[rt][b];
  __syncthreads();
}
template <int RT, int KS, int BT = STEP_MAXBT>
__device__ __forceinline__ v4f step_tile_sum(const float* red, int rt, int bt) {
  const int lane = threadIdx.x & 63;
  v4f r = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < KS; ++k) r += *reinterpret_cast<const v4f*>(red + (((k * RT + rt) * BT + bt) * 64 + lane) * 4);
  return r;
}

// The same contraction on fragment-major operands (bf16): wt[rt] = first block of row tile rt (its k steps follow
// each other), a0 / a1 = fragment-major activation segments of ns0 / ns1 k steps (batch tile bt at bt * ns blocks).
// [s_begin, s_end) = the k steps this workgroup contracts (default: all).
// `after_first_loads` runs once, behind the loads of the first round: a kernel whose operand addresses arrived in
// registers (leading kernel arguments) fetches the rest of its arguments there, in the shadow of those loads.
struct StepNoHook { __device__ __forceinline__ void operator()() const {} };
// HookLate: behind the first round's matrix operations instead (the hook's own loads then do not meet the first
// round's fragments in the register file; for kernels at the register limit whose k range takes several rounds).
template <int RT, int KS, int U, int BT, typename Hook = StepNoHook, bool HookLate = false>
__device__ __forceinline__ void step_contract_fm(const bf16_t* const (&wt)[RT], const bf16_t* a0, int ns0, const bf16_t* a1, int ns1,
                                                 int bt0, int nbt, float* red, int s_begin = 0, int s_end = 1 << 30,
                                                 Hook after_first_loads = Hook{}) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int nsteps = min(ns0 + ns1, s_end);
  bool hook_due = true;
  v4f acc[RT][BT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int b = 0; b < BT; ++b) acc[rt][b] = v4f{0.f, 0.f, 0.f, 0.f};
  for (int s0 = s_begin; s0 < nsteps; s0 += KS * U) {
    Frag<bf16_t> fw[U][RT], fx[U][BT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int s = s0 + w + KS * u;
      if (s < nsteps) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) fw[u][rt].load(wt[rt] + ((size_t)s * 64 + lane) * 8);
        const bool first = s < ns0;
        const bf16_t* a = first ? a0 : a1;
        const int ns = first ? ns0 : ns1, sl = first ? s : s - ns0;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
          if (b < nbt) fx[u][b].load(a + (((size_t)(bt0 + b) * ns + sl) * 64 + lane) * 8);
          else fx[u][b].zero();
        }
      } else {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) fw[u][rt].zero();
#pragma unroll
        for (int b = 0; b < BT; ++b) fx[u][b].zero();
      }
    }
    if (!HookLate && hook_due) { after_first_loads(); hook_due = false; }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int b = 0; b < BT; ++b) mma16(acc[rt][b], fw[u][rt], fx[u][b]);
    if (HookLate && hook_due) { after_first_loads(); hook_due = false; }
  }
  if (hook_due) after_first_loads();
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int b = 0; b < BT; ++b)
      *reinterpret_cast<v4f*>(red + (((w * RT + rt) * BT + b) * 64 + lane) * 4) = acc[rt][b];
  __syncthreads();
}

// dots[b, i] = vec[b, :] . Mat[i, b, :] for position i < len[b] of sentence b, by one wavefront
template <typename MT, typename T>
__device__ __forceinline__ void att_dots_row(const MT* __restrict__ Mat, int ldm, const T* __restrict__ vec, int ldv,
                                             const int32_t* __restrict__ len, int S, int Bp, int H, float* __restrict__ dots, int i, int b) {
  const int lane = threadIdx.x & 63;
  if (i >= S || i >= len[b]) return;
  const MT* row = Mat + ((size_t)i * Bp + b) * ldm;
  float a = 0.f;
  for (int c = lane; c < (H >> 3); c += 64) {
    Frag<T> fv;
    Frag<MT> f;
    fv.load(vec + (size_t)b * ldv + 8 * c);
    f.load(row + 8 * c);
#pragma unroll
    for (int e = 0; e < 8; ++e) a += f.get(e) * fv.get(e);
  }
  a = wave_sum(a);
  if (lane == 0) dots[(size_t)b * S + i] = a;
}

// keep-and-rescale factor of element (b, col) of a dropout slice (see DropSpec)
__device__ __forceinline__ float drop_factor(const DropSpec& d, int b, int col) {
  if (!d.on) return 1.f;
  unsigned long long x = d.key0 + (unsigned long long)b * (unsigned long long)d.width + (unsigned long long)col;
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  x ^= x >> 31;
  return (unsigned)(x >> 40) >= d.thresh ? d.scale : 0.f;
}

__device__ __forceinline__ float planes_get(const Planes& p, int b, int c) {
  float v = 0.f;
  for (int k = 0; k < p.np; ++k) v += p.p[(size_t)k * p.stride + (size_t)b * p.ld + c];
  return v;
}

// ------------------------------------------------------------------------------------------------
// Row-major -> fragment-major copies (16-bit elements)
// ------------------------------------------------------------------------------------------------
// one thread per 16-byte chunk of the destination: block (row tile, k step), lane, 8 elements
__global__ __launch_bounds__(256) void fm_pack_kernel(const bf16_t* __restrict__ src, int ld, int rows, int nsteps, bf16_t* __restrict__ dst,
                                                      int dst_nsteps, int dst_step0) {
  const size_t n = (size_t)(rows >> 4) * nsteps * 64;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const int lane = (int)(i & 63);
    const size_t blk = i >> 6;
    const int s = (int)(blk % nsteps), rt = (int)(blk / nsteps);
    const int row = rt * 16 + (lane & 15), k = s * 32 + (lane >> 4) * 8;
    const size_t o = (((size_t)rt * dst_nsteps + dst_step0 + s) * 64 + lane) * 8;
    *reinterpret_cast<uint4*>(dst + o) = *reinterpret_cast<const uint4*>(src + (size_t)row * ld + k);
  }
}
void launch_fm_pack(const void* src, int ld, int rows, int cols, void* dst, hipStream_t st, int dst_nsteps, int dst_step0) {
  const size_t n = (size_t)(rows >> 4) * (cols >> 5) * 64;
  if (n == 0) return;
  size_t g = (n + 255) / 256;
  if (g > 65535) g = 65535;
  if (dst_nsteps <= 0) { dst_nsteps = cols >> 5; dst_step0 = 0; }
  hipLaunchKernelGGL(fm_pack_kernel, dim3((unsigned)g), dim3(256), 0, st, (const bf16_t*)src, ld, rows, cols >> 5, (bf16_t*)dst, dst_nsteps,
                     dst_step0);
}
__global__ __launch_bounds__(256) void fm_pack_lstm_weights_kernel(const bf16_t* __restrict__ W, int ldw, int col0, int nsteps, int Hh,
                                                                   bf16_t* __restrict__ dst) {
  const size_t n = (size_t)(Hh >> 2) * nsteps * 64;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const int lane = (int)(i & 63);
    const size_t blk = i >> 6;
    const int s = (int)(blk % nsteps), tile = (int)(blk / nsteps);
    const int m = lane & 15;
    const int row = (m & 3) * Hh + 4 * tile + (m >> 2), k = col0 + s * 32 + (lane >> 4) * 8;
    *reinterpret_cast<uint4*>(dst + i * 8) = *reinterpret_cast<const uint4*>(W + (size_t)row * ldw + k);
  }
}
void launch_fm_pack_lstm_weights(const void* W, int ldw, int col0, int K, int Hh, void* dst, hipStream_t st) {
  const size_t n = (size_t)(Hh >> 2) * (K >> 5) * 64;
  if (n == 0) return;
  size_t g = (n + 255) / 256;
  if (g > 65535) g = 65535;
  hipLaunchKernelGGL(fm_pack_lstm_weights_kernel, dim3((unsigned)g), dim3(256), 0, st, (const bf16_t*)W, ldw, col0, K >> 5, Hh,
                     (bf16_t*)dst);
}

// ------------------------------------------------------------------------------------------------
// LSTM forward step
// ------------------------------------------------------------------------------------------------
struct LstmFwdArgs { LstmFwdDir d[STEP_MAX_INST]; };

// everything the cell update of one (sentence, unit) reads besides the GEMM result; loaded before the
// contraction so that its latency hides behind the weight stream
struct CellIn { float add[4]; float cp, hp, mask; };
__device__ __forceinline__ CellIn cell_load(const LstmFwdDir& d, int b, int u, int Hh, bool is_bf16) {
  CellIn in;
#pragma unroll
  for (int g = 0; g < 4; ++g) in.add[g] = d.gx ? d.gx[(size_t)b * d.ldgx + g * Hh + u] : d.bias[g * Hh + u];
  in.cp = d.cprev[(size_t)b * Hh + u];
  in.mask = d.mask[b];
  in.hp = is_bf16 ? bf2f(((const bf16_t*)d.hprev)[(size_t)b * d.ldh + u]) : ((const float*)d.hprev)[(size_t)b * d.ldh + u];
  return in;
}
__device__ __forceinline__ void cell_finish(const LstmFwdDir& d, int b, int u, int Hh, const float (&pre)[4], const CellIn& in,
                                            bool is_bf16) {
  float ig, fg, gg, og, tcn;
  if (is_bf16) {
    ig = sigm_of<true>(pre[0] + in.add[0]); fg = sigm_of<true>(pre[1] + in.add[1]);
    gg = tanh_of<true>(pre[2] + in.add[2]); og = sigm_of<true>(pre[3] + in.add[3]);
  } else {
    ig = sigm_of<false>(pre[0] + in.add[0]); fg = sigm_of<false>(pre[1] + in.add[1]);
    gg = tanh_of<false>(pre[2] + in.add[2]); og = sigm_of<false>(pre[3] + in.add[3]);
  }
  const float cn = fg * in.cp + ig * gg;
  tcn = is_bf16 ? tanh_of<true>(cn) : tanh_of<false>(cn);
  const float hn = og * tcn;
  const bool valid = in.mask > 0.f;
  d.cnext[(size_t)b * Hh + u] = valid ? cn : in.cp;
  float* gs = d.gsave + (size_t)b * 4 * Hh + u;
  gs[0] = ig; gs[Hh] = fg; gs[2 * Hh] = gg; gs[3 * Hh] = og;
  const float hv = valid ? hn : in.hp;
  const float yv = d.ycat ? hv * drop_factor(d.drop, b, d.drop_col0 + u) : 0.f;
  if (is_bf16) {
    ((bf16_t*)d.hnext)[(size_t)b * d.ldhn + u] = f2bf(hv);   // a carried state is already a bf16 value: exact
    if (d.ycat) ((bf16_t*)d.ycat)[(size_t)b * d.ldy + u] = f2bf(yv);
    if (d.hnext_fm) ((bf16_t*)d.hnext_fm)[fm_offset(b, u, Hh >> 5)] = f2bf(hv);
    if (d.ycat_fm) ((bf16_t*)d.ycat_fm)[fm_offset(b, u, Hh >> 5)] = f2bf(yv);
  } else {
    ((float*)d.hnext)[(size_t)b * d.ldhn + u] = hv;
    if (d.ycat) ((float*)d.ycat)[(size_t)b * d.ldy + u] = yv;
  }
}

// RT row tiles = 4 * RT hidden units x 4 gates, and BT batch tiles of 16 sentences, per workgroup; the
// whole k range inside the workgroup.  Per workgroup RT weight slabs and BT activation slabs cross L2:
// for 64 sentences RT = BT = 2 moves the fewest bytes (each weight slab is then read by two workgroups,
// which the XCD-aware numbering puts on the same L2).
// The operand addresses of the fragment-major contraction and the grid lead the argument list (for one instance:
// W_fm0, x_fm0, hprev_fm0, Kx0 are that instance's), so that they arrive in registers and the first loads go out
// before the argument buffer has been read; the rest (args) is fetched behind those loads.  The grid follows from
// Hh, Bp and the instance count as the launcher computes it.
// nlead = how many instances the leading arguments describe: 1, or 2 when the launch's two instances have no
// input segment (Kx = 0: the bottom encoder layer's directions) — then W_fm1 / hprev_fm1 are the second one's.
template <typename T, int RT, int KS, int U, int BT, bool FM = false>
__global__ __launch_bounds__(64 * KS) void lstm_fwd_kernel(const void* W_fm0, const void* x_fm0, const void* hprev_fm0,
                                                           const void* W_fm1, const void* hprev_fm1, int Kx0, int Bp, int Hh,
                                                           int ndir_nlead, LstmFwdArgs args) {
  __shared__ __align__(16) float red[KS * RT * BT * 256];
  const int ndir = ndir_nlead & 0xffff, nlead = ndir_nlead >> 16;
  const int nxd = (Hh + 4 * RT - 1) / (4 * RT);    // unit blocks per direction
  const int nx = nxd * ndir, nz = ((Bp + 15) / 16 + BT - 1) / BT;
  const StepGrid sg{nx, 1, nz};
  int x, kb, z;
  if (!decode_block(sg, x, kb, z)) return;
  const int dir = ndir == 1 ? 0 : x / nxd;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int u0 = (x - dir * nxd) * 4 * RT;
  const int bt0 = z * BT;
  const int nbt = min(BT, (Bp + 15) / 16 - bt0);
  LstmFwdDir d;
  CellIn in0;
  bool have0 = false;
  auto fetch_rest = [&]() {
    // (the instance index passes through an opaque register and a compiler barrier: otherwise the compiler moves this
    // block, which depends on nothing before it, back in front of the contraction's loads)
    int dsel = __builtin_amdgcn_readfirstlane(dir);
    asm volatile("" : "+s"(dsel) : : "memory");
    d = args.d[dsel];
    // what the epilogue needs is fetched now, not behind the barrier
    CMT_PIN_UNIFORM_PTR(d.cnext); CMT_PIN_UNIFORM_PTR(d.gsave); CMT_PIN_UNIFORM_PTR(d.hnext); CMT_PIN_UNIFORM(d.ldhn);
    CMT_PIN_UNIFORM_PTR(d.ycat); CMT_PIN_UNIFORM(d.ldy); CMT_PIN_UNIFORM_PTR(d.hnext_fm); CMT_PIN_UNIFORM_PTR(d.ycat_fm);
    CMT_PIN_UNIFORM(d.drop.on); CMT_PIN_UNIFORM(d.drop_col0);
    CMT_PIN_UNIFORM_PTR(d.gx); CMT_PIN_UNIFORM(d.ldgx); CMT_PIN_UNIFORM_PTR(d.bias); CMT_PIN_UNIFORM_PTR(d.cprev); CMT_PIN_UNIFORM_PTR(d.mask);
    CMT_PIN_UNIFORM_PTR(d.hprev); CMT_PIN_UNIFORM(d.ldh);
    // the first tile this wavefront will finish: fetch its cell inputs now
    if (w < RT * BT) {
      const int rt = w / BT, bt = w - rt * BT;
      const int u = u0 + 4 * rt + (lane >> 4), b = 16 * (bt0 + bt) + (lane & 15);
      have0 = bt < nbt && u < Hh && b < Bp;
      if (have0) in0 = cell_load(d, b, u, Hh, sizeof(T) == 2);
    }
  };
  if constexpr (FM) {
    const bf16_t *Wf = (const bf16_t*)W_fm0, *xf = (const bf16_t*)x_fm0, *hf = (const bf16_t*)hprev_fm0;
    int Kx = Kx0;
    if (dir == 1 && nlead == 2) { Wf = (const bf16_t*)W_fm1; hf = (const bf16_t*)hprev_fm1; }
    else if (dir >= nlead) {
      Wf = (const bf16_t*)args.d[dir].W_fm; xf = (const bf16_t*)args.d[dir].x_fm; hf = (const bf16_t*)args.d[dir].hprev_fm;
      Kx = args.d[dir].Kx;
    }
    const int ns0 = Kx >> 5, ns1 = Hh >> 5;
    const bf16_t* wt[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) wt[rt] = Wf + (size_t)((u0 >> 2) + rt) * (ns0 + ns1) * 512;
    step_contract_fm<RT, KS, U, BT>(wt, xf, ns0, hf, ns1, bt0, nbt, red, 0, 1 << 30, fetch_rest);
  } else {
    fetch_rest();
    // row m = lane % 16 of row tile rt: gate m % 4 of unit u0 + 4 * rt + m / 4
    const int m = lane & 15;
    const T* wrow[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
      wrow[rt] = (const T*)d.W + (size_t)((m & 3) * Hh + min(u0 + 4 * rt + (m >> 2), Hh - 1)) * d.ldw;
    step_contract<T, RT, KS, U, BT>(wrow, d.wx_off, d.wh_off, (const T*)d.x, d.ldx, d.Kx, (const T*)d.hprev, d.ldh, Hh, Bp, bt0,
                                    nbt, red);
  }
  for (int t = w; t < RT * BT; t += KS) {
    const int rt = t / BT, bt = t - rt * BT;
    if (bt >= nbt) continue;
    const v4f pre = step_tile_sum<RT, KS, BT>(red, rt, bt);
    const int u = u0 + 4 * rt + (lane >> 4);
    const int b = 16 * (bt0 + bt) + (lane & 15);
    if (u >= Hh || b >= Bp) continue;
    const float p[4] = {pre[0], pre[1], pre[2], pre[3]};
    if (t == w && have0) cell_finish(d, b, u, Hh, p, in0, sizeof(T) == 2);
    else cell_finish(d, b, u, Hh, p, cell_load(d, b, u, Hh, sizeof(T) == 2), sizeof(T) == 2);
  }
}

template <typename T, int RT, int KS, int U, int BT = STEP_MAXBT>
static void lstm_fwd_go(const LstmFwdArgs& a, int Bp, int Hh, int ndir, hipStream_t st, bool fm = false) {
  const int nbt = (Bp + 15) / 16;
  StepGrid sg{((Hh + 4 * RT - 1) / (4 * RT)) * ndir, 1, (nbt + BT - 1) / BT};
  const LstmFwdDir& d0 = a.d[0];
  const LstmFwdDir& d1 = a.d[ndir > 1 ? 1 : 0];
  const int nlead = (ndir == 2 && d0.Kx == 0 && d1.Kx == 0) ? 2 : 1;
  const int ndir_nlead = ndir | (nlead << 16);
  if constexpr (sizeof(T) == 2) {
    if (fm) {
      hipLaunchKernelGGL((lstm_fwd_kernel<T, RT, KS, U, BT, true>), dim3(step_grid_blocks(sg)), dim3(64 * KS), 0, st, d0.W_fm, d0.x_fm,
                         d0.hprev_fm, d1.W_fm, d1.hprev_fm, d0.Kx, Bp, Hh, ndir_nlead, a);
      return;
    }
  }
  hipLaunchKernelGGL((lstm_fwd_kernel<T, RT, KS, U, BT>), dim3(step_grid_blocks(sg)), dim3(64 * KS), 0, st, d0.W_fm, d0.x_fm, d0.hprev_fm,
                     d1.W_fm, d1.hprev_fm, d0.Kx, Bp, Hh, ndir_nlead, a);
}

// Shapes of the fused kernel: 16 / 32 / 64 gate rows per workgroup, with all sentences (up to 64) or
// 32 of them; fewer, fatter workgroups move less activation traffic through L2.
// `how` (env CMT_LSTM_FWD for experiments): 0 = choose by size, 1 / 2 / 4 = that many 16-row tiles x
// 64 sentences, 6 = 32 rows x 32 sentences.
static int g_lstm_fwd_how = -1;
void launch_lstm_fwd(int prec, const LstmFwdDir* dirs, int ndir, int Bp, int Hh, hipStream_t st) {
  if (g_lstm_fwd_how < 0) {
    const char* e = getenv("CMT_LSTM_FWD");
    g_lstm_fwd_how = e ? atoi(e) : 0;
  }
  LstmFwdArgs a;
  int K = 0;
  for (int i = 0; i < STEP_MAX_INST; ++i) {
    a.d[i] = dirs[i < ndir ? i : 0];
    if (i < ndir && dirs[i].Kx + Hh > K) K = dirs[i].Kx + Hh;      // instances may differ in their input width
  }
  bool fm = prec != 0;                              // fragment-major operands: every instance must bring them
  for (int i = 0; i < ndir; ++i) fm = fm && dirs[i].W_fm != nullptr;
  int how = g_lstm_fwd_how;
  const int nbt = (Bp + 15) / 16;
  // measured (bf16, hidden 1024): 64 sentences — 32 gate rows x 32 sentences per workgroup: 9.9 us against
  // 11.3 us for 16 rows x 64 sentences; more than 64 sentences — 32 rows x 64 sentences
  // (32 sentences: 16 rows x 32 sentences is faster; 640 sentences, as in beam search: 64 rows x 64 sentences,
  // 65 us against 80 us; 128 sentences: 32 rows, 14.7 us against 19.7 us)
  if (how == 0) how = (Bp >= 256) ? 4 : (Bp > 64) ? 2 : (prec && nbt == 4) ? 6 : 1;
  const int nsteps = (K / 8 + 3) / 4;
  if (prec) {
    if (how == 6) {
      if (nsteps > 32) lstm_fwd_go<bf16_t, 2, 8, 4, 2>(a, Bp, Hh, ndir, st, fm);
      else if (nsteps > 16) lstm_fwd_go<bf16_t, 2, 8, 2, 2>(a, Bp, Hh, ndir, st, fm);
      else lstm_fwd_go<bf16_t, 2, 4, 2, 2>(a, Bp, Hh, ndir, st, fm);
    }
    else if (how == 4) lstm_fwd_go<bf16_t, 4, 8, 4>(a, Bp, Hh, ndir, st, fm);
    else if (how == 2) lstm_fwd_go<bf16_t, 2, 8, 4>(a, Bp, Hh, ndir, st, fm);
    else if (nsteps > 32) lstm_fwd_go<bf16_t, 1, 16, 4>(a, Bp, Hh, ndir, st, fm);
    else if (nsteps > 16) lstm_fwd_go<bf16_t, 1, 16, 2>(a, Bp, Hh, ndir, st, fm);
    else if (nsteps > 8) lstm_fwd_go<bf16_t, 1, 8, 2>(a, Bp, Hh, ndir, st, fm);
    else lstm_fwd_go<bf16_t, 1, 4, 2>(a, Bp, Hh, ndir, st, fm);
  } else {
    if (how == 4) lstm_fwd_go<float, 4, 8, 2>(a, Bp, Hh, ndir, st);
    else if (how == 2) lstm_fwd_go<float, 2, 8, 2>(a, Bp, Hh, ndir, st);
    else if (nsteps > 16) lstm_fwd_go<float, 1, 16, 2>(a, Bp, Hh, ndir, st);
    else if (nsteps > 8) lstm_fwd_go<float, 1, 8, 2>(a, Bp, Hh, ndir, st);
    else lstm_fwd_go<float, 1, 4, 2>(a, Bp, Hh, ndir, st);
  }
}

// ------------------------------------------------------------------------------------------------
// generic step GEMM, 2-D decomposition: a workgroup owns 64 weight rows x all (<= 64) sentences x a
// k block.  Its 4 wavefronts split the k-steps; each loads every operand element it needs exactly
// once (4 weight + 4 activation fragments per k-step feed 16 MFMAs), so the bytes that cross L2
// are rows/64 * B * K for the activations instead of rows/16 * B * K.  The k blocks write planes
// out[kb][b][n] that the consumer sums.
// ------------------------------------------------------------------------------------------------
struct Step2dPlan { int kb, steps_per_block, u; };
static Step2dPlan plan2d(int prec, int N, int K, int Bp, int max_kb) {
  const int nsteps = (K / 8 + 3) / 4;
  const int nrb = (N + 63) / 64, nz = ((Bp + 15) / 16 + STEP_MAXBT - 1) / STEP_MAXBT;
  const int u = prec ? 4 : 2;
  int kb = (256 + nrb * nz - 1) / (nrb * nz);          // enough workgroups for 256 CUs
  const int kb_max = (nsteps + 3) / 4;                  // at least one k-step per wavefront
  if (kb > kb_max) kb = kb_max;
  if (kb > 8) kb = 8;
  if (max_kb > 0 && kb > max_kb) kb = max_kb;
  if (kb < 1) kb = 1;
  int spb = (nsteps + kb - 1) / kb;
  spb = (spb + 3) / 4 * 4;
  kb = (nsteps + spb - 1) / spb;
  Step2dPlan p{kb, spb, u};
  if (spb <= 4) p.u = 1;
  else if (spb <= 8 && p.u > 2) p.u = 2;
  return p;
}
int step_kblocks(int prec, int N, int K, int Bp, int max_kb) { return plan2d(prec, N, K, Bp, max_kb).kb; }

template <typename T, int U, bool FM = false>
__global__ __launch_bounds__(256) void step2d_kernel(StepGemmArgs args, int Bp, StepGrid sg, int spb) {
  __shared__ __align__(16) float red[4 * 16 * 64 * 4];
  StepGemm g = args.g[blockIdx.y];
  int x, kb, z;
  if (!decode_block(sg, x, kb, z)) return;
  if (x * 64 >= g.N) return;                       // instances of one launch may differ in N
  // what the epilogue needs is fetched now, not behind the barrier
  CMT_PIN_UNIFORM_PTR(g.bias); CMT_PIN_UNIFORM_PTR(g.best_idx);
  CMT_PIN_UNIFORM(g.N); CMT_PIN_UNIFORM(g.mode); CMT_PIN_UNIFORM_PTR(g.out); CMT_PIN_UNIFORM(g.ldout); CMT_PIN_UNIFORM(g.plane_stride);
  CMT_PIN_UNIFORM_PTR(g.outT); CMT_PIN_UNIFORM(g.ldo); CMT_PIN_UNIFORM_PTR(g.outD); CMT_PIN_UNIFORM(g.ldod); CMT_PIN_UNIFORM(g.drop.on);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int n0 = x * 64;
  const int bt0 = z * STEP_MAXBT;
  const int nbt = min(STEP_MAXBT, (Bp + 15) / 16 - bt0);
  const T* wrow[4];
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
    wrow[rt] = (const T*)g.W + (size_t)min(n0 + 16 * rt + (lane & 15), g.N - 1) * g.ldw;
  const int nc0 = g.K0 >> 3, nc = (g.K0 + g.K1) >> 3;
  const int brow = 16 * bt0 + (lane & 15);
  const T* a0 = (const T*)g.a0; const T* a1 = (const T*)g.a1;
  v4f acc[4][STEP_MAXBT];
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int b = 0; b < STEP_MAXBT; ++b) acc[rt][b] = v4f{0.f, 0.f, 0.f, 0.f};
  const int s_begin = kb * spb, s_end = s_begin + spb;
  if constexpr (FM) {
    const int ns0 = g.K0 >> 5, ns1 = g.K1 >> 5, ntile = g.N >> 4;
    const bf16_t* wt[4];
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)   // row tiles past N read the last one (their results are dropped)
      wt[rt] = (const bf16_t*)g.W_fm + (size_t)(g.w_tile0 + min((n0 >> 4) + rt, ntile - 1)) * (ns0 + ns1) * 512;
    step_contract_fm<4, 4, U, STEP_MAXBT>(wt, (const bf16_t*)g.a0_fm, ns0, (const bf16_t*)g.a1_fm, ns1, bt0, nbt, red, s_begin, s_end);
  } else {
  for (int s0 = s_begin; s0 < s_end; s0 += 4 * U) {
    Frag<T> fw[U][4], fx[U][STEP_MAXBT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int s = s0 + w + 4 * u;
      const int chunk = 4 * s + (lane >> 4);
      if (s < s_end && chunk < nc) {
        const bool first = chunk < nc0;
        const int kk = first ? chunk * 8 : (chunk - nc0) * 8;
        const int wo = (first ? g.w0_off : g.w1_off) + kk;
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) fw[u][rt].load(wrow[rt] + wo);
        const T* a = first ? a0 : a1;
        const int lda = first ? g.lda0 : g.lda1;
#pragma unroll
        for (int b = 0; b < STEP_MAXBT; ++b) {
          if (b < nbt) fx[u][b].load(a + (size_t)min(brow + 16 * b, Bp - 1) * lda + kk);
          else fx[u][b].zero();
        }
      } else {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) fw[u][rt].zero();
#pragma unroll
        for (int b = 0; b < STEP_MAXBT; ++b) fx[u][b].zero();
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int rt = 0; rt < 4; ++rt)
#pragma unroll
        for (int b = 0; b < STEP_MAXBT; ++b) mma16(acc[rt][b], fw[u][rt], fx[u][b]);
  }
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int b = 0; b < STEP_MAXBT; ++b)
      *reinterpret_cast<v4f*>(red + (((w * 4 + rt) * STEP_MAXBT + b) * 64 + lane) * 4) = acc[rt][b];
  __syncthreads();
  }
  // wavefront w finishes row tile w for all batch tiles
  const int n = n0 + 16 * w + 4 * (lane >> 4);
  if (g.mode == 2) {
    // arg-max over this workgroup's 64 columns per sentence: a lane's 4 columns, then the 4 lane groups of the
    // wavefront's row tile, then the 4 wavefronts through LDS ((value, column) order: larger value, lower column)
    __shared__ float sbv[4][16 * STEP_MAXBT];
    __shared__ int sbi[4][16 * STEP_MAXBT];
#pragma unroll
    for (int bt = 0; bt < STEP_MAXBT; ++bt) {
      float bv = -INFINITY; int bi = 0x7fffffff;
      if (bt < nbt) {
        v4f r = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < 4; ++k) r += *reinterpret_cast<const v4f*>(red + (((k * 4 + w) * STEP_MAXBT + bt) * 64 + lane) * 4);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (n + i < g.N) {
            const float v = r[i] + g.bias[n + i];
            if (v > bv) { bv = v; bi = n + i; }              // ascending columns: the first of equal values stays
          }
      }
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
      }
      if (lane < 16) { sbv[w][16 * bt + lane] = bv; sbi[w][16 * bt + lane] = bi; }
    }
    __syncthreads();
    const int t = threadIdx.x;
    if (t < 16 * STEP_MAXBT) {
      const int b = 16 * bt0 + t;
      float bv = sbv[0][t]; int bi = sbi[0][t];
#pragma unroll
      for (int k = 1; k < 4; ++k)
        if (sbv[k][t] > bv || (sbv[k][t] == bv && sbi[k][t] < bi)) { bv = sbv[k][t]; bi = sbi[k][t]; }
      if (b < Bp) { g.out[(size_t)x * Bp + b] = bv; g.best_idx[(size_t)x * Bp + b] = bi; }
    }
    return;
  }
#pragma unroll
  for (int bt = 0; bt < STEP_MAXBT; ++bt) {
    if (bt >= nbt) break;
    const int b = 16 * (bt0 + bt) + (lane & 15);
    v4f r = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 4; ++k) r += *reinterpret_cast<const v4f*>(red + (((k * 4 + w) * STEP_MAXBT + bt) * 64 + lane) * 4);
    if (b >= Bp || n >= g.N) continue;
    if (g.mode == 0 && sg.kb == 1) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (n + i < g.N) {
          const float hv = tanh_of<sizeof(T) == 2>(r[i]);
          ((T*)g.outT)[(size_t)b * g.ldo + n + i] = from_f<T>(hv);
          if (g.outD) ((T*)g.outD)[(size_t)b * g.ldod + n + i] = from_f<T>(hv * drop_factor(g.drop, b, n + i));
        }
    } else {
      float* o = g.out + (size_t)kb * g.plane_stride + (size_t)b * g.ldout + n;
      if (n + 3 < g.N && (g.ldout & 3) == 0) *reinterpret_cast<v4f*>(o) = r;
      else
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (n + i < g.N) o[i] = r[i];
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void tanh_planes_kernel(Planes p, T* __restrict__ out, int ldo, T* __restrict__ outD, int ldod,
                                                          DropSpec drop, int Bp, int N);

// mode 0 in one launch: 16 weight rows x 16 sentences per workgroup with the whole k range inside it
// (split over its wavefronts, combined through LDS), tanh and the optional dropped copy in the
// epilogue.  No planes, no second kernel; each weight slab is read by the batch's 16-sentence groups
// from the same L2.
template <typename T, int KS, int U, bool FM, bool RAW>
__device__ __forceinline__ void step_tanh_body(StepGemm& g, int Bp, const StepGrid& sg, float* red) {
  int x, kb, z;
  if (!decode_block(sg, x, kb, z)) return;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int n0 = x * 16;
  // what the epilogue needs is fetched now, not behind the barrier
  if constexpr (RAW) {
    CMT_PIN_UNIFORM_PTR(g.out); CMT_PIN_UNIFORM(g.ldout); CMT_PIN_UNIFORM(g.N);
  } else {
    CMT_PIN_UNIFORM_PTR(g.outT); CMT_PIN_UNIFORM(g.ldo); CMT_PIN_UNIFORM_PTR(g.outD); CMT_PIN_UNIFORM(g.ldod); CMT_PIN_UNIFORM_PTR(g.outF);
    CMT_PIN_UNIFORM_PTR(g.outF2); CMT_PIN_UNIFORM(g.outF2_nsteps); CMT_PIN_UNIFORM(g.outF2_k0); CMT_PIN_UNIFORM(g.N);
    CMT_PIN_UNIFORM(g.drop.on);
  }
  const bool skip0 = RAW && g.skip0;                 // (mode 3 only) segment 1 alone
  const T* wrow[1] = {(const T*)g.W + (size_t)min(n0 + (lane & 15), g.N - 1) * g.ldw};
  if constexpr (FM) {
    const int ns0 = g.K0 >> 5, ns1 = g.K1 >> 5;
    const bf16_t* wt[1] = {(const bf16_t*)g.W_fm + (size_t)(g.w_tile0 + x) * (ns0 + ns1) * 512};
    step_contract_fm<1, KS, U, 1>(wt, (const bf16_t*)g.a0_fm, ns0, (const bf16_t*)g.a1_fm, ns1, z, 1, red, skip0 ? ns0 : 0);
  } else {
    step_contract<T, 1, KS, U, 1>(wrow, g.w0_off, g.w1_off, (const T*)g.a0, g.lda0, skip0 ? 0 : g.K0, (const T*)g.a1, g.lda1, g.K1, Bp,
                                  z, 1, red);
  }
  if (w != 0) return;
  const v4f r = step_tile_sum<1, KS, 1>(red, 0, 0);
  const int n = n0 + 4 * (lane >> 4), b = 16 * z + (lane & 15);
  if (b >= Bp) return;
  if constexpr (RAW) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (n + i < g.N) g.out[(size_t)b * g.ldout + n + i] = r[i];
    return;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (n + i < g.N) {
      const float hv = tanh_of<sizeof(T) == 2>(r[i]);
      const float hd = g.outD ? hv * drop_factor(g.drop, b, n + i) : hv;
      ((T*)g.outT)[(size_t)b * g.ldo + n + i] = from_f<T>(hv);
      if (g.outD) ((T*)g.outD)[(size_t)b * g.ldod + n + i] = from_f<T>(hd);
      if (sizeof(T) == 2 && g.outF) ((T*)g.outF)[fm_offset(b, n + i, g.N >> 5)] = from_f<T>(hd);
      if (sizeof(T) == 2 && g.outF2) ((T*)g.outF2)[fm_offset(b, g.outF2_k0 + n + i, g.outF2_nsteps)] = from_f<T>(hd);
    }
}
template <typename T, int KS, int U, bool FM = false>
__global__ __launch_bounds__(64 * KS) void step_tanh_kernel(StepGemm g, int Bp, StepGrid sg) {
  __shared__ __align__(16) float red[KS * 256];
  step_tanh_body<T, KS, U, FM, false>(g, Bp, sg, red);
}

static bool step_gemm_has_fm(const StepGemm& g) {
  return g.W_fm && (g.K0 == 0 || g.a0_fm) && (g.K1 == 0 || g.a1_fm) && g.K0 % 32 == 0 && g.K1 % 32 == 0 && g.N % 16 == 0;
}

// n instances in one launch (blockIdx.y); they share the contraction length and the k-block plan,
// which is the plan of the widest instance.
void launch_step_gemm_multi(int prec, const StepGemm* gs, int n, int n_plan, int Bp, hipStream_t st) {
  const int nbt = (Bp + 15) / 16;
  StepGemmArgs a;
  int Nmax = 0;
  for (int i = 0; i < STEP_MAX_INST; ++i) {
    a.g[i] = gs[i < n ? i : 0];
    if (i < n && gs[i].N > Nmax) Nmax = gs[i].N;
  }
  if (n_plan > Nmax) Nmax = n_plan;
  const StepGemm& g = gs[0];
  const Step2dPlan pl = plan2d(prec, Nmax, g.K0 + g.K1, Bp, g.max_kb);
  StepGrid sg{(Nmax + 63) / 64, pl.kb, (nbt + STEP_MAXBT - 1) / STEP_MAXBT};
  const dim3 grid(step_grid_blocks(sg), n);
  bool fm = prec != 0;                              // fragment-major operands: every instance must bring them
  for (int i = 0; i < n; ++i) fm = fm && step_gemm_has_fm(gs[i]);
#define GO(TT, UU) hipLaunchKernelGGL((step2d_kernel<TT, UU>), grid, dim3(256), 0, st, a, Bp, sg, pl.steps_per_block)
#define GOF(UU) hipLaunchKernelGGL((step2d_kernel<bf16_t, UU, true>), grid, dim3(256), 0, st, a, Bp, sg, pl.steps_per_block)
  if (fm) { if (pl.u == 4) GOF(4); else if (pl.u == 2) GOF(2); else GOF(1); }
  else if (prec) { if (pl.u == 4) GO(bf16_t, 4); else if (pl.u == 2) GO(bf16_t, 2); else GO(bf16_t, 1); }
  else { if (pl.u == 2) GO(float, 2); else GO(float, 1); }
#undef GO
#undef GOF
}

static int g_step_tanh = -1;
void launch_step_gemm(int prec, const StepGemm& g, int Bp, hipStream_t st) {
  const int nbt = (Bp + 15) / 16;
  if (g_step_tanh < 0) {
    const char* e = getenv("CMT_STEP_TANH");
    g_step_tanh = e ? atoi(e) : 1;
  }
  if (g.mode == 0 && g_step_tanh && Bp < 256) {       // (from 256 sentences on its 16-sentence tiles re-read W too often)
    StepGrid sg{(g.N + 15) / 16, 1, nbt};
    const dim3 grid(step_grid_blocks(sg));
    const int nsteps = ((g.K0 + g.K1) / 8 + 3) / 4;
#define GO(TT, KS, UU) hipLaunchKernelGGL((step_tanh_kernel<TT, KS, UU>), grid, dim3(64 * KS), 0, st, g, Bp, sg)
#define GOF(KS, UU) hipLaunchKernelGGL((step_tanh_kernel<bf16_t, KS, UU, true>), grid, dim3(64 * KS), 0, st, g, Bp, sg)
    if (prec && step_gemm_has_fm(g)) { if (nsteps > 32) GOF(16, 4); else if (nsteps > 16) GOF(16, 2); else GOF(8, 2); }
    else if (prec) { if (nsteps > 32) GO(bf16_t, 16, 4); else if (nsteps > 16) GO(bf16_t, 16, 2); else GO(bf16_t, 8, 2); }
    else { if (nsteps > 16) GO(float, 16, 2); else GO(float, 8, 2); }
#undef GO
#undef GOF
    return;
  }
  // the other forms do not write the fragment-major copy themselves
  const bool pack_after = g.mode == 0 && prec && (g.outF || g.outF2);
  const Step2dPlan pl = plan2d(prec, g.N, g.K0 + g.K1, Bp, g.max_kb);
  StepGrid sg{(g.N + 63) / 64, pl.kb, (nbt + STEP_MAXBT - 1) / STEP_MAXBT};
  const dim3 grid(step_grid_blocks(sg));
  StepGemmArgs a;
  for (int i = 0; i < STEP_MAX_INST; ++i) a.g[i] = g;
#define GO(TT, UU) hipLaunchKernelGGL((step2d_kernel<TT, UU>), grid, dim3(256), 0, st, a, Bp, sg, pl.steps_per_block)
#define GOF(UU) hipLaunchKernelGGL((step2d_kernel<bf16_t, UU, true>), grid, dim3(256), 0, st, a, Bp, sg, pl.steps_per_block)
  if (prec && step_gemm_has_fm(g)) { if (pl.u == 4) GOF(4); else if (pl.u == 2) GOF(2); else GOF(1); }
  else if (prec) { if (pl.u == 4) GO(bf16_t, 4); else if (pl.u == 2) GO(bf16_t, 2); else GO(bf16_t, 1); }
  else { if (pl.u == 2) GO(float, 2); else GO(float, 1); }
#undef GO
#undef GOF
  if (g.mode == 0 && pl.kb > 1) {
    Planes p{g.out, g.ldout, pl.kb, g.plane_stride};
    const int n = Bp * (g.N >> 2);
    if (prec) hipLaunchKernelGGL(tanh_planes_kernel<bf16_t>, dim3((n + 255) / 256), dim3(256), 0, st, p, (bf16_t*)g.outT, g.ldo,
                                 (bf16_t*)g.outD, g.ldod, g.drop, Bp, g.N);
    else hipLaunchKernelGGL(tanh_planes_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, st, p, (float*)g.outT, g.ldo,
                            (float*)g.outD, g.ldod, g.drop, Bp, g.N);
  }
  if (pack_after && g.outF) launch_fm_pack(g.outD ? g.outD : g.outT, g.outD ? g.ldod : g.ldo, Bp, g.N, g.outF, st);
  if (pack_after && g.outF2)
    launch_fm_pack(g.outD ? g.outD : g.outT, g.outD ? g.ldod : g.ldo, Bp, g.N, g.outF2, st, g.outF2_nsteps, g.outF2_k0 >> 5);
}

// ------------------------------------------------------------------------------------------------
// LSTM cell backward (pointwise), one thread per (sentence, unit)
// ------------------------------------------------------------------------------------------------
// sum of the planes for 4 consecutive columns (c, ld and stride are multiples of 4); the loads of
// all planes (at most 8) are independent and issued together
__device__ __forceinline__ float4 planes_get4(const Planes& p, int b, int c) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  const float* base = p.p + (size_t)b * p.ld + c;
  float4 t[8];
#pragma unroll
  for (int k = 0; k < 8; ++k)
    t[k] = k < p.np ? *reinterpret_cast<const float4*>(base + (size_t)k * p.stride) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int k = 0; k < 8; ++k) { v.x += t[k].x; v.y += t[k].y; v.z += t[k].z; v.w += t[k].w; }
  for (int k = 8; k < p.np; ++k) {
    const float4 q = *reinterpret_cast<const float4*>(base + (size_t)k * p.stride);
    v.x += q.x; v.y += q.y; v.z += q.z; v.w += q.w;
  }
  return v;
}
template <typename T> __device__ __forceinline__ void store4(T* p, const float (&v)[4]);
template <> __device__ __forceinline__ void store4<float>(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t* p, const float (&v)[4]) {
  uint2 o;
  o.x = (uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16);
  o.y = (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16);
  *reinterpret_cast<uint2*>(p) = o;
}

// Cell backward of 4 consecutive units u..u+3 of sentence b.  The gradient arriving at the step's output is
// dy = p.dy planes + dy_x, the recurrent part of the state gradient is p.dhrec planes + rec_x (the _x parts are
// what a fused caller holds in registers); everything else comes from p.
struct CellBwdIn { float4 i, f, g, o, cp, cn, dc, dhp, dy, rec; float mask; };
__device__ __forceinline__ CellBwdIn cell_bwd_load(const LstmBwdPoint& p, int b, int u, int Hh) {
  CellBwdIn in;
  const size_t idx = (size_t)b * Hh + u;
  in.mask = p.mask[b];
  in.rec = planes_get4(p.dhrec, b, p.dhrec_col + u);
  in.dhp = *reinterpret_cast<const float4*>(p.dh + idx);
  in.dy = planes_get4(p.dy, b, p.dy_col + u);
  in.dc = *reinterpret_cast<const float4*>(p.dc + idx);
  const float* gs = p.gsave + (size_t)b * 4 * Hh + u;
  in.i = *reinterpret_cast<const float4*>(gs); in.f = *reinterpret_cast<const float4*>(gs + Hh);
  in.g = *reinterpret_cast<const float4*>(gs + 2 * Hh); in.o = *reinterpret_cast<const float4*>(gs + 3 * Hh);
  in.cp = *reinterpret_cast<const float4*>(p.cprev + idx); in.cn = *reinterpret_cast<const float4*>(p.cnext + idx);
  return in;
}
template <typename T>
__device__ __forceinline__ void cell_bwd_finish(const LstmBwdPoint& p, int b, int u, int Hh, const CellBwdIn& in, const float (&dy_x)[4],
                                                const float (&rec_x)[4]) {
  const size_t idx = (size_t)b * Hh + u;
  const float dh_state[4] = {in.dhp.x + (in.rec.x + rec_x[0]), in.dhp.y + (in.rec.y + rec_x[1]), in.dhp.z + (in.rec.z + rec_x[2]),
                             in.dhp.w + (in.rec.w + rec_x[3])};
  T* dg = (T*)p.dg + (size_t)b * p.lddg + u;
  const float zero[4] = {0.f, 0.f, 0.f, 0.f};
  // the same four values per gate go to the fragment-major copy (u % 4 == 0: four consecutive elements there too)
  const bool fm_copy = sizeof(T) == 2 && p.dg_fm != nullptr;
  T* const dgf = (T*)p.dg_fm;
  size_t fo[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) fo[g] = fm_offset(b, g * Hh + u, (4 * Hh) >> 5);
  if (!(in.mask > 0.f)) {                          // masked step: state passes through, no gate gradient
#pragma unroll
    for (int g = 0; g < 4; ++g) { store4<T>(dg + g * Hh, zero); if (fm_copy) store4<T>(dgf + fo[g], zero); }
    store4<float>(p.dh + idx, dh_state);           // (an output of a masked step is the constant 0: dy is dropped)
    return;
  }
  float di[4], df[4], dgg[4], dout[4], dcn[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float ig = (&in.i.x)[e], fg = (&in.f.x)[e], gg = (&in.g.x)[e], og = (&in.o.x)[e];
    const float cp = (&in.cp.x)[e], cn = (&in.cn.x)[e];
    const float tc = tanh_of<sizeof(T) == 2>(cn);
    const float dh = dh_state[e] + ((&in.dy.x)[e] + dy_x[e]) * drop_factor(p.drop_dy, b, p.dy_col + u + e);
    const float dog = dh * tc;
    const float dc = (&in.dc.x)[e] + dh * og * (1.f - tc * tc);
    di[e] = dc * gg * ig * (1.f - ig);
    df[e] = dc * cp * fg * (1.f - fg);
    dgg[e] = dc * ig * (1.f - gg * gg);
    dout[e] = dog * og * (1.f - og);
    dcn[e] = dc * fg;
  }
  store4<T>(dg, di); store4<T>(dg + Hh, df); store4<T>(dg + 2 * Hh, dgg); store4<T>(dg + 3 * Hh, dout);
  if (fm_copy) { store4<T>(dgf + fo[0], di); store4<T>(dgf + fo[1], df); store4<T>(dgf + fo[2], dgg); store4<T>(dgf + fo[3], dout); }
  store4<float>(p.dc + idx, dcn);
  store4<float>(p.dh + idx, zero);                 // the recurrent part arrives with the next step's GEMM
}

// one thread per (sentence, 4 consecutive units); single-wavefront workgroups, so that the 16 K threads
// of a 64-sentence x 1024-unit step spread over all CUs
constexpr int LSTM_BWD_POINT_THREADS = 64;
template <typename T>
__global__ __launch_bounds__(LSTM_BWD_POINT_THREADS) void lstm_bwd_point_kernel(LstmBwdPointArgs args, int Bp, int Hh) {
  const LstmBwdPoint& p = args.p[blockIdx.y];
  const int idx4 = blockIdx.x * LSTM_BWD_POINT_THREADS + threadIdx.x;
  const int hq = Hh >> 2;
  if (idx4 >= Bp * hq) return;
  int b, u;
  divmod_uniform(idx4, hq, b, u);
  u *= 4;
  const float zero[4] = {0.f, 0.f, 0.f, 0.f};
  cell_bwd_finish<T>(p, b, u, Hh, cell_bwd_load(p, b, u, Hh), zero, zero);
}

void launch_lstm_bwd_point_multi(int prec, const LstmBwdPoint* ps, int n, int Bp, int Hh, hipStream_t st) {
  LstmBwdPointArgs a;
  for (int i = 0; i < STEP_MAX_INST; ++i) a.p[i] = ps[i < n ? i : 0];
  const int cnt = Bp * (Hh >> 2);
  const dim3 grid((cnt + LSTM_BWD_POINT_THREADS - 1) / LSTM_BWD_POINT_THREADS, n);
  if (prec) hipLaunchKernelGGL(lstm_bwd_point_kernel<bf16_t>, grid, dim3(LSTM_BWD_POINT_THREADS), 0, st, a, Bp, Hh);
  else hipLaunchKernelGGL(lstm_bwd_point_kernel<float>, grid, dim3(LSTM_BWD_POINT_THREADS), 0, st, a, Bp, Hh);
}
void launch_lstm_bwd_point(int prec, const LstmBwdPoint& p, int Bp, int Hh, hipStream_t st) {
  launch_lstm_bwd_point_multi(prec, &p, 1, Bp, Hh, st);
}

// ------------------------------------------------------------------------------------------------
// backward step GEMM, whole k range per workgroup, consumer fused into the epilogue
// ------------------------------------------------------------------------------------------------
// A workgroup owns 16 output columns x BT tiles of 16 sentences; its wavefronts split the k range and
// meet in LDS as in the forward kernel.  After the reduction a lane holds 4 consecutive output columns
// of one sentence — for the cell backward that is 4 consecutive hidden units, the same unit of work a
// thread of the pointwise kernel has — so the consumer runs in registers and neither the planes nor a
// second launch exist.  The epilogue's operands are fetched before the contraction starts.
struct StepBwdArgs { StepBwd g[STEP_BWD_MAX_INST]; };

// What the fragment-major contraction of an instance needs before its first load, as leading kernel arguments
// (they arrive in registers): the operands, the contraction length and the column counts.  `on` = 0: read the
// instance's own fields instead (further instances of a launch).
struct StepBwdLead { const void* Wt_fm; const void* dg_fm; int K, wt_tile0, N, ncols0, on; };   // (on: see step_bwd_fused_kernel)
template <typename T, int KS, int U, int BT, bool FM>
__device__ __forceinline__ void step_bwd_body(const StepBwdLead& ld, const StepBwd& g, int Bp, const StepGrid& sg, float* red) {
  int x, kb, z;
  if (!decode_block(sg, x, kb, z)) return;
  const int ncols0 = ld.on ? ld.ncols0 : g.part[0].ncols;
  const int N = ld.on ? ld.N : g.part[0].ncols + g.part[1].ncols;
  const int n0 = x * 16;
  if (n0 >= N) return;                              // instances of one launch may differ in N
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int which = n0 >= ncols0 ? 1 : 0;
  const int c0 = n0 - (which ? ncols0 : 0);
  const int bt0 = z * BT;
  const int nbt = min(BT, (Bp + 15) / 16 - bt0);
  // the tile this wavefront will finish
  const int c = c0 + 4 * (lane >> 4);
  const int b = 16 * (bt0 + w) + (lane & 15);
  BwdEpi e;
  bool mine = false;
  CellBwdIn cin;
  float4 tce = make_float4(0.f, 0.f, 0.f, 0.f);
  float tho[4] = {0.f, 0.f, 0.f, 0.f};
  // the epilogue's description and operands: fetched now, not behind the barrier — and, where the contraction's
  // operands came in registers, behind its first round of loads (the opaque index keeps the compiler from moving
  // this block, which depends on nothing before it, back in front of them)
  auto fetch_rest = [&]() {
    int wsel = __builtin_amdgcn_readfirstlane(which);
    asm volatile("" : "+s"(wsel) : : "memory");
    e = g.part[wsel];
    CMT_PIN_UNIFORM(e.kind); CMT_PIN_UNIFORM(e.ncols); CMT_PIN_UNIFORM(e.hh); CMT_PIN_UNIFORM_PTR(e.out); CMT_PIN_UNIFORM(e.ldout);
    CMT_PIN_UNIFORM_PTR(e.dpre); CMT_PIN_UNIFORM(e.ldp); CMT_PIN_UNIFORM_PTR(e.dpre_fm); CMT_PIN_UNIFORM(e.drop.on);
    CMT_PIN_UNIFORM_PTR(e.cell.dg); CMT_PIN_UNIFORM(e.cell.lddg); CMT_PIN_UNIFORM_PTR(e.cell.dg_fm); CMT_PIN_UNIFORM_PTR(e.cell.dc);
    CMT_PIN_UNIFORM_PTR(e.cell.dh); CMT_PIN_UNIFORM(e.cell.drop_dy.on); CMT_PIN_UNIFORM(e.cell.dy_col);
    mine = w < nbt && b < Bp && c < e.ncols;
    if (mine) {
      if (e.kind == BWD_EPI_CELL_DY || e.kind == BWD_EPI_CELL_REC) cin = cell_bwd_load(e.cell, b, c, e.hh);
      else if (e.kind == BWD_EPI_TANH) {
        const int r = e.pos ? e.pos[b] : b;
        if (r >= 0) tce = *reinterpret_cast<const float4*>(e.dce + (size_t)r * e.hh + c);
#pragma unroll
        for (int i = 0; i < 4; ++i) tho[i] = to_f<T>(((const T*)e.Ho)[(size_t)b * e.ldho + c + i]);
      }
    }
  };
  if constexpr (FM) {
    const int ns = (ld.on ? ld.K : g.K) >> 5;
    const bf16_t* Wf = (const bf16_t*)(ld.on ? ld.Wt_fm : g.Wt_fm);
    const bf16_t* wt[1] = {Wf + (size_t)((ld.on ? ld.wt_tile0 : g.wt_tile0) + x) * ns * 512};
    step_contract_fm<1, KS, U, BT, decltype(fetch_rest), KS == 16>(wt, (const bf16_t*)(ld.on ? ld.dg_fm : g.dg_fm), ns, nullptr, 0, bt0, nbt,
                                                                   red, 0, 1 << 30, fetch_rest);
  } else {
    fetch_rest();
    const T* wrow[1] = {(const T*)g.Wt + (size_t)min(n0 + (lane & 15), N - 1) * g.ldw};
    step_contract<T, 1, KS, U, BT>(wrow, 0, 0, (const T*)g.dg, g.lddg, g.K, (const T*)nullptr, 0, 0, Bp, bt0, nbt, red);
  }
  if (!mine) return;                                // KS >= BT: wavefront w finishes sentence tile w
  const v4f r = step_tile_sum<1, KS, BT>(red, 0, w);
  const float v[4] = {r[0], r[1], r[2], r[3]};
  const float zero[4] = {0.f, 0.f, 0.f, 0.f};
  if (e.kind == BWD_EPI_STORE) {
    store4<float>(e.out + (size_t)b * e.ldout + c, v);
  } else if (e.kind == BWD_EPI_CELL_DY) {
    cell_bwd_finish<T>(e.cell, b, c, e.hh, cin, v, zero);
  } else if (e.kind == BWD_EPI_CELL_REC) {
    cell_bwd_finish<T>(e.cell, b, c, e.hh, cin, zero, v);
  } else {
    float o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = ((&tce.x)[i] + v[i]) * drop_factor(e.drop, b, c + i) * (1.f - tho[i] * tho[i]);
    store4<T>((T*)e.dpre + (size_t)b * e.ldp + c, o);
    if (sizeof(T) == 2 && e.dpre_fm) store4<T>((T*)e.dpre_fm + fm_offset(b, c, e.hh >> 5), o);
  }
}
// The leading arguments describe instance 0 and, with nlead = 2, instance 1 (same shape, its own operands: the
// bottom encoder layer's two directions).  nx = the launch's column tiles (of its widest instance).
template <typename T, int KS, int U, int BT, bool FM = false>
__global__ __launch_bounds__(64 * KS) void step_bwd_fused_kernel(const void* Wt_fm0, const void* dg_fm0, const void* Wt_fm1,
                                                                 const void* dg_fm1, int K0, int wt_tile00, int N0, int ncols00, int Bp,
                                                                 int nx_nlead, StepBwdArgs args) {
  __shared__ __align__(16) float red[KS * BT * 256];
  const int nx = nx_nlead & 0xffff, nlead = nx_nlead >> 16;
  const int inst = blockIdx.y;
  const StepBwdLead ld{inst == 1 ? Wt_fm1 : Wt_fm0, inst == 1 ? dg_fm1 : dg_fm0, K0, wt_tile00, N0, ncols00, inst < nlead ? 1 : 0};
  step_bwd_body<T, KS, U, BT, FM>(ld, args.g[inst], Bp, StepGrid{nx, 1, ((Bp + 15) / 16 + BT - 1) / BT}, red);
}
// One instance and, in further workgroups of the same launch, attention scores that depend on the same input
// alone (block n_gemm + ig * Bp + b: positions ig * KS + wavefront of sentence b).
template <typename T, int KS, int U, int BT, bool FM = false>
__global__ __launch_bounds__(64 * KS) void step_bwd_scores_kernel(const void* Wt_fm0, const void* dg_fm0, int K0, int wt_tile00, int N0,
                                                                  int ncols00, int Bp, int nx, int nz, int n_gemm, StepBwd g,
                                                                  AttScores d) {
  __shared__ __align__(16) float red[KS * BT * 256];
  const StepGrid sg{nx, 1, nz};
  if ((int)blockIdx.x >= n_gemm) {
    int ig, b;
    divmod_uniform((int)blockIdx.x - n_gemm, Bp, ig, b);
    const int i = ig * KS + (threadIdx.x >> 6);
    if (d.mat_f32) att_dots_row<float, T>((const float*)d.Mat, d.ldm, (const T*)d.vec, d.ldv, d.len, d.S, Bp, d.H, d.dots, i, b);
    else att_dots_row<T, T>((const T*)d.Mat, d.ldm, (const T*)d.vec, d.ldv, d.len, d.S, Bp, d.H, d.dots, i, b);
    return;
  }
  const StepBwdLead ld{Wt_fm0, dg_fm0, K0, wt_tile00, N0, ncols00, 1};
  step_bwd_body<T, KS, U, BT, FM>(ld, g, Bp, sg, red);
}

template <typename T, int KS, int U, int BT>
static void step_bwd_go(const StepBwdArgs& a, int n, int Nmax, int Bp, hipStream_t st, bool fm, const AttScores* sc) {
  const int nbt = (Bp + 15) / 16;
  StepGrid sg{(Nmax + 15) / 16, 1, (nbt + BT - 1) / BT};
  const StepBwd& g0 = a.g[0];
  const int N0 = g0.part[0].ncols + g0.part[1].ncols;
  if (sc) {                                        // (one instance) the scores ride in the same launch
    const int n_gemm = step_grid_blocks(sg);
    const dim3 grid(n_gemm + ((sc->S + KS - 1) / KS) * Bp);
    if constexpr (sizeof(T) == 2) {
      if (fm) {
        hipLaunchKernelGGL((step_bwd_scores_kernel<T, KS, U, BT, true>), grid, dim3(64 * KS), 0, st, g0.Wt_fm, g0.dg_fm, g0.K, g0.wt_tile0,
                           N0, g0.part[0].ncols, Bp, sg.nx, sg.nz, n_gemm, g0, *sc);
        return;
      }
    }
    hipLaunchKernelGGL((step_bwd_scores_kernel<T, KS, U, BT>), grid, dim3(64 * KS), 0, st, g0.Wt_fm, g0.dg_fm, g0.K, g0.wt_tile0, N0,
                       g0.part[0].ncols, Bp, sg.nx, sg.nz, n_gemm, g0, *sc);
    return;
  }
  const StepBwd& g1 = a.g[n > 1 ? 1 : 0];
  const bool same = n > 1 && g1.K == g0.K && g1.wt_tile0 == g0.wt_tile0 && g1.part[0].ncols == g0.part[0].ncols &&
                    g1.part[1].ncols == g0.part[1].ncols;
  const int nx_nlead = sg.nx | ((same ? 2 : 1) << 16);
  if constexpr (sizeof(T) == 2) {
    if (fm) {
      hipLaunchKernelGGL((step_bwd_fused_kernel<T, KS, U, BT, true>), dim3(step_grid_blocks(sg), n), dim3(64 * KS), 0, st, g0.Wt_fm,
                         g0.dg_fm, g1.Wt_fm, g1.dg_fm, g0.K, g0.wt_tile0, N0, g0.part[0].ncols, Bp, nx_nlead, a);
      return;
    }
  }
  hipLaunchKernelGGL((step_bwd_fused_kernel<T, KS, U, BT>), dim3(step_grid_blocks(sg), n), dim3(64 * KS), 0, st, g0.Wt_fm, g0.dg_fm,
                     g1.Wt_fm, g1.dg_fm, g0.K, g0.wt_tile0, N0, g0.part[0].ncols, Bp, nx_nlead, a);
}

void launch_step_bwd_fused(int prec, const StepBwd* gs, int n, int Bp, hipStream_t st, const AttScores* scores) {
  if (scores && n != 1) scores = nullptr;            // (callers pass one instance with scores)
  for (int base = 0; base < n; base += STEP_BWD_MAX_INST) {
    const int m = n - base < STEP_BWD_MAX_INST ? n - base : STEP_BWD_MAX_INST;
    StepBwdArgs a;
    int Nmax = 0, Kmax = 0;
    bool fm = prec != 0;                           // fragment-major operands: every instance must bring them
    for (int i = 0; i < STEP_BWD_MAX_INST; ++i) {
      a.g[i] = gs[base + (i < m ? i : 0)];
      if (i < m) {
        fm = fm && a.g[i].dg_fm && a.g[i].Wt_fm;
        Nmax = std::max(Nmax, a.g[i].part[0].ncols + a.g[i].part[1].ncols);
        Kmax = std::max(Kmax, a.g[i].K);
      }
    }
    const int nsteps = (Kmax / 8 + 3) / 4;
    const int wgs = ((Nmax + 15) / 16) * (((Bp + 15) / 16 + 1) / 2) * m;
    // 16 columns x 32 sentences per workgroup.  (64 sentences per workgroup halves the number of workgroups
    // and was measured at twice the time: 25.6 against 12.9 us for 64 sentences, 26.2 against 21.8 us for 128.)
#define GO(TT, KS, UU) step_bwd_go<TT, KS, UU, 2>(a, m, Nmax, Bp, st, fm, scores)
    if (prec) {
      // a long k range is split over 16 wavefronts while the launch is one round of workgroups; with more than 256
      // workgroups (128 sentences) 8 wavefronts, so that two workgroups share a CU instead of taking turns
      // (decoder layer at 128 sentences: 12.4 against 14.5 us; at 64 sentences: 10.2 against 9.1 us)
      if (nsteps > 64 && wgs > 256) GO(bf16_t, 8, 2); else
      if (nsteps > 64) GO(bf16_t, 16, 4); else if (nsteps > 32) GO(bf16_t, 8, 4); else if (nsteps > 16) GO(bf16_t, 8, 2); else GO(bf16_t, 4, 2);
    } else {
      if (nsteps > 32) GO(float, 16, 2); else if (nsteps > 16) GO(float, 8, 2); else GO(float, 4, 2);
    }
#undef GO
  }
}

// out[b, c] = base[b, c] + sum of planes (plain fp32 [Bp, cols])
__global__ __launch_bounds__(256) void planes_add_kernel(float* __restrict__ out, const float* __restrict__ base, Planes p,
                                                         int col0, int Bp, int cols) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= Bp * cols) return;
  int b, c;
  divmod_uniform(idx, cols, b, c);
  out[idx] = (base ? base[idx] : 0.f) + planes_get(p, b, col0 + c);
}
void launch_planes_add(float* out, const float* base, const Planes& p, int col0, int Bp, int cols, hipStream_t st) {
  hipLaunchKernelGGL(planes_add_kernel, dim3((Bp * cols + 255) / 256), dim3(256), 0, st, out, base, p, col0, Bp, cols);
}

// ------------------------------------------------------------------------------------------------
// attention: a "dots" kernel (a wavefront per (sentence, source position), or per four of them) and a "mix" kernel
// (softmax or its backward on the dots, then a weighted sum of rows), both spread over the chip
// ------------------------------------------------------------------------------------------------
// dots[b, i] = vec[b, :] . Mat[i, b, :] for i < len[b], vec a T row (forward: H_t); one wavefront per position
template <typename T>
__global__ __launch_bounds__(256) void att_dots_kernel(const T* __restrict__ Mat, int ldm, const T* __restrict__ vec, int ldv,
                                                       const int32_t* __restrict__ len, int S, int Bp, int H, float* __restrict__ dots) {
  att_dots_row<T, T>(Mat, ldm, vec, ldv, len, S, Bp, H, dots, blockIdx.x * 4 + (threadIdx.x >> 6), blockIdx.y);
}

// The scores of a step and, in other workgroups of the same launch, the plain sums of a mode-3 step GEMM (the
// attentional layer's H_t half): both depend on the top layer's new state alone, so neither waits for the other.
// Blocks [0, n_gemm) are the GEMM's; block n_gemm + ig * Bp + b takes positions ig * KS + wavefront of sentence b.
// The leading arguments (they arrive in registers) are all the fragment-major GEMM blocks need: W_fm / a1_fm / K0 /
// K1 / N / out / ldout of `g`, which those blocks then never read.
template <typename T, int KS, int U, bool FM>
__global__ __launch_bounds__(64 * KS) void att_dots_pre_kernel(const void* W_fm0, const void* a1_fm0, float* out0, int K00, int K10, int N0,
                                                               int ldout0, int Bp, int n_gemm, StepGemm g, AttScores d) {
  __shared__ __align__(16) float red[KS * 256];
  const StepGrid sg{(N0 + 15) / 16, 1, (Bp + 15) / 16};
  if constexpr (FM) {
    if ((int)blockIdx.x < n_gemm) {
      StepGemm gl{};
      gl.W_fm = W_fm0; gl.a0_fm = a1_fm0; gl.a1_fm = a1_fm0; gl.K0 = K00; gl.K1 = K10; gl.N = N0; gl.out = out0; gl.ldout = ldout0;
      gl.skip0 = 1; gl.mode = 3;
      step_tanh_body<T, KS, U, true, true>(gl, Bp, sg, red);
      return;
    }
  }
  if ((int)blockIdx.x >= n_gemm) {
    int ig, b;
    divmod_uniform((int)blockIdx.x - n_gemm, Bp, ig, b);
    att_dots_row<T, T>((const T*)d.Mat, d.ldm, (const T*)d.vec, d.ldv, d.len, d.S, Bp, d.H, d.dots, ig * KS + (threadIdx.x >> 6), b);
    return;
  }
  step_tanh_body<T, KS, U, FM, true>(g, Bp, sg, red);
}

// The same with the vector given as the sum of fp32 planes (backward: dC_s from the step GEMM).  The planes are
// summed once per workgroup into LDS and shared by its 4 x PW positions (a wavefront per position would re-read
// all planes for every one of them: 16 x the row it is dotted with); the workgroup of position 0
// also stores the summed vector to vsum[b, :] for the deferred attention gradients.
template <typename T, int PW>                             // PW = positions per wavefront
__global__ __launch_bounds__(256) void att_dots_planes_kernel(const T* __restrict__ Mat, int ldm, Planes vp, float* __restrict__ vsum,
                                                              const int32_t* __restrict__ len, int S, int Bp, int H,
                                                              float* __restrict__ dots) {
  __shared__ __align__(16) float sv[1024];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, b = blockIdx.y;
  const int i0 = blockIdx.x * (4 * PW) + w * PW;
  const int n = min(len[b], S);
  if (blockIdx.x != 0 && blockIdx.x * (4 * PW) >= n) return;   // (uniform over the workgroup)
  float a[PW];
#pragma unroll
  for (int p = 0; p < PW; ++p) a[p] = 0.f;
  for (int c0 = 0; c0 < H; c0 += 1024) {                  // 1024 columns at a time
    const int width = min(1024, H - c0);
    // the rows do not depend on the summed vector: request them first
    Frag<T> f[2][PW];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int p = 0; p < PW; ++p) {
        const int c = 8 * lane + 512 * q;
        if (c < width && i0 + p < n) f[q][p].load(Mat + ((size_t)(i0 + p) * Bp + b) * ldm + c0 + c);
        else f[q][p].zero();
      }
    if (c0) __syncthreads();                              // the previous block's readers are done
    const int col = 4 * threadIdx.x;
    if (col < width) {
      float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int k = 0; k < vp.np; ++k) {
        const float4 x = *reinterpret_cast<const float4*>(vp.p + (size_t)k * vp.stride + (size_t)b * vp.ld + c0 + col);
        sum.x += x.x; sum.y += x.y; sum.z += x.z; sum.w += x.w;
      }
      *reinterpret_cast<float4*>(&sv[col]) = sum;
      if (blockIdx.x == 0) *reinterpret_cast<float4*>(vsum + (size_t)b * H + c0 + col) = sum;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int c = 8 * lane + 512 * q;
      if (c >= width) continue;
      Frag<float> v;
      v.load(&sv[c]);
#pragma unroll
      for (int p = 0; p < PW; ++p)
#pragma unroll
        for (int e = 0; e < 8; ++e) a[p] += f[q][p].get(e) * v.get(e);
    }
  }
#pragma unroll
  for (int p = 0; p < PW; ++p) {
    if (i0 + p >= n) continue;                            // (uniform over the wavefront)
    const float d = wave_sum(a[p]);
    if (lane == 0) dots[(size_t)b * S + i0 + p] = d;
  }
}

constexpr int ATT_MAXS = 512;
struct AttDropped { void* outD; int ldod; DropSpec drop; void* outF2; int outF2_nsteps, outF2_k0; };   // MODE 2: optional copies
// MODE 0 (forward, Eq. 3 and 5): a = softmax(dots) over i < len, written by the h-chunk 0 block;
//                                out = sum_i a_i Mat[i,b,:]  -> T
// MODE 1 (backward): ds = a (dots - sum a dots), written by the h-chunk 0 block;
//                    out = add[b,:] + sum_i ds_i Mat[i,b,:]  -> fp32
// MODE 2 (forward, Eq. 3-7 with Mat = the projected rows W_c1 H_s^i): a as in mode 0;
//                    out = tanh(add[b,:] + sum_i a_i Mat[i,b,:]) -> T, its dropped copy and fragment-major copy
// grid (H / 64 column chunks, Bp); 256 threads = 8 column-octets x 32 position groups
template <typename T, int MODE>
__global__ __launch_bounds__(256) void att_mix_kernel(const T* __restrict__ Mat, int ldm, int ldo, const float* __restrict__ dots,
                                                      const float* __restrict__ a_in, const int32_t* __restrict__ len,
                                                      int S, int Bp, int H, float* __restrict__ coef_out,
                                                      void* __restrict__ out, Planes add, int add_col, LstmBwdPoint cell,
                                                      int fuse_cell, void* __restrict__ out_fm, AttDropped dropped) {
  __shared__ float sc[ATT_MAXS];
  __shared__ float part[32][65];
  const int b = blockIdx.y, t = threadIdx.x;
  const int n = min(len[b], S);
  // MODE 1 with fuse_cell: the result is the gradient at the top decoder layer's output, and the cell
  // backward of that layer's step runs here (lanes 0..15 take 4 consecutive units each) instead of in
  // a launch of its own; its operands are fetched now
  const int u4 = blockIdx.x * 64 + 4 * t;
  const bool do_cell = MODE == 1 && fuse_cell && t < 16 && u4 < H;
  CellBwdIn cin;
  if (do_cell) cin = cell_bwd_load(cell, b, u4, H);
  // the rows of the first 64 positions do not depend on the coefficients: request them (and the term added to the
  // result) now, so that they arrive while wavefront 0 works out the coefficients
  const int oct = t & 7, grp = t >> 3;                       // 8 octets = 64 columns; 32 position groups
  const int h0 = blockIdx.x * 64 + oct * 8;
  Frag<T> pre[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    if (h0 < H && grp + 32 * q < n) pre[q].load(Mat + ((size_t)(grp + 32 * q) * Bp + b) * ldm + h0);
    else pre[q].zero();
  }
  float addv = 0.f;
  if (MODE != 0 && t < 64 && blockIdx.x * 64 + t < H) addv = planes_get(add, b, add_col + blockIdx.x * 64 + t);
  if (t < 64) {
    if (MODE != 1) {
      float mx = -INFINITY;
      for (int i = t; i < n; i += 64) mx = fmaxf(mx, dots[(size_t)b * S + i]);
      mx = wave_max(mx);
      float s = 0.f;
      for (int i = t; i < n; i += 64) { const float e = expf(dots[(size_t)b * S + i] - mx); sc[i] = e; s += e; }
      s = wave_sum(s);
      const float inv = n > 0 ? 1.f / s : 0.f;
      for (int i = t; i < S; i += 64) {
        const float a = i < n ? sc[i] * inv : 0.f;
        if (i < n) sc[i] = a;
        if (blockIdx.x == 0) coef_out[(size_t)b * S + i] = a;
      }
    } else {
      float dot = 0.f;
      for (int i = t; i < n; i += 64) dot += a_in[(size_t)b * S + i] * dots[(size_t)b * S + i];
      dot = wave_sum(dot);
      for (int i = t; i < S; i += 64) {
        const float v = i < n ? a_in[(size_t)b * S + i] * (dots[(size_t)b * S + i] - dot) : 0.f;
        if (i < n) sc[i] = v;
        if (blockIdx.x == 0) coef_out[(size_t)b * S + i] = v;
      }
    }
  }
  __syncthreads();
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const float w = grp + 32 * q < n ? sc[grp + 32 * q] : 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += w * pre[q].get(e);
  }
  if (h0 < H) {
    for (int i = grp + 64; i < n; i += 32) {
      Frag<T> f;
      f.load(Mat + ((size_t)i * Bp + b) * ldm + h0);
      const float w = sc[i];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += w * f.get(e);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[grp][oct * 8 + e] = acc[e];
  __syncthreads();
  if (t < 64) {
    const int h = blockIdx.x * 64 + t;
    float s = 0.f;
    if (h < H) {
#pragma unroll
      for (int g = 0; g < 32; ++g) s += part[g][t];
      if (MODE == 0) {
        ((T*)out)[(size_t)b * ldo + h] = from_f<T>(s);
        if (sizeof(T) == 2 && out_fm) ((T*)out_fm)[fm_offset(b, h, H >> 5)] = from_f<T>(s);
      }
      else if (MODE == 2) {                                  // Eq. 7 on the projected rows: s + u is the pre-activation
        const float hv = tanh_of<sizeof(T) == 2>(s + addv);
        const float hd = dropped.outD ? hv * drop_factor(dropped.drop, b, h) : hv;
        ((T*)out)[(size_t)b * ldo + h] = from_f<T>(hv);
        if (dropped.outD) ((T*)dropped.outD)[(size_t)b * dropped.ldod + h] = from_f<T>(hd);
        if (sizeof(T) == 2 && out_fm) ((T*)out_fm)[fm_offset(b, h, H >> 5)] = from_f<T>(hd);
        if (sizeof(T) == 2 && dropped.outF2)
          ((T*)dropped.outF2)[fm_offset(b, dropped.outF2_k0 + h, dropped.outF2_nsteps)] = from_f<T>(hd);
      }
      else {
        s += addv;
        if (!fuse_cell) ((float*)out)[(size_t)b * H + h] = s;
      }
    }
    if (MODE == 1 && fuse_cell) {
      float dyx[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) dyx[e] = __shfl(s, 4 * (t & 15) + e, 64);
      const float zero[4] = {0.f, 0.f, 0.f, 0.f};
      if (do_cell) cell_bwd_finish<T>(cell, b, u4, H, cin, dyx, zero);
    }
  }
}

void launch_att_fwd(int prec, const void* Kmat, int ldk, const void* Hs, int lds, const void* Ht, int ldt,
                    const int32_t* src_len, int S, int Bp, int H, float* dots, float* a, void* Cs, int ldcs, hipStream_t st,
                    void* Cs_fm) {
  dim3 gd((S + 3) / 4, Bp), gm((H + 63) / 64, Bp);
  const Planes none{nullptr, 0, 0, 0};
  if (prec) {
    hipLaunchKernelGGL(att_dots_kernel<bf16_t>, gd, dim3(256), 0, st, (const bf16_t*)Kmat, ldk, (const bf16_t*)Ht, ldt, src_len, S, Bp, H, dots);
    hipLaunchKernelGGL((att_mix_kernel<bf16_t, 0>), gm, dim3(256), 0, st, (const bf16_t*)Hs, lds, ldcs, dots, nullptr, src_len, S, Bp, H, a, Cs, none, 0, LstmBwdPoint{}, 0, Cs_fm, AttDropped{});
  } else {
    hipLaunchKernelGGL(att_dots_kernel<float>, gd, dim3(256), 0, st, (const float*)Kmat, ldk, (const float*)Ht, ldt, src_len, S, Bp, H, dots);
    hipLaunchKernelGGL((att_mix_kernel<float, 0>), gm, dim3(256), 0, st, (const float*)Hs, lds, ldcs, dots, nullptr, src_len, S, Bp, H, a, Cs, none, 0, LstmBwdPoint{}, 0, nullptr, AttDropped{});
  }
}

void launch_att_fwd_proj(int prec, const void* Kmat, int ldk, const void* Pmat, int ldp, const void* Ht, int ldt,
                         const StepGemm& u, const AttOut& o, const int32_t* src_len, int S, int Bp, int H, float* dots, float* a,
                         hipStream_t st) {
  const int nbt = (Bp + 15) / 16;
  StepGrid sg{(u.N + 15) / 16, 1, nbt};
  const int n_gemm = step_grid_blocks(sg);
  const int nsteps = (u.K1 / 8 + 3) / 4;              // k steps of the contracted segment
  const int ks = nsteps > 16 ? 16 : 8;
  const dim3 grid(n_gemm + ((S + ks - 1) / ks) * Bp);
  const AttScores d{Kmat, ldk, Ht, ldt, src_len, S, H, dots, 0};
#define GO(TT, KS, FM) hipLaunchKernelGGL((att_dots_pre_kernel<TT, KS, 2, FM>), grid, dim3(64 * KS), 0, st, u.W_fm, u.a1_fm, u.out, u.K0, u.K1, \
                                          u.N, u.ldout, Bp, n_gemm, u, d)
  // (the fragment-major form reads the leading arguments alone: segment 1 of an unshifted W_fm)
  if (prec && step_gemm_has_fm(u) && u.skip0 && u.w_tile0 == 0) { if (ks == 16) GO(bf16_t, 16, true); else GO(bf16_t, 8, true); }
  else if (prec) { if (ks == 16) GO(bf16_t, 16, false); else GO(bf16_t, 8, false); }
  else { if (ks == 16) GO(float, 16, false); else GO(float, 8, false); }
#undef GO
  const dim3 gm((H + 63) / 64, Bp);
  const Planes up{u.out, u.ldout, 1, 0};
  const AttDropped dr{o.outD, o.ldod, o.drop, o.outF2, o.outF2_nsteps, o.outF2_k0};
  if (prec)
    hipLaunchKernelGGL((att_mix_kernel<bf16_t, 2>), gm, dim3(256), 0, st, (const bf16_t*)Pmat, ldp, o.ldo, dots, nullptr, src_len, S, Bp,
                       H, a, o.outT, up, 0, LstmBwdPoint{}, 0, o.outF, dr);
  else
    hipLaunchKernelGGL((att_mix_kernel<float, 2>), gm, dim3(256), 0, st, (const float*)Pmat, ldp, o.ldo, dots, nullptr, src_len, S, Bp,
                       H, a, o.outT, up, 0, LstmBwdPoint{}, 0, nullptr, dr);
}

// One workgroup: 64 columns of one sentence for 16 steps; the rows H_s^i pass through LDS 64 positions at a time.
template <typename T>
__global__ __launch_bounds__(256) void att_context_kernel(const T* __restrict__ Hs, int lds, const float* __restrict__ a,
                                                          const int32_t* __restrict__ len, int S, int Tn, int Bp, int H,
                                                          T* __restrict__ Cs, int ldcs) {
  __shared__ float sa[16][64];
  __shared__ float sh[64][65];
  const int t = threadIdx.x, col = t & 63, jq = t >> 6;
  const int b = blockIdx.y, j0 = blockIdx.z * 16, h0 = blockIdx.x * 64;
  const int n = min(len[b], S);
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < n; s0 += 64) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int idx = t + 256 * q, jj = idx >> 6, ss = idx & 63;
      sa[jj][ss] = (j0 + jj < Tn && s0 + ss < n) ? a[((size_t)(j0 + jj) * Bp + b) * S + s0 + ss] : 0.f;
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int f = t + 256 * q, ss = f >> 3, oct = f & 7;
      Frag<T> v;
      if (s0 + ss < n && h0 + oct * 8 < H) v.load(Hs + ((size_t)(s0 + ss) * Bp + b) * lds + h0 + oct * 8);
      else v.zero();
#pragma unroll
      for (int e = 0; e < 8; ++e) sh[ss][oct * 8 + e] = v.get(e);
    }
    __syncthreads();
    const int m = min(64, n - s0);
    for (int ss = 0; ss < m; ++ss) {
      const float hv = sh[ss][col];
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] += sa[jq * 4 + q][ss] * hv;
    }
    __syncthreads();
  }
  if (h0 + col < H)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int j = j0 + jq * 4 + q;
      if (j < Tn) Cs[((size_t)j * Bp + b) * ldcs + h0 + col] = from_f<T>(acc[q]);
    }
}
void launch_att_context(int prec, const void* Hs, int lds, const float* a, const int32_t* src_len, int S, int T, int Bp, int H,
                        void* Cs, int ldcs, hipStream_t st) {
  const dim3 grid((H + 63) / 64, Bp, (T + 15) / 16);
  if (prec) hipLaunchKernelGGL(att_context_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)Hs, lds, a, src_len, S, T, Bp, H, (bf16_t*)Cs, ldcs);
  else hipLaunchKernelGGL(att_context_kernel<float>, grid, dim3(256), 0, st, (const float*)Hs, lds, a, src_len, S, T, Bp, H, (float*)Cs, ldcs);
}

void launch_att_bwd(int prec, const void* Kmat, int ldk, const void* Hs, int lds, const Planes& dCst, float* dCs_sum, const float* a,
                    const int32_t* src_len, int S, int Bp, int H, float* dots, float* ds, float* dHt, hipStream_t st,
                    const LstmBwdPoint* cell) {
  const LstmBwdPoint cl = cell ? *cell : LstmBwdPoint{};
  const int fuse = cell ? 1 : 0;
  // dCst planes [.., Bp, 2H]: columns [0,H) = dC_s, columns [H,2H) = the direct part of dH_t
  // two positions per wavefront, 8 per workgroup (medium workload: attention backward 9.6 us per step against 10.3
  // with four and 10.5 with a wavefront per position, each summing the planes itself)
  constexpr int PW = 2;
  dim3 gd((S + 4 * PW - 1) / (4 * PW), Bp), gm((H + 63) / 64, Bp);
  if (prec) {
    hipLaunchKernelGGL((att_dots_planes_kernel<bf16_t, PW>), gd, dim3(256), 0, st, (const bf16_t*)Hs, lds, dCst, dCs_sum, src_len, S, Bp, H, dots);
    hipLaunchKernelGGL((att_mix_kernel<bf16_t, 1>), gm, dim3(256), 0, st, (const bf16_t*)Kmat, ldk, 0, dots, a, src_len, S, Bp, H, ds, dHt, dCst, H, cl, fuse, nullptr, AttDropped{});
  } else {
    hipLaunchKernelGGL((att_dots_planes_kernel<float, PW>), gd, dim3(256), 0, st, (const float*)Hs, lds, dCst, dCs_sum, src_len, S, Bp, H, dots);
    hipLaunchKernelGGL((att_mix_kernel<float, 1>), gm, dim3(256), 0, st, (const float*)Kmat, ldk, 0, dots, a, src_len, S, Bp, H, ds, dHt, dCst, H, cl, fuse, nullptr, AttDropped{});
  }
}

void launch_att_bwd_mix(int prec, const void* Kmat, int ldk, const Planes& add, int add_col, const float* a, const int32_t* src_len,
                        int S, int Bp, int H, const float* dots, float* ds, float* dHt, hipStream_t st, const LstmBwdPoint* cell) {
  const LstmBwdPoint cl = cell ? *cell : LstmBwdPoint{};
  const int fuse = cell ? 1 : 0;
  const dim3 gm((H + 63) / 64, Bp);
  if (prec)
    hipLaunchKernelGGL((att_mix_kernel<bf16_t, 1>), gm, dim3(256), 0, st, (const bf16_t*)Kmat, ldk, 0, dots, a, src_len, S, Bp, H, ds, dHt,
                       add, add_col, cl, fuse, nullptr, AttDropped{});
  else
    hipLaunchKernelGGL((att_mix_kernel<float, 1>), gm, dim3(256), 0, st, (const float*)Kmat, ldk, 0, dots, a, src_len, S, Bp, H, ds, dHt,
                       add, add_col, cl, fuse, nullptr, AttDropped{});
}

// After the decoder loop: for a block (sentence b, 256 hidden columns, ATT_DEF_IB source positions):
//   dHs[i,b,h] = sum_j a[j,b,i] dCs[j,b,h]        dK[i,b,h] = sum_j ds[j,b,i] Ht[j,b,h]
constexpr int ATT_DEF_IB = 32;                       // source positions per workgroup (each re-reads the step data once)
constexpr int ATT_DEF_JB = 256 / ATT_DEF_IB;         // decoder steps per pass: their loads are issued together
template <typename T>
__global__ __launch_bounds__(256) void att_deferred_kernel(const float* __restrict__ a, const float* __restrict__ ds,
                                                           const float* __restrict__ dCs, int lddc, const T* __restrict__ Ht,
                                                           int ldht, int S, int Tn, int Bp, int H, float* __restrict__ dHs,
                                                           T* __restrict__ dK) {
  constexpr int IB = ATT_DEF_IB, JB = ATT_DEF_JB;
  __shared__ __align__(16) float sa[JB][IB], sd[JB][IB];
  const int b = blockIdx.x, h = blockIdx.y * 256 + threadIdx.x, i0 = blockIdx.z * IB;
  float accC[IB], accK[IB];
#pragma unroll
  for (int i = 0; i < IB; ++i) { accC[i] = 0.f; accK[i] = 0.f; }
  for (int j0 = 0; j0 < Tn; j0 += JB) {
    __syncthreads();
    {
      const int jj = threadIdx.x / IB, il = threadIdx.x % IB, i = i0 + il;   // 256 threads = JB x IB
      const int j = j0 + jj;
      const bool ok = j < Tn && i < S;
      sa[jj][il] = ok ? a[((size_t)j * Bp + b) * S + i] : 0.f;
      sd[jj][il] = ok ? ds[((size_t)j * Bp + b) * S + i] : 0.f;
    }
    float dc[JB], ht[JB];
#pragma unroll
    for (int jj = 0; jj < JB; ++jj) {
      const int j = j0 + jj;
      const bool ok = h < H && j < Tn;
      dc[jj] = ok ? dCs[((size_t)j * Bp + b) * lddc + h] : 0.f;
      ht[jj] = ok ? to_f<T>(Ht[((size_t)j * Bp + b) * ldht + h]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int jj = 0; jj < JB; ++jj)                  // ascending j: the same summation order as one step at a time
#pragma unroll
      for (int i = 0; i < IB; i += 4) {              // coefficients as 16-byte LDS reads (same address in every lane)
        const float4 ca = *reinterpret_cast<const float4*>(&sa[jj][i]);
        const float4 cd = *reinterpret_cast<const float4*>(&sd[jj][i]);
        accC[i] += ca.x * dc[jj]; accC[i + 1] += ca.y * dc[jj]; accC[i + 2] += ca.z * dc[jj]; accC[i + 3] += ca.w * dc[jj];
        accK[i] += cd.x * ht[jj]; accK[i + 1] += cd.y * ht[jj]; accK[i + 2] += cd.z * ht[jj]; accK[i + 3] += cd.w * ht[jj];
      }
  }
  if (h >= H) return;
#pragma unroll
  for (int i = 0; i < IB; ++i) {
    if (i0 + i < S) {
      const size_t o = ((size_t)(i0 + i) * Bp + b) * H + h;
      dHs[o] = accC[i];
      dK[o] = from_f<T>(accK[i]);
    }
  }
}

void launch_att_deferred(int prec, const float* a, const float* ds, const float* dCs, int lddc, const void* Ht, int ldht,
                         int S, int T, int Bp, int H, float* dHs, void* dK, hipStream_t st) {
  dim3 grid(Bp, (H + 255) / 256, (S + ATT_DEF_IB - 1) / ATT_DEF_IB);
  if (prec) hipLaunchKernelGGL(att_deferred_kernel<bf16_t>, grid, dim3(256), 0, st, a, ds, dCs, lddc, (const bf16_t*)Ht, ldht, S, T,
                               Bp, H, dHs, (bf16_t*)dK);
  else hipLaunchKernelGGL(att_deferred_kernel<float>, grid, dim3(256), 0, st, a, ds, dCs, lddc, (const float*)Ht, ldht, S, T, Bp, H,
                          dHs, (float*)dK);
}

template <typename T>
__global__ __launch_bounds__(256) void tanh_planes_kernel(Planes p, T* __restrict__ out, int ldo, T* __restrict__ outD, int ldod,
                                                          DropSpec drop, int Bp, int N) {
  const int i4 = blockIdx.x * 256 + threadIdx.x;
  const int nq = N >> 2;
  if (i4 >= Bp * nq) return;
  int b, n;
  divmod_uniform(i4, nq, b, n);
  n *= 4;
  const float4 v = planes_get4(p, b, n);
  constexpr bool FAST = sizeof(T) == 2;
  const float o[4] = {tanh_of<FAST>(v.x), tanh_of<FAST>(v.y), tanh_of<FAST>(v.z), tanh_of<FAST>(v.w)};
  store4<T>(out + (size_t)b * ldo + n, o);
  if (outD) {
    const float od[4] = {o[0] * drop_factor(drop, b, n), o[1] * drop_factor(drop, b, n + 1), o[2] * drop_factor(drop, b, n + 2),
                         o[3] * drop_factor(drop, b, n + 3)};
    store4<T>(outD + (size_t)b * ldod + n, od);
  }
}
template __global__ void tanh_planes_kernel<bf16_t>(Planes, bf16_t*, int, bf16_t*, int, DropSpec, int, int);
template __global__ void tanh_planes_kernel<float>(Planes, float*, int, float*, int, DropSpec, int, int);

// dpre = (dHo_ce + feed) * (1 - Ho^2) -> T; feed arrives as planes (np = 0: none); 4 columns per thread
template <typename T>
__global__ __launch_bounds__(64) void tanh_bwd_kernel(const float* __restrict__ dce, const int32_t* __restrict__ pos, Planes feed,
                                                      const T* __restrict__ Ho, int ldho, T* __restrict__ dpre, int ldp, int Bp,
                                                      int H, DropSpec drop, T* __restrict__ dpre_fm) {
  const int i4 = blockIdx.x * 64 + threadIdx.x;        // single-wavefront workgroups: spread over all CUs
  const int hq = H >> 2;
  if (i4 >= Bp * hq) return;
  int b, h;
  divmod_uniform(i4, hq, b, h);
  h *= 4;
  const int c = pos ? pos[b] : b;                      // row of sentence b in dce
  const float4 d = c >= 0 ? *reinterpret_cast<const float4*>(dce + (size_t)c * H + h) : make_float4(0.f, 0.f, 0.f, 0.f);
  const float4 f = planes_get4(feed, b, h);
  float o[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float ho = to_f<T>(Ho[(size_t)b * ldho + h + e]);
    o[e] = ((&d.x)[e] + (&f.x)[e]) * drop_factor(drop, b, h + e) * (1.f - ho * ho);
  }
  store4<T>(dpre + (size_t)b * ldp + h, o);
  if (sizeof(T) == 2 && dpre_fm) store4<T>(dpre_fm + fm_offset(b, h, H >> 5), o);
}

void launch_tanh_bwd(int prec, const float* dHo_ce, const int32_t* pos, const Planes& feed, const void* Ho, int ldho, void* dpre,
                     int ldp, int Bp, int H, const DropSpec& drop, hipStream_t st, void* dpre_fm) {
  const int n = Bp * (H >> 2);
  if (prec) hipLaunchKernelGGL(tanh_bwd_kernel<bf16_t>, dim3((n + 63) / 64), dim3(64), 0, st, dHo_ce, pos, feed,
                               (const bf16_t*)Ho, ldho, (bf16_t*)dpre, ldp, Bp, H, drop, (bf16_t*)dpre_fm);
  else hipLaunchKernelGGL(tanh_bwd_kernel<float>, dim3((n + 63) / 64), dim3(64), 0, st, dHo_ce, pos, feed,
                          (const float*)Ho, ldho, (float*)dpre, ldp, Bp, H, drop, (float*)nullptr);
}

}  // namespace cmt
