// Device-side building blocks shared by the gfx950 kernels: storage types, MFMA fragment
// loads and the two matrix-core tile shapes used everywhere (16x16 and 32x32 outputs).
//
// Every contraction in the training step is written against one fragment convention:
// a lane holds 8 consecutive k-values of one row of an operand whose k index is contiguous in
// memory.  For bf16 that is exactly the operand of v_mfma_f32_{16x16x32,32x32x16}_bf16; for
// fp32 the same 8 values feed 8 back-to-back v_mfma_f32_{16x16x4,32x32x2}_f32 (the k order
// inside a tile is permuted identically for both operands, which leaves the sum unchanged).
// The accumulator layouts of the bf16 and fp32 instructions coincide, so every kernel is one
// template over the storage type.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cmt {

typedef uint16_t bf16_t;                                   // raw bfloat16 bits
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {           // round to nearest even (the hardware conversion)
  const __bf16 b = (__bf16)f;
  return __builtin_bit_cast(bf16_t, b);
}

template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v) { return bf2f(v); }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return f2bf(v); }

// 8 consecutive-k elements of one operand row.
template <typename T> struct Frag;
template <> struct Frag<bf16_t> {
  uint4 v;
  __device__ __forceinline__ void zero() { v = make_uint4(0, 0, 0, 0); }
  __device__ __forceinline__ void load(const bf16_t* p) { v = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ float get(int i) const {
    uint32_t w = (&v.x)[i >> 1];
    return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
  }
};
template <> struct Frag<float> {
  float4 lo, hi;
  __device__ __forceinline__ void zero() { lo = make_float4(0, 0, 0, 0); hi = lo; }
  __device__ __forceinline__ void load(const float* p) {
    lo = *reinterpret_cast<const float4*>(p);
    hi = *reinterpret_cast<const float4*>(p + 4);
  }
  __device__ __forceinline__ float get(int i) const { return i < 4 ? (&lo.x)[i] : (&hi.x)[i - 4]; }
};

// 16x16 output tile, 32 k per call.  Operand lane l: row (l % 16), k = 8 * (l / 16) + 0..7.
// Accumulator lane l, register i: row 4 * (l / 16) + i of A's rows, column (l % 16) of B's rows.
__device__ __forceinline__ void mma16(v4f& acc, const Frag<bf16_t>& a, const Frag<bf16_t>& b) {
  acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a.v), __builtin_bit_cast(v8bf, b.v), acc, 0, 0, 0);
}
__device__ __forceinline__ void mma16(v4f& acc, const Frag<float>& a, const Frag<float>& b) {
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.lo.x, b.lo.x, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.lo.y, b.lo.y, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.lo.z, b.lo.z, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.lo.w, b.lo.w, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.hi.x, b.hi.x, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.hi.y, b.hi.y, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.hi.z, b.hi.z, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.hi.w, b.hi.w, acc, 0, 0, 0);
}

// 32x32 output tile, 16 k per call.  Operand lane l: row (l % 32), k = 8 * (l / 32) + 0..7.
// Accumulator lane l, register i: row 8 * (i / 4) + 4 * (l / 32) + (i % 4), column (l % 32).
__device__ __forceinline__ void mma32(v16f& acc, const Frag<bf16_t>& a, const Frag<bf16_t>& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a.v), __builtin_bit_cast(v8bf, b.v), acc, 0, 0, 0);
}
__device__ __forceinline__ void mma32(v16f& acc, const Frag<float>& a, const Frag<float>& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.lo.x, b.lo.x, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.lo.y, b.lo.y, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.lo.z, b.lo.z, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.lo.w, b.lo.w, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.hi.x, b.hi.x, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.hi.y, b.hi.y, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.hi.z, b.hi.z, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.hi.w, b.hi.w, acc, 0, 0, 0);
}
__device__ __forceinline__ int acc32_row(int lane, int i) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

// Keeps a wavefront-uniform value (a kernel argument, a field of an argument structure picked by a uniform index)
// in a scalar register from this point on.  Without it the compiler fetches such a value where it is first used;
// in an epilogue behind a barrier that is one scalar load and one wait after the other, each a trip to the
// scalar cache, on the critical path of a kernel that lasts a few microseconds.
#define CMT_PIN_UNIFORM(x) asm volatile("" : "+s"(x))
// The same for a pointer to device memory.  The value passes through the global address space, so that what
// is reached through it afterwards is still known to be global memory (an opaque generic pointer would turn
// every access into a flat one).
#define CMT_PIN_UNIFORM_PTR(p)                                                                  \
  do {                                                                                          \
    auto cmt_gp_ = (__attribute__((address_space(1))) char*)(p);                                \
    asm volatile("" : "+s"(cmt_gp_));                                                           \
    (p) = (decltype(p))(char*)cmt_gp_;                                                          \
  } while (0)

// i / d and i % d for a wavefront-uniform divisor: a shift when d is a power of two (the usual case for widths)
__device__ __forceinline__ void divmod_uniform(int i, int d, int& q, int& r) {
  if ((d & (d - 1)) == 0) { q = i >> __builtin_ctz(d); r = i & (d - 1); }
  else { q = i / d; r = i - q * d; }
}

// Gate nonlinearities.  The fp32 path takes the full-accuracy library routines.  On the 16-bit path (FAST) the
// results are rounded to 8 significant bits or meet operands that were, so the hardware exponential and
// reciprocal (about 1e-6 relative) are as good, at a tenth of the instructions — the cell epilogues of the
// per-step kernels run on one or two wavefronts per workgroup and wait for these.
__device__ __forceinline__ float sigm(float x) { return 1.0f / (1.0f + expf(-x)); }
template <bool FAST> __device__ __forceinline__ float sigm_of(float x) {
  if (FAST) return __builtin_amdgcn_rcpf(1.0f + __expf(-x));
  return sigm(x);
}
template <bool FAST> __device__ __forceinline__ float tanh_of(float x) {
  if (FAST) return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * x));   // exp = inf -> 1, exp = 0 -> -1
  return tanhf(x);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

}  // namespace cmt
