// Device-side helpers: storage types, conversions, fixed-order wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spec {

struct bf16_t { uint16_t v; };
typedef _Float16 f16_t;

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t u) { return __uint_as_float((uint32_t)u << 16); }
// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t x = __float_as_uint(f);
  if ((x & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
  x += 0x7fffu + ((x >> 16) & 1u);
  return (uint16_t)(x >> 16);
}

template <class T> struct Conv;
template <> struct Conv<float> {
  static __device__ __forceinline__ float ld(const float *p, size_t i) { return p[i]; }
  static __device__ __forceinline__ void st(float *p, size_t i, float f) { p[i] = f; }
  static __device__ __forceinline__ float round(float f) { return f; }
};
template <> struct Conv<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t *p, size_t i) { return bf16_bits_to_f32(p[i].v); }
  static __device__ __forceinline__ void st(bf16_t *p, size_t i, float f) { p[i].v = f32_to_bf16_bits(f); }
  static __device__ __forceinline__ float round(float f) { return bf16_bits_to_f32(f32_to_bf16_bits(f)); }
};
template <> struct Conv<f16_t> {
  static __device__ __forceinline__ float ld(const f16_t *p, size_t i) { return (float)p[i]; }
  static __device__ __forceinline__ void st(f16_t *p, size_t i, float f) { p[i] = (f16_t)f; }
  static __device__ __forceinline__ float round(float f) { return (float)(f16_t)f; }
};

// Operand type of the matrix-core GEMMs, for bf16 and fp16 models alike: fp16 has three more
// significand bits than bf16, and an fp32 activation rounded once to fp16 carries the layer as
// accurately as a bf16 high part plus a bf16 low part at half the matrix work.  Weights of bf16
// models are held as fp16 times a power of two per matrix (exact, see the packing kernel);
// activations beyond the fp16 range saturate.
typedef f16_t op_t;
__device__ __forceinline__ op_t to_op(float f) {
  f = f > 65504.f ? 65504.f : (f < -65504.f ? -65504.f : f);  // NaN passes through
  return (op_t)f;
}

// to_op that also counts the values it had to clamp (sat: a device counter, or null)
__device__ __forceinline__ op_t to_op_counted(float f, unsigned int *sat) {
  if (sat && (f > 65504.f || f < -65504.f)) atomicAdd(sat, 1u);
  return to_op(f);
}

// Activations that feed a matrix-core GEMM are stored in the order the B operand is loaded:
// 16-row x 32-k tiles of 1 KB, tile (m/16, k/32) at ((m/16) * KT + k/32), inside a tile lane
// 16*((k%32)/8) + m%16 owns 8 consecutive k.  Element index of X[m][k] for a row length of 32*KT:
__host__ __device__ __forceinline__ size_t xpack_index(int m, int k, int KT) {
  return ((((size_t)(m >> 4) * KT + (k >> 5)) * 64 + (((k & 31) >> 3) << 4) + (m & 15)) << 3) + (k & 7);
}

// Butterfly sum over the 64 lanes of a wave: every lane ends with the same value and
// the order of additions is fixed by the lane numbers alone.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// (value, index) arg-max combine: larger value wins, equal values -> lower index.
__device__ __forceinline__ void argmax_combine(float &v, int &i, float ov, int oi) {
  if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}
__device__ __forceinline__ void wave_argmax(float &v, int &i) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    float ov = __shfl_xor(v, o, 64);
    int oi = __shfl_xor(i, o, 64);
    argmax_combine(v, i, ov, oi);
  }
}

}  // namespace spec

#define SPEC_DISPATCH_DTYPE(dtype, T, ...)                                   \
  do {                                                                       \
    if ((dtype) == SPEC_DTYPE_F32) { typedef float T; __VA_ARGS__; }         \
    else if ((dtype) == SPEC_DTYPE_BF16) { typedef spec::bf16_t T; __VA_ARGS__; } \
    else { typedef spec::f16_t T; __VA_ARGS__; }                             \
  } while (0)
