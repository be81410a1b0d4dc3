// Shared by the matrix-core GEMM kernels: operand types, the one MFMA instruction, and the
// tile epilogues (the layer's element-wise work on finished fp32 tiles).
#pragma once
#include "spec_internal.h"
#include "device_utils.h"
#include "mfma_gemm.h"

// No implicit fusing of multiplies and adds (see kernels_gemm_mfma.hip).
#pragma clang fp contract(off)

namespace spec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_v;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_v;
typedef __attribute__((ext_vector_type(4))) float f32x4_v;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_v;

// The one instruction: D(16x16 fp32) += A(16x32 fp16) * B(32x16 fp16).
struct Mfma16 {
  static __device__ __forceinline__ f32x4_v run(u32x4_v a, u32x4_v b, f32x4_v c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_v, a), __builtin_bit_cast(f16x8_v, b), c,
                                                  0, 0, 0);
  }
};

// Folded norm, consumer side: the sum of squares of a row of activations is taken from the fp16 operand
// fragments the GEMM reads anyway.  In the B operand lane (c, g) holds elements 8g .. 8g+7 of row c of a
// 32-k step: a lane adds its eight squares to a running fp32 sum, two at a time in ascending k (the two-element
// dot-product instruction: four instead of sixteen operations per fragment), one chain per k-slice from zero; the
// slices are added in slice order per lane, then the four lane groups of a row as (g0 + g1) + (g2 + g3).  Every
// GEMM kernel follows exactly this order, so the value depends on the row alone.
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_v;
// (the pairs are taken from the fragment cast as a whole: a bit cast of one element of a vector, x[i], compiles to a
// read of element 0 whatever i)
__device__ __forceinline__ float frag_ssq(u32x4_v x, float s) {
  const f16x8_v h = __builtin_bit_cast(f16x8_v, x);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const f16x2_v p = {h[2 * i], h[2 * i + 1]};
    s = __builtin_amdgcn_fdot2(p, p, s, false);
  }
  return s;
}
// the same chain for the plain sum of the row (folded LayerNorm: the mean)
__device__ __forceinline__ float frag_sum(u32x4_v x, float s) {
  const f16x8_v h = __builtin_bit_cast(f16x8_v, x);
  const f16x2_v one = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const f16x2_v p = {h[2 * i], h[2 * i + 1]};
    s = __builtin_amdgcn_fdot2(p, one, s, false);
  }
  return s;
}
// folded LayerNorm: per-lane slice-ordered sums of squares and sums -> 1 / std and mean of the lane's row (lane groups
// combined as below; variance as mean of squares minus squared mean, in fp32)
__device__ __forceinline__ void row_ln_from_lane(float ssq, float sum, int d, float eps, float &rinv, float &mean) {
  ssq += __shfl_xor(ssq, 16, 64);
  ssq += __shfl_xor(ssq, 32, 64);
  sum += __shfl_xor(sum, 16, 64);
  sum += __shfl_xor(sum, 32, 64);
  mean = sum / (float)d;
  const float var = fmaxf(ssq / (float)d - mean * mean, 0.f);
  rinv = 1.0f / sqrtf(var + eps);
}
// per-lane slice-ordered sum -> 1 / rms of the lane's row (all four lanes of a row get the same bits)
__device__ __forceinline__ float row_inv_from_lane_ssq(float t, int d, float eps) {
  t += __shfl_xor(t, 16, 64);
  t += __shfl_xor(t, 32, 64);
  return 1.0f / sqrtf(t / (float)d + eps);
}

// h[m][n..n+3] += v (scaled, biased): the residual update of one lane's four outputs; o4 = the updated values
// rounded to the next GEMM's operand type (also written to x_out in fragment order when that is set).
__device__ __forceinline__ void residual_update(const GemmArgs &a, f32x4_v v, int n, int m, op_t (&o4)[4]) {
  v[0] *= a.out_scale; v[1] *= a.out_scale; v[2] *= a.out_scale; v[3] *= a.out_scale;  // exact: a power of two
  if (a.bias) {
    const float4 b4 = *(const float4 *)(a.bias + n);
    v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
  }
  float4 *p = (float4 *)(a.h + (size_t)m * a.N + n);
  float4 o = *p;
  o.x += v[0]; o.y += v[1]; o.z += v[2]; o.w += v[3];
  *p = o;
  if (a.x_out) {  // the next GEMM's activations: the updated row, rounded to fp16
    o4[0] = to_op_counted(o.x, a.sat); o4[1] = to_op_counted(o.y, a.sat);
    o4[2] = to_op_counted(o.z, a.sat); o4[3] = to_op_counted(o.w, a.sat);
    *(uint2 *)((op_t *)a.x_out + xpack_index(m, n, a.N >> 5)) = *(const uint2 *)o4;
  }
}

// ------------------------------------------------------------------------- epilogues
// One finished 16x16 tile: this lane holds stored rows n .. n+3 (n = 16*nt + 4g) of
// activation row m.  The element-wise work of the layer happens here, on fp32 sums.
// rinv: 1 / rms of row m when the norm in front of this GEMM is folded into it, else 1.
template <class T, int EPI>
__device__ __forceinline__ void tile_epilogue(const GemmArgs &a, f32x4_v v, int nt, int m, int g, float rinv = 1.0f, float mean = 0.f) {
  if (nt >= a.NT) return;
  const int n = nt * 16 + 4 * g;
  if (EPI == EPI_RESIDUAL) {
    op_t o4[4];
    if (m < a.M && n < a.N) residual_update(a, v, n, m, o4);
    return;
  }
  if (a.wsum) {  // folded LayerNorm: take the mean's share out, in the packed weights' units
    const float4 ws = *(const float4 *)(a.wsum + n);
    v[0] -= mean * ws.x; v[1] -= mean * ws.y; v[2] -= mean * ws.z; v[3] -= mean * ws.w;
  }
  v[0] *= a.out_scale; v[1] *= a.out_scale; v[2] *= a.out_scale; v[3] *= a.out_scale;  // exact: a power of two
  v[0] *= rinv; v[1] *= rinv; v[2] *= rinv; v[3] *= rinv;
  if (a.bias) {
    const float4 b4 = *(const float4 *)(a.bias + n);
    v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
  }
  const bool live = m < a.M;

  if (EPI == EPI_QKV) {
    if (live && n < a.N) {
      // No per-lane integer division (it would be most of this epilogue).  A strip of 16 stored rows lies
      // inside one head of one of q, k, v (d and hd are multiples of 16), and the strip number is the same for
      // the whole wave: its place is scalar arithmetic.  The row's sequence m / q_rows comes from a float
      // product, made exact by one step either way.
      const int base = __builtin_amdgcn_readfirstlane(nt) * 16;
      const int region = base / a.d, cc0 = base - region * a.d, hh = cc0 / a.hd;
      const int cc = cc0 + 4 * g, e = cc - hh * a.hd;
      const int pos = a.row_pos[m];
      int b = (int)(((float)m + 0.5f) * (1.0f / (float)a.q_rows));
      b += ((b + 1) * a.q_rows <= m) ? 1 : 0;
      b -= (b * a.q_rows > m) ? 1 : 0;
      if (a.seq_groups > 1) b /= a.seq_groups;  // prefill passes only
      if (region < 2) {
        float r0 = v[0], r1 = v[1], r2 = v[2], r3 = v[3];
        if (a.rope && pos >= 0) {
          const float2 cs0 = a.rope[(size_t)pos * (a.hd >> 1) + (e >> 1)];
          const float2 cs1 = a.rope[(size_t)pos * (a.hd >> 1) + (e >> 1) + 1];
          r0 = v[0] * cs0.x - v[1] * cs0.y; r1 = v[1] * cs0.x + v[0] * cs0.y;
          r2 = v[2] * cs1.x - v[3] * cs1.y; r3 = v[3] * cs1.x + v[2] * cs1.y;
        }
        if (region == 0) {  // queries stay fp32: they are never cached, and the attention kernel feeds them at full width
          *(float4 *)((float *)a.q + (size_t)m * a.d + cc) = make_float4(r0, r1, r2, r3);
        } else if (pos >= 0) {
          T o4[4];
          Conv<T>::st(o4, 0, r0); Conv<T>::st(o4, 1, r1); Conv<T>::st(o4, 2, r2); Conv<T>::st(o4, 3, r3);
          *(uint2 *)((T *)a.kc + kv_k_index(a.L_pad, a.H, a.hd, b, hh, pos, e)) = *(const uint2 *)o4;
        }
      } else if (pos >= 0) {
        T *vc = (T *)a.vc;
#pragma unroll
        for (int i = 0; i < 4; ++i) Conv<T>::st(vc, kv_v_index(a.L_pad, a.H, a.hd, b, hh, pos, e + i), v[i]);
      }
    }
  } else if (EPI == EPI_SWIGLU) {
    const int j = n >> 1;  // stored rows n..n+3 = gate_j, up_j, gate_{j+1}, up_{j+1}
    if (live && j < a.f) {
      const float r0 = v[0] / (1.0f + __expf(-v[0])) * v[1], r1 = v[2] / (1.0f + __expf(-v[2])) * v[3];
      op_t o2[2] = {to_op_counted(r0, a.sat), to_op_counted(r1, a.sat)};
      const size_t at = xpack_index(m, j, a.f >> 5);
      *(uint32_t *)((op_t *)a.act + at) = *(const uint32_t *)o2;
    }
  } else if (EPI == EPI_RELU) {
    if (live && n < a.N) {
      op_t o4[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) o4[i] = to_op_counted(v[i] > 0.f ? v[i] : 0.f, a.sat);
      const size_t at = xpack_index(m, n, a.N >> 5);
      *(uint2 *)((op_t *)a.act + at) = *(const uint2 *)o4;
    }
  } else {  // EPI_LOGITS: optional dump, per-strip arg-max partial (lowest index wins ties)
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    float *dump = nullptr;  // debug / parity only
    if (live && a.logits) {
      if (a.logit_step <= 1) dump = a.logits + (size_t)m * a.N;
      else if (m % a.logit_step == a.logit_step - 1) dump = a.logits + (size_t)(m / a.logit_step) * a.N;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (n + i < a.N) {
        if (dump) dump[n + i] = v[i];
        argmax_combine(bv, bi, v[i], n + i);
      }
    for (int o = 16; o <= 32; o <<= 1) {
      float ov = __shfl_xor(bv, o, 64);
      int oi = __shfl_xor(bi, o, 64);
      argmax_combine(bv, bi, ov, oi);
    }
    if (live && g == 0) {
      a.part_val[(size_t)m * a.NT + nt] = bv;
      a.part_idx[(size_t)m * a.NT + nt] = bi;
    }
  }
}

}  // namespace spec
