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

// Folded RMS norm, consumer side: the sum of squares of a row of activations is taken from the fp16 operand
// fragments the GEMM reads anyway.  In the B operand lane (c, g) holds elements 8g .. 8g+7 of row c of a
// 32-k step: a lane adds its eight squares (exact in fp32) to a running fp32 sum by fused multiply-adds in
// ascending k, one chain per k-slice from zero; the slices are added in slice order per lane, then the four
// lane groups of a row as (g0 + g1) + (g2 + g3).  Every GEMM kernel follows exactly this order, so the value
// depends on the row alone.
__device__ __forceinline__ float frag_ssq(u32x4_v x, float s) {
  const f16x8_v h = __builtin_bit_cast(f16x8_v, x);
#pragma unroll
  for (int i = 0; i < 8; ++i) s = fmaf((float)h[i], (float)h[i], s);
  return s;
}
// per-lane slice-ordered sum -> 1 / rms of the lane's row (all four lanes of a row get the same bits)
__device__ __forceinline__ float row_inv_from_lane_ssq(float t, int d, float eps) {
  t += __shfl_xor(t, 16, 64);
  t += __shfl_xor(t, 32, 64);
  return 1.0f / sqrtf(t / (float)d + eps);
}

// h[m][n..n+3] += v (scaled, biased): the residual update of one lane's four outputs; o4 = the updated values
// rounded to the next GEMM's operand type (also written to x_out in fragment order when that is set).
__device__ __forceinline__ void residual_update(const GemmArgs &a, f32x4_v v, int n, int m, op_t (&o4)[4], float4 *h_new = nullptr) {
  v[0] *= a.out_scale; v[1] *= a.out_scale; v[2] *= a.out_scale; v[3] *= a.out_scale;  // exact: a power of two
  if (a.bias) {
    const float4 b4 = *(const float4 *)(a.bias + n);
    v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
  }
  float4 *p = (float4 *)(a.h + (size_t)m * a.N + n);
  float4 o = *p;
  o.x += v[0]; o.y += v[1]; o.z += v[2]; o.w += v[3];
  *p = o;
  if (h_new) *h_new = o;
  if (a.x_out) {  // the next GEMM's activations: the updated row, rounded to fp16
    o4[0] = to_op_counted(o.x, a.sat); o4[1] = to_op_counted(o.y, a.sat);
    o4[2] = to_op_counted(o.z, a.sat); o4[3] = to_op_counted(o.w, a.sat);
    *(uint2 *)((op_t *)a.x_out + xpack_index(m, n, a.N >> 5)) = *(const uint2 *)o4;
  }
}

// -------------------------------------------------------------------------
// RMSNorm / LayerNorm of one row of the fp32 residual stream by the first 256 threads of a workgroup.  Statistics in
// fp32 with a fixed reduction tree (per-thread strided partial, wave butterfly, then the four wave results in order),
// so a row's result never depends on which other rows are in the pass -- nor on which kernel runs this: the norm
// kernel (a 256-thread workgroup per row, row in memory) and the row-wise reduction of a split residual GEMM (a wider
// workgroup, WIDE: the others only keep the barriers company; row in LDS) execute these very instructions.
template <bool WIDE>
__device__ __forceinline__ float block_sum_256(float v, float *sh) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0 && (!WIDE || w < 4)) sh[w] = v;
  __syncthreads();
  return ((sh[0] + sh[1]) + sh[2]) + sh[3];
}

// Row held in registers: thread t owns the float4 groups t, t+256, ... (all loads issued
// before any arithmetic, so the kernel costs one memory round trip, not d/256 of them).
constexpr int NORM_MAX_V4 = 8;  // d <= 8192
constexpr int NORM_ROW_MAX = NORM_MAX_V4 * 1024;
// four consecutive parameters (index a multiple of 4) with one load
template <class T>
__device__ __forceinline__ void load4(const T *__restrict__ p, int i, float (&out)[4]) {
  struct alignas(sizeof(T) * 4) Quad { T v[4]; };
  const Quad q = *(const Quad *)(p + i);
#pragma unroll
  for (int k = 0; k < 4; ++k) out[k] = Conv<T>::ld(q.v, k);
}
// the gains and biases of the elements a thread owns (float4 groups t, t + 256, ...); zero where it owns none
template <class T, bool WIDE>
__device__ __forceinline__ void norm_params(int kind, int d, const T *__restrict__ gain, const T *__restrict__ bias,
                                            float (&gn)[NORM_MAX_V4][4], float (&bs)[NORM_MAX_V4][4]) {
  const int nv = (!WIDE || threadIdx.x < 256) ? d >> 2 : 0;
#pragma unroll
  for (int i = 0; i < NORM_MAX_V4; ++i) {
    const int c = threadIdx.x + i * 256;
#pragma unroll
    for (int k = 0; k < 4; ++k) { gn[i][k] = 0.f; bs[i][k] = 0.f; }
    if (c < nv) {
      load4(gain, 4 * c, gn[i]);
      if (kind != SPEC_NORM_RMS) load4(bias, 4 * c, bs[i]);
    }
  }
}
// gn, bs: from norm_params, fetched by the caller as early as it can (their latency then passes behind other work)
template <class T, bool WIDE>
__device__ __forceinline__ void norm_row(int kind, int d, float eps, const float4 *hr, const float (&gn)[NORM_MAX_V4][4],
                                         const float (&bs)[NORM_MAX_V4][4], int r, void *__restrict__ x, int pack_kt,
                                         unsigned int *__restrict__ sat, float *sh) {
  const bool act = !WIDE || threadIdx.x < 256;
  const int nv = act ? d >> 2 : 0;  // the passive threads of a wide workgroup own no element
  float4 v[NORM_MAX_V4];
#pragma unroll
  for (int i = 0; i < NORM_MAX_V4; ++i) {
    const int c = threadIdx.x + i * 256;
    v[i] = c < nv ? hr[c] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float mean = 0.f, inv;
  if (kind == SPEC_NORM_RMS) {
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_MAX_V4; ++i) {
      ss = fmaf(v[i].x, v[i].x, ss); ss = fmaf(v[i].y, v[i].y, ss);
      ss = fmaf(v[i].z, v[i].z, ss); ss = fmaf(v[i].w, v[i].w, ss);
    }
    ss = block_sum_256<WIDE>(ss, sh);
    inv = 1.0f / sqrtf(ss / (float)d + eps);
  } else {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_MAX_V4; ++i) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    mean = block_sum_256<WIDE>(s, sh) / (float)d;
    float vs = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_MAX_V4; ++i) {
      const int c = threadIdx.x + i * 256;
      if (c < nv) {
        float a0 = v[i].x - mean, a1 = v[i].y - mean, a2 = v[i].z - mean, a3 = v[i].w - mean;
        vs = fmaf(a0, a0, vs); vs = fmaf(a1, a1, vs); vs = fmaf(a2, a2, vs); vs = fmaf(a3, a3, vs);
      }
    }
    inv = 1.0f / sqrtf(block_sum_256<WIDE>(vs, sh) / (float)d + eps);
  }
#pragma unroll
  for (int i = 0; i < NORM_MAX_V4; ++i) {
    const int c = threadIdx.x + i * 256;
    if (c < nv) {
      const float e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
      float o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        o[k] = (e[k] - mean) * inv * gn[i][k];
        if (kind != SPEC_NORM_RMS) o[k] += bs[i][k];
      }
      if (pack_kt > 0) {
        // the consumer is a matrix-core GEMM: fp16 operands, rows stored in fragment order, where four consecutive
        // elements of a row are eight contiguous bytes
        op_t o4[4] = {to_op_counted(o[0], sat), to_op_counted(o[1], sat), to_op_counted(o[2], sat), to_op_counted(o[3], sat)};
        *(uint2 *)((op_t *)x + xpack_index(r, 4 * c, pack_kt)) = *(const uint2 *)o4;
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) Conv<T>::st((T *)x, (size_t)r * d + 4 * c + k, o[k]);
      }
    }
  }
}

// ------------------------------------------------------------------------- epilogues
// One finished 16x16 tile: this lane holds stored rows n .. n+3 (n = 16*nt + 4g) of
// activation row m.  The element-wise work of the layer happens here, on fp32 sums.
// rinv: 1 / rms of row m when the norm in front of this GEMM is folded into it, else 1.
template <class T, int EPI>
__device__ __forceinline__ void tile_epilogue(const GemmArgs &a, f32x4_v v, int nt, int m, int g, float rinv = 1.0f) {
  if (nt >= a.NT) return;
  const int n = nt * 16 + 4 * g;
  if (EPI == EPI_RESIDUAL) {
    op_t o4[4];
    if (m < a.M && n < a.N) residual_update(a, v, n, m, o4);
    return;
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
