// Verification attention on the matrix cores: the (up to 16) new query rows of one
// sequence against that sequence's KV cache, causal among the new rows.
//
// HBM-bound on the cache (a handful of flops per cached byte), so the layout is built
// around the loads: one wave owns one (sequence, head, 256-key chunk); keys stream in as
// full 256-byte rows, values as 16-byte runs of 8 consecutive positions.
//
// Transposed formulation, so that scores never move between lanes:
//   S^T[key][query]  = K . Q^T     A operand = 16 key rows,  B operand = 16 query rows
//   O^T[dim][query] += V^T . P^T   A operand = V^T (16 dims x 32 keys), B operand = P^T
// The accumulator layout of the first product (lane = query column, 4 consecutive keys per
// lane and tile) is already the B-operand layout of the second once the key rows fed to
// the first product are permuted: tile t, row 4g'+i carries key ks + 8g' + 4t + i.
//
// Numerics depend on (sequence, absolute positions) only: chunks start at multiples of 256,
// steps of 32 keys ascend inside a chunk, the chunk partials are merged in ascending order
// by a second kernel.  Masked keys contribute exact zeros and leave the running maximum
// unchanged, so the other rows of a pass never change a row's bits.
#include "spec_internal.h"
#include "device_utils.h"
#include "mfma_gemm.h"

namespace spec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_v;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_v;
typedef __attribute__((ext_vector_type(4))) float f32x4_v;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_v;

template <class T> struct MfmaA;
template <> struct MfmaA<bf16_t> {
  static __device__ __forceinline__ f32x4_v run(u32x4_v a, u32x4_v b, f32x4_v c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_v, a), __builtin_bit_cast(bf16x8_v, b), c,
                                                   0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
  }
};
template <> struct MfmaA<f16_t> {
  static __device__ __forceinline__ f32x4_v run(u32x4_v a, u32x4_v b, f32x4_v c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_v, a), __builtin_bit_cast(f16x8_v, b), c,
                                                  0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f16_t a = (f16_t)lo, b = (f16_t)hi;
    uint16_t ua, ub;
    __builtin_memcpy(&ua, &a, 2);
    __builtin_memcpy(&ub, &b, 2);
    return (uint32_t)ua | ((uint32_t)ub << 16);
  }
};

constexpr float NEG_BIG = -1.0e30f;

template <class T, int HD>
__global__ __launch_bounds__(256) void k_attn_partial(AttnArgs a) {
  constexpr int KK = HD / 32, HT = HD / 16;
  const int lane = threadIdx.x & 63;
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (unit >= a.B * a.H * a.NC) return;
  const int c = unit % a.NC, bh = unit / a.NC, hh = bh % a.H, b = bh / a.H;
  const int j = lane & 15, g = lane >> 4, r = j;
  const int d = a.H * HD;
  const int m_row = b * a.q_rows + min(j, a.q_rows - 1);
  const int pos_j = (j < a.q_rows) ? a.row_pos[b * a.q_rows + j] : -1;
  int pmax = pos_j;
#pragma unroll
  for (int o = 1; o <= 8; o <<= 1) pmax = max(pmax, __shfl_xor(pmax, o, 64));
  const int k0 = c * ATTN_CHUNK;
  if (k0 > pmax) return;  // same for the whole wave
  const int kend = min(k0 + ATTN_CHUNK, pmax + 1);
  const float scale = rsqrtf((float)HD);

  u32x4_v qf[KK];
  const T *qrow = (const T *)a.q + (size_t)m_row * d + (size_t)hh * HD;
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) qf[kk] = *(const u32x4_v *)(qrow + kk * 32 + 8 * g);

  const T *kbase = (const T *)a.kc + (size_t)bh * a.L_pad * HD;
  const T *vbase = (const T *)a.vc + (size_t)bh * (a.L_pad / KV_VBLOCK) * HD * KV_VBLOCK;

  float m_run = NEG_BIG, l_run = 0.f;
  f32x4_v acc[HT];
#pragma unroll
  for (int ht = 0; ht < HT; ++ht) acc[ht] = (f32x4_v){0.f, 0.f, 0.f, 0.f};

  for (int ks = k0; ks < kend; ks += 32) {
    // key rows of the two score tiles (see the permutation in the header comment)
    const T *kr0 = kbase + (size_t)(ks + 8 * (r >> 2) + (r & 3)) * HD + 8 * g;
    const T *kr1 = kr0 + 4 * HD;
    u32x4_v kf0[KK], kf1[KK], vf[HT];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      kf0[kk] = *(const u32x4_v *)(kr0 + kk * 32);
      kf1[kk] = *(const u32x4_v *)(kr1 + kk * 32);
    }
    const T *vr = vbase + ((size_t)(ks / KV_VBLOCK + g) * HD + r) * KV_VBLOCK;
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) vf[ht] = *(const u32x4_v *)(vr + (size_t)ht * 16 * KV_VBLOCK);

    f32x4_v s0 = (f32x4_v){0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      s0 = MfmaA<T>::run(kf0[kk], qf[kk], s0);
      s1 = MfmaA<T>::run(kf1[kk], qf[kk], s1);
    }
    // lane (query j, group g): s0[i] <-> key ks + 8g + i, s1[i] <-> key ks + 8g + 4 + i
    float sv[8];
    const int kfirst = ks + 8 * g;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      sv[i] = (kfirst + i <= pos_j) ? s0[i] : NEG_BIG;
      sv[4 + i] = (kfirst + 4 + i <= pos_j) ? s1[i] : NEG_BIG;
    }
    float smax = sv[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) smax = fmaxf(smax, sv[i]);
    smax = fmaxf(smax, __shfl_xor(smax, 16, 64));
    smax = fmaxf(smax, __shfl_xor(smax, 32, 64));
    const float m_new = fmaxf(m_run, smax);
    const float corr = __expf((m_run - m_new) * scale);
    float p[8];
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float e = (sv[i] > 0.5f * NEG_BIG) ? __expf((sv[i] - m_new) * scale) : 0.f;
      p[i] = Conv<T>::round(e);  // the product below sees the rounded weight; sum the same value
      psum += p[i];
    }
    psum += __shfl_xor(psum, 16, 64);
    psum += __shfl_xor(psum, 32, 64);
    l_run = l_run * corr + psum;
    m_run = m_new;
    u32x4_v pf;
    pf[0] = MfmaA<T>::pack2(p[0], p[1]);
    pf[1] = MfmaA<T>::pack2(p[2], p[3]);
    pf[2] = MfmaA<T>::pack2(p[4], p[5]);
    pf[3] = MfmaA<T>::pack2(p[6], p[7]);
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) {
      acc[ht][0] *= corr; acc[ht][1] *= corr; acc[ht][2] *= corr; acc[ht][3] *= corr;
      acc[ht] = MfmaA<T>::run(vf[ht], pf, acc[ht]);
    }
  }

  if (j < a.q_rows && pos_j >= k0) {
    const size_t slot = ((size_t)(b * a.q_rows + j) * a.H + hh) * a.NC + c;
    if (g == 0) { a.part_ml[slot * 2] = m_run; a.part_ml[slot * 2 + 1] = l_run; }
    float *pa = a.part_acc + slot * HD + 4 * g;
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) *(f32x4_v *)(pa + ht * 16) = acc[ht];
  }
}

// Merge of the chunk partials of one (row, head) in ascending chunk order.
template <class T, int HD>
__global__ void k_attn_combine(AttnArgs a) {
  const int m = blockIdx.x, hh = blockIdx.y, e = threadIdx.x;
  const int d = a.H * HD;
  const int pos = a.row_pos[m];
  T *out = (T *)a.out + (size_t)m * d + (size_t)hh * HD;
  if (pos < 0) { Conv<T>::st(out, e, 0.f); return; }
  const int nc = pos / ATTN_CHUNK + 1;
  const size_t slot0 = ((size_t)m * a.H + hh) * a.NC;
  const float scale = rsqrtf((float)HD);
  float mx = a.part_ml[slot0 * 2];
  for (int c = 1; c < nc; ++c) mx = fmaxf(mx, a.part_ml[(slot0 + c) * 2]);
  float den = 0.f, num = 0.f;
  for (int c = 0; c < nc; ++c) {
    const float wgt = __expf((a.part_ml[(slot0 + c) * 2] - mx) * scale);
    den += a.part_ml[(slot0 + c) * 2 + 1] * wgt;
    num += a.part_acc[(slot0 + c) * HD + e] * wgt;
  }
  Conv<T>::st(out, e, num / den);
}

template <class T>
static void launch_attn_t(const AttnArgs &a, hipStream_t st) {
  const int M = a.B * a.q_rows;
  if (M <= 0) return;
  const int units = a.B * a.H * a.NC;
  if (a.hd == 128) {
    hipLaunchKernelGGL((k_attn_partial<T, 128>), dim3((units + 3) / 4), dim3(256), 0, st, a);
    hipLaunchKernelGGL((k_attn_combine<T, 128>), dim3(M, a.H), dim3(128), 0, st, a);
  } else {
    hipLaunchKernelGGL((k_attn_partial<T, 64>), dim3((units + 3) / 4), dim3(256), 0, st, a);
    hipLaunchKernelGGL((k_attn_combine<T, 64>), dim3(M, a.H), dim3(64), 0, st, a);
  }
}

void launch_attention_mfma(int dtype, const AttnArgs &a, hipStream_t st) {
  if (dtype == SPEC_DTYPE_BF16) launch_attn_t<bf16_t>(a, st);
  else launch_attn_t<f16_t>(a, st);
}

}  // namespace spec
