// Verification attention on the matrix cores: the (up to 16) new query rows of one
// sequence against that sequence's KV cache, causal among the new rows.
//
// HBM-bound on the cache (a handful of flops per cached byte), so the layout is built
// around the loads: keys stream in as full rows (256 bytes at head_dim 128), values as
// 16-byte runs of 8 consecutive positions, and the next 32-key step is in flight while
// the current one is computed.
//
// Transposed formulation, so that scores never move between lanes:
//   S^T[key][query]  = K . Q^T     A operand = 16 key rows,  B operand = 16 query rows
//   O^T[dim][query] += V^T . P^T   A operand = V^T (16 dims x 32 keys), B operand = P^T
// The accumulator layout of the first product (lane = query column, 4 consecutive keys per
// lane and tile) is already the B-operand layout of the second once the key rows fed to
// the first product are permuted: tile t, row 4g'+i carries key ks + 8g' + 4t + i.
//
// Numerics depend on (sequence, absolute positions) only.  The cache is cut into chunks of
// 256 positions starting at multiples of 256.  Each chunk yields a fresh partial (running
// maximum, sum, un-normalised output) from an online softmax over ascending 32-key steps;
// the partials are merged pairwise in ascending chunk order.  Masked keys contribute exact
// zeros and leave the running maximum unchanged, and merging an all-masked partial is an
// exact no-op, so neither the other rows of a pass nor the launch shape change a row's
// bits.  Two launch shapes compute exactly that: one wave per (sequence, head, chunk) with
// the partials merged by a second kernel (few sequences: parallelism over chunks), or one
// wave per (sequence, head) walking its chunks and merging in registers (many sequences:
// no partial traffic).
#include "spec_internal.h"
#include "device_utils.h"
#include "mfma_gemm.h"

// No implicit fusing of multiplies and adds: which product a compiler folds into an FMA can
// differ between two instantiations of the same source, and results here must be bit-identical
// across launch shapes.  Fused operations are written out with fmaf where they are wanted.
#pragma clang fp contract(off)

namespace spec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_v;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_v;
typedef __attribute__((ext_vector_type(4))) float f32x4_v;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_v;

template <class T> struct MfmaA;
template <> struct MfmaA<bf16_t> {
  static constexpr bool HILO = true;   // queries and softmax weights as a bf16 pair (value + remainder): 16 significant bits
  static __device__ __forceinline__ f32x4_v run(u32x4_v a, u32x4_v b, f32x4_v c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_v, a), __builtin_bit_cast(bf16x8_v, b), c,
                                                   0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
  }
};
template <> struct MfmaA<f16_t> {
  static constexpr bool HILO = false;  // one fp16 word has 11 significant bits: enough
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
constexpr float LOG2E = 1.4426950408889634f;

// exp((a - b) * scale) with the scale pre-multiplied by log2(e): one subtraction, one
// multiplication, one hardware exp2 -- nothing the optimiser may legally rearrange, so every
// kernel that uses it produces the same bits.
__device__ __forceinline__ float exp_diff(float a, float b, float sl2) {
  return __builtin_amdgcn_exp2f((a - b) * sl2);
}

// (m, l, acc) <- (m, l, acc) (+) (mc, lc, accc): the one merge rule, used by both launch shapes.
__device__ __forceinline__ void merge_weights(float m, float mc, float scale, float &m_new, float &wa, float &wb) {
  m_new = fmaxf(m, mc);
  wa = exp_diff(m, m_new, scale);
  wb = exp_diff(mc, m_new, scale);
}
__device__ __forceinline__ float merge_value(float a, float wa, float b, float wb) { return fmaf(a, wa, b * wb); }

// The query fragments of a wave: row j's elements 32 kk + 8 g .. + 7 of the head, from the fp32 queries the QKV
// epilogue left.  bf16 caches: hi = bf16(q), lo = bf16(q - hi), both multiplied with every key fragment (the cache
// streams from HBM and the matrix pipes idle, so the second product is free), which takes the query's rounding
// out of the scores.
template <class T, int HD> struct QFrags {
  u32x4_v hi[HD / 32], lo[MfmaA<T>::HILO ? HD / 32 : 1];
};
template <class T, int HD>
__device__ __forceinline__ void load_q(QFrags<T, HD> &qf, const float *qrow, int g) {
#pragma unroll
  for (int kk = 0; kk < HD / 32; ++kk) {
    const float4 a = *(const float4 *)(qrow + kk * 32 + 8 * g), b = *(const float4 *)(qrow + kk * 32 + 8 * g + 4);
    const float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    float r[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = Conv<T>::round(x[i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) qf.hi[kk][i] = MfmaA<T>::pack2(r[2 * i], r[2 * i + 1]);
    if (MfmaA<T>::HILO) {
#pragma unroll
      for (int i = 0; i < 4; ++i) qf.lo[kk][i] = MfmaA<T>::pack2(x[2 * i] - r[2 * i], x[2 * i + 1] - r[2 * i + 1]);
    }
  }
}

template <int HD> struct Frags {
  u32x4_v k0[HD / 32], k1[HD / 32], v[HD / 16];
};

// STREAM: non-temporal loads.  With many sequences the cache rows of a pass are a pure stream, read once
// (measured on MI355X: 13 % faster at 64 sequences); the few long waves of a small batch were faster with
// plain loads.
template <class T, int HD, bool STREAM>
__device__ __forceinline__ void load_step(Frags<HD> &f, const T *kbase, const T *vbase, int ks, int r, int g) {
  auto ld = [](const u32x4_v *p) { return STREAM ? __builtin_nontemporal_load(p) : *p; };
  const T *kr0 = kbase + (size_t)(ks + 8 * (r >> 2) + (r & 3)) * HD + 8 * g;
  const T *kr1 = kr0 + 4 * HD;
#pragma unroll
  for (int kk = 0; kk < HD / 32; ++kk) {
    f.k0[kk] = ld((const u32x4_v *)(kr0 + kk * 32));
    f.k1[kk] = ld((const u32x4_v *)(kr1 + kk * 32));
  }
  const T *vr = vbase + ((size_t)(ks / KV_VBLOCK + g) * HD + r) * KV_VBLOCK;
#pragma unroll
  for (int ht = 0; ht < HD / 16; ++ht) f.v[ht] = ld((const u32x4_v *)(vr + (size_t)ht * 16 * KV_VBLOCK));
}

// One 32-key step of the online softmax for the 16 query columns of the wave.
template <class T, int HD>
__device__ __forceinline__ void compute_step(const Frags<HD> &f, const QFrags<T, HD> &qf, int ks, int g,
                                             int pos_j, float scale, float &m_run, float &l_run,
                                             f32x4_v (&acc)[HD / 16]) {
  f32x4_v s0 = (f32x4_v){0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
  for (int kk = 0; kk < HD / 32; ++kk) {
    s0 = MfmaA<T>::run(f.k0[kk], qf.hi[kk], s0);
    s1 = MfmaA<T>::run(f.k1[kk], qf.hi[kk], s1);
  }
  if (MfmaA<T>::HILO) {
#pragma unroll
    for (int kk = 0; kk < HD / 32; ++kk) {
      s0 = MfmaA<T>::run(f.k0[kk], qf.lo[kk], s0);
      s1 = MfmaA<T>::run(f.k1[kk], qf.lo[kk], s1);
    }
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
  const float corr = exp_diff(m_run, m_new, scale);
  // The products below see the weight rounded to the cache's type -- for bf16 as a pair (value + remainder, both
  // multiplied with the value fragments) -- and the denominator sums exactly what they see.
  float p[8], plo[8];
  float psum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float e = (sv[i] > 0.5f * NEG_BIG) ? exp_diff(sv[i], m_new, scale) : 0.f;
    p[i] = Conv<T>::round(e);
    if (MfmaA<T>::HILO) {
      plo[i] = Conv<T>::round(e - p[i]);
      psum += p[i] + plo[i];  // 16 significant bits: exact in fp32
    } else {
      psum += p[i];
    }
  }
  psum += __shfl_xor(psum, 16, 64);
  psum += __shfl_xor(psum, 32, 64);
  l_run = fmaf(l_run, corr, psum);
  m_run = m_new;
  u32x4_v pf, pfl;
#pragma unroll
  for (int i = 0; i < 4; ++i) pf[i] = MfmaA<T>::pack2(p[2 * i], p[2 * i + 1]);
  if (MfmaA<T>::HILO) {
#pragma unroll
    for (int i = 0; i < 4; ++i) pfl[i] = MfmaA<T>::pack2(plo[2 * i], plo[2 * i + 1]);
  }
#pragma unroll
  for (int ht = 0; ht < HD / 16; ++ht) {
    acc[ht][0] *= corr; acc[ht][1] *= corr; acc[ht][2] *= corr; acc[ht][3] *= corr;
    acc[ht] = MfmaA<T>::run(f.v[ht], pf, acc[ht]);
    if (MfmaA<T>::HILO) acc[ht] = MfmaA<T>::run(f.v[ht], pfl, acc[ht]);
  }
}

// Fresh partial of the chunk [k0, kend): steps of 32 keys, next step's loads in flight.
template <class T, int HD, bool STREAM>
__device__ __forceinline__ void chunk_partial(const T *kbase, const T *vbase, const QFrags<T, HD> &qf, int k0,
                                              int kend, int r, int g, int pos_j, float scale, float &m_run,
                                              float &l_run, f32x4_v (&acc)[HD / 16]) {
  m_run = NEG_BIG;
  l_run = 0.f;
#pragma unroll
  for (int ht = 0; ht < HD / 16; ++ht) acc[ht] = (f32x4_v){0.f, 0.f, 0.f, 0.f};
  // Steps in pairs; inside the loop every load is unconditional, so the wait in front of a step can leave exactly
  // the next step's loads in flight (a load behind a branch makes the compiler wait for everything at the join).
  Frags<HD> fa, fb;
  load_step<T, HD, STREAM>(fa, kbase, vbase, k0, r, g);
  const int klast = k0 + ((kend - k0 - 1) & ~31);  // where the chunk's last step starts
  int ks = k0;
  while (ks + 64 <= klast) {  // steps ks and ks + 32, and a step behind them to prefetch
    load_step<T, HD, STREAM>(fb, kbase, vbase, ks + 32, r, g);
    compute_step<T, HD>(fa, qf, ks, g, pos_j, scale, m_run, l_run, acc);
    load_step<T, HD, STREAM>(fa, kbase, vbase, ks + 64, r, g);
    compute_step<T, HD>(fb, qf, ks + 32, g, pos_j, scale, m_run, l_run, acc);
    ks += 64;
  }
  if (ks + 32 <= klast) {  // two steps left
    load_step<T, HD, STREAM>(fb, kbase, vbase, ks + 32, r, g);
    compute_step<T, HD>(fa, qf, ks, g, pos_j, scale, m_run, l_run, acc);
    compute_step<T, HD>(fb, qf, ks + 32, g, pos_j, scale, m_run, l_run, acc);
  } else {                 // one
    compute_step<T, HD>(fa, qf, ks, g, pos_j, scale, m_run, l_run, acc);
  }
}

struct WaveSetup {
  int j, g, pos_j, pmax, m_row;
};
__device__ __forceinline__ WaveSetup wave_setup(const AttnArgs &a, int b, int lane) {
  WaveSetup w;
  w.j = lane & 15;
  w.g = lane >> 4;
  w.m_row = b * a.q_rows + min(w.j, a.q_rows - 1);
  w.pos_j = (w.j < a.q_rows) ? a.row_pos[b * a.q_rows + w.j] : -1;
  int pmax = w.pos_j;
#pragma unroll
  for (int o = 1; o <= 8; o <<= 1) pmax = max(pmax, __shfl_xor(pmax, o, 64));
  w.pmax = pmax;
  return w;
}

// Launch shape 1: one wave per (sequence, head, chunk); partials go to the workspace.
template <class T, int HD, bool STREAM>
__global__ __launch_bounds__(256) void k_attn_split(AttnArgs a) {
  constexpr int HT = HD / 16;
  const int lane = threadIdx.x & 63;
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (unit >= a.B * a.H * a.NC) return;
  const int c = unit % a.NC, bh = unit / a.NC, hh = bh % a.H, b = bh / a.H;
  const WaveSetup w = wave_setup(a, b, lane);
  const int k0 = attn_chunk_begin(c);
  if (k0 > w.pmax) return;  // same for the whole wave
  const int kend = min(attn_chunk_begin(c + 1), w.pmax + 1);
  const float scale = rsqrtf((float)HD) * LOG2E;  // score scale in base-2 exponent units
  const int d = a.H * HD;
  QFrags<T, HD> qf;
  load_q<T, HD>(qf, (const float *)a.q + (size_t)w.m_row * d + (size_t)hh * HD, w.g);
  const size_t cbh = a.seq_groups > 1 ? (size_t)(b / a.seq_groups) * a.H + hh : (size_t)bh;  // whose cache: the group's sequence
  const T *kbase = (const T *)a.kc + cbh * a.L_pad * HD;
  const T *vbase = (const T *)a.vc + cbh * (a.L_pad / KV_VBLOCK) * HD * KV_VBLOCK;
  float m_run, l_run;
  f32x4_v acc[HT];
  chunk_partial<T, HD, STREAM>(kbase, vbase, qf, k0, kend, w.j, w.g, w.pos_j, scale, m_run, l_run, acc);
  if (w.j < a.q_rows && w.pos_j >= k0) {
    const size_t slot = ((size_t)(b * a.q_rows + w.j) * a.H + hh) * a.NC + c;
    if (w.g == 0) { a.part_ml[slot * 2] = m_run; a.part_ml[slot * 2 + 1] = l_run; }
    float *pa = a.part_acc + slot * HD + 4 * w.g;
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) *(f32x4_v *)(pa + ht * 16) = acc[ht];
  }
}

// Merge of the chunk partials of one (row, head), ascending.
template <class T, int HD>
__global__ void k_attn_merge(AttnArgs a) {
  const int m = blockIdx.x, hh = blockIdx.y, e = threadIdx.x;
  const int d = a.H * HD;
  const int pos = a.row_pos[m];
  const size_t at = xpack_index(m, hh * HD + e, d >> 5);
  op_t *out = (op_t *)a.out + at;
  if (pos < 0) { *out = (op_t)0.f; return; }
  const int nc = attn_chunk_of(pos) + 1;
  const size_t slot0 = ((size_t)m * a.H + hh) * a.NC;
  const float scale = rsqrtf((float)HD) * LOG2E;  // score scale in base-2 exponent units
  float mr = a.part_ml[slot0 * 2], lr = a.part_ml[slot0 * 2 + 1], ar = a.part_acc[slot0 * HD + e];
  for (int c = 1; c < nc; ++c) {
    float mn, wa, wb;
    merge_weights(mr, a.part_ml[(slot0 + c) * 2], scale, mn, wa, wb);
    lr = merge_value(lr, wa, a.part_ml[(slot0 + c) * 2 + 1], wb);
    ar = merge_value(ar, wa, a.part_acc[(slot0 + c) * HD + e], wb);
    mr = mn;
  }
  const float res = ar * (1.0f / lr);
  *out = to_op(res);
}

// Launch shape 2: one wave per (sequence, head) walks all chunks, merging in registers.
template <class T, int HD>
__global__ __launch_bounds__(256) void k_attn_seq(AttnArgs a) {  // launched with 64: the bound only keeps the register budget
  constexpr int HT = HD / 16;
  const int lane = threadIdx.x & 63;
  const int bh = blockIdx.x;  // a workgroup is one wave
  if (bh >= a.B * a.H) return;
  const int hh = bh % a.H, b = bh / a.H;
  const WaveSetup w = wave_setup(a, b, lane);
  const int d = a.H * HD;
  const float scale = rsqrtf((float)HD) * LOG2E;  // score scale in base-2 exponent units
  QFrags<T, HD> qf;
  load_q<T, HD>(qf, (const float *)a.q + (size_t)w.m_row * d + (size_t)hh * HD, w.g);
  const size_t cbh = a.seq_groups > 1 ? (size_t)(b / a.seq_groups) * a.H + hh : (size_t)bh;  // whose cache: the group's sequence
  const T *kbase = (const T *)a.kc + cbh * a.L_pad * HD;
  const T *vbase = (const T *)a.vc + cbh * (a.L_pad / KV_VBLOCK) * HD * KV_VBLOCK;
  float mr = NEG_BIG, lr = 0.f;
  f32x4_v ar[HT];
#pragma unroll
  for (int ht = 0; ht < HT; ++ht) ar[ht] = (f32x4_v){0.f, 0.f, 0.f, 0.f};
  for (int c = 0, k0 = 0; k0 <= w.pmax; k0 = attn_chunk_begin(++c)) {
    const int kend = min(attn_chunk_begin(c + 1), w.pmax + 1);
    float mc, lc;
    f32x4_v ac[HT];
    chunk_partial<T, HD, true>(kbase, vbase, qf, k0, kend, w.j, w.g, w.pos_j, scale, mc, lc, ac);
    if (k0 == 0) {
      mr = mc; lr = lc;
#pragma unroll
      for (int ht = 0; ht < HT; ++ht) ar[ht] = ac[ht];
    } else {
      float mn, wa, wb;
      merge_weights(mr, mc, scale, mn, wa, wb);
      lr = merge_value(lr, wa, lc, wb);
#pragma unroll
      for (int ht = 0; ht < HT; ++ht)
#pragma unroll
        for (int i = 0; i < 4; ++i) ar[ht][i] = merge_value(ar[ht][i], wa, ac[ht][i], wb);
      mr = mn;
    }
  }
  if (w.j < a.q_rows) {
    const int m = b * a.q_rows + w.j;
    const float inv = (w.pos_j >= 0) ? 1.0f / lr : 0.f;
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) {
      op_t o4[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) o4[i] = to_op(w.pos_j >= 0 ? ar[ht][i] * inv : 0.f);
      const size_t at = xpack_index(m, hh * HD + ht * 16 + 4 * w.g, d >> 5);
      *(uint2 *)((op_t *)a.out + at) = *(const uint2 *)o4;
    }
  }
}

// Launch shape 3: one workgroup per (sequence, head) with one wave per chunk; the partials meet in LDS and are
// merged there in ascending chunk order, the head-dimension tiles dealt to the waves.  The same partials and the
// same merge arithmetic as the other two shapes, without the merge launch and the partials' trip through memory:
// for the few sequences of a small batch, where the attention is a chain of load latencies.
template <class T, int HD, bool STREAM>
__global__ __launch_bounds__(512) void k_attn_group(AttnArgs a) {
  constexpr int HT = HD / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char attn_smem[];  // [NC][HT][64] f32x4, then [NC][64] (max, sum)
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, W = blockDim.x >> 6;
  const int bh = blockIdx.x, hh = bh % a.H, b = bh / a.H;
  const WaveSetup w = wave_setup(a, b, lane);
  const int d = a.H * HD;
  const float scale = rsqrtf((float)HD) * LOG2E;  // score scale in base-2 exponent units
  QFrags<T, HD> qf;
  load_q<T, HD>(qf, (const float *)a.q + (size_t)w.m_row * d + (size_t)hh * HD, w.g);
  const size_t cbh = a.seq_groups > 1 ? (size_t)(b / a.seq_groups) * a.H + hh : (size_t)bh;  // whose cache: the group's sequence
  const T *kbase = (const T *)a.kc + cbh * a.L_pad * HD;
  const T *vbase = (const T *)a.vc + cbh * (a.L_pad / KV_VBLOCK) * HD * KV_VBLOCK;
  f32x4_v *pacc = (f32x4_v *)attn_smem;
  float2 *pml = (float2 *)(attn_smem + (size_t)a.NC * HT * 64 * sizeof(f32x4_v));
  for (int c = wv; c < a.NC; c += W) {
    const int k0 = attn_chunk_begin(c);
    if (k0 > w.pmax) break;  // same for the whole wave; no row of the sequence reaches this chunk or a later one
    const int kend = min(attn_chunk_begin(c + 1), w.pmax + 1);
    float mc, lc;
    f32x4_v ac[HT];
    chunk_partial<T, HD, STREAM>(kbase, vbase, qf, k0, kend, w.j, w.g, w.pos_j, scale, mc, lc, ac);
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) pacc[(c * HT + ht) * 64 + lane] = ac[ht];
    pml[c * 64 + lane] = make_float2(mc, lc);
  }
  __syncthreads();
  // row j needs the chunks up to its own position; every one of them was computed (pmax >= pos_j)
  const int nc = w.pos_j >= 0 ? attn_chunk_of(w.pos_j) + 1 : 0;
  if (w.j >= a.q_rows) return;
  const int m = b * a.q_rows + w.j;
  for (int ht = wv; ht < HT; ht += W) {
    float mr = 0.f, lr = 1.f;
    f32x4_v ar = (f32x4_v){0.f, 0.f, 0.f, 0.f};
    if (nc > 0) {
      const float2 ml0 = pml[lane];
      mr = ml0.x; lr = ml0.y;
      ar = pacc[ht * 64 + lane];
      for (int c = 1; c < nc; ++c) {
        const float2 mlc = pml[c * 64 + lane];
        const f32x4_v ac = pacc[(c * HT + ht) * 64 + lane];
        float mn, wa, wb;
        merge_weights(mr, mlc.x, scale, mn, wa, wb);
        lr = merge_value(lr, wa, mlc.y, wb);
#pragma unroll
        for (int i = 0; i < 4; ++i) ar[i] = merge_value(ar[i], wa, ac[i], wb);
        mr = mn;
      }
    }
    const float inv = nc > 0 ? 1.0f / lr : 0.f;
    op_t o4[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) o4[i] = to_op(nc > 0 ? ar[i] * inv : 0.f);
    const size_t at = xpack_index(m, hh * HD + ht * 16 + 4 * w.g, d >> 5);
    *(uint2 *)((op_t *)a.out + at) = *(const uint2 *)o4;
  }
}

constexpr size_t attn_group_lds(int HD, int NC) { return (size_t)NC * ((HD / 16) * 64 * 16 + 64 * 8); }

template <class T, int HD, bool STREAM>
static void launch_attn_group(const AttnArgs &a, int pairs, hipStream_t st) {
  const int waves = a.NC < ATTN_GROUP_MAX_WAVES ? a.NC : ATTN_GROUP_MAX_WAVES;
  hipLaunchKernelGGL((k_attn_group<T, HD, STREAM>), dim3(pairs), dim3(64 * waves), attn_group_lds(HD, a.NC), st, a);
}
template <class T, int HD>
static void prepare_attn_group() {  // more than the default 64 KB of LDS has to be asked for
  const int lds = (int)attn_group_lds(HD, ATTN_GROUP_MAX_CHUNKS);
  (void)hipFuncSetAttribute((const void *)k_attn_group<T, HD, true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  (void)hipFuncSetAttribute((const void *)k_attn_group<T, HD, false>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}
void attention_prepare() {
  prepare_attn_group<bf16_t, 128>(); prepare_attn_group<bf16_t, 64>();
  prepare_attn_group<f16_t, 128>(); prepare_attn_group<f16_t, 64>();
}

template <class T, int HD>
static void launch_attn_hd(const AttnArgs &a, hipStream_t st) {
  const int M = a.B * a.q_rows;
  const int pairs = a.B * a.H;
  // One wave per (sequence, head) once there are enough pairs to fill the chip -- unless they leave the last of
  // several rounds of n_cu * 4 waves mostly empty: a compute unit's share of the HBM stream is bounded, so the
  // units that hold a second workgroup take twice as long as the others.  Measured (us per layer): 512 cached
  // positions x 32 heads, a workgroup per pair as the alternative: 33 sequences 86 against 64, 48 sequences 92
  // against 81, 32 and 64 sequences 53 and 101 against 57 and 104; 2048 positions x 52 heads, where the alternative
  // was split + merge: 20 sequences 299 against 242, 24 sequences 305 against 287, 32 sequences 326 against 378.
  const int slots = (a.n_cu > 0 ? a.n_cu : 256) * 4, rounds = (pairs + slots - 1) / slots;
  // ... with a wave per chunk, or every eighth chunk per wave -- unless the waves of the split shape all find a slot at
  // once: then their shorter chains win (one sequence x 32 heads x 2048 positions: 20.9 us against 26.5)
  const bool group_fits = a.NC <= ATTN_GROUP_MAX_WAVES || (a.NC <= ATTN_GROUP_MAX_CHUNKS && pairs * a.NC > slots);
  // (2048 positions x 52 heads, the workgroup shape with its waves at two chunks each as the alternative: 28 sequences
  // 303 against 276 us, 32 sequences 312 against 318)
  const double full = !group_fits ? 0.7 : a.NC <= ATTN_GROUP_MAX_WAVES ? 0.85 : 0.8;
  const bool fills = rounds == 1 || (double)pairs >= full * (double)rounds * slots;
  const bool seq = a.shape == 2 || (a.shape == 0 && ((pairs >= ATTN_SEQ_MIN_PAIRS && fills) || a.NC == 1));
  // few sequences: a workgroup per (sequence, head), as long as its partials fit into LDS with a wave per chunk
  const bool group = !seq && (a.shape == 3 || a.shape == 0) && group_fits;
  if (seq) {
    // workgroups of one wave: few pairs then spread over all compute units (measured, us per layer at 32 heads: 4
    // sequences x 100 positions 15.1 -> 11.8, 24 x 250 29.6 -> 26.6), and many pairs drain evenly (64 sequences x 300
    // positions 72.5 -> 71.4 against workgroups of four waves; 32 sequences x 52 heads x 2048 positions: the same)
    hipLaunchKernelGGL((k_attn_seq<T, HD>), dim3(pairs), dim3(64), 0, st, a);
  } else if (group) {
    if (pairs * a.NC >= ATTN_STREAM_MIN_WAVES) launch_attn_group<T, HD, true>(a, pairs, st);
    else launch_attn_group<T, HD, false>(a, pairs, st);
  } else {
    if (pairs * a.NC >= ATTN_STREAM_MIN_WAVES)  // enough waves that the cache rows are a stream (measured)
      hipLaunchKernelGGL((k_attn_split<T, HD, true>), dim3((pairs * a.NC + 3) / 4), dim3(256), 0, st, a);
    else
      hipLaunchKernelGGL((k_attn_split<T, HD, false>), dim3((pairs * a.NC + 3) / 4), dim3(256), 0, st, a);
    hipLaunchKernelGGL((k_attn_merge<T, HD>), dim3(M, a.H), dim3(HD), 0, st, a);
  }
}

template <class T>
static void launch_attn_t(const AttnArgs &a, hipStream_t st) {
  if (a.B * a.q_rows <= 0) return;
  if (a.hd == 128) launch_attn_hd<T, 128>(a, st);
  else launch_attn_hd<T, 64>(a, st);
}

void launch_attention_mfma(int dtype, const AttnArgs &a, hipStream_t st) {
  if (dtype == SPEC_DTYPE_BF16) launch_attn_t<bf16_t>(a, st);
  else launch_attn_t<f16_t>(a, st);
}

}  // namespace spec
