// Weight-streaming GEMMs on the matrix cores (fp16 operands, fp32 accumulate) with the
// layer's element-wise work fused into the epilogue.
//
//   Y^T[n][m] = sum_k W[n][k] * X[m][k]        W: weights [N][K], X: activations [M][K]
//
// One instruction, v_mfma_f32_16x16x32_f16, everywhere: the weight tile is the A operand
// (16 output features x 32 k), the activation tile the B operand (16 rows x 32 k).  bf16
// models run on it too: their weights become fp16 times a power of two per matrix (exact
// for all but vanishing elements), their activations are rounded from fp32 to fp16, which
// keeps three more bits than bf16 would.
//
// Packed weights.  Each 16x32 tile is stored as the 1 KB a wave loads with one 16-byte load
// per lane: lane L = 16*g + r holds W[n0 + r][k0 + 8g .. k0 + 8g + 7].  Tiles of one
// 16-row strip are contiguous in k, strips follow each other, so a wave streams its strip
// slice as one linear run of HBM addresses.
//
// Numerics are a function of the weight shape only.  K is cut into KS equal slices (KS =
// 8, 4, 2 or 1, the largest that divides K/32).  Every output element is
//     (((P_0 + P_1) + P_2) + ... + P_{KS-1}) (+ bias)
// where P_w is the chain of MFMAs over slice w in ascending k, starting from zero.  Neither
// the number of rows M, nor a row's index, nor the tiling chosen for a given M changes
// that order, so a sequence's results are bit-identical at every batch size and
// speculation length.
#include "spec_internal.h"
#include "device_utils.h"
#include "mfma_gemm.h"
#include "mfma_tiles.h"
#include <algorithm>
#include <type_traits>

// No implicit fusing of multiplies and adds: which product a compiler folds into an FMA can
// differ between two instantiations of the same source, and results here must be bit-identical
// across launch shapes.  Fused operations are written out with fmaf where they are wanted.
#pragma clang fp contract(off)

namespace spec {

// ------------------------------------------------------------------------- packing
// Largest magnitude of a tensor as an fp32 bit pattern (atomic max over non-negative floats
// ordered as integers).
template <class T>
__global__ void k_absmax(const T *__restrict__ s, size_t n, int K, const T *__restrict__ gain, uint32_t *__restrict__ out) {
  float m = 0.f;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    float v = fabsf(Conv<T>::ld(s, i));
    if (gain) v *= fabsf(Conv<T>::ld(gain, i % (size_t)K));
    if (v < INFINITY) m = fmaxf(m, v);
  }
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) atomicMax(out, __float_as_uint(m));
}
void launch_absmax(int dtype, const void *src, size_t n, int K, const void *gain, uint32_t *d_amax_bits, hipStream_t st) {
  if (!src || n == 0) return;
  const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, 2048);
  if (dtype == SPEC_DTYPE_BF16)
    hipLaunchKernelGGL(k_absmax<bf16_t>, dim3(blocks), dim3(256), 0, st, (const bf16_t *)src, n, K, (const bf16_t *)gain, d_amax_bits);
  else
    hipLaunchKernelGGL(k_absmax<f16_t>, dim3(blocks), dim3(256), 0, st, (const f16_t *)src, n, K, (const f16_t *)gain, d_amax_bits);
}

// mode 0: rows of one matrix in natural order
// mode 1: q | k | v stacked; inside every head the q and k rows are pair-interleaved
//         (stored row 2i <- canonical i, 2i+1 <- i + hd/2) so a rotary pair is lane-local
// mode 2: gate / up interleaved: stored rows 4p.. = gate[2p], up[2p], gate[2p+1], up[2p+1]
// Elements are written as fp16(weight * gain[k] * scale): gain the folded norm gain of column k (1 without
// gain), scale the matrix's power of two (1 without amax_bits).  The product of two 16-bit values is exact
// in fp32, the scaling too: one rounding per element.
template <class T>
__global__ void k_pack_weight(int mode, int N, int K, int N_pad, int K_pad, int d, int hd, const T *__restrict__ s0,
                              const T *__restrict__ s1, const T *__restrict__ s2, const T *__restrict__ gain,
                              op_t *__restrict__ dst, const uint32_t *__restrict__ amax_bits) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // one thread per 8 packed elements
  const int KT = K_pad / 32;
  const size_t total = (size_t)(N_pad / 16) * KT * 64;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const size_t tile = idx >> 6;
  const int kt = (int)(tile % KT), nt = (int)(tile / KT);
  const int r = lane & 15, g = lane >> 4;
  const int n = nt * 16 + r, k0 = kt * 32 + g * 8;
  const T *src = nullptr;
  int row = 0;
  if (n < N) {
    if (mode == 0) { src = s0; row = n; }
    else if (mode == 1) {
      int region = n / d, c = n % d, hh = c / hd, e = c % hd;
      if (region < 2) { int half = hd >> 1; e = (e & 1) ? (e >> 1) + half : (e >> 1); }
      src = region == 0 ? s0 : region == 1 ? s1 : s2;
      row = hh * hd + e;
    } else {
      int p = n >> 2, q = n & 3;
      src = (q & 1) ? s1 : s0;
      row = 2 * p + (q >> 1);
    }
  }
  const float scale = amax_bits ? weight_scale(*amax_bits) : 1.0f;
  op_t out[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
    out[i] = (src && k0 + i < K)
                 ? (op_t)(Conv<T>::ld(src, (size_t)row * K + k0 + i) * (gain ? Conv<T>::ld(gain, k0 + i) : 1.0f) * scale)
                 : (op_t)0.f;
  op_t *o = dst + idx * 8;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = out[i];
}

template <class T>
__global__ void k_pack_bias(int mode, int N, int N_pad, int d, int hd, const T *__restrict__ s0,
                            const T *__restrict__ s1, const T *__restrict__ s2, float *__restrict__ dst) {
  int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N_pad) return;
  float v = 0.f;
  if (n < N) {
    if (mode == 0) v = Conv<T>::ld(s0, n);
    else if (mode == 1) {
      int region = n / d, c = n % d, hh = c / hd, e = c % hd;
      if (region < 2) { int half = hd >> 1; e = (e & 1) ? (e >> 1) + half : (e >> 1); }
      const T *src = region == 0 ? s0 : region == 1 ? s1 : s2;
      v = Conv<T>::ld(src, hh * hd + e);
    } else {
      int p = n >> 2, q = n & 3;
      v = Conv<T>::ld((q & 1) ? s1 : s0, 2 * p + (q >> 1));
    }
  }
  dst[n] = v;
}

// Folded LayerNorm, set-up side: for every stored row n of a packed matrix (one wave per row, fixed lane assignment
// and butterfly: the same bits on every run) wsum[n] = the sum of the packed fp16 elements of the row -- what the
// epilogue multiplies the row mean with, in the packed weights' own scaled units -- and bias[n] += sum_k W[n][k] *
// b[k], the norm's bias pushed through the original weights (stored-row order as in k_pack_weight).
template <class T>
__global__ __launch_bounds__(256) void k_fold_ln(int mode, int N, int K, int N_pad, int K_pad, int d, int hd,
                                                 const T *__restrict__ s0, const T *__restrict__ s1, const T *__restrict__ s2,
                                                 const T *__restrict__ ln_bias, const op_t *__restrict__ packed,
                                                 float *__restrict__ wsum, float *__restrict__ bias) {
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (n >= N_pad) return;
  const int KT = K_pad / 32, nt = n >> 4, r = n & 15;
  float s = 0.f;
  for (int k = lane * 8; k < K_pad; k += 512) {
    const op_t *p = packed + ((((size_t)nt * KT + (k >> 5)) * 64 + (((k & 31) >> 3) << 4) + r) << 3);
#pragma unroll
    for (int i = 0; i < 8; ++i) s += (float)p[i];
  }
  s = wave_sum(s);
  float wb = 0.f;
  if (n < N) {
    const T *src;
    int row;
    if (mode == 0) { src = s0; row = n; }
    else if (mode == 1) {
      int region = n / d, c = n % d, hh = c / hd, e = c % hd;
      if (region < 2) { int half = hd >> 1; e = (e & 1) ? (e >> 1) + half : (e >> 1); }
      src = region == 0 ? s0 : region == 1 ? s1 : s2;
      row = hh * hd + e;
    } else {
      int p = n >> 2, q = n & 3;
      src = (q & 1) ? s1 : s0;
      row = 2 * p + (q >> 1);
    }
    for (int k = lane; k < K; k += 64) wb += Conv<T>::ld(src, (size_t)row * K + k) * Conv<T>::ld(ln_bias, k);
  }
  wb = wave_sum(wb);
  if (lane == 0) {
    wsum[n] = s;
    if (n < N) bias[n] += wb;
  }
}
void launch_fold_ln(int dtype, int mode, const PackedDims &p, int d, int hd, const void *s0, const void *s1, const void *s2,
                    const void *ln_bias, const void *packed, float *wsum, float *bias, hipStream_t st) {
  const unsigned blocks = (unsigned)((p.N_pad + 3) / 4);
  if (dtype == SPEC_DTYPE_BF16)
    hipLaunchKernelGGL(k_fold_ln<bf16_t>, dim3(blocks), dim3(256), 0, st, mode, p.N, p.K, p.N_pad, p.K_pad, d, hd, (const bf16_t *)s0,
                       (const bf16_t *)s1, (const bf16_t *)s2, (const bf16_t *)ln_bias, (const op_t *)packed, wsum, bias);
  else
    hipLaunchKernelGGL(k_fold_ln<f16_t>, dim3(blocks), dim3(256), 0, st, mode, p.N, p.K, p.N_pad, p.K_pad, d, hd, (const f16_t *)s0,
                       (const f16_t *)s1, (const f16_t *)s2, (const f16_t *)ln_bias, (const op_t *)packed, wsum, bias);
}

PackedDims packed_dims(int N, int K) {
  PackedDims p;
  p.N = N; p.K = K;
  p.N_pad = (N + 15) / 16 * 16;
  p.K_pad = (K + 31) / 32 * 32;
  p.NT = p.N_pad / 16;
  p.KT = p.K_pad / 32;
  p.KS = gemm_ks_for(p.KT);
  return p;
}

void launch_pack_weight(int dtype, int mode, const PackedDims &p, int d, int hd, const void *s0, const void *s1,
                        const void *s2, const void *gain, void *dst, const uint32_t *d_amax_bits, hipStream_t st) {
  size_t total = (size_t)p.NT * p.KT * 64;
  unsigned blocks = (unsigned)((total + 255) / 256);
  if (dtype == SPEC_DTYPE_BF16)
    hipLaunchKernelGGL(k_pack_weight<bf16_t>, dim3(blocks), dim3(256), 0, st, mode, p.N, p.K, p.N_pad, p.K_pad, d, hd,
                       (const bf16_t *)s0, (const bf16_t *)s1, (const bf16_t *)s2, (const bf16_t *)gain, (op_t *)dst, d_amax_bits);
  else
    hipLaunchKernelGGL(k_pack_weight<f16_t>, dim3(blocks), dim3(256), 0, st, mode, p.N, p.K, p.N_pad, p.K_pad, d, hd,
                       (const f16_t *)s0, (const f16_t *)s1, (const f16_t *)s2, (const f16_t *)gain, (op_t *)dst, d_amax_bits);
}

void launch_pack_bias(int dtype, int mode, const PackedDims &p, int d, int hd, const void *s0, const void *s1,
                      const void *s2, float *dst, hipStream_t st) {
  unsigned blocks = (unsigned)((p.N_pad + 255) / 256);
  if (dtype == SPEC_DTYPE_BF16)
    hipLaunchKernelGGL(k_pack_bias<bf16_t>, dim3(blocks), dim3(256), 0, st, mode, p.N, p.N_pad, d, hd,
                       (const bf16_t *)s0, (const bf16_t *)s1, (const bf16_t *)s2, dst);
  else
    hipLaunchKernelGGL(k_pack_bias<f16_t>, dim3(blocks), dim3(256), 0, st, mode, p.N, p.N_pad, d, hd,
                       (const f16_t *)s0, (const f16_t *)s1, (const f16_t *)s2, dst);
}

// Rotary table: rope[pos][i] = (cos, sin) of pos * theta^(-2i/hd), i < hd/2.
__global__ void k_rope_table(int L, int hd, float theta, float2 *__restrict__ tab) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  int half = hd >> 1;
  if (idx >= L * half) return;
  int pos = idx / half, i = idx % half;
  float inv_freq = powf(theta, -2.0f * (float)i / (float)hd);
  float s, c;
  sincosf((float)pos * inv_freq, &s, &c);
  tab[idx] = make_float2(c, s);
}
void launch_rope_table(int L, int hd, float theta, float2 *tab, hipStream_t st) {
  int total = L * (hd / 2);
  hipLaunchKernelGGL(k_rope_table, dim3((total + 255) / 256), dim3(256), 0, st, L, hd, theta, tab);
}

// ------------------------------------------------------------------------- the kernel
// Workgroup = KS waves; wave w owns k-slice w of NB consecutive 16-row strips of W (a strip
// group) and MT 16-row tiles of X (a pass).  Weights and activations are both read in
// fragment order, 1 KB per wave per load.  After the k loop the KS partial tiles meet in
// LDS, eight tiles at a time, and are added in slice order.
// With more than one pass the linear workgroup id is decoded so that all passes of a strip
// group run on the same XCD (workgroups are dealt round-robin to the 8 XCDs): the group's
// weights are fetched from HBM once and hit that XCD's L2 for the other passes.
template <class T, int MT, int NB, int EPI>
__global__ __launch_bounds__(512) void k_gemm_stream(GemmArgs a) {
  extern __shared__ float red[];  // [KS][min(NB*MT, 8)][256]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int KS = blockDim.x >> 6;
  int G, pass;
  if (a.passes == 1) { G = blockIdx.x; pass = 0; }
  else {
    const int id = blockIdx.x, rest = id >> 3;
    pass = rest % a.passes;
    G = (rest / a.passes) * 8 + (id & 7);
  }
  if (G >= a.groups) return;
  const int nt0 = G * NB;
  const int m_base = pass * (MT * 16);
  const int kt_per = a.KT / KS;
  const int kt0 = w * kt_per, kt1 = kt0 + kt_per;
  const int m_tiles = (a.M + 15) >> 4;

  const u32x4_v *Wp[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    int nt = min(nt0 + nb, a.NT - 1);
    Wp[nb] = (const u32x4_v *)a.W + (size_t)nt * a.KT * 64 + lane;
  }
  const u32x4_v *Xp[MT];
  bool xlive[MT];  // lanes whose activation row does not exist load nothing and feed zeros
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int tile = min((m_base >> 4) + mt, m_tiles - 1);
    Xp[mt] = (const u32x4_v *)a.X + (size_t)tile * a.KT * 64 + lane;
    xlive[mt] = m_base + mt * 16 + c < a.M;
  }
  const u32x4_v zero4 = (u32x4_v){0u, 0u, 0u, 0u};

  f32x4_v acc[NB][MT];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[nb][mt] = (f32x4_v){0.f, 0.f, 0.f, 0.f};

  constexpr bool FOLDX = EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_RELU || EPI == EPI_LOGITS;  // the GEMMs behind a norm
  const bool foldx = FOLDX && a.fold_x;
  const bool lnx = foldx && a.wsum;  // the folded norm is a LayerNorm: the plain sums as well
  float ssq[MT], sm[MT];  // this lane's part of the sum of squares (and of the sum) of its rows over the wave's k-slice
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) { ssq[mt] = 0.f; sm[mt] = 0.f; }
  constexpr int U = (NB + MT >= 12) ? 1 : (NB + MT >= 6) ? 2 : (NB + MT >= 3) ? 4 : 8;
  int kt = kt0;
  for (; kt + U <= kt1; kt += U) {
    u32x4_v wf[U][NB], xf[U][MT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) wf[u][nb] = __builtin_nontemporal_load(Wp[nb] + (size_t)(kt + u) * 64);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) xf[u][mt] = xlive[mt] ? Xp[mt][(size_t)(kt + u) * 64] : zero4;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nb][mt] = Mfma16::run(wf[u][nb], xf[u][mt], acc[nb][mt]);
    if (foldx) {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) ssq[mt] = frag_ssq(xf[u][mt], ssq[mt]);
      if (lnx) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) sm[mt] = frag_sum(xf[u][mt], sm[mt]);
      }
    }
  }
  // the steps left over (fewer than U): all their loads go out together as well, so the end of a slice costs one
  // memory latency, not one per step (a slice of the 7B down projection has 43 = 5 * 8 + 3 steps)
  const int rem = __builtin_amdgcn_readfirstlane(kt1 - kt);  // same for the whole wave: scalar branches
  if (U > 1 && rem > 0) {
    u32x4_v wf[U][NB], xf[U][MT];
#pragma unroll
    for (int u = 0; u < U - 1; ++u) {
      if (u < rem) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) wf[u][nb] = __builtin_nontemporal_load(Wp[nb] + (size_t)(kt + u) * 64);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) xf[u][mt] = xlive[mt] ? Xp[mt][(size_t)(kt + u) * 64] : zero4;
      }
    }
#pragma unroll
    for (int u = 0; u < U - 1; ++u) {
      if (u < rem) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[nb][mt] = Mfma16::run(wf[u][nb], xf[u][mt], acc[nb][mt]);
      }
    }
    if (foldx) {
#pragma unroll
      for (int u = 0; u < U - 1; ++u) {
        if (u < rem) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) ssq[mt] = frag_ssq(xf[u][mt], ssq[mt]);
          if (lnx) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) sm[mt] = frag_sum(xf[u][mt], sm[mt]);
          }
        }
      }
    }
  }

  constexpr int TILES = NB * MT;
  // folded norm from the operand fragments: the waves' slice sums meet in LDS (behind the same barrier as the
  // first round of partial tiles) and are added in slice order
  __shared__ float ssq_s[FOLDX ? 8 : 1][FOLDX ? MT * 64 : 1];
  __shared__ float sum_s[FOLDX ? 8 : 1][FOLDX ? MT * 64 : 1];
  float rinv_x[MT], mean_x[MT];
  if (foldx && KS > 1) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      ssq_s[w][mt * 64 + lane] = ssq[mt];
      if (lnx) sum_s[w][mt * 64 + lane] = sm[mt];
    }
  }
  auto finish_rinv = [&]() {
    if (!foldx) return;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float t = ssq[mt];
      if (KS > 1) {
        t = ssq_s[0][mt * 64 + lane];
        for (int s = 1; s < KS; ++s) t += ssq_s[s][mt * 64 + lane];
      }
      mean_x[mt] = 0.f;
      if (lnx) {
        float ts = sm[mt];
        if (KS > 1) {
          ts = sum_s[0][mt * 64 + lane];
          for (int s = 1; s < KS; ++s) ts += sum_s[s][mt * 64 + lane];
        }
        row_ln_from_lane(t, ts, a.ss_d, a.ss_eps, rinv_x[mt], mean_x[mt]);
      } else {
        rinv_x[mt] = row_inv_from_lane_ssq(t, a.ss_d, a.ss_eps);
      }
    }
  };
  auto rinv_of = [&](int mt) { return foldx ? rinv_x[mt] : 1.0f; };
  auto mean_of = [&](int mt) { return foldx ? mean_x[mt] : 0.f; };
  if (KS == 1) {
    finish_rinv();
#pragma unroll
    for (int t = 0; t < TILES; ++t)
      tile_epilogue<T, EPI>(a, acc[t / MT][t % MT], nt0 + t / MT, m_base + (t % MT) * 16 + c, g, rinv_of(t % MT), mean_of(t % MT));
    return;
  }
  constexpr int ROUNDS = (TILES + 7) / 8;
  constexpr int SLOTS = TILES < 8 ? TILES : 8;
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    if (r > 0) __syncthreads();
#pragma unroll
    for (int slot = 0; slot < 8; ++slot) {
      const int t = r * 8 + slot;
      if (t < TILES) *(f32x4_v *)&red[((size_t)(w * SLOTS + slot) * 64 + lane) * 4] = acc[t / MT][t % MT];
    }
    __syncthreads();
    if (r == 0) finish_rinv();
#pragma unroll
    for (int slot = 0; slot < 8; ++slot) {
      const int t = r * 8 + slot;
      if (t >= TILES) continue;
      if ((slot % KS) != w) continue;
      f32x4_v v = *(const f32x4_v *)&red[((size_t)(0 * SLOTS + slot) * 64 + lane) * 4];
      for (int s = 1; s < KS; ++s) {
        f32x4_v p = *(const f32x4_v *)&red[((size_t)(s * SLOTS + slot) * 64 + lane) * 4];
        v[0] += p[0]; v[1] += p[1]; v[2] += p[2]; v[3] += p[3];
      }
      tile_epilogue<T, EPI>(a, v, nt0 + t / MT, m_base + (t % MT) * 16 + c, g, rinv_of(t % MT), mean_of(t % MT));
    }
  }
}

template <class T, int MT, int NB>
static void launch_epi(const GemmArgs &a, int epi, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
  switch (epi) {
    case EPI_RESIDUAL: hipLaunchKernelGGL((k_gemm_stream<T, MT, NB, EPI_RESIDUAL>), grid, block, lds, st, a); break;
    case EPI_QKV: hipLaunchKernelGGL((k_gemm_stream<T, MT, NB, EPI_QKV>), grid, block, lds, st, a); break;
    case EPI_SWIGLU: hipLaunchKernelGGL((k_gemm_stream<T, MT, NB, EPI_SWIGLU>), grid, block, lds, st, a); break;
    case EPI_RELU: hipLaunchKernelGGL((k_gemm_stream<T, MT, NB, EPI_RELU>), grid, block, lds, st, a); break;
    default: hipLaunchKernelGGL((k_gemm_stream<T, MT, NB, EPI_LOGITS>), grid, block, lds, st, a); break;
  }
}

// Wide outputs go to the LDS-tiled kernel (same bits, weights fetched once per up to 256 rows) from 65 rows
// on, the widest (gate-up, LM head) already from 33: the streaming kernel's waves each fetch their own copy
// of the activations, the tiled kernel shares them through LDS.  The narrow residual GEMMs run it one k-slice
// per workgroup when the context has the scratch for the slices: worth the second kernel from 33 rows on
// when a slice has at least 32 steps (down projection), and from 5 row passes of the streaming kernel.
static bool goes_to_tile_kernel(const GemmArgs &a, int epi) {
  const bool split_ok = a.part && a.KS > 1 && (a.N & 3) == 0 && (a.KT / a.KS >= 32 || a.M > 256);
  const int tile_min_m = a.NT >= 1024 ? 33 : 65;
  return a.NT >= 64 && (epi != EPI_RESIDUAL ? a.M >= tile_min_m : (split_ok && a.M >= 33));
}
bool gemm_can_leave_ssq(const GemmArgs &a) {  // the row-wise reduction keeps the fp16 row in LDS: rows of up to 8192
  return a.x_out && a.M > 64 && (a.N & 31) == 0 && a.N <= 8192 && goes_to_tile_kernel(a, EPI_RESIDUAL);
}
bool gemm_wants_row_inv(const GemmArgs &a, int epi) {
  return a.M > 0 && goes_to_tile_kernel(a, epi) && gemm_tile_wants_row_inv(a, epi);
}

template <class T>
static void launch_gemm_t(GemmArgs a, int epi, hipStream_t st) {
  if (a.M <= 0) return;
  if (goes_to_tile_kernel(a, epi)) {
    launch_gemm_tile(std::is_same<T, bf16_t>::value ? SPEC_DTYPE_BF16 : SPEC_DTYPE_F16, a, epi, st);
    return;
  }
  if (launch_gemm_rowres(std::is_same<T, bf16_t>::value ? SPEC_DTYPE_BF16 : SPEC_DTYPE_F16, a, epi, st)) return;
  const int KS = a.KS;
  // rows per pass: MT tiles of 16; strips per workgroup: NB.  Neither changes any result.
  // A compute unit keeps a bounded number of cache-line requests in flight, and that is what a launch here is bound
  // by; a workgroup asks for NB weight fragments (from HBM the first time a strip is read, from L2 for the other row
  // passes) and MT activation fragments (L2) per 32-k step, so the unit with the most workgroups sets the time:
  // ceil(workgroups / units) * (NB * weight cost + MT * activation cost), with a request that goes to HBM about three
  // times as dear as one that hits L2 (measured).  Against doubling NB up to MT: QKV at d_model 4096 with 17..64
  // rows 27..36 -> 23..31 us (three strips per workgroup: one workgroup per unit).  Small matrices (a draft model's)
  // come out with two row tiles per workgroup and more row passes: their few strips then spread over more units.
  const int n_cu = a.n_cu > 0 ? a.n_cu : 256;
  const int mt_max = a.M <= 16 ? 1 : a.M <= 32 ? 2 : 4;
  int MT = mt_max, NB = 1;
  if (mt_max > 1 && epi != EPI_LOGITS) {
    static const int cand[] = {1, 2, 3, 4, 6, 8};
    long best = -1;
    for (int mt = mt_max; mt >= 1; mt >>= 1) {
      const int passes = (a.M + mt * 16 - 1) / (mt * 16);
      for (int nb : cand) {
        if (mt == 1 && nb > 1) break;  // one row tile per workgroup is built with one strip only
        const long wgs = (long)((a.NT + nb - 1) / nb) * passes;
        const long per_cu = (wgs + n_cu - 1) / n_cu;
        const long w_cost = (3000 + 1000 * (passes - 1)) / passes;  // per strip and step, averaged over the row passes
        const long cost = per_cu * (nb * w_cost + mt * 1000);
        if (best < 0 || cost < best) { best = cost; NB = nb; MT = mt; }
      }
    }
  } else if (mt_max > 1) {
    // the LM head, with its arg-max epilogue per strip, measured better with fewer strips per workgroup than that
    // estimate picks: as many as row tiles while 160 workgroups remain
    const int passes = (a.M + MT * 16 - 1) / (MT * 16);
    while (NB < MT && (a.NT / (NB * 2)) * passes >= 160) NB *= 2;
    if (MT == 4 && NB == 4 && (a.NT / 8) * passes >= 160) NB = 8;
  }
  a.passes = (a.M + MT * 16 - 1) / (MT * 16);
  a.groups = (a.NT + NB - 1) / NB;
  const int blocks = a.passes == 1 ? a.groups : ((a.groups + 7) / 8) * 8 * a.passes;
  dim3 grid(blocks), block(KS * 64);
  const int tiles = NB * MT;
  size_t lds = KS > 1 ? (size_t)KS * (tiles < 8 ? tiles : 8) * 1024 : 0;
  // Up to 16 rows the kernel needs few registers and little LDS, and three workgroups would fit a compute unit; two
  // measured best (QKV and LM head at 8 rows: three +2..5 us, one +25 %): more requests than the unit keeps in flight
  // only queue up.  Asking for more LDS than a third of the unit's holds the third workgroup off.
  if (MT == 1 && lds < 56 * 1024) lds = 56 * 1024;
  if (MT == 1) launch_epi<T, 1, 1>(a, epi, grid, block, lds, st);
  else if (MT == 2) {
    switch (NB) {
      case 1: launch_epi<T, 2, 1>(a, epi, grid, block, lds, st); break;
      case 2: launch_epi<T, 2, 2>(a, epi, grid, block, lds, st); break;
      case 3: launch_epi<T, 2, 3>(a, epi, grid, block, lds, st); break;
      case 4: launch_epi<T, 2, 4>(a, epi, grid, block, lds, st); break;
      case 6: launch_epi<T, 2, 6>(a, epi, grid, block, lds, st); break;
      default: launch_epi<T, 2, 8>(a, epi, grid, block, lds, st); break;
    }
  } else {
    switch (NB) {
      case 1: launch_epi<T, 4, 1>(a, epi, grid, block, lds, st); break;
      case 2: launch_epi<T, 4, 2>(a, epi, grid, block, lds, st); break;
      case 3: launch_epi<T, 4, 3>(a, epi, grid, block, lds, st); break;
      case 4: launch_epi<T, 4, 4>(a, epi, grid, block, lds, st); break;
      case 6: launch_epi<T, 4, 6>(a, epi, grid, block, lds, st); break;
      default: launch_epi<T, 4, 8>(a, epi, grid, block, lds, st); break;
    }
  }
}

void launch_gemm_mfma(int dtype, const GemmArgs &a, int epi, hipStream_t st) {
  if (dtype == SPEC_DTYPE_BF16) launch_gemm_t<bf16_t>(a, epi, st);
  else launch_gemm_t<f16_t>(a, epi, st);
}

// Second stage of the fused arg-max: one block per row over the per-strip partials.
// row_step > 0: output row m takes the partials of GEMM row m * row_step + row_step - 1 (the last row of its group).
__global__ void k_argmax_partials(const float *__restrict__ pv, const int32_t *__restrict__ pi, int row_step, int NT, int V,
                                  int q, int out_stride, int32_t *__restrict__ out) {
  __shared__ float shv[4];
  __shared__ int shi[4];
  const int m = blockIdx.x;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  const size_t src = row_step > 0 ? (size_t)m * row_step + row_step - 1 : (size_t)m;
  for (int t = threadIdx.x; t < NT; t += 256) argmax_combine(bv, bi, pv[src * NT + t], pi[src * NT + t]);
  wave_argmax(bv, bi);
  if ((threadIdx.x & 63) == 0) { shv[threadIdx.x >> 6] = bv; shi[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) argmax_combine(bv, bi, shv[w], shi[w]);
    if (bi < 0 || bi >= V) bi = 0;
    out[(size_t)(m / q) * out_stride + m % q] = bi;
  }
}
void launch_argmax_partials(const float *pv, const int32_t *pi, int M, int row_step, int NT, int V, int q, int out_stride,
                            int32_t *out, hipStream_t st) {
  if (M <= 0) return;
  hipLaunchKernelGGL(k_argmax_partials, dim3(M), dim3(256), 0, st, pv, pi, row_step, NT, V, q, out_stride, out);
}

}  // namespace spec
