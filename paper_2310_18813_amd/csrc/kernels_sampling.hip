// Speculative sampling: the non-greedy form of the acceptance step (Sec. 2 describes speculative decoding and
// cites this rule for sampling; Alg. 1 itself is greedy).
//
//   q_j = softmax(draft logits of step j / T),  p_j = softmax(target logits of row j / T)
//   keep proposal t_j  if  u * q_j[t_j] < p_j[t_j];  at the first j that fails, emit one token drawn from
//   max(0, p_j - q_j) (normalised) and stop;  if all are kept, emit one token drawn from the next target row.
// Proposals that come from no distribution (a table) count as point masses: q_j[t_j] = 1.
// A draw from weights w with a uniform number u is the smallest index whose cumulative weight exceeds u * sum(w).
//
// The kernels here only replace the "greedy tokens of the target" by tokens chosen so that the unchanged
// longest-matching-prefix rule reproduces the outcome: entry j is t_{j+1} while proposals are kept, the drawn token
// at the first rejection (never equal to the rejected proposal: its residual weight is zero), the bonus draw
// behind s kept proposals.  Commit, roll-back, end token and budgets then work as in the greedy case.
//
// One workgroup per row (proposal draws) or per sequence (verification); a thread owns a contiguous chunk of the
// vocabulary; chunk sums are added in thread order by every thread alike, so a draw depends on the row alone.
#include "spec_internal.h"
#include "device_utils.h"

namespace spec {

#pragma clang fp contract(off)

constexpr int SMP_THREADS = 256;

struct Chunk { int k0, k1; };
__device__ __forceinline__ Chunk my_chunk(int V) {
  const int per = ((V + SMP_THREADS - 1) / SMP_THREADS + 3) & ~3;  // a multiple of four: chunks start 16-byte aligned
  Chunk c;
  c.k0 = min(V, (int)threadIdx.x * per);
  c.k1 = min(V, c.k0 + per);
  return c;
}

// z[k .. k+3] (k a multiple of four), `fill` beyond the row; one 16-byte load when the row allows it
__device__ __forceinline__ void load4z(const float *__restrict__ z, int k, int V, bool vec, float fill, float (&o)[4]) {
  if (vec) {
    const float4 v = *(const float4 *)(z + k);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = k + i < V ? z[k + i] : fill;
  }
}
__device__ __forceinline__ bool row_vec(const float *z, int V) { return (V & 3) == 0 && ((uintptr_t)z & 15) == 0; }

// Workgroup-wide maximum / sum / exclusive prefix of one value per thread.  The order of the additions is fixed by the
// thread numbers alone (shuffles inside a wave, then the waves in order), so every thread sees the same bits and a
// row's result does not depend on anything but the row.  sh: at least SMP_THREADS / 64 + 1 floats.
__device__ __forceinline__ float block_max_all(float v, float *sh) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  __syncthreads();  // sh may still be read by the previous user
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float m = sh[0];
#pragma unroll
  for (int i = 1; i < SMP_THREADS / 64; ++i) m = fmaxf(m, sh[i]);
  return m;
}
// inclusive prefix inside the wave (lane l: v_0 + ... + v_l, added pairwise by doubling distances), the waves' totals
// through LDS; returns the exclusive prefix of this thread, *total = the sum over the workgroup
__device__ __forceinline__ float block_prefix(float v, float *sh, float *total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  float inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const float up = __shfl_up(inc, o, 64);
    if (lane >= o) inc += up;
  }
  __syncthreads();
  if (lane == 63) sh[wv] = inc;
  __syncthreads();
  float before = 0.f, all = 0.f;
#pragma unroll
  for (int i = 0; i < SMP_THREADS / 64; ++i) {
    if (i == wv) before = all;
    all += sh[i];
  }
  *total = all;
  return before + (inc - v);
}

// max over the row and sum of exp((z - max) * inv_T), the same bits in every thread
template <bool WANT_SUM = true>
__device__ __forceinline__ void row_stats(const float *__restrict__ z, int V, float inv_T, float *sh, float &m, float &Z) {
  const Chunk c = my_chunk(V);
  const bool vec = row_vec(z, V);
  float lm = -INFINITY;
#pragma unroll 8
  for (int k = c.k0; k < c.k1; k += 4) {
    float v[4];
    load4z(z, k, V, vec, -INFINITY, v);
    lm = fmaxf(fmaxf(lm, v[0]), fmaxf(fmaxf(v[1], v[2]), v[3]));
  }
  m = block_max_all(lm, sh);
  Z = 0.f;
  if (!WANT_SUM) return;
  float ls = 0.f;
#pragma unroll 8
  for (int k = c.k0; k < c.k1; k += 4) {
    float v[4];
    load4z(z, k, V, vec, -INFINITY, v);  // exp(-inf) = 0 beyond the row
#pragma unroll
    for (int i = 0; i < 4; ++i) ls += __expf((v[i] - m) * inv_T);
  }
  block_prefix(ls, sh, &Z);
}

// Draw with u from the weights w4(k, out) -> weights of k .. k+3 (zero beyond the row), k a multiple of four:
// every thread returns the same index.  *total_out: the sum of all weights.
template <class W4>
__device__ __forceinline__ int block_draw(int V, W4 w4, float u, float *sh, int *sh_i, float *total_out = nullptr) {
  const Chunk c = my_chunk(V);
  float local = 0.f;
#pragma unroll 8
  for (int k = c.k0; k < c.k1; k += 4) {
    float w[4];
    w4(k, w);
#pragma unroll
    for (int i = 0; i < 4; ++i) local += w[i];
  }
  float total;
  const float excl = block_prefix(local, sh, &total);
  if (threadIdx.x == 0) *sh_i = -1;
  if (total_out) *total_out = total;
  float x = u * total;
  if (!(x < total)) x = total * 0.99999994f;  // u < 1, but the product may round up to the total
  __syncthreads();
  // the owner of x: the last thread with weight whose prefix does not exceed x (the prefixes come from sums in
  // different associations, so "prefix <= x < prefix + local" could leave a hair's gap between neighbours)
  if (local > 0.f && excl <= x) atomicMax(sh_i, (int)threadIdx.x);
  __syncthreads();
  const int owner = *sh_i;
  __syncthreads();
  if ((int)threadIdx.x == owner) {
    float run = excl;
    int pick = -1, last = -1;
  #pragma unroll 8
  for (int k = c.k0; k < c.k1; k += 4) {
      float w[4];
      w4(k, w);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (w[i] > 0.f) last = k + i;
        run += w[i];
        if (pick < 0 && run > x) pick = k + i;
      }
    }
    *sh_i = pick >= 0 ? pick : last;  // the walk may end a hair below x: then the chunk's last token
  } else if (owner < 0 && threadIdx.x == 0) {
    *sh_i = 0;  // all weights zero or not finite: the lowest index, as the greedy rule does for a row of NaNs
  }
  __syncthreads();
  return *sh_i;
}

// weights exp((z - m) * inv_T) of a row, optionally with one token removed
struct ExpW {
  const float *z; int V; bool vec; float m, inv_T; int drop;
  __device__ __forceinline__ void operator()(int k, float (&w)[4]) const {
    float v[4];
    load4z(z, k, V, vec, -INFINITY, v);
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (k + i == drop) ? 0.f : __expf((v[i] - m) * inv_T);
  }
};
// residual weights max(0, p - q) of a target and a draft row
struct ResidW {
  ExpW p, q; float ip, iq;
  __device__ __forceinline__ void operator()(int k, float (&w)[4]) const {
    float a[4], b[4];
    p(k, a); q(k, b);
#pragma unroll
    for (int i = 0; i < 4; ++i) { const float r = a[i] * ip - b[i] * iq; w[i] = r > 0.f ? r : 0.f; }
  }
};

__device__ __forceinline__ float uniform_at(const float *__restrict__ u, const int32_t *__restrict__ n, int b, int off,
                                            int u_rows, int kind) {
  // with lengths: a table [B][u_rows][3] indexed by the absolute position of the token the number decides;
  // without: [B][u_rows][3] indexed by the row of the round
  const int row = n ? min(n[b] + off, u_rows - 1) : off;
  return u[((size_t)b * u_rows + row) * 3 + kind];
}

// One proposal per sequence: a draw from softmax(logits[b] / T).  out[b * out_stride].
__global__ __launch_bounds__(SMP_THREADS) void k_sample_rows(const float *__restrict__ logits, int V, float inv_T,
                                                             const float *__restrict__ u, const int32_t *__restrict__ n,
                                                             int off, int u_rows, int32_t *__restrict__ out, int out_stride) {
  __shared__ float sh[SMP_THREADS];
  __shared__ int sh_i;
  const int b = blockIdx.x;
  const float *z = logits + (size_t)b * V;
  float m, Z;  // a draw needs the maximum only: its own pass over the row adds the weights up
  row_stats<false>(z, V, inv_T, sh, m, Z);
  const float uu = n ? uniform_at(u, n, b, off, u_rows, 0) : u[b];
  const int tok = block_draw(V, ExpW{z, V, row_vec(z, V), m, inv_T, -1}, uu, sh, &sh_i);
  if (threadIdx.x == 0) out[(size_t)b * out_stride] = tok;
}

// Verification of one sequence's proposals; writes a[b][0..s_b] (see the head of this file).
//   tl: target logits, row b * (s + 1) + j;  dl: draft logits of step j + 1 at ((size_t)j * d_rows + b) * V, or null
__global__ __launch_bounds__(SMP_THREADS) void k_sample_verify(const float *__restrict__ tl, const float *__restrict__ dl,
                                                               int d_rows, int s, int V, float inv_T,
                                                               const int32_t *__restrict__ t, int t_stride,
                                                               const int32_t *__restrict__ seq_s,
                                                               const float *__restrict__ u, const int32_t *__restrict__ n,
                                                               int u_rows, int32_t *__restrict__ a, int a_stride) {
  __shared__ float sh[SMP_THREADS];
  __shared__ int sh_i;
  const int b = blockIdx.x;
  const int sb = seq_s ? min(s, max(0, seq_s[b])) : s;
  int32_t *ab = a + (size_t)b * a_stride;
  for (int j = 0; j <= sb; ++j) {
    const float *zp = tl + ((size_t)b * (s + 1) + j) * V;
    float mp, Zp;
    row_stats(zp, V, inv_T, sh, mp, Zp);
    const float us = uniform_at(u, n, b, j, u_rows, 2);
    const ExpW wp{zp, V, row_vec(zp, V), mp, inv_T, -1};
    if (j == sb) {  // every proposal kept: the bonus draw from the target's next row
      const int tok = block_draw(V, wp, us, sh, &sh_i);
      if (threadIdx.x == 0) ab[j] = tok;
      break;
    }
    const int tj = t[(size_t)b * t_stride + j];
    const bool valid = tj >= 0 && tj < V;
    const float ua = uniform_at(u, n, b, j, u_rows, 1);
    const float pt = valid ? __expf((zp[tj] - mp) * inv_T) * (1.0f / Zp) : 0.f;
    int tok;
    if (dl) {
      const float *zq = dl + ((size_t)j * d_rows + b) * V;
      float mq, Zq;
      row_stats(zq, V, inv_T, sh, mq, Zq);
      const float qt = valid ? __expf((zq[tj] - mq) * inv_T) * (1.0f / Zq) : 1.f;
      if (ua * qt < pt) {
        if (threadIdx.x == 0) ab[j] = tj;
        continue;
      }
      float total;
      tok = block_draw(V, ResidW{wp, ExpW{zq, V, row_vec(zq, V), mq, inv_T, -1}, 1.0f / Zp, 1.0f / Zq}, us, sh, &sh_i, &total);
      // p = q everywhere leaves no residual (not reachable with u < 1 and a valid proposal): draw from p
      if (!(total > 0.f)) tok = block_draw(V, wp, us, sh, &sh_i);
    } else {
      if (ua < pt) {
        if (threadIdx.x == 0) ab[j] = tj;
        continue;
      }
      tok = block_draw(V, ExpW{zp, V, row_vec(zp, V), mp, inv_T, valid ? tj : -1}, us, sh, &sh_i);
    }
    if (threadIdx.x == 0) {
      ab[j] = tok;
      for (int i = j + 1; i <= s; ++i) ab[i] = -1;
    }
    break;
  }
}

void launch_sample_rows(const float *logits, int rows, int V, float temperature, const float *u, const int32_t *n, int off,
                        int u_rows, int32_t *out, int out_stride, hipStream_t st) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(k_sample_rows, dim3(rows), dim3(SMP_THREADS), 0, st, logits, V, 1.0f / temperature, u, n, off, u_rows,
                     out, out_stride);
}
void launch_sample_verify(const float *tl, const float *dl, int d_rows, int B, int s, int V, float temperature,
                          const int32_t *t, int t_stride, const int32_t *seq_s, const float *u, const int32_t *n, int u_rows,
                          int32_t *a, int a_stride, hipStream_t st) {
  if (B <= 0) return;
  hipLaunchKernelGGL(k_sample_verify, dim3(B), dim3(SMP_THREADS), 0, st, tl, dl, d_rows, s, V, 1.0f / temperature, t, t_stride,
                     seq_s, u, n, u_rows, a, a_stride);
}

// acceptance count and emitted tokens from (proposals, chosen tokens): the stand-alone entry point's last step
__global__ void k_sample_emit(int B, int s, const int32_t *__restrict__ t, const int32_t *__restrict__ a,
                              int32_t *__restrict__ accepted, int32_t *__restrict__ emitted) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int32_t *ab = a + (size_t)b * (s + 1);
  int l = 0;
  while (l < s && t[(size_t)b * s + l] == ab[l]) ++l;
  accepted[b] = l;
  int32_t *e = emitted + (size_t)b * (s + 1);
  const int32_t last = ab[l];
  for (int i = 0; i <= s; ++i) e[i] = i < l ? ab[i] : -1;
  e[l] = last;
}

}  // namespace spec

using namespace spec;

extern "C" int spec_sample_tokens(void *hip_stream, const float *d_logits, int32_t rows, int32_t vocab, float temperature,
                                  const float *d_uniforms, int32_t *d_tokens) {
  if (rows < 0 || vocab < 1) return fail_noctx(SPEC_ERR_INVALID_ARG, "spec_sample_tokens: rows=%d vocab=%d", rows, vocab);
  if (!(temperature > 0.f)) return fail_noctx(SPEC_ERR_INVALID_ARG, "spec_sample_tokens: temperature must be positive");
  if (rows == 0) return SPEC_OK;
  if (!d_logits || !d_uniforms || !d_tokens) return fail_noctx(SPEC_ERR_INVALID_ARG, "spec_sample_tokens: null pointer");
  if (rows > 65535 * 16) return fail_noctx(SPEC_ERR_CAPACITY, "spec_sample_tokens: rows=%d beyond 1048560", rows);
  launch_sample_rows(d_logits, rows, vocab, temperature, d_uniforms, nullptr, 0, 1, d_tokens, 1, (hipStream_t)hip_stream);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_noctx(SPEC_ERR_HIP, "spec_sample_tokens: %s", hipGetErrorString(e));
  return SPEC_OK;
}

extern "C" int spec_sample_accept(void *hip_stream, const float *d_target_logits, const float *d_draft_logits,
                                  const int32_t *d_proposals, const float *d_uniforms, int32_t B, int32_t s, int32_t vocab,
                                  float temperature, int32_t *d_chosen, int32_t *d_accepted, int32_t *d_emitted) {
  if (B < 0 || s < 0 || vocab < 1) return fail_noctx(SPEC_ERR_INVALID_ARG, "spec_sample_accept: B=%d s=%d vocab=%d", B, s, vocab);
  if (!(temperature > 0.f)) return fail_noctx(SPEC_ERR_INVALID_ARG, "spec_sample_accept: temperature must be positive");
  if (s > 15) return fail_noctx(SPEC_ERR_CAPACITY, "spec_sample_accept: s=%d beyond 15", s);
  if (B == 0) return SPEC_OK;
  if (!d_target_logits || !d_uniforms || !d_chosen || !d_accepted || !d_emitted || (s > 0 && !d_proposals))
    return fail_noctx(SPEC_ERR_INVALID_ARG, "spec_sample_accept: null pointer");
  hipStream_t st = (hipStream_t)hip_stream;
  launch_sample_verify(d_target_logits, d_draft_logits, B, B, s, vocab, temperature, d_proposals, s, nullptr, d_uniforms, nullptr,
                       s + 1, d_chosen, s + 1, st);
  hipLaunchKernelGGL(k_sample_emit, dim3((B + 63) / 64), dim3(64), 0, st, B, s, d_proposals, d_chosen, d_accepted, d_emitted);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_noctx(SPEC_ERR_HIP, "spec_sample_accept: %s", hipGetErrorString(e));
  return SPEC_OK;
}
