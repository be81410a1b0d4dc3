// Weight-streaming GEMM for up to 16 activation rows with the rows resident in registers.
//
// The streaming kernel (kernels_gemm_mfma.hip) gives every 16-row strip of W a workgroup of its own: each of its
// waves fetches the activation fragments of its k-slice again for every strip.  Those fetches hit L2, but they
// take places in the compute unit's queue of outstanding cache-line requests, which is what bounds a unit's share
// of the HBM stream: with 9 to 16 live rows a fragment is eight 128-byte lines, as many as the weight fragment
// beside it.  Here a workgroup is the same eight waves = eight k-slices, but it stays: wave w loads its k-slice of
// the activations once, keeps it in registers, and walks the strips blockIdx.x, blockIdx.x + gridDim.x, ... with
// half a strip slice of weight loads in flight (a ring of KTP / 2 fragment registers: the slot a multiply has
// just read is refilled with the fragment KTP / 2 steps ahead in the wave's stream; deeper rings and whole-slice
// bursts were measured slower).  Per strip the eight partial tiles meet in LDS, double-buffered so that one
// barrier per strip suffices, and a ninth wave adds them in slice order and runs the epilogue while the eight go
// on: their loop then holds no memory operation but its own loads.
//
// Same bits as the streaming kernel: the same instruction, every k-slice a chain from zero in ascending k, the
// slices added in order, the same epilogue code, the same sum-of-squares order for the folded norm.
//
// Covers k-slices of exactly 16 or 20 32-k steps (d_model 4096 and 5120 with eight slices) and the epilogues
// whose k is d_model and whose output is wide (QKV, gate-up / fc1, LM head).
#include "mfma_tiles.h"

namespace spec {

#pragma clang fp contract(off)

// The ring's loads are issued and awaited by hand: the compiler does not know of them, so it neither waits for all
// of them at the loop head (which it does for loads it tracks across the back edge) nor anywhere else.
// stream_load: non-temporal 16-byte load per lane into r, in flight when it returns.  stream_wait<N>(r): at most N
// of this wave's loads still in flight; r is tied to it so that no use of r can be moved in front of the wait.
__device__ __forceinline__ void stream_load(u32x4_v &r, const u32x4_v *p) {
  asm volatile("global_load_dwordx4 %0, %1, off nt" : "=&v"(r) : "v"(p) : "memory");
}
template <int N>
__device__ __forceinline__ void stream_wait(u32x4_v &r) {
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(r) : "n"(N) : "memory");
}

template <class T, int MT, int KTP, int R, int EPI>
__global__ __launch_bounds__(576) void k_gemm_rowres(GemmArgs a) {
  static_assert(KTP % R == 0 && R <= 32, "ring slots per strip slice");
  __shared__ f32x4_v red[2][8][MT][64];
  __shared__ float ssq_s[8][MT * 64];
  __shared__ float sum_s[8][MT * 64];
  const bool lnx = a.fold_x && a.wsum;  // the folded norm is a LayerNorm: the plain sums as well
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 15, g = lane >> 4;
  const int n_mine = (a.NT - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;  // host: gridDim.x <= NT
  // A bare barrier: __syncthreads() would wait for the loads in flight.  Before it this wave's LDS writes are done.
  auto wg_barrier = [&]() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  if (w == 8) {
    // the ninth wave streams nothing: per strip it adds the eight slices in slice order and runs the epilogue,
    // so that the streaming waves' loop holds no memory operation but its own loads
    wg_barrier();  // the sums of squares are in LDS
    float rinv[MT], mean[MT];  // folded norm: 1 / rms (or 1 / std and mean) of this lane's rows, the slice sums added in slice order
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      rinv[mt] = 1.0f; mean[mt] = 0.f;
      if (a.fold_x) {
        float t = ssq_s[0][mt * 64 + lane];
#pragma unroll
        for (int s = 1; s < 8; ++s) t += ssq_s[s][mt * 64 + lane];
        if (lnx) {
          float ts = sum_s[0][mt * 64 + lane];
#pragma unroll
          for (int s = 1; s < 8; ++s) ts += sum_s[s][mt * 64 + lane];
          row_ln_from_lane(t, ts, a.ss_d, a.ss_eps, rinv[mt], mean[mt]);
        } else {
          rinv[mt] = row_inv_from_lane_ssq(t, a.ss_d, a.ss_eps);
        }
      }
    }
    int strip = blockIdx.x;
    for (int i = 0; i < n_mine; ++i) {
      wg_barrier();  // strip i's partial tiles are in LDS buffer i & 1
      const int buf = i & 1;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        f32x4_v v = red[buf][0][mt][lane];
#pragma unroll
        for (int s = 1; s < 8; ++s) {
          const f32x4_v p = red[buf][s][mt][lane];
          v[0] += p[0]; v[1] += p[1]; v[2] += p[2]; v[3] += p[3];
        }
        tile_epilogue<T, EPI>(a, v, strip, mt * 16 + c, g, rinv[mt], mean[mt]);
      }
      // buffer `buf` is written again two strips on, behind the next barrier, which this wave reaches only now
      strip += gridDim.x;
    }
    return;
  }

  const int kt0 = w * KTP;
  const int m_tiles = (a.M + 15) >> 4;
  const u32x4_v zero4 = (u32x4_v){0u, 0u, 0u, 0u};
  // the weight stream of this wave: strip s, steps kt0 .. kt0 + KTP - 1; the first R steps go out at once
  const size_t strip_stride = (size_t)a.KT * 64;
  const u32x4_v *wp = (const u32x4_v *)a.W + (size_t)blockIdx.x * strip_stride + (size_t)kt0 * 64 + lane;
  u32x4_v ring[R];
#pragma unroll
  for (int r = 0; r < R; ++r) stream_load(ring[r], wp + (size_t)r * 64);

  // the activations of this wave's k-slice, once
  u32x4_v xf[MT][KTP];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int tile = min(mt, m_tiles - 1);
    const u32x4_v *xp = (const u32x4_v *)a.X + (size_t)tile * a.KT * 64 + (size_t)kt0 * 64 + lane;
    const bool live = mt * 16 + c < a.M;  // lanes whose row does not exist load nothing and feed zeros
#pragma unroll
    for (int u = 0; u < KTP; ++u) xf[mt][u] = live ? xp[(size_t)u * 64] : zero4;
  }
  if (a.fold_x) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float s = 0.f;
#pragma unroll
      for (int u = 0; u < KTP; ++u) s = frag_ssq(xf[mt][u], s);
      ssq_s[w][mt * 64 + lane] = s;
      if (lnx) {
        float t = 0.f;
#pragma unroll
        for (int u = 0; u < KTP; ++u) t = frag_sum(xf[mt][u], t);
        sum_s[w][mt * 64 + lane] = t;
      }
    }
  }
  // A use of every activation fragment in front of the loop: the compiler places its wait for those loads here and
  // has none pending inside the loop (left pending, it would wait for "all loads" in front of the first multiply
  // of every strip).  From here on the only loads in flight are the ring's, R at a time, returning in order.
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int u = 0; u < KTP; ++u) asm volatile("" ::"v"(xf[mt][u]));
  wg_barrier();

  for (int i = 0; i < n_mine; ++i) {
    // the slot a multiply has read is refilled with the step R further on in the wave's stream: the same strip, then
    // the next one -- after the last strip the wave's own activation slice (in bounds, and cache hits rather than
    // weights from HBM once more), so that the loop has no conditional load and exactly R loads are in flight in
    // front of every multiply
    const u32x4_v *wp_next = (i + 1 < n_mine) ? wp + (size_t)gridDim.x * strip_stride
                                              : (const u32x4_v *)a.X + (size_t)kt0 * 64 + lane;
    f32x4_v acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = (f32x4_v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < KTP; ++u) {
      stream_wait<R - 1>(ring[u % R]);  // the oldest of the R loads in flight has landed
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt] = Mfma16::run(ring[u % R], xf[mt][u], acc[mt]);
      stream_load(ring[u % R], u + R < KTP ? wp + (size_t)(u + R) * 64 : wp_next + (size_t)(u + R - KTP) * 64);
    }
    const int buf = i & 1;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) red[buf][w][mt][lane] = acc[mt];
    wg_barrier();
    wp = wp_next;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the over-fetched tail
}

template <class T, int MT, int KTP, int R>
static void launch_rowres_epi(const GemmArgs &a, int epi, int blocks, hipStream_t st) {
  switch (epi) {
    case EPI_QKV: hipLaunchKernelGGL((k_gemm_rowres<T, MT, KTP, R, EPI_QKV>), dim3(blocks), dim3(576), 0, st, a); break;
    case EPI_SWIGLU: hipLaunchKernelGGL((k_gemm_rowres<T, MT, KTP, R, EPI_SWIGLU>), dim3(blocks), dim3(576), 0, st, a); break;
    case EPI_RELU: hipLaunchKernelGGL((k_gemm_rowres<T, MT, KTP, R, EPI_RELU>), dim3(blocks), dim3(576), 0, st, a); break;
    default: hipLaunchKernelGGL((k_gemm_rowres<T, MT, KTP, R, EPI_LOGITS>), dim3(blocks), dim3(576), 0, st, a); break;
  }
}

template <class T>
static bool launch_rowres_t(const GemmArgs &a, int epi, hipStream_t st) {
  if (a.tune & TUNE_ROWRES_OFF) return false;
  if (epi != EPI_QKV && epi != EPI_SWIGLU && epi != EPI_RELU && epi != EPI_LOGITS) return false;
  // Measured on MI355X (d_model 4096): with 9 to 16 rows it beats the streaming kernel by 4 % of a pass (the
  // activation fragments are 8 cache lines per step there, fetched once instead of once per strip); with up to
  // 8 rows (4 lines) the streaming kernel's many short-lived workgroups are 2 % ahead.
  const int m_lo = (a.tune & TUNE_ROWRES_ALWAYS) ? 1 : 9;
  if (a.M < m_lo || a.M > 16 || a.KS != 8) return false;
  const int ktp = a.KT / 8, n_cu = a.n_cu > 0 ? a.n_cu : 256;
  if (a.NT < 2 * n_cu) return false;  // fewer than two strips per workgroup: nothing to keep the rows for
  if (ktp != 16 && ktp != 20) return false;
  int blocks = n_cu;
  if (blocks > a.NT) blocks = a.NT;
  if (ktp == 16) launch_rowres_epi<T, 1, 16, 8>(a, epi, blocks, st);
  else launch_rowres_epi<T, 1, 20, 10>(a, epi, blocks, st);
  return true;
}

bool launch_gemm_rowres(int dtype, const GemmArgs &a, int epi, hipStream_t st) {
  return dtype == SPEC_DTYPE_BF16 ? launch_rowres_t<bf16_t>(a, epi, st) : launch_rowres_t<f16_t>(a, epi, st);
}

}  // namespace spec
