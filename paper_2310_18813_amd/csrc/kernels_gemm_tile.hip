// GEMM for more than 64 activation rows and wide outputs (QKV, gate-up / fc1, LM head).
//
// The streaming kernel covers 64 rows per pass and re-streams the weights for every pass.
// Here one workgroup holds up to 256 rows of a group of weight strips, so a weight byte is
// fetched once per 256 rows, and both operands reach the waves through LDS:
//
//   workgroup = 8 waves = 2 (strip halves) x 4 (row quarters); wave tile = NBW strips x MTW
//   16-row tiles; workgroup tile = 2*NBW strips x 4*MTW row tiles.
//   Per 32-k step the workgroup needs 2*NBW weight fragments and 4*MTW activation
//   fragments of 1 KB each.  Weights and activations are both stored in
//   fragment order in global memory, so a fragment is one 16-byte load per lane, issued two
//   steps ahead, parked in registers and written to the LDS stage that is not being read; the
//   waves then read their fragments back with one 16-byte LDS load per lane, conflict-free.
//
// Results are bit-identical to the streaming kernel: the same instruction, every k-slice a
// chain of MFMAs from zero in ascending k, the slices added in order, the same epilogue code.
#include "mfma_tiles.h"
#include <cstdio>
#include <cstdlib>

namespace spec {

#pragma clang fp contract(off)

// Two LDS stages of fragments; global loads run three steps ahead of the LDS writes through
// three register sets (global -> VGPR -> LDS).  The direct global->LDS path was measured at about
// 18 bytes per clock and CU on this part, a third of what the ordinary load path sustains, so
// it is not used here.
//
// The eight waves work as two groups of four (one wave of each group per SIMD) half a step
// apart: while one group issues the MFMAs of its step, the other does its LDS traffic (fragment
// reads for its next MFMA phase, the hand-over of prefetched global data into the other stage),
// and at the next barrier they swap.  The matrix pipe and the LDS pipe of a SIMD are then busy
// at the same time although every wave runs its phases strictly in order.
template <class T, int MTW, int NBW, int EPI>
__global__ __launch_bounds__(512) void k_gemm_tile(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NBG = 2 * NBW, MTG = 4 * MTW;
  constexpr int FRAGS = NBG + MTG;  // 1 KB fragments per stage
  constexpr int STAGE = FRAGS * 1024;
  constexpr int LPW = (FRAGS + 7) / 8;  // fragments each wave fetches per step
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int grp = w >> 2;               // phase group; waves w and w + 4 share a SIMD
  const int wn = w & 1, wm = ((w >> 1) & 1) | (grp << 1);
  const int c = lane & 15, g = lane >> 4;
  int G, pass;
  if (a.passes == 1) { G = blockIdx.x; pass = 0; }
  else {  // all passes of a strip group on one XCD (see the streaming kernel)
    const int id = blockIdx.x, rest = id >> 3;
    pass = rest % a.passes;
    G = (rest / a.passes) * 8 + (id & 7);
  }
  if (G >= a.groups) return;
  const int nt0 = G * NBG;
  const int mtile0 = pass * MTG;
  const int m_tiles = (a.M + 15) >> 4;

  // fragment f of a stage: f < NBG weight strip nt0 + f; else activation tile f - NBG.
  // Wave w fetches fragments w, w + 8, ...; every wave issues exactly LPW loads per step (a wave with
  // nothing left re-reads its last fragment and drops it) so that one vmcnt value fits all waves.
  const u32x4_v *src[LPW];
  int dst[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int f = w + 8 * i;
    dst[i] = f < FRAGS ? f * 1024 + lane * 16 : -1;
    const int fc = min(f, FRAGS - 1);
    if (fc < NBG) {
      const int nt = min(nt0 + fc, a.NT - 1);
      src[i] = (const u32x4_v *)a.W + (size_t)nt * a.KT * 64 + lane;
    } else {
      const int tile = min(mtile0 + fc - NBG, m_tiles - 1);
      src[i] = (const u32x4_v *)a.X + (size_t)tile * a.KT * 64 + lane;
    }
  }

  f32x4_v cur[NBW][MTW], tot[NBW][MTW];
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
      cur[nb][mt] = (f32x4_v){0.f, 0.f, 0.f, 0.f};
      tot[nb][mt] = (f32x4_v){0.f, 0.f, 0.f, 0.f};
    }

  u32x4_v r0[LPW], r1[LPW], r2[LPW];  // three steps on their way from global memory
  auto fetch = [&](u32x4_v (&r)[LPW], int kt) {
#pragma unroll
    for (int i = 0; i < LPW; ++i) r[i] = src[i][(size_t)min(kt, a.KT - 1) * 64];
  };

  auto stash = [&](const u32x4_v (&r)[LPW], int stage) {
#pragma unroll
    for (int i = 0; i < LPW; ++i)
      if (dst[i] >= 0) *(u32x4_v *)(smem + stage * STAGE + dst[i]) = r[i];
  };
  // A bare barrier, not __syncthreads(): the fence of the latter would wait for the global loads in
  // flight.  Ordered by hand: before it, this wave's LDS reads have returned and its LDS writes are
  // done; nothing may be scheduled across it, so that the phases stay phases.
  auto phase_end = [&]() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
  };

  const int kt_per = a.KT / a.KS;
  int in_slice = 0, slice = 0;
  // prologue: step 0 into LDS stage 0, steps 1, 2 and 3 into the register sets
  fetch(r0, 0);
  fetch(r1, 1);
  fetch(r2, 2);
  stash(r0, 0);
  fetch(r0, 3);
  phase_end();
  if (grp) phase_end();  // the second group runs half a step behind the first

  u32x4_v wf[NBW], xf[MTW];
  // LDS phase of step kt: this wave's fragments of step kt out of stage kt&1; step kt+1, prefetched three
  // steps ago, into the other stage (its last readers finished before the previous barrier: the own
  // group a whole step ago, the other group in the phase just ended); that register set then fetches
  // step kt+4.  The register sets rotate with period three: the loop below is unrolled by three so that
  // each set has a fixed role per copy and the compiler's wait-count bookkeeping stays exact.
#define SPEC_TILE_STEP(rset, kt_)                                                         \
  {                                                                                       \
    const int stage_ = (kt_) & 1;                                                         \
    const unsigned char *sb = smem + stage_ * STAGE + lane * 16;                          \
    _Pragma("unroll") for (int nb = 0; nb < NBW; ++nb)                                    \
        wf[nb] = *(const u32x4_v *)(sb + (wn * NBW + nb) * 1024);                         \
    _Pragma("unroll") for (int mt = 0; mt < MTW; ++mt)                                    \
        xf[mt] = *(const u32x4_v *)(sb + (NBG + wm * MTW + mt) * 1024);                   \
    stash(rset, stage_ ^ 1);                                                              \
    fetch(rset, (kt_) + 4);                                                               \
    phase_end();                                                                          \
    compute();                                                                            \
    phase_end();                                                                          \
  }
  auto compute = [&]() {
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
      for (int mt = 0; mt < MTW; ++mt) cur[nb][mt] = Mfma16::run(wf[nb], xf[mt], cur[nb][mt]);
    __builtin_amdgcn_s_setprio(0);
    if (++in_slice == kt_per) {  // slice finished: add it to the running total, in slice order
#pragma unroll
      for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
          if (slice == 0) tot[nb][mt] = cur[nb][mt];
          else {
            tot[nb][mt][0] += cur[nb][mt][0]; tot[nb][mt][1] += cur[nb][mt][1];
            tot[nb][mt][2] += cur[nb][mt][2]; tot[nb][mt][3] += cur[nb][mt][3];
          }
          cur[nb][mt] = (f32x4_v){0.f, 0.f, 0.f, 0.f};
        }
      in_slice = 0;
      ++slice;
    }
  };
  int kt = 0;
  for (; kt + 2 < a.KT; kt += 3) {
    SPEC_TILE_STEP(r1, kt)
    SPEC_TILE_STEP(r2, kt + 1)
    SPEC_TILE_STEP(r0, kt + 2)
  }
  if (kt < a.KT) SPEC_TILE_STEP(r1, kt)
  if (kt + 1 < a.KT) SPEC_TILE_STEP(r2, kt + 1)
#undef SPEC_TILE_STEP
  if (!grp) phase_end();  // every wave passes the same number of barriers
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // drain the over-fetched tail before the epilogue

#pragma unroll
  for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
      tile_epilogue<T, EPI>(a, tot[nb][mt], nt0 + wn * NBW + nb, (mtile0 + wm * MTW + mt) * 16 + c, g);
}

template <class T, int MTW, int NBW, int EPI>
static void launch_one(const GemmArgs &a, int blocks, hipStream_t st) {
  constexpr size_t lds = 2 * (size_t)(2 * NBW + 4 * MTW) * 1024;
  static bool attr_set = false;  // the kernel may use more than the default 64 KB of LDS
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)k_gemm_tile<T, MTW, NBW, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds);
    attr_set = true;
  }
  hipLaunchKernelGGL((k_gemm_tile<T, MTW, NBW, EPI>), dim3(blocks), dim3(512), lds, st, a);
}

template <class T, int MTW, int NBW>
static void launch_epi_tile(const GemmArgs &a, int epi, int blocks, hipStream_t st) {
  switch (epi) {
    case EPI_QKV: launch_one<T, MTW, NBW, EPI_QKV>(a, blocks, st); break;
    case EPI_SWIGLU: launch_one<T, MTW, NBW, EPI_SWIGLU>(a, blocks, st); break;
    case EPI_RELU: launch_one<T, MTW, NBW, EPI_RELU>(a, blocks, st); break;
    default: launch_one<T, MTW, NBW, EPI_LOGITS>(a, blocks, st); break;
  }
}

template <class T, int MTW>
static void launch_nb_tile(const GemmArgs &a, int NBW, int epi, int blocks, hipStream_t st) {
  if (NBW == 2) launch_epi_tile<T, MTW, 2>(a, epi, blocks, st);
  else if (NBW == 3) launch_epi_tile<T, MTW, 3>(a, epi, blocks, st);
  else launch_epi_tile<T, MTW, 4>(a, epi, blocks, st);
}

// Wave tile (MTW 16-row tiles x NBW strips) for M rows and NT strips.  One workgroup occupies a CU, so
// a launch takes ceil(workgroups / CUs) rounds of KT steps; a step lasts two phases, each as long as the
// slower of one group's MFMAs (16 clocks each) and the other group's LDS traffic (8 clocks per 1 KB
// fragment read or written).  SPEC_GEMM_TILE="mtw,nbw" in the environment overrides the choice (tuning aid).
static void choose_tile(int M, int NT, int n_cu, int &MTW, int &NBW) {
  static int force_mt = -1, force_nb = 0;
  if (force_mt < 0) {
    force_mt = 0;
    const char *e = getenv("SPEC_GEMM_TILE");
    int mt = 0, nb = 0;
    if (e && sscanf(e, "%d,%d", &mt, &nb) == 2 && mt >= 2 && mt <= 4 && nb >= 2 && nb <= 4) { force_mt = mt; force_nb = nb; }
  }
  if (force_mt > 0) { MTW = force_mt; NBW = force_nb; return; }
  long best = -1;
  for (int mt = 2; mt <= 4; ++mt)
    for (int nb = 2; nb <= 4; ++nb) {
      const int passes = (M + 64 * mt - 1) / (64 * mt);
      const int wgs = passes * ((NT + 2 * nb - 1) / (2 * nb));
      const int rounds = (wgs + n_cu - 1) / n_cu;
      const int frags = 2 * nb + 4 * mt;
      const int mfma = mt * nb * 16;
      const int lds = 4 * (mt + nb + 2 * ((frags + 7) / 8)) * 8;  // writes run at half the rate of reads
      const long cost = (long)rounds * (2 * (mfma > lds ? mfma : lds) + 100);
      if (best < 0 || cost < best || (cost == best && mt * nb > MTW * NBW)) { best = cost; MTW = mt; NBW = nb; }
    }
}

template <class T>
static void launch_tile_t(GemmArgs a, int epi, hipStream_t st) {
  static int n_cu = 0;
  if (!n_cu) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n_cu = prop.multiProcessorCount;
    if (n_cu <= 0) n_cu = 256;
  }
  int MTW = 2, NBW = 2;
  choose_tile(a.M, a.NT, n_cu, MTW, NBW);
  a.passes = (a.M + 64 * MTW - 1) / (64 * MTW);
  a.groups = (a.NT + 2 * NBW - 1) / (2 * NBW);
  const int blocks = a.passes == 1 ? a.groups : ((a.groups + 7) / 8) * 8 * a.passes;
  if (MTW == 2) launch_nb_tile<T, 2>(a, NBW, epi, blocks, st);
  else if (MTW == 3) launch_nb_tile<T, 3>(a, NBW, epi, blocks, st);
  else launch_nb_tile<T, 4>(a, NBW, epi, blocks, st);
}

void launch_gemm_tile(int dtype, GemmArgs a, int epi, hipStream_t st) {
  if (dtype == SPEC_DTYPE_BF16) launch_tile_t<bf16_t>(a, epi, st);
  else launch_tile_t<f16_t>(a, epi, st);
}

}  // namespace spec
