// GEMM for more than 64 activation rows (gate-up / fc1 and the LM head: from 33 rows on).
//
// The streaming kernel covers 64 rows per pass and re-streams the weights for every pass.
// Here one workgroup holds up to 256 rows of a group of weight strips, so a weight byte is
// fetched once per up to 256 rows, and both operands reach the waves through LDS:
//
//   workgroup = 8 waves = 2 (strip halves) x 4 (row quarters); wave tile = NBW strips x MTW
//   16-row tiles; workgroup tile = 2*NBW strips x 4*MTW row tiles.
//   Per 32-k step the workgroup needs 2*NBW weight fragments and 4*MTW activation
//   fragments of 1 KB each.  Weights and activations are both stored in fragment order in
//   global memory, so a fragment is one 16-byte load per lane, issued three steps ahead, parked
//   in registers and written to the LDS stage nobody reads; the waves then read their fragments
//   back with one 16-byte LDS load per lane, conflict-free.
//
// Wide outputs (QKV, gate-up / fc1, LM head) walk all of k in one workgroup.  Narrow outputs (the
// residual GEMMs, N = d_model) would leave most CUs idle that way: there each workgroup takes
// one k-slice of its tile (EPI_PARTIAL) and k_partial_reduce adds the slices in slice order.
//
// Results are bit-identical to the streaming kernel: the same instruction, every k-slice a
// chain of MFMAs from zero in ascending k, the slices added in order, the same epilogue code.
#include "mfma_tiles.h"

namespace spec {

#pragma clang fp contract(off)

// Three LDS stages of fragments.  Global loads run three steps ahead of the LDS writes through
// three register sets (global -> VGPR -> LDS; direct global->LDS loads into deeper rings of stages run at
// the same rate on this part and were measured no faster for this loop: the operand stream itself, weights
// from HBM mixed with activations from L2 through one CU's vector L1, is what bounds it).
// The waves read their fragments of step k+1 into a second set of fragment registers before they
// issue the MFMAs of step k, so the LDS pipe, the global loads and the matrix pipe of a SIMD work at
// the same time, with one barrier per step.
template <class T, int MTW, int NBW, int EPI>
__global__ __launch_bounds__(512) void k_gemm_tile(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NBG = 2 * NBW, MTG = 4 * MTW;
  constexpr int FRAGS = NBG + MTG;  // 1 KB fragments per stage
  constexpr int STAGE = FRAGS * 1024;
  constexpr int LPW = (FRAGS + 7) / 8;  // fragments each wave fetches per step
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wn = w & 1, wm = w >> 1;
  const int c = lane & 15, g = lane >> 4;
  constexpr bool PARTIAL = EPI == EPI_PARTIAL;
  int G, pass, slice_id = 0;
  if (!PARTIAL && a.passes == 1) { G = blockIdx.x; pass = 0; }
  else if (PARTIAL && a.KS == 8) {
    // one k-slice per workgroup, and one k-slice per XCD (workgroups are dealt round-robin to the 8 XCDs): all
    // workgroups on an XCD read the same k-slice of the activations, which its L2 then fetches once for the chip
    const int id = blockIdx.x, rest = id >> 3;
    slice_id = id & 7;
    pass = rest % a.passes;
    G = rest / a.passes;
  } else {  // all passes of a strip group on one XCD (see the streaming kernel)
    const int id = blockIdx.x;
    int rest = id >> 3;
    pass = rest % a.passes;
    rest /= a.passes;
    if (PARTIAL) {  // one k-slice per workgroup, the strip groups of a slice neighbours in launch order
      const int gpx = (a.groups + 7) >> 3;
      slice_id = rest / gpx;
      rest %= gpx;
    }
    G = rest * 8 + (id & 7);
  }
  if (G >= a.groups) return;
  const int kt_per = a.KT / a.KS;
  const int KTL = PARTIAL ? kt_per : a.KT;          // steps of this workgroup
  const int kt_lo = PARTIAL ? slice_id * kt_per : 0;  // first k-tile
  const int nt0 = G * NBG;
  const int mtile0 = pass * MTG;
  const int m_tiles = (a.M + 15) >> 4;

  // fragment f of a stage: f < NBG weight strip nt0 + f; else activation tile f - NBG.
  // Wave w fetches fragments w, w + 8, ...; every wave issues exactly LPW loads and LDS writes per step (a
  // wave with nothing left repeats the last fragment: the same bytes to the same place) so that the step is
  // branch-free and one wait count fits all waves.
  const u32x4_v *src[LPW];
  int dst[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int f = w + 8 * i;
    const int fc = min(f, FRAGS - 1);
    dst[i] = fc * 1024 + lane * 16;
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

  // Folded norm.  With one row tile per wave the sum of squares comes from the operand fragments inside the
  // loop (frag_ssq: per lane, one chain per k-slice, slices added in order), where it costs nothing; with larger
  // wave tiles the loop has no issue slots to spare (measured: +10 %) and k_row_inv_x has left 1 / rms per row.
  constexpr bool FOLD_EPI = EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_RELU || EPI == EPI_LOGITS;
  constexpr bool INLOOP = FOLD_EPI && MTW == 1;
  const bool inloop = INLOOP && a.fold_x;
  const bool lnx = a.fold_x && a.wsum;  // the folded norm is a LayerNorm: the plain sums as well
  float ssq_cur = 0.f, ssq_tot = 0.f, sum_cur = 0.f, sum_tot = 0.f;

  u32x4_v r0[LPW], r1[LPW], r2[LPW];  // three steps on their way from global memory
  auto fetch = [&](u32x4_v (&r)[LPW], int kt) {
#pragma unroll
    for (int i = 0; i < LPW; ++i) r[i] = src[i][(size_t)(kt_lo + min(kt, KTL - 1)) * 64];
  };
  auto stash = [&](const u32x4_v (&r)[LPW], int stage) {
#pragma unroll
    for (int i = 0; i < LPW; ++i) *(u32x4_v *)(smem + stage * STAGE + dst[i]) = r[i];
  };
  struct Frags { u32x4_v wf[NBW], xf[MTW]; };
  auto read_frags = [&](Frags &f, int stage) {
    const unsigned char *sb = smem + stage * STAGE + lane * 16;
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) f.wf[nb] = *(const u32x4_v *)(sb + (wn * NBW + nb) * 1024);
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) f.xf[mt] = *(const u32x4_v *)(sb + (NBG + wm * MTW + mt) * 1024);
  };
  // A bare barrier, not __syncthreads(): the fence of the latter would wait for the global loads in
  // flight.  Ordered by hand: before it this wave's LDS writes are done; the NBW + MTW fragment reads
  // issued after them may still be on their way (LDS operations of a wave complete in order).
  auto step_end = [&]() {
    static_assert(NBW + MTW <= 15, "wait count field");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(NBW + MTW) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  int in_slice = 0, slice = 0;
  auto mfmas = [&](const Frags &f) {
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
      for (int mt = 0; mt < MTW; ++mt) cur[nb][mt] = Mfma16::run(f.wf[nb], f.xf[mt], cur[nb][mt]);
    if (inloop) {
      ssq_cur = frag_ssq(f.xf[0], ssq_cur);
      if (lnx) sum_cur = frag_sum(f.xf[0], sum_cur);
    }
  };
  auto slice_end = [&]() {
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
      if (inloop) {
        ssq_tot = slice == 0 ? ssq_cur : ssq_tot + ssq_cur;
        ssq_cur = 0.f;
        sum_tot = slice == 0 ? sum_cur : sum_tot + sum_cur;
        sum_cur = 0.f;
      }
      in_slice = 0;
      ++slice;
    }
  };

  // prologue: steps 0 and 1 into LDS stages 0 and 1, steps 2, 3, 4 into the register sets, fragments of step 0
  Frags f0, f1;
  fetch(r0, 0);
  fetch(r1, 1);
  fetch(r2, 2);
  stash(r0, 0);
  fetch(r0, 3);
  stash(r1, 1);
  fetch(r1, 4);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  read_frags(f0, 0);
  // Step j lives in LDS stage j % 3.  Invariant at the top of step kt: stages kt % 3 and (kt+1) % 3 hold
  // steps kt and kt+1; every wave's reads of stage (kt+2) % 3 (step kt-1) have returned (their MFMAs were
  // issued before the last barrier); the fragment set of parity kt&1 holds step kt or is on its way; the
  // register set of the step holds step kt+2 (possibly still in flight).  Fragment sets alternate, register
  // sets and stages rotate with period three: the loop is unrolled by six so that each has a fixed role
  // per copy and the compiler's wait-count bookkeeping stays exact.
  // The instruction order inside a step is pinned: the LDS queue of the CU is short, and a wave that
  // issues its LDS traffic in one burst waits for queue slots before it reaches its MFMAs.  Spread between
  // the MFMAs (writes first, then reads: the wait before the barrier counts on that order) the LDS and
  // global-memory instructions find their slots while the matrix pipe works.
  auto interleave = [&]() {
    constexpr int NM = NBW * MTW, NO = 2 * LPW + NBW + MTW;  // MFMAs; other instructions: writes, loads, reads
#pragma unroll
    for (int i = 0, o = 0; i < NM; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
      // others due after MFMA i: spread evenly, in program order (writes, global loads, reads)
      const int due = ((i + 1) * NO) / NM;
      for (; o < due; ++o) {
        if (o < LPW) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);            // LDS write
        else if (o < 2 * LPW) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // global load
        else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                    // LDS read
      }
    }
  };
#define SPEC_TILE_STEP(fcur, fnext, rset, kt_, i_)                               \
  {                                                                              \
    stash(rset, ((i_) + 2) % 3);                                                 \
    fetch(rset, (kt_) + 5);                                                      \
    read_frags(fnext, ((i_) + 1) % 3);                                           \
    mfmas(fcur);                                                                 \
    interleave();                                                                \
    slice_end();                                                                 \
    step_end();                                                                  \
  }
  int kt = 0;
  for (; kt + 5 < KTL; kt += 6) {
    SPEC_TILE_STEP(f0, f1, r2, kt, 0)
    SPEC_TILE_STEP(f1, f0, r0, kt + 1, 1)
    SPEC_TILE_STEP(f0, f1, r1, kt + 2, 2)
    SPEC_TILE_STEP(f1, f0, r2, kt + 3, 3)
    SPEC_TILE_STEP(f0, f1, r0, kt + 4, 4)
    SPEC_TILE_STEP(f1, f0, r1, kt + 5, 5)
  }
  if (kt < KTL) SPEC_TILE_STEP(f0, f1, r2, kt, 0)
  if (kt + 1 < KTL) SPEC_TILE_STEP(f1, f0, r0, kt + 1, 1)
  if (kt + 2 < KTL) SPEC_TILE_STEP(f0, f1, r1, kt + 2, 2)
  if (kt + 3 < KTL) SPEC_TILE_STEP(f1, f0, r2, kt + 3, 3)
  if (kt + 4 < KTL) SPEC_TILE_STEP(f0, f1, r0, kt + 4, 4)
#undef SPEC_TILE_STEP
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // drain the over-fetched tail before the epilogue
  // 1 / rms of this lane's rows, fetched only now: the loop has no register to spare for them
  float rv[MTW], mv[MTW];
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt) {
    const int m = (mtile0 + wm * MTW + mt) * 16 + c;
    rv[mt] = 1.0f; mv[mt] = 0.f;
    if (FOLD_EPI && !INLOOP && a.fold_x && m < a.M) {
      rv[mt] = a.rinv_ws[m];
      if (lnx) mv[mt] = a.mean_ws[m];
    }
  }
  if (inloop) {
    if (lnx) row_ln_from_lane(ssq_tot, sum_tot, a.ss_d, a.ss_eps, rv[0], mv[0]);
    else rv[0] = row_inv_from_lane_ssq(ssq_tot, a.ss_d, a.ss_eps);
  }

#pragma unroll
  for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
      const int nt = nt0 + wn * NBW + nb, m = (mtile0 + wm * MTW + mt) * 16 + c;
      if (PARTIAL) {  // the slice's chain as it is; k_partial_reduce adds the slices in order
        const int n = nt * 16 + 4 * g;
        if (nt < a.NT && m < a.M && n < a.N)
          *(f32x4_v *)(a.part + ((size_t)slice_id * a.part_rows + m) * a.N + n) = tot[nb][mt];
      } else {
        tile_epilogue<T, EPI == EPI_PARTIAL ? EPI_RESIDUAL : EPI>(a, tot[nb][mt], nt, m, g,
                                                                 rv[mt], mv[mt]);
      }
    }
}

// ((P_0 + P_1) + ...) + P_{KS-1} for four consecutive outputs; with eight slices all loads go out before the first add
__device__ __forceinline__ f32x4_v sum_slices(const float *__restrict__ p, size_t stride, int KS) {
  if (KS == 8) {
    f32x4_v q[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) q[s] = *(const f32x4_v *)(p + s * stride);
    f32x4_v v = q[0];
#pragma unroll
    for (int s = 1; s < 8; ++s) { v[0] += q[s][0]; v[1] += q[s][1]; v[2] += q[s][2]; v[3] += q[s][3]; }
    return v;
  }
  f32x4_v v = *(const f32x4_v *)p;
  for (int s = 1; s < KS; ++s) {
    const f32x4_v q = *(const f32x4_v *)(p + s * stride);
    v[0] += q[0]; v[1] += q[1]; v[2] += q[2]; v[3] += q[3];
  }
  return v;
}

// Second half of a split residual GEMM: out = ((P_0 + P_1) + ...) + P_{KS-1}, then the same epilogue as
// everywhere (scale, bias, h += out).  One thread per four consecutive outputs of a row.
template <class T>
__global__ __launch_bounds__(256) void k_partial_reduce(GemmArgs a) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int n4 = a.N >> 2;
  if (idx >= (size_t)a.M * n4) return;
  const int m = (int)(idx / n4), n = (int)(idx % n4) * 4;
  const float *p = a.part + (size_t)m * a.N + n;
  const size_t stride = (size_t)a.part_rows * a.N;
  tile_epilogue<T, EPI_RESIDUAL>(a, sum_slices(p, stride, a.KS), n >> 4, m, (n & 15) >> 2);
}


// The same reduction, one workgroup per row, for the producer of the next GEMM's activations.  After the update the
// row's fp16-rounded values sit in LDS, and one thread per (k-slice of the next GEMM, lane group) adds their squares
// up exactly as that GEMM would take them from its operand fragments (frag_ssq: eight consecutive elements per 32-k
// step, ascending, one chain per k-slice); the slices are added in order, then the lane groups as
// row_inv_from_lane_ssq pairs them: a.rinv_ws[m] = 1 / rms of the row, the very bits k_row_inv_x would leave --
// which then need not run.  a.ssq_ks = the k-slices of the next GEMM (at most 8).
// A LayerNorm folded into the next GEMM (a.mean_ws set) wants the plain sums too, taken the same way (frag_sum):
// a.mean_ws[m] = the row's mean and a.rinv_ws[m] = 1 / std, as row_ln_from_lane computes them.
template <class T>
__global__ __launch_bounds__(1024) void k_partial_reduce_rows(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char reduce_smem[];
  op_t *xs = (op_t *)reduce_smem;  // [N] fp16: the updated row as the next GEMM will read it
  __shared__ float ssq_s[8][4];
  const int m = blockIdx.x, n4 = a.N >> 2;
  const size_t stride = (size_t)a.part_rows * a.N;
  for (int i = threadIdx.x; i < n4; i += blockDim.x) {
    const int n = i * 4;
    const float *p = a.part + (size_t)m * a.N + n;
    op_t o4[4];
    residual_update(a, sum_slices(p, stride, a.KS), n, m, o4);
    *(uint2 *)(xs + n) = *(const uint2 *)o4;
  }
  __syncthreads();
  const int steps = (a.N >> 5) / a.ssq_ks;
  __shared__ float sum_s2[8][4];
  const bool lnx = a.mean_ws != nullptr;  // the next GEMM folds a LayerNorm: the plain sums and the mean as well
  if ((int)threadIdx.x < a.ssq_ks * 4) {
    const int w = threadIdx.x >> 2, g = threadIdx.x & 3;
    float s = 0.f, t = 0.f;
    for (int u = 0; u < steps; ++u) {
      const u32x4_v f = *(const u32x4_v *)(xs + (w * steps + u) * 32 + g * 8);
      s = frag_ssq(f, s);
      if (lnx) t = frag_sum(f, t);
    }
    ssq_s[w][g] = s;
    sum_s2[w][g] = t;
  }
  __syncthreads();
  if (threadIdx.x < 4) {  // one lane per lane group: the slices in order, then the pairs as the GEMM kernels add them
    const int g = threadIdx.x;
    float t = ssq_s[0][g], ts = sum_s2[0][g];
    for (int w = 1; w < a.ssq_ks; ++w) { t += ssq_s[w][g]; ts += sum_s2[w][g]; }
    t += __shfl_xor(t, 1, 64);
    t += __shfl_xor(t, 2, 64);
    ts += __shfl_xor(ts, 1, 64);
    ts += __shfl_xor(ts, 2, 64);
    if (g == 0) {
      if (lnx) {
        const float mean = ts / (float)a.ss_d, var = fmaxf(t / (float)a.ss_d - mean * mean, 0.f);
        a.rinv_ws[m] = 1.0f / sqrtf(var + a.ss_eps);
        a.mean_ws[m] = mean;
      } else {
        a.rinv_ws[m] = 1.0f / sqrtf(t / (float)a.ss_d + a.ss_eps);
      }
    }
  }
}

// 1 / rms of every row of the fp16 activations X, in exactly the order the GEMM kernels add the squares up
// themselves (frag_ssq): one workgroup per 16-row tile, wave w walks k-slice w, the slice sums meet in LDS and are
// added in slice order.  For the tiled kernel with more than one row tile per wave.
__global__ __launch_bounds__(512) void k_row_inv_x(const void *__restrict__ X, int M, int KT, int KS, int d, float eps,
                                                   float *__restrict__ rinv, float *__restrict__ mean_out) {
  __shared__ float ssq_s[8][64];
  __shared__ float sum_s[8][64];
  const bool lnx = mean_out != nullptr;  // folded LayerNorm: mean and 1 / std instead of 1 / rms
  float t = 0.f;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, c = lane & 15, g = lane >> 4;
  const int tile = blockIdx.x, kt_per = KT / KS;
  const u32x4_v *xp = (const u32x4_v *)X + (size_t)tile * KT * 64 + lane;
  float s = 0.f;
  int kt = w * kt_per;
  const int kt1 = kt + kt_per;
  for (; kt + 8 <= kt1; kt += 8) {
    u32x4_v xf[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) xf[u] = xp[(size_t)(kt + u) * 64];
#pragma unroll
    for (int u = 0; u < 8; ++u) s = frag_ssq(xf[u], s);
    if (lnx) {
#pragma unroll
      for (int u = 0; u < 8; ++u) t = frag_sum(xf[u], t);
    }
  }
  for (; kt < kt1; ++kt) {
    const u32x4_v f = xp[(size_t)kt * 64];
    s = frag_ssq(f, s);
    if (lnx) t = frag_sum(f, t);
  }
  if (KS > 1) {
    ssq_s[w][lane] = s;
    sum_s[w][lane] = t;
    __syncthreads();
    s = ssq_s[0][lane];
    t = sum_s[0][lane];
    for (int i = 1; i < KS; ++i) { s += ssq_s[i][lane]; t += sum_s[i][lane]; }
  }
  float v, mean = 0.f;
  if (lnx) row_ln_from_lane(s, t, d, eps, v, mean);
  else v = row_inv_from_lane_ssq(s, d, eps);
  const int m = tile * 16 + c;
  if (w == 0 && g == 0 && m < M) {
    rinv[m] = v;
    if (lnx) mean_out[m] = mean;
  }
}

template <class T, int MTW, int NBW, int EPI>
static void launch_one(const GemmArgs &a, int blocks, hipStream_t st) {
  constexpr size_t lds = 3 * (size_t)(2 * NBW + 4 * MTW) * 1024;
  if (blocks < 0) {  // preparation pass: the kernel may use more than the default 64 KB of LDS
    (void)hipFuncSetAttribute((const void *)k_gemm_tile<T, MTW, NBW, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds);
    return;
  }
  hipLaunchKernelGGL((k_gemm_tile<T, MTW, NBW, EPI>), dim3(blocks), dim3(512), lds, st, a);
}

template <class T, int MTW, int NBW>
static void launch_epi_tile(const GemmArgs &a, int epi, int blocks, hipStream_t st) {
  switch (epi) {
    case EPI_QKV: launch_one<T, MTW, NBW, EPI_QKV>(a, blocks, st); break;
    case EPI_SWIGLU: launch_one<T, MTW, NBW, EPI_SWIGLU>(a, blocks, st); break;
    case EPI_RELU: launch_one<T, MTW, NBW, EPI_RELU>(a, blocks, st); break;
    case EPI_PARTIAL: launch_one<T, MTW, NBW, EPI_PARTIAL>(a, blocks, st); break;
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
// a launch takes ceil(workgroups / CUs) rounds of KT steps.  Measured on MI355X a step costs about
// 150 + 45 * MTW * NBW + 40 * (MTW + NBW) clocks (two waves per SIMD at 16 clocks per MFMA are 32 of the
// 45; the last term is the LDS traffic).
static void choose_tile(int M, int NT, int n_cu, int steps, int wg_mult, int &MTW, int &NBW) {
  long best = -1;
  for (int mt = 1; mt <= 4; ++mt)
    for (int nb = 2; nb <= 4; ++nb) {
      const int passes = (M + 64 * mt - 1) / (64 * mt);
      const int wgs = passes * ((NT + 2 * nb - 1) / (2 * nb)) * wg_mult;
      const int rounds = (wgs + n_cu - 1) / n_cu;
      // per round: the steps, plus filling the pipeline and the epilogue (about 2 us)
      const long cost = (long)rounds * ((long)steps * (150 + 45 * mt * nb + 40 * (mt + nb)) + 5000);
      if (best < 0 || cost < best || (cost == best && mt * nb > MTW * NBW)) { best = cost; MTW = mt; NBW = nb; }
    }
}

// wave tile of the launch for these arguments (epi as given by the caller, EPI_RESIDUAL = split by k-slice)
static void tile_for(const GemmArgs &a, int epi, int &MTW, int &NBW) {
  const int f_mt = a.tune & TUNE_TILE_MTW_MASK, f_nb = (a.tune >> TUNE_TILE_NBW_SHIFT) & 0xf;
  if (f_mt >= 1 && f_mt <= 4 && f_nb >= 2 && f_nb <= 4) { MTW = f_mt; NBW = f_nb; return; }  // test / tuning aid
  const bool split = epi == EPI_RESIDUAL;
  MTW = 2; NBW = 2;
  choose_tile(a.M, a.NT, a.n_cu > 0 ? a.n_cu : 256, split ? a.KT / a.KS : a.KT, split ? a.KS : 1, MTW, NBW);
}

// With more than one row tile per wave the kernel reads 1 / rms of its rows from a.rinv_ws: the caller runs
// launch_row_inv_x first when this says so.
bool gemm_tile_wants_row_inv(const GemmArgs &a, int epi) {
  if (!a.fold_x || (epi != EPI_QKV && epi != EPI_SWIGLU && epi != EPI_RELU && epi != EPI_LOGITS)) return false;
  int MTW, NBW;
  tile_for(a, epi, MTW, NBW);
  return MTW > 1;
}
void launch_row_inv_x(const GemmArgs &a, hipStream_t st) {
  if (a.M <= 0) return;
  hipLaunchKernelGGL(k_row_inv_x, dim3((a.M + 15) / 16), dim3(a.KS * 64), 0, st, a.X, a.M, a.KT, a.KS, a.ss_d, a.ss_eps, a.rinv_ws,
                     a.wsum ? a.mean_ws : nullptr);
}

template <class T>
static void launch_tile_t(GemmArgs a, int epi, hipStream_t st) {
  int MTW, NBW;
  tile_for(a, epi, MTW, NBW);
  const bool split = epi == EPI_RESIDUAL;  // narrow outputs: one k-slice per workgroup, slices added by a second kernel
  if (split) epi = EPI_PARTIAL;
  a.passes = (a.M + 64 * MTW - 1) / (64 * MTW);
  a.groups = (a.NT + 2 * NBW - 1) / (2 * NBW);
  const int blocks = split ? (a.KS == 8 ? a.groups * a.passes * 8 : ((a.groups + 7) / 8) * 8 * a.passes * a.KS)
                           : a.passes == 1 ? a.groups : ((a.groups + 7) / 8) * 8 * a.passes;
  if (MTW == 1) launch_nb_tile<T, 1>(a, NBW, epi, blocks, st);
  else if (MTW == 2) launch_nb_tile<T, 2>(a, NBW, epi, blocks, st);
  else if (MTW == 3) launch_nb_tile<T, 3>(a, NBW, epi, blocks, st);
  else launch_nb_tile<T, 4>(a, NBW, epi, blocks, st);
  const int rr_threads = std::min(1024, ((a.N >> 2) + 63) / 64 * 64);  // one float4 of outputs per thread where that fits
  if (split && a.ssq_ks > 0 && a.x_out) {
    hipLaunchKernelGGL(k_partial_reduce_rows<T>, dim3(a.M), dim3(rr_threads), (size_t)a.N * sizeof(op_t), st, a);
  } else if (split) {
    const size_t total = (size_t)a.M * (a.N >> 2);
    hipLaunchKernelGGL(k_partial_reduce<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
  }
}

void gemm_tile_prepare() {
  GemmArgs a{};
  for (int epi : {(int)EPI_QKV, (int)EPI_SWIGLU, (int)EPI_RELU, (int)EPI_PARTIAL, (int)EPI_LOGITS})
    for (int nbw = 2; nbw <= 4; ++nbw) {
      launch_nb_tile<bf16_t, 1>(a, nbw, epi, -1, nullptr); launch_nb_tile<f16_t, 1>(a, nbw, epi, -1, nullptr);
      launch_nb_tile<bf16_t, 2>(a, nbw, epi, -1, nullptr); launch_nb_tile<f16_t, 2>(a, nbw, epi, -1, nullptr);
      launch_nb_tile<bf16_t, 3>(a, nbw, epi, -1, nullptr); launch_nb_tile<f16_t, 3>(a, nbw, epi, -1, nullptr);
      launch_nb_tile<bf16_t, 4>(a, nbw, epi, -1, nullptr); launch_nb_tile<f16_t, 4>(a, nbw, epi, -1, nullptr);
    }
}

void launch_gemm_tile(int dtype, GemmArgs a, int epi, hipStream_t st) {
  if (dtype == SPEC_DTYPE_BF16) launch_tile_t<bf16_t>(a, epi, st);
  else launch_tile_t<f16_t>(a, epi, st);
}

}  // namespace spec
