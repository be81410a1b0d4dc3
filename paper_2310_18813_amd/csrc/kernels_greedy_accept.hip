// Greedy tokens and acceptance on logits the caller already has (Sec. 2; Alg. 1): for a caller that runs the
// target model itself and wants only a_i = argmax o_i, the accepted count l_b and the emitted tokens.
//
// Two kernels.  k_ga_partials: one workgroup per (row, 4096-logit chunk) leaves the chunk's (value, index)
// arg-max in scratch.  k_ga_accept: one wave per sequence reduces the chunks of its s + 1 rows (lowest index wins
// ties, at every stage) and applies the first-mismatch rule.  Every partial the second kernel reads was written by
// the first in the same call, so the scratch needs no clearing.
//
// The scratch is the caller's workspace (spec_greedy_accept) or a file-scope device array
// (spec_greedy_accept_noalloc, for callers that cannot allocate).
#include "spec_internal.h"
#include "device_utils.h"
#include <mutex>

namespace spec {

constexpr int GA_CHUNK = 4096;                      // logits per first-stage workgroup

struct GaPartial { float v; int32_t i; };

__global__ __launch_bounds__(256) void k_ga_partials(const float *__restrict__ logits, int V, int n_chunks,
                                                     GaPartial *__restrict__ part) {
  __shared__ float shv[4];
  __shared__ int shi[4];
  const int row = blockIdx.x, chunk = blockIdx.y;
  const float *src = logits + (size_t)row * V;
  const int c0 = chunk * GA_CHUNK, c1 = min(c0 + GA_CHUNK, V);
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int c = c0 + threadIdx.x; c < c1; c += 256) argmax_combine(bv, bi, src[c], c);
  wave_argmax(bv, bi);
  if ((threadIdx.x & 63) == 0) { shv[threadIdx.x >> 6] = bv; shi[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) argmax_combine(bv, bi, shv[w], shi[w]);
    part[(size_t)row * n_chunks + chunk] = GaPartial{bv, bi};
  }
}

// One wave per sequence.  emitted: t_1..t_l, a_l, then -1 up to s + 1 entries.
__global__ __launch_bounds__(64) void k_ga_accept(const GaPartial *__restrict__ part, int n_chunks, int V, int s,
                                                  const int32_t *__restrict__ proposals, int32_t *__restrict__ accepted,
                                                  int32_t *__restrict__ emitted) {
  __shared__ int a_sh[16];
  const int b = blockIdx.x, lane = threadIdx.x;
  for (int i = 0; i <= s; ++i) {
    const GaPartial *p = part + (size_t)(b * (s + 1) + i) * n_chunks;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int c = lane; c < n_chunks; c += 64) argmax_combine(bv, bi, p[c].v, p[c].i);
    wave_argmax(bv, bi);
    if (lane == 0) a_sh[i] = (bi < 0 || bi >= V) ? 0 : bi;
  }
  __syncthreads();
  if (lane == 0) {
    const int32_t *t = proposals + (size_t)b * s;
    int l = 0;
    while (l < s && t[l] == a_sh[l]) ++l;
    accepted[b] = l;
    int32_t *e = emitted + (size_t)b * (s + 1);
    for (int i = 0; i <= s; ++i) e[i] = i < l ? t[i] : (i == l ? a_sh[l] : -1);
  }
}

static int ga_check(const char *who, const float *d_logits, const int32_t *d_proposals, int B, int s, int vocab,
                    const int32_t *d_accepted, const int32_t *d_emitted) {
  if (!d_logits || !d_accepted || !d_emitted || (s > 0 && !d_proposals))
    return fail_noctx(SPEC_ERR_INVALID_ARG, "%s: null argument", who);
  if (B < 1 || vocab < 1 || s < 0) return fail_noctx(SPEC_ERR_INVALID_ARG, "%s: B and vocab must be positive, s non-negative", who);
  if (s > 15 || B > 65535 || vocab > (1 << 28))
    return fail_noctx(SPEC_ERR_CAPACITY, "%s: at most s = 15, B = 65535, vocab = 2^28", who);
  return SPEC_OK;
}
static size_t ga_bytes(int B, int s, int vocab) {
  const size_t n_chunks = ((size_t)vocab + GA_CHUNK - 1) / GA_CHUNK;
  return (size_t)B * (s + 1) * n_chunks * sizeof(GaPartial);
}
static int ga_launch(hipStream_t st, const float *d_logits, const int32_t *d_proposals, int B, int s, int vocab, void *scratch,
                     int32_t *d_accepted, int32_t *d_emitted) {
  const int n_chunks = (vocab + GA_CHUNK - 1) / GA_CHUNK;
  hipLaunchKernelGGL(k_ga_partials, dim3(B * (s + 1), n_chunks), dim3(256), 0, st, d_logits, vocab, n_chunks, (GaPartial *)scratch);
  hipLaunchKernelGGL(k_ga_accept, dim3(B), dim3(64), 0, st, (const GaPartial *)scratch, n_chunks, vocab, s, d_proposals,
                     d_accepted, d_emitted);
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? SPEC_OK : fail_noctx(SPEC_ERR_HIP, "greedy accept launch: %s", hipGetErrorString(e));
}

}  // namespace spec

using namespace spec;

extern "C" int spec_greedy_accept_workspace_bytes(int32_t B, int32_t s, int32_t vocab, size_t *bytes) {
  if (!bytes || B < 1 || s < 0 || vocab < 1)
    return fail_noctx(SPEC_ERR_INVALID_ARG, "spec_greedy_accept_workspace_bytes: bytes is null, or B, s or vocab out of range");
  if (s > 15 || B > 65535 || vocab > (1 << 28))
    return fail_noctx(SPEC_ERR_CAPACITY, "spec_greedy_accept_workspace_bytes: at most s = 15, B = 65535, vocab = 2^28");
  *bytes = ga_bytes(B, s, vocab);
  return SPEC_OK;
}

extern "C" int spec_greedy_accept(void *hip_stream, const float *d_logits, const int32_t *d_proposals, int32_t B, int32_t s,
                                  int32_t vocab, void *d_workspace, size_t workspace_bytes, int32_t *d_accepted,
                                  int32_t *d_emitted) {
  int rc = ga_check("spec_greedy_accept", d_logits, d_proposals, B, s, vocab, d_accepted, d_emitted);
  if (rc) return rc;
  if (!d_workspace || ((uintptr_t)d_workspace & 7) != 0 || workspace_bytes < ga_bytes(B, s, vocab))
    return fail_noctx(SPEC_ERR_WORKSPACE, "spec_greedy_accept: workspace null, not 8-byte aligned, or smaller than %zu bytes",
                      ga_bytes(B, s, vocab));
  return ga_launch((hipStream_t)hip_stream, d_logits, d_proposals, B, s, vocab, d_workspace, d_accepted, d_emitted);
}

// ---------------------------------------------------------------- no-allocation variant
namespace spec {
constexpr size_t GA_STATIC_BYTES = 1u << 20;  // 131072 (row, chunk) partials: e.g. 1024 rows of a 500k vocabulary, 16384 rows of a 32k one
constexpr int GA_MAX_DEVICES = 64;
// The no-allocation variant's scratch.  In host code this name is a stand-in, not a device address: the address
// comes from hipGetSymbolAddress, once per device (every GPU holds its own copy of the array).
static __device__ __align__(256) unsigned char ga_scratch[GA_STATIC_BYTES];
static void *g_ga_scratch_ptr[GA_MAX_DEVICES];
static std::mutex g_ga_mutex;

// Device address of the current device's copy of the scratch array; null on failure.
static void *ga_static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= GA_MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_ga_mutex);
  if (!g_ga_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(ga_scratch)) != hipSuccess) return nullptr;
    g_ga_scratch_ptr[dev] = p;
  }
  return g_ga_scratch_ptr[dev];
}
}  // namespace spec

extern "C" int spec_greedy_accept_noalloc(void *hip_stream, const float *d_logits, const int32_t *d_proposals, int32_t B,
                                          int32_t s, int32_t vocab, int32_t *d_accepted, int32_t *d_emitted) {
  int rc = ga_check("spec_greedy_accept_noalloc", d_logits, d_proposals, B, s, vocab, d_accepted, d_emitted);
  if (rc) return rc;
  if (ga_bytes(B, s, vocab) > GA_STATIC_BYTES)
    return fail_noctx(SPEC_ERR_CAPACITY,
                      "spec_greedy_accept_noalloc: B * (s + 1) * ceil(vocab / %d) = %zu partials exceed the built-in scratch of %zu; "
                      "use spec_greedy_accept with a workspace",
                      GA_CHUNK, ga_bytes(B, s, vocab) / sizeof(GaPartial), GA_STATIC_BYTES / sizeof(GaPartial));
  void *scratch = ga_static_scratch();
  if (!scratch) return fail_noctx(SPEC_ERR_HIP, "spec_greedy_accept_noalloc: hipGetSymbolAddress failed for the scratch array");
  return ga_launch((hipStream_t)hip_stream, d_logits, d_proposals, B, s, vocab, scratch, d_accepted, d_emitted);
}
