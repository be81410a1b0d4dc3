// Internal declarations shared by the host runtime and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>
#include <string>
#include <vector>
#include "../../include/spec.h"
#include "mfma_gemm.h"

namespace spec {

constexpr int WAVE = 64;
constexpr int KV_VBLOCK = 8;  // values of 8 consecutive positions are stored together (see kv_v_index)
constexpr int KV_LPAD = 32;   // cache rows per sequence are padded to the attention kernel's 32-key step

// ---------------------------------------------------------------- layouts
// KV cache of one model: for each layer a K area and a V area, each
// [B_max][H][L_pad][hd] elements, L_pad = L_max rounded up to KV_LPAD.
//   K: row-major over positions; inside a row the head's elements are stored
//      pair-interleaved: canonical element i (i < hd/2) sits at 2i, its rotary
//      partner i + hd/2 at 2i+1.  Q is produced in the same order, so q.k is unchanged.
//   V: blocked by KV_VBLOCK positions: [pos / 8][hd][pos % 8], canonical element order,
//      so that 8 consecutive positions of one element are one 16-byte load.
__host__ __device__ inline int hd_interleave(int i, int hd) {
  int half = hd >> 1;
  return i < half ? 2 * i : 2 * (i - half) + 1;
}
__host__ __device__ inline size_t kv_k_index(int L_pad, int H, int hd, int b, int h, int pos, int i_stored) {
  return (((size_t)b * H + h) * L_pad + pos) * hd + i_stored;
}
__host__ __device__ inline size_t kv_v_index(int L_pad, int H, int hd, int b, int h, int pos, int i) {
  return ((((size_t)b * H + h) * (L_pad / KV_VBLOCK) + pos / KV_VBLOCK) * hd + i) * KV_VBLOCK + pos % KV_VBLOCK;
}

// ---------------------------------------------------------------- model on device
struct LayerW {
  // canonical-layout copies used by the generic kernels, or packed tiles for the MFMA kernels
  const void *attn_norm_w, *attn_norm_b, *ffn_norm_w, *ffn_norm_b;
  const void *wqkv, *bqkv;  // [3d][d] (rows: q heads, k heads, v heads), bias [3d]
  const void *wo, *bo;      // [d][d]
  const void *w13, *b13;    // SwiGLU: [2f][d] gate/up rows; ReLU: [f][d]
  const void *w2, *b2;      // [d][f]
  float s_qkv = 1.f, s_o = 1.f, s_13 = 1.f, s_2 = 1.f;  // MFMA path: 1 / scale of the packed fp16 weights
  const float *wsum_qkv = nullptr, *wsum_13 = nullptr;   // MFMA path, folded LayerNorm: row sums of the packed weights
};

struct Model {
  bool present = false;
  spec_model_desc desc{};
  int hd = 0, L_pad = 0;
  bool fast = false;  // MFMA kernels (16-bit dtypes with supported shapes) or generic kernels
  // MFMA path: the norms live inside the GEMMs behind them (gain in the packed weights, 1 / rms in the epilogue)
  bool fold_ln = false;    // ... and they are LayerNorms (mean taken out in the epilogue, bias pushed through the weights)
  const float *wsum_head = nullptr, *b_head = nullptr;
  const void *tok_emb = nullptr, *pos_emb = nullptr, *final_norm_w = nullptr, *final_norm_b = nullptr,
             *lm_head = nullptr;
  std::vector<LayerW> layers;
  PackedDims p_qkv{}, p_o{}, p_13{}, p_2{}, p_head{};  // MFMA path: packed shapes
  float s_head = 1.f;                                  // MFMA path: 1 / scale of the packed LM head
  const float2 *rope = nullptr;                        // MFMA path: (cos, sin) table [L_max][hd/2]
  void *kcache = nullptr, *vcache = nullptr;  // [n_layers] x area
  size_t kv_area_elems = 0;                   // elements per layer per K (or V) area
  int32_t *kv_len = nullptr;                  // draft only: device [B_max] valid cache length
};

// What a forward pass feeds in.
enum PassKind {
  PASS_VERIFY = 0,      // rows (b,i), i=0..q-1: pending token then proposals, positions n_b-1+i
  PASS_DRAFT_FIRST = 1, // rows (b,i): committed tokens at positions n_b-j-q+i; rows before kv_len_b are dead
  PASS_DRAFT_NEXT = 2,  // q = 1: proposal t_{j-1} at position n_b+j-2
  PASS_PREFILL = 3      // rows (b,i): prompt tokens at positions base+i; rows >= P-1 are dead
};

struct Workspace {
  // activations (shared by both models; sized for the larger)
  float *h = nullptr;       // [M_max][d]   fp32 residual stream
  void *x = nullptr;        // [M_max][d]   normed rows, model dtype (MFMA path: fp16 operands, as attn and act)
  void *q = nullptr;        // [M_max][d]   queries, pair-interleaved per head: fp32 (matrix-core path) or model dtype (generic)
  void *attn = nullptr;     // [M_max][d]   attention output, model dtype
  void *act = nullptr;      // [M_max][f]   FFN activation, model dtype
  float *y32 = nullptr;     // [M_max][max(3d, 2f)] fp32 GEMM output (generic path)
  float *logits = nullptr;  // [M_max][vocab] fp32 (generic path / debug)
  float *attn_part = nullptr, *attn_ml = nullptr;  // split-KV partials (MFMA path)
  float *row_mean = nullptr;                       // [M_max] their means (folded LayerNorm)
  float *row_inv = nullptr;                        // [M_max] 1 / rms of the rows of h (folded norm, tiled GEMM with large wave tiles)
  float *gemm_part = nullptr;                      // k-slice sums of the split residual GEMMs (M_max > 32)
  float *head_part = nullptr;                      // per-strip arg-max partials (MFMA path)
  int32_t *head_part_idx = nullptr;
  int32_t *row_tok = nullptr, *row_pos = nullptr, *row_seq = nullptr;  // [M_max]
};

struct State {
  int32_t *seq = nullptr;     // [B_max][L_max] committed tokens (prompt + emitted)
  int32_t *n = nullptr;       // [B_max] committed length
  int32_t *P_b = nullptr;     // [B_max] prompt length of the sequence in the slot (admissions may differ from the batch's)
  int32_t *gen_cap = nullptr; // [B_max] tokens the sequence may emit: gen_max, or fewer once it has emitted the end token
  int32_t *t = nullptr;       // [B_max][s_max]   proposals of the round
  int32_t *a = nullptr;       // [B_max][s_max+1] target greedy tokens of the round
  int32_t *l_last = nullptr;  // [B_max]
  int32_t *draft_arg = nullptr;  // [B_max] where the draft's greedy token goes when the proposals come from outside
  unsigned long long *hist = nullptr;  // [s_max+1]
  unsigned long long *counters = nullptr;  // [0] emitted tokens total, [1] rounds
  unsigned int *sat = nullptr;             // activations clamped to the fp16 range since spec_init (matrix-core path)
};

}  // namespace spec

struct spec_ctx {
  spec_run_desc run{};
  spec::Model tgt, drf;
  spec::Workspace ws;
  spec::State st;
  hipStream_t stream = nullptr;
  int M_max = 0;
  int NC_max = 1;         // attention chunks that cover L_max
  int n_ub = 0;           // host upper bound of every sequence's committed length
  // host-side bookkeeping
  int B = 0, P = 0;       // current batch; P: prompt length given to the last reset
  int32_t eos = -1;       // end-of-sequence token (-1: none)
  std::vector<int32_t> P_host;  // [B] prompt length per slot (host mirror of st.P_b)
  bool active = false;
  int draft_j = 0;        // draft steps done this round
  int draft_lag = 1;      // upper bound of n_b - kv_draft_b
  int verified_s = -1;    // s of the verify step waiting for accept_commit, or -1
  bool proposals_ready = false;
  const int32_t *prop_table = nullptr;
  const int32_t *seq_s = nullptr;  // [B] per-sequence cap of the speculation length (caller's device memory), or null
  float *hidden_dump = nullptr;
  float *draft_logits = nullptr;  // parity aid: where every draft step leaves the logits behind its proposals
  // speculative sampling (off while smp_u is null): temperature, the caller's table of uniform numbers
  // [B_max][L_max][3], and the caller's buffers for the target's logits [M_max][vocab] and the draft's
  // [s_max][B_max][vocab] of a round
  bool x_ssq = false;  // ws.row_inv already holds 1 / rms of the rows now in ws.x (left by a split residual GEMM)
  float smp_T = 0.f;
  const float *smp_u = nullptr;
  float *smp_tl = nullptr, *smp_dl = nullptr;
  int attn_shape = 0;
  int gemm_tune = 0;      // GemmTune bits (spec_set_gemm_tuning)
  int n_cu = 256;         // compute units of the context's device
  std::vector<int32_t> lut_B, lut_s;
  std::string err;
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  // optional per-kernel-class timing (spec_kernel_timing)
  bool kt_on = false;
  std::vector<hipEvent_t> kt_ev;   // start/stop pairs
  std::vector<int> kt_cls;         // class of pair i
  size_t kt_used = 0;              // pairs recorded since the last read
};

namespace spec {
// Brackets the launches of one kernel class with a HIP event pair while timing is on.
struct KScope {
  spec_ctx *c;
  size_t slot = 0;
  bool on;
  KScope(spec_ctx *ctx, int cls) : c(ctx), on(ctx->kt_on && cls >= 0) {
    if (!on) return;
    if (c->kt_used * 2 + 2 > c->kt_ev.size()) {
      hipEvent_t a = nullptr, b = nullptr;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
      c->kt_ev.push_back(a);
      c->kt_ev.push_back(b);
      c->kt_cls.push_back(cls);
    }
    slot = c->kt_used++;
    c->kt_cls[slot] = cls;
    (void)hipEventRecord(c->kt_ev[2 * slot], c->stream);
  }
  ~KScope() {
    if (on) (void)hipEventRecord(c->kt_ev[2 * slot + 1], c->stream);
  }
};
}  // namespace spec

namespace spec {

// ---- launchers implemented in the kernel files (all asynchronous on `st`) ----
struct PassArgs {
  PassKind kind;
  int B, q;      // rows M = B*q
  int j;         // draft step index (PASS_DRAFT_NEXT) / prefill base position (PASS_PREFILL) /
                 // PASS_DRAFT_FIRST: how many positions before n_b the pass ends (0: at n_b - 1)
  int P;         // prompt length (PASS_PREFILL)
  int s_max, L_max;
  int b0 = 0;    // first batch slot of the pass: its rows are the sequences b0 .. b0 + B - 1
  int seq_groups = 1;  // PASS_PREFILL: this many consecutive groups of q rows belong to one sequence (B counts groups):
                       // group g of a sequence holds positions base + g*q .. and all its groups share the sequence's cache
};

void launch_assemble_embed(const spec_ctx *c, const Model &m, const PassArgs &pa, hipStream_t st);
void launch_norm(const spec_ctx *c, const Model &m, const float *h, const void *gain, const void *bias, void *x,
                 int M, int last_of_q, hipStream_t st);
void launch_argmax_rows(const float *logits, int M, int V, int q, int out_stride, int32_t *out, hipStream_t st);
void launch_accept(spec_ctx *c, int s, hipStream_t st);
// speculative sampling (kernels_sampling.hip): one draw per row from softmax(logits / T); the verification of a
// round's proposals, which leaves in a[] the tokens under which the longest-matching-prefix rule gives the outcome
void launch_sample_rows(const float *logits, int rows, int V, float temperature, const float *u, const int32_t *n, int off,
                        int u_rows, int32_t *out, int out_stride, hipStream_t st);
void launch_sample_verify(const float *tl, const float *dl, int d_rows, int B, int s, int V, float temperature,
                          const int32_t *t, int t_stride, const int32_t *seq_s, const float *u, const int32_t *n, int u_rows,
                          int32_t *a, int a_stride, hipStream_t st);
void launch_fill_proposals(spec_ctx *c, int s, hipStream_t st);
void launch_copy_proposals(spec_ctx *c, const int32_t *d_tok, int s, hipStream_t st);
void launch_state_reset(spec_ctx *c, const int32_t *d_prompt, int P_stride, bool ragged, hipStream_t st);
void launch_state_admit(spec_ctx *c, int b, const int32_t *d_prompt, int P, hipStream_t st);
void launch_kv_convert(spec_ctx *c, const Model &m, int layer, int B, int len, void *k, void *v, bool import_,
                       hipStream_t st);

// generic kernels (any dtype, any shape)
void generic_repack_top(spec_ctx *c, Model &m, const spec_weights *w, void *&cursor, hipStream_t st);
void generic_repack_layer(spec_ctx *c, Model &m, int layer, const spec_weights *w, void *&cursor, hipStream_t st);
void generic_layer(spec_ctx *c, const Model &m, int layer, int M, int q_rows, int b0, int seq_groups, hipStream_t st);
void generic_head(spec_ctx *c, const Model &m, int Mh, int last_of_q, float *logits, hipStream_t st);
size_t generic_packed_bytes(const spec_model_desc &d, int dtype);
void generic_copy(const void *src, void *dst, size_t bytes, hipStream_t st);
void generic_zero(void *dst, size_t bytes, hipStream_t st);

size_t dtype_bytes(int dtype);
int fail_noctx(int code, const char *fmt, ...);  // records the message spec_last_error(NULL) returns; returns code

// matrix-core path (16-bit dtypes)
bool fast_supported(const spec_model_desc &D, int dtype);
size_t fast_packed_bytes(const spec_model_desc &D, int dtype, int L_max);
bool fast_setup_model(spec_ctx *c, Model &m, const spec_weights *w, void *&cursor, hipStream_t st);  // false: HIP error
void fast_layer(spec_ctx *c, const Model &m, int layer, int B, int q_rows, int b0, int seq_groups, int max_pos, hipStream_t st);
void fast_head(spec_ctx *c, const Model &m, int Mh, int last_of_q, float *logits_or_null, int q, int arg_stride,
               int32_t *arg_out, hipStream_t st);

}  // namespace spec
