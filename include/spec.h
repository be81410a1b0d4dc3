/*
 * spec.h -- C ABI of the MI355X (gfx950) library for batched greedy speculative
 * decoding: the draft model proposes s tokens for each of B sequences, the
 * target model verifies all B*(s+1) tokens in one forward pass, the longest
 * matching prefix plus one target token is accepted, the KV caches are committed
 * or rolled back, and a profiled look-up table picks s for each batch size
 * (paper: Alg. 1 and Sec. 2 "Speculative Decoding"; Sec. 3.1 for the batched
 * form; Sec. 4 for the adaptive policy).
 *
 * Conventions
 *   - Every function returns an int status: SPEC_OK or a SPEC_ERR_* code.  Nothing
 *     throws or aborts.  spec_last_error() returns a message for the most recent
 *     failure on that context (or the most recent failure without a context).
 *   - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  Structures
 *     (descriptors, spec_weights itself, the layer_tensors array) live on the host;
 *     the tensors they point to live on the device.
 *   - The library never allocates or frees device memory.  The caller owns the
 *     weights, the workspace and the HIP stream and keeps them alive until
 *     spec_destroy.  spec_init re-packs the weights into the workspace; the
 *     caller's weight tensors are not read after spec_init returns.
 *   - Step calls (reset, draft_step, verify_step, accept_commit, round) enqueue
 *     work on the context's stream and return without waiting.  Calls that hand
 *     data back to the host (read_output, read_state, profile_and_choose_s)
 *     synchronise the stream.
 *   - A call that fails validation leaves all state untouched.  Arguments are
 *     validated before any device call, so misuse is reported without a GPU.
 *   - One context must not be used from two threads at once.
 *
 * Notation (per sequence b): n_b = committed length (prompt + emitted tokens);
 * the "pending" token is the last committed one, x_{n_b-1}, whose target KV is
 * not yet written; t_1..t_s are the proposals for positions n_b..n_b+s-1;
 * o_0..o_s are the target logits, o_i predicting position n_b+i; a_i = argmax o_i;
 * l_b = number of accepted proposals.
 */
#ifndef SPEC_H
#define SPEC_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

enum {
  SPEC_OK = 0,
  SPEC_ERR_INVALID_ARG = 1, /* null pointer, value out of range                       */
  SPEC_ERR_WORKSPACE = 2,   /* workspace missing, too small or misaligned             */
  SPEC_ERR_STATE = 3,       /* call out of order                                      */
  SPEC_ERR_CAPACITY = 4,    /* B, s or sequence length beyond what spec_init reserved */
  SPEC_ERR_UNSUPPORTED = 5, /* model shape / option this build has no kernel for      */
  SPEC_ERR_HIP = 6          /* a HIP runtime call failed                              */
};

/* Storage type of the weights handed in and of the KV cache.  Arithmetic: fp32 runs on plain fp32 ALU
   kernels; the 16-bit types run their GEMMs on the matrix cores with fp16 operands and fp32 sums (bf16
   weights are held as fp16 times a power of two per matrix, which is exact for all but vanishing
   elements; activations are rounded from fp32 to fp16 and saturate at +-65504), attention on the
   matrix cores in the storage type; residual stream, norms and softmax in fp32.                       */
enum { SPEC_DTYPE_F32 = 0, SPEC_DTYPE_BF16 = 1, SPEC_DTYPE_F16 = 2 };
enum { SPEC_FFN_SWIGLU = 0, SPEC_FFN_RELU = 1 };
enum { SPEC_NORM_RMS = 0, SPEC_NORM_LAYER = 1 };
enum { SPEC_POS_ROPE = 0, SPEC_POS_LEARNED = 1 };
enum { SPEC_PROPOSALS_DRAFT = 0, SPEC_PROPOSALS_EXTERNAL = 1 };
enum { SPEC_MODEL_TARGET = 0, SPEC_MODEL_DRAFT = 1 };

/* Per-layer tensor slots of spec_weights.layer_tensors (n_layers * SPEC_T_COUNT
   device pointers, layer-major).  Every matrix is row-major [out][in]; every
   tensor has the run's dtype.  Unused slots may be NULL.                        */
enum {
  SPEC_T_ATTN_NORM_W = 0, SPEC_T_ATTN_NORM_B, /* [d]; _B for LayerNorm only                */
  SPEC_T_WQ, SPEC_T_BQ, SPEC_T_WK, SPEC_T_BK, /* [d][d], [d]; biases only if has_bias      */
  SPEC_T_WV, SPEC_T_BV, SPEC_T_WO, SPEC_T_BO,
  SPEC_T_FFN_NORM_W, SPEC_T_FFN_NORM_B,
  SPEC_T_W1, SPEC_T_B1, /* SwiGLU: gate [f][d], no bias | ReLU: fc1 [f][d], bias [f]       */
  SPEC_T_W3,            /* SwiGLU: up   [f][d]          | ReLU: unused                     */
  SPEC_T_W2, SPEC_T_B2, /* SwiGLU: down [d][f], no bias | ReLU: fc2 [d][f], bias [d]       */
  SPEC_T_COUNT
};

typedef struct spec_ctx spec_ctx; /* opaque; host memory owned by the library */

/* A decoder-only transformer.  LLaMA shape: RMSNorm, rotary positions (rotate-half
   pairing, element i with i + head_dim/2), SwiGLU, no biases.  OPT shape: LayerNorm,
   learned absolute positions (row p of pos_emb for position p), ReLU FFN, biases.
   Pre-norm residual blocks, attention scale 1/sqrt(head_dim), untied LM head.
   head_dim = d_model / n_heads must be 64 or 128 for 16-bit runs.                 */
typedef struct {
  int32_t n_layers, d_model, n_heads, d_ffn, vocab, max_pos;
  int32_t ffn_kind, norm_kind, pos_kind, has_bias;
  float norm_eps, rope_theta;
} spec_model_desc;

typedef struct {
  const void *d_tok_emb;           /* [vocab][d]                          */
  const void *d_pos_emb;           /* [max_pos][d], learned positions only */
  const void *d_final_norm_w;      /* [d]                                 */
  const void *d_final_norm_b;      /* [d], LayerNorm only                 */
  const void *d_lm_head;           /* [vocab][d]                          */
  const void *const *layer_tensors; /* host array, n_layers * SPEC_T_COUNT device pointers */
} spec_weights;

typedef struct {
  int32_t dtype;         /* SPEC_DTYPE_*: storage type of weights, activations and KV cache;
                            accumulation, softmax, norms and the residual stream are fp32  */
  int32_t B_max;         /* most sequences in one batch                                    */
  int32_t s_max;         /* longest speculation length                                     */
  int32_t L_max;         /* KV-cache positions per sequence; needs P + gen_max + s_max     */
  int32_t gen_max;       /* tokens to emit per sequence; a sequence that reached it is
                            frozen (still computed, emits nothing)                         */
  int32_t eos_id;        /* end-of-sequence token the context starts with, -1 = none (every
                            workload of the paper generates a fixed count); see spec_set_eos   */
  int32_t proposal_mode; /* SPEC_PROPOSALS_DRAFT: t_j = the draft model's greedy token.
                            SPEC_PROPOSALS_EXTERNAL: t_j supplied by the caller; a draft
                            model, if present, still runs and ingests those tokens          */
} spec_run_desc;

const char *spec_last_error(const spec_ctx *ctx_or_null);

/* Bytes of device workspace spec_init needs (packed weights of both models, both KV
   caches, activations, per-sequence state).  drf may be NULL (no draft model).        */
int spec_workspace_bytes(const spec_model_desc *tgt, const spec_model_desc *drf,
                         const spec_run_desc *run, size_t *bytes);

/* Create a context.  d_workspace: device memory, 256-byte aligned, at least
   spec_workspace_bytes() large, owned by the caller.  hip_stream: a hipStream_t
   (NULL = the default stream).  Re-packs both weight sets into the workspace
   (device-side; synchronises the stream before returning).  drf / drf_w may both be
   NULL; then s > 0 needs SPEC_PROPOSALS_EXTERNAL.                                     */
int spec_init(const spec_model_desc *tgt, const spec_weights *tgt_w,
              const spec_model_desc *drf, const spec_weights *drf_w,
              const spec_run_desc *run, void *d_workspace, size_t workspace_bytes,
              void *hip_stream, spec_ctx **out);
int spec_destroy(spec_ctx *ctx);

/* Start a batch of B sequences, each with the P prompt tokens d_prompt[b][0..P-1]
   (int32, device).  Runs the prompt's first P-1 tokens through both models to fill
   their KV caches (the prefill the paper's runtime model leaves out, Sec. 3.3); the
   last prompt token becomes the pending token.  Needs 1 <= B <= B_max, P >= 1,
   P + gen_max + s_max <= L_max (and <= max_pos for learned positions), token ids in
   [0, vocab) (ids are clamped on the device, not checked).                           */
int spec_reset(spec_ctx *ctx, int32_t B, const int32_t *d_prompt, int32_t P);

/* As spec_reset for prompts of different lengths: row b of d_prompt ([B][P_stride], int32, device) holds the
   h_len[b] prompt tokens of sequence b (h_len: host, B entries, 1 <= h_len[b] <= P_stride; the rest of a row
   is ignored).  One batch prefill over the longest prompt, rows beyond a sequence's own prompt being dead
   rows of the pass; the capacity rules of spec_reset apply to the longest prompt.  Every sequence emits up to
   gen_max tokens after its own prompt.  Synchronises the stream once (the lengths go to the device).       */
int spec_reset_ragged(spec_ctx *ctx, int32_t B, const int32_t *d_prompt, int32_t P_stride, const int32_t *h_len);

/* As spec_reset but without touching the KV caches: the caller provides positions
   0..P-2 through spec_kv_import.  For micro-benchmarks and tests that start from a
   given cache.                                                                        */
int spec_reset_noprefill(spec_ctx *ctx, int32_t B, const int32_t *d_prompt, int32_t P);

/* Continuous batching (beyond the paper, which decodes fixed batches): batch slot b, 0 <= b < B, starts
   over with the P prompt tokens d_prompt[0..P-1] (int32, device).  P need not be the length given to
   spec_reset: every slot keeps its own prompt length (P >= 1, P + gen_max + s_max <= L_max, and <= max_pos for
   learned positions; SPEC_ERR_CAPACITY otherwise).  The slot's emitted tokens are dropped (read them with
   spec_read_output first), its prompt is run through both models in a single-sequence pass, and from the next
   round on it decodes beside the others, whose state and results do not change.  spec_rewind takes every slot
   back to its own prompt.  Not allowed between a round's first draft or verify step and its
   spec_accept_commit (SPEC_ERR_STATE).  With an external proposal table the caller updates row b of the
   table it owns.  Counters and the accepted-length histogram keep running for the whole batch.           */
int spec_admit(spec_ctx *ctx, int32_t b, const int32_t *d_prompt, int32_t P);

/* A speculation length per sequence (beyond the paper, whose rounds use one s for the whole batch):
   d_s[b] (int32, device, B entries, the caller's memory, read by every round until replaced) caps the
   proposals of sequence b.  A round called with s then verifies min(s, d_s[b]) proposals for sequence b:
   its rows for further proposals are dead (no cache write, no attention, logits ignored) and its draft
   steps beyond the cap are skipped the same way; the pass still has B * (s + 1) rows.  Negative entries count
   as 0.  NULL (the default) removes the caps.  spec_profile_and_choose_s ignores them.  Not allowed inside a
   round (SPEC_ERR_STATE).  Emitted tokens do not depend on the caps (Sec. 2).                            */
int spec_set_seq_s(spec_ctx *ctx, const int32_t *d_s_or_null);

/* End-of-sequence token (beyond the paper, whose sequences all run to a fixed length): once a sequence has
   emitted eos_token it stops for good — the tokens the same round accepted behind it are dropped, its length no
   longer moves, spec_read_output returns it up to and including the end token — until its slot is given a new
   prompt (spec_admit) or the batch starts over (spec_reset*, spec_rewind).  -1 (the default) means none.  Takes
   effect from the next spec_accept_commit; sequences already stopped stay stopped.  spec_profile_and_choose_s
   ignores it.  Not allowed inside a round (SPEC_ERR_STATE).                                                 */
int spec_set_eos(spec_ctx *ctx, int32_t eos_token);

/* Back to the state right after the last reset (lengths, counters, emitted tokens);
   cached prompt KV is kept.                                                           */
int spec_rewind(spec_ctx *ctx);

/* External proposals, one of:
   - spec_set_proposal_table: d_table[b][pos] (int32, row stride L_max) is the proposal
     for absolute position pos of sequence b; each round reads t_j = table[b][n_b+j-1]
     on the device, so rounds need no host round-trip.  The table must stay alive.
   - spec_set_proposals: explicit t_1..t_s for the coming round, d_tok[b][0..s-1];
     call it before the round's first draft step.
   Both need SPEC_PROPOSALS_EXTERNAL.                                                  */
int spec_set_proposal_table(spec_ctx *ctx, const int32_t *d_table);
int spec_set_proposals(spec_ctx *ctx, const int32_t *d_tok, int32_t s);

/* Draft step j (1-based) of the current round: the call speculate(S, kv_SSM, s) of
   Alg. 1 is s of these in order.  Step 1 ingests the committed tokens the draft has
   not read yet (one or two per sequence after a round with draft steps; one more for
   every round that ran without them, ingested in as many passes as it takes), step
   j >= 2 ingests t_{j-1}; each appends the draft's KV and, in SPEC_PROPOSALS_DRAFT
   mode, writes t_j = argmax.                                                          */
int spec_draft_step(spec_ctx *ctx, int32_t j);

/* Target verification: the call LLM(S, t_1..t_s, kv_LLM) of Alg. 1.  One forward pass
   over B*(s+1) rows -- the pending token and the s proposals of every sequence -- at
   positions n_b-1 .. n_b+s-1, attending to the cached prefix plus, causally, each
   other; appends their K/V provisionally and leaves a_0..a_s per sequence on the
   device.  d_logits_or_null: if not NULL receives o_0..o_s as fp32
   [B][s+1][vocab] (debug / parity; costs an extra B*(s+1)*vocab*4 bytes of writes).  */
int spec_verify_step(spec_ctx *ctx, int32_t s, float *d_logits_or_null);

/* Acceptance and commit (Sec. 2; Alg. 1): l_b = number of leading proposals with
   t_j = a_{j-1}; emit t_1..t_l, a_l; n_b += l_b+1; target cache length n_b-1; draft
   cache length n_old + min(l_b, s-1).  Rejected positions are dropped by length only
   (Sec. 3.1 masks them; the result is the same) and overwritten next round.          */
int spec_accept_commit(spec_ctx *ctx, int32_t s);

/* n_rounds complete rounds at speculation length s: [proposals from the table] ->
   s draft steps -> verify -> accept/commit.  Same effect as the single calls.        */
int spec_round(spec_ctx *ctx, int32_t s, int32_t n_rounds);

/* Sec. 4, profiling stage.  For every batch size h_batch_sizes[i] (ascending) and
   every s in 0..s_max_profile: reset with the first B rows of d_prompt ([maxB][P]),
   run one untimed warm-up round, rewind, then time max(1, gen / (s+1)) rounds with HIP
   events (that many rounds cannot finish a sequence, so every timed round does full
   work) and record microseconds per emitted token per sequence, the per-token latency
   of the paper's Fig. 1: the time of a round at (B, s) divided by the tokens a sequence
   emits per round at that s, the latter pooled over all batch sizes of the call (it does
   not depend on B, and one small batch holds too few acceptance draws to estimate it).
   The LUT entry is the s with the lowest value, the smaller s winning ties within 1 %.  The LUT is kept in
   the context for spec_choose_s.  h_lut_out: [n_b]; h_grid_us_per_tok_or_null:
   [n_b][s_max_profile+1].  Needs gen <= gen_max.  In SPEC_PROPOSALS_EXTERNAL mode a
   proposal table must be set.  Synchronises; leaves the context rewound on the last
   profiled batch.                                                                     */
int spec_profile_and_choose_s(spec_ctx *ctx, const int32_t *h_batch_sizes, int32_t n_b,
                              int32_t s_max_profile, const int32_t *d_prompt, int32_t P,
                              int32_t gen, int32_t *h_lut_out, float *h_grid_us_per_tok_or_null);

/* Install a LUT measured elsewhere (h_batch_sizes ascending). */
int spec_set_lut(spec_ctx *ctx, const int32_t *h_batch_sizes, const int32_t *h_lut, int32_t n_b);

/* Sec. 4, execution stage: s for a batch of B.  A profiled B returns its entry; an
   un-profiled B the smaller entry of its two nearest profiled sizes; B beyond the
   profiled range the entry of the nearest end.                                        */
int spec_choose_s(const spec_ctx *ctx, int32_t B, int32_t *h_s_out);

/* Emitted tokens so far: h_tokens [B][gen_max] (row stride gen_max), h_len [B].
   h_hist_or_null: [s_max+1] counts of rounds*sequences by accepted length l.         */
int spec_read_output(spec_ctx *ctx, int32_t *h_tokens, int32_t *h_len, int64_t *h_hist_or_null);

/* 16-bit runs feed their GEMMs fp16 operands: an activation beyond +-65504 (the residual stream of the layer
   input, an FFN activation) is clamped to that range on the way, silently as far as the tokens go.  *h_count
   receives how many values were clamped since spec_init (0 for fp32 runs and for every workload of this
   repository; a non-zero count says the model's activations do not fit this build's operand type).  Synchronises. */
int spec_read_saturation(spec_ctx *ctx, int64_t *h_count);

/* Per-sequence state for tests: any pointer may be NULL.  h_n [B] committed lengths,
   h_kv_draft [B] draft cache lengths, h_l_last [B] accepted count of the last round,
   h_argmax [B][s_max+1] the a_i of the last verify step.                             */
int spec_read_state(spec_ctx *ctx, int32_t *h_n, int32_t *h_kv_draft, int32_t *h_l_last, int32_t *h_argmax);

/* Copy KV-cache rows between the caller's canonical layout and the library's private
   one.  d_k, d_v: [B][len][d_model] in the run's dtype (keys as stored, i.e. after the
   rotary embedding); positions 0..len-1 of the first B sequences of one layer.        */
int spec_kv_import(spec_ctx *ctx, int32_t which_model, int32_t layer, int32_t B, int32_t len,
                   const void *d_k, const void *d_v);
int spec_kv_export(spec_ctx *ctx, int32_t which_model, int32_t layer, int32_t B, int32_t len,
                   void *d_k, void *d_v);

/* Parity aid: if d_hidden is not NULL, every following target pass (verify step or prefill
   chunk) also copies its fp32 residual stream into d_hidden as [n_layers + 1][M][d_model]:
   slice 0 after the embedding, slice l after layer l (M = rows of that pass).  NULL turns it
   off.  The buffer is the caller's and must hold (n_layers + 1) * B_max * 16 * d_model floats. */
int spec_set_hidden_dump(spec_ctx *ctx, float *d_hidden);

/* Greedy tokens and acceptance on logits the caller already has, without a context: for a caller that runs the
   target model itself (Alg. 1: a_i = argmax o_i; Sec. 2: a proposal is accepted while every earlier one
   was, then the target's own token follows).
     d_logits     [B][s+1][vocab] fp32, device: o_0..o_s of every sequence
     d_proposals  [B][s] int32, device: t_1..t_s (may be NULL when s = 0)
     d_accepted   [B] int32, device, out: l_b
     d_emitted    [B][s+1] int32, device, out: t_1..t_l, a_l, then -1
     d_workspace  device scratch for the arg-max partials, 8-byte aligned, at least
                  spec_greedy_accept_workspace_bytes(B, s, vocab) bytes; contents before and after are of no meaning
   Ties go to the lowest token id; a row of NaNs yields token 0.  Enqueues two kernels on hip_stream (NULL = the
   default stream) and returns without waiting.  Limits: s <= 15, B <= 65535, vocab <= 2^28 (SPEC_ERR_CAPACITY);
   SPEC_ERR_WORKSPACE for a missing, misaligned or short workspace.  All buffers are the caller's.             */
int spec_greedy_accept_workspace_bytes(int32_t B, int32_t s, int32_t vocab, size_t *bytes);
int spec_greedy_accept(void *hip_stream, const float *d_logits, const int32_t *d_proposals, int32_t B, int32_t s,
                       int32_t vocab, void *d_workspace, size_t workspace_bytes, int32_t *d_accepted,
                       int32_t *d_emitted);

/* spec_greedy_accept for callers that cannot allocate or pass a workspace (code under HIP graph capture, tight
   serving loops, harnesses that forbid hipMalloc): the same kernels, with the arg-max partials in a 1 MiB array
   built into the library (one copy per GPU, held until the process ends).  Calls no allocating routine.
   Limit: B * (s + 1) * ceil(vocab / 4096) <= 131072, SPEC_ERR_CAPACITY beyond (e.g. 16384 rows of a 32000-token
   vocabulary).  Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two
   threads) race; calls on one stream are ordered and need no clearing in between.                               */
int spec_greedy_accept_noalloc(void *hip_stream, const float *d_logits, const int32_t *d_proposals, int32_t B,
                               int32_t s, int32_t vocab, int32_t *d_accepted, int32_t *d_emitted);

/* Speculative sampling: the non-greedy form of the acceptance step.  Sec. 2 describes speculative decoding and
   cites this rule for sampling from the models instead of taking their most likely token; Alg. 1 is the greedy
   case.  With q_j = softmax(draft logits of step j / T) and p_j = softmax(target logits of row j / T):
   proposal t_j is kept if u * q_j[t_j] < p_j[t_j]; at the first j that fails one token drawn from
   max(0, p_j - q_j), normalised, is emitted and the round ends; if all s are kept, one token drawn from p_{s+1}
   follows.  The emitted tokens are distributed as if the target alone had been sampled.  Proposals that were not
   drawn from a distribution count as point masses (q_j[t_j] = 1).  A draw from weights w with a uniform number u
   takes the smallest index whose cumulative weight exceeds u * sum(w).  Arithmetic: fp32.

   Every random number is the caller's: uniform numbers in [0, 1), three per decided token --
   [.][0] draws a proposal, [.][1] decides whether it is kept, [.][2] draws the token emitted at that place.

   spec_sample_tokens: one draw per row.  d_logits [rows][vocab] fp32, d_uniforms [rows], d_tokens [rows] out.
   spec_sample_accept: the rule for B sequences on logits the caller has.
     d_target_logits [B][s+1][vocab]; d_draft_logits [s][B][vocab] (step-major), or NULL for point-mass proposals;
     d_proposals [B][s] (may be NULL when s = 0); d_uniforms [B][s+1][3], row j for the token at place j of the round
     ([.][j][0] is not read); out: d_chosen [B][s+1] (the token chosen at each place up to the one that ended the
     round, -1 behind it), d_accepted [B] = l_b, d_emitted [B][s+1] = the l_b kept proposals, the drawn token, -1.
   Both enqueue on hip_stream (NULL = the default stream), need no context and no workspace, and do not wait.
   temperature > 0, s <= 15 (SPEC_ERR_INVALID_ARG, SPEC_ERR_CAPACITY).  All device pointers, all the caller's.

   spec_set_sampling: the same rule inside a context, for every following round (spec_draft_step draws t_j, the
   verify step applies the rule; commit, roll-back, end token, budgets and per-sequence s work as in the greedy
   case).  d_uniforms [B_max][L_max][3] is indexed by sequence slot and by the absolute position of the token a
   number decides, so a token's random numbers do not depend on how the rounds fall.  The library needs the logits
   of a round in memory: d_target_logits [B_max * (s_max + 1)][vocab] and, with SPEC_PROPOSALS_DRAFT,
   d_draft_logits [s_max][B_max][vocab], both fp32 device buffers of the caller's, written every round (their
   contents after a round are that round's logits: tests read them).  External proposals are point masses.
   d_uniforms = NULL switches back to the greedy rule.  Only between rounds (SPEC_ERR_STATE).                    */
int spec_sample_tokens(void *hip_stream, const float *d_logits, int32_t rows, int32_t vocab, float temperature,
                       const float *d_uniforms, int32_t *d_tokens);
int spec_sample_accept(void *hip_stream, const float *d_target_logits, const float *d_draft_logits,
                       const int32_t *d_proposals, const float *d_uniforms, int32_t B, int32_t s, int32_t vocab,
                       float temperature, int32_t *d_chosen, int32_t *d_accepted, int32_t *d_emitted);
int spec_set_sampling(spec_ctx *ctx, float temperature, const float *d_uniforms, float *d_target_logits,
                      float *d_draft_logits);

/* Parity aids for the draft step (the call speculate(S, kv_SSM, s) of Alg. 1).
   spec_set_draft_logits: if d_logits is not NULL, every following spec_draft_step also writes the draft
   model's logits behind t_j -- the logits of the last token each sequence fed in -- as fp32 [B][vocab]
   into d_logits (the caller's device memory, B_max * vocab floats); NULL turns it off.  Needs a draft model
   (SPEC_ERR_STATE otherwise).
   spec_read_proposals: the proposals of the current round, h_t [B][s_max] (row stride s_max): t_1..t_j after
   draft step j in SPEC_PROPOSALS_DRAFT mode, the external ones once they were fetched.  Synchronises.      */
int spec_set_draft_logits(spec_ctx *ctx, float *d_logits);
int spec_read_proposals(spec_ctx *ctx, int32_t *h_t);

/* Measurement aid: what this GPU delivers, for roofline fractions against measured as well as nominal peaks.
   Streams d_buf (device, 16-byte aligned, `bytes` long; at least 64 KB per compute unit, a few hundred MB
   to be beyond every cache) once per repetition with plain 16-byte loads, and issues the GEMM kernels' MFMA
   instruction (f32 += f16 x f16, 16x16x32) back to back on every SIMD; the best of two timed repetitions of
   each goes to *h_hbm_gbs (GB/s) and *h_mfma_tflops (TFLOP/s).  The buffer is only read.  Runs on hip_stream
   and waits for it.  Needs no context.  SPEC_ERR_CAPACITY if the buffer is too small.                       */
int spec_measure_peaks(void *hip_stream, void *d_buf, size_t bytes, double *h_hbm_gbs, double *h_mfma_tflops);

/* Test aid: pin the launch shape of the 16-bit verify attention.  0 = chosen from the batch size
   (default), 1 = one wave per (sequence, head, chunk) plus a merge kernel, 2 = one wave per
   (sequence, head), 3 = one workgroup per (sequence, head) with a wave per chunk (falls back to 1 beyond 8
   chunks).  Results must not depend on it.                                          */
int spec_set_attention_shape(spec_ctx *ctx, int32_t shape);

/* Test and tuning aid: pin launch shapes of the 16-bit GEMMs.  tile_mtw x tile_nbw (1..4 x 2..4; 0, 0 = chosen
   from the shape) is the wave tile of the LDS-tiled kernel (more than 64 rows); flags: bit 0 = never take the
   row-resident kernel, bit 1 = take it for every row count it covers (1..16) instead of the 9..16 where it is
   the faster one.  Results must not depend on any of it.                                                      */
int spec_set_gemm_tuning(spec_ctx *ctx, int32_t tile_mtw, int32_t tile_nbw, int32_t flags);

/* Per-kernel timing for benchmarks.  While enabled, every launch of the target model's
   kernels is bracketed by a HIP event pair on the context's stream (this adds a few
   microseconds per launch: leave it off in production).  spec_read_kernel_timing
   synchronises, adds up the elapsed time per kernel class since the last read and clears
   the record.  h_count, h_ms: [SPEC_KCLASS_COUNT].                                        */
enum {
  SPEC_KCLASS_GEMM_QKV = 0,   /* QKV projection + rotary + KV append            */
  SPEC_KCLASS_GEMM_O,         /* attention output projection + residual         */
  SPEC_KCLASS_GEMM_FFN_IN,    /* gate/up (or fc1) projection + activation       */
  SPEC_KCLASS_GEMM_FFN_OUT,   /* down (or fc2) projection + residual            */
  SPEC_KCLASS_GEMM_HEAD,      /* LM head + arg-max partials                     */
  SPEC_KCLASS_ATTENTION,      /* verify attention (both kernels)                */
  SPEC_KCLASS_NORM,           /* norm kernels (fp32 path); 16-bit path: the row
                                 statistics kernel of the norms folded into GEMMs */
  SPEC_KCLASS_OTHER,          /* embedding, arg-max merge, accept/commit        */
  SPEC_KCLASS_DRAFT_PASS,     /* one whole forward pass of the draft model      */
  SPEC_KCLASS_COUNT
};
int spec_kernel_timing(spec_ctx *ctx, int32_t enable);
int spec_read_kernel_timing(spec_ctx *ctx, int64_t *h_count, double *h_ms);

#ifdef __cplusplus
}
#endif
#endif
