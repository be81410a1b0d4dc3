// Declarations of the matrix-core kernels (GEMM with fused epilogues, attention).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spec {

enum GemmEpilogue {
  EPI_RESIDUAL = 0,  // h[m][n] += y            (O projection, down projection / fc2)
  EPI_QKV = 1,       // rotary on q,k; q -> buffer, k,v -> cache at the row's position
  EPI_SWIGLU = 2,    // act[m][j] = silu(gate_j) * up_j
  EPI_RELU = 3,      // act[m][n] = max(y, 0)
  EPI_LOGITS = 4,    // per-strip arg-max partials (+ optional fp32 logits dump)
  EPI_PARTIAL = 5    // tiled kernel only: raw fp32 sums of one k-slice -> part[slice][m][n]
};

struct PackedDims {
  int N, K, N_pad, K_pad, NT, KT, KS;
  size_t bytes(size_t esz) const { return (size_t)N_pad * K_pad * esz; }
};
PackedDims packed_dims(int N, int K);
// k-slices of a GEMM with KT 32-k steps: fixed by the shape alone (it fixes the order of every sum)
inline int gemm_ks_for(int KT) { return (KT % 8 == 0) ? 8 : (KT % 4 == 0) ? 4 : (KT % 2 == 0) ? 2 : 1; }

struct GemmArgs {
  // operands
  const void *W;      // packed tiles
  const float *bias;  // [N_pad] in stored-row order, or null
  const void *X;      // fp16 activations in fragment order (xpack_index), ceil(M/16) x KT tiles
  float out_scale;    // 1 / (power of two the packed weights were multiplied by)
  int M, N, NT, KT, KS, K_pad;
  int passes, groups;  // filled by the launcher
  unsigned int *sat;   // counts activations clamped to the fp16 range on their way to a GEMM operand (or null)
  int n_cu;            // compute units of the device (0: 256)
  int tune;            // launch-shape overrides of spec_set_gemm_tuning (0: none); never change a result
  // epilogue targets (those the chosen epilogue uses)
  float *h;                  // EPI_RESIDUAL: [M][N] fp32
  // RMS norm folded into the GEMMs around it: the gain sits in the packed weights of the consumer, whose
  // activations are the fp16-rounded rows of h themselves, written by the producer of h; the consumer's
  // epilogue multiplies by 1 / rms of the row, which it takes from the operand fragments it reads anyway.
  int fold_x;                // consumer: norm folded in (row length ss_d, epsilon ss_eps)
  int ss_d;
  float ss_eps;
  int ssq_ks;                // producer (below): the k-slices of the GEMM that will consume x_out, gemm_ks_for(N / 32); else 0
  // consumer (tiled kernel with more than one row tile per wave): [M] 1 / rms per row, left by k_row_inv_x or by the
  // split residual GEMM that produced X.  producer (EPI_RESIDUAL, split by k-slice, x_out set, ssq_ks > 0): where the
  // 1 / rms of the updated rows goes (row length ss_d = N, epsilon ss_eps).
  float *rinv_ws;
  void *x_out;               // EPI_RESIDUAL producer: fp16 copy of the updated rows, fragment order
  // LayerNorm folded into the GEMM behind it: (W diag(g)) (x - mean) / std + (W b + bias) = ((W diag(g)) x - mean * wsum) / std
  // + bias', with wsum[n] the sum of row n of the packed weights (in their scaled units) and bias' folded at set-up.
  // consumer: wsum non-null says the folded norm is a LayerNorm; mean_ws [M]: the row means where the kernel reads
  // 1 / std from rinv_ws instead of taking both from its operand fragments.  producer (row-wise reduction): where the
  // mean goes beside rinv_ws.
  const float *wsum;
  float *mean_ws;
  float *part;               // EPI_RESIDUAL with more than 64 rows: scratch [KS][part_rows][N] fp32, or null
  int part_rows;             // M rounded up to 16
  void *q, *kc, *vc;         // EPI_QKV: q [M][d] fp32 (un-rounded: the attention kernel decides how to feed it), caches in the model dtype
  const int32_t *row_pos;    // EPI_QKV: absolute position per row, -1 = dead row
  const float2 *rope;        // EPI_QKV: (cos, sin) table [L][hd/2] or null
  int q_rows, d, hd, H, L_pad;
  int seq_groups;            // EPI_QKV: consecutive groups of q_rows rows per sequence (0 or 1: one)
  void *act;                 // EPI_SWIGLU / EPI_RELU: fp16, fragment order, row length f (resp. N)
  int f;
  float *logits;             // EPI_LOGITS: optional [M][N] fp32
  int logit_step;            // EPI_LOGITS: > 1: only the last row of every group of logit_step rows is dumped, as row m / logit_step
  float *part_val;           // EPI_LOGITS: [M][NT]
  int32_t *part_idx;
};

// The kernels take GemmArgs by value: it is the explicit part of their kernel-argument segment (the code objects
// declare that size plus 256 bytes of hidden arguments).
static_assert(sizeof(GemmArgs) % 8 == 0 && sizeof(GemmArgs) <= 288 && alignof(GemmArgs) == 8, "kernel argument block of the GEMM kernels");

// Packed weights are fp16 = weight * 2^k, k per matrix so that the largest magnitude lands in
// [2^13, 2^14): every bf16 value within 2^-31 of the largest is then an exact fp16 number (smaller
// ones round to a multiple of 2^-24 / 2^k).  amax_bits holds the fp32 bit pattern of that largest
// magnitude (0 = no scaling, fp16 sources).
__host__ __device__ inline float weight_scale(uint32_t amax_bits) {
  const int e = (int)((amax_bits >> 23) & 0xffu) - 127;  // floor(log2(amax))
  if (amax_bits == 0 || e < -90 || e > 90) return 1.0f;
  return __builtin_bit_cast(float, (uint32_t)(13 - e + 127) << 23);
}
// gain: per-column factor [K] folded into the weights (model dtype), or null
void launch_absmax(int dtype, const void *src, size_t n, int K, const void *gain, uint32_t *d_amax_bits, hipStream_t st);
void launch_pack_weight(int dtype, int mode, const PackedDims &p, int d, int hd, const void *s0, const void *s1,
                        const void *s2, const void *gain, void *dst, const uint32_t *d_amax_bits, hipStream_t st);
void launch_pack_bias(int dtype, int mode, const PackedDims &p, int d, int hd, const void *s0, const void *s1,
                      const void *s2, float *dst, hipStream_t st);
// folded LayerNorm: wsum[n] = sum of the packed row n; bias[n] += (W b)[n] (bias must hold the GEMM's own bias, or zeros)
void launch_fold_ln(int dtype, int mode, const PackedDims &p, int d, int hd, const void *s0, const void *s1, const void *s2,
                    const void *ln_bias, const void *packed, float *wsum, float *bias, hipStream_t st);
void launch_rope_table(int L, int hd, float theta, float2 *tab, hipStream_t st);
void launch_gemm_mfma(int dtype, const GemmArgs &a, int epi, hipStream_t st);
void launch_gemm_tile(int dtype, GemmArgs a, int epi, hipStream_t st);  // more than 64 rows, wide outputs
// Folded norm: true when the launch for these arguments reads 1 / rms of its rows from a.rinv_ws (tiled kernel
// with more than one row tile per wave); launch_row_inv_x then has to run first.  Every other launch takes the
// value from its own operand fragments.
bool gemm_wants_row_inv(const GemmArgs &a, int epi);
bool gemm_tile_wants_row_inv(const GemmArgs &a, int epi);
void launch_row_inv_x(const GemmArgs &a, hipStream_t st);
// True when this EPI_RESIDUAL launch (x_out set) goes through the split kernel's row-wise reduction, which can leave
// 1 / rms of the updated rows behind (set ssq_ks, ss_d, ss_eps and rinv_ws before the launch): the consumer then needs
// no k_row_inv_x.
bool gemm_can_leave_ssq(const GemmArgs &a);
void launch_argmax_partials(const float *pv, const int32_t *pi, int M, int row_step, int NT, int V, int q, int out_stride,
                            int32_t *out, hipStream_t st);
// once per context, with its device current: lets the kernels that need it use more than 64 KB of LDS
void gemm_tile_prepare();
void attention_prepare();
// Up to 16 rows, wide outputs with a short k-slice: a wave keeps its slice of the activations in registers and
// walks several weight strips (kernels_gemm_rowres.hip).  launch_gemm_rowres returns false when the shape is not
// covered (the caller then takes the streaming kernel).
bool launch_gemm_rowres(int dtype, const GemmArgs &a, int epi, hipStream_t st);
// bits of GemmArgs::tune
enum GemmTune {
  TUNE_TILE_MTW_MASK = 0x00f,   // tiled kernel: force MTW (1..4) ...
  TUNE_TILE_NBW_SHIFT = 4,      // ... and NBW (2..4), both or neither
  TUNE_ROWRES_OFF = 0x100,      // never take the row-resident kernel
  TUNE_ROWRES_ALWAYS = 0x200    // take it for every row count it covers (1..16), not only where it was measured faster
};

struct AttnArgs {
  const void *q;            // [M][d] fp32, pair-interleaved heads (rounded to the cache's type, as a pair for bf16, by the kernel)
  const void *kc, *vc;      // this layer's cache areas
  const int32_t *row_pos;   // [M]
  void *out;                // [M][d] fp16, canonical element order, fragment layout
  float *part_acc;          // [M][H][NC][hd] un-normalised partial outputs
  float *part_ml;           // [M][H][NC][2] running max (raw score units) and sum
  int shape;                // 0 auto, 1 split + merge, 2 one wave per (sequence, head), 3 one workgroup per (sequence, head)
  int B, q_rows, H, hd, L_pad, NC;  // NC = chunks launched (upper bound over the batch)
  int seq_groups;           // consecutive groups of q_rows rows that belong to one sequence and share its cache (0 or 1: one)
  int n_cu;                 // compute units of the device (0: 256)
};
// Keys per split.  The chunk boundaries are fixed positions, the same for every launch shape and batch (they decide
// the order of the softmax merges, hence the bits): 128 keys each up to position 512, where the attention of a small
// batch is a chain of load latencies and twice the waves halve it, 256 keys beyond.
constexpr int ATTN_CHUNK = 256, ATTN_FINE_CHUNK = 128, ATTN_FINE_END = 512, ATTN_FINE_CHUNKS = ATTN_FINE_END / ATTN_FINE_CHUNK;
__host__ __device__ inline int attn_chunk_begin(int c) {
  return c < ATTN_FINE_CHUNKS ? c * ATTN_FINE_CHUNK : ATTN_FINE_END + (c - ATTN_FINE_CHUNKS) * ATTN_CHUNK;
}
__host__ __device__ inline int attn_chunk_of(int pos) {  // the chunk that holds key position pos >= 0
  return pos < ATTN_FINE_END ? pos / ATTN_FINE_CHUNK : ATTN_FINE_CHUNKS + (pos - ATTN_FINE_END) / ATTN_CHUNK;
}
constexpr int ATTN_STREAM_MIN_WAVES = 2048;  // (sequence, head, chunk) waves from which the chunk kernels load non-temporally (8 sequences x 32 heads x 512 positions: 18.8 us with, 17.1 without; 16 sequences: 32.7 with, 34.2 without)
constexpr int ATTN_SEQ_MIN_PAIRS = 768;   // (sequence, head) pairs from which one wave walks all chunks (measured: 24 sequences x 32 heads 55 -> 45 us)
constexpr int ATTN_GROUP_MAX_WAVES = 8;  // waves of the one-workgroup-per-(sequence, head) shape, a chunk each (four waves with the register budget of the split kernel were measured no faster, and slower at 16 sequences)
constexpr int ATTN_GROUP_MAX_CHUNKS = 16;  // ... or every eighth chunk each when there are more: 139 KB of partials at head_dim 128 (2560 positions)
void launch_attention_mfma(int dtype, const AttnArgs &a, hipStream_t st);

}  // namespace spec
