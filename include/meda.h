/*
 * libmeda -- prefill-time KV-cache compression pass of MEDA (arXiv 2502.17599) for AMD MI355X
 * (gfx950).  C ABI: plain pointers and sizes, no framework types.
 *
 * One call compresses the KV cache of one sequence (or of a batch of equally shaped sequences) over all layers:
 *   1. attention of an observation window (the last W prompt positions) against every cached
 *      key: causal softmax rows, cumulative attention score per key      (Section 3.3, A_s)
 *   2. cross-modal attention entropy of every layer                       (Section 3.2, E_CM)
 *   3. per-layer budgets S_l proportional to exp(E_CM), summing to the total budget
 *                                                   (Section 3.2 allocation, Appendix A.3)
 *   4. per kv head: text-prior boost, recent window M_l, Top-N_l          (Section 3.3, selection)
 *   5. nearest conserved key by cosine similarity for every other key     (Section 3.3, matrix U)
 *   6. average merging of keys and, with the same assignment, values      (Section 3.3, merging)
 *   7. ragged per-layer compressed cache
 *
 * Memory: every data pointer is a DEVICE pointer owned by the caller; the library never
 * allocates or frees device memory, never modifies the inputs and never synchronises the
 * stream: work is enqueued on `hip_stream` and the call returns.  `params` is a host pointer.
 * Errors: every function that can fail returns a meda_status; on an error detected on the host
 * nothing has been launched and the outputs are untouched.
 * Results are deterministic: the same inputs give bit-identical outputs on every run.
 */
#ifndef MEDA_H
#define MEDA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MEDA_OK = 0,
  MEDA_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, Hq % Hkv != 0, window > seq_len ...  */
  MEDA_ERR_BUDGET = 2,      /* total_budget outside [L*min(W,T), L*T]                               */
  MEDA_ERR_UNSUPPORTED = 3, /* head_dim / dtype / group size (Hq / Hkv > 32) / sizes outside the built set */
  MEDA_ERR_WORKSPACE = 4,   /* workspace null, misaligned or smaller than meda_workspace_bytes()    */
  MEDA_ERR_HIP = 5,         /* a HIP call or kernel launch failed                                    */
  MEDA_ERR_SCRATCH_LIMIT = 6 /* meda_decode_attention_noalloc: the step needs more scratch than the
                               library's built-in array holds (MEDA_DECODE_NOALLOC_MAX_BYTES)        */
} meda_status;

typedef enum { MEDA_F32 = 0, MEDA_BF16 = 1 } meda_dtype;

/* flags */
#define MEDA_FLAG_UNIFORM_BUDGET 1 /* skip the entropy softmax: S_l = B/L (+1 on the lowest layers)  */
#define MEDA_FLAG_NO_MERGE 2       /* evict instead of merge: conserved rows are copied unchanged    */
#define MEDA_FLAG_FULL_PROMPT 4    /* every prompt position scores the keys (Section 3.3 sums A_p over all
                                      prompt rows, Section 3.2 takes all text / vision queries): q_win
                                      is then [L][Hq][T][d]; `window` stays the lower bound of the recent
                                      part and of the layer budgets                                    */

typedef struct {
  int32_t n_layers;     /* L, 1..256                                                               */
  int32_t n_q_heads;    /* Hq                                                                      */
  int32_t n_kv_heads;   /* Hkv, Hq % Hkv == 0; query head h reads kv head h / (Hq/Hkv)             */
  int32_t head_dim;     /* d: 64 or 128                                                            */
  int32_t seq_len;      /* T: cached positions per layer; T*d*sizeof(element) < 2^31, N*L*Hkv*T < 2^31
                           and N*L*Hq*max(128, scoring rows) < 2^31 (MEDA_ERR_UNSUPPORTED beyond)      */
  int32_t window;       /* W: rows of q_win = the last W positions, 1 <= W <= T                      */
  int64_t total_budget; /* B = sum_l S_l, kept positions per kv head summed over layers            */
  int32_t recent_num;   /* M_l = max(min(W,S_l), floor(S_l*num/den)); 3/4 is the paper's 3:1 split */
  int32_t recent_den;   /*   (Section 4.3); den > 0, 0 <= num <= den                               */
  int32_t dtype;        /* meda_dtype of q_win, k, v, k_out, v_out                                 */
  float softmax_scale;  /* 0 -> 1/sqrt(head_dim)                                                   */
  int32_t flags;        /* MEDA_FLAG_*                                                             */
  int32_t n_seqs;       /* N: sequences of this shape compressed by the call (0 means 1); every array
                           gains a leading [N] dimension, see meda_compress; N * L <= 256             */
} meda_params;

/* Bytes of device scratch meda_compress needs for these parameters; 0 if they are invalid.       */
size_t meda_workspace_bytes(const meda_params* params);

/*
 * The compression pass (Sections 3.2 and 3.3).
 *
 * Inputs (device, read-only):
 *   q_win     [L][Hq][W][d]   queries of the last W positions (row i sits at position T-W+i)
 *   k, v      [L][Hkv][T][d]  contiguous
 *   modality  [T] uint8       0 = text position, 1 = vision position
 * Outputs (device):
 *   k_out, v_out   ragged: layer l holds [Hkv][S_l][d] starting at row layer_off[l]*Hkv; rows of
 *                  a (layer, head) are in ascending original position; capacity B*Hkv*d elements
 *   layer_len      [L]   int32  S_l
 *   layer_off      [L+1] int64  prefix sums of S_l, layer_off[L] == B
 *   entropy        [L]   double E_CM per layer; may be NULL
 *   sel_idx        [B*Hkv] int32 original position of every output row, same ragged layout; may be NULL
 *   merge_assign   [L][Hkv][T] int32 for every position the slot (row within its (layer, head)
 *                  block) it was kept in or merged into (-1 for evicted positions when
 *                  MEDA_FLAG_NO_MERGE is set); may be NULL
 *   workspace      at least meda_workspace_bytes(params) bytes, 256-byte aligned
 *   hip_stream     hipStream_t (NULL = the default stream)
 * Calls that share a workspace must not overlap.
 *
 * Several sequences (n_seqs = N > 1; the paper's throughput figures are taken on batches, Table 6): the
 * sequences are independent and share every parameter (each gets the budget B).  Inputs are stacked:
 * q_win [N][L][Hq][W][d], k, v [N][L][Hkv][T][d], modality [N][T].  Outputs: one ragged cache for the whole
 * batch, sequence n occupying the rows [n*B*Hkv, (n+1)*B*Hkv); layer_len [N][L]; layer_off [N][L+1] holds
 * ABSOLUTE offsets (layer_off[n][0] = n*B, layer_off[n][L] = (n+1)*B), so the slices of sequence n can be
 * handed to meda_decode_attention as they are; entropy [N][L]; sel_idx [N*B*Hkv]; merge_assign [N][L][Hkv][T].
 * The result of every sequence is bit-identical to a call of its own.
 */
meda_status meda_compress(const meda_params* params, const void* q_win, const void* k, const void* v,
                          const uint8_t* modality, void* k_out, void* v_out, int32_t* layer_len,
                          int64_t* layer_off, double* entropy, int32_t* sel_idx, int32_t* merge_assign,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Where an intermediate result lives inside the workspace after meda_compress (for tests and
 * profiling tools).  Returns MEDA_ERR_INVALID_ARG for an unknown region or invalid params.
 */
typedef enum {
  MEDA_REGION_COL_SCORES = 0, /* float [L][Hkv][T]: cumulative attention score A_s (Section 3.3)    */
  MEDA_REGION_INV_NORM = 1,   /* float [L][Hkv][T]: 1/|k| of every key                              */
  MEDA_REGION_ROW_STATS = 2,  /* float [L][Hq][4][Wp], Wp = W rounded up to 32: four planes of one value per window
                                 row: log2-domain row max, 1/Z over all visible keys, then the row's cross-modal
                                 1/Z as the factor for vision columns (text rows, else 0) and for text columns
                                 (vision rows, else 0).  With more than 128 scoring rows R (W, or T with
                                 MEDA_FLAG_FULL_PROMPT): [L][Hq][4][R], one value per row: -(max + log2 Z) / (scale * log2 e), Z / Z_vision (text
                                 rows, else 0), Z / Z_text (vision rows, else 0), unused                */
  MEDA_REGION_ALLOC = 3,      /* int32 [L][4]: S_l, M_l, N_l, layer of rank l by decreasing S (with n_seqs = N
                                 > 1: [N*L][4], ranks of the sequences interleaved)                  */
  MEDA_REGION_LESS_IDX = 4,   /* int32 ragged: layer l, head g at ((l*T - off[l])*Hkv + g*(T-S_l)): the keys
                                 that are not conserved, ascending, as row ids (l*Hkv+g)*T + position */
  MEDA_REGION_LESS_SLOT = 5   /* int32, same layout: slot each of them merges into                   */
} meda_region;
meda_status meda_workspace_region(const meda_params* params, int region, size_t* offset, size_t* bytes);

/*
 * Per-phase GPU timing.  While enabled, meda_compress records HIP events on its stream around
 * its kernels; meda_profile_read waits for the recorded calls and returns, per phase, the
 * summed kernel time in milliseconds and the number of calls since the last reset.
 * meda_profile_enable(0) switches it off, (1) brackets every kernel, (2 + p) brackets only the
 * kernel of phase p (two events per call instead of nine; the other phases read 0).
 */
#define MEDA_N_PHASES 8
/* phases: 0 row statistics + key norms, 1 statistics combine, 2 column scores + entropy,
 *         3 layer budgets, 4 selection, 5 similarity + argmax, 6 segment sort, 7 merge + write   */
meda_status meda_profile_enable(int enable);
meda_status meda_profile_read(double* phase_ms /* [MEDA_N_PHASES] */, int32_t* n_calls, int reset);
const char* meda_phase_name(int phase);

const char* meda_status_string(meda_status status);

/*
 * One decoding step over the compressed cache (Section 3.1, "Decoding with Multimodal KV Cache"):
 * for every layer and query head, out = Softmax(q K^T * scale) V over the rows the compression pass
 * kept for that layer (the ragged layout meda_compress writes: layer l holds [Hkv][S_l][d] from row
 * layer_off[l] * Hkv) followed by the rows appended since then, K = [K, k_t], V = [V, v_t].  Query
 * head h reads kv head h / (Hq/Hkv).  The order of the rows has no influence on the result.
 */
typedef struct {
  int32_t n_layers;     /* L                                                                        */
  int32_t n_q_heads;    /* Hq                                                                       */
  int32_t n_kv_heads;   /* Hkv, Hq % Hkv == 0, Hq / Hkv <= 8                                        */
  int32_t head_dim;     /* d: 64 or 128                                                             */
  int32_t n_new;        /* rows appended per layer and kv head since the cache was compressed (>= 0) */
  int32_t dtype;        /* meda_dtype of q, the caches, the appended rows and out                    */
  int64_t total_budget; /* B = sum_l S_l (used to size the split of the work; >= L)                  */
  float softmax_scale;  /* 0 -> 1/sqrt(head_dim)                                                    */
} meda_decode_params;

/* Bytes of workspace meda_decode_attention needs (multiple of 256); 0 if the parameters are invalid. */
size_t meda_decode_workspace_bytes(const meda_decode_params* params);

/*
 * q        [L][Hq][d]                    the query of the new position, one per layer and head
 * k_cache, v_cache                       ragged compressed cache, B * Hkv rows of d elements
 * layer_len [L] int32, layer_off [L+1] int64   DEVICE arrays as written by meda_compress
 * k_new, v_new [L][Hkv][n_new][d]        rows appended since; may be NULL when n_new == 0
 * out      [L][Hq][d]                    attention output, one rounding to the storage type
 * workspace                              256-byte aligned, at least meda_decode_workspace_bytes()
 * All data pointers are device pointers, 16-byte aligned; nothing is allocated; the work is enqueued on
 * hip_stream.  Errors as for meda_compress (MEDA_ERR_UNSUPPORTED for a group size above 8).
 */
meda_status meda_decode_attention(const meda_decode_params* params, const void* q, const void* k_cache,
                                  const void* v_cache, const int32_t* layer_len, const int64_t* layer_off,
                                  const void* k_new, const void* v_new, void* out, void* workspace,
                                  size_t workspace_bytes, void* hip_stream);

/*
 * meda_decode_attention for callers that cannot allocate or hand over device scratch: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs, kernels and results as
 * meda_decode_attention, without the workspace arguments: the chunk partials of the step live in a device array
 * built into the library (MEDA_DECODE_NOALLOC_MAX_BYTES per GPU, held until the process ends).  The call
 * allocates and frees nothing, on the host side of HIP or through any library.
 *   - returns MEDA_ERR_SCRATCH_LIMIT, with nothing launched, when meda_decode_workspace_bytes(params) exceeds
 *     MEDA_DECODE_NOALLOC_MAX_BYTES (the five benchmark shapes fit; the need grows with L * Hq * chunks)
 *   - the array belongs to the current device of the calling thread, which must be the device of hip_stream
 *   - all calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams,
 *     or different threads) race; calls on one stream are ordered and safe.  Nothing in the array has to start
 *     at zero: every partial a call reads was written by the same call.
 */
#define MEDA_DECODE_NOALLOC_MAX_BYTES (40u << 20)
meda_status meda_decode_attention_noalloc(const meda_decode_params* params, const void* q, const void* k_cache,
                                          const void* v_cache, const int32_t* layer_len, const int64_t* layer_off,
                                          const void* k_new, const void* v_new, void* out, void* hip_stream);

/*
 * 8-bit storage of a compressed cache.  The paper names quantisation of the KV cache as a technique that can be
 * combined with its method (Limitations) and fixes no scheme; this one is the library's own.  Per row of
 * head_dim elements:
 *   scale  = max|x| / 448 in fp32 (1 for an all-zero row)
 *   code_i = E4M3(clamp(x_i / scale, -448, 448)): fp32 division, round to nearest, ties to even, where E4M3 is
 *            the 8-bit format of the OCP 8-bit floating point specification (1 sign, 4 exponent bits with
 *            bias 7, 3 mantissa bits, no infinities, largest magnitude 448); a NaN code is never written
 *   x_i   ~= value(code_i) * scale
 * rows    [n_rows][head_dim] of `dtype` (meda_dtype), e.g. k_out or v_out of meda_compress (read-only)
 * codes   [n_rows][head_dim] uint8, scales [n_rows] float (outputs)
 * head_dim 64 or 128; n_rows >= 0; device pointers, 16-byte aligned; enqueued on hip_stream, nothing allocated.
 * meda_dequantize_fp8 is the inverse map (one rounding to `dtype`; exact for MEDA_BF16 and MEDA_F32 up to the
 * product with the scale).
 */
meda_status meda_quantize_fp8(const void* rows, int32_t dtype, int64_t n_rows, int32_t head_dim, uint8_t* codes,
                              float* scales, void* hip_stream);
meda_status meda_dequantize_fp8(const uint8_t* codes, const float* scales, int32_t dtype, int64_t n_rows,
                                int32_t head_dim, void* rows, void* hip_stream);

/*
 * meda_decode_attention over a cache stored with meda_quantize_fp8: k_codes, v_codes [B*Hkv][d] uint8 and
 * k_scales, v_scales [B*Hkv] float in the ragged layout of meda_compress; q, the appended rows k_new / v_new and
 * out are of params->dtype, which must be MEDA_BF16 (MEDA_ERR_UNSUPPORTED otherwise).  The step computes
 * Softmax(q K^T * scale) V with K = value(k_codes) * k_scales and V likewise (Section 3.1); it reads half the
 * bytes of the bf16 cache.  Workspace and all other arguments as for meda_decode_attention.
 */
meda_status meda_decode_attention_fp8(const meda_decode_params* params, const void* q, const uint8_t* k_codes,
                                      const uint8_t* v_codes, const float* k_scales, const float* v_scales,
                                      const int32_t* layer_len, const int64_t* layer_off, const void* k_new,
                                      const void* v_new, void* out, void* workspace, size_t workspace_bytes,
                                      void* hip_stream);

/*
 * Measurement aids for the benchmark: what this GPU delivers to the simplest kernel of each of the two kinds the
 * pass is made of.  Both only enqueue one kernel on hip_stream; the caller times them (events on that stream).
 *   meda_peak_stream_read   reads `bytes` bytes (multiple of 16 used; src device pointer, 16-byte aligned) once,
 *                           with 16-byte streaming loads, eight in flight per lane; nothing is written.
 *                           Rate = bytes / time: the HBM read rate a kernel of the scoring / merge kind can reach.
 *   meda_peak_mfma_bf16     every SIMD of the chip issues `mfma_per_wave` (rounded down to a multiple of 16,
 *                           >= 16) bf16 32x32x16 matrix instructions from registers, two waves per SIMD, four
 *                           independent accumulator chains per wave; *total_mfma (host pointer) receives the
 *                           number issued over the whole chip.  Rate = total_mfma * 32768 flop / time.
 *                           random_operands = 0: operands nearly constant; 1: pseudo-random signs and mantissas
 *                           (more bits toggle per step, the chip draws more power and holds a lower clock: the
 *                           rate a kernel working on real data can hope for).
 *   meda_peak_mfma_valu     how much vector work fits beside the matrix instructions: every wave runs `rounds`
 *                           (1 .. 2^22) rounds of 16 bf16 32x32x16 matrix instructions (two accumulator chains,
 *                           nearly constant operands) and 16 * valu_per_mfma (0, 4, 6 or 8) independent fp32
 *                           multiply-adds, written right behind each matrix instruction (interleaved != 0) or all
 *                           after the sixteenth (a matrix phase, then a vector phase); waves_per_simd (1 or 2)
 *                           workgroups of one wave per SIMD run on every CU.  Time per round against the run with
 *                           valu_per_mfma = 0 tells what the vector work costs.  MEDA_ERR_INVALID_ARG for other
 *                           values.
 * `sink` is a 4-byte aligned device word that is never actually written (it keeps the work alive).
 */
meda_status meda_peak_stream_read(const void* src, size_t bytes, void* sink, void* hip_stream);
meda_status meda_peak_mfma_bf16(int64_t mfma_per_wave, int32_t random_operands, int64_t* total_mfma, void* sink,
                                void* hip_stream);
meda_status meda_peak_mfma_valu(int64_t rounds, int32_t valu_per_mfma, int32_t interleaved, int32_t waves_per_simd,
                                void* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MEDA_H */
