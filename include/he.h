/*
 * he.h -- C ABI of the MI355X actor-generation engine.
 *
 * The engine runs the inference half of the paper's Hybrid Engine (Section 4):
 * the experience-generation phase of RLHF step 3, i.e. the actor model run
 * over the prompt once and then once per generated token with a KV cache
 * (Section 5.3 (I): 256 prompt tokens, 256 generated tokens, memory-bandwidth
 * bound).  The model is an OPT-style decoder (Section 2 names the family):
 * pre-LayerNorm, learned positions, causal multi-head attention with biases,
 * ReLU feed-forward, final LayerNorm, LM head.
 *
 * Conventions
 *  - Every pointer whose name starts with d_ and every weight pointer is a
 *    DEVICE pointer on cfg.device.  Structs and scalars are host memory.
 *  - Linear weights are row-major [out, in]:  y = x W^T + b.
 *  - dtype HE_F32: weights, biases, LayerNorm parameters and the KV cache are
 *    float.  dtype HE_BF16: the caller's weights, biases and LayerNorm
 *    parameters are bfloat16 (raw 16-bit, upper half of an IEEE float).
 *    Accumulation, residual stream, LayerNorm statistics, softmax, logits and
 *    log-probs are float in both cases.  Inside the engine the HE_BF16 path
 *    feeds the matrix cores IEEE binary16 operands: the tiled copies hold the
 *    caller's bf16 weights converted to binary16 (the same value for
 *    magnitudes from 2^-14 to 65504, the nearest multiple of 2^-24 below that,
 *    infinity above -- no trained weight is that large), every GEMM input and
 *    the KV cache are float values rounded once, to nearest even, to binary16.
 *  - The caller owns weights and all input/output buffers.  The engine
 *    borrows the weight pointers until he_destroy; it owns only its KV arena,
 *    workspace and (bf16) MFMA-tiled copies of the GEMM matrices, all
 *    allocated once in he_create -- the engine allocates no device memory on
 *    the generation path (Section 4: pre-reserved KV cache and intermediate
 *    buffers).  One exception is the runtime's, not the engine's: the first
 *    he_generate / he_generate_ragged with a new (batch, answer length)
 *    captures the decode step into a HIP graph and instantiates it, and the
 *    runtime may back that with memory of its own; later calls of that shape
 *    replay the graph.  he_decode_step_static is the call for a caller that
 *    tolerates no allocation at all.  After the caller overwrites weights in
 *    place (a training update between two generation phases) it calls
 *    he_refresh_weights.
 *  - All work is enqueued on cfg.stream (a hipStream_t, NULL = default
 *    stream) and is asynchronous; only he_create / he_refresh_weights /
 *    he_destroy synchronise.  Outputs are valid once the stream has drained.
 *  - Every call validates its arguments and returns a status; nothing throws
 *    across the boundary.  After an error the engine is reusable once
 *    he_reset has been called.  An engine is not thread-safe.
 *  - he_prefill / he_generate: all sequences of a batch have the same prompt
 *    length and exactly G tokens are generated per sequence (no stop token);
 *    the _ragged variants lift both restrictions.
 */
#ifndef HE_H
#define HE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct he_engine he_engine; /* opaque */

typedef enum {
    HE_OK = 0,
    HE_ERR_INVALID_ARG = 1, /* null pointer, bad enum, non-positive size */
    HE_ERR_SHAPE = 2,       /* dimensions the kernels do not support */
    HE_ERR_CAPACITY = 3,    /* batch, sequence length or positions exceed what he_create reserved */
    HE_ERR_OOM = 4,         /* device allocation failed in he_create */
    HE_ERR_DEVICE = 5,      /* a HIP call failed; he_last_error has the text */
    HE_ERR_STATE = 6        /* call order: decode before prefill, prefill on a non-empty cache */
} he_status;

typedef enum { HE_F32 = 0, HE_BF16 = 1 } he_dtype;

typedef struct {
    int n_layers;      /* L >= 0 */
    int hidden;        /* H, multiple of 64 */
    int n_heads;       /* nh; head_dim d = H / nh must be 64 or 128 on the bf16 path, any multiple of 8 <= 256 on f32 */
    int ffn;           /* F, multiple of 64 */
    int vocab;         /* V */
    int max_positions; /* rows of pos_emb minus pos_offset */
    int pos_offset;    /* position t reads pos_emb row t + pos_offset */
    float ln_eps;
    he_dtype dtype;
    int max_batch;     /* KV arena holds max_batch sequences ... */
    int max_seq_len;   /* ... of at most max_seq_len positions (prompt + generated) */
    int device;        /* HIP device ordinal */
    void* stream;      /* hipStream_t or NULL */
    int impl;          /* 0 = default kernels for the dtype; 1 = the plain (f32-path) kernels
                          instantiated for this dtype -- a slow comparator for tests */
    int weights_tiled; /* bf16, impl 0 only.  0: wqkv, wo, w1, w2 and lm_head are row-major and the engine
                          keeps MFMA-tiled copies of them (twice the memory).  1: the caller passes those
                          five kinds of matrices already tiled by he_tile_matrix and the engine uses them
                          in place, no copies -- for models whose weights fill more than half of HBM.
                          tok_emb is row-major in both cases (with a tied head and weights_tiled = 1,
                          lm_head is the tiled copy of tok_emb). */
    int weights_fp8;   /* bf16, impl 0, weights_tiled 0 only.  1: the engine keeps the four matrices of every layer
                          (wqkv, wo, w1, w2) as 8-bit codes instead of bf16 copies -- half the bytes a decode step
                          streams, half the engine's weight memory.  Row n of a matrix is stored as OCP FP8 E4M3
                          codes q[n][:] and a scale 2^e[n], e[n] the smallest integer with max|W[n][:]| 2^-e[n] <= 448,
                          q the nearest E4M3 value of W 2^-e (ties to even); the model then computes with the
                          dequantised weights q 2^e (bf16 values again, so everything else is unchanged:
                          accumulation, activations, tolerances).  The LM head and the embeddings stay bf16.
                          This goes beyond the paper, which streams 16-bit weights (Section 5.3 (I): generation is
                          bound by the bytes read per token).  Decode steps of up to 32 sequences read the codes
                          directly; prompt rows, scoring and larger batches dequantise a layer at a time into one
                          layer of scratch.  Not combinable with he_refresh_weights_lora. */
} he_config;

typedef struct {
    const void *ln1_g, *ln1_b; /* [H] */
    const void *wqkv;          /* [3H, H]: rows 0..H-1 query, H..2H-1 key, 2H..3H-1 value */
    const void *bqkv;          /* [3H] */
    const void *wo, *bo;       /* [H, H], [H] */
    const void *ln2_g, *ln2_b; /* [H] */
    const void *w1, *b1;       /* [F, H], [F] */
    const void *w2, *b2;       /* [H, F], [H] */
} he_layer_weights;

typedef struct {
    const void* tok_emb;            /* [V, H] */
    const void* pos_emb;            /* [max_positions + pos_offset, H] */
    const void *lnf_g, *lnf_b;      /* [H] final LayerNorm */
    const void* lm_head;            /* [V, H], no bias; may alias tok_emb (tied) */
    const he_layer_weights* layers; /* host array of n_layers entries (copied by he_create) */
} he_weights;

typedef struct {
    int mode;          /* 0 greedy: argmax z.  1 Gumbel-max: argmax (z / temperature + g) */
    float temperature; /* > 0, used in mode 1 only */
    uint64_t seed;     /* g = -log(-log u), u from Philox4x32-10 keyed by seed at counter (v, step, b, 0) */
} he_sampling;

/* Bytes of the MFMA-tiled form of a bf16 [rows, cols] matrix (rows padded to a multiple of 32;
 * cols must be a multiple of 16), and the conversion itself: d_src row-major bf16 [rows, cols],
 * d_dst the tiled form, distinct buffers, on `stream`.  The tiled form is [rows/32][cols/16]
 * blocks of 64 lanes x 8 values: lane 32*((c%16)/8) + r%32 holds columns 16*(c/16) + 8*(lane/32)
 * + 0..7 of row r -- one MFMA 32x32x16 operand per block.  The 16-bit values of the tiled form are
 * IEEE binary16, each the bf16 source value converted as the conventions above state. */
size_t he_tiled_bytes(int rows, int cols);
he_status he_tile_matrix(const void* d_src, void* d_dst, int rows, int cols, void* stream);
/* The same with a low-rank adapter folded in: d_dst = tiled bf16(src + scale * B A), d_a bf16 [rank, cols],
 * d_b bf16 [rows, rank], summed as he_refresh_weights_lora states (for callers that keep the tiled
 * matrices themselves, weights_tiled = 1). */
he_status he_tile_matrix_lora(const void* d_src, void* d_dst, int rows, int cols, const void* d_a, const void* d_b,
                              int rank, float scale, void* stream);

/* Bytes of device memory he_create will allocate for cfg (KV arena, workspace,
 * tiled weight copies).  Pure host computation; 0 if cfg is invalid. */
size_t he_workspace_bytes(const he_config* cfg);

/* Validates cfg, allocates arena and workspace, prepares weights.  *out is
 * set only on HE_OK.  Synchronises the whole device first (the weights may have
 * been written on any stream), then cfg.stream. */
he_status he_create(const he_config* cfg, const he_weights* weights, he_engine** out);

/* Re-reads the borrowed weight pointers after the caller changed the values
 * in place (re-tiles the GEMM matrices on the bf16 path).  Synchronises the
 * device before and cfg.stream after. */
he_status he_refresh_weights(he_engine* e);

/* Prompt pass (Section 5.3 (I): "initial prompt").  d_prompt_ids is [B, S]
 * int32 row-major, 1 <= B <= max_batch, 1 <= S <= max_seq_len, S within
 * max_positions.  Requires an empty cache (fresh engine or he_reset).
 * Fills the KV cache for positions 0..S-1 and samples generation step 0 from
 * the last position's logits z:  d_next_ids [B] int32, d_logprobs [B] float
 * = log_softmax(z)[id] (untempered).  d_logits_opt, if not NULL, receives z
 * as [B, V] float. */
he_status he_prefill(he_engine* e, const int32_t* d_prompt_ids, int B, int S, const he_sampling* sampling,
                     int32_t* d_next_ids, float* d_logprobs, float* d_logits_opt);

/* One KV-cached decode step (Section 5.3 (I): the actor "once for each"
 * generated token): feeds d_in_ids [B] at position cur_len, appends its K/V,
 * samples the next generation step.  Outputs as in he_prefill.  B is the
 * batch of the preceding he_prefill.  HE_ERR_CAPACITY when the cache or the
 * position table is full. */
he_status he_decode_step(he_engine* e, const int32_t* d_in_ids, const he_sampling* sampling, int32_t* d_next_ids,
                         float* d_logprobs, float* d_logits_opt);

/* he_decode_step for callers that cannot allocate device memory or tolerate a call that might: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results
 * (bit for bit) as he_decode_step.  The step's scratch -- the k-split partial sums of the out-projection
 * and FC2, the column-group statistics and arrival counters of the folded LayerNorms, and the LM head's
 * per-tile soft-max / arg-max partials -- lives in a file-scope device array of 16 MiB inside the library
 * (every GPU the library runs on holds its own copy until the process ends) instead of the engine's
 * workspace; the call makes no hipMalloc / hipFree / event or graph creation and launches its kernels one by
 * one on cfg.stream.  KV arena, activations and weights are still the engine's (he_create allocated them).
 * Limits: dtype bf16 with impl 0; at most 64 sequences (32 with weights_fp8); HE_ERR_CAPACITY with the byte
 * counts in he_last_error when model width, vocabulary and batch together need more than the 16 MiB
 * (the OPT-13B-shaped headline workload needs about 5.3 MiB); HE_ERR_STATE when the engine's device is not the
 * current device.  All engines on one GPU share that GPU's array, which keeps the last call's contents:
 * the call clears what must start at zero itself, and two such calls that overlap in time on one GPU
 * (different streams, different engines) race -- serialise them. */
he_status he_decode_step_static(he_engine* e, const int32_t* d_in_ids, const he_sampling* sampling, int32_t* d_next_ids,
                                float* d_logprobs, float* d_logits_opt);

/* The whole generation phase: reset, prefill, then G-1 decode steps that feed
 * each sampled token back (the steps run as replays of one captured HIP
 * graph).  d_out_ids [B, G] int32 and d_out_logprobs [B, G] float, row-major.
 * Requires S + G - 1 <= max_seq_len and within max_positions. */
he_status he_generate(he_engine* e, const int32_t* d_prompt_ids, int B, int S, int G, const he_sampling* sampling,
                      int32_t* d_out_ids, float* d_out_logprobs);

/* Hand-over from the training phase (Section 4: the Hybrid Engine switches one actor between a
 * training mode, where memory-saving techniques such as LoRA are in use, and an inference mode that
 * runs the generation kernels, and reconfigures memory between the two modes).
 *
 * he_refresh_weights_lora is he_refresh_weights with low-rank adapters folded in on the way: the
 * engine's tiled copy of a matrix W [out, in] becomes bf16(W + scale * B A), A bf16 [rank, in] and
 * B bf16 [out, rank] row-major device pointers (a == b == NULL: no adapter on that matrix).  The sum is
 * taken in float: the products B[o][j] A[j][i] added one by one for j = 0 .. rank-1, then
 * W + scale * that, each operation rounded separately, then rounded to nearest-even bf16.  The
 * caller's W is not written, so a later plain he_refresh_weights undoes the merge.  `adapters` is a
 * host array of n_layers entries (copied); the factors are read during the call only.  Needs dtype
 * bf16, impl 0, weights_tiled 0.
 *
 * he_release_arena frees the KV arena (the cache is emptied first) so that the training phase can
 * have the memory; he_acquire_arena allocates it again (HE_ERR_OOM if that fails; the engine then
 * stays released).  While released, prefill / decode / generate / score return HE_ERR_STATE.  These
 * two calls are the only ones after he_create that allocate or free device memory. */
typedef struct { const void* a; const void* b; } he_lora;
typedef struct { he_lora wqkv, wo, w1, w2; } he_lora_layer;
he_status he_refresh_weights_lora(he_engine* e, const he_lora_layer* adapters, int rank, float scale);
he_status he_release_arena(he_engine* e);
he_status he_acquire_arena(he_engine* e);

/* Prompts of different lengths and answers that end early (Section 5.3 (I) pads or cuts every
 * prompt to one length and lets every answer run to the cap; real prompts are shorter and sit
 * right-aligned behind padding, and an answer is over once the end-of-sequence token has come).
 * d_prompt_ids is [B, S] int32 row-major, LEFT-padded: row b's tokens are its last d_prompt_lens[b]
 * entries (1 <= len <= S; values outside are clamped), whatever stands before them is ignored.
 * Padding is not part of a sequence: sequence b is computed exactly as if it were run alone on its own
 * tokens at positions 0, 1, 2, ... (only its row number b enters, through the sampling noise), and its
 * cache holds len[b] positions after the prompt.  Capacity is checked as for S tokens per sequence.
 *
 * he_prefill_ragged is he_prefill for such a batch; he_decode_step then continues every sequence at
 * its own position.
 *
 * he_generate_ragged is he_generate for such a batch with an end token: once a sequence has produced
 * eos_id (eos_id < 0: never) it produces nothing more -- its remaining d_out_ids are pad_id and their
 * d_out_logprobs 0 -- and d_out_lens [B] int32 receives the number of tokens each sequence produced,
 * the end token included.  When every sequence has ended, the remaining steps are skipped (the count
 * of running sequences is read back every 16 steps, which synchronises cfg.stream).  A sequence that has
 * ended skips attention at once; at those read-backs, on the HE_BF16 path, the rows of ended sequences are
 * dropped from the following steps whenever that makes a step cheaper (the row count falls to fewer 16-row
 * halves of the weight-streaming GEMMs' activation slices, up to 64 rows, or to fewer 128-row matrix-core
 * tiles above): the running sequences move up in order, every result still goes to its sequence's place,
 * and the sampling noise stays keyed by the sequence's number b -- results do not depend on it. */
he_status he_prefill_ragged(he_engine* e, const int32_t* d_prompt_ids, const int32_t* d_prompt_lens, int B, int S,
                            const he_sampling* sampling, int32_t* d_next_ids, float* d_logprobs, float* d_logits_opt);
he_status he_generate_ragged(he_engine* e, const int32_t* d_prompt_ids, const int32_t* d_prompt_lens, int B, int S, int G,
                             const he_sampling* sampling, int eos_id, int pad_id, int32_t* d_out_ids,
                             float* d_out_logprobs, int32_t* d_out_lens);

/* Scoring pass: the log-probability the model gives every token of a sequence after its prefix
 * (Section 4: the inference phase of an RLHF iteration produces the inputs of the training phase --
 * after the answer is generated, prompt plus answer goes through the model once more and the
 * log-probabilities of the tokens that are there are kept; Section 5.3 (I) counts this with the
 * generation phase).  d_ids is [B, T] int32 row-major, 1 <= B <= max_batch, 2 <= T <= max_seq_len and
 * within max_positions.  d_out_logprobs is [B, T-1] float:
 *   out[b][t] = log_softmax(logits at position t of sequence b)[d_ids[b][t+1]],  t = 0 .. T-2.
 * All T positions go through the prompt-pass kernels at once; the LM head is fused with the
 * log-softmax and the gather, so the [B*T, V] logits are never stored.  Uses the KV arena as
 * scratch: the cache is emptied before and after (as by he_reset). */
he_status he_score(he_engine* e, const int32_t* d_ids, int B, int T, float* d_out_logprobs);

/* Empties the KV cache (lengths to zero; memory is kept). */
he_status he_reset(he_engine* e);

/* Frees everything the engine owns.  NULL is accepted. */
he_status he_destroy(he_engine* e);

/* Text of the last error on this engine (engine-owned, valid until the next
 * call); with e == NULL, the text of the last he_create failure. */
const char* he_last_error(const he_engine* e);

/* Current number of cached positions per sequence, or -1 if e is NULL. */
int he_cache_len(const he_engine* e);
/* Test hook: rows of the last decode step of the last he_generate / he_generate_ragged (fewer than its batch once
 * he_generate_ragged has dropped the rows of ended sequences); -1 for a NULL engine. */
int he_last_step_rows(const he_engine* e);

/* Measurement hook (bf16 path).  While on, he_prefill / he_decode_step / he_generate
 * launch their decode-shaped kernels one by one (no graph replay) and bracket every
 * launch of each kernel class below with a pair of HIP events on cfg.stream.
 * he_timing_read synchronises the stream, returns the summed elapsed milliseconds
 * and launch counts per class since the last read, and clears them.  Events are
 * created on demand while the hook is on (the one place the engine allocates after
 * he_create); results are unaffected. */
enum {
    HE_K_LAYERNORM = 0, /* decode rows: the embedding kernel (their LayerNorms are folded into the GEMMs) */
    HE_K_QKV = 1,       /* fused QKV projection, K/V appended to the cache */
    HE_K_ATTENTION = 2, /* attention over the cache */
    HE_K_OUT_PROJ = 3,
    HE_K_FC1 = 4,       /* + bias + ReLU */
    HE_K_FC2 = 5,
    HE_K_LM_HEAD = 6,   /* LM head + log-softmax + sampling (both of its kernels) */
    HE_K_EMPTY = 7,     /* an event pair with no launch between (once per pass): what the pair itself costs */
    HE_K_COUNT = 8
};
he_status he_timing_enable(he_engine* e, int on);
he_status he_timing_read(he_engine* e, double* ms_per_class, long* launches_per_class, int n_classes);

/* Measurement hook (bf16 path, after a prefill): launches the decode-shaped GEMM of one
 * class (HE_K_OUT_PROJ, HE_K_FC1 or HE_K_FC2) once per layer, layer after layer, `reps`
 * times, on cfg.stream -- each launch streams a different layer's matrix, as in a decode
 * step, with the engine's current activations as the other operand.  Only workspace that the
 * next decode step overwrites anyway is written; the KV cache and the generation state are
 * untouched.  One event pair around the call gives the kernel's launch duration without the
 * per-launch cost of an event pair. */
he_status he_kernel_sweep(he_engine* e, int kernel_class, int reps);

/* Utility and test hook: the row quantisation weights_fp8 applies.  d_src bf16 [rows, cols] row-major (cols a
 * multiple of 8); d_codes receives the E4M3 codes [rows, cols] uint8 row-major, d_exps [rows] int32 the
 * exponents e[n], d_scales [rows] float the scales 2^e[n].  On `stream`. */
he_status he_fp8_quantize_rows(const void* d_src, int rows, int cols, void* d_codes, int32_t* d_exps, float* d_scales,
                               void* stream);

/* Test hook, host logic only (no device work): how a decode-shaped GEMM of M <= 64 rows with an [N, K] weight
 * matrix is shared out over `cus` compute units (0 = the current device's count, 256 if there is none): weight
 * rows per unit (32, or 16 for the half-tile kernel), units per workgroup, and k-splits (always 1 unless
 * ksplit_allowed, i.e. for the out-projection and FC2, whose partial sums go through scratch_floats floats of
 * scratch; 0 = unlimited).  N and K multiples of 32. */
he_status he_plan_decode_gemm(int M, int N, int K, int ksplit_allowed, size_t scratch_floats, int cus, int* unit_rows,
                              int* units_per_workgroup, int* ksplit);

/* Test hook, host logic only (no device work, no engine): what the k-split GEMM of a decode step of B <= 64
 * sequences (which = 0: out-projection, 1: FC2) would index in an engine created with cfg, next to what he_create
 * reserves for it.  The partial sums of one launch cross workgroups through scratch, each (column group, row
 * slice, split) in words of its own, and one arrival counter per (column group, row slice); the account comes
 * from the launcher's own choice of kernel variant and grid.  cus as in he_plan_decode_gemm.  bf16, impl 0 only. */
typedef struct {
    size_t scratch_floats;   /* floats of scratch the launch indexes (0 without a k-split) */
    size_t scratch_reserved; /* floats he_create reserves */
    size_t static_floats;    /* floats he_decode_step_static sets aside for this launch */
    int counters;            /* arrival counters the launch indexes */
    int counters_reserved;
    int stat_pairs;          /* (mean, sum of squares) pairs of column-group statistics it writes */
    int stat_pairs_reserved;
    int ksplit;
} he_scratch_account;
he_status he_decode_scratch_account(const he_config* cfg, int B, int which, int cus, he_scratch_account* out);

/* Test hook: waits for the engine's stream, then counts the engine's arrival counters that are not zero.  Every
 * k-split launch leaves its counters at zero for the next one (its last workgroup clears them), and he_reset
 * clears them all: between calls the answer is 0.  bf16, impl 0 only. */
he_status he_arrival_counters_nonzero(he_engine* e, int* nonzero);

/* Test hook, host logic only: how a GEMM of a prompt or scoring pass (M rows, [N, K] weights) is cut into tiles on
 * `cus` compute units (0 = the current device's count, 256 if there is none).  *tile_cols: columns of a tile (256 or
 * 320 with 256 rows; 0 if the pass is too small for these tiles and takes the 256 x 128 ones); *ksplit, *split_col:
 * with may_cut (the out-projection and FC2, whose partial sums the following LayerNorm adds; scratch_floats floats
 * of scratch, 0 = unlimited), the tiles of columns >= *split_col are cut into *ksplit k ranges (1: none are). */
he_status he_plan_prompt_gemm(int M, int N, int K, int may_cut, size_t scratch_floats, int cus, int* tile_cols,
                              int* ksplit, int* split_col);

/* Measurement hook: a plain copy kernel (reads `bytes`, writes `bytes`, a multiple of 16,
 * device pointers, on `stream`).  Hardware byte counters (rocprofv3 FETCH_SIZE /
 * WRITE_SIZE) are scaled by what they read for this kernel of known size. */
he_status he_calibration_copy(const void* d_src, void* d_dst, size_t bytes, void* stream);

/* Test hook for the sampler's counter-based generator: writes the `count`
 * 32-bit words for vocabulary ids v0 .. v0+count-1 of (seed, sequence b,
 * generation step n) to d_out [count] uint32, on `stream`. */
he_status he_rng_words(uint64_t seed, uint32_t b, uint32_t n, uint32_t v0, int count, uint32_t* d_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HE_H */
