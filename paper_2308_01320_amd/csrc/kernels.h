// Host-side launchers of the engine's kernels (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

struct he_dev_state;

enum { EPI_STORE = 0, EPI_BIAS_RELU = 1, EPI_QKV = 2 };

// ---- plain kernels (kernels_plain.hip): float activations, row-major; bf16 != 0 selects bf16 storage
void plain_embed(hipStream_t s, int bf16, const int32_t* ids, const void* tok, const void* pos, float* x,
                 const he_dev_state* st, int M, int S, int H, int V, int pos_offset);
void plain_ln(hipStream_t s, int bf16, float* r, const float* y, const void* ybias, const void* g, const void* b,
              float* a, int rows, int H, float eps, int in_mul, int in_add, int writeback);
void plain_gemm(hipStream_t s, int bf16, const float* A, const void* W, const void* bias, int M, int N, int K, int epi,
                float* out, void* kv, const he_dev_state* st, int S, int layer, int H, int n_heads, int max_batch,
                int max_seq, float qscale);
void plain_attn(hipStream_t s, int bf16, const float* q, const void* kv, float* o, const he_dev_state* st, int M, int S,
                int layer, int H, int n_heads, int max_batch, int max_seq);
void plain_lm_head(hipStream_t s, int bf16, const float* xf, const void* W, float* logits, int B, int H, int V);

// ---- shared small kernels
void launch_sample(hipStream_t s, const float* logits, int B, int V, const he_dev_state* st, int32_t* ids_out,
                   float* lp_out, int out_stride, int out_at_step, int32_t* cur_ids);
void launch_set_state(hipStream_t s, he_dev_state* st, int cur_len, int step, int set_pos, int mode, float temperature,
                      uint64_t seed);
void launch_advance_state(hipStream_t s, he_dev_state* st, int tokens);
void launch_rng_words(hipStream_t s, uint64_t seed, uint32_t b, uint32_t n, uint32_t v0, int count, uint32_t* out);
void launch_copy_out(hipStream_t s, const int32_t* ids, const float* lp, int32_t* out_ids, float* out_lp, int count);
