// Internal definitions shared by the engine and its kernels (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;  // raw bfloat16: the upper 16 bits of an IEEE float
typedef uint16_t half_t;  // raw IEEE half (what the bf16 path's matrix-core operands and KV cache hold)

// Device-resident generation state.  Every kernel reads positions, step
// numbers and sampling parameters from here rather than from launch
// arguments, so a captured decode step can be replayed unchanged.
struct he_dev_state {
    int cur_len;       // positions already in the KV cache, per sequence (uniform batches)
    int step;          // generation step n of the token about to be sampled
    int mode;          // 0 greedy, 1 Gumbel-max
    float temperature;
    uint32_t seed_lo, seed_hi;
    int ragged;        // 1: sequences differ in length -- per-sequence numbers live in seq[]
    int max_batch;
    int eos_id, pad_id;  // end-of-sequence stop (eos_id < 0: none) and the filler written after it
    int n_active;      // sequences that have not produced eos_id yet
    int reserved[5];
    // [0 .. max_batch): cached positions of sequence b;  [max_batch .. 2 max_batch): left padding of
    // the rows now going through the model (0 outside a prompt pass);  [2 .. 3 max_batch): 1 once the
    // sequence has produced eos_id;  [3 .. 4 max_batch): tokens produced so far;  [4 .. 5 max_batch): the
    // sequence whose token goes through row r of a decode step (r itself, until he_generate_ragged drops the
    // rows of sequences that have ended)
    int seq[1];
};

__host__ __device__ inline size_t he_dev_state_bytes(int max_batch) {
    return sizeof(he_dev_state) + (size_t)5 * max_batch * sizeof(int);
}
// positions of sequence b already in the cache
__device__ __forceinline__ int seq_len(const he_dev_state* st, int b) { return st->ragged ? st->seq[b] : st->cur_len; }
// leading rows of sequence b in this pass that are padding, not tokens
__device__ __forceinline__ int row_pad(const he_dev_state* st, int b) { return st->ragged ? st->seq[st->max_batch + b] : 0; }
__device__ __forceinline__ bool seq_done(const he_dev_state* st, int b) {
    return st->ragged && st->seq[2 * st->max_batch + b] != 0;
}
// The sequence of row m of a pass of S rows per sequence.  Rows of a decode step (S = 1) go through the map;
// cache slot, per-sequence state, sampling noise and outputs belong to the sequence, activations to the row.
__device__ __forceinline__ int row_seq(const he_dev_state* st, int m, int S) {
    if (S != 1) return m / S;
    return st->ragged ? st->seq[4 * st->max_batch + m] : m;
}

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// Two floats -> two bf16 in one word (first argument in the low half), round to nearest, ties to even:
// the hardware's packed conversion, one instruction for the pair.
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
    typedef float he_f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 he_bf16x2 __attribute__((ext_vector_type(2)));
    const he_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, he_bf16x2));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(f32x2_to_bf16x2(f, 0.f) & 0xFFFFu); }

__device__ __forceinline__ float ld_f32(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld_f32(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void st_val(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st_val(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }

// ---- Philox-4x32-10 (Salmon et al., SC'11): word 0 for counter (v, n, b, 0), key = seed ----
__device__ __forceinline__ uint32_t philox_word0(uint32_t v, uint32_t n, uint32_t b, uint32_t k0, uint32_t k1) {
    uint32_t c0 = v, c1 = n, c2 = b, c3 = 0u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return c0;
}

// Gumbel noise for vocabulary id v: u = ((x >> 9) + 1/2) 2^-23 lies strictly in (0,1)
__device__ __forceinline__ float gumbel_from_word(uint32_t x) {
    const float u = ((float)(x >> 9) + 0.5f) * 1.1920928955078125e-07f;  // 2^-23
    return -logf(-logf(u));
}

// KV arena: [layer][k|v][max_batch][head][max_seq_len][head_dim]
__host__ __device__ __forceinline__ size_t kv_index(int layer, int kv, int b, int h, int t, int max_batch, int n_heads,
                                                    int max_seq, int d) {
    return ((((size_t)(layer * 2 + kv) * max_batch + b) * n_heads + h) * max_seq + t) * (size_t)d;
}
