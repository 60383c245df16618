// Shared by the kernel files of the bf16 path (the model's weights are bfloat16) for gfx950 (CDNA4, 64-wide
// wavefronts, MFMA 32x32x16 and 16x16x32 on IEEE half operands).
//
// Operand format.  Everything the matrix cores multiply is IEEE half (fp16): the engine's tiled copies of
// the weight matrices hold the caller's bf16 values converted to half -- exact for every weight of
// magnitude 2^-14 .. 65504 (8 significant bits fit into 11), to the nearest multiple of 2^-24 below that --
// and activations are rounded once to half (11 significant bits, 3 more than bf16) by the kernel that
// produces them.  The KV cache is half as well.  Accumulation, residual stream, LayerNorm statistics,
// soft-max, logits are float.  Measured against the unrounded definition on OPT-13B-shaped layers this sits
// at 5e-3 of the logits; bf16 activations and a bf16 cache (one rounding each) sit at 4e-2.
//
// Tiled operand layout ("blocks"): a matrix R[rows, K] of halves is stored as
// [rows/32][K/16][64 lanes][8 values]; lane = 32*((k%16)/8) + r%32 holds
// R[r][16*kb + 8*(lane/32) + 0..7].  One block is 1 KiB, contiguous, and is
// exactly the per-lane register image of one MFMA operand, so a wavefront
// fetches an operand with a single fully coalesced 16-byte-per-lane load and
// feeds it to the matrix core with no shuffling.  Weights are tiled once at
// engine creation; activations are written in this layout by the kernel that
// produces them (LayerNorm, ReLU epilogue, attention).
//
// Every GEMM computes D[n][m] = sum_k W[n][k] X[m][k] with W blocks as the A
// operand and X blocks as the B operand: lane l then holds, for column
// m = l%32, rows n = 8*(r/4) + 4*(l/32) + r%4 (r = 0..15 accumulators),
// i.e. runs of four consecutive n -- what the epilogues store.
#pragma once
#include <algorithm>
#include <cstdlib>

#include "he_common.h"
#include "kernels.h"

namespace he_bf16 {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one lane's 16 bytes of a block

__device__ __forceinline__ f32x16 mfma_f16(const u32x4& a, const u32x4& b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// two floats -> two halves in one word (first argument in the low half), round to nearest, ties to even
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    typedef float v2f __attribute__((ext_vector_type(2)));
    typedef _Float16 v2h __attribute__((ext_vector_type(2)));
    const v2f v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, v2h));
}
// the two halves of a word as floats
__device__ __forceinline__ float half_lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xFFFFu)); }
__device__ __forceinline__ float half_hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }
// the two bfloat16 of a word (the caller's parameters: biases, gains, embeddings) as floats
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// x in two half terms, hi = half(x), lo = half(x - hi): 22 significant bits (the prompt-pass attention feeds
// its queries and probabilities to the matrix cores this way)
__device__ __forceinline__ void split2(float a, float b, uint32_t& hi, uint32_t& lo) {
    hi = pack2(a, b);
    lo = pack2(a - half_lo(hi), b - half_hi(hi));
}

// index (in 16-byte units) of the slot holding R[r][k0..k0+7], k0 % 8 == 0
__device__ __forceinline__ size_t block_slot(int r, int k0, int KB) {
    return ((size_t)(r >> 5) * KB + (k0 >> 4)) * 64 + (((k0 >> 3) & 1) << 5) + (r & 31);
}

// 16 bytes per lane, global memory -> LDS with no staging registers: lane i's bytes land at lds_block + 16*i
__device__ __forceinline__ void load_block_to_lds(const u32x4* gsrc_lane, u32x4* lds_block) {
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gsrc_lane,
                                     (void __attribute__((address_space(3)))*)lds_block, 16, 0, 0);
}

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14; other counters left at their maxima)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// ----------------------------------------------------------------- epilogues

struct Epi {
    int M, N;               // valid rows (m) and columns (n) of the product
    const bf16_t* bias;     // [N] or null
    float* out;             // STORE: partial sums [ksplit][M][N]; QKV: q [M][H]
    size_t out_split;       // elements between two k-splits of `out`
    u32x4* out_blocks;      // BIAS_RELU: tiled half [M/32][N/16] blocks
    half_t* kv;             // QKV: the KV arena
    const he_dev_state* st;
    int S, layer, H, n_heads, d, max_batch, max_seq;
    float qscale;
    // LM head
    float* logits;          // optional [M][N]
    float* stats;           // [M][n_tiles][4]: max z, sum exp(z - max), best score, z at best
    int* stats_idx;         // [M][n_tiles]: id of best score
    int n_tiles;
    // LayerNorm folded into this GEMM (BIAS_RELU, QKV, LMHEAD on decode rows): X is gamma * x, not
    // normalised; ln_stats[(mt*ln_groups + g)*32 + m%32] = (mean, sum of squared deviations) of x[m]
    // over column group g (ln_gw columns, the last group may be short); c1 = W gamma, c2 = W beta.
    const float2* ln_stats;  // null: X is already normalised
    int ln_groups, ln_gw, ln_cols;
    float ln_eps;
    const float *c1, *c2;   // [N]
    // STORE_LN: the workgroup that finishes a column group last adds the k-split partial sums,
    // bias and residual, and hands the next GEMM gamma * x (out_blocks) and the
    // group's statistics
    float* resid;           // [M][N] residual stream, updated in place
    const bf16_t* gamma;    // [N] gain of the LayerNorm that follows
    float2* stats_out;      // [m_tiles][groups][32]
    int* counters;          // [groups][m_tiles], zero between launches
    // SCORE (tiled LM head over every position): row m = b*S + t is scored on the token that
    // follows it, ids[m + 1]; sc_stats[m][part] = (max z, sum exp(z - max)) over a 128-wide slice
    // of the vocabulary, sc_tgt[m] = z at that token
    const int32_t* ids;
    float2* sc_stats;
    float* sc_tgt;
    int sc_parts;
    // 8-bit weights (half-tile kernel): the accumulators are sums over E4M3 codes; row n of the result
    // is scaled by wscale[n] = 2^e[n]
    const float* wscale;
};

enum { MODE_STORE = 0, MODE_BIAS_RELU = 1, MODE_QKV = 2, MODE_LMHEAD = 3, MODE_STORE_LN = 4, MODE_SCORE = 5 };

// bias words for outputs n0..n0+3 and the cache length, fetched ahead of the epilogue
template <int MODE>
__device__ __forceinline__ uint2 epilogue_bias(const Epi& p, int n0) {
    if ((MODE == MODE_BIAS_RELU || MODE == MODE_QKV) && n0 < p.N) return *reinterpret_cast<const uint2*>(p.bias + n0);
    return make_uint2(0, 0);
}
template <int MODE>
__device__ __forceinline__ int epilogue_len(const Epi& p) {
    if (MODE != MODE_QKV) return 0;
    // two independent loads and a select: a branch on the first would make the second wait for it
    const int ragged = p.st->ragged, len = p.st->cur_len;
    return ragged ? -1 : len;  // -1: look the sequence up
}

// four consecutive outputs D[n0..n0+3][m] (n0 % 4 == 0); bb = their bias, cur_len = cached positions
template <int MODE>
__device__ __forceinline__ void epilogue4(const Epi& p, int m, int n0, int ks, float v0, float v1, float v2, float v3,
                                          uint2 bb, int cur_len) {
    if (m >= p.M || n0 >= p.N) return;  // N is a multiple of 4 wherever this is used
    if (MODE == MODE_STORE) {
        *reinterpret_cast<float4*>(p.out + (size_t)ks * p.out_split + (size_t)m * p.N + n0) =
            make_float4(v0, v1, v2, v3);
    } else if (MODE == MODE_BIAS_RELU) {
        v0 = fmaxf(v0 + bf_lo(bb.x), 0.f);
        v1 = fmaxf(v1 + bf_hi(bb.x), 0.f);
        v2 = fmaxf(v2 + bf_lo(bb.y), 0.f);
        v3 = fmaxf(v3 + bf_hi(bb.y), 0.f);
        const size_t slot = block_slot(m, n0 & ~7, p.N >> 4);
        reinterpret_cast<uint2*>(p.out_blocks + slot)[(n0 >> 2) & 1] = make_uint2(pack2(v0, v1), pack2(v2, v3));
    } else if (MODE == MODE_QKV) {
        v0 += bf_lo(bb.x);
        v1 += bf_hi(bb.x);
        v2 += bf_lo(bb.y);
        v3 += bf_hi(bb.y);
        if (n0 < p.H) {
            *reinterpret_cast<float4*>(p.out + (size_t)m * p.H + n0) =
                make_float4(v0 * p.qscale, v1 * p.qscale, v2 * p.qscale, v3 * p.qscale);
        } else {
            const int which = n0 >= 2 * p.H, c = n0 - (which ? 2 * p.H : p.H);
            const int b = row_seq(p.st, m, p.S);
            int t = cur_len + (m % p.S);
            if (cur_len < 0) {  // sequences of different lengths; padding rows append nothing
                const int tr = m % p.S - row_pad(p.st, b);
                if (tr < 0) return;
                t = seq_len(p.st, b) + tr;
            }
            half_t* dst = p.kv + kv_index(p.layer, which, b, c / p.d, t, p.max_batch, p.n_heads, p.max_seq, p.d) + (c % p.d);
            *reinterpret_cast<uint2*>(dst) = make_uint2(pack2(v0, v1), pack2(v2, v3));
        }
    }
}

// Folded LayerNorm, consumer side: mean and 1/sqrt(var + eps) of each of the 32 rows of a slice from the
// per-column-group statistics the producer left ([group][32 rows](mean, sum of squared deviations)).
// Pairwise-update form, pivoted on the first group's mean so that the cross terms stay small.  The work is
// spread over a workgroup and taken off the tail of the kernel: wavefront w takes the groups
// g = 2w + lane/32 (mod 2 WAVES), a lane one row of them; the loads are issued (ln_issue) before the first
// weight loads, the partial sums formed (ln_partial) while those weights are in flight and left in LDS ahead
// of the barrier that ends the k loop; after it every lane adds the WAVES partial sums of the rows it needs in
// wavefront order (ln_finish).
constexpr int kLnBatch = 6;  // statistics a lane keeps in flight; more groups than 2 WAVES kLnBatch are loaded late
struct LnLoads { float2 e[kLnBatch]; float pivot; };

template <int WAVES>
__device__ __forceinline__ void ln_issue(LnLoads& L, const Epi& p, int mt, int wave, int lane) {
    const float2* gs = p.ln_stats + (size_t)mt * p.ln_groups * 32 + (lane & 31);
    L.pivot = gs[0].x;
    const int g0 = 2 * wave + (lane >> 5);
#pragma unroll
    for (int i = 0; i < kLnBatch; ++i) {
        const int g = g0 + i * 2 * WAVES;
        L.e[i] = g < p.ln_groups ? gs[(size_t)g * 32] : make_float2(0.f, 0.f);
    }
}

// lnp: [WAVES][4][32] floats of LDS
template <int WAVES>
__device__ __forceinline__ void ln_partial(const LnLoads& L, const Epi& p, int mt, int wave, int lane, float* lnp) {
    const int g0 = 2 * wave + (lane >> 5);
    float s1 = 0.f, s2 = 0.f, sm = 0.f;
    auto add = [&](int g, float2 e) {
        const float cnt = (float)min(p.ln_gw, p.ln_cols - g * p.ln_gw), dlt = e.x - L.pivot;
        s1 += cnt * dlt;
        s2 += cnt * dlt * dlt;
        sm += e.y;
    };
#pragma unroll
    for (int i = 0; i < kLnBatch; ++i) {
        const int g = g0 + i * 2 * WAVES;
        if (g < p.ln_groups) add(g, L.e[i]);
    }
    const float2* gs = p.ln_stats + (size_t)mt * p.ln_groups * 32 + (lane & 31);
    for (int g = g0 + kLnBatch * 2 * WAVES; g < p.ln_groups; g += 2 * WAVES) add(g, gs[(size_t)g * 32]);
    s1 += __shfl_xor(s1, 32);
    s2 += __shfl_xor(s2, 32);
    sm += __shfl_xor(sm, 32);
    if (lane < 32) {
        float* o = lnp + wave * 4 * 32 + lane;
        o[0] = s1; o[32] = s2; o[64] = sm; o[96] = L.pivot;
    }
}

template <int WAVES>
__device__ __forceinline__ float2 ln_finish(const float* lnp, int row, const Epi& p) {
    float s1 = 0.f, s2 = 0.f, sm = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        const float* o = lnp + w * 4 * 32 + row;
        s1 += o[0]; s2 += o[32]; sm += o[64];
    }
    const float pivot = lnp[96 + row];
    const float inv = 1.0f / (float)p.ln_cols;
    const float mean = pivot + s1 * inv;
    const float var = fmaxf((sm + s2 - s1 * s1 * inv) * inv, 0.f);
    return make_float2(mean, 1.0f / sqrtf(var + p.ln_eps));
}

// Compute units of the current device (256 on an MI355X; also the answer when there is no device).
inline int num_cus() {
    static int n_cus = 0;
    if (n_cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        n_cus = n;
    }
    return n_cus;
}

inline Epi make_epi(int M, int N, const bf16_gemm_args& a) {
    Epi p{};
    p.M = M; p.N = N; p.bias = (const bf16_t*)a.bias; p.out = a.out; p.out_split = a.out_split;
    p.out_blocks = (u32x4*)a.out_blocks; p.kv = (half_t*)a.kv; p.st = a.st;
    p.S = a.S; p.layer = a.layer; p.H = a.H; p.n_heads = a.n_heads; p.d = a.n_heads ? a.H / a.n_heads : 0;
    p.max_batch = a.max_batch; p.max_seq = a.max_seq; p.qscale = a.qscale;
    p.ln_stats = (const float2*)a.ln_stats; p.ln_groups = a.ln_groups; p.ln_gw = a.ln_gw; p.ln_cols = a.ln_cols;
    p.ln_eps = a.ln_eps; p.c1 = a.c1; p.c2 = a.c2;
    p.resid = a.resid; p.gamma = (const bf16_t*)a.gamma; p.stats_out = (float2*)a.stats_out; p.counters = a.counters;
    p.wscale = a.wscale;
    return p;
}

}  // namespace he_bf16
