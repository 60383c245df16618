// bf16 path kernels for gfx950 (CDNA4, 64-wide wavefronts, MFMA 32x32x16 bf16).
//
// Tiled operand layout ("blocks"): a bf16 matrix R[rows, K] is stored as
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
//
// All
// GEMM activations are carried as two bf16 terms, x = hi + lo with
// lo = bf16(x - hi): a second MFMA per block against the same weight registers
// takes the activation rounding error from 2^-9 to 2^-17.  Decode-shaped GEMMs
// are bound by the weight stream, so there it costs no time; the prompt pass
// pays twice the matrix-core work for it.
#include <algorithm>
#include <cstdlib>

#include "he_common.h"
#include "kernels.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one lane's 16 bytes of a block

__device__ __forceinline__ f32x16 mfma_bf16(const u32x4& a, const u32x4& b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// x = hi + lo in two bf16 terms
__device__ __forceinline__ void split2(float a, float b, uint32_t& hi, uint32_t& lo) {
    const bf16_t ha = f32_to_bf16(a), hb = f32_to_bf16(b);
    hi = (uint32_t)ha | ((uint32_t)hb << 16);
    lo = pack2(a - bf16_to_f32(ha), b - bf16_to_f32(hb));
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

// ----------------------------------------------------------------- weight tiling

__global__ void tile_rows_kernel(const bf16_t* __restrict__ src, u32x4* __restrict__ dst, int R, int K, size_t total) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int KB = K >> 4;
    const int lane = (int)(idx & 63);
    const int kb = (int)((idx >> 6) % KB);
    const int rt = (int)((idx >> 6) / KB);
    const int r = rt * 32 + (lane & 31), k = kb * 16 + (lane >> 5) * 8;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (r < R) v = *reinterpret_cast<const u32x4*>(src + (size_t)r * K + k);
    dst[idx] = v;
}

// The same with a low-rank adapter folded in: dst = tiled bf16(W + scale * B A), A [rank, K], B [R, rank].
// The sum fixes a bf16 rounding, so its order is part of the definition: products B[r][j] A[j][k]
// (exact in float for bf16 inputs) are added one by one for j = 0..rank-1, then W + scale * that, every
// operation a separate float rounding (no fused multiply-add).
__global__ void tile_rows_lora_kernel(const bf16_t* __restrict__ src, u32x4* __restrict__ dst, int R, int K, size_t total,
                                      const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, int rank, float scale) {
#pragma clang fp contract(off)  // scale * t and the addition to W round separately, as stated
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int KB = K >> 4;
    const int lane = (int)(idx & 63);
    const int kb = (int)((idx >> 6) % KB);
    const int rt = (int)((idx >> 6) / KB);
    const int r = rt * 32 + (lane & 31), k = kb * 16 + (lane >> 5) * 8;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (r < R) {
        const u32x4 w = *reinterpret_cast<const u32x4*>(src + (size_t)r * K + k);
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
        float t[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int j = 0; j < rank; ++j) {
            const float b = bf16_to_f32(B[(size_t)r * rank + j]);
            const u32x4 a = *reinterpret_cast<const u32x4*>(A + (size_t)j * K + k);
            const uint32_t aw[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p0 = b * __uint_as_float(aw[i] << 16), p1 = b * __uint_as_float(aw[i] & 0xFFFF0000u);
                t[2 * i] = t[2 * i] + p0;
                t[2 * i + 1] = t[2 * i + 1] + p1;
            }
        }
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float s0 = scale * t[2 * i], s1 = scale * t[2 * i + 1];  // plain operators: the pragma above covers them
            const float lo = __uint_as_float(ww[i] << 16) + s0;
            const float hi = __uint_as_float(ww[i] & 0xFFFF0000u) + s1;
            o[i] = pack2(lo, hi);
        }
        v = u32x4{o[0], o[1], o[2], o[3]};
    }
    dst[idx] = v;
}

// ----------------------------------------------------------------- 8-bit weight storage
//
// Row n of a weight matrix is kept as E4M3 codes q[n][:] and a power-of-two scale 2^e[n], e[n] the
// smallest integer with max|W[n][:]| 2^-e[n] <= 448; q = nearest E4M3 value of W 2^-e (ties to even).
// Scaling by a power of two is exact, so the codes are a rounding decision on the weights' own values.

// one wavefront per row: e[n] and 2^e[n]
__global__ __launch_bounds__(256) void row_exp_kernel(const bf16_t* __restrict__ src, int R, int K, int* __restrict__ exps,
                                                      float* __restrict__ scales) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= R) return;
    float amax = 0.f;
    for (int k = lane * 8; k < K; k += 512) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(src + (size_t)row * K + k);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            amax = fmaxf(amax, fabsf(__uint_as_float(w[j] << 16)));
            amax = fmaxf(amax, fabsf(__uint_as_float(w[j] & 0xFFFF0000u)));
        }
    }
    for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    if (lane == 0) {
        int x = 0, e = 0;
        if (amax > 0.f) {
            const float f = frexpf(amax, &x);  // amax = f 2^x, f in [0.5, 1); 448 = 0.875 2^9
            e = f <= 0.875f ? x - 9 : x - 8;
        }
        exps[row] = e;
        scales[row] = ldexpf(1.0f, e);
    }
}

// eight bf16 values (one 16-byte load) -> eight E4M3 codes
__device__ __forceinline__ uint2 quant8_e4m3(const u32x4& v, float inv_scale) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float f[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f[2 * j] = __uint_as_float(w[j] << 16) * inv_scale;
        f[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u) * inv_scale;
    }
    int lo = 0, hi = 0;
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
    return make_uint2((uint32_t)lo, (uint32_t)hi);
}

// row-major codes (a utility, and what the tests compare bit for bit)
__global__ void quant_rows_kernel(const bf16_t* __restrict__ src, const int* __restrict__ exps, uint2* __restrict__ codes,
                                  int R, int K) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)R * (K / 8)) return;
    const int row = (int)(idx / (K / 8));
    codes[idx] = quant8_e4m3(reinterpret_cast<const u32x4*>(src)[idx], ldexpf(1.0f, -exps[row]));
}

// codes in the half-tile kernel's units: [R/16][K/64][64 lanes][16 bytes]
__global__ void quant_units_kernel(const bf16_t* __restrict__ src, const int* __restrict__ exps, u32x4* __restrict__ dst,
                                   int R, int K, size_t total) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int KQ = K >> 6;
    const int lane = (int)(idx & 63);
    const int j = (int)((idx >> 6) % KQ), g = (int)((idx >> 6) / KQ);
    const int row = g * 16 + (lane & 15), k0 = j * 64 + 8 * (lane >> 4);
    u32x4 out = u32x4{0u, 0u, 0u, 0u};
    if (row < R) {
        const float inv = ldexpf(1.0f, -exps[row]);
        const uint2 a = quant8_e4m3(*reinterpret_cast<const u32x4*>(src + (size_t)row * K + k0), inv);
        const uint2 b = quant8_e4m3(*reinterpret_cast<const u32x4*>(src + (size_t)row * K + k0 + 32), inv);
        out = u32x4{a.x, a.y, b.x, b.y};
    }
    dst[idx] = out;
}

// units -> the bf16 32x16 blocks the tiled GEMMs read (the dequantised weights are bf16 values exactly)
__global__ void dequant_units_kernel(const u32x4* __restrict__ units, const float* __restrict__ scales,
                                     u32x4* __restrict__ dst, int R, int K, size_t total) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int KB = K >> 4, KQ = K >> 6;
    const int lane = (int)(idx & 63);
    const int kb = (int)((idx >> 6) % KB), rt = (int)((idx >> 6) / KB);
    const int row = rt * 32 + (lane & 31), k0 = kb * 16 + 8 * (lane >> 5);
    u32x4 out = u32x4{0u, 0u, 0u, 0u};
    if (row < R) {
        const int g = row >> 4, j = k0 >> 6, off = k0 & 63;
        const u32x4 u = units[((size_t)g * KQ + j) * 64 + 16 * ((off & 31) >> 3) + (row & 15)];
        const uint32_t c0 = off & 32 ? u.z : u.x, c1 = off & 32 ? u.w : u.y;
        const float sc = scales[row];
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        const f32x2 f0 = __builtin_amdgcn_cvt_pk_f32_fp8(c0, false), f1 = __builtin_amdgcn_cvt_pk_f32_fp8(c0, true);
        const f32x2 f2 = __builtin_amdgcn_cvt_pk_f32_fp8(c1, false), f3 = __builtin_amdgcn_cvt_pk_f32_fp8(c1, true);
        out = u32x4{pack2(f0.x * sc, f0.y * sc), pack2(f1.x * sc, f1.y * sc), pack2(f2.x * sc, f2.y * sc),
                    pack2(f3.x * sc, f3.y * sc)};
    }
    dst[idx] = out;
}

// ----------------------------------------------------------------- epilogues

struct Epi {
    int M, N;               // valid rows (m) and columns (n) of the product
    const bf16_t* bias;     // [N] or null
    float* out;             // STORE: partial sums [ksplit][M][N]; QKV: q [M][H]
    size_t out_split;       // elements between two k-splits of `out`
    u32x4* out_blocks;      // BIAS_RELU: tiled bf16 [M/32][N/16] blocks (hi term)
    u32x4* out_blocks_lo;   // BIAS_RELU: lo term, or null
    bf16_t* kv;             // QKV: the KV arena
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
    // bias and residual, and hands the next GEMM gamma * x (out_blocks, out_blocks_lo) and the
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
    return MODE == MODE_QKV ? (p.st->ragged ? -1 : p.st->cur_len) : 0;  // -1: look the sequence up
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
        v0 = fmaxf(v0 + __uint_as_float(bb.x << 16), 0.f);
        v1 = fmaxf(v1 + __uint_as_float(bb.x & 0xFFFF0000u), 0.f);
        v2 = fmaxf(v2 + __uint_as_float(bb.y << 16), 0.f);
        v3 = fmaxf(v3 + __uint_as_float(bb.y & 0xFFFF0000u), 0.f);
        const size_t slot = block_slot(m, n0 & ~7, p.N >> 4);
        uint32_t h0, h1, l0, l1;
        split2(v0, v1, h0, l0);
        split2(v2, v3, h1, l1);
        reinterpret_cast<uint2*>(p.out_blocks + slot)[(n0 >> 2) & 1] = make_uint2(h0, h1);
        if (p.out_blocks_lo) reinterpret_cast<uint2*>(p.out_blocks_lo + slot)[(n0 >> 2) & 1] = make_uint2(l0, l1);
    } else if (MODE == MODE_QKV) {
        v0 += __uint_as_float(bb.x << 16);
        v1 += __uint_as_float(bb.x & 0xFFFF0000u);
        v2 += __uint_as_float(bb.y << 16);
        v3 += __uint_as_float(bb.y & 0xFFFF0000u);
        if (n0 < p.H) {
            *reinterpret_cast<float4*>(p.out + (size_t)m * p.H + n0) =
                make_float4(v0 * p.qscale, v1 * p.qscale, v2 * p.qscale, v3 * p.qscale);
        } else {
            const int which = n0 >= 2 * p.H, c = n0 - (which ? 2 * p.H : p.H);
            const int b = m / p.S;
            int t = cur_len + (m % p.S);
            if (cur_len < 0) {  // sequences of different lengths; padding rows append nothing
                const int tr = m % p.S - row_pad(p.st, b);
                if (tr < 0) return;
                t = seq_len(p.st, b) + tr;
            }
            bf16_t* dst = p.kv + kv_index(p.layer, which, b, c / p.d, t, p.max_batch, p.n_heads, p.max_seq, p.d) + (c % p.d);
            *reinterpret_cast<uint2*>(dst) = make_uint2(pack2(v0, v1), pack2(v2, v3));
        }
    }
}

// Folded LayerNorm, consumer side: mean and 1/sqrt(var + eps) of row `row` (0..31 of this slice of
// rows) from the per-column-group statistics the producer left, staged in LDS as
// [group][32 rows](mean, sum of squared deviations).  Pairwise-update form, pivoted on the first
// group's mean so that the cross terms stay small.
__device__ __forceinline__ float2 ln_row_from_groups(const float* lds_stats, int row, const Epi& p) {
    const float2* gs = reinterpret_cast<const float2*>(lds_stats) + row;
    const float pivot = gs[0].x;
    float s1 = 0.f, s2 = 0.f, sm = 0.f;
    for (int g = 0; g < p.ln_groups; ++g) {
        const float2 e = gs[g * 32];
        const float cnt = (float)min(p.ln_gw, p.ln_cols - g * p.ln_gw), dlt = e.x - pivot;
        s1 += cnt * dlt;
        s2 += cnt * dlt * dlt;
        sm += e.y;
    }
    const float inv = 1.0f / (float)p.ln_cols;
    const float mean = pivot + s1 * inv;
    const float var = fmaxf((sm + s2 - s1 * s1 * inv) * inv, 0.f);
    return make_float2(mean, 1.0f / sqrtf(var + p.ln_eps));
}

// ----------------------------------------------------------------- k-split GEMM -> residual rows + next LayerNorm's input
//
// Tail of the decode-shaped out-projection / FC2 GEMMs (MODE_STORE_LN), shared by the 32-row and the
// 16-row kernel.  On entry every thread holds ITEMS quads v[i][0..3]: this workgroup's k-split partial
// sums of outputs n0[i]..n0[i]+3 of row mrow[i] (live[i]: the quad exists).  rslot[i] says which of the
// lane's 32/LG rows the quad belongs to: lanes with equal lane % LG hold different columns of the same
// rows (LG = 32: one row per lane; LG = 16: two).
//
// The partial sums cross workgroups (and XCDs, each with an L2 of its own) inside one launch.  They
// travel as agent-scope atomic words -- written through to, and read from, the level every XCD shares
// -- so no cache has to be flushed or invalidated (an agent-scope fence does that to whole L2s and cost
// 45 us per launch).  The words of one (split, item, r) are laid out thread after thread: every access
// is a contiguous 256 bytes per wavefront.  Each workgroup publishes its partial sums, waits for the
// stores to be acknowledged and counts itself in; whoever counts last for the column group reads all
// splits back -- its own included -- and adds them in split order, so the sum does not depend on which
// workgroup that was.  Nobody waits for anybody: the others are done.  The last one adds bias and
// residual, writes the residual rows back, gamma * x as two-term blocks, and the group's statistics
// (mean and sum of squared deviations per row over the group's `cnt` columns, fixed summation order).
// Returns to the caller, who returns.
template <int ITEMS, int WAVES, int LG>
__device__ __forceinline__ void store_ln_tail(const Epi& p, int ksplit, int ks, int grp, int groups, int mt, float cnt,
                                              const float (&v)[ITEMS][4], const int (&mrow)[ITEMS],
                                              const int (&n0)[ITEMS], const bool (&live)[ITEMS],
                                              const int (&rslot)[ITEMS]) {
    constexpr int NSLOT = 32 / LG;
    __shared__ int s_last;
    __shared__ float sred[2][WAVES][32];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t cell = (size_t)grp * gridDim.y + mt;
    constexpr size_t kPer = (size_t)ITEMS * 4 * WAVES * 64;  // words of one split of one column group
    float* scratch = p.out + cell * ksplit * kPer + threadIdx.x;
    if (ksplit > 1) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            if (!live[i]) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                __hip_atomic_store(scratch + (ks * kPer + (size_t)(i * 4 + r) * WAVES * 64), v[i][r], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0)
            s_last = __hip_atomic_fetch_add(p.counters + cell, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == ksplit - 1;
        __syncthreads();
        if (!s_last) return;
    }
    float x[ITEMS][4];
    float srow[NSLOT];
#pragma unroll
    for (int r = 0; r < NSLOT; ++r) srow[r] = 0.f;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        x[i][0] = x[i][1] = x[i][2] = x[i][3] = 0.f;
        if (!live[i]) continue;
        const size_t at = (size_t)mrow[i] * p.N + n0[i];
        const float4 rr = *reinterpret_cast<const float4*>(p.resid + at);
        const uint2 bb = *reinterpret_cast<const uint2*>(p.bias + n0[i]);
        const uint2 gg = *reinterpret_cast<const uint2*>(p.gamma + n0[i]);
        float4 tot = make_float4(v[i][0], v[i][1], v[i][2], v[i][3]);
        if (ksplit > 1) {
            float y[8][4];
#pragma unroll
            for (int k = 0; k < 8; ++k)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    y[k][r] = __hip_atomic_load(scratch + (min(k, ksplit - 1) * kPer + (size_t)(i * 4 + r) * WAVES * 64),
                                                __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            tot = make_float4(y[0][0], y[0][1], y[0][2], y[0][3]);
#pragma unroll
            for (int k = 1; k < 8; ++k)
                if (k < ksplit) { tot.x += y[k][0]; tot.y += y[k][1]; tot.z += y[k][2]; tot.w += y[k][3]; }
        }
        x[i][0] = rr.x + (tot.x + __uint_as_float(bb.x << 16));
        x[i][1] = rr.y + (tot.y + __uint_as_float(bb.x & 0xFFFF0000u));
        x[i][2] = rr.z + (tot.z + __uint_as_float(bb.y << 16));
        x[i][3] = rr.w + (tot.w + __uint_as_float(bb.y & 0xFFFF0000u));
        *reinterpret_cast<float4*>(p.resid + at) = make_float4(x[i][0], x[i][1], x[i][2], x[i][3]);
        uint32_t h0, h1, l0, l1;
        split2(x[i][0] * __uint_as_float(gg.x << 16), x[i][1] * __uint_as_float(gg.x & 0xFFFF0000u), h0, l0);
        split2(x[i][2] * __uint_as_float(gg.y << 16), x[i][3] * __uint_as_float(gg.y & 0xFFFF0000u), h1, l1);
        const size_t slot = block_slot(mrow[i], n0[i] & ~7, p.N >> 4);
        reinterpret_cast<uint2*>(p.out_blocks + slot)[(n0[i] >> 2) & 1] = make_uint2(h0, h1);
        reinterpret_cast<uint2*>(p.out_blocks_lo + slot)[(n0[i] >> 2) & 1] = make_uint2(l0, l1);
        const float part = (x[i][0] + x[i][1]) + (x[i][2] + x[i][3]);
#pragma unroll
        for (int r = 0; r < NSLOT; ++r)
            if (rslot[i] == r) srow[r] += part;
    }
    // row sums over the lanes that share a row, then over the wavefronts
#pragma unroll
    for (int r = 0; r < NSLOT; ++r) {
#pragma unroll
        for (int o = LG; o < 64; o <<= 1) srow[r] += __shfl_xor(srow[r], o);
        if (lane < LG) sred[0][wave][LG * r + lane] = srow[r];
    }
    __syncthreads();
    float mean[NSLOT], q[NSLOT];
#pragma unroll
    for (int r = 0; r < NSLOT; ++r) {
        float tot = 0.f;
#pragma unroll
        for (int ww = 0; ww < WAVES; ++ww) tot += sred[0][ww][LG * r + (lane & (LG - 1))];
        mean[r] = tot / cnt;
        q[r] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        if (!live[i]) continue;
#pragma unroll
        for (int r = 0; r < NSLOT; ++r)
            if (rslot[i] == r) {
                const float d0 = x[i][0] - mean[r], d1 = x[i][1] - mean[r], d2 = x[i][2] - mean[r], d3 = x[i][3] - mean[r];
                q[r] += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
            }
    }
#pragma unroll
    for (int r = 0; r < NSLOT; ++r) {
#pragma unroll
        for (int o = LG; o < 64; o <<= 1) q[r] += __shfl_xor(q[r], o);
        if (lane < LG) sred[1][wave][LG * r + lane] = q[r];
    }
    __syncthreads();
    if (threadIdx.x < 32) {
        float m2 = 0.f, tot = 0.f;
#pragma unroll
        for (int ww = 0; ww < WAVES; ++ww) { m2 += sred[1][ww][lane]; tot += sred[0][ww][lane]; }
        p.stats_out[((size_t)mt * groups + grp) * 32 + lane] = make_float2(tot / cnt, m2);
    }
    if (threadIdx.x == 0 && ksplit > 1)  // ready for the next launch
        __hip_atomic_store(p.counters + cell, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ----------------------------------------------------------------- skinny GEMM (decode, LM head)
//
// At most 32 rows per grid.y slice: weights are streamed exactly once from HBM,
// straight from global memory into MFMA operand registers.  A workgroup of four
// wavefronts owns NT consecutive 32-row weight tiles and one k-split; its
// wavefronts divide the k range, keep U blocks per stream in flight (NT weight
// streams plus the hi and lo activation streams out of L2, which every weight
// tile reuses from registers), and combine their accumulators through LDS.  The
// sum over k-splits (STORE mode) is taken, in a fixed order, by the LayerNorm
// kernel that consumes it.
//
// What bounds this kernel is the number of bytes one CU can keep in flight, so
// the launcher picks NT (and the k-split) to put one equally loaded workgroup on
// as many of the CUs as the shape allows: more workgroups than CUs double up
// on some CUs and the whole launch waits for those.

template <int NT, int U>
struct SkinnyRegs {
    u32x4 w[NT][U], xh[U], xl[U];
};

template <int NT, int U>
__device__ __forceinline__ void skinny_load(SkinnyRegs<NT, U>& r, const u32x4* (&w)[NT], const u32x4*& xh,
                                            const u32x4*& xl) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int t = 0; t < NT; ++t) r.w[t][u] = __builtin_nontemporal_load(w[t] + u * 64);
        r.xh[u] = xh[u * 64];
        r.xl[u] = xl[u * 64];
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) w[t] += U * 64;
    xh += U * 64;
    xl += U * 64;
}

template <int NT, int U>
__device__ __forceinline__ void skinny_mma(const SkinnyRegs<NT, U>& r, f32x16 (&acc)[NT]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = mfma_bf16(r.w[t][u], r.xh[u], acc[t]);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = mfma_bf16(r.w[t][u], r.xl[u], acc[t]);
    }
}

template <int MODE, int NT, int U, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gemm_skinny_kernel(const u32x4* __restrict__ Wp,
                                                                 const u32x4* __restrict__ Xhi,
                                                                 const u32x4* __restrict__ Xlo, int KB, int n_tiles,
                                                                 int ksplit, Epi p) {
    __shared__ float red[WAVES][NT][16][64];
    extern __shared__ float dyn_lds[];  // LayerNorm statistics of this slice of rows, when folded
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int grp = blockIdx.x / ksplit, ks = blockIdx.x % ksplit;
    const int mt = blockIdx.y;
    const int parts = ksplit * WAVES, part = ks * WAVES + wave;
    const int kb0 = (int)(((long)part * KB) / parts), kb1 = (int)(((long)(part + 1) * KB) / parts);
    constexpr bool FOLDABLE = MODE == MODE_BIAS_RELU || MODE == MODE_QKV || MODE == MODE_LMHEAD;
    const bool fold = FOLDABLE && p.ln_stats != nullptr;
    if (fold) {  // statistics go straight to LDS, 1 KiB per instruction; they are read after the k loop
        const int chunks = (p.ln_groups * 32 * (int)sizeof(float2) + 1023) >> 10;  // the buffer is padded to this
        const u32x4* src = reinterpret_cast<const u32x4*>(p.ln_stats + (size_t)mt * p.ln_groups * 32);
        for (int c = wave; c < chunks; c += WAVES)
            load_block_to_lds(src + c * 64 + lane, reinterpret_cast<u32x4*>(dyn_lds) + c * 64);
    }
    const u32x4* w[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)  // tiles past the last one are computed from the last one, never stored
        w[t] = Wp + ((size_t)min(grp * NT + t, n_tiles - 1) * KB + kb0) * 64 + lane;
    const u32x4* xh = Xhi + ((size_t)mt * KB + kb0) * 64 + lane;
    const u32x4* xl = Xlo + ((size_t)mt * KB + kb0) * 64 + lane;
    // After the k loop the NT*4 (tile, row-quad) items of the workgroup are shared out over its
    // wavefronts: item = wave + i*WAVES -> tile item/4, rows 8*(item%4) + 4*(lane/32) + 0..3.
    constexpr int ITEMS = (NT * 4 + WAVES - 1) / WAVES;
    // epilogue operands are requested now, long before they are used
    uint2 bias_w[ITEMS];
    float4 c1w[ITEMS], c2w[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int item = wave + i * WAVES, tile = grp * NT + (item >> 2);
        const int n0 = tile * 32 + 8 * (item & 3) + 4 * (lane >> 5);
        const bool live = item < NT * 4 && tile < n_tiles;
        bias_w[i] = live ? epilogue_bias<MODE>(p, n0) : make_uint2(0, 0);
        if (FOLDABLE) {
            c1w[i] = c2w[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (fold && live) {  // c1 and c2 are padded to whole tiles
                c1w[i] = *reinterpret_cast<const float4*>(p.c1 + n0);
                c2w[i] = *reinterpret_cast<const float4*>(p.c2 + n0);
            }
        }
    }
    const int cur_len = epilogue_len<MODE>(p);
    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x16{};
    int n = kb1 - kb0;
    if (n >= U) {
        SkinnyRegs<NT, U> ra;
        skinny_load<NT, U>(ra, w, xh, xl);
        n -= U;
        while (n >= U) {
            SkinnyRegs<NT, U> rb;
            skinny_load<NT, U>(rb, w, xh, xl);
            n -= U;
            skinny_mma<NT, U>(ra, acc);
            ra = rb;
        }
        skinny_mma<NT, U>(ra, acc);
    }
    for (; n > 0; --n) {
        SkinnyRegs<NT, 1> r1;
        skinny_load<NT, 1>(r1, w, xh, xl);
        skinny_mma<NT, 1>(r1, acc);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave][t][r][lane] = acc[t][r];
    if (FOLDABLE) wait_vmcnt<0>();  // the statistics have landed in LDS
    __syncthreads();
    const int m = mt * 32 + (lane & 31);
    float v[ITEMS][4];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int item = wave + i * WAVES, t = item >> 2, q = item & 3;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float sum = 0.f;
            if (item < NT * 4) {
#pragma unroll
                for (int ww = 0; ww < WAVES; ww += 2) sum += red[ww][t][q * 4 + r][lane] + red[ww + 1][t][q * 4 + r][lane];
            }
            v[i][r] = sum;
        }
    }
    if (fold) {  // W LN(x) = rstd * (W (gamma x) - mean * W gamma) + W beta
        const float2 mr = ln_row_from_groups(dyn_lds, lane & 31, p);
        const float mean = mr.x, rstd = mr.y;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            v[i][0] = rstd * (v[i][0] - mean * c1w[i].x) + c2w[i].x;
            v[i][1] = rstd * (v[i][1] - mean * c1w[i].y) + c2w[i].y;
            v[i][2] = rstd * (v[i][2] - mean * c1w[i].z) + c2w[i].z;
            v[i][3] = rstd * (v[i][3] - mean * c1w[i].w) + c2w[i].w;
        }
    }
    if (MODE == MODE_STORE_LN) {
        int mrow[ITEMS], n0[ITEMS], rslot[ITEMS];
        bool live[ITEMS];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int item = wave + i * WAVES, tile = grp * NT + (item >> 2);
            mrow[i] = m;
            n0[i] = tile * 32 + 8 * (item & 3) + 4 * (lane >> 5);
            live[i] = item < NT * 4 && tile < n_tiles && m < p.M;
            rslot[i] = 0;
        }
        store_ln_tail<ITEMS, WAVES, 32>(p, ksplit, ks, grp, (n_tiles + NT - 1) / NT, mt,
                                        32.f * (float)min(NT, n_tiles - grp * NT), v, mrow, n0, live, rslot);
        return;
    }
    float (*zt)[32][33] = reinterpret_cast<float (*)[32][33]>(&red[0][0][0][0]);  // logits tiles reuse the LDS
    if (MODE == MODE_LMHEAD) __syncthreads();                                      // once every partial is read
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int item = wave + i * WAVES, t = item >> 2, tile = grp * NT + t;
        const int nl = 8 * (item & 3) + 4 * (lane >> 5);  // first of this lane's four rows inside the tile
        if (item >= NT * 4) continue;
        if (MODE != MODE_LMHEAD) {
            if (tile < n_tiles) epilogue4<MODE>(p, m, tile * 32 + nl, ks, v[i][0], v[i][1], v[i][2], v[i][3], bias_w[i], cur_len);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) zt[t][nl + r][lane & 31] = v[i][r];
        }
    }
    if (MODE == MODE_LMHEAD) {
        // logits tiles -> per-(row, tile) softmax and arg-max partials
        __syncthreads();
        for (int i0 = threadIdx.x; i0 < NT * 32; i0 += WAVES * 64) {
            const int t = i0 >> 5, mm = mt * 32 + (i0 & 31), tile = grp * NT + t;
            if (mm >= p.M || tile >= n_tiles) continue;
            const int mode = p.st->mode, step = p.st->step;
            const float temp = p.st->temperature;
            const uint32_t k0 = p.st->seed_lo, k1 = p.st->seed_hi;
            float mx = -INFINITY, best = -INFINITY, bestz = 0.f;
            int besti = 0x7FFFFFFF;
            const int nv = min(32, p.N - tile * 32);
            for (int i = 0; i < nv; ++i) {
                const float z = zt[t][i][i0 & 31];
                const int vid = tile * 32 + i;
                if (p.logits) p.logits[(size_t)mm * p.N + vid] = z;
                mx = fmaxf(mx, z);
                float s = z;
                if (mode == 1)
                    s = z / temp + gumbel_from_word(philox_word0((uint32_t)vid, (uint32_t)step, (uint32_t)mm, k0, k1));
                if (s > best) { best = s; besti = vid; bestz = z; }  // ascending ids: strict > keeps the lowest
            }
            float sum = 0.f;
            for (int i = 0; i < nv; ++i) sum += expf(zt[t][i][i0 & 31] - mx);
            float* sp = p.stats + ((size_t)mm * p.n_tiles + tile) * 4;
            sp[0] = mx; sp[1] = sum; sp[2] = best; sp[3] = bestz;
            p.stats_idx[(size_t)mm * p.n_tiles + tile] = besti;
        }
    }
}

// ----------------------------------------------------------------- skinny GEMM on 16-row units
//
// The kernel above hands out weight rows in units of 32, so a launch can only be balanced over
// the CUs when the number of 32-row tiles happens to divide well: 640 tiles (FC1 of the 13B
// shape) give 214 workgroups of three, and 42 CUs idle.  This variant hands out units of 16 rows
// -- 1280 of them are five per CU on all 256 -- using the 16x16x32 matrix instruction: its A
// operand is 16 rows x 32 k, i.e. one half (rows 0-15 or 16-31) of two consecutive 32x16 blocks,
// which a wavefront gathers from the unchanged tiled layout as four 256-byte runs (lane l: k-block
// l/32, k half (l/16)%2, row l%16).  The activations are gathered the same way, 16 of the 32 rows
// per instruction.  Lane l ends up with D[n = 16 g + 4 (l/16) + 0..3][m = 16 mh + l%16]: four
// consecutive outputs of one row, as the epilogues want them.  Everything else -- k split over the
// wavefronts, double-buffered loads, reduction through LDS, folded LayerNorm, last-arriving
// workgroup for the k-split modes -- is as above.

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma16_bf16(const u32x4& a, const u32x4& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
}

// 16 E4M3 codes -> two bf16 operand registers (exact: an E4M3 value has four significant bits).
// Bytes 0-7 are the lane's eight k values of the first 32-wide k range, bytes 8-15 those of the second.
__device__ __forceinline__ uint32_t e4m3x2_to_bf16x2(uint32_t word, bool upper) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 f = upper ? __builtin_amdgcn_cvt_pk_f32_fp8(word, true) : __builtin_amdgcn_cvt_pk_f32_fp8(word, false);
    return (__float_as_uint(f.x) >> 16) | (__float_as_uint(f.y) & 0xFFFF0000u);
}
__device__ __forceinline__ void e4m3x16_to_bf16(const u32x4& w, u32x4& a0, u32x4& a1) {
    a0 = u32x4{e4m3x2_to_bf16x2(w.x, false), e4m3x2_to_bf16x2(w.x, true), e4m3x2_to_bf16x2(w.y, false),
               e4m3x2_to_bf16x2(w.y, true)};
    a1 = u32x4{e4m3x2_to_bf16x2(w.z, false), e4m3x2_to_bf16x2(w.z, true), e4m3x2_to_bf16x2(w.w, false),
               e4m3x2_to_bf16x2(w.w, true)};
}

// One loop step of a wavefront covers KU = 1 (bf16 weights) or 2 (8-bit weights: one 16-byte load holds
// two) k ranges of 32, U steps per round of loads.
template <int HT, int U, bool W8>
struct HalfRegs {
    static constexpr int KU = W8 ? 2 : 1;
    u32x4 w[HT][U], xh[2][U * KU], xl[2][U * KU];
};

template <int HT, int U, bool W8>
__device__ __forceinline__ void half_load(HalfRegs<HT, U, W8>& r, const u32x4* (&w)[HT], const u32x4*& xh, const u32x4*& xl) {
    constexpr int KU = W8 ? 2 : 1, WSTEP = W8 ? 64 : 128;
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int t = 0; t < HT; ++t) r.w[t][u] = __builtin_nontemporal_load(w[t] + u * WSTEP);
#pragma unroll
        for (int kp = 0; kp < KU; ++kp)
#pragma unroll
            for (int mh = 0; mh < 2; ++mh) {
                r.xh[mh][u * KU + kp] = xh[(u * KU + kp) * 128 + mh * 16];
                r.xl[mh][u * KU + kp] = xl[(u * KU + kp) * 128 + mh * 16];
            }
    }
#pragma unroll
    for (int t = 0; t < HT; ++t) w[t] += U * WSTEP;
    xh += U * KU * 128;
    xl += U * KU * 128;
}

template <int HT, int U, bool W8>
__device__ __forceinline__ void half_mma(const HalfRegs<HT, U, W8>& r, f32x4 (&acc)[HT][2]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (W8) {
#pragma unroll
            for (int t = 0; t < HT; ++t) {
                u32x4 a[2];
                e4m3x16_to_bf16(r.w[t][u], a[0], a[1]);
#pragma unroll
                for (int kp = 0; kp < 2; ++kp)
#pragma unroll
                    for (int mh = 0; mh < 2; ++mh) {
                        acc[t][mh] = mfma16_bf16(a[kp], r.xh[mh][u * 2 + kp], acc[t][mh]);
                        acc[t][mh] = mfma16_bf16(a[kp], r.xl[mh][u * 2 + kp], acc[t][mh]);
                    }
            }
        } else {
#pragma unroll
            for (int t = 0; t < HT; ++t)
#pragma unroll
                for (int mh = 0; mh < 2; ++mh) acc[t][mh] = mfma16_bf16(r.w[t][u], r.xh[mh][u], acc[t][mh]);
#pragma unroll
            for (int t = 0; t < HT; ++t)
#pragma unroll
                for (int mh = 0; mh < 2; ++mh) acc[t][mh] = mfma16_bf16(r.w[t][u], r.xl[mh][u], acc[t][mh]);
        }
    }
}

// n_half = number of 16-row units of the weight matrix (N / 16); a workgroup owns HT of them.
// W8: the weights are E4M3 codes in units of [16 rows][64 k] -- lane l holds, for row l%16, the eight k
// values 8 (l/16) + 0..7 of the unit's first 32 k in bytes 0-7 and those of its second 32 k in bytes
// 8-15: one contiguous 1 KiB load per unit, two matrix-instruction operands after conversion.
template <int MODE, int HT, int U, int WAVES, bool W8>
__global__ __launch_bounds__(WAVES * 64) void gemm_half_kernel(const u32x4* __restrict__ Wp, const u32x4* __restrict__ Xhi,
                                                               const u32x4* __restrict__ Xlo, int KB, int n_half,
                                                               int ksplit, Epi p) {
    constexpr int NI = HT * 2;  // (unit, row half) items of a workgroup
    __shared__ float red[WAVES][NI][4][64];
    extern __shared__ float dyn_lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int grp = blockIdx.x / ksplit, ks = blockIdx.x % ksplit;
    const int mt = blockIdx.y;
    constexpr int KU = W8 ? 2 : 1;       // 32-wide k ranges per loop step
    const int KP = KB / (2 * KU);        // loop steps over the whole of k
    const int parts = ksplit * WAVES, part = ks * WAVES + wave;
    const int kp0 = (int)(((long)part * KP) / parts), kp1 = (int)(((long)(part + 1) * KP) / parts);
    constexpr bool FOLDABLE = MODE == MODE_BIAS_RELU || MODE == MODE_QKV;
    const bool fold = FOLDABLE && p.ln_stats != nullptr;
    if (fold) {
        const int chunks = (p.ln_groups * 32 * (int)sizeof(float2) + 1023) >> 10;
        const u32x4* src = reinterpret_cast<const u32x4*>(p.ln_stats + (size_t)mt * p.ln_groups * 32);
        for (int c = wave; c < chunks; c += WAVES)
            load_block_to_lds(src + c * 64 + lane, reinterpret_cast<u32x4*>(dyn_lds) + c * 64);
    }
    // this lane's 16 bytes inside a pair of 32x16 blocks: k-block lane/32, slot 32*(k half) + row
    const int in_pair = (lane >> 5) * 64 + 32 * ((lane >> 4) & 1) + (lane & 15);
    const u32x4* w[HT];
#pragma unroll
    for (int t = 0; t < HT; ++t) {  // units past the last one are computed from the last one, never stored
        const int g = min(grp * HT + t, n_half - 1);
        if (W8) w[t] = Wp + ((size_t)g * KP + kp0) * 64 + lane;
        else w[t] = Wp + ((size_t)(g >> 1) * KB + 2 * kp0) * 64 + in_pair + 16 * (g & 1);
    }
    const u32x4* xh = Xhi + ((size_t)mt * KB + 2 * KU * kp0) * 64 + in_pair;
    const u32x4* xl = Xlo + ((size_t)mt * KB + 2 * KU * kp0) * 64 + in_pair;
    constexpr int ITEMS = (NI + WAVES - 1) / WAVES;  // item = wave + i*WAVES -> unit item/2, row half item%2
    uint2 bias_w[ITEMS];
    float4 c1w[ITEMS], c2w[ITEMS], wsc[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int item = wave + i * WAVES, g = grp * HT + (item >> 1);
        const int n0 = g * 16 + 4 * (lane >> 4);
        const bool live = item < NI && g < n_half;
        bias_w[i] = live ? epilogue_bias<MODE>(p, n0) : make_uint2(0, 0);
        wsc[i] = make_float4(1.f, 1.f, 1.f, 1.f);
        if (W8 && live) wsc[i] = *reinterpret_cast<const float4*>(p.wscale + n0);
        c1w[i] = c2w[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (FOLDABLE && fold && live) {
            c1w[i] = *reinterpret_cast<const float4*>(p.c1 + n0);
            c2w[i] = *reinterpret_cast<const float4*>(p.c2 + n0);
        }
    }
    const int cur_len = epilogue_len<MODE>(p);
    f32x4 acc[HT][2];
#pragma unroll
    for (int t = 0; t < HT; ++t) acc[t][0] = acc[t][1] = f32x4{0.f, 0.f, 0.f, 0.f};
    int n = kp1 - kp0;
    if (n >= U) {
        HalfRegs<HT, U, W8> ra;
        half_load<HT, U, W8>(ra, w, xh, xl);
        n -= U;
        while (n >= U) {
            HalfRegs<HT, U, W8> rb;
            half_load<HT, U, W8>(rb, w, xh, xl);
            n -= U;
            half_mma<HT, U, W8>(ra, acc);
            ra = rb;
        }
        half_mma<HT, U, W8>(ra, acc);
    }
    for (; n > 0; --n) {
        HalfRegs<HT, 1, W8> r1;
        half_load<HT, 1, W8>(r1, w, xh, xl);
        half_mma<HT, 1, W8>(r1, acc);
    }
#pragma unroll
    for (int t = 0; t < HT; ++t)
#pragma unroll
        for (int mh = 0; mh < 2; ++mh)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[wave][t * 2 + mh][r][lane] = acc[t][mh][r];
    if (FOLDABLE) wait_vmcnt<0>();  // the statistics have landed in LDS
    __syncthreads();
    float v[ITEMS][4];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int item = wave + i * WAVES;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float sum = 0.f;
            if (item < NI) {
#pragma unroll
                for (int ww = 0; ww < WAVES; ww += 2) sum += red[ww][item][r][lane] + red[ww + 1][item][r][lane];
            }
            v[i][r] = sum;
        }
    }
    if (W8) {  // sums over codes -> sums over weights: exact, the scales are powers of two
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            v[i][0] *= wsc[i].x; v[i][1] *= wsc[i].y; v[i][2] *= wsc[i].z; v[i][3] *= wsc[i].w;
        }
    }
    if (fold) {  // W LN(x) = rstd * (W (gamma x) - mean * W gamma) + W beta; a lane's items sit in two rows
        float2 mr[2];
#pragma unroll
        for (int mh = 0; mh < 2; ++mh) mr[mh] = ln_row_from_groups(dyn_lds, 16 * mh + (lane & 15), p);
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int mh = (wave + i * WAVES) & 1;
            const float mean = mr[mh].x, rstd = mr[mh].y;
            v[i][0] = rstd * (v[i][0] - mean * c1w[i].x) + c2w[i].x;
            v[i][1] = rstd * (v[i][1] - mean * c1w[i].y) + c2w[i].y;
            v[i][2] = rstd * (v[i][2] - mean * c1w[i].z) + c2w[i].z;
            v[i][3] = rstd * (v[i][3] - mean * c1w[i].w) + c2w[i].w;
        }
    }
    if (MODE == MODE_STORE_LN) {
        int mrow[ITEMS], n0[ITEMS], rslot[ITEMS];
        bool live[ITEMS];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int item = wave + i * WAVES, g = grp * HT + (item >> 1);
            mrow[i] = mt * 32 + 16 * (item & 1) + (lane & 15);
            n0[i] = g * 16 + 4 * (lane >> 4);
            live[i] = item < NI && g < n_half && mrow[i] < p.M;
            rslot[i] = item & 1;
        }
        store_ln_tail<ITEMS, WAVES, 16>(p, ksplit, ks, grp, (n_half + HT - 1) / HT, mt,
                                        16.f * (float)min(HT, n_half - grp * HT), v, mrow, n0, live, rslot);
        return;
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int item = wave + i * WAVES, g = grp * HT + (item >> 1);
        if (item >= NI || g >= n_half) continue;
        epilogue4<MODE>(p, mt * 32 + 16 * (item & 1) + (lane & 15), g * 16 + 4 * (lane >> 4), ks, v[i][0], v[i][1], v[i][2],
                        v[i][3], bias_w[i], cur_len);
    }
}

// One block per sequence: combines the LM-head tile partials in tile order
// (deterministic), writes token id and its untempered log-probability.
__global__ void lm_reduce_kernel(const float* __restrict__ stats, const int* __restrict__ stats_idx, int n_tiles,
                                 const he_dev_state* __restrict__ st, int32_t* __restrict__ ids_out,
                                 float* __restrict__ lp_out, int out_stride, int out_at_step,
                                 int32_t* __restrict__ cur_ids) {
    __shared__ float smx[4], ssum[4], sbest[4], sz[4];
    __shared__ int sidx[4];
    const int b = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const float* sp = stats + (size_t)b * n_tiles * 4;
    const int* ip = stats_idx + (size_t)b * n_tiles;
    float mx = -INFINITY;
    for (int t = threadIdx.x; t < n_tiles; t += blockDim.x) mx = fmaxf(mx, sp[t * 4]);
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if (lane == 0) smx[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(smx[0], smx[1]), fmaxf(smx[2], smx[3]));
    float sum = 0.f, best = -INFINITY, bz = 0.f;
    int bi = 0x7FFFFFFF;
    for (int t = threadIdx.x; t < n_tiles; t += blockDim.x) {
        sum += sp[t * 4 + 1] * expf(sp[t * 4] - mx);
        const float s = sp[t * 4 + 2];
        const int i = ip[t];
        if (s > best || (s == best && i < bi)) { best = s; bi = i; bz = sp[t * 4 + 3]; }
    }
    for (int o = 32; o > 0; o >>= 1) {
        sum += __shfl_xor(sum, o);
        const float os = __shfl_xor(best, o), oz = __shfl_xor(bz, o);
        const int oi = __shfl_xor(bi, o);
        if (os > best || (os == best && oi < bi)) { best = os; bi = oi; bz = oz; }
    }
    if (lane == 0) { ssum[wave] = sum; sbest[wave] = best; sidx[wave] = bi; sz[wave] = bz; }
    __syncthreads();
    if (threadIdx.x == 0) {
        sum = (ssum[0] + ssum[1]) + (ssum[2] + ssum[3]);
        best = sbest[0]; bi = sidx[0]; bz = sz[0];
        for (int w = 1; w < 4; ++w)
            if (sbest[w] > best || (sbest[w] == best && sidx[w] < bi)) { best = sbest[w]; bi = sidx[w]; bz = sz[w]; }
        const size_t at = (size_t)b * out_stride + (out_at_step ? st->step : 0);
        ids_out[at] = bi;
        lp_out[at] = bz - (mx + logf(sum));
        if (cur_ids) cur_ids[b] = bi;
    }
}

// ----------------------------------------------------------------- tiled GEMM (prompt pass)
//
// 256 (n) x 128 (m) output tile per workgroup, four wavefronts in a 2x2 grid of
// 128x64 sub-tiles (4x2 MFMA tiles each: 8 LDS operand reads feed 16 MFMAs per
// k-block).  Operands arrive as 1 KiB blocks whose layout is the lane order, so
// they are moved global -> LDS directly (global_load_lds, 16 bytes per lane, no
// staging registers) into a ring of stages; loads run several stages (about 3000
// MFMA cycles) ahead of the arithmetic, which is what it takes to cover an L2 /
// infinity-cache round trip; one barrier per stage.
// Activations are the two-term form here as well (hi and lo blocks against the
// same weight registers), which keeps keys and values of the prompt within a
// rounding of the exact ones before they are stored as bf16.
//
// Two ring shapes.  PAIR = 0: four stages of two k-blocks (128 KiB), one workgroup per CU -- for launches
// with fewer tiles than CUs (few rows; the k-split GEMMs of a wide decode step).  PAIR = 1: five stages of
// one k-block (80 KiB) and at most 256 registers, so that TWO workgroups share a CU: while one of them
// sits at its barrier, waits for operands or writes its results, the other one's MFMAs keep the matrix
// cores busy (one workgroup per CU left them idle 40-50 % of the time, and a 256-row tile that moves a
// quarter less operand data per flop, but fits only once, still 39 %).

constexpr int TN = 256, TM = 128;
constexpr int TNB = TN / 32;   // 32-row operand blocks on the n side
constexpr int MW = 2;          // 32-row m blocks per wavefront
template <int PAIR> struct TiledShape {
    static constexpr int TMB = 2 * MW;                 // 32-row operand blocks on the m side
    static constexpr int TMR = TMB * 32;               // rows of the m tile
    static constexpr int KSTAGE = PAIR ? 1 : 2;        // k-blocks (16 values of k each) per stage
    static constexpr int NSTG = PAIR ? 5 : 4;          // ring depth
    static constexpr int STAGE_BLOCKS = (TNB + 2 * TMB) * KSTAGE;
};

template <int MODE, int PAIR>
__global__ __launch_bounds__(256, PAIR ? 2 : 1) void gemm_tiled_kernel(const u32x4* __restrict__ Wp, const u32x4* __restrict__ Xhi,
                                                         const u32x4* __restrict__ Xlo, int KB, int NT32, int MT32,
                                                         int tiles_n, int tiles_m, int ksplit, Epi p) {
    // ring[stage][block][lane]; blocks of a stage: W tile i, k-block j at 2i+j; X hi at 16+2i+j; X lo at 24+2i+j
    constexpr int TMB = TiledShape<PAIR>::TMB, TMR = TiledShape<PAIR>::TMR, NSTG = TiledShape<PAIR>::NSTG;
    constexpr int KSTAGE = TiledShape<PAIR>::KSTAGE;
    constexpr int STAGE_BLOCKS = TiledShape<PAIR>::STAGE_BLOCKS;
    __shared__ u32x4 ring[NSTG][STAGE_BLOCKS][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // XCD-aware order: consecutive workgroups land on different XCDs, so give each XCD a
    // contiguous run of tiles; within a run, tiles sharing an m panel are neighbours.  With few
    // rows (a decode step of a large batch) the tiles alone do not fill the chip: each is then cut
    // into ksplit k ranges (MODE_STORE only; the partial sums go to separate slots).
    const int nblk = tiles_n * tiles_m;
    const int nitem = nblk * ksplit;
    const int per_xcd = (nitem + 7) / 8;
    const int item = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (item >= nitem) return;
    // PAIR: k range after k range, so that the tiles an XCD works on at once still share their panels;
    // the few tiles of a wide decode step: all k ranges of a tile next to each other
    const int lin = PAIR ? item % nblk : item / ksplit, ks = PAIR ? item / nblk : item % ksplit;
    const int GROUP = 8;  // m-tiles per super-row: the tiles an XCD works on at once (8 x 4, or 8 x 8 when two share
                          // a CU) use the same few W and X panels
    const int gsize = GROUP * tiles_n;
    const int g = lin / gsize, first_m = g * GROUP;
    const int gm = min(GROUP, tiles_m - first_m);
    const int tm = first_m + (lin % gsize) % gm, tn = (lin % gsize) / gm;

    const int wn = wave & 1, wm = wave >> 1;  // this wavefront's 128 (n) x 32 MW (m) sub-tile
    const int cur_len = epilogue_len<MODE>(p);
    f32x16 acc[4][MW];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < MW; ++j) acc[i][j] = f32x16{};

    // this wavefront brings in W row-tiles 2w, 2w+1 and XW row-tiles of X hi and X lo per k-block
    constexpr int XW = TMB / 4;
    const u32x4* wsrc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) wsrc[i] = Wp + (size_t)min(tn * TNB + wave * 2 + i, NT32 - 1) * KB * 64 + lane;
    const u32x4 *hsrc[XW], *lsrc[XW];
#pragma unroll
    for (int x = 0; x < XW; ++x) {
        const int xrt = min(tm * TMB + wave * XW + x, MT32 - 1);
        hsrc[x] = Xhi + (size_t)xrt * KB * 64 + lane;
        lsrc[x] = Xlo + (size_t)xrt * KB * 64 + lane;
    }
    const int nst_all = KB / KSTAGE;  // KB is even (K % 32 == 0)
    const int st0 = (int)((long)ks * nst_all / ksplit);
    const int nstage = (int)((long)(ks + 1) * nst_all / ksplit) - st0;  // this workgroup's stages: st0 .. st0+nstage-1
    {
        const size_t skip = (size_t)st0 * KSTAGE * 64;
        wsrc[0] += skip; wsrc[1] += skip;
#pragma unroll
        for (int x = 0; x < XW; ++x) { hsrc[x] += skip; lsrc[x] += skip; }
    }
    auto issue = [&](int st) {
        u32x4 (*slot)[64] = ring[st % NSTG];
#pragma unroll
        for (int j = 0; j < KSTAGE; ++j) {
            const size_t off = ((size_t)st * KSTAGE + j) * 64;
            load_block_to_lds(wsrc[0] + off, &slot[(wave * 2 + 0) * KSTAGE + j][0]);
            load_block_to_lds(wsrc[1] + off, &slot[(wave * 2 + 1) * KSTAGE + j][0]);
#pragma unroll
            for (int x = 0; x < XW; ++x) {
                load_block_to_lds(hsrc[x] + off, &slot[(TNB + wave * XW + x) * KSTAGE + j][0]);
                load_block_to_lds(lsrc[x] + off, &slot[(TNB + TMB + wave * XW + x) * KSTAGE + j][0]);
            }
        }
    };
    constexpr int kLoadsPerStage = (2 + 2 * XW) * KSTAGE;  // per wavefront
    // operand registers of one k-block: 4 weight blocks, MW activation tiles x (hi, lo)
    struct Ops { u32x4 a[4], b[2][MW]; };
    auto read_ops = [&](Ops& o, int st, int j) {
        u32x4 (*slot)[64] = ring[st % NSTG];
#pragma unroll
        for (int i = 0; i < 4; ++i) o.a[i] = slot[(wn * 4 + i) * KSTAGE + j][lane];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < MW; ++i) o.b[t][i] = slot[(TNB + t * TMB + wm * MW + i) * KSTAGE + j][lane];
    };
    auto mma_ops = [&](const Ops& o) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int jj = 0; jj < MW; ++jj) acc[i][jj] = mfma_bf16(o.a[i], o.b[t][jj], acc[i][jj]);
            }
    };
    // Stage st is usable once this wavefront's own loads of it have landed (at most the loads of the
    // stages issued after it may still be outstanding) and every other wavefront says the same.
    auto stage_ready = [&](int st, int last_issued) {
        const int later = min(last_issued, nstage - 1) - st;  // 0 .. NSTG-2
        if (later >= 4) wait_vmcnt<4 * kLoadsPerStage>();
        else if (later == 3) wait_vmcnt<3 * kLoadsPerStage>();
        else if (later == 2) wait_vmcnt<2 * kLoadsPerStage>();
        else if (later == 1) wait_vmcnt<kLoadsPerStage>();
        else wait_vmcnt<0>();
        __syncthreads();
    };
#pragma unroll
    for (int st = 0; st < NSTG - 1; ++st)
        if (st < nstage) issue(st);
    // Two operand register sets, used in turn.  No set is ever copied into the other: a copy would
    // have to wait for the LDS reads it copies, in the middle of the MFMAs.  A stage's slot is
    // refilled behind the barrier that every wavefront passes only after its MFMAs of that stage.
    Ops opa, opb;
    if constexpr (KSTAGE == 2) {
        // first k-block of a stage from A while B loads, second from B while A loads from the next
        // stage; the barrier that opens stage s+1 sits before the last k-block of stage s
        stage_ready(0, NSTG - 2);
        read_ops(opa, 0, 0);
        for (int s = 0; s < nstage; ++s) {
            read_ops(opb, s, KSTAGE - 1);
            mma_ops(opa);
            if (s + 1 < nstage) {
                stage_ready(s + 1, s + NSTG - 2);
                if (s + NSTG - 1 < nstage) issue(s + NSTG - 1);
                read_ops(opa, s + 1, 0);
            }
            mma_ops(opb);
        }
    } else {
        // One k-block per stage, an even number of stages (the launcher sees to that): even stages
        // from A, odd ones from B.  In the steady state a stage is opened while the NSTG-3 stages
        // issued after it are still in flight, and the slot just finished with is refilled.
        constexpr int kAhead = (NSTG - 3) * kLoadsPerStage;
        int s = 0;
        if (nstage > NSTG) {  // then the prologue has issued NSTG-1 stages
            wait_vmcnt<(NSTG - 2) * kLoadsPerStage>();
            __syncthreads();
            read_ops(opa, 0, 0);
            for (; s + NSTG < nstage; s += 2) {
                wait_vmcnt<kAhead>();
                __syncthreads();
                issue(s + NSTG - 1);
                read_ops(opb, s + 1, 0);
                mma_ops(opa);
                wait_vmcnt<kAhead>();
                __syncthreads();
                issue(s + NSTG);
                read_ops(opa, s + 2, 0);
                mma_ops(opb);
            }
        }
        // the last stages: issue the one that may still be missing (into the slot of stage s-1, which
        // every wavefront has left once it is past the barrier), then one wait covers them all
        __syncthreads();
        if (s + NSTG - 1 < nstage) issue(s + NSTG - 1);
        wait_vmcnt<0>();
        __syncthreads();
        if (s == 0) read_ops(opa, 0, 0);
        for (; s < nstage; s += 2) {
            read_ops(opb, s + 1, 0);
            mma_ops(opa);
            if (s + 2 < nstage) read_ops(opa, s + 2, 0);
            mma_ops(opb);
        }
    }
    if (MODE == MODE_SCORE) {
        // The logits never leave the registers: per row, the soft-max partials of this wavefront's
        // 128 vocabulary entries and, if the row's next token is among them, its logit.
#pragma unroll
        for (int j = 0; j < MW; ++j) {
            const int m = tm * TMR + (wm * MW + j) * 32 + (lane & 31);
            int tgt = -1;
            if (m < p.M && m % p.S != p.S - 1) {
                tgt = p.ids[m + 1];
                tgt = tgt < 0 ? 0 : (tgt >= p.N ? p.N - 1 : tgt);  // clamped like the embedding's ids
            }
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int n = tn * TN + (wn * 4 + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    const float z = n < p.N ? acc[i][j][r] : -INFINITY;
                    acc[i][j][r] = z;
                    mx = fmaxf(mx, z);
                    if (n == tgt) p.sc_tgt[m] = z;
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            float sum = 0.f;
            if (mx > -INFINITY) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sum += expf(acc[i][j][r] - mx);
            }
            sum += __shfl_xor(sum, 32);
            if (lane < 32 && m < p.M) p.sc_stats[(size_t)m * p.sc_parts + tn * 2 + wn] = make_float2(mx, sum);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < MW; ++j) {
            const int m = tm * TMR + (wm * MW + j) * 32 + (lane & 31);
            const int nb = tn * TN + (wn * 4 + i) * 32 + 4 * (lane >> 5);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                epilogue4<MODE>(p, m, nb + 8 * q, ks, acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2],
                                acc[i][j][q * 4 + 3], epilogue_bias<MODE>(p, nb + 8 * q), cur_len);
        }
}

// One wavefront per scored row: log-sum-exp over the vocabulary slices in slice order, then
// out[b][t] = z[next token] - lse  (out is [B][S-1]; the last position of a sequence scores nothing).
__global__ __launch_bounds__(256) void score_reduce_kernel(const float2* __restrict__ stats, const float* __restrict__ tgt,
                                                           int parts, int M, int S, float* __restrict__ out) {
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (m >= M || m % S == S - 1) return;
    const float2* sp = stats + (size_t)m * parts;
    float mx = -INFINITY;
    for (int i = lane; i < parts; i += 64) mx = fmaxf(mx, sp[i].x);
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float sum = 0.f;
    for (int i = lane; i < parts; i += 64) {
        const float2 e = sp[i];
        if (e.x > -INFINITY) sum += e.y * expf(e.x - mx);
    }
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) out[(size_t)(m / S) * (S - 1) + m % S] = tgt[m] - (mx + logf(sum));
}


// ----------------------------------------------------------------- LayerNorm (+ residual update)
//
// Row `src = m*in_mul + in_add`: r += sum of k-split partials + bias (fixed order),
// written back when asked; a = LayerNorm(r) is emitted as tiled bf16 blocks.
__global__ __launch_bounds__(1024) void ln_blocks_kernel(float* __restrict__ r, const float* __restrict__ part,
                                                        int ksplit, size_t part_split,
                                                        const bf16_t* __restrict__ pbias,
                                                        const bf16_t* __restrict__ gamma,
                                                        const bf16_t* __restrict__ beta, u32x4* __restrict__ a,
                                                        u32x4* __restrict__ a_lo, int H, float eps, int in_mul,
                                                        int in_add, int writeback) {
    extern __shared__ __align__(16) float row[];
    __shared__ float red[16];
    const int m = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nwave = blockDim.x >> 6;
    const size_t src = (size_t)m * in_mul + in_add;
    float4* rr = reinterpret_cast<float4*>(r + src * H);
    float s = 0.f;
    for (int i = threadIdx.x; i < H / 4; i += blockDim.x) {
        float4 v = rr[i];
        if (part) {
            for (int k = 0; k < ksplit; ++k) {
                const float4 y = *reinterpret_cast<const float4*>(part + (size_t)k * part_split + src * H + 4 * i);
                v.x += y.x; v.y += y.y; v.z += y.z; v.w += y.w;
            }
            const uint2 bb = *reinterpret_cast<const uint2*>(pbias + 4 * i);
            v.x += __uint_as_float(bb.x << 16); v.y += __uint_as_float(bb.x & 0xFFFF0000u);
            v.z += __uint_as_float(bb.y << 16); v.w += __uint_as_float(bb.y & 0xFFFF0000u);
            if (writeback) rr[i] = v;
        }
        reinterpret_cast<float4*>(row)[i] = v;
        s += (v.x + v.y) + (v.z + v.w);
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    float tot = 0.f;
    for (int i = 0; i < nwave; ++i) tot += red[i];
    const float mean = tot / H;
    float q = 0.f;
    for (int i = threadIdx.x; i < H; i += blockDim.x) { const float dlt = row[i] - mean; q += dlt * dlt; }
    for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o);
    __syncthreads();
    if (lane == 0) red[wave] = q;
    __syncthreads();
    tot = 0.f;
    for (int i = 0; i < nwave; ++i) tot += red[i];
    const float rstd = 1.0f / sqrtf(tot / H + eps);
    const int KB = H >> 4;
    for (int c = threadIdx.x; c < H / 8; c += blockDim.x) {
        const int k0 = c * 8;
        const u32x4 gg = *reinterpret_cast<const u32x4*>(gamma + k0), bb = *reinterpret_cast<const u32x4*>(beta + k0);
        const uint32_t gw[4] = {gg.x, gg.y, gg.z, gg.w}, bw[4] = {bb.x, bb.y, bb.z, bb.w};
        uint32_t o[4], ol[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float e0 = (row[k0 + 2 * j] - mean) * rstd * __uint_as_float(gw[j] << 16) + __uint_as_float(bw[j] << 16);
            const float e1 = (row[k0 + 2 * j + 1] - mean) * rstd * __uint_as_float(gw[j] & 0xFFFF0000u) +
                             __uint_as_float(bw[j] & 0xFFFF0000u);
            split2(e0, e1, o[j], ol[j]);
        }
        const size_t slot = block_slot(m, k0, KB);
        a[slot] = u32x4{o[0], o[1], o[2], o[3]};
        if (a_lo) a_lo[slot] = u32x4{ol[0], ol[1], ol[2], ol[3]};
    }
}

// The same operation with every value of the row held in registers (NV float4 per thread) and all
// loads -- residual, k-split partials, bias, gamma, beta -- issued before the first reduction.
// For the few rows of a decode step one 1024-thread workgroup per row (the kernel's time is then the
// length of its dependent-load chain); for the many rows of a prompt pass 256 threads per row.
template <int NV, int THREADS>
__global__ __launch_bounds__(THREADS) void ln_row_kernel(float* __restrict__ r, const float* __restrict__ part, int ksplit,
                                                      size_t part_split, const bf16_t* __restrict__ pbias,
                                                      const bf16_t* __restrict__ gamma,
                                                      const bf16_t* __restrict__ beta, u32x4* __restrict__ a,
                                                      u32x4* __restrict__ a_lo, int H, float eps, int in_mul,
                                                      int in_add, int writeback) {
    constexpr int NW = THREADS / 64;
    __shared__ float red[2][NW];
    const int m = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t src = (size_t)m * in_mul + in_add;
    const int nq = H >> 2;  // float4 per row
    float4 v[NV];
    uint2 gg[NV], bb[NV];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int i = threadIdx.x + j * THREADS;
        v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        gg[j] = bb[j] = make_uint2(0, 0);
        if (i < nq) {
            v[j] = *reinterpret_cast<const float4*>(r + src * H + 4 * i);
            gg[j] = *reinterpret_cast<const uint2*>(gamma + 4 * i);
            bb[j] = *reinterpret_cast<const uint2*>(beta + 4 * i);
        }
    }
    if (part) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = threadIdx.x + j * THREADS;
            if (i >= nq) continue;
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int k = 0; k < ksplit; ++k) {  // fixed order: the sum does not depend on scheduling
                const float4 y = *reinterpret_cast<const float4*>(part + (size_t)k * part_split + src * H + 4 * i);
                acc.x += y.x; acc.y += y.y; acc.z += y.z; acc.w += y.w;
            }
            const uint2 pb = *reinterpret_cast<const uint2*>(pbias + 4 * i);
            v[j].x += acc.x + __uint_as_float(pb.x << 16);
            v[j].y += acc.y + __uint_as_float(pb.x & 0xFFFF0000u);
            v[j].z += acc.z + __uint_as_float(pb.y << 16);
            v[j].w += acc.w + __uint_as_float(pb.y & 0xFFFF0000u);
            if (writeback) *reinterpret_cast<float4*>(r + src * H + 4 * i) = v[j];
        }
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) s += (v[j].x + v[j].y) + (v[j].z + v[j].w);  // lanes past the row hold zeros
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) red[0][wave] = s;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) tot += red[0][i];
    const float mean = tot / H;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        if (threadIdx.x + j * THREADS < nq) {
            const float d0 = v[j].x - mean, d1 = v[j].y - mean, d2 = v[j].z - mean, d3 = v[j].w - mean;
            q += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
        }
    }
    for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o);
    if (lane == 0) red[1][wave] = q;
    __syncthreads();
    tot = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) tot += red[1][i];
    const float rstd = 1.0f / sqrtf(tot / H + eps);
    const int KB = H >> 4;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int i = threadIdx.x + j * THREADS;
        if (i >= nq) continue;
        const float e0 = (v[j].x - mean) * rstd * __uint_as_float(gg[j].x << 16) + __uint_as_float(bb[j].x << 16);
        const float e1 = (v[j].y - mean) * rstd * __uint_as_float(gg[j].x & 0xFFFF0000u) + __uint_as_float(bb[j].x & 0xFFFF0000u);
        const float e2 = (v[j].z - mean) * rstd * __uint_as_float(gg[j].y << 16) + __uint_as_float(bb[j].y << 16);
        const float e3 = (v[j].w - mean) * rstd * __uint_as_float(gg[j].y & 0xFFFF0000u) + __uint_as_float(bb[j].y & 0xFFFF0000u);
        uint32_t h0, h1, l0, l1;
        split2(e0, e1, h0, l0);
        split2(e2, e3, h1, l1);
        const int k0 = 4 * i;  // four values: half of a 16-byte slot
        const size_t slot = block_slot(m, k0 & ~7, KB);
        reinterpret_cast<uint2*>(a + slot)[(k0 >> 2) & 1] = make_uint2(h0, h1);
        if (a_lo) reinterpret_cast<uint2*>(a_lo + slot)[(k0 >> 2) & 1] = make_uint2(l0, l1);
    }
}

// ----------------------------------------------------------------- LayerNorm folded into the next GEMM (decode rows)
//
// For the few rows of a decode step a LayerNorm kernel of its own is all latency.  Instead
//   W LN(x) + b = rstd * (W (gamma . x) - mean * (W gamma)) + W beta + b,
// so the kernel that produces x (the embedding below, or the out-projection / FC2 GEMM
// through its last-arriving workgroup) writes gamma . x as two-term blocks plus per-column-
// group statistics of x, the consuming GEMM multiplies those blocks by the unchanged bf16
// weights and applies mean and rstd in its epilogue, and W gamma, W beta are vectors computed
// once per weight update.

// Row m of a decode step: x = tok_emb[id] + pos_emb[cur_len + pos_offset]; one wavefront per
// (column group, row), four columns per lane (gw <= 256).
__global__ __launch_bounds__(64) void embed_ln_kernel(const int32_t* __restrict__ ids, int id_stride,
                                                      const bf16_t* __restrict__ tok, const bf16_t* __restrict__ pos,
                                                      const he_dev_state* __restrict__ st, int V, int pos_offset,
                                                      int H, int gw, int groups, const bf16_t* __restrict__ gamma,
                                                      float* __restrict__ r, u32x4* __restrict__ xb,
                                                      u32x4* __restrict__ xb_lo, float2* __restrict__ stats) {
    const int g = blockIdx.x, m = blockIdx.y, lane = threadIdx.x;
    int id = ids[(size_t)m * id_stride];
    id = id < 0 ? 0 : (id >= V ? V - 1 : id);
    const size_t prow = (size_t)(seq_len(st, m) + pos_offset);  // one row per sequence here
    const int cols = min(gw, H - g * gw), c0 = g * gw + 4 * lane;
    const bool live = 4 * lane < cols;
    float x0 = 0.f, x1 = 0.f, x2 = 0.f, x3 = 0.f;
    if (live) {
        const uint2 t = *reinterpret_cast<const uint2*>(tok + (size_t)id * H + c0);
        const uint2 q = *reinterpret_cast<const uint2*>(pos + prow * H + c0);
        const uint2 gg = *reinterpret_cast<const uint2*>(gamma + c0);
        x0 = __uint_as_float(t.x << 16) + __uint_as_float(q.x << 16);
        x1 = __uint_as_float(t.x & 0xFFFF0000u) + __uint_as_float(q.x & 0xFFFF0000u);
        x2 = __uint_as_float(t.y << 16) + __uint_as_float(q.y << 16);
        x3 = __uint_as_float(t.y & 0xFFFF0000u) + __uint_as_float(q.y & 0xFFFF0000u);
        *reinterpret_cast<float4*>(r + (size_t)m * H + c0) = make_float4(x0, x1, x2, x3);
        uint32_t h0, h1, l0, l1;
        split2(x0 * __uint_as_float(gg.x << 16), x1 * __uint_as_float(gg.x & 0xFFFF0000u), h0, l0);
        split2(x2 * __uint_as_float(gg.y << 16), x3 * __uint_as_float(gg.y & 0xFFFF0000u), h1, l1);
        const size_t slot = block_slot(m, c0 & ~7, H >> 4);
        reinterpret_cast<uint2*>(xb + slot)[(c0 >> 2) & 1] = make_uint2(h0, h1);
        reinterpret_cast<uint2*>(xb_lo + slot)[(c0 >> 2) & 1] = make_uint2(l0, l1);
    }
    float s = (x0 + x1) + (x2 + x3);
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    const float mean = s / (float)cols;
    float q2 = 0.f;
    if (live) {
        const float d0 = x0 - mean, d1 = x1 - mean, d2 = x2 - mean, d3 = x3 - mean;
        q2 = (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
    }
    for (int o = 32; o > 0; o >>= 1) q2 += __shfl_xor(q2, o);
    if (lane == 0) stats[((size_t)(m >> 5) * groups + g) * 32 + (m & 31)] = make_float2(mean, q2);
}

// c1[n] = sum_k W[n][k] gamma[k], c2[n] = sum_k W[n][k] beta[k] from the tiled weights: one
// wavefront per 32-row tile (lane = row and k half), float accumulation in k order.
__global__ __launch_bounds__(256) void wvec_kernel(const u32x4* __restrict__ Wp, int KB, int n_tiles,
                                                   const bf16_t* __restrict__ gamma, const bf16_t* __restrict__ beta,
                                                   float* __restrict__ c1, float* __restrict__ c2) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int tile = blockIdx.x * 4 + wave;
    if (tile >= n_tiles) return;
    const u32x4* w = Wp + (size_t)tile * KB * 64 + lane;
    float a1 = 0.f, a2 = 0.f;
    for (int kb = 0; kb < KB; ++kb) {
        const u32x4 wv = w[(size_t)kb * 64];
        const int k0 = kb * 16 + (lane >> 5) * 8;
        const u32x4 gv = *reinterpret_cast<const u32x4*>(gamma + k0), bv = *reinterpret_cast<const u32x4*>(beta + k0);
        const uint32_t ww[4] = {wv.x, wv.y, wv.z, wv.w}, gg[4] = {gv.x, gv.y, gv.z, gv.w}, bb[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float w0 = __uint_as_float(ww[j] << 16), w1 = __uint_as_float(ww[j] & 0xFFFF0000u);
            a1 = fmaf(w0, __uint_as_float(gg[j] << 16), a1);
            a1 = fmaf(w1, __uint_as_float(gg[j] & 0xFFFF0000u), a1);
            a2 = fmaf(w0, __uint_as_float(bb[j] << 16), a2);
            a2 = fmaf(w1, __uint_as_float(bb[j] & 0xFFFF0000u), a2);
        }
    }
    a1 += __shfl_xor(a1, 32);
    a2 += __shfl_xor(a2, 32);
    if (lane < 32) {  // rows past the matrix are zero blocks: their entries come out zero
        c1[tile * 32 + lane] = a1;
        c2[tile * 32 + lane] = a2;
    }
}

// ----------------------------------------------------------------- attention over the KV cache
//
// One workgroup per (row m, head h); the query at position cur_len + (m % S)
// sees keys 0..that position.  D/8 adjacent lanes own one key (16 bytes each, a
// whole row of K or V per group, coalesced); scores are reduced with wavefront
// shuffles, kept in LDS, soft-maxed, then the same lanes accumulate p_j * V[j].
// The output goes out as tiled bf16 blocks for the out-projection GEMM.
template <int D>
__global__ __launch_bounds__(256) void attn_kernel(const float* __restrict__ q, const bf16_t* __restrict__ kv,
                                                   u32x4* __restrict__ o, u32x4* __restrict__ o_lo,
                                                   const he_dev_state* __restrict__ st, int S, int layer, int H,
                                                   int n_heads, int max_batch, int max_seq) {
    constexpr int LPK = D / 8;     // lanes per key
    constexpr int KPW = 64 / LPK;  // keys per wavefront load
    constexpr int KR = 4 * KPW;    // keys per workgroup round
    constexpr int U = 4;
    extern __shared__ float sc[];  // [max_seq] scores, then probabilities
    __shared__ float red[8];
    __shared__ float ored[4][LPK * 8];
    const int m = blockIdx.x, h = blockIdx.y;
    const int b = m / S, T = seq_len(st, b) + (m % S) - row_pad(st, b) + 1;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sub = lane % LPK, grp = lane / LPK;
    if (seq_done(st, b)) return;  // the sequence has ended: its row's output is not used any more
    if (T <= 0) {                 // a padding row: nothing to attend to, nothing reads the output; keep it finite
        if (wave == 0 && grp == 0) {
            const size_t slot = block_slot(m, h * D + sub * 8, H >> 4);
            o[slot] = u32x4{0u, 0u, 0u, 0u};
            if (o_lo) o_lo[slot] = u32x4{0u, 0u, 0u, 0u};
        }
        return;
    }
    const float4 qa = *reinterpret_cast<const float4*>(q + (size_t)m * H + h * D + sub * 8);
    const float4 qb = *reinterpret_cast<const float4*>(q + (size_t)m * H + h * D + sub * 8 + 4);
    const u32x4* Kp = reinterpret_cast<const u32x4*>(kv + kv_index(layer, 0, b, h, 0, max_batch, n_heads, max_seq, D));
    const u32x4* Vp = reinterpret_cast<const u32x4*>(kv + kv_index(layer, 1, b, h, 0, max_batch, n_heads, max_seq, D));
    const int jw = wave * KPW + grp;
    constexpr int STEP = KR * U;  // keys per workgroup iteration
    auto load_rows = [&](u32x4 (&dst)[U], const u32x4* src, int base) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = base + u * KR + jw;
            dst[u] = j < T ? __builtin_nontemporal_load(src + (size_t)j * LPK + sub) : u32x4{0u, 0u, 0u, 0u};
        }
    };
    // loads run one iteration ahead of the arithmetic, and the first values are requested
    // before the soft-max barrier, so the memory pipe never drains between the phases
    float mx = -INFINITY;
    u32x4 cur[U], nxt[U];
    load_rows(cur, Kp, 0);
    for (int base = 0; base < T; base += STEP) {
        if (base + STEP < T) load_rows(nxt, Kp, base + STEP);
        else load_rows(nxt, Vp, 0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = base + u * KR + jw;
            float s = qa.x * __uint_as_float(cur[u].x << 16);
            s = fmaf(qa.y, __uint_as_float(cur[u].x & 0xFFFF0000u), s);
            s = fmaf(qa.z, __uint_as_float(cur[u].y << 16), s);
            s = fmaf(qa.w, __uint_as_float(cur[u].y & 0xFFFF0000u), s);
            s = fmaf(qb.x, __uint_as_float(cur[u].z << 16), s);
            s = fmaf(qb.y, __uint_as_float(cur[u].z & 0xFFFF0000u), s);
            s = fmaf(qb.z, __uint_as_float(cur[u].w << 16), s);
            s = fmaf(qb.w, __uint_as_float(cur[u].w & 0xFFFF0000u), s);
#pragma unroll
            for (int o2 = 1; o2 < LPK; o2 <<= 1) s += __shfl_xor(s, o2);
            if (j < T) {
                if (sub == 0) sc[j] = s;
                mx = fmaxf(mx, s);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) cur[u] = nxt[u];
    }
    // cur now holds the first values
    for (int o2 = 32; o2 > 0; o2 >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o2));
    if (lane == 0) red[wave] = mx;
    __syncthreads();  // also publishes sc[]
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float sum = 0.f;
    for (int j = threadIdx.x; j < T; j += 256) {
        const float pj = expf(sc[j] - mx);
        sc[j] = pj;
        sum += pj;
    }
    for (int o2 = 32; o2 > 0; o2 >>= 1) sum += __shfl_xor(sum, o2);
    if (lane == 0) red[4 + wave] = sum;
    __syncthreads();  // also publishes the probabilities
    sum = (red[4] + red[5]) + (red[6] + red[7]);
    float acc[8] = {};
    for (int base = 0; base < T; base += STEP) {
        if (base + STEP < T) load_rows(nxt, Vp, base + STEP);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = base + u * KR + jw;
            const float pj = j < T ? sc[j] : 0.f;
            acc[0] = fmaf(pj, __uint_as_float(cur[u].x << 16), acc[0]);
            acc[1] = fmaf(pj, __uint_as_float(cur[u].x & 0xFFFF0000u), acc[1]);
            acc[2] = fmaf(pj, __uint_as_float(cur[u].y << 16), acc[2]);
            acc[3] = fmaf(pj, __uint_as_float(cur[u].y & 0xFFFF0000u), acc[3]);
            acc[4] = fmaf(pj, __uint_as_float(cur[u].z << 16), acc[4]);
            acc[5] = fmaf(pj, __uint_as_float(cur[u].z & 0xFFFF0000u), acc[5]);
            acc[6] = fmaf(pj, __uint_as_float(cur[u].w << 16), acc[6]);
            acc[7] = fmaf(pj, __uint_as_float(cur[u].w & 0xFFFF0000u), acc[7]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) cur[u] = nxt[u];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
        for (int o2 = LPK; o2 < 64; o2 <<= 1) acc[e] += __shfl_xor(acc[e], o2);
    }
    if (grp == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) ored[wave][sub * 8 + e] = acc[e];
    }
    __syncthreads();
    if (threadIdx.x < LPK) {
        float ov[8];
        const float inv = 1.0f / sum;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int i = threadIdx.x * 8 + e;
            ov[e] = ((ored[0][i] + ored[1][i]) + (ored[2][i] + ored[3][i])) * inv;
        }
        uint32_t oh[4], ol[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) split2(ov[2 * e], ov[2 * e + 1], oh[e], ol[e]);
        const size_t slot = block_slot(m, h * D + threadIdx.x * 8, H >> 4);
        o[slot] = u32x4{oh[0], oh[1], oh[2], oh[3]};
        if (o_lo) o_lo[slot] = u32x4{ol[0], ol[1], ol[2], ol[3]};
    }
}

// ----------------------------------------------------------------- attention, prompt rows
//
// Same arithmetic as attn_kernel for a block of QB consecutive queries of one (sequence, head):
// every K and V row fetched once serves all QB queries, which cuts the L2 traffic of the prompt
// pass by QB.  The QB partial dot products of a key are reduced over the D/8 lanes that share
// the key with a halving butterfly (each step sends half of the values and keeps the other
// half), so the lanes end up owning different queries.  Query t0+i sees keys <= cur_len + t0 + i.
constexpr int QB = 8;

template <int D>
__global__ __launch_bounds__(256) void attn_prompt_kernel(const float* __restrict__ q, const bf16_t* __restrict__ kv,
                                                          u32x4* __restrict__ o, u32x4* __restrict__ o_lo,
                                                          const he_dev_state* __restrict__ st, int S, int layer, int H,
                                                          int n_heads, int max_batch, int max_seq) {
    constexpr int LPK = D / 8, KPW = 64 / LPK, KR = 4 * KPW, U = 2, STEP = KR * U;
    extern __shared__ float sc[];  // [QB][max_seq] scores, then probabilities
    __shared__ float ored[4][QB][D];
    __shared__ float inv_sum[QB];
    const int t0 = blockIdx.x * QB, h = blockIdx.y, b = blockIdx.z;
    const int nq = min(QB, S - t0);
    const int cur = seq_len(st, b) - row_pad(st, b);  // cache position of row 0: negative while rows are padding
    const int T = cur + t0 + nq;  // keys any query of the block may see
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sub = lane % LPK, grp = lane / LPK;
    float qv[QB][8];
#pragma unroll
    for (int i = 0; i < QB; ++i) {
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f), c = a;
        if (i < nq) {
            const float* qp = q + (size_t)(b * S + t0 + i) * H + h * D + sub * 8;
            a = *reinterpret_cast<const float4*>(qp);
            c = *reinterpret_cast<const float4*>(qp + 4);
        }
        qv[i][0] = a.x; qv[i][1] = a.y; qv[i][2] = a.z; qv[i][3] = a.w;
        qv[i][4] = c.x; qv[i][5] = c.y; qv[i][6] = c.z; qv[i][7] = c.w;
    }
    const u32x4* Kp = reinterpret_cast<const u32x4*>(kv + kv_index(layer, 0, b, h, 0, max_batch, n_heads, max_seq, D));
    const u32x4* Vp = reinterpret_cast<const u32x4*>(kv + kv_index(layer, 1, b, h, 0, max_batch, n_heads, max_seq, D));
    const int jw = wave * KPW + grp;
    auto load_rows = [&](u32x4 (&dst)[U], const u32x4* src, int base) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = base + u * KR + jw;
            dst[u] = j < T ? src[(size_t)j * LPK + sub] : u32x4{0u, 0u, 0u, 0u};
        }
    };
    // which query this lane owns after the butterfly
    int qown = 0;
    {
        int nval = QB;
#pragma unroll
        for (int off = LPK / 2; off >= 1; off >>= 1)
            if (nval > 1) { nval >>= 1; if (sub & off) qown += nval; }
    }
    constexpr bool kPairs = LPK > QB;  // two lanes end up with the same query: the even one stores
    u32x4 cur_r[U], nxt_r[U];
    load_rows(cur_r, Kp, 0);
    for (int base = 0; base < T; base += STEP) {
        if (base + STEP < T) load_rows(nxt_r, Kp, base + STEP);
        else load_rows(nxt_r, Vp, 0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = base + u * KR + jw;
            const float k0 = __uint_as_float(cur_r[u].x << 16), k1 = __uint_as_float(cur_r[u].x & 0xFFFF0000u);
            const float k2 = __uint_as_float(cur_r[u].y << 16), k3 = __uint_as_float(cur_r[u].y & 0xFFFF0000u);
            const float k4 = __uint_as_float(cur_r[u].z << 16), k5 = __uint_as_float(cur_r[u].z & 0xFFFF0000u);
            const float k6 = __uint_as_float(cur_r[u].w << 16), k7 = __uint_as_float(cur_r[u].w & 0xFFFF0000u);
            float part[QB];
#pragma unroll
            for (int i = 0; i < QB; ++i) {
                float s = qv[i][0] * k0;
                s = fmaf(qv[i][1], k1, s); s = fmaf(qv[i][2], k2, s); s = fmaf(qv[i][3], k3, s);
                s = fmaf(qv[i][4], k4, s); s = fmaf(qv[i][5], k5, s); s = fmaf(qv[i][6], k6, s);
                part[i] = fmaf(qv[i][7], k7, s);
            }
            int nval = QB;
#pragma unroll
            for (int off = LPK / 2; off >= 1; off >>= 1) {
                if (nval > 1) {
                    nval >>= 1;
                    const bool upper = (sub & off) != 0;
#pragma unroll
                    for (int c = 0; c < QB / 2; ++c) {
                        if (c < nval) {
                            const float send = upper ? part[c] : part[c + nval];
                            const float keep = upper ? part[c + nval] : part[c];
                            part[c] = keep + __shfl_xor(send, off);
                        }
                    }
                } else {
                    part[0] += __shfl_xor(part[0], off);
                }
            }
            if (j < T && (!kPairs || (sub & 1) == 0))
                sc[qown * max_seq + j] = j <= max(cur + t0 + qown, 0) ? part[0] : -INFINITY;  // a padding row looks at key 0
        }
#pragma unroll
        for (int u = 0; u < U; ++u) cur_r[u] = nxt_r[u];
    }
    __syncthreads();
    {   // soft-max of query 2*wave + (lane / 32) over its 32 lanes
        const int qi = 2 * wave + (lane >> 5), l32 = lane & 31;
        float* row = sc + qi * max_seq;
        float mx = -INFINITY;
        for (int j = l32; j < T; j += 32) mx = fmaxf(mx, row[j]);
        for (int o2 = 16; o2 > 0; o2 >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o2));
        float sum = 0.f;
        for (int j = l32; j < T; j += 32) {
            const float pj = expf(row[j] - mx);
            row[j] = pj;
            sum += pj;
        }
        for (int o2 = 16; o2 > 0; o2 >>= 1) sum += __shfl_xor(sum, o2);
        if (l32 == 0) inv_sum[qi] = sum > 0.f ? 1.0f / sum : 0.f;  // no keys at all: a block of padding rows
    }
    __syncthreads();
    float acc[QB][8] = {};
    for (int base = 0; base < T; base += STEP) {
        if (base + STEP < T) load_rows(nxt_r, Vp, base + STEP);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = base + u * KR + jw;
            if (j < T) {
                const float v0 = __uint_as_float(cur_r[u].x << 16), v1 = __uint_as_float(cur_r[u].x & 0xFFFF0000u);
                const float v2 = __uint_as_float(cur_r[u].y << 16), v3 = __uint_as_float(cur_r[u].y & 0xFFFF0000u);
                const float v4 = __uint_as_float(cur_r[u].z << 16), v5 = __uint_as_float(cur_r[u].z & 0xFFFF0000u);
                const float v6 = __uint_as_float(cur_r[u].w << 16), v7 = __uint_as_float(cur_r[u].w & 0xFFFF0000u);
#pragma unroll
                for (int i = 0; i < QB; ++i) {
                    const float pj = sc[i * max_seq + j];
                    acc[i][0] = fmaf(pj, v0, acc[i][0]); acc[i][1] = fmaf(pj, v1, acc[i][1]);
                    acc[i][2] = fmaf(pj, v2, acc[i][2]); acc[i][3] = fmaf(pj, v3, acc[i][3]);
                    acc[i][4] = fmaf(pj, v4, acc[i][4]); acc[i][5] = fmaf(pj, v5, acc[i][5]);
                    acc[i][6] = fmaf(pj, v6, acc[i][6]); acc[i][7] = fmaf(pj, v7, acc[i][7]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) cur_r[u] = nxt_r[u];
    }
#pragma unroll
    for (int i = 0; i < QB; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
#pragma unroll
            for (int o2 = LPK; o2 < 64; o2 <<= 1) acc[i][e] += __shfl_xor(acc[i][e], o2);
        }
    if (grp == 0) {
#pragma unroll
        for (int i = 0; i < QB; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) ored[wave][i][sub * 8 + e] = acc[i][e];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < QB * LPK; idx += 256) {
        const int i = idx / LPK, c = idx % LPK;
        if (i >= nq) continue;
        float ov[8];
        const float inv = inv_sum[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int d0 = c * 8 + e;
            ov[e] = ((ored[0][i][d0] + ored[1][i][d0]) + (ored[2][i][d0] + ored[3][i][d0])) * inv;
        }
        uint32_t oh[4], ol[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) split2(ov[2 * e], ov[2 * e + 1], oh[e], ol[e]);
        const size_t slot = block_slot(b * S + t0 + i, h * D + c * 8, H >> 4);
        o[slot] = u32x4{oh[0], oh[1], oh[2], oh[3]};
        if (o_lo) o_lo[slot] = u32x4{ol[0], ol[1], ol[2], ol[3]};
    }
}

// ----------------------------------------------------------------- attention, prompt rows, on the matrix cores
//
// Flash-style causal attention for the prompt pass.  One wavefront owns 32 queries of one
// (sequence, head); the four wavefronts of a workgroup share each 32-key tile of K and V through
// LDS.  Everything is computed transposed so that a lane owns ONE query: S^T = K Q^T puts the
// scores of query lane%32 in that lane's 16 accumulators (online soft-max needs one exchange
// with lane^32), and O^T = V^T P^T accumulates that query's output column, so the soft-max
// rescaling is a per-lane scalar.  Q and P enter the MFMA as two bf16 terms (hi + lo).  The
// keys of a PV step are taken in the order the score accumulators already hold them; V is
// transposed into that order while it is staged in LDS.
template <int D>
__global__ __launch_bounds__(256) void attn_prompt_mfma_kernel(const float* __restrict__ q,
                                                               const bf16_t* __restrict__ kv, u32x4* __restrict__ o,
                                                               u32x4* __restrict__ o_lo,
                                                               const he_dev_state* __restrict__ st, int S, int layer,
                                                               int H, int n_heads, int max_batch, int max_seq) {
    constexpr int KBD = D / 16;      // k-blocks over the head dimension
    constexpr int DB = D / 32;       // 32-wide blocks of output dimensions
    constexpr int KPITCH = D + 8;    // bf16 per K row in LDS (16 bytes of padding)
    __shared__ __align__(16) bf16_t ks[32 * KPITCH];
    __shared__ __align__(16) bf16_t vt[DB * 2 * 2 * 32 * 8];  // [dim block][k-step][lane half][dim][8 keys]
    const int h = blockIdx.y, b = blockIdx.z;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int j = lane & 31, hh = lane >> 5;
    const int cur = seq_len(st, b) - row_pad(st, b);  // cache position of row 0: negative while rows are padding
    const int T = cur + S;                          // keys in the cache once this pass is stored
    const int t0 = (blockIdx.x * 4 + wave) * 32;    // this wavefront's first query
    const bool live = t0 < S;
    const int qpos = max(cur + t0 + j, 0);          // last key this lane's query may see (a padding row looks at key 0)
    const int wg_last = min(T - 1, cur + min(S, (int)(blockIdx.x * 4 + 4) * 32) - 1);
    const int n_tiles = wg_last / 32 + 1;
    const int my_last_tile = live ? min(T - 1, cur + t0 + 31) / 32 : -1;

    u32x4 qhi[KBD], qlo[KBD];
    {
        const bool ok = t0 + j < S;
        const float* qp = q + (size_t)(b * S + (ok ? t0 + j : 0)) * H + h * D + hh * 8;
#pragma unroll
        for (int kb = 0; kb < KBD; ++kb) {
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), c = a;
            if (ok) {
                a = *reinterpret_cast<const float4*>(qp + kb * 16);
                c = *reinterpret_cast<const float4*>(qp + kb * 16 + 4);
            }
            uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
            split2(a.x, a.y, h0, l0); split2(a.z, a.w, h1, l1); split2(c.x, c.y, h2, l2); split2(c.z, c.w, h3, l3);
            qhi[kb] = u32x4{h0, h1, h2, h3};
            qlo[kb] = u32x4{l0, l1, l2, l3};
        }
    }
    const bf16_t* Kg = kv + kv_index(layer, 0, b, h, 0, max_batch, n_heads, max_seq, D);
    const bf16_t* Vg = kv + kv_index(layer, 1, b, h, 0, max_batch, n_heads, max_seq, D);
    f32x16 oacc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i) oacc[i] = f32x16{};
    float m_run = -INFINITY, l_run = 0.f;

    for (int kt = 0; kt < n_tiles; ++kt) {
        __syncthreads();  // the previous tile has been consumed
        // stage K rows as they are, V transposed into the PV operand order
        for (int c = threadIdx.x; c < 32 * (D / 8); c += 256) {
            const int key = c / (D / 8), d0 = (c % (D / 8)) * 8, kabs = kt * 32 + key;
            u32x4 kk = u32x4{0u, 0u, 0u, 0u}, vv = kk;
            if (kabs < T) {
                kk = *reinterpret_cast<const u32x4*>(Kg + (size_t)kabs * D + d0);
                vv = *reinterpret_cast<const u32x4*>(Vg + (size_t)kabs * D + d0);
            }
            *reinterpret_cast<u32x4*>(&ks[key * KPITCH + d0]) = kk;
            const int s2 = key >> 4, k16 = key & 15, vh = (k16 >> 2) & 1, e = 4 * (k16 >> 3) + (k16 & 3);
            const uint32_t w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const int d = d0 + x;
                vt[((((d >> 5) * 2 + s2) * 2 + vh) * 32 + (d & 31)) * 8 + e] = (bf16_t)(w[x >> 1] >> ((x & 1) * 16));
            }
        }
        __syncthreads();
        if (kt > my_last_tile) continue;  // wholly above the diagonal for this wavefront (uniform per wavefront)
        f32x16 sacc = f32x16{};
#pragma unroll
        for (int kb = 0; kb < KBD; ++kb) {
            const u32x4 kblk = *reinterpret_cast<const u32x4*>(&ks[j * KPITCH + kb * 16 + hh * 8]);
            sacc = mfma_bf16(kblk, qhi[kb], sacc);
            sacc = mfma_bf16(kblk, qlo[kb], sacc);
        }
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int kabs = kt * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (kabs > qpos) sacc[r] = -INFINITY;
            mx = fmaxf(mx, sacc[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);  // finite from the first tile on: key 0 is visible to every query
        const float alpha = expf(m_run - m_new);
        float psum = 0.f;
        float pr[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) { pr[r] = expf(sacc[r] - m_new); psum += pr[r]; }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            uint32_t ph[4], pl[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) split2(pr[8 * s2 + 2 * x], pr[8 * s2 + 2 * x + 1], ph[x], pl[x]);
            const u32x4 phi = u32x4{ph[0], ph[1], ph[2], ph[3]}, plo = u32x4{pl[0], pl[1], pl[2], pl[3]};
#pragma unroll
            for (int i = 0; i < DB; ++i) {
                const u32x4 vblk = *reinterpret_cast<const u32x4*>(&vt[(((i * 2 + s2) * 2 + hh) * 32 + j) * 8]);
                oacc[i] = mfma_bf16(vblk, phi, oacc[i]);
                oacc[i] = mfma_bf16(vblk, plo, oacc[i]);
            }
        }
    }
    if (!live || t0 + j >= S) return;
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;  // 0: a wavefront of padding rows saw no tile
    const int m = b * S + t0 + j;
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int dim = h * D + i * 32 + 8 * qd + 4 * hh;  // four consecutive output dimensions
            uint32_t h0, h1, l0, l1;
            split2(oacc[i][qd * 4 + 0] * inv, oacc[i][qd * 4 + 1] * inv, h0, l0);
            split2(oacc[i][qd * 4 + 2] * inv, oacc[i][qd * 4 + 3] * inv, h1, l1);
            const size_t slot = block_slot(m, dim & ~7, H >> 4);
            reinterpret_cast<uint2*>(o + slot)[(dim >> 2) & 1] = make_uint2(h0, h1);
            if (o_lo) reinterpret_cast<uint2*>(o_lo + slot)[(dim >> 2) & 1] = make_uint2(l0, l1);
        }
}

static int g_num_cus = 0;

int num_cus() {
    if (g_num_cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        g_num_cus = n;
    }
    return g_num_cus;
}

#ifndef HE_SKINNY_U
#define HE_SKINNY_U(NT) ((NT) <= 4 ? 4 : 2)
#endif
#ifndef HE_SKINNY_W8_MAXNT
#define HE_SKINNY_W8_MAXNT 2
#endif
template <int MODE, int NT>
void launch_skinny_nt(hipStream_t s, const void* Wp, const void* Xhi, const void* Xlo, int KB, int n_tiles,
                      int m_tiles, int ksplit, const Epi& p) {
    constexpr int U = HE_SKINNY_U(NT);
    dim3 grid(((n_tiles + NT - 1) / NT) * ksplit, m_tiles);
    // What bounds a wavefront is its serial chain of load rounds (K/16 blocks / wavefronts / U
    // rounds, about 1.7 us each under load): eight wavefronts halve the chain when K leaves each
    // of them two rounds (and their accumulators still fit in LDS for the final reduction).
    const bool eight = NT <= HE_SKINNY_W8_MAXNT && KB / (ksplit * 8) >= 2 * U;
    // Ask for more than half of a CU's LDS so that no two workgroups share a CU: with at most one
    // workgroup per CU the dispatcher has to spread a launch of <= #CUs workgroups evenly.
    constexpr size_t kWant = 84 * 1024;
    const size_t ln_bytes = p.ln_stats ? (((size_t)p.ln_groups * 32 * sizeof(float2) + 1023) & ~(size_t)1023) : 0;
    if (eight) {
        constexpr size_t kStatic = (size_t)8 * NT * 16 * 64 * sizeof(float);
        const size_t pad = std::max(kStatic >= kWant ? 0 : kWant - kStatic, ln_bytes);
        gemm_skinny_kernel<MODE, NT <= HE_SKINNY_W8_MAXNT ? NT : 1, U, 8><<<grid, 512, pad, s>>>(
            (const u32x4*)Wp, (const u32x4*)Xhi, (const u32x4*)Xlo, KB, n_tiles, ksplit, p);
    } else {
        constexpr size_t kStatic = (size_t)4 * NT * 16 * 64 * sizeof(float);
        const size_t pad = std::max(kStatic >= kWant ? 0 : kWant - kStatic, ln_bytes);
        gemm_skinny_kernel<MODE, NT, U, 4><<<grid, 256, pad, s>>>((const u32x4*)Wp, (const u32x4*)Xhi,
                                                                  (const u32x4*)Xlo, KB, n_tiles, ksplit, p);
    }
}

template <int MODE, int HT, bool W8>
void launch_half_ht(hipStream_t s, const void* Wp, const void* Xhi, const void* Xlo, int KB, int n_half, int m_tiles,
                    int ksplit, const Epi& p) {
    // loads per wavefront and round: (HT + 4) U 16-byte loads with bf16 weights, (HT + 8) U with 8-bit ones
    constexpr int U = W8 ? (HT <= 3 ? 2 : 1) : (HT <= 3 ? 4 : 2);
    constexpr int KU = W8 ? 2 : 1;
    dim3 grid(((n_half + HT - 1) / HT) * ksplit, m_tiles);
    const bool eight = HT <= 4 && (KB / (2 * KU)) / (ksplit * 8) >= 2 * U;  // short chains per wavefront, as above
    constexpr size_t kWant = 84 * 1024;                                     // one workgroup per CU
    const size_t ln_bytes = p.ln_stats ? (((size_t)p.ln_groups * 32 * sizeof(float2) + 1023) & ~(size_t)1023) : 0;
    if (eight) {
        constexpr size_t kStatic = (size_t)8 * HT * 2 * 4 * 64 * sizeof(float);
        const size_t pad = std::max(kStatic >= kWant ? 0 : kWant - kStatic, ln_bytes);
        gemm_half_kernel<MODE, HT <= 4 ? HT : 2, U, 8, W8><<<grid, 512, pad, s>>>(
            (const u32x4*)Wp, (const u32x4*)Xhi, (const u32x4*)Xlo, KB, n_half, ksplit, p);
    } else {
        constexpr size_t kStatic = (size_t)4 * HT * 2 * 4 * 64 * sizeof(float);
        const size_t pad = std::max(kStatic >= kWant ? 0 : kWant - kStatic, ln_bytes);
        gemm_half_kernel<MODE, HT, U, 4, W8><<<grid, 256, pad, s>>>((const u32x4*)Wp, (const u32x4*)Xhi, (const u32x4*)Xlo,
                                                                    KB, n_half, ksplit, p);
    }
}

constexpr int kHalfMin = 2, kHalfMax = 10;  // 16-row units per workgroup the half-tile kernel is built for (8-bit: from 1)

template <int MODE, bool W8>
void launch_half(hipStream_t s, const void* Wp, const void* Xhi, const void* Xlo, int KB, int n_half, int m_tiles, int ht,
                 int ksplit, const Epi& p) {
    switch (ht) {
        case 1:
            if constexpr (W8) { launch_half_ht<MODE, 1, W8>(s, Wp, Xhi, Xlo, KB, n_half, m_tiles, ksplit, p); break; }
            [[fallthrough]];
        case 2: launch_half_ht<MODE, 2, W8>(s, Wp, Xhi, Xlo, KB, n_half, m_tiles, ksplit, p); break;
        case 3: launch_half_ht<MODE, 3, W8>(s, Wp, Xhi, Xlo, KB, n_half, m_tiles, ksplit, p); break;
        case 4: launch_half_ht<MODE, 4, W8>(s, Wp, Xhi, Xlo, KB, n_half, m_tiles, ksplit, p); break;
        case 5: launch_half_ht<MODE, 5, W8>(s, Wp, Xhi, Xlo, KB, n_half, m_tiles, ksplit, p); break;
        case 6: launch_half_ht<MODE, 6, W8>(s, Wp, Xhi, Xlo, KB, n_half, m_tiles, ksplit, p); break;
        case 7: launch_half_ht<MODE, 7, W8>(s, Wp, Xhi, Xlo, KB, n_half, m_tiles, ksplit, p); break;
        case 8: launch_half_ht<MODE, 8, W8>(s, Wp, Xhi, Xlo, KB, n_half, m_tiles, ksplit, p); break;
        case 9: launch_half_ht<MODE, 9, W8>(s, Wp, Xhi, Xlo, KB, n_half, m_tiles, ksplit, p); break;
        default: launch_half_ht<MODE, 10, W8>(s, Wp, Xhi, Xlo, KB, n_half, m_tiles, ksplit, p); break;
    }
}

// nt weight tiles per workgroup (1..8)
template <int MODE>
void launch_skinny(hipStream_t s, const void* Wp, const void* Xhi, const void* Xlo, int KB, int n_tiles, int m_tiles,
                   int nt, int ksplit, const Epi& p) {
    switch (nt) {
        case 1: launch_skinny_nt<MODE, 1>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, ksplit, p); break;
        case 2: launch_skinny_nt<MODE, 2>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, ksplit, p); break;
        case 3: launch_skinny_nt<MODE, 3>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, ksplit, p); break;
        case 4: launch_skinny_nt<MODE, 4>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, ksplit, p); break;
        case 5: launch_skinny_nt<MODE, 5>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, ksplit, p); break;
        case 6: launch_skinny_nt<MODE, 6>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, ksplit, p); break;
        case 7: launch_skinny_nt<MODE, 7>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, ksplit, p); break;
        default: launch_skinny_nt<MODE, 8>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, ksplit, p); break;
    }
}

// Tiles per workgroup for a GEMM whose epilogue needs the whole sum in one workgroup: the
// smallest count that fits all workgroups on the chip at once (one per CU), at most 8.
int skinny_nt_fused(int n_tiles, int m_tiles) {
    const int cus = num_cus();
    int nt = (n_tiles * m_tiles + cus - 1) / cus;
    return nt < 1 ? 1 : (nt > 8 ? 8 : nt);
}

template <int MODE>
void launch_tiled(hipStream_t s, const void* Wp, const void* Xhi, const void* Xlo, int KB, int N, int M, const Epi& p,
                  int ksplit = 1) {
    const int NT32 = (N + 31) / 32, MT32 = (M + 31) / 32;
    const int tiles_n = (N + TN - 1) / TN, tiles_m = (M + TM - 1) / TM;
    const int nitem = tiles_n * tiles_m * ksplit;
    const int grid = ((nitem + 7) / 8) * 8;
    // two workgroups per CU once there are that many (their k ranges must hold an even number of k-blocks
    // each: that ring alternates two register sets)
    const bool pair = nitem >= 2 * num_cus() && KB % (2 * ksplit) == 0;
    if (pair)
        gemm_tiled_kernel<MODE, 1><<<grid, 256, 0, s>>>((const u32x4*)Wp, (const u32x4*)Xhi, (const u32x4*)Xlo, KB, NT32,
                                                        MT32, tiles_n, tiles_m, ksplit, p);
    else
        gemm_tiled_kernel<MODE, 0><<<grid, 256, 0, s>>>((const u32x4*)Wp, (const u32x4*)Xhi, (const u32x4*)Xlo, KB, NT32,
                                                        MT32, tiles_n, tiles_m, ksplit, p);
}

// After a k-split MODE_STORE GEMM whose epilogue needs the whole sum: adds the partial sums in split
// order and applies the epilogue of MODE (bias + ReLU into blocks, or the QKV hand-out).
template <int MODE>
__global__ __launch_bounds__(256) void finish_kernel(const float* __restrict__ part, int ksplit, size_t split, Epi p) {
    const int quads = p.N >> 2;  // N is a multiple of 4 here
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)p.M * quads) return;
    const int m = (int)(idx / quads), n0 = (int)(idx % quads) * 4;
    float4 v = *reinterpret_cast<const float4*>(part + (size_t)m * p.N + n0);
    for (int k = 1; k < ksplit; ++k) {
        const float4 y = *reinterpret_cast<const float4*>(part + (size_t)k * split + (size_t)m * p.N + n0);
        v.x += y.x; v.y += y.y; v.z += y.z; v.w += y.w;
    }
    epilogue4<MODE>(p, m, n0, 0, v.x, v.y, v.z, v.w, epilogue_bias<MODE>(p, n0), epilogue_len<MODE>(p));
}

}  // namespace

// ------------------------------------------------------------------ launchers

size_t bf16_tiled_bytes(int rows, int K) { return (size_t)((rows + 31) / 32) * (K / 16) * 1024; }

void bf16_tile_rows(hipStream_t s, const void* src, void* dst, int R, int K) {
    const size_t total = (size_t)((R + 31) / 32) * (K / 16) * 64;
    tile_rows_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const bf16_t*)src, (u32x4*)dst, R, K, total);
}

size_t fp8_units_bytes(int rows, int K) { return (size_t)((rows + 15) / 16) * (K / 64) * 1024; }

void fp8_row_exponents(hipStream_t s, const void* src, int R, int K, int* exps, float* scales) {
    row_exp_kernel<<<(R + 3) / 4, 256, 0, s>>>((const bf16_t*)src, R, K, exps, scales);
}

void fp8_quant_rows(hipStream_t s, const void* src, const int* exps, void* codes, int R, int K) {
    const size_t total = (size_t)R * (K / 8);
    quant_rows_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const bf16_t*)src, exps, (uint2*)codes, R, K);
}

void fp8_quant_units(hipStream_t s, const void* src, const int* exps, void* units, int R, int K) {
    const size_t total = (size_t)((R + 15) / 16) * (K / 64) * 64;
    quant_units_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const bf16_t*)src, exps, (u32x4*)units, R, K, total);
}

void fp8_dequant_units(hipStream_t s, const void* units, const float* scales, void* dst_blocks, int R, int K) {
    const size_t total = (size_t)((R + 31) / 32) * (K / 16) * 64;
    dequant_units_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const u32x4*)units, scales, (u32x4*)dst_blocks, R, K,
                                                                        total);
}

void bf16_tile_rows_lora(hipStream_t s, const void* src, void* dst, int R, int K, const void* A, const void* B, int rank,
                         float scale) {
    const size_t total = (size_t)((R + 31) / 32) * (K / 16) * 64;
    tile_rows_lora_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const bf16_t*)src, (u32x4*)dst, R, K, total,
                                                                          (const bf16_t*)A, (const bf16_t*)B, rank, scale);
}

// Shape of a decode-shaped STORE GEMM: nt tiles per workgroup and ks k-splits such that about one
// workgroup lands on every CU.  Four tiles per workgroup (activation blocks reused four times)
// as long as each wavefront keeps 8 k-blocks, else two tiles and half the splits.  (Two tiles and
// three splits for the 5120x5120 out-projection measured 2 us slower than four and six, more
// than the LayerNorm that adds up the partial sums gained.)
static void store_shape(int N, int K, int* nt, int* ks) {
    const int tiles = (N + 31) / 32, kb = K / 16, cus = num_cus();
    int n = 4, groups = (tiles + 3) / 4;
    int k = cus / groups;
    if (k < 1) k = 1;
    if (kb / (k * 4) < 8) {
        n = 2;
        groups = (tiles + 1) / 2;
        k = cus / groups;
        if (k < 1) k = 1;
        while (k > 1 && kb / (k * 4) < 8) --k;
    }
    if (k > 8) k = 8;
    *nt = n;
    *ks = k;
}

void bf16_store_shape(int M, int N, int K, int* nt, int* ks) {
    store_shape(N, K, nt, ks);
    const int n_tiles = (N + 31) / 32, m_tiles = (M + 31) / 32;
    if (m_tiles > 1) *nt = *ks > 1 ? 2 : skinny_nt_fused(n_tiles, m_tiles);  // several row slices: keep the launch balanced
}

// How a decode-shaped GEMM is cut up: weight rows in units of 32 (the skinny kernel) or 16 (the
// half-tile kernel), `per_wg` units per workgroup, ks k-splits.  The launch waits for its most
// loaded workgroup, so the plan with the fewest weight bytes per workgroup wins, as long as all of
// its workgroups fit on the chip at once and every wavefront keeps at least 8 k-blocks.
struct GemmPlan { bool half; int per_wg, ks; };

static GemmPlan plan_fused(int M, int N) {  // epilogue needs the whole sum: no k-split
    const int n_tiles = (N + 31) / 32, m_tiles = (M + 31) / 32, cus = num_cus();
    GemmPlan g{false, skinny_nt_fused(n_tiles, m_tiles), 1};
    if (m_tiles > 1 || N % 16) return g;
    const int n_half = N / 16, ht = (n_half + cus - 1) / cus;
    if (ht >= kHalfMin && ht <= kHalfMax && 16 * ht < 32 * g.per_wg) g = GemmPlan{true, ht, 1};
    return g;
}

// capacity: floats the k-split scratch can hold (0 = not checked)
static GemmPlan plan_store(int M, int N, int K, size_t capacity) {
    GemmPlan g{false, 0, 0};
    bf16_store_shape(M, N, K, &g.per_wg, &g.ks);
    if ((M + 31) / 32 > 1 || N % 16) return g;
    const int n_half = N / 16, kb = K / 16, cus = num_cus();
    double best = (double)g.per_wg * 32 / g.ks;  // rows x (k share) per workgroup
    for (int ht = kHalfMax; ht >= kHalfMin; --ht) {
        const int groups = (n_half + ht - 1) / ht;
        int ks = cus / groups;
        if (ks < 1) continue;
        if (ks > 8) ks = 8;
        while (ks > 1 && kb / (ks * 4) < 8) --ks;
        // scratch the kernel will index: groups x splits x (items rounded up to the wavefronts) x 256 words
        if (capacity && (size_t)groups * ks * (size_t)(2 * ht + 7) * 256 > capacity) continue;
        const double load = (double)ht * 16 / ks;
        // fewer, longer k ranges per wavefront cost a 16-row plan some of its balance back (measured on the
        // 5120x5120 and 5120x20480 shapes: 6 % less load per workgroup ran no faster), so it has to win clearly
        if (load < best * 0.9) { best = load; g = GemmPlan{true, ht, ks}; }
    }
    return g;
}

// 8-bit weights: always the 16-row-unit kernel
static GemmPlan plan_fused_w8(int N) {
    const int n_half = N / 16, cus = num_cus();
    int ht = (n_half + cus - 1) / cus;
    if (ht > kHalfMax) ht = kHalfMax;
    return GemmPlan{true, ht < 1 ? 1 : ht, 1};
}

static GemmPlan plan_store_w8(int N, int K, size_t capacity) {
    const int n_half = N / 16, kq = K / 64, cus = num_cus();
    GemmPlan g{true, kHalfMax, 1};
    double best = 1e30;
    for (int ht = kHalfMax; ht >= 1; --ht) {
        const int groups = (n_half + ht - 1) / ht;
        int ks = cus / groups;
        if (ks < 1) ks = 1;
        if (ks > 8) ks = 8;
        while (ks > 1 && kq / (ks * 4) < 4) --ks;  // at least four 64-wide steps per wavefront
        if (capacity && (size_t)groups * ks * (size_t)(2 * ht + 7) * 256 > capacity) continue;
        const double load = (double)ht * 16 / ks * (groups * ks > cus ? (double)(groups * ks + cus - 1) / cus : 1.0);
        if (load < best * 0.999) { best = load; g = GemmPlan{true, ht, ks}; }
    }
    return g;
}

void bf16_store_plan_w8(int N, int K, size_t capacity, int* group_cols, int* ks) {
    const GemmPlan g = plan_store_w8(N, K, capacity);
    *group_cols = g.per_wg * 16;
    *ks = g.ks;
}

void bf16_plan_query(int M, int N, int K, int store, size_t capacity, int cus, int* unit_rows, int* per_wg, int* ks) {
    const int saved = g_num_cus;
    if (cus > 0) g_num_cus = cus;
    const GemmPlan g = store ? plan_store(M, N, K, capacity) : plan_fused(M, N);
    g_num_cus = saved;
    *unit_rows = g.half ? 16 : 32;
    *per_wg = g.per_wg;
    *ks = g.ks;
}

void bf16_store_plan(int M, int N, int K, size_t capacity, int* group_cols, int* ks) {
    const GemmPlan g = plan_store(M, N, K, capacity);
    *group_cols = g.per_wg * (g.half ? 16 : 32);
    *ks = g.ks;
}

static Epi make_epi(int M, int N, const bf16_gemm_args& a) {
    Epi p{};
    p.M = M; p.N = N; p.bias = (const bf16_t*)a.bias; p.out = a.out; p.out_split = a.out_split;
    p.out_blocks = (u32x4*)a.out_blocks; p.out_blocks_lo = (u32x4*)a.out_blocks_lo; p.kv = (bf16_t*)a.kv; p.st = a.st;
    p.S = a.S; p.layer = a.layer; p.H = a.H; p.n_heads = a.n_heads; p.d = a.n_heads ? a.H / a.n_heads : 0;
    p.max_batch = a.max_batch; p.max_seq = a.max_seq; p.qscale = a.qscale;
    p.ln_stats = (const float2*)a.ln_stats; p.ln_groups = a.ln_groups; p.ln_gw = a.ln_gw; p.ln_cols = a.ln_cols;
    p.ln_eps = a.ln_eps; p.c1 = a.c1; p.c2 = a.c2;
    p.resid = a.resid; p.gamma = (const bf16_t*)a.gamma; p.stats_out = (float2*)a.stats_out; p.counters = a.counters;
    p.wscale = a.wscale;
    return p;
}

void bf16_gemm_skinny(hipStream_t s, int mode, const void* Wp, const void* Xhi, const void* Xlo, int M, int N, int K,
                      int ksplit, const bf16_gemm_args& a) {
    (void)ksplit;
    const Epi p = make_epi(M, N, a);
    const int KB = K / 16, n_tiles = (N + 31) / 32, m_tiles = (M + 31) / 32;
    if (a.wscale) {  // 8-bit weights: Wp holds E4M3 units; one row slice only
        if (mode == EPI_STORE_LN) {
            const GemmPlan g = plan_store_w8(N, K, a.out_capacity);
            launch_half<MODE_STORE_LN, true>(s, Wp, Xhi, Xlo, KB, N / 16, m_tiles, g.per_wg, g.ks, p);
        } else {
            const GemmPlan g = plan_fused_w8(N);
            if (mode == EPI_BIAS_RELU) launch_half<MODE_BIAS_RELU, true>(s, Wp, Xhi, Xlo, KB, N / 16, m_tiles, g.per_wg, 1, p);
            else launch_half<MODE_QKV, true>(s, Wp, Xhi, Xlo, KB, N / 16, m_tiles, g.per_wg, 1, p);
        }
        return;
    }
    if (mode == EPI_STORE_LN) {  // the k-split is the one bf16_store_plan reports for this shape
        const GemmPlan g = plan_store(M, N, K, a.out_capacity);
        if (g.half) launch_half<MODE_STORE_LN, false>(s, Wp, Xhi, Xlo, KB, N / 16, m_tiles, g.per_wg, g.ks, p);
        else launch_skinny<MODE_STORE_LN>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, g.per_wg, g.ks, p);
        return;
    }
    const GemmPlan g = plan_fused(M, N);
    if (mode == EPI_BIAS_RELU) {
        if (g.half) launch_half<MODE_BIAS_RELU, false>(s, Wp, Xhi, Xlo, KB, N / 16, m_tiles, g.per_wg, 1, p);
        else launch_skinny<MODE_BIAS_RELU>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, g.per_wg, 1, p);
    } else {
        if (g.half) launch_half<MODE_QKV, false>(s, Wp, Xhi, Xlo, KB, N / 16, m_tiles, g.per_wg, 1, p);
        else launch_skinny<MODE_QKV>(s, Wp, Xhi, Xlo, KB, n_tiles, m_tiles, g.per_wg, 1, p);
    }
}

void bf16_gemm_tiled(hipStream_t s, int mode, const void* Wp, const void* Xhi, const void* Xlo, int M, int N, int K,
                     const bf16_gemm_args& a) {
    const Epi p = make_epi(M, N, a);
    if (mode == EPI_STORE) launch_tiled<MODE_STORE>(s, Wp, Xhi, Xlo, K / 16, N, M, p);
    else if (mode == EPI_BIAS_RELU) launch_tiled<MODE_BIAS_RELU>(s, Wp, Xhi, Xlo, K / 16, N, M, p);
    else launch_tiled<MODE_QKV>(s, Wp, Xhi, Xlo, K / 16, N, M, p);
}

int bf16_tiled_ksplit(int M, int N, int K) {
    const int tiles = ((N + TN - 1) / TN) * ((M + TM - 1) / TM), stages = K / 16 / TiledShape<0>::KSTAGE;
    int ks = num_cus() / tiles;
    if (ks > 8) ks = 8;
    while (ks > 1 && stages / ks < 8) --ks;  // keep the ring worth filling
    return ks < 1 ? 1 : ks;
}

// Many-row MODE_STORE GEMMs (out-projection and FC2 of a prompt pass): the tiles come in rounds of two per
// CU, and a last round that is partly empty costs as much as a full one (1280 tiles on 256 CUs: three rounds
// for the work of two and a half).  Cutting every tile into ks k ranges makes the rounds shorter and the
// last one fuller; the price is ks sets of partial sums for the following LayerNorm to add.
int bf16_tiled_store_ksplit(int M, int N, int K, size_t capacity_floats) {
    const long slots = 2L * num_cus(), tiles = (long)((N + TN - 1) / TN) * ((M + TM - 1) / TM);
    const int KB = K / 16;
    if (tiles < slots || KB % 2) return 1;
    int best = 1;
    double best_cost = (double)((tiles + slots - 1) / slots);  // in units of one full-K tile
    for (int ks = 2; ks <= 4; ++ks) {
        if (KB % (2 * ks) || KB / ks < 8 * TiledShape<1>::NSTG || (size_t)ks * M * N > capacity_floats) continue;
        const double cost = (double)((tiles * ks + slots - 1) / slots) / ks * (1.0 + 0.02 * ks);
        if (cost < 0.95 * best_cost) { best_cost = cost; best = ks; }
    }
    return best;
}

void bf16_gemm_tiled_ksplit(hipStream_t s, int mode, const void* Wp, const void* Xhi, const void* Xlo, int M, int N, int K,
                            int ksplit, float* part, size_t part_split, const bf16_gemm_args& a) {
    if (ksplit == 1 && mode != EPI_STORE) {  // the tiles alone fill the chip: the epilogue runs in the GEMM
        bf16_gemm_tiled(s, mode, Wp, Xhi, Xlo, M, N, K, a);
        return;
    }
    bf16_gemm_args st = a;
    st.out = part; st.out_split = part_split;
    const Epi ps = make_epi(M, N, st);
    launch_tiled<MODE_STORE>(s, Wp, Xhi, Xlo, K / 16, N, M, ps, ksplit);
    if (mode == EPI_STORE) return;  // the consumer (a LayerNorm) adds the partial sums
    const Epi p = make_epi(M, N, a);
    const unsigned grid = (unsigned)(((size_t)M * (N / 4) + 255) / 256);
    if (mode == EPI_BIAS_RELU) finish_kernel<MODE_BIAS_RELU><<<grid, 256, 0, s>>>(part, ksplit, part_split, p);
    else finish_kernel<MODE_QKV><<<grid, 256, 0, s>>>(part, ksplit, part_split, p);
}

void bf16_embed_ln(hipStream_t s, const int32_t* ids, int id_stride, const void* tok, const void* pos,
                   const he_dev_state* st, int B, int H, int V, int pos_offset, int gw, const void* gamma, float* r,
                   void* x_blocks, void* x_blocks_lo, float* stats) {
    const int groups = (H + gw - 1) / gw;
    embed_ln_kernel<<<dim3(groups, B), 64, 0, s>>>(ids, id_stride, (const bf16_t*)tok, (const bf16_t*)pos, st, V,
                                                   pos_offset, H, gw, groups, (const bf16_t*)gamma, r,
                                                   (u32x4*)x_blocks, (u32x4*)x_blocks_lo, (float2*)stats);
}

void bf16_wvec(hipStream_t s, const void* Wp, int N, int K, const void* gamma, const void* beta, float* c1, float* c2) {
    const int n_tiles = (N + 31) / 32;
    wvec_kernel<<<(n_tiles + 3) / 4, 256, 0, s>>>((const u32x4*)Wp, K / 16, n_tiles, (const bf16_t*)gamma,
                                                  (const bf16_t*)beta, c1, c2);
}

int bf16_score_parts(int V) { return 2 * ((V + TN - 1) / TN); }

void bf16_score_head(hipStream_t s, const void* Wp, const void* Xhi, const void* Xlo, int M, int S, int V, int K,
                     const int32_t* ids, float* stats, float* tgt, float* out) {
    Epi p{};
    p.M = M; p.N = V; p.S = S; p.ids = ids; p.sc_stats = (float2*)stats; p.sc_tgt = tgt; p.sc_parts = bf16_score_parts(V);
    launch_tiled<MODE_SCORE>(s, Wp, Xhi, Xlo, K / 16, V, M, p);
    score_reduce_kernel<<<(M + 3) / 4, 256, 0, s>>>((const float2*)stats, tgt, p.sc_parts, M, S, out);
}

void bf16_lm_head(hipStream_t s, const void* Wp, const void* Xhi, const void* Xlo, int B, int V, int K,
                  const he_dev_state* st, float* logits_opt, float* stats, int* stats_idx, int32_t* ids_out,
                  float* lp_out, int out_stride, int out_at_step, int32_t* cur_ids, const bf16_gemm_args* fold) {
    Epi p{};
    if (fold) p = make_epi(B, V, *fold);
    p.M = B; p.N = V; p.st = st; p.logits = logits_opt; p.stats = stats; p.stats_idx = stats_idx;
    p.n_tiles = (V + 31) / 32;
    const int m_tiles = (B + 31) / 32;
    launch_skinny<MODE_LMHEAD>(s, Wp, Xhi, Xlo, K / 16, p.n_tiles, m_tiles, skinny_nt_fused(p.n_tiles, m_tiles), 1, p);
    lm_reduce_kernel<<<B, 256, 0, s>>>(stats, stats_idx, p.n_tiles, st, ids_out, lp_out, out_stride, out_at_step,
                                       cur_ids);
}

void bf16_ln(hipStream_t s, float* r, const float* part, int ksplit, size_t part_split, const void* pbias,
             const void* gamma, const void* beta, void* a_blocks, void* a_blocks_lo, int rows, int H, float eps,
             int in_mul, int in_add, int writeback) {
    const int nv = (H / 4 + 1023) / 1024, nv256 = (H / 4 + 255) / 256;
#define HE_LN_ROW(NV, T)                                                                                                \
    ln_row_kernel<NV, T><<<rows, T, 0, s>>>(r, part, ksplit, part_split, (const bf16_t*)pbias, (const bf16_t*)gamma,    \
                                            (const bf16_t*)beta, (u32x4*)a_blocks, (u32x4*)a_blocks_lo, H, eps, in_mul, \
                                            in_add, writeback)
    if (rows <= 256 && nv <= 3) {  // a decode step
        if (nv == 1) HE_LN_ROW(1, 1024);
        else if (nv == 2) HE_LN_ROW(2, 1024);
        else HE_LN_ROW(3, 1024);
        return;
    }
    if (nv256 <= 10) {  // prompt rows, hidden sizes up to 10240
        switch (nv256) {
            case 1: HE_LN_ROW(1, 256); break;
            case 2: HE_LN_ROW(2, 256); break;
            case 3: HE_LN_ROW(3, 256); break;
            case 4: HE_LN_ROW(4, 256); break;
            case 5: HE_LN_ROW(5, 256); break;
            case 6: HE_LN_ROW(6, 256); break;
            case 7: HE_LN_ROW(7, 256); break;
            case 8: HE_LN_ROW(8, 256); break;
            case 9: HE_LN_ROW(9, 256); break;
            default: HE_LN_ROW(10, 256); break;
        }
        return;
    }
#undef HE_LN_ROW
    ln_blocks_kernel<<<rows, 256, (size_t)H * sizeof(float), s>>>(
        r, part, ksplit, part_split, (const bf16_t*)pbias, (const bf16_t*)gamma, (const bf16_t*)beta, (u32x4*)a_blocks,
        (u32x4*)a_blocks_lo, H, eps, in_mul, in_add, writeback);
}

void bf16_attn(hipStream_t s, const float* q, const void* kv, void* o_blocks, void* o_blocks_lo,
               const he_dev_state* st, int M, int S, int layer, int H, int n_heads, int max_batch, int max_seq) {
    if (S >= 32) {  // prompt rows: 32 queries per wavefront on the matrix cores
        dim3 fgrid((S + 127) / 128, n_heads, M / S);
        if (H / n_heads == 128)
            attn_prompt_mfma_kernel<128><<<fgrid, 256, 0, s>>>(q, (const bf16_t*)kv, (u32x4*)o_blocks,
                                                               (u32x4*)o_blocks_lo, st, S, layer, H, n_heads,
                                                               max_batch, max_seq);
        else
            attn_prompt_mfma_kernel<64><<<fgrid, 256, 0, s>>>(q, (const bf16_t*)kv, (u32x4*)o_blocks,
                                                              (u32x4*)o_blocks_lo, st, S, layer, H, n_heads,
                                                              max_batch, max_seq);
        return;
    }
    const size_t prompt_shm = (size_t)QB * max_seq * sizeof(float);
    if (S >= QB && prompt_shm <= 96 * 1024) {  // short prompts: blocks of QB queries per workgroup
        dim3 pgrid((S + QB - 1) / QB, n_heads, M / S);
        if (H / n_heads == 128)
            attn_prompt_kernel<128><<<pgrid, 256, prompt_shm, s>>>(q, (const bf16_t*)kv, (u32x4*)o_blocks,
                                                                   (u32x4*)o_blocks_lo, st, S, layer, H, n_heads,
                                                                   max_batch, max_seq);
        else
            attn_prompt_kernel<64><<<pgrid, 256, prompt_shm, s>>>(q, (const bf16_t*)kv, (u32x4*)o_blocks,
                                                                  (u32x4*)o_blocks_lo, st, S, layer, H, n_heads,
                                                                  max_batch, max_seq);
        return;
    }
    dim3 grid(M, n_heads);
    const size_t shm = (size_t)max_seq * sizeof(float);
    if (H / n_heads == 128)
        attn_kernel<128><<<grid, 256, shm, s>>>(q, (const bf16_t*)kv, (u32x4*)o_blocks, (u32x4*)o_blocks_lo, st, S,
                                                layer, H, n_heads, max_batch, max_seq);
    else
        attn_kernel<64><<<grid, 256, shm, s>>>(q, (const bf16_t*)kv, (u32x4*)o_blocks, (u32x4*)o_blocks_lo, st, S,
                                               layer, H, n_heads, max_batch, max_seq);
}
