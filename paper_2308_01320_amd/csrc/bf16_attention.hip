// bf16 path: attention over the KV cache of IEEE halves (decode rows, short prompts, prompt rows on the matrix cores).
#include "bf16_common.h"

using namespace he_bf16;

namespace {

// ----------------------------------------------------------------- attention over the KV cache
//
// One workgroup per (row m, head h); the query at position cur_len + (m % S)
// sees keys 0..that position.  D/8 adjacent lanes own one key (16 bytes each, a
// whole row of K or V per group, coalesced); scores are reduced with wavefront
// shuffles, kept in LDS, soft-maxed, then the same lanes accumulate p_j * V[j].
// The output goes out as tiled half blocks for the out-projection GEMM.
template <int D>
__global__ __launch_bounds__(256) void attn_kernel(const float* __restrict__ q, const half_t* __restrict__ kv,
                                                   u32x4* __restrict__ o,
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
    const int b = row_seq(st, m, S), T = seq_len(st, b) + (m % S) - row_pad(st, b) + 1;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sub = lane % LPK, grp = lane / LPK;
    if (seq_done(st, b)) return;  // the sequence has ended: its row's output is not used any more
    if (T <= 0) {                 // a padding row: nothing to attend to, nothing reads the output; keep it finite
        if (wave == 0 && grp == 0) {
            const size_t slot = block_slot(m, h * D + sub * 8, H >> 4);
            o[slot] = u32x4{0u, 0u, 0u, 0u};
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
            float s = qa.x * half_lo(cur[u].x);
            s = fmaf(qa.y, half_hi(cur[u].x), s);
            s = fmaf(qa.z, half_lo(cur[u].y), s);
            s = fmaf(qa.w, half_hi(cur[u].y), s);
            s = fmaf(qb.x, half_lo(cur[u].z), s);
            s = fmaf(qb.y, half_hi(cur[u].z), s);
            s = fmaf(qb.z, half_lo(cur[u].w), s);
            s = fmaf(qb.w, half_hi(cur[u].w), s);
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
            acc[0] = fmaf(pj, half_lo(cur[u].x), acc[0]);
            acc[1] = fmaf(pj, half_hi(cur[u].x), acc[1]);
            acc[2] = fmaf(pj, half_lo(cur[u].y), acc[2]);
            acc[3] = fmaf(pj, half_hi(cur[u].y), acc[3]);
            acc[4] = fmaf(pj, half_lo(cur[u].z), acc[4]);
            acc[5] = fmaf(pj, half_hi(cur[u].z), acc[5]);
            acc[6] = fmaf(pj, half_lo(cur[u].w), acc[6]);
            acc[7] = fmaf(pj, half_hi(cur[u].w), acc[7]);
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
        const size_t slot = block_slot(m, h * D + threadIdx.x * 8, H >> 4);
        o[slot] = u32x4{pack2(ov[0], ov[1]), pack2(ov[2], ov[3]), pack2(ov[4], ov[5]), pack2(ov[6], ov[7])};
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
__global__ __launch_bounds__(256) void attn_prompt_kernel(const float* __restrict__ q, const half_t* __restrict__ kv,
                                                          u32x4* __restrict__ o,
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
            const float k0 = half_lo(cur_r[u].x), k1 = half_hi(cur_r[u].x);
            const float k2 = half_lo(cur_r[u].y), k3 = half_hi(cur_r[u].y);
            const float k4 = half_lo(cur_r[u].z), k5 = half_hi(cur_r[u].z);
            const float k6 = half_lo(cur_r[u].w), k7 = half_hi(cur_r[u].w);
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
                const float v0 = half_lo(cur_r[u].x), v1 = half_hi(cur_r[u].x);
                const float v2 = half_lo(cur_r[u].y), v3 = half_hi(cur_r[u].y);
                const float v4 = half_lo(cur_r[u].z), v5 = half_hi(cur_r[u].z);
                const float v6 = half_lo(cur_r[u].w), v7 = half_hi(cur_r[u].w);
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
        const size_t slot = block_slot(b * S + t0 + i, h * D + c * 8, H >> 4);
        o[slot] = u32x4{pack2(ov[0], ov[1]), pack2(ov[2], ov[3]), pack2(ov[4], ov[5]), pack2(ov[6], ov[7])};
    }
}

// ----------------------------------------------------------------- attention, prompt rows, on the matrix cores
//
// Flash-style causal attention for the prompt pass.  One wavefront owns 32 queries of one
// (sequence, head); the four wavefronts of a workgroup share each 32-key tile of K and V through
// LDS.  Everything is computed transposed so that a lane owns ONE query: S^T = K Q^T puts the
// scores of query lane%32 in that lane's 16 accumulators (online soft-max needs one exchange
// with lane^32), and O^T = V^T P^T accumulates that query's output column, so the soft-max
// rescaling is a per-lane scalar.  Q and P enter the MFMA as two half terms (hi + lo).  The
// keys of a PV step are taken in the order the score accumulators already hold them; the V^T
// operand is gathered in that order from the staged rows with 16-bit LDS reads.
template <int D>
__global__ __launch_bounds__(256, 2) void attn_prompt_mfma_kernel(const float* __restrict__ q,
                                                               const half_t* __restrict__ kv, u32x4* __restrict__ o,
                                                               const he_dev_state* __restrict__ st, int S, int layer,
                                                               int H, int n_heads, int max_batch, int max_seq) {
    constexpr int KBD = D / 16;      // k-blocks over the head dimension
    constexpr int DB = D / 32;       // 32-wide blocks of output dimensions
    constexpr int KPITCH = D + 8;    // halves per K row in LDS (16 bytes of padding)
    __shared__ __align__(16) half_t ks[32 * KPITCH];
    __shared__ __align__(16) half_t vs[32 * KPITCH];
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
    const half_t* Kg = kv + kv_index(layer, 0, b, h, 0, max_batch, n_heads, max_seq, D);
    const half_t* Vg = kv + kv_index(layer, 1, b, h, 0, max_batch, n_heads, max_seq, D);
    f32x16 oacc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i) oacc[i] = f32x16{};
    float m_run = -INFINITY, l_run = 0.f;

    // A tile's K and V rows are requested one tile ahead and wait in registers while the tile before
    // them is multiplied, so that their latency is not paid between two barriers.
    constexpr int NI = 32 * (D / 8) / 256;  // 16-byte pieces of K (and of V) per thread and tile
    u32x4 kreg[NI], vreg[NI];
    auto request_tile = [&](int kt) {
#pragma unroll
        for (int n = 0; n < NI; ++n) {
            const int c = threadIdx.x + n * 256;
            const int key = c / (D / 8), d0 = (c % (D / 8)) * 8, kabs = kt * 32 + key;
            kreg[n] = vreg[n] = u32x4{0u, 0u, 0u, 0u};
            if (kabs < T) {
                kreg[n] = *reinterpret_cast<const u32x4*>(Kg + (size_t)kabs * D + d0);
                vreg[n] = *reinterpret_cast<const u32x4*>(Vg + (size_t)kabs * D + d0);
            }
        }
    };
    request_tile(0);
    for (int kt = 0; kt < n_tiles; ++kt) {
        __syncthreads();  // the previous tile has been consumed
        // stage the K and V rows as they are (a padded pitch keeps the reads below off each other's banks)
#pragma unroll
        for (int n = 0; n < NI; ++n) {
            const int c = threadIdx.x + n * 256;
            const int key = c / (D / 8), d0 = (c % (D / 8)) * 8;
            *reinterpret_cast<u32x4*>(&ks[key * KPITCH + d0]) = kreg[n];
            *reinterpret_cast<u32x4*>(&vs[key * KPITCH + d0]) = vreg[n];
        }
        __syncthreads();
        if (kt + 1 < n_tiles) request_tile(kt + 1);
        if (kt > my_last_tile) continue;  // wholly above the diagonal for this wavefront (uniform per wavefront)
        // two accumulators (one per term of Q), so that consecutive MFMAs do not wait for each other's result
        f32x16 sacc = f32x16{}, sacc_lo = f32x16{};
#pragma unroll
        for (int kb = 0; kb < KBD; ++kb) {
            const u32x4 kblk = *reinterpret_cast<const u32x4*>(&ks[j * KPITCH + kb * 16 + hh * 8]);
            sacc = mfma_f16(kblk, qhi[kb], sacc);
            sacc_lo = mfma_f16(kblk, qlo[kb], sacc_lo);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] += sacc_lo[r];
        float mx = -INFINITY;
        if (kt * 32 + 31 > cur + t0) {  // the tile reaches past the first query's last key: mask per query
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kabs = kt * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
                if (kabs > qpos) sacc[r] = -INFINITY;
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);  // finite from the first tile on: key 0 is visible to every query
        // the hardware's exponential (2^(x log2 e), a few ulp): the library routine's ~20 instructions per
        // value were more work per tile than its matrix products
        const float alpha = __expf(m_run - m_new);
        float psum = 0.f;
        float pr[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) { pr[r] = __expf(sacc[r] - m_new); psum += pr[r]; }
        l_run = l_run * alpha + psum;
        if (__any(m_new != m_run)) {  // no query of this wavefront met a larger score: nothing to rescale
#pragma unroll
            for (int i = 0; i < DB; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
        }
        m_run = m_new;
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            uint32_t ph[4], pl[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) split2(pr[8 * s2 + 2 * x], pr[8 * s2 + 2 * x + 1], ph[x], pl[x]);
            const u32x4 phi = u32x4{ph[0], ph[1], ph[2], ph[3]}, plo = u32x4{pl[0], pl[1], pl[2], pl[3]};
#pragma unroll
            for (int i = 0; i < DB; ++i) {
                // V^T operand: this lane's output dimension, the eight keys in the order the score
                // accumulators hold them (16-bit reads down a column of the staged rows: the 32 lanes of
                // a half read 64 consecutive bytes, the two halves sit 16 banks apart)
                const half_t* vcol = &vs[(s2 * 16 + 4 * hh) * KPITCH + i * 32 + j];
                uint32_t vw[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int k0 = 8 * (x >> 1) + 2 * (x & 1);  // element 2x of the operand; 2x+1 is the next key
                    vw[x] = (uint32_t)vcol[k0 * KPITCH] | ((uint32_t)vcol[(k0 + 1) * KPITCH] << 16);
                }
                const u32x4 vblk = u32x4{vw[0], vw[1], vw[2], vw[3]};
                oacc[i] = mfma_f16(vblk, phi, oacc[i]);
                oacc[i] = mfma_f16(vblk, plo, oacc[i]);
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
            const size_t slot = block_slot(m, dim & ~7, H >> 4);
            reinterpret_cast<uint2*>(o + slot)[(dim >> 2) & 1] =
                make_uint2(pack2(oacc[i][qd * 4 + 0] * inv, oacc[i][qd * 4 + 1] * inv),
                           pack2(oacc[i][qd * 4 + 2] * inv, oacc[i][qd * 4 + 3] * inv));
        }
}

}  // namespace

// ------------------------------------------------------------------ launchers

void bf16_attn(hipStream_t s, const float* q, const void* kv, void* o_blocks, const he_dev_state* st, int M, int S, int layer, int H, int n_heads, int max_batch, int max_seq) {
    if (S >= 32) {  // prompt rows: 32 queries per wavefront on the matrix cores
        dim3 fgrid((S + 127) / 128, n_heads, M / S);
        if (H / n_heads == 128)
            attn_prompt_mfma_kernel<128><<<fgrid, 256, 0, s>>>(q, (const half_t*)kv, (u32x4*)o_blocks, st, S, layer, H, n_heads,
                                                               max_batch, max_seq);
        else
            attn_prompt_mfma_kernel<64><<<fgrid, 256, 0, s>>>(q, (const half_t*)kv, (u32x4*)o_blocks, st, S, layer, H, n_heads,
                                                              max_batch, max_seq);
        return;
    }
    const size_t prompt_shm = (size_t)QB * max_seq * sizeof(float);
    if (S >= QB && prompt_shm <= 96 * 1024) {  // short prompts: blocks of QB queries per workgroup
        dim3 pgrid((S + QB - 1) / QB, n_heads, M / S);
        if (H / n_heads == 128)
            attn_prompt_kernel<128><<<pgrid, 256, prompt_shm, s>>>(q, (const half_t*)kv, (u32x4*)o_blocks, st, S, layer, H, n_heads,
                                                                   max_batch, max_seq);
        else
            attn_prompt_kernel<64><<<pgrid, 256, prompt_shm, s>>>(q, (const half_t*)kv, (u32x4*)o_blocks, st, S, layer, H, n_heads,
                                                                  max_batch, max_seq);
        return;
    }
    dim3 grid(M, n_heads);
    const size_t shm = (size_t)max_seq * sizeof(float);
    if (H / n_heads == 128)
        attn_kernel<128><<<grid, 256, shm, s>>>(q, (const half_t*)kv, (u32x4*)o_blocks, st, S,
                                                layer, H, n_heads, max_batch, max_seq);
    else
        attn_kernel<64><<<grid, 256, shm, s>>>(q, (const half_t*)kv, (u32x4*)o_blocks, st, S,
                                               layer, H, n_heads, max_batch, max_seq);
}
