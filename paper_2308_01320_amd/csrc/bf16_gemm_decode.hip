// bf16 path: the weight-streaming GEMMs of a decode step (at most 32 rows per slice) and the LM head
// fused with log-softmax and sampling.  Weights and activations are tiled blocks of IEEE halves.
#include "bf16_common.h"

using namespace he_bf16;

namespace {

// Quads of outputs a thread of a workgroup holds after the k loop: the workgroup's (tile or unit, row part) items
// dealt out over its wavefronts.  One definition for the kernels and for the launchers' account of the scratch a
// launch indexes.
constexpr int items_per_wave(int items, int waves) { return (items + waves - 1) / waves; }
// Floats of k-split scratch one split of one column group covers (store_ln_tail's layout).
constexpr size_t tail_floats_per_split(int items, int waves) { return (size_t)items * 4 * waves * 64; }

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
// 45 us per launch).  The 64-bit words of one (split, item, pair) are laid out thread after thread: every
// access is a contiguous 512 bytes per wavefront.  Each workgroup publishes its partial sums, waits for the
// stores to be acknowledged and counts itself in; whoever counts last for the column group reads all splits
// back -- its own included -- and adds them in split order, so the sum does not depend on which
// workgroup that was.  Nobody waits for anybody: the others are done.  The last one adds bias and
// residual, writes the residual rows back, gamma * x as half blocks, and the group's statistics
// (mean and sum of squared deviations per row over the group's `cnt` columns, fixed summation order).
// Returns to the caller, who returns.
// MT: 32-row slices the workgroup holds (rows mt*32 .. mt*32 + 32 MT - 1; mt = its first slice).
template <int ITEMS, int WAVES, int LG, int MT = 1>
__device__ __forceinline__ void store_ln_tail(const Epi& p, int ksplit, int ks, int grp, int groups, int mt, float cnt,
                                              const float (&v)[ITEMS][4], const int (&mrow)[ITEMS],
                                              const int (&n0)[ITEMS], const bool (&live)[ITEMS],
                                              const int (&rslot)[ITEMS]) {
    constexpr int NSLOT = 32 * MT / LG;
    __shared__ int s_last;
    __shared__ float sred[2][WAVES][32 * MT];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t cell = (size_t)grp * gridDim.y + blockIdx.y;
    constexpr size_t kPer = tail_floats_per_split(ITEMS, WAVES);  // words of one split of one column group
    // 64-bit words (two sums each): a wavefront can have 63 loads outstanding, and the wider they are, the more
    // of the last workgroup's read-back is in flight at once
    uint64_t* scratch = reinterpret_cast<uint64_t*>(p.out + cell * ksplit * kPer) + threadIdx.x;
    constexpr size_t kPer2 = kPer / 2;
    auto pair_bits = [](float a, float b) { return (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32); };
    if (ksplit > 1) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            if (!live[i]) continue;
#pragma unroll
            for (int h = 0; h < 2; ++h)
                __hip_atomic_store(scratch + (ks * kPer2 + (size_t)(i * 2 + h) * WAVES * 64), pair_bits(v[i][2 * h], v[i][2 * h + 1]),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
    // The splits' partial sums come from the level all XCDs share, a microsecond or two away.  All loads of
    // a chunk of items are issued before anything is stored: with loads and stores outstanding together the
    // hardware counter no longer tells which have returned, and every wait would drain them all.
    constexpr int CH = ITEMS < 4 ? ITEMS : 4;
    auto lo32 = [](uint64_t w) { return __uint_as_float((uint32_t)w); };
    auto hi32 = [](uint64_t w) { return __uint_as_float((uint32_t)(w >> 32)); };
#pragma unroll
    for (int c0 = 0; c0 < ITEMS; c0 += CH) {
        uint64_t y[CH][8][2];
        float4 rr[CH];
        uint2 bb[CH], gg[CH];
        uint2 hh[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int i = c0 + c;
            if (i >= ITEMS) continue;
            // every lane loads (rows and columns past the end are clamped, their results never stored):
            // no per-lane branches around the loads
            const int mc = min(mrow[i], p.M - 1), nc = min(n0[i], p.N - 4);
            rr[c] = *reinterpret_cast<const float4*>(p.resid + (size_t)mc * p.N + nc);
            bb[c] = *reinterpret_cast<const uint2*>(p.bias + nc);
            gg[c] = *reinterpret_cast<const uint2*>(p.gamma + nc);
        }
        if (ksplit > 1) {  // every split's sums, this workgroup's own included: one uniform test per split
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (k >= ksplit) break;
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const int i = c0 + c;
                    if (i >= ITEMS) continue;
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        y[c][k][h] = __hip_atomic_load(scratch + (k * kPer2 + (size_t)(i * 2 + h) * WAVES * 64),
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int i = c0 + c;
            if (i >= ITEMS) continue;
            x[i][0] = x[i][1] = x[i][2] = x[i][3] = 0.f;
            if (!live[i]) continue;
            float4 tot = make_float4(v[i][0], v[i][1], v[i][2], v[i][3]);
            if (ksplit > 1) {  // in split order, whichever split this workgroup was
                tot = make_float4(lo32(y[c][0][0]), hi32(y[c][0][0]), lo32(y[c][0][1]), hi32(y[c][0][1]));
#pragma unroll
                for (int k = 1; k < 8; ++k)
                    if (k < ksplit) {
                        tot.x += lo32(y[c][k][0]); tot.y += hi32(y[c][k][0]);
                        tot.z += lo32(y[c][k][1]); tot.w += hi32(y[c][k][1]);
                    }
            }
            x[i][0] = rr[c].x + (tot.x + bf_lo(bb[c].x));
            x[i][1] = rr[c].y + (tot.y + bf_hi(bb[c].x));
            x[i][2] = rr[c].z + (tot.z + bf_lo(bb[c].y));
            x[i][3] = rr[c].w + (tot.w + bf_hi(bb[c].y));
            hh[c].x = pack2(x[i][0] * bf_lo(gg[c].x), x[i][1] * bf_hi(gg[c].x));
            hh[c].y = pack2(x[i][2] * bf_lo(gg[c].y), x[i][3] * bf_hi(gg[c].y));
            const float part = (x[i][0] + x[i][1]) + (x[i][2] + x[i][3]);
#pragma unroll
            for (int r = 0; r < NSLOT; ++r)
                if (rslot[i] == r) srow[r] += part;
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int i = c0 + c;
            if (i >= ITEMS || !live[i]) continue;
            *reinterpret_cast<float4*>(p.resid + (size_t)mrow[i] * p.N + n0[i]) = make_float4(x[i][0], x[i][1], x[i][2], x[i][3]);
            const size_t slot = block_slot(mrow[i], n0[i] & ~7, p.N >> 4);
            reinterpret_cast<uint2*>(p.out_blocks + slot)[(n0[i] >> 2) & 1] = hh[c];
        }
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
    if (threadIdx.x < 32 * MT) {  // (wavefront 0: lane = row)
        float m2 = 0.f, tot = 0.f;
#pragma unroll
        for (int ww = 0; ww < WAVES; ++ww) { m2 += sred[1][ww][lane]; tot += sred[0][ww][lane]; }
        p.stats_out[((size_t)(mt + (lane >> 5)) * groups + grp) * 32 + (lane & 31)] = make_float2(tot / cnt, m2);
    }
    if (threadIdx.x == 0 && ksplit > 1)  // ready for the next launch
        __hip_atomic_store(p.counters + cell, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ----------------------------------------------------------------- skinny GEMM (decode, LM head)
//
// At most 32 rows per grid.y slice: weights are streamed exactly once from HBM,
// straight from global memory into MFMA operand registers.  A workgroup of four
// or eight wavefronts owns NT consecutive 32-row weight tiles and one k-split; its
// wavefronts divide the k range, keep U blocks per stream in flight (NT weight
// streams plus the activation stream out of L2, which every weight
// tile reuses from registers), and combine their accumulators through LDS.  The
// sum over k-splits (MODE_STORE_LN) is taken by the last-arriving workgroup (above).
//
// The launcher picks NT (and the k-split) to put one equally loaded workgroup on
// as many of the CUs as the shape allows: more workgroups than CUs double up
// on some CUs and the whole launch waits for those.  Measured on the 13B shapes:
// the stream itself runs at the HBM rate; what it competes for is the path from
// L2 to the CU, which carries the activation panel (half as many bytes again as the
// weights when NT = 2) next to the weights.  Everything executed once per launch
// (prologue, epilogue) is instruction-bound -- a wavefront issues one vector
// instruction per four cycles -- so the code around the loop is kept short and
// what the epilogue needs is requested behind the first round of weight loads.

template <int NT, int U>
struct SkinnyRegs {
    u32x4 w[NT][U], x[U];
};

template <int NT, int U>
__device__ __forceinline__ void skinny_load(SkinnyRegs<NT, U>& r, const u32x4* (&w)[NT], const u32x4*& xh) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int t = 0; t < NT; ++t) r.w[t][u] = __builtin_nontemporal_load(w[t] + u * 64);
        r.x[u] = xh[u * 64];
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) w[t] += U * 64;
    xh += U * 64;
}

template <int NT, int U>
__device__ __forceinline__ void skinny_mma(const SkinnyRegs<NT, U>& r, f32x16 (&acc)[NT]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = mfma_f16(r.w[t][u], r.x[u], acc[t]);
    }
}

template <int MODE, int NT, int U, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gemm_skinny_kernel(const u32x4* __restrict__ Wp,
                                                                 const u32x4* __restrict__ Xhi, int KB, int n_tiles,
                                                                 int ksplit, Epi p) {
    __shared__ float red[WAVES][NT][16][64];
    __shared__ float lnp[WAVES * 4 * 32];  // folded LayerNorm: the wavefronts' partial sums of the row statistics
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int bx = blockIdx.x, mt = blockIdx.y;
    if (MODE == MODE_LMHEAD && gridDim.y > 1) {
        // Several 32-row slices each stream the whole matrix.  Workgroups go round the XCDs by index: the slices
        // of one group of tiles are placed on ONE XCD, next to each other in dispatch order, so that they run
        // side by side and all but the first of them find the weights in that XCD's L2 (the grid's x is padded
        // to a multiple of eight for this).
        const int lid = blockIdx.y * gridDim.x + blockIdx.x, span = 8 * gridDim.y;
        bx = (lid / span) * 8 + (lid % span) % 8;
        mt = (lid % span) / 8;
        if (bx >= (n_tiles + NT - 1) / NT) return;  // the whole workgroup
    }
    const int grp = bx / ksplit, ks = bx % ksplit;
    const int parts = ksplit * WAVES, part = ks * WAVES + wave;
    const int kb0 = (int)(((long)part * KB) / parts), kb1 = (int)(((long)(part + 1) * KB) / parts);
    constexpr bool FOLDABLE = MODE == MODE_BIAS_RELU || MODE == MODE_QKV || MODE == MODE_LMHEAD;
    const u32x4* w[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)  // tiles past the last one are computed from the last one, never stored
        w[t] = Wp + ((size_t)min(grp * NT + t, n_tiles - 1) * KB + kb0) * 64 + lane;
    const u32x4* xh = Xhi + ((size_t)mt * KB + kb0) * 64 + lane;
    // After the k loop the NT*4 (tile, row-quad) items of the workgroup are shared out over its
    // wavefronts: item = wave + i*WAVES -> tile item/4, rows 8*(item%4) + 4*(lane/32) + 0..3.
    constexpr int ITEMS = items_per_wave(NT * 4, WAVES);
    // What the epilogue needs (bias, the folded LayerNorm's vectors and statistics, the cache length) is
    // requested right behind the first round of weight loads: long before it is used, and without holding
    // up the start of the weight stream, which then waits for three pointers and three sizes only.
    uint2 bias_w[ITEMS];
    float4 c1w[ITEMS], c2w[ITEMS];
    LnLoads lnl;
    bool fold = false;
    int cur_len = 0;
    auto request_epilogue_operands = [&]() {
        fold = FOLDABLE && p.ln_stats != nullptr;
        if (fold) ln_issue<WAVES>(lnl, p, mt, wave, lane);
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
        cur_len = epilogue_len<MODE>(p);
    };
    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x16{};
    int n = kb1 - kb0;
    if (n >= U) {
        SkinnyRegs<NT, U> ra;
        skinny_load<NT, U>(ra, w, xh);
        n -= U;
        request_epilogue_operands();
        // the statistics are used once the second round is on its way as well (first trip peeled off
        // the loop: a test inside it cost the loop its schedule)
        if (n >= U) {
            SkinnyRegs<NT, U> rb;
            skinny_load<NT, U>(rb, w, xh);
            n -= U;
            if (fold) ln_partial<WAVES>(lnl, p, mt, wave, lane, lnp);
            skinny_mma<NT, U>(ra, acc);
            ra = rb;
        } else if (fold) {
            ln_partial<WAVES>(lnl, p, mt, wave, lane, lnp);
        }
        while (n >= U) {
            SkinnyRegs<NT, U> rb;
            skinny_load<NT, U>(rb, w, xh);
            n -= U;
            skinny_mma<NT, U>(ra, acc);
            ra = rb;
        }
        skinny_mma<NT, U>(ra, acc);
    } else {
        request_epilogue_operands();
        if (fold) ln_partial<WAVES>(lnl, p, mt, wave, lane, lnp);
    }
    for (; n > 0; --n) {
        SkinnyRegs<NT, 1> r1;
        skinny_load<NT, 1>(r1, w, xh);
        skinny_mma<NT, 1>(r1, acc);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave][t][r][lane] = acc[t][r];
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
        const float2 mr = ln_finish<WAVES>(lnp, lane & 31, p);
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
            const uint32_t seq = (uint32_t)row_seq(p.st, mm, 1);  // the noise is keyed by the sequence, not by its row
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
                    s = z / temp + gumbel_from_word(philox_word0((uint32_t)vid, (uint32_t)step, seq, k0, k1));
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

__device__ __forceinline__ f32x4 mfma16_f16(const u32x4& a, const u32x4& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// 16 E4M3 codes -> two half operand registers (exact: an E4M3 value has four significant bits and lies in
// 2^-9 .. 448).  Bytes 0-7 are the lane's eight k values of the first 32-wide k range, bytes 8-15 those of the second.
__device__ __forceinline__ uint32_t e4m3x2_to_f16x2(uint32_t word, bool upper) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 f = upper ? __builtin_amdgcn_cvt_pk_f32_fp8(word, true) : __builtin_amdgcn_cvt_pk_f32_fp8(word, false);
    return pack2(f.x, f.y);
}
__device__ __forceinline__ void e4m3x16_to_f16(const u32x4& w, u32x4& a0, u32x4& a1) {
    a0 = u32x4{e4m3x2_to_f16x2(w.x, false), e4m3x2_to_f16x2(w.x, true), e4m3x2_to_f16x2(w.y, false),
               e4m3x2_to_f16x2(w.y, true)};
    a1 = u32x4{e4m3x2_to_f16x2(w.z, false), e4m3x2_to_f16x2(w.z, true), e4m3x2_to_f16x2(w.w, false),
               e4m3x2_to_f16x2(w.w, true)};
}

// One loop step of a wavefront covers KU = 1 (bf16 weights) or 2 (8-bit weights: one 16-byte load holds
// two) k ranges of 32, U steps per round of loads.
// MH: 16-row halves of the activation rows a workgroup multiplies its weights by: 2 = one 32-row slice, 4 = two
// slices (decode steps of 33..64 sequences: the weights are still streamed once), 1 = the first half only (at
// most 16 sequences: the other half's loads and products would be thrown away); xstride = 16-byte units
// between two slices
template <int HT, int U, bool W8, int MH = 2>
struct HalfRegs {
    static constexpr int KU = W8 ? 2 : 1;
    u32x4 w[HT][U], xh[MH][U * KU];
};

template <int HT, int U, bool W8, int MH = 2>
__device__ __forceinline__ void half_load(HalfRegs<HT, U, W8, MH>& r, const u32x4* (&w)[HT], const u32x4*& xh,
                                          size_t xstride = 0) {
    constexpr int KU = W8 ? 2 : 1, WSTEP = W8 ? 64 : 128;
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int t = 0; t < HT; ++t) r.w[t][u] = __builtin_nontemporal_load(w[t] + u * WSTEP);
#pragma unroll
        for (int kp = 0; kp < KU; ++kp)
#pragma unroll
            for (int mh = 0; mh < MH; ++mh)
                r.xh[mh][u * KU + kp] = xh[(u * KU + kp) * 128 + (mh & 1) * 16 + (mh >> 1) * xstride];
    }
#pragma unroll
    for (int t = 0; t < HT; ++t) w[t] += U * WSTEP;
    xh += U * KU * 128;
}

template <int HT, int U, bool W8, int MH = 2>
__device__ __forceinline__ void half_mma(const HalfRegs<HT, U, W8, MH>& r, f32x4 (&acc)[HT][MH]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (W8) {
#pragma unroll
            for (int t = 0; t < HT; ++t) {
                u32x4 a[2];
                e4m3x16_to_f16(r.w[t][u], a[0], a[1]);
#pragma unroll
                for (int kp = 0; kp < 2; ++kp)
#pragma unroll
                    for (int mh = 0; mh < MH; ++mh) acc[t][mh] = mfma16_f16(a[kp], r.xh[mh][u * 2 + kp], acc[t][mh]);
            }
        } else {
#pragma unroll
            for (int t = 0; t < HT; ++t)
#pragma unroll
                for (int mh = 0; mh < MH; ++mh) acc[t][mh] = mfma16_f16(r.w[t][u], r.xh[mh][u], acc[t][mh]);
        }
    }
}

// n_half = number of 16-row units of the weight matrix (N / 16); a workgroup owns HT of them.
// W8: the weights are E4M3 codes in units of [16 rows][64 k] -- lane l holds, for row l%16, the eight k
// values 8 (l/16) + 0..7 of the unit's first 32 k in bytes 0-7 and those of its second 32 k in bytes
// 8-15: one contiguous 1 KiB load per unit, two matrix-instruction operands after conversion.
template <int MODE, int HT, int U, int WAVES, bool W8, int MT = 1, int HALVES = 0>
__global__ __launch_bounds__(WAVES * 64) void gemm_half_kernel(const u32x4* __restrict__ Wp, const u32x4* __restrict__ Xhi,
                                                               int KB, int n_half, int ksplit, Epi p) {
    // 16-row halves of the activation rows: both of every slice, or only the first HALVES of them when no more
    // are in use (at most 16 rows of one slice, at most 48 of two): the rest would be loaded and multiplied for nothing
    static_assert(HALVES == 0 || (HALVES < 2 * MT && HALVES > 2 * (MT - 1)), "HALVES ends inside the last slice");
    constexpr int MH = HALVES ? HALVES : 2 * MT;
    constexpr int NI = HT * MH;  // (unit, row half) items of a workgroup
    __shared__ float red[WAVES][NI][4][64];
    __shared__ float lnp[MT][WAVES * 4 * 32];  // folded LayerNorm: the wavefronts' partial sums of the row statistics
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int grp = blockIdx.x / ksplit, ks = blockIdx.x % ksplit;
    const int mt = blockIdx.y * MT;  // first 32-row slice
    const size_t xstride = (size_t)KB * 64;
    constexpr int KU = W8 ? 2 : 1;       // 32-wide k ranges per loop step
    const int KP = KB / (2 * KU);        // loop steps over the whole of k
    const int parts = ksplit * WAVES, part = ks * WAVES + wave;
    const int kp0 = (int)(((long)part * KP) / parts), kp1 = (int)(((long)(part + 1) * KP) / parts);
    constexpr bool FOLDABLE = MODE == MODE_BIAS_RELU || MODE == MODE_QKV;
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
    constexpr int ITEMS = items_per_wave(NI, WAVES);  // item = wave + i*WAVES -> unit item/MH, row half item%MH
    // epilogue operands: requested right behind the first round of weight loads (see gemm_skinny_kernel)
    uint2 bias_w[ITEMS];
    float4 c1w[ITEMS], c2w[ITEMS], wsc[ITEMS];
    LnLoads lnl[MT];
    bool fold = false;
    int cur_len = 0;
    auto request_epilogue_operands = [&]() {
        fold = FOLDABLE && p.ln_stats != nullptr;
        if (fold) {
#pragma unroll
            for (int s2 = 0; s2 < MT; ++s2) ln_issue<WAVES>(lnl[s2], p, mt + s2, wave, lane);
        }
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int item = wave + i * WAVES, g = grp * HT + item / MH;
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
        cur_len = epilogue_len<MODE>(p);
    };
    f32x4 acc[HT][MH];
#pragma unroll
    for (int t = 0; t < HT; ++t)
#pragma unroll
        for (int mh = 0; mh < MH; ++mh) acc[t][mh] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto ln_partials = [&]() {
#pragma unroll
        for (int s2 = 0; s2 < MT; ++s2) ln_partial<WAVES>(lnl[s2], p, mt + s2, wave, lane, lnp[s2]);
    };
    int n = kp1 - kp0;
    if (n >= U) {
        HalfRegs<HT, U, W8, MH> ra;
        half_load<HT, U, W8, MH>(ra, w, xh, xstride);
        n -= U;
        request_epilogue_operands();
        // the statistics are used once the second round is on its way as well (first trip peeled off the loop)
        if (n >= U) {
            HalfRegs<HT, U, W8, MH> rb;
            half_load<HT, U, W8, MH>(rb, w, xh, xstride);
            n -= U;
            if (fold) ln_partials();
            half_mma<HT, U, W8, MH>(ra, acc);
            ra = rb;
        } else if (fold) {
            ln_partials();
        }
        while (n >= U) {
            HalfRegs<HT, U, W8, MH> rb;
            half_load<HT, U, W8, MH>(rb, w, xh, xstride);
            n -= U;
            half_mma<HT, U, W8, MH>(ra, acc);
            ra = rb;
        }
        half_mma<HT, U, W8, MH>(ra, acc);
    } else {
        request_epilogue_operands();
        if (fold) ln_partials();
    }
    for (; n > 0; --n) {
        HalfRegs<HT, 1, W8, MH> r1;
        half_load<HT, 1, W8, MH>(r1, w, xh, xstride);
        half_mma<HT, 1, W8, MH>(r1, acc);
    }
#pragma unroll
    for (int t = 0; t < HT; ++t)
#pragma unroll
        for (int mh = 0; mh < MH; ++mh)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[wave][t * MH + mh][r][lane] = acc[t][mh][r];
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
        // (selected, not indexed: an array indexed at run time would live in LDS, whose addressing
        // reads the dispatch packet -- microseconds, here in the tail of the kernel)
        const float2 mr0 = ln_finish<WAVES>(lnp[0], lane & 15, p), mr1 = ln_finish<WAVES>(lnp[0], 16 + (lane & 15), p);
        float2 mr2 = mr0, mr3 = mr1;
        if (MT == 2) {
            mr2 = ln_finish<WAVES>(lnp[MT - 1], lane & 15, p);
            mr3 = ln_finish<WAVES>(lnp[MT - 1], 16 + (lane & 15), p);
        }
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int rh = (wave + i * WAVES) % MH;
            const bool odd = rh & 1, second = rh >= 2;
            const float mean = second ? (odd ? mr3.x : mr2.x) : (odd ? mr1.x : mr0.x);
            const float rstd = second ? (odd ? mr3.y : mr2.y) : (odd ? mr1.y : mr0.y);
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
            const int item = wave + i * WAVES, g = grp * HT + item / MH;
            mrow[i] = mt * 32 + 16 * (item % MH) + (lane & 15);
            n0[i] = g * 16 + 4 * (lane >> 4);
            live[i] = item < NI && g < n_half && mrow[i] < p.M;
            rslot[i] = item % MH;
        }
        store_ln_tail<ITEMS, WAVES, 16, MT>(p, ksplit, ks, grp, (n_half + HT - 1) / HT, mt,
                                            16.f * (float)min(HT, n_half - grp * HT), v, mrow, n0, live, rslot);
        return;
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int item = wave + i * WAVES, g = grp * HT + item / MH;
        if (item >= NI || g >= n_half) continue;
        epilogue4<MODE>(p, mt * 32 + 16 * (item % MH) + (lane & 15), g * 16 + 4 * (lane >> 4), ks, v[i][0], v[i][1], v[i][2],
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
        const int q = row_seq(st, b, 1);  // outputs and the next input belong to the row's sequence
        const size_t at = (size_t)q * out_stride + (out_at_step ? st->step : 0);
        ids_out[at] = bi;
        lp_out[at] = bz - (mx + logf(sum));
        if (cur_ids) cur_ids[q] = bi;
    }
}

// Launch shapes are sized for the current device's CU count, or for the count a planner query names.
int g_cus_override = 0;
int plan_cus() { return g_cus_override > 0 ? g_cus_override : num_cus(); }

#ifndef HE_SKINNY_U
#define HE_SKINNY_U(NT) ((NT) <= 4 ? 4 : 2)
#endif
#ifndef HE_SKINNY_W8_MAXNT
#define HE_SKINNY_W8_MAXNT 2
#endif
// Host-side account of a MODE_STORE_LN launch: when `g_dry` is set the launchers below go through their choice of
// kernel variant and grid as usual, then record what that launch would index instead of launching it.
struct StoreFootprint { size_t scratch_floats; int cells; int stat_groups; int ksplit; };
StoreFootprint* g_dry = nullptr;
// grid: the launch's; items, waves: of the kernel variant chosen.  True if the launch is to be left out.
inline bool dry_run(const dim3& grid, int ksplit, int items, int waves) {
    if (!g_dry) return false;
    const int groups = grid.x / ksplit;
    g_dry->cells = groups * grid.y;
    g_dry->stat_groups = groups;
    g_dry->ksplit = ksplit;
    g_dry->scratch_floats = ksplit > 1 ? (size_t)g_dry->cells * ksplit * tail_floats_per_split(items, waves) : 0;
    return true;
}

template <int MODE, int NT>
void launch_skinny_nt(hipStream_t s, const void* Wp, const void* Xhi, int KB, int n_tiles,
                      int m_tiles, int ksplit, const Epi& p) {
    constexpr int U = HE_SKINNY_U(NT);
    dim3 grid(((n_tiles + NT - 1) / NT) * ksplit, m_tiles);
    if (MODE == MODE_LMHEAD && m_tiles > 1) grid.x = (grid.x + 7) / 8 * 8;  // see the kernel: slices of a tile group share an XCD
    // What bounds a wavefront is its serial chain of load rounds (K/16 blocks / wavefronts / U
    // rounds, about 1.7 us each under load): eight wavefronts halve the chain when K leaves each
    // of them two rounds (and their accumulators still fit in LDS for the final reduction).
    const bool eight = NT <= HE_SKINNY_W8_MAXNT && KB / (ksplit * 8) >= 2 * U;
    // Ask for more than half of a CU's LDS so that no two workgroups share a CU: with at most one
    // workgroup per CU the dispatcher has to spread a launch of <= #CUs workgroups evenly.
    constexpr size_t kWant = 84 * 1024;
    if (dry_run(grid, ksplit, items_per_wave(NT * 4, eight ? 8 : 4), eight ? 8 : 4)) return;
    if (eight) {
        constexpr size_t kStatic = (size_t)8 * NT * 16 * 64 * sizeof(float);
        const size_t pad = kStatic >= kWant ? 0 : kWant - kStatic;
        gemm_skinny_kernel<MODE, NT <= HE_SKINNY_W8_MAXNT ? NT : 1, U, 8><<<grid, 512, pad, s>>>(
            (const u32x4*)Wp, (const u32x4*)Xhi, KB, n_tiles, ksplit, p);
    } else {
        constexpr size_t kStatic = (size_t)4 * NT * 16 * 64 * sizeof(float);
        const size_t pad = kStatic >= kWant ? 0 : kWant - kStatic;
        gemm_skinny_kernel<MODE, NT, U, 4><<<grid, 256, pad, s>>>((const u32x4*)Wp, (const u32x4*)Xhi,
                                                                  KB, n_tiles, ksplit, p);
    }
}

template <int MODE, int HT, bool W8>
void launch_half_ht(hipStream_t s, const void* Wp, const void* Xhi, int KB, int n_half, int m_tiles,
                    int ksplit, const Epi& p) {
    // loads per wavefront and round: (HT + 4) U 16-byte loads with bf16 weights, (HT + 8) U with 8-bit ones
    // (with the activations' second term gone there are registers for deeper rounds at four to six units; three or
    // four blocks per round measured 1-3 % slower than two on the 13B shapes)
    constexpr int U = W8 ? (HT <= 3 ? 2 : 1) : (HT <= 3 ? 4 : 2);
    constexpr int KU = W8 ? 2 : 1;
    dim3 grid(((n_half + HT - 1) / HT) * ksplit, m_tiles);
    if constexpr (!W8 && HT <= 8) {  // (the accumulators of more units than that do not fit in LDS for the reduction)
        if (m_tiles == 2) {  // both 32-row slices in one workgroup: the weights are streamed once
            constexpr int U2 = HT <= 6 ? 2 : 1;
            constexpr size_t kWant2 = 84 * 1024;
            grid.y = 1;
            if (dry_run(grid, ksplit, items_per_wave(HT * (p.M <= 48 ? 3 : 4), 4), 4)) return;
            if (p.M <= 48) {  // the last 16 of the 64 rows are not in use
                constexpr size_t kStatic = (size_t)4 * HT * 3 * 4 * 64 * sizeof(float);
                const size_t pad = kStatic >= kWant2 ? 0 : kWant2 - kStatic;
                gemm_half_kernel<MODE, HT, U2, 4, false, 2, 3><<<grid, 256, pad, s>>>(
                    (const u32x4*)Wp, (const u32x4*)Xhi, KB, n_half, ksplit, p);
                return;
            }
            constexpr size_t kStatic = (size_t)4 * HT * 4 * 4 * 64 * sizeof(float);
            const size_t pad = kStatic >= kWant2 ? 0 : kWant2 - kStatic;
            gemm_half_kernel<MODE, HT, U2, 4, false, 2><<<grid, 256, pad, s>>>((const u32x4*)Wp, (const u32x4*)Xhi,
                                                                               KB, n_half, ksplit, p);
            return;
        }
    }
    // eight wavefronts have 256 registers each: three units with four rounds of operands twice over do not fit
    constexpr int U8 = (!W8 && HT == 3) ? 2 : U;
    const bool eight = HT <= 4 && (KB / (2 * KU)) / (ksplit * 8) >= 2 * U8;  // short chains per wavefront, as above
    constexpr size_t kWant = 84 * 1024;                                      // one workgroup per CU
    if constexpr (!W8) {
        if (m_tiles == 1 && p.M <= 16) {  // the second half of the 32 activation rows is not in use: leave it out
            if (dry_run(grid, ksplit, items_per_wave(HT, eight ? 8 : 4), eight ? 8 : 4)) return;
            if (eight) {
                constexpr size_t kStatic = (size_t)8 * HT * 4 * 64 * sizeof(float);
                const size_t pad = kStatic >= kWant ? 0 : kWant - kStatic;
                gemm_half_kernel<MODE, HT <= 4 ? HT : 2, U8, 8, false, 1, 1><<<grid, 512, pad, s>>>(
                    (const u32x4*)Wp, (const u32x4*)Xhi, KB, n_half, ksplit, p);
            } else {
                constexpr size_t kStatic = (size_t)4 * HT * 4 * 64 * sizeof(float);
                const size_t pad = kStatic >= kWant ? 0 : kWant - kStatic;
                gemm_half_kernel<MODE, HT, U, 4, false, 1, 1><<<grid, 256, pad, s>>>(
                    (const u32x4*)Wp, (const u32x4*)Xhi, KB, n_half, ksplit, p);
            }
            return;
        }
    }
    if (dry_run(grid, ksplit, items_per_wave(HT * 2, eight ? 8 : 4), eight ? 8 : 4)) return;
    if (eight) {
        constexpr size_t kStatic = (size_t)8 * HT * 2 * 4 * 64 * sizeof(float);
        const size_t pad = kStatic >= kWant ? 0 : kWant - kStatic;
        gemm_half_kernel<MODE, HT <= 4 ? HT : 2, U8, 8, W8><<<grid, 512, pad, s>>>(
            (const u32x4*)Wp, (const u32x4*)Xhi, KB, n_half, ksplit, p);
    } else {
        constexpr size_t kStatic = (size_t)4 * HT * 2 * 4 * 64 * sizeof(float);
        const size_t pad = kStatic >= kWant ? 0 : kWant - kStatic;
        gemm_half_kernel<MODE, HT, U, 4, W8><<<grid, 256, pad, s>>>((const u32x4*)Wp, (const u32x4*)Xhi,
                                                                    KB, n_half, ksplit, p);
    }
}

constexpr int kHalfMin = 2, kHalfMax = 10;  // 16-row units per workgroup the half-tile kernel is built for (8-bit: from 1)
constexpr int kHalfMax2 = 8;                // ... with two 32-row activation slices per workgroup

template <int MODE, bool W8>
void launch_half(hipStream_t s, const void* Wp, const void* Xhi, int KB, int n_half, int m_tiles, int ht,
                 int ksplit, const Epi& p) {
    switch (ht) {
        case 1:
            if constexpr (W8) { launch_half_ht<MODE, 1, W8>(s, Wp, Xhi, KB, n_half, m_tiles, ksplit, p); break; }
            [[fallthrough]];
        case 2: launch_half_ht<MODE, 2, W8>(s, Wp, Xhi, KB, n_half, m_tiles, ksplit, p); break;
        case 3: launch_half_ht<MODE, 3, W8>(s, Wp, Xhi, KB, n_half, m_tiles, ksplit, p); break;
        case 4: launch_half_ht<MODE, 4, W8>(s, Wp, Xhi, KB, n_half, m_tiles, ksplit, p); break;
        case 5: launch_half_ht<MODE, 5, W8>(s, Wp, Xhi, KB, n_half, m_tiles, ksplit, p); break;
        case 6: launch_half_ht<MODE, 6, W8>(s, Wp, Xhi, KB, n_half, m_tiles, ksplit, p); break;
        case 7: launch_half_ht<MODE, 7, W8>(s, Wp, Xhi, KB, n_half, m_tiles, ksplit, p); break;
        case 8: launch_half_ht<MODE, 8, W8>(s, Wp, Xhi, KB, n_half, m_tiles, ksplit, p); break;
        case 9: launch_half_ht<MODE, 9, W8>(s, Wp, Xhi, KB, n_half, m_tiles, ksplit, p); break;
        default: launch_half_ht<MODE, 10, W8>(s, Wp, Xhi, KB, n_half, m_tiles, ksplit, p); break;
    }
}

// nt weight tiles per workgroup (1..8)
template <int MODE>
void launch_skinny(hipStream_t s, const void* Wp, const void* Xhi, int KB, int n_tiles, int m_tiles,
                   int nt, int ksplit, const Epi& p) {
    switch (nt) {
        case 1: launch_skinny_nt<MODE, 1>(s, Wp, Xhi, KB, n_tiles, m_tiles, ksplit, p); break;
        case 2: launch_skinny_nt<MODE, 2>(s, Wp, Xhi, KB, n_tiles, m_tiles, ksplit, p); break;
        case 3: launch_skinny_nt<MODE, 3>(s, Wp, Xhi, KB, n_tiles, m_tiles, ksplit, p); break;
        case 4: launch_skinny_nt<MODE, 4>(s, Wp, Xhi, KB, n_tiles, m_tiles, ksplit, p); break;
        case 5: launch_skinny_nt<MODE, 5>(s, Wp, Xhi, KB, n_tiles, m_tiles, ksplit, p); break;
        case 6: launch_skinny_nt<MODE, 6>(s, Wp, Xhi, KB, n_tiles, m_tiles, ksplit, p); break;
        case 7: launch_skinny_nt<MODE, 7>(s, Wp, Xhi, KB, n_tiles, m_tiles, ksplit, p); break;
        default: launch_skinny_nt<MODE, 8>(s, Wp, Xhi, KB, n_tiles, m_tiles, ksplit, p); break;
    }
}

// Tiles per workgroup for a GEMM whose epilogue needs the whole sum in one workgroup: the
// smallest count that fits all workgroups on the chip at once (one per CU), at most 8.
int skinny_nt_fused(int n_tiles, int m_tiles) {
    const int cus = plan_cus();
    int nt = (n_tiles * m_tiles + cus - 1) / cus;
    return nt < 1 ? 1 : (nt > 8 ? 8 : nt);
}

}  // namespace

// ------------------------------------------------------------------ launchers

// Shape of a decode-shaped STORE GEMM: nt tiles per workgroup and ks k-splits such that about one
// workgroup lands on every CU.  Four tiles per workgroup (activation blocks reused four times)
// as long as each wavefront keeps 8 k-blocks, else two tiles and half the splits.  (Two tiles and
// three splits for the 5120x5120 out-projection measured 2 us slower than four and six, more
// than the LayerNorm that adds up the partial sums gained.)
static void store_shape(int N, int K, int* nt, int* ks) {
    const int tiles = (N + 31) / 32, kb = K / 16, cus = plan_cus();
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
    const int n_tiles = (N + 31) / 32, m_tiles = (M + 31) / 32, cus = plan_cus();
    GemmPlan g{false, skinny_nt_fused(n_tiles, m_tiles), 1};
    if (m_tiles > 2 || N % 16) return g;
    const int n_half = N / 16, ht = (n_half + cus - 1) / cus;
    if (m_tiles == 2) {  // two row slices per workgroup (16-row-unit kernel only): the weights are streamed once
        if (ht >= kHalfMin && ht <= kHalfMax2) g = GemmPlan{true, ht, 1};
        return g;
    }
    // up to 16 rows the 16-row-unit kernel also leaves out the unused half of the activation panel: it wins ties
    if (ht >= kHalfMin && ht <= kHalfMax && (16 * ht < 32 * g.per_wg || (M <= 16 && 16 * ht == 32 * g.per_wg)))
        g = GemmPlan{true, ht, 1};
    return g;
}

// capacity: floats the k-split scratch can hold (0 = not checked)
//
// Cost of a one-slice plan, in microseconds, fitted to launches of the 13B and 6.7B shapes: what the most loaded
// workgroup moves (its weight rows and the activation rows over its k range, at the ~48 GB/s one CU
// sustains while all stream; never less than the whole matrix takes at the HBM rate) plus the tail after the
// stream: ~0.6 us per k-split whose partial sums the last arriver waits for and reads back, ~0.2 us per quad of
// outputs a thread finishes.  (Balance alone, the earlier criterion, chose four 32-row tiles and six splits on
// 5120x5120 and 5120x20480; five 16-row units and four splits move 12 % more bytes per workgroup and run 1-2 us
// faster; on 4096x4096 four units and four splits run 3.4 us faster than four tiles and eight splits.)
static double store_cost_us(int N, int K, int rows, int items, int ks, int wgs, int cus, double act = 64.0) {
    // weight rows and the activation panel (act bytes per k: 32 rows of halves) at 48 GB/s into the CU
    const double per_cu = (double)K / ks * (2.0 * rows + act) / 48e3;
    // the whole matrix at 6.5 TB/s; CUs left without a workgroup request nothing, and the stream slows by about
    // half their share (9216x36864: 216 workgroups on 256 CUs ran 8 % slower than 256)
    const double idle = wgs < cus ? 1.0 - (double)wgs / cus : 0.0;
    const double hbm = 2.0 * N * K / 6.5e6 * (1.0 + 0.5 * idle);
    return (per_cu > hbm ? per_cu : hbm) + 0.2 * items + 0.6 * ks;
}

static GemmPlan plan_store(int M, int N, int K, size_t capacity) {
    GemmPlan g{false, 0, 0};
    bf16_store_shape(M, N, K, &g.per_wg, &g.ks);
    const int m_tiles = (M + 31) / 32;
    if (m_tiles > 2 || N % 16) return g;
    const int n_half = N / 16, kb = K / 16, cus = plan_cus();
    // two row slices: only the 16-row-unit kernel takes both in one workgroup, so any such plan beats the rest;
    // among them the one with the fewest weight rows x k share on a workgroup
    double best = m_tiles == 2 ? 1e30
                               : store_cost_us(N, K, g.per_wg * 32, g.per_wg, g.ks,
                                               ((N + 31) / 32 + g.per_wg - 1) / g.per_wg * g.ks, cus);
    const int mh = 2 * m_tiles;
    for (int ht = m_tiles == 2 ? kHalfMax2 : kHalfMax; ht >= kHalfMin; --ht) {
        const int groups = (n_half + ht - 1) / ht;
        int ks = cus / groups;
        if (ks < 1) continue;
        if (ks > 8) ks = 8;
        while (ks > 1 && kb / (ks * 4) < 8) --ks;
        // scratch the kernel will index: groups x splits x (items rounded up to the wavefronts) x 256 words
        if (capacity && (size_t)groups * ks * (size_t)(mh * ht + 7) * 256 > capacity) continue;
        const double cost = m_tiles == 2 ? (double)ht * 16 / ks : store_cost_us(N, K, ht * 16, (ht * (M <= 16 ? 1 : mh) + 3) / 4, ks, groups * ks, cus, M <= 16 ? 32.0 : 64.0);
        if (cost < best) { best = cost; g = GemmPlan{true, ht, ks}; }
    }
    return g;
}

// 8-bit weights: always the 16-row-unit kernel
static GemmPlan plan_fused_w8(int N) {
    const int n_half = N / 16, cus = plan_cus();
    int ht = (n_half + cus - 1) / cus;
    if (ht > kHalfMax) ht = kHalfMax;
    return GemmPlan{true, ht < 1 ? 1 : ht, 1};
}

static GemmPlan plan_store_w8(int N, int K, size_t capacity) {
    const int n_half = N / 16, kq = K / 64, cus = plan_cus();
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
    g_cus_override = cus;
    const GemmPlan g = store ? plan_store(M, N, K, capacity) : plan_fused(M, N);
    g_cus_override = 0;
    *unit_rows = g.half ? 16 : 32;
    *per_wg = g.per_wg;
    *ks = g.ks;
}

// What the MODE_STORE_LN launch of this shape indexes (host logic only): floats of k-split scratch, arrival
// counters, column groups of statistics per 32-row slice, and its k-split.
void bf16_store_footprint(int M, int N, int K, size_t capacity, int w8, int cus, size_t* scratch_floats,
                          size_t* need_floats, int* cells, int* stat_groups, int* ksplit) {
    StoreFootprint f{};
    g_cus_override = cus;
    bf16_gemm_args a{};
    a.out_capacity = capacity;
    float one = 1.f;
    if (w8) a.wscale = &one;  // (never read: nothing is launched)
    g_dry = &f;
    bf16_gemm_skinny(nullptr, EPI_STORE_LN, nullptr, nullptr, M, N, K, 0, a);
    g_dry = nullptr;
    *need_floats = bf16_store_need(M, N, K, capacity, w8);
    g_cus_override = 0;
    *scratch_floats = f.scratch_floats;
    *cells = f.cells;
    *stat_groups = f.stat_groups;
    *ksplit = f.ksplit;
}

void bf16_store_plan(int M, int N, int K, size_t capacity, int* group_cols, int* ks) {
    const GemmPlan g = plan_store(M, N, K, capacity);
    *group_cols = g.per_wg * (g.half ? 16 : 32);
    *ks = g.ks;
}

// Floats of k-split scratch the EPI_STORE_LN launch of this shape may index (an upper bound: per column
// group, row-slice pair and split, one 256-float run per item, items rounded up to whole wavefronts).
size_t bf16_store_need(int M, int N, int K, size_t capacity, int w8) {
    const int m_tiles = (M + 31) / 32;
    if (w8) {
        const GemmPlan g = plan_store_w8(N, K, capacity);
        const size_t groups = (size_t)(N / 16 + g.per_wg - 1) / g.per_wg;
        return groups * m_tiles * g.ks * (size_t)(2 * g.per_wg + 7) * 256;
    }
    const GemmPlan g = plan_store(M, N, K, capacity);
    if (g.half) {
        const size_t groups = (size_t)(N / 16 + g.per_wg - 1) / g.per_wg;
        const int grid_y = m_tiles == 2 ? 1 : m_tiles, mh = m_tiles == 2 ? 4 : 2;
        return groups * grid_y * g.ks * (size_t)(mh * g.per_wg + 7) * 256;
    }
    const size_t groups = (size_t)((N + 31) / 32 + g.per_wg - 1) / g.per_wg;
    return groups * m_tiles * g.ks * (size_t)(4 * g.per_wg + 7) * 256;
}

void bf16_gemm_skinny(hipStream_t s, int mode, const void* Wp, const void* Xhi, int M, int N, int K,
                      int ksplit, const bf16_gemm_args& a) {
    (void)ksplit;
    const Epi p = make_epi(M, N, a);
    const int KB = K / 16, n_tiles = (N + 31) / 32, m_tiles = (M + 31) / 32;
    if (a.wscale) {  // 8-bit weights: Wp holds E4M3 units; one row slice only
        if (mode == EPI_STORE_LN) {
            const GemmPlan g = plan_store_w8(N, K, a.out_capacity);
            launch_half<MODE_STORE_LN, true>(s, Wp, Xhi, KB, N / 16, m_tiles, g.per_wg, g.ks, p);
        } else {
            const GemmPlan g = plan_fused_w8(N);
            if (mode == EPI_BIAS_RELU) launch_half<MODE_BIAS_RELU, true>(s, Wp, Xhi, KB, N / 16, m_tiles, g.per_wg, 1, p);
            else launch_half<MODE_QKV, true>(s, Wp, Xhi, KB, N / 16, m_tiles, g.per_wg, 1, p);
        }
        return;
    }
    if (mode == EPI_STORE_LN) {  // the k-split is the one bf16_store_plan reports for this shape
        const GemmPlan g = plan_store(M, N, K, a.out_capacity);
        if (g.half) launch_half<MODE_STORE_LN, false>(s, Wp, Xhi, KB, N / 16, m_tiles, g.per_wg, g.ks, p);
        else launch_skinny<MODE_STORE_LN>(s, Wp, Xhi, KB, n_tiles, m_tiles, g.per_wg, g.ks, p);
        return;
    }
    const GemmPlan g = plan_fused(M, N);
    if (mode == EPI_BIAS_RELU) {
        if (g.half) launch_half<MODE_BIAS_RELU, false>(s, Wp, Xhi, KB, N / 16, m_tiles, g.per_wg, 1, p);
        else launch_skinny<MODE_BIAS_RELU>(s, Wp, Xhi, KB, n_tiles, m_tiles, g.per_wg, 1, p);
    } else {
        if (g.half) launch_half<MODE_QKV, false>(s, Wp, Xhi, KB, N / 16, m_tiles, g.per_wg, 1, p);
        else launch_skinny<MODE_QKV>(s, Wp, Xhi, KB, n_tiles, m_tiles, g.per_wg, 1, p);
    }
}

void bf16_lm_head(hipStream_t s, const void* Wp, const void* Xhi, int B, int V, int K,
                  const he_dev_state* st, float* logits_opt, float* stats, int* stats_idx, int32_t* ids_out,
                  float* lp_out, int out_stride, int out_at_step, int32_t* cur_ids, const bf16_gemm_args* fold) {
    Epi p{};
    if (fold) p = make_epi(B, V, *fold);
    p.M = B; p.N = V; p.st = st; p.logits = logits_opt; p.stats = stats; p.stats_idx = stats_idx;
    p.n_tiles = (V + 31) / 32;
    const int m_tiles = (B + 31) / 32;
    launch_skinny<MODE_LMHEAD>(s, Wp, Xhi, K / 16, p.n_tiles, m_tiles, skinny_nt_fused(p.n_tiles, m_tiles), 1, p);
    lm_reduce_kernel<<<B, 256, 0, s>>>(stats, stats_idx, p.n_tiles, st, ids_out, lp_out, out_stride, out_at_step,
                                       cur_ids);
}

