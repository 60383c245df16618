// bf16 path: LayerNorm kernels, and the producer side of LayerNorms folded into the next GEMM.
#include "bf16_common.h"

using namespace he_bf16;

namespace {

// ----------------------------------------------------------------- LayerNorm (+ residual update)
//
// Row `src = m*in_mul + in_add`: r += sum of k-split partials + bias (fixed order),
// written back when asked; a = LayerNorm(r) is emitted as tiled half blocks.
__global__ __launch_bounds__(1024) void ln_blocks_kernel(float* __restrict__ r, const float* __restrict__ part,
                                                        int ksplit, size_t part_split,
                                                        const bf16_t* __restrict__ pbias,
                                                        const bf16_t* __restrict__ gamma,
                                                        const bf16_t* __restrict__ beta, u32x4* __restrict__ a,
                                                        int H, float eps, int in_mul, int in_add, int writeback,
                                                        int split_col) {
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
                if (k > 0 && 4 * i < split_col) break;  // columns before split_col have one whole sum
                const float4 y = *reinterpret_cast<const float4*>(part + (size_t)k * part_split + src * H + 4 * i);
                v.x += y.x; v.y += y.y; v.z += y.z; v.w += y.w;
            }
            const uint2 bb = *reinterpret_cast<const uint2*>(pbias + 4 * i);
            v.x += bf_lo(bb.x); v.y += bf_hi(bb.x);
            v.z += bf_lo(bb.y); v.w += bf_hi(bb.y);
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
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float e0 = (row[k0 + 2 * j] - mean) * rstd * bf_lo(gw[j]) + bf_lo(bw[j]);
            const float e1 = (row[k0 + 2 * j + 1] - mean) * rstd * bf_hi(gw[j]) + bf_hi(bw[j]);
            o[j] = pack2(e0, e1);
        }
        a[block_slot(m, k0, KB)] = u32x4{o[0], o[1], o[2], o[3]};
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
                                                      int H, float eps, int in_mul, int in_add, int writeback,
                                                      int rows, int split_col) {
    constexpr int NW = THREADS / 64;
    __shared__ float red[2][NW];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int m = blockIdx.x;
    if (THREADS == 256) {
        // Many rows: a row writes 16-byte slots of the 32-row blocks, 512 bytes apart, and the 32 rows of a block
        // together fill whole cache lines.  Workgroups go round the eight XCDs by index, so the rows of one block
        // are kept on one XCD (block b on XCD b mod 8): its L2 then holds complete lines to write back.
        const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
        m = (((j >> 5) << 3) + x) * 32 + (j & 31);
        if (m >= rows) return;  // the whole workgroup: the grid is padded to eight blocks
    }
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
    if (part && ksplit <= 2) {  // the usual cases, with every load of the row requested before the first is used
        float4 y0[NV], y1[NV];
        uint2 pb[NV];
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = threadIdx.x + j * THREADS;
            y0[j] = y1[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            pb[j] = make_uint2(0, 0);
            if (i >= nq) continue;
            y0[j] = *reinterpret_cast<const float4*>(part + src * H + 4 * i);
            // (columns before split_col have one whole sum; a multiple of 256 or 320)
            if (ksplit == 2 && 4 * i >= split_col) y1[j] = *reinterpret_cast<const float4*>(part + part_split + src * H + 4 * i);
            pb[j] = *reinterpret_cast<const uint2*>(pbias + 4 * i);
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = threadIdx.x + j * THREADS;
            if (i >= nq) continue;
            v[j].x += (y0[j].x + y1[j].x) + bf_lo(pb[j].x);
            v[j].y += (y0[j].y + y1[j].y) + bf_hi(pb[j].x);
            v[j].z += (y0[j].z + y1[j].z) + bf_lo(pb[j].y);
            v[j].w += (y0[j].w + y1[j].w) + bf_hi(pb[j].y);
            if (writeback) *reinterpret_cast<float4*>(r + src * H + 4 * i) = v[j];
        }
    } else if (part) {
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
            v[j].x += acc.x + bf_lo(pb.x);
            v[j].y += acc.y + bf_hi(pb.x);
            v[j].z += acc.z + bf_lo(pb.y);
            v[j].w += acc.w + bf_hi(pb.y);
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
        const float e0 = (v[j].x - mean) * rstd * bf_lo(gg[j].x) + bf_lo(bb[j].x);
        const float e1 = (v[j].y - mean) * rstd * bf_hi(gg[j].x) + bf_hi(bb[j].x);
        const float e2 = (v[j].z - mean) * rstd * bf_lo(gg[j].y) + bf_lo(bb[j].y);
        const float e3 = (v[j].w - mean) * rstd * bf_hi(gg[j].y) + bf_hi(bb[j].y);
        const int k0 = 4 * i;  // four values: half of a 16-byte slot
        const size_t slot = block_slot(m, k0 & ~7, KB);
        reinterpret_cast<uint2*>(a + slot)[(k0 >> 2) & 1] = make_uint2(pack2(e0, e1), pack2(e2, e3));
    }
}

// ----------------------------------------------------------------- LayerNorm folded into the next GEMM (decode rows)
//
// For the few rows of a decode step a LayerNorm kernel of its own is all latency.  Instead
//   W LN(x) + b = rstd * (W (gamma . x) - mean * (W gamma)) + W beta + b,
// so the kernel that produces x (the embedding below, or the out-projection / FC2 GEMM
// through its last-arriving workgroup) writes gamma . x as half blocks plus per-column-
// group statistics of x, the consuming GEMM multiplies those blocks by the unchanged
// weights and applies mean and rstd in its epilogue, and W gamma, W beta are vectors computed
// once per weight update.

// Row m of a decode step: x = tok_emb[id] + pos_emb[cur_len + pos_offset]; one wavefront per
// (column group, row), four columns per lane (gw <= 256).
__global__ __launch_bounds__(64) void embed_ln_kernel(const int32_t* __restrict__ ids, int id_stride,
                                                      const bf16_t* __restrict__ tok, const bf16_t* __restrict__ pos,
                                                      const he_dev_state* __restrict__ st, int V, int pos_offset,
                                                      int H, int gw, int groups, const bf16_t* __restrict__ gamma,
                                                      float* __restrict__ r, u32x4* __restrict__ xb,
                                                      float2* __restrict__ stats) {
    const int g = blockIdx.x, m = blockIdx.y, lane = threadIdx.x;
    const int b = row_seq(st, m, 1);  // one row per running sequence here
    int id = ids[(size_t)b * id_stride];
    id = id < 0 ? 0 : (id >= V ? V - 1 : id);
    const size_t prow = (size_t)(seq_len(st, b) + pos_offset);
    const int cols = min(gw, H - g * gw), c0 = g * gw + 4 * lane;
    const bool live = 4 * lane < cols;
    float x0 = 0.f, x1 = 0.f, x2 = 0.f, x3 = 0.f;
    if (live) {
        const uint2 t = *reinterpret_cast<const uint2*>(tok + (size_t)id * H + c0);
        const uint2 q = *reinterpret_cast<const uint2*>(pos + prow * H + c0);
        const uint2 gg = *reinterpret_cast<const uint2*>(gamma + c0);
        x0 = bf_lo(t.x) + bf_lo(q.x);
        x1 = bf_hi(t.x) + bf_hi(q.x);
        x2 = bf_lo(t.y) + bf_lo(q.y);
        x3 = bf_hi(t.y) + bf_hi(q.y);
        *reinterpret_cast<float4*>(r + (size_t)m * H + c0) = make_float4(x0, x1, x2, x3);
        const size_t slot = block_slot(m, c0 & ~7, H >> 4);
        reinterpret_cast<uint2*>(xb + slot)[(c0 >> 2) & 1] =
            make_uint2(pack2(x0 * bf_lo(gg.x), x1 * bf_hi(gg.x)), pack2(x2 * bf_lo(gg.y), x3 * bf_hi(gg.y)));
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
            const float w0 = half_lo(ww[j]), w1 = half_hi(ww[j]);
            a1 = fmaf(w0, bf_lo(gg[j]), a1);
            a1 = fmaf(w1, bf_hi(gg[j]), a1);
            a2 = fmaf(w0, bf_lo(bb[j]), a2);
            a2 = fmaf(w1, bf_hi(bb[j]), a2);
        }
    }
    a1 += __shfl_xor(a1, 32);
    a2 += __shfl_xor(a2, 32);
    if (lane < 32) {  // rows past the matrix are zero blocks: their entries come out zero
        c1[tile * 32 + lane] = a1;
        c2[tile * 32 + lane] = a2;
    }
}

// Rows b*S + S-1 (each sequence's last prompt row) of two [B*S][H] float arrays -> rows b of two [B][H] arrays.
__global__ __launch_bounds__(256) void gather_last_rows_kernel(const float* __restrict__ r, const float* __restrict__ q,
                                                               float* __restrict__ r_out, float* __restrict__ q_out, int S,
                                                               int H) {
    const size_t src = ((size_t)blockIdx.x * S + S - 1) * H, dst = (size_t)blockIdx.x * H;
    for (int i = threadIdx.x; i < H / 4; i += 256) {
        reinterpret_cast<float4*>(r_out + dst)[i] = reinterpret_cast<const float4*>(r + src)[i];
        reinterpret_cast<float4*>(q_out + dst)[i] = reinterpret_cast<const float4*>(q + src)[i];
    }
}

}  // namespace

// ------------------------------------------------------------------ launchers

void bf16_gather_last_rows(hipStream_t s, const float* r, const float* q, float* r_out, float* q_out, int B, int S, int H) {
    gather_last_rows_kernel<<<B, 256, 0, s>>>(r, q, r_out, q_out, S, H);
}

void bf16_embed_ln(hipStream_t s, const int32_t* ids, int id_stride, const void* tok, const void* pos,
                   const he_dev_state* st, int B, int H, int V, int pos_offset, int gw, const void* gamma, float* r,
                   void* x_blocks, float* stats) {
    const int groups = (H + gw - 1) / gw;
    embed_ln_kernel<<<dim3(groups, B), 64, 0, s>>>(ids, id_stride, (const bf16_t*)tok, (const bf16_t*)pos, st, V,
                                                   pos_offset, H, gw, groups, (const bf16_t*)gamma, r,
                                                   (u32x4*)x_blocks, (float2*)stats);
}

void bf16_wvec(hipStream_t s, const void* Wp, int N, int K, const void* gamma, const void* beta, float* c1, float* c2) {
    const int n_tiles = (N + 31) / 32;
    wvec_kernel<<<(n_tiles + 3) / 4, 256, 0, s>>>((const u32x4*)Wp, K / 16, n_tiles, (const bf16_t*)gamma,
                                                  (const bf16_t*)beta, c1, c2);
}

void bf16_ln(hipStream_t s, float* r, const float* part, int ksplit, size_t part_split, const void* pbias,
             const void* gamma, const void* beta, void* a_blocks, int rows, int H, float eps, int in_mul, int in_add,
             int writeback, int split_col) {
    if (ksplit != 2) split_col = 0;  // (only the two-range form knows partly cut rows)
    const int nv = (H / 4 + 1023) / 1024, nv256 = (H / 4 + 255) / 256;
#define HE_LN_ROW(NV, T)                                                                                                \
    ln_row_kernel<NV, T><<<(T == 256 ? (rows + 255) / 256 * 256 : rows), T, 0, s>>>(                                    \
        r, part, ksplit, part_split, (const bf16_t*)pbias, (const bf16_t*)gamma, (const bf16_t*)beta, (u32x4*)a_blocks, \
        H, eps, in_mul, in_add, writeback, rows, split_col)
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
        H, eps, in_mul, in_add, writeback, split_col);
}

