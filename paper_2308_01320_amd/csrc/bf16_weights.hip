// bf16 path: weight preparation -- the caller's bf16 matrices converted to IEEE half and tiled into MFMA
// operand blocks (optionally with low-rank adapters folded in), and 8-bit E4M3 row quantisation.
#include "bf16_common.h"

using namespace he_bf16;

namespace {

// ----------------------------------------------------------------- weight tiling

// eight bf16 values -> eight halves: exact for magnitudes 2^-14 .. 65504 (8 significant bits into 11), nearest
// multiple of 2^-24 (ties to even) below that
__device__ __forceinline__ u32x4 bf16x8_to_half(const u32x4& w) {
    return u32x4{pack2(bf_lo(w.x), bf_hi(w.x)), pack2(bf_lo(w.y), bf_hi(w.y)), pack2(bf_lo(w.z), bf_hi(w.z)),
                 pack2(bf_lo(w.w), bf_hi(w.w))};
}
// two floats -> two bf16 in one word, round to nearest even (the LoRA merge rounds to the model's own format)
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) { return f32x2_to_bf16x2(lo, hi); }

__global__ void tile_rows_kernel(const bf16_t* __restrict__ src, u32x4* __restrict__ dst, int R, int K, size_t total) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int KB = K >> 4;
    const int lane = (int)(idx & 63);
    const int kb = (int)((idx >> 6) % KB);
    const int rt = (int)((idx >> 6) / KB);
    const int r = rt * 32 + (lane & 31), k = kb * 16 + (lane >> 5) * 8;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (r < R) v = bf16x8_to_half(*reinterpret_cast<const u32x4*>(src + (size_t)r * K + k));
    dst[idx] = v;
}

// The same with a low-rank adapter folded in: dst = tiled half(bf16(W + scale * B A)), A [rank, K], B [R, rank].
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
                const float p0 = b * bf_lo(aw[i]), p1 = b * bf_hi(aw[i]);
                t[2 * i] = t[2 * i] + p0;
                t[2 * i + 1] = t[2 * i + 1] + p1;
            }
        }
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float s0 = scale * t[2 * i], s1 = scale * t[2 * i + 1];  // plain operators: the pragma above covers them
            const float lo = bf_lo(ww[i]) + s0;
            const float hi = bf_hi(ww[i]) + s1;
            o[i] = pack2_bf16(lo, hi);  // the merged weight is a bf16 value ...
        }
        v = bf16x8_to_half(u32x4{o[0], o[1], o[2], o[3]});  // ... held as a half like every other weight
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
            amax = fmaxf(amax, fabsf(bf_lo(w[j])));
            amax = fmaxf(amax, fabsf(bf_hi(w[j])));
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
        f[2 * j] = bf_lo(w[j]) * inv_scale;
        f[2 * j + 1] = bf_hi(w[j]) * inv_scale;
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

// units -> the half 32x16 blocks the tiled GEMMs read (a dequantised weight q 2^e has four significant bits: exact
// as a half down to 2^-24, which only rows whose largest weight is below 448 * 2^-15 = 0.014 can undercut)
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

