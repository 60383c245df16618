// Plain kernels: the f32 path of the engine (and, instantiated for bf16 storage,
// a slow comparator for the tuned bf16 kernels).  One obvious kernel per step of
// the decoder; activations are float, row-major [rows, features].
#include "he_common.h"
#include "kernels.h"

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float block_sum(float v, float* red) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < nw; ++i) t += red[i];
    return t;
}

__device__ __forceinline__ float block_max(float v, float* red) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = red[0];
    for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
    return t;
}

// Row m = b*S + t:  x[m,:] = tok_emb[ids[b*id_stride + t],:] + pos_emb[cur_len + t + pos_offset,:]
template <typename ST>
__global__ void embed_kernel(const int32_t* __restrict__ ids, int id_stride, const ST* __restrict__ tok,
                             const ST* __restrict__ pos, float* __restrict__ x, const he_dev_state* __restrict__ st,
                             int S, int H, int V, int pos_offset) {
    const int m = blockIdx.x, b = row_seq(st, m, S), t = m % S - row_pad(st, b);
    if (t < 0) {  // a padding row: not a token, nothing downstream uses it
        for (int i = threadIdx.x; i < H; i += blockDim.x) x[(size_t)m * H + i] = 0.f;
        return;
    }
    int id = ids[(size_t)b * id_stride + (m % S)];
    id = id < 0 ? 0 : (id >= V ? V - 1 : id);  // out-of-range ids are clamped, never read out of bounds
    const size_t p = (size_t)(seq_len(st, b) + t + pos_offset);
    for (int i = threadIdx.x; i < H; i += blockDim.x)
        x[(size_t)m * H + i] = ld_f32(tok, (size_t)id * H + i) + ld_f32(pos, p * H + i);
}

// Row `row = m*in_mul + in_add` of the residual stream: r += y + bias (when y is given,
// written back when writeback), then a[m,:] = LayerNorm(r).
template <typename ST>
__global__ void ln_kernel(float* __restrict__ r, const float* __restrict__ y, const ST* __restrict__ ybias,
                          const ST* __restrict__ gamma, const ST* __restrict__ beta, float* __restrict__ a, int H,
                          float eps, int in_mul, int in_add, int writeback) {
    __shared__ float red[8];
    const int m = blockIdx.x;
    const size_t row = (size_t)m * in_mul + in_add;
    float* rr = r + row * H;
    float s = 0.f;
    for (int i = threadIdx.x; i < H; i += blockDim.x) {
        float v = rr[i];
        if (y) v += y[row * H + i] + ld_f32(ybias, i);
        if (y && writeback) rr[i] = v;
        a[(size_t)m * H + i] = v;  // staged; normalised below
        s += v;
    }
    const float mean = block_sum(s, red) / H;
    float q = 0.f;
    for (int i = threadIdx.x; i < H; i += blockDim.x) {
        const float dlt = a[(size_t)m * H + i] - mean;
        q += dlt * dlt;
    }
    const float rstd = 1.0f / sqrtf(block_sum(q, red) / H + eps);
    for (int i = threadIdx.x; i < H; i += blockDim.x) {
        const float v = a[(size_t)m * H + i];
        a[(size_t)m * H + i] = (v - mean) * rstd * ld_f32(gamma, i) + ld_f32(beta, i);
    }
}

// C[m,n] = sum_k A[m,k] W[n,k]; 64x64 tile, 4x4 outputs per thread, K staged 16 at a time.
template <typename ST>
__global__ void gemm_kernel(const float* __restrict__ A, const ST* __restrict__ W, const ST* __restrict__ bias, int M,
                            int N, int K, int epi, float* __restrict__ out, float* __restrict__ kv,
                            const he_dev_state* __restrict__ st, int S, int layer, int H, int n_heads, int max_batch,
                            int max_seq, float qscale) {
    __shared__ float As[16][65];
    __shared__ float Ws[16][65];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int i = threadIdx.x; i < 64 * 16; i += kThreads) {
            const int r = i >> 4, c = i & 15;
            As[c][r] = (m0 + r < M && k0 + c < K) ? A[(size_t)(m0 + r) * K + k0 + c] : 0.f;
            Ws[c][r] = (n0 + r < N && k0 + c < K) ? ld_f32(W, (size_t)(n0 + r) * K + k0 + c) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            float av[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { av[i] = As[c][ty * 4 + i]; wv[i] = Ws[c][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
    const int d = H / n_heads;
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = acc[i][j];
            if (epi == EPI_STORE) {
                out[(size_t)m * N + n] = v;
            } else if (epi == EPI_BIAS_RELU) {
                v += ld_f32(bias, n);
                out[(size_t)m * N + n] = v > 0.f ? v : 0.f;
            } else {  // EPI_QKV: q scaled to `out`, k and v appended to the cache at cur_len + t
                v += ld_f32(bias, n);
                if (n < H) {
                    out[(size_t)m * H + n] = v * qscale;
                } else {
                    const int which = (n >= 2 * H), c = n - (which ? 2 * H : H);
                    const int b = m / S, tr = m % S - row_pad(st, b);  // padding rows append nothing
                    if (tr >= 0)
                        st_val(kv, kv_index(layer, which, b, c / d, seq_len(st, b) + tr, max_batch, n_heads, max_seq, d) + (c % d), v);
                }
            }
        }
    }
}

// One block per (row m, head h): scores over keys 0..cur_len+t, softmax, weighted sum of values.
__global__ void attn_kernel(const float* __restrict__ q, const float* __restrict__ kv, float* __restrict__ o,
                            const he_dev_state* __restrict__ st, int S, int layer, int H, int n_heads, int max_batch,
                            int max_seq) {
    extern __shared__ float smem[];
    __shared__ float red[8];
    const int d = H / n_heads;
    float* qs = smem;      // [d]
    float* sc = smem + d;  // [max_seq]
    const int m = blockIdx.x, h = blockIdx.y;
    const int b = m / S, nkeys = seq_len(st, b) + (m % S) - row_pad(st, b) + 1;
    if (nkeys <= 0 || seq_done(st, b)) {  // a padding row, or a sequence that has ended: nothing reads this output
        for (int e = threadIdx.x; e < d; e += blockDim.x) o[(size_t)m * H + h * d + e] = 0.f;
        return;
    }
    const float* Kp = kv + kv_index(layer, 0, b, h, 0, max_batch, n_heads, max_seq, d);
    const float* Vp = kv + kv_index(layer, 1, b, h, 0, max_batch, n_heads, max_seq, d);
    for (int e = threadIdx.x; e < d; e += blockDim.x) qs[e] = q[(size_t)m * H + h * d + e];
    __syncthreads();
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < nkeys; j += blockDim.x) {
        float s = 0.f;
        for (int e = 0; e < d; ++e) s = fmaf(qs[e], ld_f32(Kp, (size_t)j * d + e), s);
        sc[j] = s;
        mx = fmaxf(mx, s);
    }
    mx = block_max(mx, red);
    float sum = 0.f;
    for (int j = threadIdx.x; j < nkeys; j += blockDim.x) {
        const float p = expf(sc[j] - mx);
        sc[j] = p;
        sum += p;
    }
    sum = block_sum(sum, red);  // also orders the sc[] writes before the reads below
    for (int e = threadIdx.x; e < d; e += blockDim.x) {
        float acc = 0.f;
        for (int j = 0; j < nkeys; ++j) acc = fmaf(sc[j], ld_f32(Vp, (size_t)j * d + e), acc);
        o[(size_t)m * H + h * d + e] = acc / sum;
    }
}

// logits[b,v] = sum_k xf[b,k] Wlm[v,k]: one wave per vocabulary row, all batch rows at once.
template <typename ST>
__global__ void lm_head_kernel(const float* __restrict__ xf, const ST* __restrict__ W, float* __restrict__ logits,
                               int B, int H, int V) {
    const int v = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (v >= V) return;
    for (int b0 = 0; b0 < B; b0 += 8) {
        float acc[8] = {};
        for (int k = lane; k < H; k += 64) {
            const float w = ld_f32(W, (size_t)v * H + k);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (b0 + i < B) acc[i] = fmaf(w, xf[(size_t)(b0 + i) * H + k], acc[i]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float a = acc[i];
            for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
            if (lane == 0 && b0 + i < B) logits[(size_t)(b0 + i) * V + v] = a;
        }
    }
}

// One block per sequence: token = argmax of z (greedy) or of z/temperature + Gumbel noise, ties
// to the lowest id; logprob = z[token] - logsumexp(z).
__global__ void sample_kernel(const float* __restrict__ logits, int V, const he_dev_state* __restrict__ st,
                              int32_t* __restrict__ ids_out, float* __restrict__ lp_out, int out_stride,
                              int out_at_step, int32_t* __restrict__ cur_ids) {
    __shared__ float red[8];
    __shared__ float bs[kThreads / 64];
    __shared__ int bi[kThreads / 64];
    const int b = blockIdx.x;
    const float* z = logits + (size_t)b * V;
    const int mode = st->mode, n = st->step;
    const float temp = st->temperature;
    const uint32_t k0 = st->seed_lo, k1 = st->seed_hi;
    float best = -INFINITY, mx = -INFINITY;
    int besti = 0x7FFFFFFF;
    for (int v = threadIdx.x; v < V; v += blockDim.x) {
        const float zv = z[v];
        mx = fmaxf(mx, zv);
        float s = zv;
        if (mode == 1) s = zv / temp + gumbel_from_word(philox_word0((uint32_t)v, (uint32_t)n, (uint32_t)b, k0, k1));
        if (s > best || (s == best && v < besti)) { best = s; besti = v; }
    }
    for (int o = 32; o > 0; o >>= 1) {
        const float os = __shfl_xor(best, o);
        const int oi = __shfl_xor(besti, o);
        if (os > best || (os == best && oi < besti)) { best = os; besti = oi; }
    }
    if ((threadIdx.x & 63) == 0) { bs[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = besti; }
    mx = block_max(mx, red);  // contains the barriers that publish bs/bi
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w)
        if (bs[w] > best || (bs[w] == best && bi[w] < besti)) { best = bs[w]; besti = bi[w]; }
    float sum = 0.f;
    for (int v = threadIdx.x; v < V; v += blockDim.x) sum += expf(z[v] - mx);
    sum = block_sum(sum, red);
    if (threadIdx.x == 0) {
        const size_t at = (size_t)b * out_stride + (out_at_step ? n : 0);
        ids_out[at] = besti;
        lp_out[at] = z[besti] - (mx + logf(sum));
        if (cur_ids) cur_ids[b] = besti;
    }
}

__global__ void set_state_kernel(he_dev_state* st, int cur_len, int step, int set_pos, int mode, float temperature,
                                 uint32_t seed_lo, uint32_t seed_hi) {
    if (set_pos) { st->cur_len = cur_len; st->step = step; st->ragged = 0; }
    st->mode = mode; st->temperature = temperature; st->seed_lo = seed_lo; st->seed_hi = seed_hi;
}

__global__ void init_state_kernel(he_dev_state* st, int max_batch) {
    for (int i = threadIdx.x; i < 4 * max_batch; i += blockDim.x) st->seq[i] = 0;
    for (int i = threadIdx.x; i < max_batch; i += blockDim.x) st->seq[4 * max_batch + i] = i;
    if (threadIdx.x == 0) {
        st->cur_len = 0; st->step = 0; st->mode = 0; st->temperature = 1.f; st->seed_lo = st->seed_hi = 0u;
        st->ragged = 0; st->max_batch = max_batch; st->eos_id = -1; st->pad_id = 0; st->n_active = 0;
    }
}

// Start of a ragged batch: B left-padded prompt rows of S entries, lens[b] of them tokens.
__global__ void set_ragged_kernel(he_dev_state* st, const int32_t* __restrict__ lens, int B, int S, int eos_id,
                                  int pad_id) {
    const int mb = st->max_batch;
    for (int b = threadIdx.x; b < mb; b += blockDim.x) {
        int n = b < B ? lens[b] : S;
        n = n < 1 ? 1 : (n > S ? S : n);  // lengths are clamped to what the rows can hold
        st->seq[b] = 0;
        st->seq[mb + b] = S - n;
        st->seq[2 * mb + b] = 0;
        st->seq[3 * mb + b] = 0;
        st->seq[4 * mb + b] = b;
    }
    if (threadIdx.x == 0) { st->ragged = 1; st->eos_id = eos_id; st->pad_id = pad_id; st->n_active = B; }
}

// End of a pass that fed `tokens` rows per sequence (padding included) and sampled `steps` tokens.
__global__ void advance_state_kernel(he_dev_state* st, int tokens, int steps) {
    if (st->ragged) {
        const int mb = st->max_batch;
        for (int b = threadIdx.x; b < mb; b += blockDim.x) {
            if (!st->seq[2 * mb + b]) st->seq[b] += tokens - st->seq[mb + b];
            st->seq[mb + b] = 0;
        }
    }
    if (threadIdx.x == 0) {
        st->cur_len += tokens;
        st->step += steps;
    }
}

// he_generate_ragged, after a step's sampling: a sequence that has ended keeps producing the
// filler (log-probability 0); one that has just produced eos_id ends here.
__global__ void ragged_post_kernel(he_dev_state* st, int32_t* __restrict__ gen_ids, float* __restrict__ gen_lp,
                                   int32_t* __restrict__ cur_ids, int G, int B) {
    __shared__ int active;
    if (threadIdx.x == 0) active = 0;
    __syncthreads();
    const int mb = st->max_batch, n = st->step;
    for (int r = threadIdx.x; r < B; r += blockDim.x) {  // the B rows of the step (sequences without a row have ended)
        const int b = st->seq[4 * mb + r];
        const size_t at = (size_t)b * G + n;
        if (st->seq[2 * mb + b]) {
            gen_ids[at] = st->pad_id;
            gen_lp[at] = 0.f;
            cur_ids[b] = st->pad_id;
        } else {
            st->seq[3 * mb + b] = n + 1;
            if (gen_ids[at] == st->eos_id) st->seq[2 * mb + b] = 1;
            else atomicAdd(&active, 1);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) st->n_active = active;
}

// he_generate_ragged, between two steps: the rows of sequences that have ended are dropped, the others move up
// in order.  rows: rows of the steps so far (new count = the running sequences: st->n_active).  One thread: the
// order has to be the same every time, and there are a few hundred rows at most.
__global__ void compact_rows_kernel(he_dev_state* st, int rows) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int mb = st->max_batch;
    int k = 0;
    for (int r = 0; r < rows; ++r) {
        const int b = st->seq[4 * mb + r];
        if (!st->seq[2 * mb + b]) st->seq[4 * mb + k++] = b;
    }
    for (; k < mb; ++k) st->seq[4 * mb + k] = k;  // (not in use: any valid sequence number)
}
// ... and back to one row per sequence, in sequence order.
__global__ void identity_rows_kernel(he_dev_state* st) {
    const int mb = st->max_batch;
    for (int i = threadIdx.x; i < mb; i += blockDim.x) st->seq[4 * mb + i] = i;
}

__global__ void fill_gen_kernel(int32_t* ids, float* lp, int count, const he_dev_state* st) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) { ids[i] = st->pad_id; lp[i] = 0.f; }
}

__global__ void copy_lens_kernel(const he_dev_state* st, int32_t* out, int B) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) out[b] = st->seq[3 * st->max_batch + b];
}

__global__ void rng_words_kernel(uint32_t* out, int count, uint32_t v0, uint32_t n, uint32_t b, uint32_t k0,
                                 uint32_t k1) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = philox_word0(v0 + (uint32_t)i, n, b, k0, k1);
}

// plain 16-byte-per-thread copy: the known-size reference that profiler byte counters are scaled by
__global__ void calibration_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ void copy_out_kernel(const int32_t* __restrict__ ids, const float* __restrict__ lp,
                                int32_t* __restrict__ out_ids, float* __restrict__ out_lp, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) { out_ids[i] = ids[i]; out_lp[i] = lp[i]; }
}

}  // namespace

// ------------------------------------------------------------------ launchers

template <typename ST>
static void plain_embed_t(hipStream_t s, const int32_t* ids, int id_stride, const void* tok, const void* pos,
                          float* x, const he_dev_state* st, int M, int S, int H, int V, int pos_offset) {
    embed_kernel<ST><<<M, kThreads, 0, s>>>(ids, id_stride, (const ST*)tok, (const ST*)pos, x, st, S, H, V, pos_offset);
}
void plain_embed(hipStream_t s, int bf16, const int32_t* ids, int id_stride, const void* tok, const void* pos, float* x,
                 const he_dev_state* st, int M, int S, int H, int V, int pos_offset) {
    if (bf16) plain_embed_t<bf16_t>(s, ids, id_stride, tok, pos, x, st, M, S, H, V, pos_offset);
    else plain_embed_t<float>(s, ids, id_stride, tok, pos, x, st, M, S, H, V, pos_offset);
}

void plain_ln(hipStream_t s, int bf16, float* r, const float* y, const void* ybias, const void* g, const void* b,
              float* a, int rows, int H, float eps, int in_mul, int in_add, int writeback) {
    if (bf16)
        ln_kernel<bf16_t><<<rows, kThreads, 0, s>>>(r, y, (const bf16_t*)ybias, (const bf16_t*)g, (const bf16_t*)b, a,
                                                    H, eps, in_mul, in_add, writeback);
    else
        ln_kernel<float><<<rows, kThreads, 0, s>>>(r, y, (const float*)ybias, (const float*)g, (const float*)b, a, H,
                                                   eps, in_mul, in_add, writeback);
}

void plain_gemm(hipStream_t s, int bf16, const float* A, const void* W, const void* bias, int M, int N, int K, int epi,
                float* out, void* kv, const he_dev_state* st, int S, int layer, int H, int n_heads, int max_batch,
                int max_seq, float qscale) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    if (bf16)
        gemm_kernel<bf16_t><<<grid, kThreads, 0, s>>>(A, (const bf16_t*)W, (const bf16_t*)bias, M, N, K, epi, out,
                                                      (float*)kv, st, S, layer, H, n_heads, max_batch, max_seq,
                                                      qscale);
    else
        gemm_kernel<float><<<grid, kThreads, 0, s>>>(A, (const float*)W, (const float*)bias, M, N, K, epi, out,
                                                     (float*)kv, st, S, layer, H, n_heads, max_batch, max_seq, qscale);
}

void plain_attn(hipStream_t s, int bf16, const float* q, const void* kv, float* o, const he_dev_state* st, int M, int S,
                int layer, int H, int n_heads, int max_batch, int max_seq) {
    dim3 grid(M, n_heads);
    const size_t shm = (size_t)(H / n_heads + max_seq) * sizeof(float);
    (void)bf16;  // the plain kernels keep keys and values as floats whatever the weights' type
    attn_kernel<<<grid, 128, shm, s>>>(q, (const float*)kv, o, st, S, layer, H, n_heads, max_batch, max_seq);
}

void plain_lm_head(hipStream_t s, int bf16, const float* xf, const void* W, float* logits, int B, int H, int V) {
    const int grid = (V + 3) / 4;
    if (bf16) lm_head_kernel<bf16_t><<<grid, kThreads, 0, s>>>(xf, (const bf16_t*)W, logits, B, H, V);
    else lm_head_kernel<float><<<grid, kThreads, 0, s>>>(xf, (const float*)W, logits, B, H, V);
}

// one workgroup per row: log-sum-exp of the row's logits, then the next token's log-probability
__global__ void score_rows_kernel(const float* __restrict__ logits, const int32_t* __restrict__ ids, int row0, int S,
                                  int V, float* __restrict__ out) {
    __shared__ float red[kThreads];
    const int m = row0 + blockIdx.x;
    if (m % S == S - 1) return;
    const float* z = logits + (size_t)blockIdx.x * V;
    float mx = -INFINITY;
    for (int i = threadIdx.x; i < V; i += blockDim.x) mx = fmaxf(mx, z[i]);
    red[threadIdx.x] = mx;
    __syncthreads();
    for (int o = blockDim.x / 2; o > 0; o >>= 1) {
        if (threadIdx.x < o) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + o]);
        __syncthreads();
    }
    mx = red[0];
    __syncthreads();
    float sum = 0.f;
    for (int i = threadIdx.x; i < V; i += blockDim.x) sum += expf(z[i] - mx);
    red[threadIdx.x] = sum;
    __syncthreads();
    for (int o = blockDim.x / 2; o > 0; o >>= 1) {
        if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        int t = ids[m + 1];
        t = t < 0 ? 0 : (t >= V ? V - 1 : t);
        out[(size_t)(m / S) * (S - 1) + m % S] = z[t] - (mx + logf(red[0]));
    }
}

void plain_score_rows(hipStream_t s, const float* logits, const int32_t* ids, int row0, int n, int S, int V, float* out) {
    score_rows_kernel<<<n, kThreads, 0, s>>>(logits, ids, row0, S, V, out);
}

void launch_sample(hipStream_t s, const float* logits, int B, int V, const he_dev_state* st, int32_t* ids_out,
                   float* lp_out, int out_stride, int out_at_step, int32_t* cur_ids) {
    sample_kernel<<<B, kThreads, 0, s>>>(logits, V, st, ids_out, lp_out, out_stride, out_at_step, cur_ids);
}

void launch_set_state(hipStream_t s, he_dev_state* st, int cur_len, int step, int set_pos, int mode, float temperature,
                      uint64_t seed) {
    set_state_kernel<<<1, 1, 0, s>>>(st, cur_len, step, set_pos, mode, temperature, (uint32_t)(seed & 0xFFFFFFFFu),
                                     (uint32_t)(seed >> 32));
}

void launch_init_state(hipStream_t s, he_dev_state* st, int max_batch) { init_state_kernel<<<1, 256, 0, s>>>(st, max_batch); }
void launch_set_ragged(hipStream_t s, he_dev_state* st, const int32_t* lens, int B, int S, int eos_id, int pad_id) {
    set_ragged_kernel<<<1, 256, 0, s>>>(st, lens, B, S, eos_id, pad_id);
}
void launch_ragged_post(hipStream_t s, he_dev_state* st, int32_t* gen_ids, float* gen_lp, int32_t* cur_ids, int G, int B) {
    ragged_post_kernel<<<1, 256, 0, s>>>(st, gen_ids, gen_lp, cur_ids, G, B);
}
void launch_compact_rows(hipStream_t s, he_dev_state* st, int rows) { compact_rows_kernel<<<1, 64, 0, s>>>(st, rows); }
void launch_identity_rows(hipStream_t s, he_dev_state* st) { identity_rows_kernel<<<1, 256, 0, s>>>(st); }
void launch_fill_gen(hipStream_t s, int32_t* ids, float* lp, int count, const he_dev_state* st) {
    fill_gen_kernel<<<(count + 255) / 256, 256, 0, s>>>(ids, lp, count, st);
}
void launch_copy_lens(hipStream_t s, const he_dev_state* st, int32_t* out, int B) {
    copy_lens_kernel<<<(B + 255) / 256, 256, 0, s>>>(st, out, B);
}
void launch_advance_state(hipStream_t s, he_dev_state* st, int tokens, int steps) {
    advance_state_kernel<<<1, 64, 0, s>>>(st, tokens, steps);
}

void launch_rng_words(hipStream_t s, uint64_t seed, uint32_t b, uint32_t n, uint32_t v0, int count, uint32_t* out) {
    rng_words_kernel<<<(count + 255) / 256, 256, 0, s>>>(out, count, v0, n, b, (uint32_t)(seed & 0xFFFFFFFFu),
                                                         (uint32_t)(seed >> 32));
}

void launch_calibration_copy(hipStream_t s, const void* src, void* dst, size_t bytes) {
    calibration_copy_kernel<<<4096, 256, 0, s>>>((const uint4*)src, (uint4*)dst, bytes / 16);
}

void launch_copy_out(hipStream_t s, const int32_t* ids, const float* lp, int32_t* out_ids, float* out_lp, int count) {
    copy_out_kernel<<<(count + 255) / 256, 256, 0, s>>>(ids, lp, out_ids, out_lp, count);
}
