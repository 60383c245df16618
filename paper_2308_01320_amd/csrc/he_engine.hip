// The engine behind the C ABI in include/he.h: argument validation, the KV arena
// and workspace (allocated once), and the stream-ordered kernel sequence of a
// prompt pass / decode step of the actor's generation phase (paper Section 4
// and Section 5.3 (I)).
#include <algorithm>
#include <string>
#include <vector>

#include "../../include/he.h"
#include "he_common.h"
#include "kernels.h"

struct he_engine {
    he_config cfg{};
    int d = 0;          // head_dim
    bool bf16 = false;  // storage type of weights / KV
    hipStream_t stream = nullptr;
    he_weights w{};
    std::vector<he_layer_weights> layers;

    std::vector<void*> allocs;  // everything the engine owns on the device
    void* kv = nullptr;
    he_dev_state* st = nullptr;
    float *resid = nullptr, *abuf = nullptr, *qbuf = nullptr, *obuf = nullptr, *ybuf = nullptr, *hbuf = nullptr;
    float *xf = nullptr, *logits = nullptr, *gen_lp = nullptr;
    int32_t *cur_ids = nullptr, *gen_ids = nullptr;

    // bf16 path: MFMA-tiled copies of the GEMM matrices (IEEE halves) and tiled activation buffers
    bool fast = false;
    struct Tiled { void *wqkv, *wo, *w1, *w2; };
    std::vector<Tiled> tiled;
    void *lm_tiled = nullptr, *ablk = nullptr, *oblk = nullptr, *hblk = nullptr, *xfblk = nullptr;
    // 8-bit weights: tiled[] then holds E4M3 units, wscale_buf the row scales (per layer 3H + H + F + H floats),
    // scratch one layer's dequantised half blocks for the GEMMs that read those
    bool w8 = false;
    float* wscale_buf = nullptr;
    int* exps_tmp = nullptr;
    Tiled scratch{nullptr, nullptr, nullptr, nullptr};
    float *part = nullptr, *stats = nullptr;
    size_t part_floats = 0;  // capacity of `part`
    int* stats_idx = nullptr;
    // decode rows: LayerNorms folded into the GEMMs around them
    float *cvec = nullptr;     // per layer W gamma, W beta for wqkv (2 x 3H) and w1 (2 x F), then the LM head's (2 x V), padded to 32
    float *ln_stats = nullptr; // per-column-group mean / squared deviations of the residual rows
    int* ln_counters = nullptr;
    float *score_stats = nullptr, *score_tgt = nullptr;  // scoring pass: soft-max partials per row and vocabulary slice
    float* tail_buf = nullptr;  // prompt pass: residual and query rows of each sequence's last token, 2 x [max_batch][H]

    // one decode step captured as a HIP graph (he_generate replays it); keyed by (B, G)
    hipGraphExec_t step_graph = nullptr;   // one decode step of he_generate
    hipGraphExec_t multi_graph = nullptr;  // kGraphSteps of them in a row (nullptr if the answer is shorter)
    int graph_B = 0, graph_G = 0;
    bool graph_ragged = false;

    // measurement hook: HIP events around every launch of a kernel class of the decode step
    bool timing = false;
    std::vector<hipEvent_t> ev_pool;
    std::vector<std::pair<int, size_t>> ev_used;  // (class, index of the start event)
    size_t ev_next = 0;

    // host mirror of the device state
    int cur_len = 0, step = 0, batch = 0;  // cur_len: the longest sequence's, when they differ
    std::vector<he_lora_layer> lora;  // adapters folded into the tiled copies by the last refresh (empty: none)
    int lora_rank = 0;
    float lora_scale = 0.f;
    bool arena_released = false;
    size_t kv_bytes = 0;
    bool ragged_gen = false;   // he_generate_ragged is running: sampling is followed by the end-token bookkeeping
    int* host_active = nullptr;  // pinned: sequences still generating, read back every few steps
    int last_rows = 0;           // rows of the last decode step of the last he_generate / he_generate_ragged
    std::string err;
};

static std::string g_create_error;

// ---- he_decode_step_static: the decode step's scratch in memory that is never allocated
//
// A file-scope device array that every GPU the library runs on holds from load to exit.  In host code the
// array's name is only a stand-in; the device address is looked up once per device (with that device
// current) and kept, and only that pointer is ever handed to kernels.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char he_static_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_static_ptr[kMaxDevices] = {};

// zeroes `count` 32-bit words (a kernel, not hipMemsetAsync: the caller may be capturing a graph)
__global__ void zero_words_kernel(uint32_t* __restrict__ p, size_t count) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

namespace {

struct Sizes {
    size_t kv, rowsH, rowsF, xf, logits, gen, total;
    // bf16 path
    size_t tiled_layer, tiled_lm, ablk, hblk, xfblk, part, stats, stats_idx, cvec, ln_stats, ln_counters, score_stats, tail;
};

bool is_fast(const he_config& c) { return c.dtype == HE_BF16 && c.impl == 0; }
constexpr int kMaxKSplit = 8;  // no GEMM plan splits k further

// bytes per cached key / value element: IEEE halves on the tuned bf16 path, floats for the plain kernels
size_t kv_elt_bytes(const he_config& c) { return is_fast(c) ? 2 : 4; }

const char* check_config(const he_config* c) {
    if (!c) return "config is NULL";
    if (c->n_layers < 0 || c->hidden <= 0 || c->n_heads <= 0 || c->ffn <= 0 || c->vocab <= 0) return "non-positive model dimension";
    if (c->max_positions <= 0 || c->pos_offset < 0 || c->max_batch <= 0 || c->max_seq_len <= 0) return "non-positive capacity";
    if (c->dtype != HE_F32 && c->dtype != HE_BF16) return "unknown dtype";
    if (c->impl != 0 && c->impl != 1) return "unknown impl";
    if (c->weights_tiled != 0 && c->weights_tiled != 1) return "weights_tiled must be 0 or 1";
    if (c->weights_tiled && !(c->dtype == HE_BF16 && c->impl == 0)) return "weights_tiled needs dtype bf16 and impl 0";
    if (c->weights_fp8 != 0 && c->weights_fp8 != 1) return "weights_fp8 must be 0 or 1";
    if (c->weights_fp8 && !(c->dtype == HE_BF16 && c->impl == 0 && !c->weights_tiled))
        return "weights_fp8 needs dtype bf16, impl 0 and weights_tiled 0";
    if (!(c->ln_eps > 0.f)) return "ln_eps must be positive";
    return nullptr;
}

const char* check_shape(const he_config* c) {
    if (c->hidden % c->n_heads) return "hidden is not a multiple of n_heads";
    const int d = c->hidden / c->n_heads;
    if (d % 8 || d > 256) return "head_dim must be a multiple of 8 and at most 256";
    if (c->max_seq_len > 8192) return "max_seq_len above 8192 is not supported";
    if (is_fast(*c)) {
        if (c->hidden % 64 || c->ffn % 64) return "bf16 path: hidden and ffn must be multiples of 64";
        if (d != 64 && d != 128) return "bf16 path: head_dim must be 64 or 128";
    }
    return nullptr;
}

Sizes sizes_of(const he_config& c) {
    Sizes s{};
    const size_t rows = (size_t)c.max_batch * c.max_seq_len;
    s.kv = (size_t)c.n_layers * 2 * rows * c.hidden * kv_elt_bytes(c);
    s.rowsH = rows * c.hidden * sizeof(float);
    s.rowsF = rows * c.ffn * sizeof(float);
    s.xf = (size_t)c.max_batch * c.hidden * sizeof(float);
    s.logits = (size_t)c.max_batch * c.vocab * sizeof(float);
    s.gen = rows * sizeof(float);
    s.total = s.kv + s.logits + 2 * s.gen + c.max_batch * sizeof(int32_t) + he_dev_state_bytes(c.max_batch);
    if (!is_fast(c)) {
        s.total += 5 * s.rowsH + s.rowsF + s.xf;
        return s;
    }
    const int H = c.hidden, F = c.ffn;
    s.tiled_layer = bf16_tiled_bytes(3 * H, H) + bf16_tiled_bytes(H, H) + bf16_tiled_bytes(F, H) + bf16_tiled_bytes(H, F);
    s.tiled_lm = bf16_tiled_bytes(c.vocab, H);
    s.ablk = bf16_tiled_bytes((int)rows, H);
    s.hblk = bf16_tiled_bytes((int)rows, F);
    s.xfblk = bf16_tiled_bytes(c.max_batch, H);
    // prompt rows, or the decode step's k-split scratch: splits x rows padded to 32, twice (a
    // workgroup of eight wavefronts on a single tile leaves half of its slots unused)
    const size_t drow = (size_t)2 * kMaxKSplit * (((size_t)c.max_batch + 31) / 32 * 32);
    // ... or, for decode steps of more than 32 rows, the k-split partial sums of the widest GEMM
    const size_t wide = (size_t)(3 * c.hidden > c.ffn ? 3 * c.hidden : c.ffn);
    const size_t mrow = c.max_batch > 32 ? ((size_t)kMaxKSplit * c.max_batch * wide + c.hidden - 1) / c.hidden : 0;
    const size_t prow = std::max(std::max(rows, drow), mrow);
    s.part = prow * H * sizeof(float);
    const size_t ntile = (size_t)(c.vocab + 31) / 32;
    s.stats = (size_t)c.max_batch * ntile * 4 * sizeof(float);
    s.stats_idx = (size_t)c.max_batch * ntile * sizeof(int);
    const size_t vpad = ((size_t)c.vocab + 31) / 32 * 32, mtiles = ((size_t)c.max_batch + 31) / 32;
    s.cvec = ((size_t)c.n_layers * 2 * (3 * H + F) + 2 * vpad) * sizeof(float);
    // column groups of the k-split GEMMs: at most one per 16 columns (8-bit weights on a narrow model; 16-bit
    // weights never go below 32)
    s.ln_stats = mtiles * (H / 16) * 32 * 2 * sizeof(float) + 1024;
    s.ln_counters = mtiles * (H / 16) * sizeof(int);
    s.score_stats = rows * bf16_score_parts(c.vocab) * 2 * sizeof(float);
    s.tail = (size_t)2 * c.max_batch * H * sizeof(float);
    s.total += s.cvec + s.ln_stats + s.ln_counters + s.score_stats + s.gen + s.tail;
    if (c.weights_fp8) {  // E4M3 units (half the bytes), row scales, one layer of bf16 scratch
        const size_t q8_layer = fp8_units_bytes(3 * H, H) + fp8_units_bytes(H, H) + fp8_units_bytes(F, H) + fp8_units_bytes(H, F);
        s.total += (size_t)c.n_layers * (q8_layer + (size_t)(5 * H + F) * sizeof(float)) + s.tiled_layer + s.tiled_lm +
                   wide * sizeof(int);
    }
    s.total += 2 * s.rowsH /* resid, q */ + (c.weights_tiled || c.weights_fp8 ? 0 : (size_t)c.n_layers * s.tiled_layer + s.tiled_lm) +
               2 * s.ablk + s.hblk + s.xfblk + s.part + s.stats + s.stats_idx;
    return s;
}

he_status fail(he_engine* e, he_status code, const std::string& msg) {
    if (e) e->err = msg;
    return code;
}

he_status check_hip(he_engine* e, hipError_t r, const char* what) {
    if (r == hipSuccess) return HE_OK;
    return fail(e, HE_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(r));
}

template <typename T>
hipError_t dev_alloc(he_engine* e, T** p, size_t bytes) {
    void* q = nullptr;
    hipError_t r = hipMalloc(&q, bytes ? bytes : 1);
    if (r == hipSuccess) {
        e->allocs.push_back(q);
        *p = (T*)q;
    }
    return r;
}

void free_all(he_engine* e) {
    for (void* p : e->allocs) (void)hipFree(p);
    e->allocs.clear();
    if (e->host_active) (void)hipHostFree(e->host_active);
    e->host_active = nullptr;
}

// Brackets the launches made during its lifetime with a pair of events when timing is on.
struct LaunchTimer {
    he_engine* e;
    bool on;
    LaunchTimer(he_engine* eng, int cls) : e(eng), on(eng->timing) {
        if (!on) return;
        while (e->ev_pool.size() < e->ev_next + 2) {
            hipEvent_t ev;
            if (hipEventCreate(&ev) != hipSuccess) { on = false; return; }
            e->ev_pool.push_back(ev);
        }
        e->ev_used.emplace_back(cls, e->ev_next);
        (void)hipEventRecord(e->ev_pool[e->ev_next], e->stream);
    }
    ~LaunchTimer() {
        if (!on) return;
        (void)hipEventRecord(e->ev_pool[e->ev_next + 1], e->stream);
        e->ev_next += 2;
    }
};

// 8-bit weights: where the row scales of layer l live, and the layer as bf16 blocks (dequantised into the
// scratch layer, on the engine's stream, for the GEMMs that read 32x16 blocks: prompt rows, scoring,
// decode steps of more than 32 rows).
struct Scales { float *wqkv, *wo, *w1, *w2; };
Scales scales_of(const he_engine* e, int l) {
    const size_t H = e->cfg.hidden, F = e->cfg.ffn;
    float* p = e->wscale_buf + (size_t)l * (5 * H + F);
    return {p, p + 3 * H, p + 4 * H, p + 4 * H + F};
}
he_engine::Tiled layer_blocks(he_engine* e, int l) {
    if (!e->w8) return e->tiled[l];
    const int H = e->cfg.hidden, F = e->cfg.ffn;
    const Scales sc = scales_of(e, l);
    fp8_dequant_units(e->stream, e->tiled[l].wqkv, sc.wqkv, e->scratch.wqkv, 3 * H, H);
    fp8_dequant_units(e->stream, e->tiled[l].wo, sc.wo, e->scratch.wo, H, H);
    fp8_dequant_units(e->stream, e->tiled[l].w1, sc.w1, e->scratch.w1, F, H);
    fp8_dequant_units(e->stream, e->tiled[l].w2, sc.w2, e->scratch.w2, H, F);
    return e->scratch;
}

// bf16 path, prompt rows: Sp tokens per sequence through the tiled MFMA GEMMs.  From all but each sequence's
// last token only the K/V cache is wanted, so the final layer stops once its keys and values are stored (the
// last tokens' rows are then finished by pass_last_token_bf16, or, where that does not apply, the last token
// is left out here and takes the whole decode-shaped pass).
// With `full` (the scoring pass) every layer is completed and the last FC2's output is left
// pending, as k-split partial sums plus *pend_bias, for the final LayerNorm.
void pass_tiled_bf16(he_engine* e, const int32_t* d_ids, int id_stride, int B, int Sp, bool full = false,
                     const void** pend_bias = nullptr, int* pend_ksplit = nullptr, int advance = -1,
                     int* pend_split_col = nullptr) {
    const he_config& c = e->cfg;
    hipStream_t s = e->stream;
    const int M = B * Sp, H = c.hidden, F = c.ffn;
    bf16_gemm_args base;
    base.st = e->st; base.S = Sp; base.H = H; base.n_heads = c.n_heads; base.max_batch = c.max_batch;
    base.max_seq = c.max_seq_len;
    plain_embed(s, 1, d_ids, id_stride, e->w.tok_emb, e->w.pos_emb, e->resid, e->st, M, Sp, H, c.vocab, c.pos_offset);
    const float* pend = nullptr;  // GEMM output not yet added to the residual stream
    const void* pend_b = nullptr;
    const size_t split = (size_t)M * H;
    // k ranges per tile of the two GEMMs whose partial sums the next LayerNorm adds, and the first column whose
    // tiles are cut at all
    int kso, sco, nao, ks2, sc2, na2;
    bf16_tiled_store_split(M, H, H, e->part_floats, &kso, &sco, &nao);
    bf16_tiled_store_split(M, H, F, e->part_floats, &ks2, &sc2, &na2);
    int pend_ks = 1, pend_sc = 0;
    for (int l = 0; l < c.n_layers; ++l) {
        const he_layer_weights& lw = e->layers[l];
        const he_engine::Tiled tw = layer_blocks(e, l);
        bf16_ln(s, e->resid, pend, pend_ks, split, pend_b, lw.ln1_g, lw.ln1_b, e->ablk, M, H, c.ln_eps, 1, 0, 1, pend_sc);
        bf16_gemm_args a = base;
        a.layer = l; a.bias = lw.bqkv; a.out = e->qbuf; a.kv = e->kv; a.qscale = 1.0f / sqrtf((float)e->d);
        bf16_gemm_tiled(s, EPI_QKV, tw.wqkv, e->ablk, M, 3 * H, H, a);
        if (l == c.n_layers - 1 && !full) break;
        bf16_attn(s, e->qbuf, e->kv, e->oblk, e->st, M, Sp, l, H, c.n_heads, c.max_batch, c.max_seq_len);
        a = base; a.split_col = sco; a.tile_na = nao;
        bf16_gemm_tiled_ksplit(s, EPI_STORE, tw.wo, e->oblk, M, H, H, kso, e->part, split, a);
        bf16_ln(s, e->resid, e->part, kso, split, lw.bo, lw.ln2_g, lw.ln2_b, e->ablk, M, H, c.ln_eps, 1, 0, 1, sco);
        a = base; a.bias = lw.b1; a.out_blocks = e->hblk;
        bf16_gemm_tiled(s, EPI_BIAS_RELU, tw.w1, e->ablk, M, F, H, a);
        a = base; a.split_col = sc2; a.tile_na = na2;
        bf16_gemm_tiled_ksplit(s, EPI_STORE, tw.w2, e->hblk, M, H, F, ks2, e->part, split, a);
        pend = e->part; pend_b = lw.b2; pend_ks = ks2; pend_sc = sc2;
    }
    if (pend_bias) *pend_bias = pend_b;
    if (pend_ksplit) *pend_ksplit = pend_ks;
    if (pend_split_col) *pend_split_col = pend_sc;
    if (advance < 0) advance = Sp;  // (the caller that finishes the last token itself advances by one row less)
    launch_advance_state(s, e->st, advance, 0);
    e->cur_len += advance;
}

// Where the vectors W gamma (c1) and W beta (c2) of the GEMMs that follow a LayerNorm live.
struct CVec { float *c1, *c2; };
CVec cvec_qkv(const he_engine* e, int l) {
    const size_t H = e->cfg.hidden, F = e->cfg.ffn;
    float* p = e->cvec + (size_t)l * 2 * (3 * H + F);
    return {p, p + 3 * H};
}
CVec cvec_fc1(const he_engine* e, int l) {
    const size_t H = e->cfg.hidden, F = e->cfg.ffn;
    float* p = e->cvec + (size_t)l * 2 * (3 * H + F) + 6 * H;
    return {p, p + F};
}
CVec cvec_lm(const he_engine* e) {
    const size_t H = e->cfg.hidden, F = e->cfg.ffn, vpad = ((size_t)e->cfg.vocab + 31) / 32 * 32;
    float* p = e->cvec + (size_t)e->cfg.n_layers * 2 * (3 * H + F);
    return {p, p + vpad};
}

// bf16 path, one new token per sequence (a decode step, or the last prompt token):
// weight-streaming GEMMs, attention over the cache, LM head
// fused with log-softmax and sampling.
void pass_decode_bf16(he_engine* e, const int32_t* d_ids, int id_stride, int B, int32_t* ids_out, float* lp_out,
                      int out_stride, int out_at_step, float* d_logits_opt) {
    const he_config& c = e->cfg;
    hipStream_t s = e->stream;
    const int H = c.hidden, F = c.ffn, L = c.n_layers;
    bf16_gemm_args base;
    base.st = e->st; base.S = 1; base.H = H; base.n_heads = c.n_heads; base.max_batch = c.max_batch;
    base.max_seq = c.max_seq_len;
    // No LayerNorm kernels here: each one is folded into the GEMM after it.  Whoever produces a
    // residual row (the embedding, the out-projection, FC2) leaves gamma * x as half blocks
    // and statistics per group of columns; the column groups are the producer's workgroups.
    int gw1, ks1, gw2, ks2;  // column-group widths after the out-projection / after FC2 and the embedding
    if (e->w8) {
        bf16_store_plan_w8(H, H, e->part_floats, &gw1, &ks1);
        bf16_store_plan_w8(H, F, e->part_floats, &gw2, &ks2);
    } else {
        bf16_store_plan(B, H, H, e->part_floats, &gw1, &ks1);
        bf16_store_plan(B, H, F, e->part_floats, &gw2, &ks2);
    }
    if (!L) gw2 = 128;
    const size_t split = (size_t)B * H;
    auto fold = [&](bf16_gemm_args& a, int gw, const CVec& cv) {
        a.ln_stats = e->ln_stats; a.ln_gw = gw; a.ln_groups = (H + gw - 1) / gw; a.ln_cols = H; a.ln_eps = c.ln_eps;
        a.c1 = cv.c1; a.c2 = cv.c2;
    };
    auto store_ln = [&](bf16_gemm_args& a, const void* bias, const void* gamma, void* blk) {
        a.out = e->part; a.out_split = split; a.out_capacity = e->part_floats; a.bias = bias; a.resid = e->resid; a.gamma = gamma;
        a.out_blocks = blk; a.stats_out = e->ln_stats; a.counters = e->ln_counters;
    };
    {
        LaunchTimer t(e, HE_K_LAYERNORM);
        const bool last = L == 0;
        bf16_embed_ln(s, d_ids, id_stride, e->w.tok_emb, e->w.pos_emb, e->st, B, H, c.vocab, c.pos_offset, gw2,
                      last ? e->w.lnf_g : e->layers[0].ln1_g, e->resid, last ? e->xfblk : e->ablk, e->ln_stats);
    }
    for (int l = 0; l < L; ++l) {
        const he_layer_weights& lw = e->layers[l];
        const he_engine::Tiled& tw = e->tiled[l];  // bf16 blocks, or E4M3 units with 8-bit weights
        bf16_gemm_args a = base;
        a.layer = l; a.bias = lw.bqkv; a.out = e->qbuf; a.kv = e->kv; a.qscale = 1.0f / sqrtf((float)e->d);
        fold(a, gw2, cvec_qkv(e, l));
        const Scales sc = e->w8 ? scales_of(e, l) : Scales{nullptr, nullptr, nullptr, nullptr};
        a.wscale = sc.wqkv;
        {
            LaunchTimer t(e, HE_K_QKV);
            bf16_gemm_skinny(s, EPI_QKV, tw.wqkv, e->ablk, B, 3 * H, H, 1, a);
        }
        {
            LaunchTimer t(e, HE_K_ATTENTION);
            bf16_attn(s, e->qbuf, e->kv, e->oblk, e->st, B, 1, l, H, c.n_heads, c.max_batch, c.max_seq_len);
        }
        a = base;
        store_ln(a, lw.bo, lw.ln2_g, e->ablk);
        a.wscale = sc.wo;
        {
            LaunchTimer t(e, HE_K_OUT_PROJ);
            bf16_gemm_skinny(s, EPI_STORE_LN, tw.wo, e->oblk, B, H, H, ks1, a);
        }
        a = base; a.bias = lw.b1; a.out_blocks = e->hblk;
        fold(a, gw1, cvec_fc1(e, l));
        a.wscale = sc.w1;
        {
            LaunchTimer t(e, HE_K_FC1);
            bf16_gemm_skinny(s, EPI_BIAS_RELU, tw.w1, e->ablk, B, F, H, 1, a);
        }
        a = base;
        const bool last = l == L - 1;
        store_ln(a, lw.b2, last ? e->w.lnf_g : e->layers[l + 1].ln1_g, last ? e->xfblk : e->ablk);
        a.wscale = sc.w2;
        {
            LaunchTimer t(e, HE_K_FC2);
            bf16_gemm_skinny(s, EPI_STORE_LN, tw.w2, e->hblk, B, H, F, ks2, a);
        }
    }
    {
        LaunchTimer t(e, HE_K_LM_HEAD);
        bf16_gemm_args a = base;
        fold(a, gw2, cvec_lm(e));
        bf16_lm_head(s, e->lm_tiled, e->xfblk, B, c.vocab, H, e->st, d_logits_opt, e->stats, e->stats_idx,
                     ids_out, lp_out, out_stride, out_at_step, e->cur_ids, &a);
    }
    { LaunchTimer t(e, HE_K_EMPTY); }
    if (e->ragged_gen) launch_ragged_post(s, e->st, ids_out, lp_out, e->cur_ids, out_stride, B);
    launch_advance_state(s, e->st, 1, 1);
    e->cur_len += 1;
    e->step += 1;
}

// The end of a prompt pass whose tiled GEMMs took every token up to the last layer's QKV projection: what is
// left of that layer, for each sequence's LAST token only -- attention over the cache, out-projection, FC1, FC2
// on the weight-streaming kernels -- then the LM head and sampling.  (The last token used to take the whole
// decode-shaped pass, streaming all layers' weights once more: one decode step's time per prompt pass.)
// On entry the device state still counts the last token as not cached (cur_len = S - 1), as in a decode step
// after its QKV projection.
void pass_last_token_bf16(he_engine* e, int B, int S, int32_t* ids_out, float* lp_out, int out_stride, int out_at_step,
                          float* d_logits_opt) {
    const he_config& c = e->cfg;
    hipStream_t s = e->stream;
    const int H = c.hidden, F = c.ffn, l = c.n_layers - 1;
    bf16_gemm_args base;
    base.st = e->st; base.S = 1; base.H = H; base.n_heads = c.n_heads; base.max_batch = c.max_batch;
    base.max_seq = c.max_seq_len;
    int gw1, ks1, gw2, ks2;
    if (e->w8) {
        bf16_store_plan_w8(H, H, e->part_floats, &gw1, &ks1);
        bf16_store_plan_w8(H, F, e->part_floats, &gw2, &ks2);
    } else {
        bf16_store_plan(B, H, H, e->part_floats, &gw1, &ks1);
        bf16_store_plan(B, H, F, e->part_floats, &gw2, &ks2);
    }
    const size_t split = (size_t)B * H;
    float *r_last = e->tail_buf, *q_last = e->tail_buf + (size_t)c.max_batch * H;
    bf16_gather_last_rows(s, e->resid, e->qbuf, r_last, q_last, B, S, H);
    const he_layer_weights& lw = e->layers[l];
    const he_engine::Tiled& tw = e->tiled[l];
    const Scales sc = e->w8 ? scales_of(e, l) : Scales{nullptr, nullptr, nullptr, nullptr};
    auto fold = [&](bf16_gemm_args& a, int gw, const CVec& cv) {
        a.ln_stats = e->ln_stats; a.ln_gw = gw; a.ln_groups = (H + gw - 1) / gw; a.ln_cols = H; a.ln_eps = c.ln_eps;
        a.c1 = cv.c1; a.c2 = cv.c2;
    };
    auto store_ln = [&](bf16_gemm_args& a, const void* bias, const void* gamma, void* blk) {
        a.out = e->part; a.out_split = split; a.out_capacity = e->part_floats; a.bias = bias; a.resid = r_last; a.gamma = gamma;
        a.out_blocks = blk; a.stats_out = e->ln_stats; a.counters = e->ln_counters;
    };
    {
        LaunchTimer t(e, HE_K_ATTENTION);
        bf16_attn(s, q_last, e->kv, e->oblk, e->st, B, 1, l, H, c.n_heads, c.max_batch, c.max_seq_len);
    }
    bf16_gemm_args a = base;
    store_ln(a, lw.bo, lw.ln2_g, e->ablk);
    a.wscale = sc.wo;
    {
        LaunchTimer t(e, HE_K_OUT_PROJ);
        bf16_gemm_skinny(s, EPI_STORE_LN, tw.wo, e->oblk, B, H, H, ks1, a);
    }
    a = base; a.bias = lw.b1; a.out_blocks = e->hblk;
    fold(a, gw1, cvec_fc1(e, l));
    a.wscale = sc.w1;
    {
        LaunchTimer t(e, HE_K_FC1);
        bf16_gemm_skinny(s, EPI_BIAS_RELU, tw.w1, e->ablk, B, F, H, 1, a);
    }
    a = base;
    store_ln(a, lw.b2, e->w.lnf_g, e->xfblk);
    a.wscale = sc.w2;
    {
        LaunchTimer t(e, HE_K_FC2);
        bf16_gemm_skinny(s, EPI_STORE_LN, tw.w2, e->hblk, B, H, F, ks2, a);
    }
    {
        LaunchTimer t(e, HE_K_LM_HEAD);
        a = base;
        fold(a, gw2, cvec_lm(e));
        bf16_lm_head(s, e->lm_tiled, e->xfblk, B, c.vocab, H, e->st, d_logits_opt, e->stats, e->stats_idx, ids_out, lp_out,
                     out_stride, out_at_step, e->cur_ids, &a);
    }
    { LaunchTimer t(e, HE_K_EMPTY); }
    if (e->ragged_gen) launch_ragged_post(s, e->st, ids_out, lp_out, e->cur_ids, out_stride, B);
    launch_advance_state(s, e->st, 1, 1);
    e->cur_len += 1;
    e->step += 1;
}

// The same pass for more than 64 sequences (more than 32 with 8-bit weights): the rows no longer fit the
// weight-streaming kernels, so the GEMMs are the prompt-pass tiles (weights shared through LDS by all rows), cut along k until they fill the
// chip; LayerNorms are kernels of their own again and add the partial sums.
void pass_decode_wide_bf16(he_engine* e, const int32_t* d_ids, int id_stride, int B, int32_t* ids_out, float* lp_out,
                           int out_stride, int out_at_step, float* d_logits_opt) {
    const he_config& c = e->cfg;
    hipStream_t s = e->stream;
    const int H = c.hidden, F = c.ffn;
    bf16_gemm_args base;
    base.st = e->st; base.S = 1; base.H = H; base.n_heads = c.n_heads; base.max_batch = c.max_batch;
    base.max_seq = c.max_seq_len;
    plain_embed(s, 1, d_ids, id_stride, e->w.tok_emb, e->w.pos_emb, e->resid, e->st, B, 1, H, c.vocab, c.pos_offset);
    const float* pend = nullptr;
    int pend_ks = 0;
    const void* pend_b = nullptr;
    const size_t split = (size_t)B * H;
    const int ksq = bf16_tiled_ksplit(B, 3 * H, H), kso = bf16_tiled_ksplit(B, H, H);
    const int ks1 = bf16_tiled_ksplit(B, F, H), ks2 = bf16_tiled_ksplit(B, H, F);
    for (int l = 0; l < c.n_layers; ++l) {
        const he_layer_weights& lw = e->layers[l];
        const he_engine::Tiled tw = layer_blocks(e, l);
        {
            LaunchTimer t(e, HE_K_LAYERNORM);
            bf16_ln(s, e->resid, pend, pend_ks, split, pend_b, lw.ln1_g, lw.ln1_b, e->ablk, B, H, c.ln_eps, 1, 0, 1);
        }
        bf16_gemm_args a = base;
        a.layer = l; a.bias = lw.bqkv; a.out = e->qbuf; a.kv = e->kv; a.qscale = 1.0f / sqrtf((float)e->d);
        {
            LaunchTimer t(e, HE_K_QKV);
            bf16_gemm_tiled_ksplit(s, EPI_QKV, tw.wqkv, e->ablk, B, 3 * H, H, ksq, e->part, (size_t)B * 3 * H, a);
        }
        {
            LaunchTimer t(e, HE_K_ATTENTION);
            bf16_attn(s, e->qbuf, e->kv, e->oblk, e->st, B, 1, l, H, c.n_heads, c.max_batch, c.max_seq_len);
        }
        a = base;
        {
            LaunchTimer t(e, HE_K_OUT_PROJ);
            bf16_gemm_tiled_ksplit(s, EPI_STORE, tw.wo, e->oblk, B, H, H, kso, e->part, split, a);
        }
        {
            LaunchTimer t(e, HE_K_LAYERNORM);
            bf16_ln(s, e->resid, e->part, kso, split, lw.bo, lw.ln2_g, lw.ln2_b, e->ablk, B, H, c.ln_eps, 1, 0, 1);
        }
        a = base; a.bias = lw.b1; a.out_blocks = e->hblk;
        {
            LaunchTimer t(e, HE_K_FC1);
            bf16_gemm_tiled_ksplit(s, EPI_BIAS_RELU, tw.w1, e->ablk, B, F, H, ks1, e->part, (size_t)B * F, a);
        }
        a = base;
        {
            LaunchTimer t(e, HE_K_FC2);
            bf16_gemm_tiled_ksplit(s, EPI_STORE, tw.w2, e->hblk, B, H, F, ks2, e->part, split, a);
        }
        pend = e->part; pend_ks = ks2; pend_b = lw.b2;
    }
    {
        LaunchTimer t(e, HE_K_LAYERNORM);
        bf16_ln(s, e->resid, pend, pend_ks, split, pend_b, e->w.lnf_g, e->w.lnf_b, e->xfblk, B, H, c.ln_eps, 1, 0, 0);
    }
    {
        LaunchTimer t(e, HE_K_LM_HEAD);
        bf16_lm_head(s, e->lm_tiled, e->xfblk, B, c.vocab, H, e->st, d_logits_opt, e->stats, e->stats_idx,
                     ids_out, lp_out, out_stride, out_at_step, e->cur_ids);
    }
    { LaunchTimer t(e, HE_K_EMPTY); }
    if (e->ragged_gen) launch_ragged_post(s, e->st, ids_out, lp_out, e->cur_ids, out_stride, B);
    launch_advance_state(s, e->st, 1, 1);
    e->cur_len += 1;
    e->step += 1;
}

// Decode steps of up to 32 sequences, and of up to 64 with bf16 weights (two 32-row slices per workgroup),
// stream the weights through the decode GEMMs; larger ones take the prompt pass's tiles.
bool wide_decode(const he_engine* e, int B) { return B > 64 || (B > 32 && e->w8); }

he_status run_forward_bf16(he_engine* e, const int32_t* d_ids, int B, int S, int32_t* ids_out, float* lp_out,
                           int out_stride, int out_at_step, float* d_logits_opt) {
    if (S > 1 && e->cfg.n_layers > 0 && !wide_decode(e, B)) {
        // every prompt token through the tiled GEMMs up to the last layer's keys and values, then the rest of
        // that layer for the last tokens alone
        pass_tiled_bf16(e, d_ids, S, B, S, false, nullptr, nullptr, S - 1);
        pass_last_token_bf16(e, B, S, ids_out, lp_out, out_stride, out_at_step, d_logits_opt);
        return check_hip(e, hipGetLastError(), "kernel launch");
    }
    if (S > 1) pass_tiled_bf16(e, d_ids, S, B, S - 1);
    if (wide_decode(e, B)) pass_decode_wide_bf16(e, d_ids + (S - 1), S, B, ids_out, lp_out, out_stride, out_at_step, d_logits_opt);
    else pass_decode_bf16(e, d_ids + (S - 1), S, B, ids_out, lp_out, out_stride, out_at_step, d_logits_opt);
    return check_hip(e, hipGetLastError(), "kernel launch");
}

// (Re)builds the MFMA-tiled copies from the caller's row-major matrices
// and the vectors W gamma, W beta of every GEMM that follows a LayerNorm.
void tile_weights(he_engine* e) {
    const he_config& c = e->cfg;
    const int H = c.hidden, F = c.ffn;
    if (e->w8) {
        // E4M3 units and row scales of every layer matrix; the vectors W gamma, W beta from the dequantised
        // layer (the weights the GEMMs really multiply by)
        auto quant = [&](const void* src, void* units, float* scales, int R, int K) {
            fp8_row_exponents(e->stream, src, R, K, e->exps_tmp, scales);
            fp8_quant_units(e->stream, src, e->exps_tmp, units, R, K);
        };
        for (int l = 0; l < c.n_layers; ++l) {
            const he_layer_weights& lw = e->layers[l];
            const Scales sc = scales_of(e, l);
            quant(lw.wqkv, e->tiled[l].wqkv, sc.wqkv, 3 * H, H);
            quant(lw.wo, e->tiled[l].wo, sc.wo, H, H);
            quant(lw.w1, e->tiled[l].w1, sc.w1, F, H);
            quant(lw.w2, e->tiled[l].w2, sc.w2, H, F);
            const he_engine::Tiled blk = layer_blocks(e, l);
            const CVec q = cvec_qkv(e, l), f = cvec_fc1(e, l);
            bf16_wvec(e->stream, blk.wqkv, 3 * H, H, lw.ln1_g, lw.ln1_b, q.c1, q.c2);
            bf16_wvec(e->stream, blk.w1, F, H, lw.ln2_g, lw.ln2_b, f.c1, f.c2);
        }
        bf16_tile_rows(e->stream, e->w.lm_head, e->lm_tiled, c.vocab, H);
        const CVec v = cvec_lm(e);
        bf16_wvec(e->stream, e->lm_tiled, c.vocab, H, e->w.lnf_g, e->w.lnf_b, v.c1, v.c2);
        return;
    }
    if (!c.weights_tiled) {  // else the caller's matrices are used in place
        auto tile = [&](const void* src, void* dst, int R, int K, const he_lora* ad) {
            if (ad && ad->a && ad->b && e->lora_rank > 0)
                bf16_tile_rows_lora(e->stream, src, dst, R, K, ad->a, ad->b, e->lora_rank, e->lora_scale);
            else
                bf16_tile_rows(e->stream, src, dst, R, K);
        };
        for (int l = 0; l < c.n_layers; ++l) {
            const he_lora_layer* ad = e->lora.empty() ? nullptr : &e->lora[l];
            tile(e->layers[l].wqkv, e->tiled[l].wqkv, 3 * H, H, ad ? &ad->wqkv : nullptr);
            tile(e->layers[l].wo, e->tiled[l].wo, H, H, ad ? &ad->wo : nullptr);
            tile(e->layers[l].w1, e->tiled[l].w1, F, H, ad ? &ad->w1 : nullptr);
            tile(e->layers[l].w2, e->tiled[l].w2, H, F, ad ? &ad->w2 : nullptr);
        }
        bf16_tile_rows(e->stream, e->w.lm_head, e->lm_tiled, c.vocab, H);
    }
    for (int l = 0; l < c.n_layers; ++l) {
        const he_layer_weights& lw = e->layers[l];
        const CVec q = cvec_qkv(e, l), f = cvec_fc1(e, l);
        bf16_wvec(e->stream, e->tiled[l].wqkv, 3 * H, H, lw.ln1_g, lw.ln1_b, q.c1, q.c2);
        bf16_wvec(e->stream, e->tiled[l].w1, F, H, lw.ln2_g, lw.ln2_b, f.c1, f.c2);
    }
    const CVec v = cvec_lm(e);
    bf16_wvec(e->stream, e->lm_tiled, c.vocab, H, e->w.lnf_g, e->w.lnf_b, v.c1, v.c2);
}

// One pass of the decoder over M = B*S new rows (S = prompt length, or 1 for a
// decode step) followed by the LM head on each sequence's last row and sampling.
he_status run_forward(he_engine* e, const int32_t* d_ids, int B, int S, int32_t* ids_out, float* lp_out,
                      int out_stride, int out_at_step, float* d_logits_opt) {
    if (e->fast) return run_forward_bf16(e, d_ids, B, S, ids_out, lp_out, out_stride, out_at_step, d_logits_opt);
    const he_config& c = e->cfg;
    hipStream_t s = e->stream;
    const int M = B * S, H = c.hidden, F = c.ffn, bf = e->bf16;
    const float qscale = 1.0f / sqrtf((float)e->d);

    plain_embed(s, bf, d_ids, S, e->w.tok_emb, e->w.pos_emb, e->resid, e->st, M, S, H, c.vocab, c.pos_offset);
    const float* pend_y = nullptr;  // GEMM output not yet added to the residual stream
    const void* pend_b = nullptr;
    for (int l = 0; l < c.n_layers; ++l) {
        const he_layer_weights& lw = e->layers[l];
        plain_ln(s, bf, e->resid, pend_y, pend_b, lw.ln1_g, lw.ln1_b, e->abuf, M, H, c.ln_eps, 1, 0, 1);
        plain_gemm(s, bf, e->abuf, lw.wqkv, lw.bqkv, M, 3 * H, H, EPI_QKV, e->qbuf, e->kv, e->st, S, l, H, c.n_heads,
                   c.max_batch, c.max_seq_len, qscale);
        plain_attn(s, bf, e->qbuf, e->kv, e->obuf, e->st, M, S, l, H, c.n_heads, c.max_batch, c.max_seq_len);
        plain_gemm(s, bf, e->obuf, lw.wo, nullptr, M, H, H, EPI_STORE, e->ybuf, nullptr, e->st, S, l, H, c.n_heads,
                   c.max_batch, c.max_seq_len, 1.f);
        plain_ln(s, bf, e->resid, e->ybuf, lw.bo, lw.ln2_g, lw.ln2_b, e->abuf, M, H, c.ln_eps, 1, 0, 1);
        plain_gemm(s, bf, e->abuf, lw.w1, lw.b1, M, F, H, EPI_BIAS_RELU, e->hbuf, nullptr, e->st, S, l, H, c.n_heads,
                   c.max_batch, c.max_seq_len, 1.f);
        plain_gemm(s, bf, e->hbuf, lw.w2, nullptr, M, H, F, EPI_STORE, e->ybuf, nullptr, e->st, S, l, H, c.n_heads,
                   c.max_batch, c.max_seq_len, 1.f);
        pend_y = e->ybuf;
        pend_b = lw.b2;
    }
    // final LayerNorm on each sequence's last row only
    plain_ln(s, bf, e->resid, pend_y, pend_b, e->w.lnf_g, e->w.lnf_b, e->xf, B, H, c.ln_eps, S, S - 1, 0);
    float* logits = d_logits_opt ? d_logits_opt : e->logits;
    plain_lm_head(s, bf, e->xf, e->w.lm_head, logits, B, H, c.vocab);
    launch_sample(s, logits, B, c.vocab, e->st, ids_out, lp_out, out_stride, out_at_step, e->cur_ids);
    if (e->ragged_gen) launch_ragged_post(s, e->st, ids_out, lp_out, e->cur_ids, out_stride, B);
    launch_advance_state(s, e->st, S, 1);
    e->cur_len += S;
    e->step += 1;
    return check_hip(e, hipGetLastError(), "kernel launch");
}

// What a decode step of `rows` rows costs, as far as the row count decides it: 16-row halves of the activation
// slices the weight-streaming GEMMs multiply by (up to 64 rows), 128-row tiles of the matrix-core GEMMs above.
int step_cost_class(const he_engine* e, int rows) {
    return wide_decode(e, rows) ? 4 + (rows + 127) / 128 : (rows + 15) / 16;
}

void drop_step_graph(he_engine* e) {
    if (e->step_graph) (void)hipGraphExecDestroy(e->step_graph);
    if (e->multi_graph) (void)hipGraphExecDestroy(e->multi_graph);
    e->step_graph = e->multi_graph = nullptr;
    e->graph_B = e->graph_G = 0;
    e->graph_ragged = false;
}

// Decode steps of he_generate as HIP graphs (input ids from cur_ids, outputs into the engine's [B, G] generation
// buffers at the device-side step index): one step, and kGraphSteps steps in a row -- between two graph launches
// the device idles for 8-9 us, between two kernels of one graph for 0.7.
constexpr int kGraphSteps = 8;

he_status capture_steps(he_engine* e, int B, int G, int steps, hipGraphExec_t* out) {
    const int len = e->cur_len, step = e->step;
    hipError_t r = hipStreamBeginCapture(e->stream, hipStreamCaptureModeThreadLocal);
    if (r != hipSuccess) return check_hip(e, r, "hipStreamBeginCapture");
    he_status rc = HE_OK;
    for (int i = 0; i < steps && rc == HE_OK; ++i) rc = run_forward(e, e->cur_ids, B, 1, e->gen_ids, e->gen_lp, G, 1, nullptr);
    e->cur_len = len;  // capturing runs nothing
    e->step = step;
    hipGraph_t g = nullptr;
    r = hipStreamEndCapture(e->stream, &g);
    if (rc != HE_OK) {
        if (g) (void)hipGraphDestroy(g);
        return rc;
    }
    if (r != hipSuccess) return check_hip(e, r, "hipStreamEndCapture");
    r = hipGraphInstantiate(out, g, nullptr, nullptr, 0);
    (void)hipGraphDestroy(g);
    if (r != hipSuccess) {
        *out = nullptr;
        return check_hip(e, r, "hipGraphInstantiate");
    }
    return HE_OK;
}

he_status ensure_step_graph(he_engine* e, int B, int G) {
    if (e->step_graph && e->graph_B == B && e->graph_G == G && e->graph_ragged == e->ragged_gen) return HE_OK;
    drop_step_graph(e);
    he_status rc = capture_steps(e, B, G, 1, &e->step_graph);
    // (the run of steps is captured where it is first needed: a call that is already close to its last step, as
    // after rows were dropped late in an answer, gets along with the single step)
    if (rc == HE_OK && G - 1 - e->step >= 2 * kGraphSteps) rc = capture_steps(e, B, G, kGraphSteps, &e->multi_graph);
    if (rc != HE_OK) {
        drop_step_graph(e);
        return rc;
    }
    e->graph_B = B;
    e->graph_ragged = e->ragged_gen;
    e->graph_G = G;
    return HE_OK;
}

const char* check_sampling(const he_sampling* sp) {
    if (!sp) return "sampling is NULL";
    if (sp->mode != 0 && sp->mode != 1) return "sampling mode must be 0 (greedy) or 1 (Gumbel-max)";
    if (sp->mode == 1 && !(sp->temperature > 0.f)) return "temperature must be positive";
    return nullptr;
}

}  // namespace

extern "C" {

size_t he_workspace_bytes(const he_config* cfg) {
    if (check_config(cfg) || check_shape(cfg)) return 0;
    return sizes_of(*cfg).total;
}

he_status he_create(const he_config* cfg, const he_weights* weights, he_engine** out) {
    if (!out) { g_create_error = "out is NULL"; return HE_ERR_INVALID_ARG; }
    if (const char* m = check_config(cfg)) { g_create_error = m; return HE_ERR_INVALID_ARG; }
    if (const char* m = check_shape(cfg)) { g_create_error = m; return HE_ERR_SHAPE; }
    if (!weights || !weights->tok_emb || !weights->pos_emb || !weights->lnf_g || !weights->lnf_b || !weights->lm_head ||
        (cfg->n_layers > 0 && !weights->layers)) {
        g_create_error = "a weight pointer is NULL";
        return HE_ERR_INVALID_ARG;
    }
    for (int l = 0; l < cfg->n_layers; ++l) {
        const he_layer_weights& lw = weights->layers[l];
        const void* ps[] = {lw.ln1_g, lw.ln1_b, lw.wqkv, lw.bqkv, lw.wo, lw.bo, lw.ln2_g, lw.ln2_b, lw.w1, lw.b1, lw.w2, lw.b2};
        for (const void* p : ps)
            if (!p) { g_create_error = "a layer weight pointer is NULL"; return HE_ERR_INVALID_ARG; }
    }
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev) {
        g_create_error = "no such HIP device";
        return HE_ERR_DEVICE;
    }
    if (hipSetDevice(cfg->device) != hipSuccess) { g_create_error = "hipSetDevice failed"; return HE_ERR_DEVICE; }

    he_engine* e = new he_engine();
    e->cfg = *cfg;
    e->d = cfg->hidden / cfg->n_heads;
    e->bf16 = cfg->dtype == HE_BF16;
    e->stream = (hipStream_t)cfg->stream;
    e->w = *weights;
    e->layers.assign(weights->layers, weights->layers + cfg->n_layers);
    e->w.layers = e->layers.data();

    const Sizes z = sizes_of(*cfg);
    hipError_t r = hipSuccess;
    auto A = [&](auto** p, size_t bytes) { if (r == hipSuccess) r = dev_alloc(e, p, bytes); };
    e->fast = is_fast(*cfg);
    A(&e->kv, z.kv);
    e->kv_bytes = z.kv;
    A(&e->st, he_dev_state_bytes(cfg->max_batch));
    A(&e->resid, z.rowsH); A(&e->qbuf, z.rowsH);
    A(&e->logits, z.logits);
    if (!e->fast) {
        A(&e->abuf, z.rowsH); A(&e->obuf, z.rowsH); A(&e->ybuf, z.rowsH);
        A(&e->hbuf, z.rowsF);
        A(&e->xf, z.xf);
    } else {
        const int H = cfg->hidden, F = cfg->ffn;
        e->tiled.resize(cfg->n_layers);
        if (cfg->weights_tiled) {  // the caller's matrices are tiled already: used in place
            for (int l = 0; l < cfg->n_layers; ++l) {
                const he_layer_weights& lw = e->layers[l];
                e->tiled[l] = {const_cast<void*>(lw.wqkv), const_cast<void*>(lw.wo), const_cast<void*>(lw.w1),
                               const_cast<void*>(lw.w2)};
            }
            e->lm_tiled = const_cast<void*>(e->w.lm_head);
        } else if (cfg->weights_fp8) {
            e->w8 = true;
            for (auto& t : e->tiled) {
                A(&t.wqkv, fp8_units_bytes(3 * H, H)); A(&t.wo, fp8_units_bytes(H, H));
                A(&t.w1, fp8_units_bytes(F, H)); A(&t.w2, fp8_units_bytes(H, F));
            }
            A(&e->wscale_buf, (size_t)cfg->n_layers * (5 * H + F) * sizeof(float));
            A(&e->exps_tmp, (size_t)(3 * H > F ? 3 * H : F) * sizeof(int));
            A(&e->scratch.wqkv, bf16_tiled_bytes(3 * H, H)); A(&e->scratch.wo, bf16_tiled_bytes(H, H));
            A(&e->scratch.w1, bf16_tiled_bytes(F, H)); A(&e->scratch.w2, bf16_tiled_bytes(H, F));
            A(&e->lm_tiled, z.tiled_lm);
        } else {
            for (auto& t : e->tiled) {
                A(&t.wqkv, bf16_tiled_bytes(3 * H, H)); A(&t.wo, bf16_tiled_bytes(H, H));
                A(&t.w1, bf16_tiled_bytes(F, H)); A(&t.w2, bf16_tiled_bytes(H, F));
            }
            A(&e->lm_tiled, z.tiled_lm);
        }
        A(&e->ablk, z.ablk); A(&e->oblk, z.ablk); A(&e->hblk, z.hblk); A(&e->xfblk, z.xfblk);
        A(&e->part, z.part); e->part_floats = z.part / sizeof(float); A(&e->stats, z.stats); A(&e->stats_idx, z.stats_idx);
        A(&e->cvec, z.cvec); A(&e->ln_stats, z.ln_stats); A(&e->ln_counters, z.ln_counters);
        A(&e->score_stats, z.score_stats); A(&e->score_tgt, z.gen); A(&e->tail_buf, z.tail);
    }
    A(&e->gen_lp, z.gen); A(&e->gen_ids, z.gen);
    A(&e->cur_ids, cfg->max_batch * sizeof(int32_t));
    if (r != hipSuccess) {
        g_create_error = std::string("device allocation failed: ") + hipGetErrorString(r);
        (void)hipGetLastError();
        free_all(e);
        delete e;
        return r == hipErrorOutOfMemory ? HE_ERR_OOM : HE_ERR_DEVICE;
    }
    // the caller's weights may still be in the making on another stream: wait for the whole device
    r = hipDeviceSynchronize();
    if (r == hipSuccess) r = hipHostMalloc((void**)&e->host_active, sizeof(int), hipHostMallocDefault);
    if (r != hipSuccess) {
        g_create_error = std::string("he_create: ") + hipGetErrorString(r);
        (void)hipGetLastError();
        free_all(e);
        delete e;
        return HE_ERR_DEVICE;
    }
    launch_init_state(e->stream, e->st, cfg->max_batch);
    if (e->fast) {
        // rows of the last 32-row tile beyond the batch are read by the matrix cores (their
        // products are never stored): give them defined contents once
        (void)hipMemsetAsync(e->ablk, 0, z.ablk, e->stream);
        (void)hipMemsetAsync(e->oblk, 0, z.ablk, e->stream);
        (void)hipMemsetAsync(e->hblk, 0, z.hblk, e->stream);
        (void)hipMemsetAsync(e->xfblk, 0, z.xfblk, e->stream);
        (void)hipMemsetAsync(e->ln_stats, 0, z.ln_stats, e->stream);
        (void)hipMemsetAsync(e->ln_counters, 0, z.ln_counters, e->stream);
        tile_weights(e);
    }
    r = hipStreamSynchronize(e->stream);
    if (r == hipSuccess) r = hipGetLastError();
    if (r != hipSuccess) {
        g_create_error = std::string("he_create: ") + hipGetErrorString(r);
        free_all(e);
        delete e;
        return HE_ERR_DEVICE;
    }
    *out = e;
    return HE_OK;
}

he_status he_refresh_weights(he_engine* e) {
    if (!e) return HE_ERR_INVALID_ARG;
    e->lora.clear();
    e->lora_rank = 0;
    he_status rc = check_hip(e, hipDeviceSynchronize(), "he_refresh_weights");  // the update may be on any stream
    if (rc != HE_OK) return rc;
    if (e->fast) tile_weights(e);
    return check_hip(e, hipStreamSynchronize(e->stream), "he_refresh_weights");
}

he_status he_refresh_weights_lora(he_engine* e, const he_lora_layer* adapters, int rank, float scale) {
    if (!e) return HE_ERR_INVALID_ARG;
    if (!adapters || rank < 1) return fail(e, HE_ERR_INVALID_ARG, "he_refresh_weights_lora: adapters NULL or rank < 1");
    if (!e->fast || e->cfg.weights_tiled || e->w8)
        return fail(e, HE_ERR_STATE, "he_refresh_weights_lora: needs dtype bf16, impl 0 and engine-owned bf16 tiled copies (weights_tiled = 0, weights_fp8 = 0)");
    for (int l = 0; l < e->cfg.n_layers; ++l) {
        const he_lora* ps[] = {&adapters[l].wqkv, &adapters[l].wo, &adapters[l].w1, &adapters[l].w2};
        for (const he_lora* p : ps)
            if ((p->a == nullptr) != (p->b == nullptr))
                return fail(e, HE_ERR_INVALID_ARG, "he_refresh_weights_lora: an adapter needs both factors");
    }
    e->lora.assign(adapters, adapters + e->cfg.n_layers);
    e->lora_rank = rank;
    e->lora_scale = scale;
    he_status rc = check_hip(e, hipDeviceSynchronize(), "he_refresh_weights_lora");
    if (rc != HE_OK) return rc;
    tile_weights(e);
    return check_hip(e, hipStreamSynchronize(e->stream), "he_refresh_weights_lora");
}

he_status he_release_arena(he_engine* e) {
    if (!e) return HE_ERR_INVALID_ARG;
    if (e->arena_released) return HE_OK;
    he_status rc = he_reset(e);
    if (rc != HE_OK) return rc;
    rc = check_hip(e, hipStreamSynchronize(e->stream), "he_release_arena");
    if (rc != HE_OK) return rc;
    drop_step_graph(e);  // the captured step holds the arena's address
    for (auto it = e->allocs.begin(); it != e->allocs.end(); ++it)
        if (*it == e->kv) { e->allocs.erase(it); break; }
    rc = check_hip(e, hipFree(e->kv), "he_release_arena");
    e->kv = nullptr;
    e->arena_released = true;
    return rc;
}

he_status he_acquire_arena(he_engine* e) {
    if (!e) return HE_ERR_INVALID_ARG;
    if (!e->arena_released) return HE_OK;
    const hipError_t r = dev_alloc(e, &e->kv, e->kv_bytes);
    if (r != hipSuccess) {
        (void)hipGetLastError();
        return fail(e, r == hipErrorOutOfMemory ? HE_ERR_OOM : HE_ERR_DEVICE,
                    std::string("he_acquire_arena: ") + hipGetErrorString(r));
    }
    e->arena_released = false;
    return HE_OK;
}

he_status he_reset(he_engine* e) {
    if (!e) return HE_ERR_INVALID_ARG;
    e->cur_len = 0; e->step = 0; e->batch = 0;
    e->ragged_gen = false;
    launch_set_state(e->stream, e->st, 0, 0, 1, 0, 1.f, 0);
    // the arrival counters of the k-split GEMMs clear themselves; after a launch that failed half-way they
    // may not have, so a reset clears them too (outside any captured graph)
    if (e->ln_counters) (void)hipMemsetAsync(e->ln_counters, 0, sizes_of(e->cfg).ln_counters, e->stream);
    return check_hip(e, hipGetLastError(), "he_reset");
}

static he_status prefill_impl(he_engine* e, const char* who, const int32_t* d_prompt_ids, const int32_t* d_prompt_lens,
                              bool ragged, int B, int S, const he_sampling* sampling, int32_t* d_next_ids,
                              float* d_logprobs, float* d_logits_opt) {
    if (!e) return HE_ERR_INVALID_ARG;
    const std::string w(who);
    if (!d_prompt_ids || !d_next_ids || !d_logprobs || (ragged && !d_prompt_lens))
        return fail(e, HE_ERR_INVALID_ARG, w + ": NULL buffer");
    if (const char* m = check_sampling(sampling)) return fail(e, HE_ERR_INVALID_ARG, m);
    if (B < 1 || S < 1) return fail(e, HE_ERR_INVALID_ARG, w + ": B and S must be positive");
    if (B > e->cfg.max_batch) return fail(e, HE_ERR_CAPACITY, w + ": B exceeds max_batch");
    if (S > e->cfg.max_seq_len) return fail(e, HE_ERR_CAPACITY, w + ": S exceeds max_seq_len");
    if (S > e->cfg.max_positions) return fail(e, HE_ERR_CAPACITY, w + ": S exceeds max_positions");
    if (e->arena_released) return fail(e, HE_ERR_STATE, w + ": the KV arena is released (call he_acquire_arena)");
    if (e->cur_len != 0) return fail(e, HE_ERR_STATE, w + ": cache is not empty (call he_reset)");
    e->batch = B;
    e->step = 0;
    launch_set_state(e->stream, e->st, 0, 0, 1, sampling->mode, sampling->temperature, sampling->seed);
    if (ragged) launch_set_ragged(e->stream, e->st, d_prompt_lens, B, S, -1, 0);
    return run_forward(e, d_prompt_ids, B, S, d_next_ids, d_logprobs, 1, 0, d_logits_opt);
}

he_status he_prefill(he_engine* e, const int32_t* d_prompt_ids, int B, int S, const he_sampling* sampling,
                     int32_t* d_next_ids, float* d_logprobs, float* d_logits_opt) {
    return prefill_impl(e, "he_prefill", d_prompt_ids, nullptr, false, B, S, sampling, d_next_ids, d_logprobs, d_logits_opt);
}

he_status he_prefill_ragged(he_engine* e, const int32_t* d_prompt_ids, const int32_t* d_prompt_lens, int B, int S,
                            const he_sampling* sampling, int32_t* d_next_ids, float* d_logprobs, float* d_logits_opt) {
    return prefill_impl(e, "he_prefill_ragged", d_prompt_ids, d_prompt_lens, true, B, S, sampling, d_next_ids, d_logprobs,
                        d_logits_opt);
}

he_status he_decode_step(he_engine* e, const int32_t* d_in_ids, const he_sampling* sampling, int32_t* d_next_ids,
                         float* d_logprobs, float* d_logits_opt) {
    if (!e) return HE_ERR_INVALID_ARG;
    if (!d_in_ids || !d_next_ids || !d_logprobs) return fail(e, HE_ERR_INVALID_ARG, "he_decode_step: NULL buffer");
    if (const char* m = check_sampling(sampling)) return fail(e, HE_ERR_INVALID_ARG, m);
    if (e->cur_len == 0 || e->batch == 0) return fail(e, HE_ERR_STATE, "he_decode_step: no prompt has been prefilled");
    if (e->cur_len + 1 > e->cfg.max_seq_len) return fail(e, HE_ERR_CAPACITY, "he_decode_step: KV cache is full");
    if (e->cur_len + 1 > e->cfg.max_positions) return fail(e, HE_ERR_CAPACITY, "he_decode_step: position table exhausted");
    launch_set_state(e->stream, e->st, 0, 0, 0, sampling->mode, sampling->temperature, sampling->seed);
    return run_forward(e, d_in_ids, e->batch, 1, d_next_ids, d_logprobs, 1, 0, d_logits_opt);
}

// How the static array is shared out for a decode step of engine e (256-byte aligned pieces):
// k-split partial sums | column-group statistics | arrival counters | LM-head partials | their ids.
struct StaticLayout { size_t part, ln_stats, ln_counters, stats, stats_idx, total, part_floats; };
static StaticLayout static_layout(const he_engine* e, int B) {
    const he_config& c = e->cfg;
    const int H = c.hidden, F = c.ffn;
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    StaticLayout L{};
    // what the two k-split GEMMs of this step will index, planned exactly as he_decode_step plans them
    const size_t n1 = bf16_store_need(B, H, H, e->part_floats, e->w8), n2 = bf16_store_need(B, H, F, e->part_floats, e->w8);
    L.part_floats = std::max(n1, n2);
    const Sizes z = sizes_of(c);
    L.part = 0;
    L.ln_stats = up(L.part + L.part_floats * sizeof(float));
    L.ln_counters = up(L.ln_stats + z.ln_stats);
    L.stats = up(L.ln_counters + z.ln_counters);
    L.stats_idx = up(L.stats + z.stats);
    L.total = up(L.stats_idx + z.stats_idx);
    return L;
}

he_status he_decode_step_static(he_engine* e, const int32_t* d_in_ids, const he_sampling* sampling, int32_t* d_next_ids,
                                float* d_logprobs, float* d_logits_opt) {
    if (!e) return HE_ERR_INVALID_ARG;
    if (!d_in_ids || !d_next_ids || !d_logprobs) return fail(e, HE_ERR_INVALID_ARG, "he_decode_step_static: NULL buffer");
    if (const char* m = check_sampling(sampling)) return fail(e, HE_ERR_INVALID_ARG, m);
    if (!e->fast) return fail(e, HE_ERR_STATE, "he_decode_step_static: dtype bf16, impl 0 only");
    if (e->cur_len == 0 || e->batch == 0) return fail(e, HE_ERR_STATE, "he_decode_step_static: no prompt has been prefilled");
    if (e->cur_len + 1 > e->cfg.max_seq_len) return fail(e, HE_ERR_CAPACITY, "he_decode_step_static: KV cache is full");
    if (e->cur_len + 1 > e->cfg.max_positions) return fail(e, HE_ERR_CAPACITY, "he_decode_step_static: position table exhausted");
    if (wide_decode(e, e->batch))
        return fail(e, HE_ERR_CAPACITY, "he_decode_step_static: the batch is too large for the weight-streaming decode kernels "
                                        "(at most 64 sequences, 32 with 8-bit weights)");
    const StaticLayout L = static_layout(e, e->batch);
    if (L.total > kStaticScratchBytes)
        return fail(e, HE_ERR_CAPACITY, "he_decode_step_static: this model and batch need " + std::to_string(L.total) +
                                            " bytes of scratch, the static array holds " + std::to_string(kStaticScratchBytes));
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != e->cfg.device)
        return fail(e, HE_ERR_STATE, "he_decode_step_static: the engine's device is not the current device");
    if (dev >= kMaxDevices) return fail(e, HE_ERR_CAPACITY, "he_decode_step_static: device ordinal beyond the table");
    if (!g_static_ptr[dev]) {  // once per device, with that device current
        void* ptr = nullptr;
        const hipError_t r = hipGetSymbolAddress(&ptr, HIP_SYMBOL(he_static_scratch));
        if (r != hipSuccess || !ptr) return check_hip(e, r != hipSuccess ? r : hipErrorInvalidSymbol, "hipGetSymbolAddress");
        g_static_ptr[dev] = ptr;
    }
    unsigned char* base = (unsigned char*)g_static_ptr[dev];
    // The array keeps the last call's contents: statistics and counters start from zero (the k-split partial
    // sums and the LM-head partials are written before they are read).
    const size_t zero_words = (L.stats - L.ln_stats) / sizeof(uint32_t);
    zero_words_kernel<<<(unsigned)std::min<size_t>((zero_words + 255) / 256, 64), 256, 0, e->stream>>>(
        (uint32_t*)(base + L.ln_stats), zero_words);
    launch_set_state(e->stream, e->st, 0, 0, 0, sampling->mode, sampling->temperature, sampling->seed);
    // the step itself: the same launches as he_decode_step, one by one, with the five scratch pointers swapped
    float *part = e->part, *ln_stats = e->ln_stats, *stats = e->stats;
    int *ln_counters = e->ln_counters, *stats_idx = e->stats_idx;
    e->part = (float*)(base + L.part); e->ln_stats = (float*)(base + L.ln_stats); e->ln_counters = (int*)(base + L.ln_counters);
    e->stats = (float*)(base + L.stats); e->stats_idx = (int*)(base + L.stats_idx);
    const bool timing = e->timing;  // the timing hook creates events on demand: off for this call
    e->timing = false;
    const he_status rc = run_forward(e, d_in_ids, e->batch, 1, d_next_ids, d_logprobs, 1, 0, d_logits_opt);
    e->timing = timing;
    e->part = part; e->ln_stats = ln_stats; e->ln_counters = ln_counters; e->stats = stats; e->stats_idx = stats_idx;
    return rc;
}

static he_status generate_impl(he_engine* e, const char* who, const int32_t* d_prompt_ids, const int32_t* d_prompt_lens,
                               bool ragged, int B, int S, int G, const he_sampling* sampling, int eos_id, int pad_id,
                               int32_t* d_out_ids, float* d_out_logprobs, int32_t* d_out_lens) {
    if (!e) return HE_ERR_INVALID_ARG;
    const std::string w(who);
    if (!d_prompt_ids || !d_out_ids || !d_out_logprobs || (ragged && (!d_prompt_lens || !d_out_lens)))
        return fail(e, HE_ERR_INVALID_ARG, w + ": NULL buffer");
    if (const char* m = check_sampling(sampling)) return fail(e, HE_ERR_INVALID_ARG, m);
    if (B < 1 || S < 1 || G < 1) return fail(e, HE_ERR_INVALID_ARG, w + ": B, S and G must be positive");
    if (ragged && (pad_id < 0 || pad_id >= e->cfg.vocab || eos_id >= e->cfg.vocab))
        return fail(e, HE_ERR_INVALID_ARG, w + ": pad_id must be a vocabulary id, eos_id a vocabulary id or negative");
    if (B > e->cfg.max_batch) return fail(e, HE_ERR_CAPACITY, w + ": B exceeds max_batch");
    if ((long)S + G - 1 > e->cfg.max_seq_len) return fail(e, HE_ERR_CAPACITY, w + ": S + G - 1 exceeds max_seq_len");
    if ((long)S + G - 1 > e->cfg.max_positions) return fail(e, HE_ERR_CAPACITY, w + ": S + G - 1 exceeds max_positions");
    if (e->arena_released) return fail(e, HE_ERR_STATE, w + ": the KV arena is released (call he_acquire_arena)");
    he_status rc = he_reset(e);
    if (rc != HE_OK) return rc;
    e->batch = B;
    launch_set_state(e->stream, e->st, 0, 0, 1, sampling->mode, sampling->temperature, sampling->seed);
    if (ragged) {
        launch_set_ragged(e->stream, e->st, d_prompt_lens, B, S, eos_id, pad_id);
        launch_fill_gen(e->stream, e->gen_ids, e->gen_lp, B * G, e->st);  // steps never run stay filler
        e->ragged_gen = true;
    }
    rc = run_forward(e, d_prompt_ids, B, S, e->gen_ids, e->gen_lp, G, 1, nullptr);
    if (rc != HE_OK) return rc;
    // Every later step is the same launch sequence (positions, step number and sampling
    // parameters live in device memory), so it is captured once and replayed.  Capture needs a
    // stream of its own: on the NULL stream, and while per-kernel timing is on, the steps are
    // launched one by one instead -- same kernels, same results.
    const bool use_graph = e->stream != nullptr && !e->timing && G > 2;
    if (use_graph) rc = ensure_step_graph(e, B, G);
    // With an end token, the number of sequences still running is read back every kCheck steps
    // (one small copy and a stream synchronisation): once it is zero the remaining steps are skipped, and once
    // enough sequences have ended for the step to get cheaper, their rows are dropped (bf16 path): the running
    // sequences move up in order, the following steps run on that many rows (a new graph for the new count).
    constexpr int kCheck = 16;
    static_assert(kCheck % kGraphSteps == 0, "a run of steps ends where the running count is read back, not beyond");
    int rows = B;  // rows of a decode step: row r carries the r-th running sequence
    for (int n = 1; n < G && rc == HE_OK; ++n) {  // n: the step about to run; after the body, the last one that ran
        if (use_graph && e->multi_graph && (n - 1) % kGraphSteps == 0 && n + kGraphSteps <= G) {
            rc = check_hip(e, hipGraphLaunch(e->multi_graph, e->stream), "hipGraphLaunch");
            e->cur_len += kGraphSteps;
            e->step += kGraphSteps;
            n += kGraphSteps - 1;
        } else if (use_graph) {
            rc = check_hip(e, hipGraphLaunch(e->step_graph, e->stream), "hipGraphLaunch");
            e->cur_len += 1;
            e->step += 1;
        } else {
            rc = run_forward(e, e->cur_ids, rows, 1, e->gen_ids, e->gen_lp, G, 1, nullptr);
        }
        if (rc == HE_OK && ragged && eos_id >= 0 && n % kCheck == 0 && n + 1 < G) {
            hipError_t r = hipMemcpyAsync(e->host_active, &e->st->n_active, sizeof(int), hipMemcpyDeviceToHost, e->stream);
            if (r == hipSuccess) r = hipStreamSynchronize(e->stream);
            rc = check_hip(e, r, "reading the active count");
            const int active = *e->host_active;
            if (rc == HE_OK && active == 0) break;
            if (rc == HE_OK && e->fast && active < rows && step_cost_class(e, active) < step_cost_class(e, rows)) {
                launch_compact_rows(e->stream, e->st, rows);
                rows = active;
                if (use_graph) rc = ensure_step_graph(e, rows, G);
            }
        }
    }
    e->last_rows = rows;
    if (rows != B) launch_identity_rows(e->stream, e->st);  // later he_decode_step calls: one row per sequence again
    if (rc != HE_OK) return rc;
    launch_copy_out(e->stream, e->gen_ids, e->gen_lp, d_out_ids, d_out_logprobs, B * G);
    if (ragged) launch_copy_lens(e->stream, e->st, d_out_lens, B);
    e->ragged_gen = false;
    return check_hip(e, hipGetLastError(), who);
}

he_status he_generate(he_engine* e, const int32_t* d_prompt_ids, int B, int S, int G, const he_sampling* sampling,
                      int32_t* d_out_ids, float* d_out_logprobs) {
    return generate_impl(e, "he_generate", d_prompt_ids, nullptr, false, B, S, G, sampling, -1, 0, d_out_ids,
                         d_out_logprobs, nullptr);
}

he_status he_generate_ragged(he_engine* e, const int32_t* d_prompt_ids, const int32_t* d_prompt_lens, int B, int S, int G,
                             const he_sampling* sampling, int eos_id, int pad_id, int32_t* d_out_ids,
                             float* d_out_logprobs, int32_t* d_out_lens) {
    return generate_impl(e, "he_generate_ragged", d_prompt_ids, d_prompt_lens, true, B, S, G, sampling, eos_id, pad_id,
                         d_out_ids, d_out_logprobs, d_out_lens);
}

he_status he_score(he_engine* e, const int32_t* d_ids, int B, int T, float* d_out_logprobs) {
    if (!e) return HE_ERR_INVALID_ARG;
    if (!d_ids || !d_out_logprobs) return fail(e, HE_ERR_INVALID_ARG, "he_score: NULL buffer");
    if (B < 1 || T < 2) return fail(e, HE_ERR_INVALID_ARG, "he_score: B must be positive and T at least 2");
    if (B > e->cfg.max_batch) return fail(e, HE_ERR_CAPACITY, "he_score: B exceeds max_batch");
    if (T > e->cfg.max_seq_len) return fail(e, HE_ERR_CAPACITY, "he_score: T exceeds max_seq_len");
    if (T > e->cfg.max_positions) return fail(e, HE_ERR_CAPACITY, "he_score: T exceeds max_positions");
    if (e->arena_released) return fail(e, HE_ERR_STATE, "he_score: the KV arena is released (call he_acquire_arena)");
    he_status rc = he_reset(e);
    if (rc != HE_OK) return rc;
    const he_config& c = e->cfg;
    hipStream_t s = e->stream;
    const int M = B * T, H = c.hidden, F = c.ffn, V = c.vocab;
    if (e->fast) {
        const void* pend_b = nullptr;
        int pend_ks = 1, pend_sc = 0;
        pass_tiled_bf16(e, d_ids, T, B, T, true, &pend_b, &pend_ks, -1, &pend_sc);
        bf16_ln(s, e->resid, c.n_layers ? e->part : nullptr, pend_ks, (size_t)M * H, pend_b, e->w.lnf_g, e->w.lnf_b, e->ablk,
                M, H, c.ln_eps, 1, 0, 0, pend_sc);
        bf16_score_head(s, e->lm_tiled, e->ablk, M, T, V, H, d_ids, e->score_stats, e->score_tgt, d_out_logprobs);
    } else {
        const int bf = e->bf16;
        const float qscale = 1.0f / sqrtf((float)e->d);
        plain_embed(s, bf, d_ids, T, e->w.tok_emb, e->w.pos_emb, e->resid, e->st, M, T, H, V, c.pos_offset);
        const float* pend_y = nullptr;
        const void* pend_b = nullptr;
        for (int l = 0; l < c.n_layers; ++l) {
            const he_layer_weights& lw = e->layers[l];
            plain_ln(s, bf, e->resid, pend_y, pend_b, lw.ln1_g, lw.ln1_b, e->abuf, M, H, c.ln_eps, 1, 0, 1);
            plain_gemm(s, bf, e->abuf, lw.wqkv, lw.bqkv, M, 3 * H, H, EPI_QKV, e->qbuf, e->kv, e->st, T, l, H, c.n_heads,
                       c.max_batch, c.max_seq_len, qscale);
            plain_attn(s, bf, e->qbuf, e->kv, e->obuf, e->st, M, T, l, H, c.n_heads, c.max_batch, c.max_seq_len);
            plain_gemm(s, bf, e->obuf, lw.wo, nullptr, M, H, H, EPI_STORE, e->ybuf, nullptr, e->st, T, l, H, c.n_heads,
                       c.max_batch, c.max_seq_len, 1.f);
            plain_ln(s, bf, e->resid, e->ybuf, lw.bo, lw.ln2_g, lw.ln2_b, e->abuf, M, H, c.ln_eps, 1, 0, 1);
            plain_gemm(s, bf, e->abuf, lw.w1, lw.b1, M, F, H, EPI_BIAS_RELU, e->hbuf, nullptr, e->st, T, l, H, c.n_heads,
                       c.max_batch, c.max_seq_len, 1.f);
            plain_gemm(s, bf, e->hbuf, lw.w2, nullptr, M, H, F, EPI_STORE, e->ybuf, nullptr, e->st, T, l, H, c.n_heads,
                       c.max_batch, c.max_seq_len, 1.f);
            pend_y = e->ybuf;
            pend_b = lw.b2;
        }
        // final LayerNorm of every row into abuf, then the LM head max_batch rows at a time
        plain_ln(s, bf, e->resid, pend_y, pend_b, e->w.lnf_g, e->w.lnf_b, e->abuf, M, H, c.ln_eps, 1, 0, 0);
        for (int r0 = 0; r0 < M; r0 += c.max_batch) {
            const int n = M - r0 < c.max_batch ? M - r0 : c.max_batch;
            plain_lm_head(s, bf, e->abuf + (size_t)r0 * H, e->w.lm_head, e->logits, n, H, V);
            plain_score_rows(s, e->logits, d_ids, r0, n, T, V, d_out_logprobs);
        }
    }
    rc = check_hip(e, hipGetLastError(), "he_score");
    const he_status rc2 = he_reset(e);  // the arena held this sequence's keys and values only as scratch
    return rc != HE_OK ? rc : rc2;
}

he_status he_destroy(he_engine* e) {
    if (!e) return HE_OK;
    (void)hipStreamSynchronize(e->stream);
    drop_step_graph(e);
    for (hipEvent_t ev : e->ev_pool) (void)hipEventDestroy(ev);
    free_all(e);
    delete e;
    return HE_OK;
}

he_status he_timing_enable(he_engine* e, int on) {
    if (!e) return HE_ERR_INVALID_ARG;
    e->timing = on != 0;
    e->ev_used.clear();
    e->ev_next = 0;
    return HE_OK;
}

he_status he_timing_read(he_engine* e, double* ms_per_class, long* launches_per_class, int n_classes) {
    if (!e || !ms_per_class || !launches_per_class || n_classes < HE_K_COUNT) return HE_ERR_INVALID_ARG;
    for (int i = 0; i < n_classes; ++i) { ms_per_class[i] = 0.0; launches_per_class[i] = 0; }
    const hipError_t r = hipStreamSynchronize(e->stream);
    if (r != hipSuccess) return check_hip(e, r, "he_timing_read");
    for (const auto& u : e->ev_used) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e->ev_pool[u.second], e->ev_pool[u.second + 1]) != hipSuccess) continue;
        ms_per_class[u.first] += ms;
        launches_per_class[u.first] += 1;
    }
    e->ev_used.clear();
    e->ev_next = 0;
    return HE_OK;
}

const char* he_last_error(const he_engine* e) { return e ? e->err.c_str() : g_create_error.c_str(); }

int he_cache_len(const he_engine* e) { return e ? e->cur_len : -1; }
int he_last_step_rows(const he_engine* e) { return e ? e->last_rows : -1; }

size_t he_tiled_bytes(int rows, int cols) {
    if (rows <= 0 || cols <= 0 || cols % 16) return 0;
    return bf16_tiled_bytes(rows, cols);
}

he_status he_tile_matrix(const void* d_src, void* d_dst, int rows, int cols, void* stream) {
    if (!d_src || !d_dst || d_src == d_dst || rows <= 0 || cols <= 0 || cols % 16) return HE_ERR_INVALID_ARG;
    bf16_tile_rows((hipStream_t)stream, d_src, d_dst, rows, cols);
    return hipGetLastError() == hipSuccess ? HE_OK : HE_ERR_DEVICE;
}

he_status he_tile_matrix_lora(const void* d_src, void* d_dst, int rows, int cols, const void* d_a, const void* d_b,
                              int rank, float scale, void* stream) {
    if (!d_src || !d_dst || d_src == d_dst || rows <= 0 || cols <= 0 || cols % 16 || !d_a || !d_b || rank < 1)
        return HE_ERR_INVALID_ARG;
    bf16_tile_rows_lora((hipStream_t)stream, d_src, d_dst, rows, cols, d_a, d_b, rank, scale);
    return hipGetLastError() == hipSuccess ? HE_OK : HE_ERR_DEVICE;
}

he_status he_fp8_quantize_rows(const void* d_src, int rows, int cols, void* d_codes, int32_t* d_exps, float* d_scales,
                               void* stream) {
    if (!d_src || !d_codes || !d_exps || !d_scales || rows <= 0 || cols <= 0 || cols % 8) return HE_ERR_INVALID_ARG;
    fp8_row_exponents((hipStream_t)stream, d_src, rows, cols, d_exps, d_scales);
    fp8_quant_rows((hipStream_t)stream, d_src, d_exps, d_codes, rows, cols);
    return hipGetLastError() == hipSuccess ? HE_OK : HE_ERR_DEVICE;
}

he_status he_plan_decode_gemm(int M, int N, int K, int ksplit_allowed, size_t scratch_floats, int cus, int* unit_rows,
                              int* units_per_workgroup, int* ksplit) {
    if (M < 1 || N < 1 || K < 1 || N % 32 || K % 32 || !unit_rows || !units_per_workgroup || !ksplit) return HE_ERR_INVALID_ARG;
    bf16_plan_query(M, N, K, ksplit_allowed, scratch_floats, cus, unit_rows, units_per_workgroup, ksplit);
    return HE_OK;
}

he_status he_plan_prompt_gemm(int M, int N, int K, int may_cut, size_t scratch_floats, int cus, int* tile_cols,
                              int* ksplit, int* split_col) {
    if (M < 1 || N < 1 || K < 1 || N % 32 || K % 32 || cus < 0 || !tile_cols || !ksplit || !split_col) return HE_ERR_INVALID_ARG;
    bf16_tiled_plan_query(M, N, K, may_cut, scratch_floats, cus, tile_cols, ksplit, split_col);
    return HE_OK;
}

he_status he_decode_scratch_account(const he_config* cfg, int B, int which, int cus, he_scratch_account* out) {
    if (!out || check_config(cfg) || check_shape(cfg) || !is_fast(*cfg)) return HE_ERR_INVALID_ARG;
    if (B < 1 || B > cfg->max_batch || B > 64 || (which != 0 && which != 1) || cus < 0) return HE_ERR_INVALID_ARG;
    if (cfg->weights_fp8 && B > 32) return HE_ERR_INVALID_ARG;  // those steps take the wide path
    const Sizes z = sizes_of(*cfg);
    const int H = cfg->hidden, K = which ? cfg->ffn : H;
    const size_t cap = z.part / sizeof(float);
    size_t need = 0;
    int groups = 0;
    bf16_store_footprint(B, H, K, cap, cfg->weights_fp8, cus, &out->scratch_floats, &need, &out->counters, &groups,
                         &out->ksplit);
    out->scratch_reserved = cap;
    out->static_floats = need;
    out->counters_reserved = (int)(z.ln_counters / sizeof(int));
    out->stat_pairs = (B + 31) / 32 * groups * 32;
    out->stat_pairs_reserved = (int)(z.ln_stats / (2 * sizeof(float)));
    return HE_OK;
}

he_status he_arrival_counters_nonzero(he_engine* e, int* nonzero) {
    if (!e || !nonzero) return HE_ERR_INVALID_ARG;
    if (!e->fast || !e->ln_counters) return fail(e, HE_ERR_STATE, "he_arrival_counters_nonzero: bf16 path only");
    const size_t n = sizes_of(e->cfg).ln_counters / sizeof(int);
    std::vector<int> host(n);
    hipError_t r = hipStreamSynchronize(e->stream);
    if (r == hipSuccess) r = hipMemcpy(host.data(), e->ln_counters, n * sizeof(int), hipMemcpyDeviceToHost);
    if (r != hipSuccess) return check_hip(e, r, "he_arrival_counters_nonzero");
    int c = 0;
    for (int v : host) c += v != 0;
    *nonzero = c;
    return HE_OK;
}

he_status he_kernel_sweep(he_engine* e, int kernel_class, int reps) {
    if (!e) return HE_ERR_INVALID_ARG;
    if (!e->fast) return fail(e, HE_ERR_STATE, "he_kernel_sweep: bf16 path only");
    if (kernel_class != HE_K_OUT_PROJ && kernel_class != HE_K_FC1 && kernel_class != HE_K_FC2)
        return fail(e, HE_ERR_INVALID_ARG, "he_kernel_sweep: class must be HE_K_OUT_PROJ, HE_K_FC1 or HE_K_FC2");
    if (e->batch == 0 || reps < 1) return fail(e, HE_ERR_STATE, "he_kernel_sweep: needs a prefilled batch and reps >= 1");
    const he_config& c = e->cfg;
    const int B = e->batch, H = c.hidden, F = c.ffn;
    bf16_gemm_args base;
    base.st = e->st; base.S = 1; base.H = H; base.n_heads = c.n_heads; base.max_batch = c.max_batch;
    base.max_seq = c.max_seq_len;
    const size_t split = (size_t)B * H;
    for (int r = 0; r < reps; ++r)
        for (int l = 0; l < c.n_layers; ++l) {
            bf16_gemm_args a = base;
            if (wide_decode(e, B)) {  // the GEMMs of the wide decode step
                if (e->w8) return fail(e, HE_ERR_STATE, "he_kernel_sweep: with 8-bit weights only for batches up to 32");
                if (kernel_class == HE_K_FC1) {
                    a.bias = e->layers[l].b1; a.out_blocks = e->hblk;
                    bf16_gemm_tiled_ksplit(e->stream, EPI_BIAS_RELU, e->tiled[l].w1, e->ablk, B, F, H,
                                           bf16_tiled_ksplit(B, F, H), e->part, (size_t)B * F, a);
                } else if (kernel_class == HE_K_FC2) {
                    bf16_gemm_tiled_ksplit(e->stream, EPI_STORE, e->tiled[l].w2, e->hblk, B, H, F,
                                           bf16_tiled_ksplit(B, H, F), e->part, split, a);
                } else {
                    bf16_gemm_tiled_ksplit(e->stream, EPI_STORE, e->tiled[l].wo, e->oblk, B, H, H,
                                           bf16_tiled_ksplit(B, H, H), e->part, split, a);
                }
                continue;
            }
            if (kernel_class == HE_K_FC1) {
                a.bias = e->layers[l].b1; a.out_blocks = e->hblk;
                int gw1, ks1;
                if (e->w8) bf16_store_plan_w8(H, H, e->part_floats, &gw1, &ks1);
                else bf16_store_plan(B, H, H, e->part_floats, &gw1, &ks1);
                if (e->w8) a.wscale = scales_of(e, l).w1;
                a.ln_stats = e->ln_stats; a.ln_gw = gw1; a.ln_groups = (H + a.ln_gw - 1) / a.ln_gw; a.ln_cols = H;
                a.ln_eps = c.ln_eps; a.c1 = cvec_fc1(e, l).c1; a.c2 = cvec_fc1(e, l).c2;
                bf16_gemm_skinny(e->stream, EPI_BIAS_RELU, e->tiled[l].w1, e->ablk, B, F, H, 1, a);
            } else {
                // as in a decode step: the last workgroup of each column group folds the partial sums
                // into the residual rows and rewrites the blocks and statistics the next GEMM reads
                const bool fc2 = kernel_class == HE_K_FC2;
                int gw, ks;
                if (e->w8) bf16_store_plan_w8(H, fc2 ? F : H, e->part_floats, &gw, &ks);
                else bf16_store_plan(B, H, fc2 ? F : H, e->part_floats, &gw, &ks);
                if (e->w8) a.wscale = fc2 ? scales_of(e, l).w2 : scales_of(e, l).wo;
                a.out = e->part; a.out_split = split; a.out_capacity = e->part_floats; a.resid = e->resid;
                a.bias = fc2 ? e->layers[l].b2 : e->layers[l].bo;
                a.gamma = fc2 ? e->layers[l].ln1_g : e->layers[l].ln2_g;
                a.out_blocks = e->ablk; a.stats_out = e->ln_stats; a.counters = e->ln_counters;
                if (fc2) bf16_gemm_skinny(e->stream, EPI_STORE_LN, e->tiled[l].w2, e->hblk, B, H, F, ks, a);
                else bf16_gemm_skinny(e->stream, EPI_STORE_LN, e->tiled[l].wo, e->oblk, B, H, H, ks, a);
            }
        }
    return check_hip(e, hipGetLastError(), "he_kernel_sweep");
}

he_status he_calibration_copy(const void* d_src, void* d_dst, size_t bytes, void* stream) {
    if (!d_src || !d_dst || bytes % 16) return HE_ERR_INVALID_ARG;
    if (bytes == 0) return HE_OK;
    launch_calibration_copy((hipStream_t)stream, d_src, d_dst, bytes);
    return hipGetLastError() == hipSuccess ? HE_OK : HE_ERR_DEVICE;
}

he_status he_rng_words(uint64_t seed, uint32_t b, uint32_t n, uint32_t v0, int count, uint32_t* d_out, void* stream) {
    if (!d_out || count < 0) return HE_ERR_INVALID_ARG;
    if (count == 0) return HE_OK;
    launch_rng_words((hipStream_t)stream, seed, b, n, v0, count, d_out);
    return hipGetLastError() == hipSuccess ? HE_OK : HE_ERR_DEVICE;
}

}  // extern "C"
