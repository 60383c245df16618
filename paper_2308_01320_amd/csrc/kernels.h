// Host-side launchers of the engine's kernels (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

struct he_dev_state;

enum { EPI_STORE = 0, EPI_BIAS_RELU = 1, EPI_QKV = 2, EPI_STORE_LN = 3 };

// ---- plain kernels (kernels_plain.hip): float activations, row-major; bf16 != 0 selects bf16 storage
void plain_embed(hipStream_t s, int bf16, const int32_t* ids, int id_stride, const void* tok, const void* pos, float* x,
                 const he_dev_state* st, int M, int S, int H, int V, int pos_offset);
void plain_ln(hipStream_t s, int bf16, float* r, const float* y, const void* ybias, const void* g, const void* b,
              float* a, int rows, int H, float eps, int in_mul, int in_add, int writeback);
void plain_gemm(hipStream_t s, int bf16, const float* A, const void* W, const void* bias, int M, int N, int K, int epi,
                float* out, void* kv, const he_dev_state* st, int S, int layer, int H, int n_heads, int max_batch,
                int max_seq, float qscale);
void plain_attn(hipStream_t s, int bf16, const float* q, const void* kv, float* o, const he_dev_state* st, int M, int S,
                int layer, int H, int n_heads, int max_batch, int max_seq);
void plain_lm_head(hipStream_t s, int bf16, const float* xf, const void* W, float* logits, int B, int H, int V);
// rows row0 .. row0+n-1 of the M = B*S positions, given their logits [n][V]: out[b][t] = log_softmax(z)[ids[m+1]]
void plain_score_rows(hipStream_t s, const float* logits, const int32_t* ids, int row0, int n, int S, int V, float* out);

// ---- shared small kernels
void launch_sample(hipStream_t s, const float* logits, int B, int V, const he_dev_state* st, int32_t* ids_out,
                   float* lp_out, int out_stride, int out_at_step, int32_t* cur_ids);
void launch_set_state(hipStream_t s, he_dev_state* st, int cur_len, int step, int set_pos, int mode, float temperature,
                      uint64_t seed);
void launch_advance_state(hipStream_t s, he_dev_state* st, int tokens, int steps);
void launch_init_state(hipStream_t s, he_dev_state* st, int max_batch);
// sequences of different lengths: B left-padded rows of S entries, lens[b] of them tokens
void launch_set_ragged(hipStream_t s, he_dev_state* st, const int32_t* lens, int B, int S, int eos_id, int pad_id);
void launch_ragged_post(hipStream_t s, he_dev_state* st, int32_t* gen_ids, float* gen_lp, int32_t* cur_ids, int G, int B);
void launch_fill_gen(hipStream_t s, int32_t* ids, float* lp, int count, const he_dev_state* st);
// Drops the rows of sequences that have ended from the row -> sequence map of the decode steps (`rows` rows so far;
// afterwards as many as sequences are running), and the map back to one row per sequence.
void launch_compact_rows(hipStream_t s, he_dev_state* st, int rows);
void launch_identity_rows(hipStream_t s, he_dev_state* st);
void launch_copy_lens(hipStream_t s, const he_dev_state* st, int32_t* out, int B);
void launch_rng_words(hipStream_t s, uint64_t seed, uint32_t b, uint32_t n, uint32_t v0, int count, uint32_t* out);
void launch_calibration_copy(hipStream_t s, const void* src, void* dst, size_t bytes);
void launch_copy_out(hipStream_t s, const int32_t* ids, const float* lp, int32_t* out_ids, float* out_lp, int count);

// ---- bf16 path (bf16_*.hip): matrix-core operands are tiled blocks of IEEE halves, see bf16_common.h
struct bf16_gemm_args {
    const void* bias = nullptr;      // bf16 [N]
    float* out = nullptr;            // EPI_STORE: partials [ksplit][M][N]; EPI_QKV: q [M][H]
    size_t out_split = 0;            // elements between k-splits
    int split_col = 0;               // EPI_STORE on the big tiles with a k-split: first column that has one
    int tile_na = 0;                 // ... and the tiles' width as bf16_tiled_store_split planned it
    size_t out_capacity = 0;         // EPI_STORE_LN: floats `out` can hold (0 = not checked)
    void* out_blocks = nullptr;      // EPI_BIAS_RELU: tiled half output
    void* kv = nullptr;              // EPI_QKV
    const he_dev_state* st = nullptr;
    int S = 1, layer = 0, H = 0, n_heads = 0, max_batch = 0, max_seq = 0;
    float qscale = 1.f;
    // LayerNorm folded into the GEMM that consumes it (EPI_BIAS_RELU, EPI_QKV, LM head; decode rows):
    // the activations are gamma * x and ln_stats holds per-column-group statistics of x
    const float* ln_stats = nullptr;  // [m_tiles][ln_groups][32][2] (+ 1 KiB of padding); null = not folded
    int ln_groups = 0, ln_gw = 0, ln_cols = 0;
    float ln_eps = 0.f;
    const float* c1 = nullptr;        // [N padded to 32] W gamma
    const float* c2 = nullptr;        // [N padded to 32] W beta
    // EPI_STORE_LN: k-split sum + bias + residual, gamma * x blocks (out_blocks) and statistics
    float* resid = nullptr;           // [M][N]
    const void* gamma = nullptr;      // bf16 [N] (the caller's parameter)
    float* stats_out = nullptr;       // [m_tiles][groups][32][2]
    int* counters = nullptr;          // [groups * m_tiles] zeros
    // 8-bit weights (bf16_gemm_skinny only): Wp holds E4M3 codes in 16-row units, wscale [N] the row scales 2^e
    const float* wscale = nullptr;
};
size_t bf16_tiled_bytes(int rows, int K);
void bf16_tile_rows(hipStream_t s, const void* src, void* dst, int R, int K);
// dst = tiled bf16(src + scale * B A): A bf16 [rank, K], B bf16 [R, rank]
void bf16_tile_rows_lora(hipStream_t s, const void* src, void* dst, int R, int K, const void* A, const void* B, int rank,
                         float scale);
// decode-shaped STORE GEMM of M rows: weight tiles per workgroup (its column group is 32*nt wide) and k-splits
void bf16_store_shape(int M, int N, int K, int* nt, int* ks);
// EPI_STORE_LN GEMM of M <= 32 rows: columns per workgroup (= per group of LayerNorm statistics) and k-splits;
// capacity = floats of k-split scratch available (the value passed as bf16_gemm_args.out_capacity)
void bf16_store_plan(int M, int N, int K, size_t capacity, int* group_cols, int* ks);
// floats of k-split scratch that launch may index (upper bound); w8 != 0: the 8-bit-weight plan
size_t bf16_store_need(int M, int N, int K, size_t capacity, int w8);
// What that launch indexes, from the launcher's own choice of kernel variant and grid (host logic, no launch).
// cus: compute units to plan for (0 = the current device's).  need_floats: what bf16_store_need answers.
void bf16_store_footprint(int M, int N, int K, size_t capacity, int w8, int cus, size_t* scratch_floats,
                          size_t* need_floats, int* cells, int* stat_groups, int* ksplit);
// the launch plan itself (host logic only; cus > 0 overrides the device's CU count): rows per unit (32 or 16),
// units per workgroup, k-splits; store != 0 for the k-split GEMMs
void bf16_plan_query(int M, int N, int K, int store, size_t capacity, int cus, int* unit_rows, int* per_wg, int* ks);
void bf16_embed_ln(hipStream_t s, const int32_t* ids, int id_stride, const void* tok, const void* pos,
                   const he_dev_state* st, int B, int H, int V, int pos_offset, int gw, const void* gamma, float* r,
                   void* x_blocks, float* stats);
// rows b*S + S-1 of r and q ([B*S][H] floats) -> rows b of r_out and q_out ([B][H])
void bf16_gather_last_rows(hipStream_t s, const float* r, const float* q, float* r_out, float* q_out, int B, int S, int H);
void bf16_wvec(hipStream_t s, const void* Wp, int N, int K, const void* gamma, const void* beta, float* c1, float* c2);
// rows in slices of 32 (a decode step of up to 32 sequences): EPI_BIAS_RELU, EPI_QKV or EPI_STORE_LN;
// X: the activations as tiled half blocks; ksplit is ignored (the plan decides)
void bf16_gemm_skinny(hipStream_t s, int mode, const void* Wp, const void* X, int M, int N, int K, int ksplit,
                      const bf16_gemm_args& a);
// many rows (prompt pass)
void bf16_gemm_tiled(hipStream_t s, int mode, const void* Wp, const void* X, int M, int N, int K, const bf16_gemm_args& a);
// a decode step of more than 32 rows: the same tiles, cut into k ranges so that they fill the chip.  The
// partial sums go to part [ksplit][M][N]; for EPI_STORE the caller's LayerNorm adds them, for the other
// modes a second kernel adds them and applies the epilogue.
int bf16_tiled_ksplit(int M, int N, int K);
// k ranges per tile for a many-row MODE_STORE GEMM whose tiles do not come out in whole rounds of one per CU
// (1 if they do, or if ks x M x N partial sums do not fit capacity_floats)
int bf16_tiled_store_ksplit(int M, int N, int K, size_t capacity_floats);
// ... and for the 256 x 256 tiles: *ks k ranges for the tiles of columns >= *split_col, one for the columns before
// (*na: the tiles' width in 64 columns, to be handed on in bf16_gemm_args.tile_na; 0 for other tile shapes)
void bf16_tiled_store_split(int M, int N, int K, size_t capacity_floats, int* ks, int* split_col, int* na);
// The plan of a many-row GEMM for a planner query (cus: compute units to plan for, 0 = the current device's)
void bf16_tiled_plan_query(int M, int N, int K, int may_cut, size_t capacity_floats, int cus, int* tile_cols, int* ks,
                           int* split_col);
void bf16_gemm_tiled_ksplit(hipStream_t s, int mode, const void* Wp, const void* X, int M, int N, int K, int ksplit,
                            float* part, size_t part_split, const bf16_gemm_args& a);
// ---- 8-bit weight storage: E4M3 codes with one power-of-two scale per row
size_t fp8_units_bytes(int rows, int K);  // codes in the half-tile kernel's units: [rows/16][K/64][64 lanes][16 bytes]
void fp8_row_exponents(hipStream_t s, const void* src, int R, int K, int* exps, float* scales);  // e[n], 2^e[n]
void fp8_quant_rows(hipStream_t s, const void* src, const int* exps, void* codes, int R, int K);  // row-major codes
void fp8_quant_units(hipStream_t s, const void* src, const int* exps, void* units, int R, int K);
// units -> half 32x16 blocks (what the tiled GEMMs read)
void fp8_dequant_units(hipStream_t s, const void* units, const float* scales, void* dst_blocks, int R, int K);
void bf16_store_plan_w8(int N, int K, size_t capacity, int* group_cols, int* ks);
void bf16_lm_head(hipStream_t s, const void* Wp, const void* X, int B, int V, int K,
                  const he_dev_state* st, float* logits_opt, float* stats, int* stats_idx, int32_t* ids_out,
                  float* lp_out, int out_stride, int out_at_step, int32_t* cur_ids,
                  const bf16_gemm_args* fold = nullptr);
// LM head over all M = B*S positions fused with log-softmax and the gather of each position's next
// token: out [B][S-1]; stats [M][bf16_score_parts(V)][2] and tgt [M] are scratch
int bf16_score_parts(int V);
void bf16_score_head(hipStream_t s, const void* Wp, const void* X, int M, int S, int V, int K,
                     const int32_t* ids, float* stats, float* tgt, float* out);
// split_col: with two k ranges, the first column that has the second partial sum (0: every column; a multiple of 256)
void bf16_ln(hipStream_t s, float* r, const float* part, int ksplit, size_t part_split, const void* pbias,
             const void* gamma, const void* beta, void* a_blocks, int rows, int H, float eps, int in_mul, int in_add,
             int writeback, int split_col = 0);
void bf16_attn(hipStream_t s, const float* q, const void* kv, void* o_blocks, const he_dev_state* st, int M, int S,
               int layer, int H, int n_heads, int max_batch, int max_seq);
