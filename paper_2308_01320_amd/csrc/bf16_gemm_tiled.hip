// bf16 path: the LDS-tiled MFMA GEMM of prompt rows, scoring passes and wide decode steps.
#include "bf16_common.h"

using namespace he_bf16;

namespace {

// ----------------------------------------------------------------- tiled GEMM (prompt pass)
//
// 256 (n) x 128 (m) output tile per workgroup, four wavefronts in a 2x2 grid of
// 128x64 sub-tiles (4x2 MFMA tiles each: 8 LDS operand reads feed 16 MFMAs per
// k-block).  Operands arrive as 1 KiB blocks whose layout is the lane order, so
// they are moved global -> LDS directly (global_load_lds, 16 bytes per lane, no
// staging registers) into a ring of stages; loads run several stages (about 3000
// MFMA cycles) ahead of the arithmetic, which is what it takes to cover an L2 /
// infinity-cache round trip; one barrier per stage.
//
// Two ring shapes.  PAIR = 0: four stages of two k-blocks (128 KiB), one workgroup per CU -- for launches
// with fewer tiles than CUs (few rows; the k-split GEMMs of a wide decode step).  PAIR = 1: five stages of
// one k-block (80 KiB) and at most 256 registers, so that TWO workgroups share a CU: while one of them
// sits at its barrier, waits for operands or writes its results, the other one's MFMAs keep the matrix
// cores busy (one workgroup per CU left them idle 40-50 % of the time, and a 256-row tile that moves a
// quarter less operand data per flop, but fits only once, still 39 %).

constexpr int TN = 256;
constexpr int TNB = TN / 32;   // 32-row operand blocks on the n side
// MW: 32-row m blocks per wavefront (2: a 128-row m tile; 4: a 256-row m tile whose 16 accumulator tiles take a
// wavefront's whole register file, so one workgroup per CU)
template <int PAIR, int MW> struct TiledShape {
    static constexpr int TMB = 2 * MW;                 // 32-row operand blocks on the m side
    static constexpr int TMR = TMB * 32;               // rows of the m tile
    static constexpr int KSTAGE = PAIR ? 1 : 2;        // k-blocks (16 values of k each) per stage
    static constexpr int NSTG = PAIR ? (MW == 4 ? 8 : 5) : 4;  // ring depth
    static constexpr int STAGE_BLOCKS = (TNB + TMB) * KSTAGE;
};

template <int MODE, int PAIR, int MW>
__global__ __launch_bounds__(256, (PAIR && MW == 2) ? 2 : 1) void gemm_tiled_kernel(const u32x4* __restrict__ Wp, const u32x4* __restrict__ Xhi,
                                                         int KB, int NT32, int MT32,
                                                         int tiles_n, int tiles_m, int ksplit, Epi p) {
    // ring[stage][block][lane]; blocks of a stage: W tile i, k-block j at KSTAGE i + j; X tile i at KSTAGE (TNB + i) + j
    typedef TiledShape<PAIR, MW> Shape;
    constexpr int TMB = Shape::TMB, TMR = Shape::TMR, NSTG = Shape::NSTG;
    constexpr int KSTAGE = Shape::KSTAGE;
    constexpr int STAGE_BLOCKS = Shape::STAGE_BLOCKS;
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

    // this wavefront brings in W row-tiles 2w, 2w+1 and XW row-tiles of X per k-block
    constexpr int XW = TMB / 4;
    const u32x4* wsrc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) wsrc[i] = Wp + (size_t)min(tn * TNB + wave * 2 + i, NT32 - 1) * KB * 64 + lane;
    const u32x4 *hsrc[XW];
#pragma unroll
    for (int x = 0; x < XW; ++x) {
        const int xrt = min(tm * TMB + wave * XW + x, MT32 - 1);
        hsrc[x] = Xhi + (size_t)xrt * KB * 64 + lane;
    }
    const int nst_all = KB / KSTAGE;  // KB is even (K % 32 == 0)
    const int st0 = (int)((long)ks * nst_all / ksplit);
    const int nstage = (int)((long)(ks + 1) * nst_all / ksplit) - st0;  // this workgroup's stages: st0 .. st0+nstage-1
    {
        const size_t skip = (size_t)st0 * KSTAGE * 64;
        wsrc[0] += skip; wsrc[1] += skip;
#pragma unroll
        for (int x = 0; x < XW; ++x) hsrc[x] += skip;
    }
    auto issue = [&](int st) {
        u32x4 (*slot)[64] = ring[st % NSTG];
#pragma unroll
        for (int j = 0; j < KSTAGE; ++j) {
            const size_t off = ((size_t)st * KSTAGE + j) * 64;
            load_block_to_lds(wsrc[0] + off, &slot[(wave * 2 + 0) * KSTAGE + j][0]);
            load_block_to_lds(wsrc[1] + off, &slot[(wave * 2 + 1) * KSTAGE + j][0]);
#pragma unroll
            for (int x = 0; x < XW; ++x) load_block_to_lds(hsrc[x] + off, &slot[(TNB + wave * XW + x) * KSTAGE + j][0]);
        }
    };
    constexpr int kLoadsPerStage = (2 + XW) * KSTAGE;  // per wavefront
    // operand registers of one k-block: 4 weight blocks, MW activation tiles
    struct Ops { u32x4 a[4], b[MW]; };
    auto read_ops = [&](Ops& o, int st, int j) {
        u32x4 (*slot)[64] = ring[st % NSTG];
#pragma unroll
        for (int i = 0; i < 4; ++i) o.a[i] = slot[(wn * 4 + i) * KSTAGE + j][lane];
#pragma unroll
        for (int i = 0; i < MW; ++i) o.b[i] = slot[(TNB + wm * MW + i) * KSTAGE + j][lane];
    };
    auto mma_ops = [&](const Ops& o) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int jj = 0; jj < MW; ++jj) acc[i][jj] = mfma_f16(o.a[i], o.b[jj], acc[i][jj]);
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

// ----------------------------------------------------------------- 256 x 256 tiles (prompt and scoring passes)
//
// With one half term per activation the 256 x 128 tile above no longer keeps the matrix cores busy: it pulls
// 12 KiB of operands out of L2 for every 32 matrix instructions, and at eight rounds of 512 tiles on 256 CUs that
// is 10 TB/s -- what the L2s deliver.  This kernel takes 16 KiB for 64: a 256 x 256 tile per workgroup, four
// wavefronts with a 128 x 128 sub-tile each (16 accumulator tiles: the whole accumulator file, so one workgroup
// per CU).  Nothing else runs on a CU while its four wavefronts sit at a barrier or issue loads, so the schedule is
// laid out by hand: a stage is two k-blocks (32 KiB, ring of four); LDS reads and global -> LDS copies are dealt out
// between pairs of matrix instructions, every read at least eight matrix instructions ahead of the wait that
// covers it.  Measured on the 8160 x 20480 x 5120 product (loop only): matrix instructions alone on random operands
// 1015 us (the clock drops under data toggling), + LDS reads 1082 us, + copies 1280 us = 1.34 PFLOP/s (1310 us with
// one read per pair all through a half: the compiler's wait at the top of a half is for all reads, the newest
// included); with reads and copies issued in bursts after the barrier, as a compiler left to itself schedules
// them, 1690 us.  Copies issued by odd and even wavefronts behind different pairs: no change.
// A lane of a 32x32 accumulator tile holds columns 8q + 4 (lane / 32) + 0..3 of row lane % 32: four halves of an
// eight-column slot, the other four in the lane 32 away.  For a pair of slots (q even, q odd) packed as x, y: the
// lower lane gets the whole even slot, the upper lane the whole odd one -- 16-byte stores instead of 8-byte ones
// (the epilogue is bound by the number of store instructions).
__device__ __forceinline__ u32x4 join_halves(uint2 x, uint2 y) {
    const auto a = __builtin_amdgcn_permlane32_swap(x.x, y.x, false, false);  // [x low lanes | y low lanes], [x high | y high]
    const auto b = __builtin_amdgcn_permlane32_swap(x.y, y.y, false, false);
    return u32x4{a[0], b[0], a[1], b[1]};
}

// The big kernel's result stores, 16 bytes per lane.  (Nontemporal stores were tried: no gain for the half blocks,
// 6 % slower for the float rows.)
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store16(void* dst, u32x4 v) { *reinterpret_cast<u32x4*>(dst) = v; }
__device__ __forceinline__ void store16(void* dst, float a, float b, float c, float d) {
    *reinterpret_cast<f32x4*>(dst) = f32x4{a, b, c, d};
}

// One matrix instruction with the accumulator tile pinned to a register file: the accumulation registers (VG =
// false) or the vector registers.  Twenty accumulator tiles do not fit into the 256 accumulation registers, and left
// to itself the compiler keeps them all there and moves the overflow in and out around every instruction (832 moves
// per stage).  Written as assembly the instruction is opaque to the compiler's hazard recogniser: nothing but these
// instructions touches an accumulator inside the k loop, and the caller waits out the matrix pipeline before the
// epilogue reads them.
template <bool VG>
__device__ __forceinline__ void mfma_f16_pinned(f32x16& c, const u32x4& a, const u32x4& b) {
    if constexpr (VG) asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

constexpr int BM = 256;  // rows of X per tile of the big kernel; its width is 64 NA columns (NA = 4 or 5)
constexpr int BSTAGES = 4;

// NA: 32-column blocks of a wavefront's sub-tile (its 32 NA x 128 accumulators: 4 NA tiles of 32 x 32).  NA = 4 is the
// 256-column tile described above.  NA = 5, a 320-column tile, takes 18 KiB of operands for 80 matrix instructions
// (a tenth fewer bytes per flop), keeps a fifth of its accumulators in the vector registers, and is chosen where
// its tiles divide the matrix and the CUs better: at hidden size 5120 the QKV GEMM is six full rounds instead of
// seven and a half, FC1 eight instead of ten, and the out-projection and FC2 two, with nothing left to cut along k.
// Measured on 8192 rows with the same operands launch after launch: FC1 1506 -> 1391 us, the QKV shape 1187 -> 1048;
// inside the prompt pass, where every launch streams new weights, 180.2 -> 177.2 ms for the pass on one box (with
// the wide tile for QKV and FC1 only: 178.9).
template <int MODE, int NA>
__global__ __launch_bounds__(256, 1) void gemm_tiled256_kernel(const u32x4* __restrict__ Wp, const u32x4* __restrict__ X,
                                                               const u32x4* __restrict__ bias8, int KB, int NT32, int MT32,
                                                               int tiles_n, int tiles_m, int ksplit, int split_tn, Epi p) {
    constexpr int BN = 64 * NA;       // columns of the tile
    constexpr int XOFF = 4 * NA;      // blocks of a stage: W row-tile i, k-block j at 2 i + j; X row-tile i at XOFF + 2 i + j
    constexpr int SB = 4 * NA + 16;   // blocks of a stage (two k-blocks of 2 NA W row-tiles and 8 X row-tiles)
    __shared__ u32x4 ring[BSTAGES][SB][64];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    // Work items, in launch order: the tiles of the first split_tn columns of tiles with their whole k range, then
    // the tiles of the other columns once per k range (k range after k range).  Each of the two parts is dealt out
    // so that an XCD gets a contiguous run of it.
    const int n_whole = split_tn * tiles_m, whole_pad = (n_whole + 7) / 8 * 8;
    const bool cut = (int)blockIdx.x >= whole_pad;
    const int idx = cut ? blockIdx.x - whole_pad : blockIdx.x;
    const int cols = cut ? tiles_n - split_tn : split_tn;  // columns of tiles of this part
    const int nblk = cols * tiles_m;
    const int nitem = cut ? nblk * ksplit : nblk;
    const int per_xcd = (nitem + 7) / 8;
    const int item = (idx % 8) * per_xcd + idx / 8;
    if (item >= nitem) return;
    const int lin = item % nblk, ks = item / nblk;
    const int nks = cut ? ksplit : 1;  // k ranges of this tile
    constexpr int GROUP = 4;  // m-tiles per super-row: the 32 tiles an XCD works on at once share 4 X panels and 8 W panels
    const int gsize = GROUP * cols;
    const int g = lin / gsize, first_m = g * GROUP;
    const int gm = min(GROUP, tiles_m - first_m);
    const int tm = first_m + (lin % gsize) % gm, tn = (cut ? split_tn : 0) + (lin % gsize) / gm;
    const int wn = wave & 1, wm = wave >> 1;  // this wavefront's 32 NA (n) x 128 (m) sub-tile
    const int cur_len = epilogue_len<MODE>(p);
    f32x16 acc[NA][4];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x16{};

    const int nst_all = KB / 2;  // KB is even (K % 32 == 0)
    const int st0 = (int)((long)ks * nst_all / nks);
    const int nstage = (int)((long)(ks + 1) * nst_all / nks) - st0;
    // The SB blocks of a stage are copied by the four wavefronts, CW each: wavefront w copies blocks w CW .. w CW + CW - 1
    // (block c < XOFF: W row-tile c / 2, k-block c % 2; else X row-tile (c - XOFF) / 2).  Row-tiles past the matrix:
    // the last one (computed, never stored).
    constexpr int CW = NA + 4;  // copies per wavefront and stage
    const u32x4* src[CW];
#pragma unroll
    for (int q = 0; q < CW; ++q) {
        const int c = wave * CW + q;
        const bool isw = c < XOFF;
        const int rt = isw ? min(tn * 2 * NA + (c >> 1), NT32 - 1) : min(tm * 8 + ((c - XOFF) >> 1), MT32 - 1);
        src[q] = (isw ? Wp : X) + ((size_t)rt * KB + (size_t)st0 * 2 + (c & 1)) * 64 + lane;
    }
    auto copy1 = [&](int st, int q) {
        load_block_to_lds(src[q] + (size_t)st * 128, &ring[st & (BSTAGES - 1)][wave * CW + q][0]);
    };
    auto issue = [&](int st) {
#pragma unroll
        for (int q = 0; q < CW; ++q) copy1(st, q);
    };
    constexpr int C2 = CW / 2;  // copies 0 .. C2-1 of a stage go out in the second half of stage t-3, the rest in the first of t-2
    struct Ops { u32x4 a[NA], b[4]; };
    // LDS read q (0 .. NA+3) of a k-block, in the order the matrix instructions below first need the operands:
    // a0, b0, b1, b2, b3, a1, a2, ...
    constexpr int NR = NA + 4;
    auto read1 = [&](Ops& o, int st, int j, int q) {
        u32x4 (*slot)[64] = ring[st & (BSTAGES - 1)];
        if (q == 0) o.a[0] = slot[(wn * NA) * 2 + j][lane];
        else if (q <= 4) o.b[q - 1] = slot[XOFF + (wm * 4 + q - 1) * 2 + j][lane];
        else o.a[q - 4] = slot[(wn * NA + q - 4) * 2 + j][lane];
    };
    auto read_ops = [&](Ops& o, int st, int j) {
#pragma unroll
        for (int q = 0; q < NR; ++q) read1(o, st, j, q);
    };
    // matrix instruction n (0 .. 4 NA - 1) of a k-block: accumulator tile (n / 4, n % 4)
    // (NA = 5: the tiles of the first four column blocks live in the accumulation registers, the fifth block's in
    // the vector registers)
    auto mma1 = [&](const Ops& o, int n) {
        if constexpr (NA > 4) {
            if ((n >> 2) < 4) mfma_f16_pinned<false>(acc[n >> 2][n & 3], o.a[n >> 2], o.b[n & 3]);
            else mfma_f16_pinned<true>(acc[n >> 2][n & 3], o.a[n >> 2], o.b[n & 3]);
        } else {
            acc[n >> 2][n & 3] = mfma_f16(o.a[n >> 2], o.b[n & 3], acc[n >> 2][n & 3]);
        }
    };
    auto mma_all = [&](const Ops& o) {
#pragma unroll
        for (int n = 0; n < 4 * NA; ++n) mma1(o, n);
    };
    // The prologue issues what would fall before stage 0.
    issue(0);
    if (nstage >= 2) issue(1);
    if (nstage >= 3) {
#pragma unroll
        for (int q = 0; q < C2; ++q) copy1(2, q);
        wait_vmcnt<CW + C2>();
    } else if (nstage == 2) {
        wait_vmcnt<CW>();
    } else {
        wait_vmcnt<0>();
    }
    __syncthreads();
    Ops opa, opb;
    read_ops(opa, 0, 0);
    int s = 0;
    // Steady state: stage s+1 and the first copies of stage s+2 are in flight; the first half of stage s requests the
    // rest of stage s+2 (into the slot stage s-2 left: everybody passed the barrier of stage s-1 since), the second
    // half the first copies of stage s+3 (into the slot of stage s-1, behind this stage's barrier).  Scheduling
    // barriers keep the order written here.  The workgroup barrier is the bare instruction: what it orders are the
    // copies, which the wait before it covers -- the LDS reads in flight across it belong to the stage in use, not to
    // the slot about to be refilled (a fence would wait for them).
    // In each half of a stage (2 NA pairs of matrix instructions) the first pairs are followed by two LDS reads each
    // (the operands of the other half: the last of them is at least eight matrix instructions old when the half
    // ends, so the wait for the reads at the top of a half finds them done), the last ones by one copy each.
    constexpr int NP = 2 * NA;  // pairs of matrix instructions per half
    static_assert((NR + 1) / 2 + (CW - C2) <= NP, "reads and copies of a half fit behind its pairs");
    for (; s + 3 < nstage; ++s) {
#pragma unroll
        for (int q = 0; q < NP; ++q) {
            mma1(opa, 2 * q);
            mma1(opa, 2 * q + 1);
            if (2 * q < NR) {
                read1(opb, s, 1, 2 * q);
                if (2 * q + 1 < NR) read1(opb, s, 1, 2 * q + 1);
            } else if (q >= NP - (CW - C2)) {
                copy1(s + 2, C2 + q - (NP - (CW - C2)));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        wait_vmcnt<CW>();  // this wavefront's copies of stage s+1 have landed ...
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();  // ... and everybody's; everybody is done with stage s-1
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < NP; ++q) {
            mma1(opb, 2 * q);
            mma1(opb, 2 * q + 1);
            if (2 * q < NR) {
                read1(opa, s + 1, 0, 2 * q);
                if (2 * q + 1 < NR) read1(opa, s + 1, 0, 2 * q + 1);
            } else if (q >= NP - C2) {
                copy1(s + 3, q - (NP - C2));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    for (; s < nstage; ++s) {  // the last three stages: only the late copies of the last one are left to request
        if (s + 2 < nstage) {
#pragma unroll
            for (int q = C2; q < CW; ++q) copy1(s + 2, q);
        }
        read_ops(opb, s, 1);
        mma_all(opa);
        if (s + 1 < nstage) {
            if (s + 2 < nstage) wait_vmcnt<CW>();
            else wait_vmcnt<0>();
            __syncthreads();
            read_ops(opa, s + 1, 0);
        }
        mma_all(opb);
    }
    if constexpr (NA > 4) asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // the last matrix instructions' results are in
    // Epilogue.  The CU runs nothing else meanwhile, so it is written out per mode with everything that depends on
    // the row alone (sequence, cache position, row base address) computed once per 32-row block and everything
    // that depends on the column alone wave-uniform (the generic per-quad form recomputes both, with run-time
    // integer divisions, for each of a lane's 64 quads: 22 us per tile for FC1, 44 us for QKV, against 130 us of
    // matrix instructions).  N is a multiple of 32 here, so a 32-column block is inside or outside as a whole.
    const int hh = lane >> 5;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int m = tm * BM + (wm * 4 + j) * 32 + (lane & 31);
        if (m >= p.M) continue;
        size_t row = 0;       // MODE_STORE: float index of (m, 4 hh); BIAS_RELU: 16-byte slot of (m, k half hh) in
                              // the first block of its row of blocks; QKV: float index into q
        size_t kvrow = 0;     // QKV: half index of (sequence, head 0, position, 0) inside one (layer, k|v) plane
        bool append = true;   // QKV: the row is a token (not padding): its key and value go into the cache
        if (MODE == MODE_STORE) {
            row = (size_t)ks * p.out_split + (size_t)m * p.N + 4 * hh;
        } else if (MODE == MODE_BIAS_RELU) {
            row = (size_t)(m >> 5) * (p.N >> 4) * 64 + 32 * hh + (m & 31);
        } else {
            row = (size_t)m * p.H + 4 * hh;
            const int b = row_seq(p.st, m, p.S), r = m % p.S;
            int t = cur_len + r;
            if (cur_len < 0) {  // sequences of different lengths; padding rows append nothing
                const int tr = r - row_pad(p.st, b);
                append = tr >= 0;
                t = seq_len(p.st, b) + tr;
            }
            kvrow = ((size_t)b * p.n_heads * p.max_seq + t) * p.d;
        }
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int n32 = tn * BN + (wn * NA + i) * 32;  // wave-uniform
            if (n32 >= p.N) continue;
            if (MODE == MODE_STORE) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    store16(p.out + row + n32 + 8 * q, acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2],
                            acc[i][j][q * 4 + 3]);
            } else if (MODE == MODE_BIAS_RELU) {
                u32x4* ob = p.out_blocks + row + (size_t)(n32 >> 4) * 64;
                uint2 h4[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const u32x4 b8 = bias8[(n32 >> 3) + q];  // wave-uniform address: a scalar load
                    const uint2 bb = hh ? make_uint2(b8.z, b8.w) : make_uint2(b8.x, b8.y);
                    const float v0 = fmaxf(acc[i][j][q * 4 + 0] + bf_lo(bb.x), 0.f), v1 = fmaxf(acc[i][j][q * 4 + 1] + bf_hi(bb.x), 0.f);
                    const float v2 = fmaxf(acc[i][j][q * 4 + 2] + bf_lo(bb.y), 0.f), v3 = fmaxf(acc[i][j][q * 4 + 3] + bf_hi(bb.y), 0.f);
                    h4[q] = make_uint2(pack2(v0, v1), pack2(v2, v3));
                }
#pragma unroll
                for (int qq = 0; qq < 2; ++qq) store16(ob + qq * 64, join_halves(h4[2 * qq], h4[2 * qq + 1]));
            } else {
                const int part = n32 >= 2 * p.H ? 2 : (n32 >= p.H ? 1 : 0);  // query, key or value columns (uniform)
                half_t* kvcol = nullptr;
                if (part) {
                    const int c32 = n32 - part * p.H, head = c32 / p.d;
                    kvcol = p.kv + (((size_t)(p.layer * 2 + (part - 1)) * p.max_batch) * p.n_heads + head) * p.max_seq * (size_t)p.d +
                            (c32 - head * p.d);
                }
                uint2 h4[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const u32x4 b8 = bias8[(n32 >> 3) + q];
                    const uint2 bb = hh ? make_uint2(b8.z, b8.w) : make_uint2(b8.x, b8.y);
                    const float v0 = acc[i][j][q * 4 + 0] + bf_lo(bb.x), v1 = acc[i][j][q * 4 + 1] + bf_hi(bb.x);
                    const float v2 = acc[i][j][q * 4 + 2] + bf_lo(bb.y), v3 = acc[i][j][q * 4 + 3] + bf_hi(bb.y);
                    if (!part)
                        store16(p.out + row + n32 + 8 * q, v0 * p.qscale, v1 * p.qscale, v2 * p.qscale, v3 * p.qscale);
                    else
                        h4[q] = make_uint2(pack2(v0, v1), pack2(v2, v3));
                }
                if (part) {  // (uniform) keys / values: eight halves of a row per lane
#pragma unroll
                    for (int qq = 0; qq < 2; ++qq) {
                        const u32x4 v8 = join_halves(h4[2 * qq], h4[2 * qq + 1]);
                        if (append) store16(kvcol + kvrow + 8 * (2 * qq + hh), v8);
                    }
                }
            }
        }
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


// Many rows (a prompt or scoring pass): 256 x 256 tiles, one workgroup per CU, once there are enough of them to
// give every CU one.
static int g_tiled_cus_override = 0;  // a planner query's CU count
static int tiled_cus() { return g_tiled_cus_override > 0 ? g_tiled_cus_override : num_cus(); }
static bool use_big_tile(int M, int N) {
    return M >= 1024 && (long)((N + TN - 1) / TN) * ((M + 255) / 256) >= tiled_cus();
}

// How a many-row GEMM is cut into tiles of 256 rows: 64 na columns wide (na = 4 or 5), and, where the partial sums
// may go through scratch (may_cut), the tiles of the columns from split_col on in ks = 2 k ranges.  The tiles come in
// rounds of one per CU and a partly empty round costs a full one; the cost is in units of a whole 256-column tile.
struct BigPlan { int na, ks, split_col; };
static BigPlan big_plan(int M, int N, int KB, bool may_cut) {
    const long cus = tiled_cus(), tm = (M + BM - 1) / BM;
    may_cut = may_cut && KB % 4 == 0 && KB / 2 >= 8 * BSTAGES;
    BigPlan best{4, 1, 0};
    double best_cost = 1e30;
    for (int na = 4; na <= 5; ++na) {
        const long tn = (N + 64 * na - 1) / (64 * na);
        // a 320-column tile is five quarters of the work, done with a tenth fewer operand bytes per flop
        const double unit = na == 5 ? 1.25 * 0.98 : 1.0;
        for (long s = 0; s <= (may_cut ? tn : 0); ++s) {  // s columns of tiles cut in two
            const long whole = (tn - s) * tm, cutn = 2 * s * tm;
            // a cut tile costs a little more than half (its own ramp and epilogue), and every cut column a second
            // set of partial sums for the LayerNorm to read
            const double cost = ((double)((whole + cus - 1) / cus) + 0.52 * (double)((cutn + cus - 1) / cus) + 0.004 * s) * unit;
            if (cost < best_cost - 1e-9) {
                best_cost = cost;
                best = BigPlan{na, s ? 2 : 1, s ? (int)(tn - s) * 64 * na : 0};
            }
        }
    }
    return best;
}

// split_col: with a k-split on the big tiles, the first column whose tiles are cut into k ranges (0: all of them);
// tile_na: their width as planned by the caller (0: plan here, no cut)
template <int MODE>
void launch_tiled(hipStream_t s, const void* Wp, const void* Xhi, int KB, int N, int M, const Epi& p, int ksplit = 1,
                  int split_col = 0, int tile_na = 0) {
    const int NT32 = (N + 31) / 32, MT32 = (M + 31) / 32;
    // (the scoring head's epilogue keeps a soft-max over all of a wavefront's accumulators: it does not fit next to 16 of them)
    const bool big = MODE != MODE_SCORE && use_big_tile(M, N);
    const int TM = big ? 256 : 128;
    const int tiles_n = (N + TN - 1) / TN, tiles_m = (M + TM - 1) / TM;
    const int nitem = tiles_n * tiles_m * ksplit;
    const int grid = ((nitem + 7) / 8) * 8;
    if constexpr (MODE != MODE_SCORE) {
        if (big) {
            // (the bias through a pointer of its own: declared never to alias the outputs, its values can be fetched
            // with scalar loads, which do not queue behind the epilogue's stores)
            const int na = tile_na ? tile_na : big_plan(M, N, KB, false).na;
            const int bn = 64 * na, tn_big = (N + bn - 1) / bn;
            const int split_tn = ksplit > 1 ? split_col / bn : tn_big;  // without a k-split every tile is whole
            const int whole = split_tn * tiles_m, cutn = (tn_big - split_tn) * tiles_m * ksplit;
            const int grid2 = (whole + 7) / 8 * 8 + (cutn + 7) / 8 * 8;
            if (na == 5)
                gemm_tiled256_kernel<MODE, 5><<<grid2, 256, 0, s>>>((const u32x4*)Wp, (const u32x4*)Xhi, (const u32x4*)p.bias,
                                                                    KB, NT32, MT32, tn_big, tiles_m, ksplit, split_tn, p);
            else
                gemm_tiled256_kernel<MODE, 4><<<grid2, 256, 0, s>>>((const u32x4*)Wp, (const u32x4*)Xhi, (const u32x4*)p.bias,
                                                                    KB, NT32, MT32, tn_big, tiles_m, ksplit, split_tn, p);
            return;
        }
    }
    // two workgroups per CU once there are that many (their k ranges must hold an even number of k-blocks
    // each: that ring alternates two register sets)
    const bool pair = nitem >= 2 * num_cus() && KB % (2 * ksplit) == 0;
    if (pair)
        gemm_tiled_kernel<MODE, 1, 2><<<grid, 256, 0, s>>>((const u32x4*)Wp, (const u32x4*)Xhi, KB, NT32, MT32, tiles_n,
                                                           tiles_m, ksplit, p);
    else
        gemm_tiled_kernel<MODE, 0, 2><<<grid, 256, 0, s>>>((const u32x4*)Wp, (const u32x4*)Xhi, KB, NT32, MT32, tiles_n,
                                                           tiles_m, ksplit, p);
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

void bf16_gemm_tiled(hipStream_t s, int mode, const void* Wp, const void* Xhi, int M, int N, int K,
                     const bf16_gemm_args& a) {
    const Epi p = make_epi(M, N, a);
    if (mode == EPI_STORE) launch_tiled<MODE_STORE>(s, Wp, Xhi, K / 16, N, M, p);
    else if (mode == EPI_BIAS_RELU) launch_tiled<MODE_BIAS_RELU>(s, Wp, Xhi, K / 16, N, M, p);
    else launch_tiled<MODE_QKV>(s, Wp, Xhi, K / 16, N, M, p);
}

int bf16_tiled_ksplit(int M, int N, int K) {
    const int tiles = ((N + TN - 1) / TN) * ((M + 127) / 128), stages = K / 16 / TiledShape<0, 2>::KSTAGE;
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
    const bool big = use_big_tile(M, N);
    const long slots = (big ? 1L : 2L) * tiled_cus(), tiles = (long)((N + TN - 1) / TN) * ((M + (big ? 255 : 127)) / (big ? 256 : 128));
    const int KB = K / 16;
    if (tiles < slots || KB % 2) return 1;
    int best = 1;
    double best_cost = (double)((tiles + slots - 1) / slots);  // in units of one full-K tile
    for (int ks = 2; ks <= 4; ++ks) {
        if (KB % (2 * ks) || KB / ks < 8 * TiledShape<1, 2>::NSTG || (size_t)ks * M * N > capacity_floats) continue;
        const double cost = (double)((tiles * ks + slots - 1) / slots) / ks * (1.0 + 0.02 * ks);
        if (cost < 0.95 * best_cost) { best_cost = cost; best = ks; }
    }
    return best;
}

// The same decision for the big tiles, which can cut the tiles of the last columns only: *split_col is the first
// column whose tiles are cut into *ks k ranges (0: all; columns before it get one whole-k sum), *na the tiles' width
// in 64 columns.  The whole tiles come first, in rounds of one per CU, and the cut ones fill the last, shorter round:
// 640 tiles of 256 columns on 256 CUs are two rounds of whole tiles and one of 256 half tiles, with a second set of
// partial sums for a fifth of the columns only (and 512 tiles of 320 columns are two rounds with nothing to cut).
// Other tile shapes: bf16_tiled_store_ksplit, every tile cut.
void bf16_tiled_store_split(int M, int N, int K, size_t capacity_floats, int* ks, int* split_col, int* na) {
    *ks = bf16_tiled_store_ksplit(M, N, K, capacity_floats);
    *split_col = 0;
    *na = 0;
    if (!use_big_tile(M, N)) return;
    const BigPlan g = big_plan(M, N, K / 16, (size_t)2 * M * N <= capacity_floats);
    *ks = g.ks;
    *split_col = g.split_col;
    *na = g.na;
}

void bf16_tiled_plan_query(int M, int N, int K, int may_cut, size_t capacity_floats, int cus, int* tile_cols, int* ks,
                           int* split_col) {
    g_tiled_cus_override = cus;
    *tile_cols = 0; *ks = 1; *split_col = 0;
    if (use_big_tile(M, N)) {
        const bool room = capacity_floats == 0 || (size_t)2 * M * N <= capacity_floats;
        const BigPlan g = big_plan(M, N, K / 16, may_cut && room);
        *tile_cols = 64 * g.na; *ks = g.ks; *split_col = g.split_col;
    } else if (may_cut) {
        *ks = bf16_tiled_store_ksplit(M, N, K, capacity_floats ? capacity_floats : (size_t)-1);
    }
    g_tiled_cus_override = 0;
}

void bf16_gemm_tiled_ksplit(hipStream_t s, int mode, const void* Wp, const void* Xhi, int M, int N, int K,
                            int ksplit, float* part, size_t part_split, const bf16_gemm_args& a) {
    if (ksplit == 1 && mode != EPI_STORE) {  // the tiles alone fill the chip: the epilogue runs in the GEMM
        bf16_gemm_tiled(s, mode, Wp, Xhi, M, N, K, a);
        return;
    }
    bf16_gemm_args st = a;
    st.out = part; st.out_split = part_split;
    const Epi ps = make_epi(M, N, st);
    launch_tiled<MODE_STORE>(s, Wp, Xhi, K / 16, N, M, ps, ksplit, a.split_col, a.tile_na);
    if (mode == EPI_STORE) return;  // the consumer (a LayerNorm) adds the partial sums
    const Epi p = make_epi(M, N, a);
    const unsigned grid = (unsigned)(((size_t)M * (N / 4) + 255) / 256);
    if (mode == EPI_BIAS_RELU) finish_kernel<MODE_BIAS_RELU><<<grid, 256, 0, s>>>(part, ksplit, part_split, p);
    else finish_kernel<MODE_QKV><<<grid, 256, 0, s>>>(part, ksplit, part_split, p);
}

int bf16_score_parts(int V) { return 2 * ((V + TN - 1) / TN); }

void bf16_score_head(hipStream_t s, const void* Wp, const void* Xhi, int M, int S, int V, int K,
                     const int32_t* ids, float* stats, float* tgt, float* out) {
    Epi p{};
    p.M = M; p.N = V; p.S = S; p.ids = ids; p.sc_stats = (float2*)stats; p.sc_tgt = tgt; p.sc_parts = bf16_score_parts(V);
    launch_tiled<MODE_SCORE>(s, Wp, Xhi, K / 16, V, M, p);
    score_reduce_kernel<<<(M + 3) / 4, 256, 0, s>>>((const float2*)stats, tgt, p.sc_parts, M, S, out);
}

