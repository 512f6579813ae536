// Machinery shared by the LM-head kernels: the persistent, XCD-aware sweep of
// 256 x 256 MFMA tiles (W-role rows x token-role rows, K contiguous in both
// operands) with a pluggable per-lane epilogue.  The forward pass plugs in the
// online log-softmax; the backward pass plugs in the softmax-derivative writer
// and a plain tile store (which makes the same sweep an "NT" GEMM).
#pragma once
#include <stdlib.h>

#include <atomic>
#include <type_traits>

#include "common.h"

namespace tppo {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kMaxSplits = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -3.0e38f;    // finite stand-in for -inf (keeps exp2(m - m') NaN-free)

struct HeadParams {
    const uint16_t* hidden;
    const uint16_t* w;
    const int32_t* sel_rows;
    const int32_t* sel_targets;
    const int64_t* m_actual;
    float* part;                       // [3][splits][M]: max (log2 domain), sumexp, target logit
    int64_t n_rows, ld_h, ld_w, M;
    int H, V, row_tiles, splits, vocab_tiles;
    int unit_splits, unit_cols, n_units;   // persistent schedule, see head_mfma_kernel
    int unit_rows, col_major;              // col_major: the 8 XCDs sweep the same vocabulary slice together
    int32_t* unit_arrivals;                // [n_units] zeroed before the launch
    // used by the epilogues of the backward pass only
    const float* aux0;                     // per-token scalars (lse)
    const float* aux1;                     // per-token scalars (upstream derivative)
    const int32_t* aux_index;              // where token t's scalars sit in aux0/aux1 (NULL: at t)
    void* out;                             // tile output
    int64_t ld_out, out_cols;              // leading dimension / columns of `out` that exist
    int accumulate;                        // add to `out` instead of overwriting it
};

// Compile-time shape of one kernel variant: a kTileV x kTileT (vocabulary x
// tokens) output tile per workgroup, kWavesV x kWavesT wavefronts, kBK
// K-elements per LDS stage, a ring of kStages stages.
//
// LDS staging layout.  A stage holds kTileV + kTileT rows of kBK bf16 (W rows
// first, then token rows), each row as kBK/8 chunks of 16 bytes.  Chunk c of
// row r sits in slot c ^ swz(r).  The LDS serves 64 banks x 4 B = 256 B per
// cycle, i.e. 16 lanes of a ds_read_b128; those 16 lanes read the same chunk
// of 16 consecutive rows, and the swizzle spreads them over all 16 slots of
// the 256-byte bank window (measured: SQ_LDS_BANK_CONFLICT = 0).
//
// MI selects the MFMA instruction: 32 = v_mfma_f32_32x32x16_bf16, 16 =
// v_mfma_f32_16x16x32_bf16.  Same flops per cycle and the same LDS bytes per
// flop, but at the chip's power limit the 16x16x32 form sustains more (MFMA
// loop on LDS-fed fragments: 1.65 vs 1.55 PFLOP/s; on register-resident ones 2.10
// vs 1.83).  In both forms lane l of a wave holds, for an MI x MI block,
// column l % MI (a token) and the rows (e/4)*(4G) + (l/MI)*4 + e%4 for
// e < MI*MI/64, G = 64/MI lane groups (vocabulary entries), and reads its
// operand fragments as 16 bytes: row l % MI, K chunk l / MI of the MFMA's K range.
template <int TV, int TT, int WV, int WT, int BK, int ST, int WGS_PER_CU, int SPREAD = 0, int MI = 32, int SUBDIV = 2>
struct HeadCfg {
    static_assert(MI == 32 || MI == 16, "MFMA block shape");
    static constexpr int kMI = MI, kGroups = 64 / MI, kAccElems = MI * MI / 64, kQuads = kAccElems / 4;
    typedef float Acc __attribute__((__vector_size__(kAccElems * sizeof(float))));
    static constexpr int kTileV = TV, kTileT = TT, kWavesV = WV, kWavesT = WT, kBK = BK, kStages = ST;
    static constexpr int kWgsPerCu = WGS_PER_CU;
    // 0: a wave issues the transfers of a stage back to back; n > 0: one by one
    // between its next n MFMAs, so the wave never sits in a full memory queue
    static constexpr int kSpread = SPREAD;
    static constexpr int kWaves = WV * WT, kThreads = kWaves * 64;
    static constexpr int kWaveV = TV / WV, kWaveT = TT / WT;              // wave tile
    static constexpr int kVB = kWaveV / MI, kTB = kWaveT / MI;            // MI x MI blocks per wave
    // an MFMA step: the 32x32x16 form covers all W blocks over 16 K; the 16x16x32 form 1/kSubdiv of them over 32 K
    static constexpr int kSubdiv = MI == 32 ? 1 : SUBDIV;
    static constexpr int kSubVB = kVB / kSubdiv;
    static constexpr int kMfmaPerStep = kSubVB * kTB;
    static constexpr int kRowBytes = BK * 2, kChunks = BK / 8;
    static constexpr int kRows = TV + TT;
    static constexpr int kStageBytes = kRows * kRowBytes;
    static constexpr int kLdsBytes = ST * kStageBytes;
    static constexpr int kRowsPerDma = 1024 / kRowBytes;                  // one wave-wide 16 B/lane transfer
    static constexpr int kDmaPerStage = kRows / kRowsPerDma;
    static constexpr int kDmaPerWave = kDmaPerStage / kWaves;
    static constexpr int kKSteps = MI == 32 ? BK / 16 : (BK / 32) * kSubdiv;
    static_assert(kDmaPerWave * kWaves == kDmaPerStage, "transfers must divide evenly over the waves");
    static_assert(TV % kRowsPerDma == 0, "a transfer may not straddle W and token rows");
    static_assert(kKSteps % 2 == 0, "fragment double buffering assumes an even number of K steps");
    static_assert(WV * 3 * TT * 4 <= kLdsBytes, "merge buffer must fit in the idle stages");
    static_assert(MI == 32 || (kVB % kSubdiv == 0 && BK % 32 == 0), "16x16x32: W blocks in equal parts, K in steps of 32");
    static_assert(SPREAD == 0 || (ST == 2 && SPREAD <= kKSteps * kMfmaPerStep),
                  "spread issue: two stages, at most one stage's worth of MFMAs");
    __device__ static __forceinline__ int swz(int r) {
        return BK == 64 ? ((r >> 1) & 7) : ((r >> 2) & 3);
    }
    __device__ static __forceinline__ int chunk_off(int r, int c) {
        return r * kRowBytes + ((c ^ swz(r)) << 4);
    }
    // row (inside the wave tile's W rows) of accumulator element e of block vb, for lane group g = lane / MI
    __device__ static __forceinline__ int row_in_wave(int vb, int e, int g) {
        return vb * MI + (e >> 2) * (4 * kGroups) + g * 4 + (e & 3);
    }
};

// One wave-wide global -> LDS transfer without a register round trip: lane l's
// 16 bytes at `src` land at LDS byte address lds_base + 16*l (lds_base is
// wave-uniform and goes through M0).  Written as inline assembly so that the
// transfer stays asynchronous: completion is awaited by hand (vmcnt) right
// before the workgroup barrier that publishes the stage.
__device__ __forceinline__ void dma_16b_per_lane(const void* src, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_base), "v"(src)
                 : "memory", "m0");
}

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8); }

// Schedule.  The grid is persistent: 256 workgroups, one per CU, hardware id
// b runs on XCD b % 8 (ids go round-robin over the 8 XCDs, each with its own
// L2).  The work is cut into units of 8 token tiles x unit_splits (<= 4)
// vocabulary splits; the 32 workgroups of an XCD take one unit together, one
// (token tile, split) pair each, then the XCD's next unit.  Inside a unit every
// W tile is wanted by 8 workgroups and every hidden tile by up to 4 at the same
// step of the same sweep, so one of them pays the L2 miss and the others hit;
// equal work per pair keeps them in step for the whole sweep, which a
// free-running grid of independent workgroups does not.  The splits of a unit
// may differ by one vocabulary tile, so the workgroups of an XCD re-align at
// every unit boundary with an arrival counter.  That wait is only a hint for
// the caches: it is bounded and falls through, and nothing depends on it.
// Across XCDs the units are handed out so that the 8 XCDs sweep the SAME
// vocabulary slice at the same time, each for its own 8 token tiles: W then
// leaves HBM once per round instead of once per XCD (the later readers find it
// in the memory-side cache), which is worth 1-2 % at the chip's power limit.
constexpr int kAlignSpins = 4096;
__device__ __forceinline__ void align_unit(int32_t* arrivals, int expected) {
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(arrivals, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int spin = 0; spin < kAlignSpins; ++spin) {
            if (__hip_atomic_load(arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= expected) break;
            __builtin_amdgcn_s_sleep(8);
        }
    }
    __syncthreads();
}
// Epi (the per-lane epilogue) provides
//   init(p, tok0, m_eff, wt, lane)                          once per (token tile, split) sweep,
//   fold(acc, p, tok0, m_eff, vt, wv, wt, lane)             after each finished tile of 256 W rows; clears acc,
//   finish(p, lds_scratch, tok0, m_eff, sp, wv, wt, lane, tid)  after the sweep (workgroup-wide).
template <class C, template <class> class Epi>
__global__ __launch_bounds__(C::kThreads, C::kWgsPerCu* C::kWaves / 4) void head_mfma_kernel(HeadParams p) {
    constexpr int kTileV = C::kTileV, kTileT = C::kTileT, kWaveV = C::kWaveV, kWaveT = C::kWaveT;
    constexpr int kVB = C::kVB, kTB = C::kTB, kBK = C::kBK, kStages = C::kStages;
    constexpr int kDmaPerWave = C::kDmaPerWave, kKSteps = C::kKSteps;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int tile_in_unit = slot & 7, split_in_unit = slot >> 3;
    if (split_in_unit >= p.unit_splits) return;
    const int64_t m_eff = p.m_actual ? min(p.M, *p.m_actual) : p.M;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wv = wave / C::kWavesT, wt = wave % C::kWavesT;
    const int frag_row = lane % C::kMI, frag_grp = lane / C::kMI;
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;

    for (int unit = xcd; unit < p.n_units; unit += 8) {
    int unit_row, unit_col;
    if (p.col_major) {
        // round j of the grid: rows 8g .. 8g+7 (one per XCD) of column j % unit_cols; the rows
        // left over after the last full group of 8 are dealt out column by column
        const int j = unit >> 3, full = p.unit_rows >> 3, left = p.unit_rows & 7;
        if (j < full * p.unit_cols) {
            unit_row = (j / p.unit_cols) * 8 + xcd;
            unit_col = j % p.unit_cols;
        } else {
            const int t = (j - full * p.unit_cols) * 8 + xcd;
            unit_col = t / left;
            unit_row = full * 8 + t - unit_col * left;
        }
    } else {
        unit_row = unit / p.unit_cols;
        unit_col = unit - unit_row * p.unit_cols;
    }
    const int rt = unit_row * 8 + tile_in_unit, sp = unit_col * p.unit_splits + split_in_unit;
    const int64_t tok0 = (int64_t)rt * kTileT;
    if (unit >= 8) align_unit(p.unit_arrivals + unit, 8 * p.unit_splits);   // the first unit starts aligned
    if (rt >= p.row_tiles || tok0 >= m_eff) continue;       // uniform over the workgroup
    const int vt_begin = (int)((int64_t)p.vocab_tiles * sp / p.splits);
    const int vt_end = (int)((int64_t)p.vocab_tiles * (sp + 1) / p.splits);
    const int k_tiles = p.H / kBK;
    const int total_iters = (vt_end - vt_begin) * k_tiles;

    // ---- loader role: transfers wave*kDmaPerWave + q, each kRowsPerDma staged rows
    const int ld_row0 = wave * kDmaPerWave * C::kRowsPerDma + lane / C::kChunks;   // + q * kRowsPerDma
    const int ld_slot = lane % C::kChunks;
    const uint16_t* src[kDmaPerWave];
    int issue_vt = vt_begin, issue_kt = 0, issue_stage = 0, issue_kpos = 0;
    auto point_at_tile = [&](int vt, bool w_only) {
#pragma unroll
        for (int q = 0; q < kDmaPerWave; ++q) {
            const int r = ld_row0 + q * C::kRowsPerDma;                 // staged row; < kTileV means a W row
            const int chunk = (ld_slot ^ C::swz(r)) * 8;
            if (r < kTileV) {
                const int64_t v = min((int64_t)vt * kTileV + r, (int64_t)p.V - 1);
                src[q] = p.w + v * p.ld_w + chunk;
            } else if (!w_only) {
                const int64_t t = min(tok0 + (r - kTileV), m_eff - 1);
                int64_t row = p.sel_rows ? (int64_t)p.sel_rows[t] : t;      // no list: rows in order
                row = min(max(row, (int64_t)0), p.n_rows - 1);
                src[q] = p.hidden + row * p.ld_h + chunk;
            }
        }
    };
    point_at_tile(vt_begin, false);
    auto issue_one = [&](int q) {
        const unsigned dst = lds_base + issue_stage * C::kStageBytes + wave * kDmaPerWave * 1024;
        dma_16b_per_lane(src[q] + issue_kpos, dst + q * 1024);
    };
    auto issue_advance = [&]() {        // next (vocabulary tile, k tile) in sweep order
        issue_kpos += kBK;
        if (++issue_stage == kStages) issue_stage = 0;
        if (++issue_kt == k_tiles) {
            issue_kt = 0;
            issue_kpos = 0;
            ++issue_vt;
            point_at_tile(min(issue_vt, vt_end - 1), true);
        }
    };
    auto issue = [&]() {
#pragma unroll
        for (int q = 0; q < kDmaPerWave; ++q) issue_one(q);
        issue_advance();
    };

    Epi<C> epi;
    epi.init(p, tok0, m_eff, wt, lane);

    typename C::Acc acc[kVB][kTB];
#pragma unroll
    for (int vb = 0; vb < kVB; ++vb)
#pragma unroll
        for (int tb = 0; tb < kTB; ++tb)
#pragma unroll
            for (int e = 0; e < C::kAccElems; ++e) acc[vb][tb][e] = 0.f;

    // Fragments of MFMA step `step` of a stage (kKSteps steps per stage), double buffered.
    //   32x32x16: step = K step of 16; all kVB W fragments and the kTB token fragments, K chunks 2*step + group.
    //   16x16x32: step = (K step of 32) * kSubdiv + part; the W fragments of that part of the blocks, K chunks
    //             4*(step/kSubdiv) + group; the token fragments once per K step of 32 (with part 0).
    constexpr int kSubVB = C::kSubVB;
    bf16x8 fa[2][kSubVB], fb[2][kTB];
    // `par`: parity of the K iteration the fragments belong to.  With 32-deep stages a stage holds ONE K step of
    // 32, so the token fragments of consecutive iterations must alternate between the two buffers (the next
    // stage's first fragments are fetched before this stage's last MFMAs); with 64-deep stages the two K steps
    // of a stage alternate by themselves.
    auto fb_slot = [](int k32, int par) { return C::kBK == 32 ? ((k32 + par) & 1) : (k32 & 1); };
    auto load_frags = [&](int stage, int step, auto par_c) {
        constexpr int par = decltype(par_c)::value;
        const unsigned char* st = smem + stage * C::kStageBytes;
        const unsigned char* a_base = st + (wv * kWaveV) * C::kRowBytes;
        const unsigned char* b_base = st + (kTileV + wt * kWaveT) * C::kRowBytes;
        if (C::kMI == 32) {
            const int c = step * 2 + frag_grp;
#pragma unroll
            for (int vb = 0; vb < kSubVB; ++vb)
                fa[step & 1][vb] = *reinterpret_cast<const bf16x8*>(a_base + C::chunk_off(vb * 32 + frag_row, c));
#pragma unroll
            for (int tb = 0; tb < kTB; ++tb)
                fb[step & 1][tb] = *reinterpret_cast<const bf16x8*>(b_base + C::chunk_off(tb * 32 + frag_row, c));
        } else {
            const int k32 = step / C::kSubdiv, part = step % C::kSubdiv, c = k32 * 4 + frag_grp;
#pragma unroll
            for (int j = 0; j < kSubVB; ++j)
                fa[step & 1][j] = *reinterpret_cast<const bf16x8*>(a_base + C::chunk_off((part * kSubVB + j) * 16 + frag_row, c));
            if (part == 0) {
#pragma unroll
                for (int tb = 0; tb < kTB; ++tb)
                    fb[fb_slot(k32, par)][tb] = *reinterpret_cast<const bf16x8*>(b_base + C::chunk_off(tb * 16 + frag_row, c));
            }
        }
    };
    auto mfma_one = [&](int step, int j, int tb, auto par_c) {
        constexpr int par = decltype(par_c)::value;
        if constexpr (C::kMI == 32) {
            acc[j][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[step & 1][j], fb[step & 1][tb], acc[j][tb], 0, 0, 0);
        } else {
            const int vb = (step % C::kSubdiv) * kSubVB + j;
            acc[vb][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[step & 1][j], fb[fb_slot(step / C::kSubdiv, par)][tb], acc[vb][tb], 0, 0, 0);
        }
    };
    auto mfma_step = [&](int step, auto par_c) {
#pragma unroll
        for (int j = 0; j < kSubVB; ++j)
#pragma unroll
            for (int tb = 0; tb < kTB; ++tb) mfma_one(step, j, tb, par_c);
    };
    // The same K step with this wave's transfers first .. first + n - 1 of the
    // stage being refilled issued between the MFMAs (`on` is workgroup-uniform).
    // Transfer j of the stage being refilled follows MFMA number
    // floor(j * kSpread / kDmaPerWave), counted from the barrier that freed it.
    constexpr int kMfmaPerStep = C::kMfmaPerStep;
    constexpr int kSpreadSteps = (C::kSpread + kMfmaPerStep - 1) / kMfmaPerStep;   // MFMA steps the issue touches
    auto mfma_step_issuing = [&](int step, int part, bool on, auto par_c) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int vb = 0; vb < kSubVB; ++vb)
#pragma unroll
            for (int tb = 0; tb < kTB; ++tb) {
                mfma_one(step, vb, tb, par_c);
                const int g = part * kMfmaPerStep + vb * kTB + tb;
                if (on) {
#pragma unroll
                    for (int j = 0; j < kDmaPerWave; ++j)
                        if (C::kSpread && j * C::kSpread / kDmaPerWave == g) issue_one(j);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
    };

    // ---- fill the ring, publish stage 0, start on its first fragments
#pragma unroll
    for (int s = 0; s < kStages - 1; ++s)
        if (s < total_iters) issue();
    if (total_iters >= kStages - 1)
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((kStages - 2) * kDmaPerWave));
    else
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    if (kStages - 1 < total_iters) issue();
    typedef std::integral_constant<int, 0> Even;
    typedef std::integral_constant<int, 1> Odd;
    load_frags(0, 0, Even());

    int kt = 0, vt = vt_begin, stage = 0;
    bool refill = false;                // spread issue: transfers of the stage freed at the last barrier are pending
    // one K iteration (one stage); par_c = the iteration's parity where it matters (32-deep stages), else Even
    auto iteration = [&](int it, auto par_c) {
        constexpr int par = decltype(par_c)::value;
        typedef std::integral_constant<int, (C::kBK == 32 ? par ^ 1 : 0)> Next;
#pragma unroll
        for (int ks = 0; ks + 1 < kKSteps; ++ks) {
            load_frags(stage, ks + 1, par_c);
            if (C::kSpread && ks + 1 < kSpreadSteps) {
                mfma_step_issuing(ks, ks + 1, refill, par_c);
                if (ks + 2 == kSpreadSteps && refill) issue_advance();
            } else {
                mfma_step(ks, par_c);
            }
        }
        // The stage's last fragments are in registers.  Hand the stage back,
        // publish the next one and fetch its first fragments BEFORE issuing the
        // last MFMAs, so the barrier and the LDS latency hide behind them.
        const int next_stage = stage + 1 == kStages ? 0 : stage + 1;
        refill = false;
        if (it + 1 < total_iters) {
            if (total_iters - it - 2 >= kStages - 2)
                __builtin_amdgcn_s_waitcnt(vmcnt_imm((kStages - 2) * kDmaPerWave));
            else
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            __syncthreads();            // stage it+1 landed for everyone; everyone left stage it
            if (it + kStages < total_iters) {
                if (C::kSpread) refill = true;
                else issue();
            }
            load_frags(next_stage, 0, Next());
        }
        if (C::kSpread) {
            mfma_step_issuing(kKSteps - 1, 0, refill, par_c);
            if (kSpreadSteps == 1 && refill) issue_advance();
        } else {
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(kKSteps - 1, par_c);
        }
        stage = next_stage;
        if (++kt == k_tiles) {          // a vocabulary tile is complete
            epi.fold(acc, p, tok0, m_eff, vt, wv, wt, lane);
            kt = 0;
            ++vt;
        }
    };
    if constexpr (C::kBK == 32) {
        for (int it = 0; it < total_iters; it += 2) {
            iteration(it, Even());
            if (it + 1 < total_iters) iteration(it + 1, Odd());
        }
    } else {
        for (int it = 0; it < total_iters; ++it) iteration(it, Even());
    }
    __syncthreads();                    // every fragment read is done before the stages are reused
    epi.finish(p, reinterpret_cast<float*>(smem), tok0, m_eff, sp, wv, wt, lane, tid);
    __syncthreads();                    // merge buffer is read before the next unit's transfers land
    }
}

static __global__ __launch_bounds__(256) void head_clear_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

struct HeadVariant {
    void (*kernel)(HeadParams);
    int tile_v, tile_t, threads, lds_bytes, wgs_per_cu;
    // what a unit costs besides its tiles, in tile times (pipeline fill, the wait at the unit boundary, and for
    // the log-softmax the merge of the splits): 0.25 measured for sweeps over H-deep tiles with a merge
    double unit_cost = 0.25;
    int col_major = 1;                  // 1: the 8 XCDs sweep the same W-role slice together; 0: the same token rows
};
// Number of vocabulary splits.  A unit is 8 token tiles x min(splits, 4 per CU slot) splits
// and every XCD works through ceil(units / 8) units of ceil(vocab_tiles /
// splits) vocabulary tiles each; pick the count (1, 2, 3 or a multiple of 4)
// that minimises that product, with a small per-unit overhead (1 .. us - 1, or a multiple of us).
static int choose_splits(const HeadVariant& hv, int64_t M, int64_t V) {
    const int64_t row_tiles = (M + hv.tile_t - 1) / hv.tile_t, vocab_tiles = (V + hv.tile_v - 1) / hv.tile_v;
    const int64_t unit_rows = (row_tiles + 7) / 8;
    const int max_s = (int)(vocab_tiles < kMaxSplits ? vocab_tiles : kMaxSplits);
    const int us = 4 * hv.wgs_per_cu;                       // splits a unit holds: 32 workgroups per XCD and per CU slot
#ifdef TPPO_TUNING
    if (const char* e = getenv("TPPO_HEAD_SPLITS")) {       // tuning builds only
        const int forced = atoi(e);
        if (forced >= 1 && (forced < us || forced % us == 0)) return forced < max_s ? forced : max_s < us ? max_s : max_s / us * us;
    }
#endif
    int best = 1;
    double best_cost = 1e300;
    for (int s = 1; s <= max_s; ++s) {
        if (s > us && s % us != 0) continue;
        const int64_t units = unit_rows * (s <= us ? 1 : s / us);
        const double rounds = (double)((units + 7) / 8);
        const double per = (double)((vocab_tiles + s - 1) / s) + hv.unit_cost;
        // fewer than `us` splits leave CUs idle: 8*s of the 8*us workgroups of an XCD work
        const double cost = rounds * per;
        if (cost < best_cost - 1e-9) {
            best_cost = cost;
            best = s;
        }
    }
    return best;
}

// arrival counters of the persistent schedule: one per unit, at the end of the workspace
static size_t arrivals_bytes(int64_t M) { return round_up((size_t)((M / 128 / 8 + 2) * (kMaxSplits / 4)) * 4, 256); }   // (token tiles of >= 128)


// Fill in the schedule fields of `p` for M token-role rows and V W-role rows.
static void plan_sweep(HeadParams& p, const HeadVariant& hv, int64_t M, int64_t V, void* arrivals,
                       const char* tune_splits = nullptr, const char* tune_order = nullptr) {
    p.M = M;
    p.V = (int)V;
    p.row_tiles = (int)((M + hv.tile_t - 1) / hv.tile_t);
    p.vocab_tiles = (int)((V + hv.tile_v - 1) / hv.tile_v);
    p.splits = choose_splits(hv, M, V);
#ifdef TPPO_TUNING
    if (const char* e = tune_splits ? getenv(tune_splits) : nullptr) {
        const int forced = atoi(e), us4 = 4 * hv.wgs_per_cu;
        if (forced >= 1 && forced <= p.vocab_tiles && forced <= kMaxSplits && (forced < us4 || forced % us4 == 0)) p.splits = forced;
    }
#endif
    const int us = 4 * hv.wgs_per_cu;
    p.unit_splits = p.splits < us ? p.splits : us;
    p.unit_cols = p.splits / p.unit_splits;
    p.unit_rows = (p.row_tiles + 7) / 8;
    p.n_units = p.unit_rows * p.unit_cols;
    p.col_major = hv.col_major;
#ifdef TPPO_TUNING
    if (const char* e = getenv("TPPO_HEAD_ORDER")) p.col_major = atoi(e);     // tuning builds only: 0 = row-major units
    if (const char* e = tune_order ? getenv(tune_order) : nullptr) p.col_major = atoi(e);
#endif
    p.unit_arrivals = static_cast<int32_t*>(arrivals);
}

// The schedule above is laid out for the whole MI355X: 256 compute units, hardware workgroup id b on XCD b % 8.
constexpr int kSweepGroups = 256;

// A kernel that wants more than 64 KiB of LDS has to be told so once per device.
static bool allow_lds(const HeadVariant& hv) {
    constexpr int kMaxDevices = 64, kMaxKernels = 8;
    static std::atomic<const void*> done[kMaxDevices][kMaxKernels];
    const void* fn = reinterpret_cast<const void*>(hv.kernel);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return false;
    std::atomic<const void*>* row = dev < kMaxDevices ? done[dev] : nullptr;
    int free_slot = -1;
    if (row) {
        for (int i = 0; i < kMaxKernels; ++i) {
            const void* seen = row[i].load(std::memory_order_acquire);
            if (seen == fn) return true;
            if (!seen && free_slot < 0) free_slot = i;
        }
    }
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, hv.lds_bytes) != hipSuccess) return false;
    if (row && free_slot >= 0) row[free_slot].store(fn, std::memory_order_release);   // (a lost race only repeats the call)
    return true;
}

// Clear the arrival counters and launch one sweep (persistent: one workgroup per CU).  A device that does not
// report 256 compute units (a partition of the chip, another chip) is refused: the sweep would still be
// correct there, but its workgroups would take turns instead of running side by side.
static int launch_sweep(const HeadVariant& hv, const HeadParams& p, hipStream_t s) {
    if (device_compute_units() != kSweepGroups) return TPPO_ERR_LAUNCH;
    if (!allow_lds(hv)) return TPPO_ERR_LAUNCH;
    hipLaunchKernelGGL(head_clear_kernel, dim3((p.n_units + 255) / 256), dim3(256), 0, s, p.unit_arrivals, p.n_units);
    if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
    hipLaunchKernelGGL(hv.kernel, dim3(kSweepGroups * hv.wgs_per_cu), dim3(hv.threads), hv.lds_bytes, s, p);
    return launch_result();
}

}  // namespace tppo
