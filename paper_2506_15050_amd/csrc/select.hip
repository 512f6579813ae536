// tppo_select: token filter of Sec. 3.2 as a segmented compaction.
//   kernel 1 (one workgroup per 1024 sequences): per-sequence window / keep lengths, their prefix
//            sums (resp_off, sel_off), the counts and a list of tiles of the compact
//            output (<= 1024 kept tokens of one sequence each);
//   kernel 2 (persistent grid): walks the compact list; a tile's descriptor says
//            which sequence and which window positions it covers, so every
//            thread emits (row, target id, response-packed index) for 4
//            consecutive kept tokens without searching the offset arrays;
//   and, if the caller wants one, the work plan of the response-packed domain
//   (plan.h) that tppo_egae* and the loss entry points take, built from the
//   offsets kernel 1 has just written.
#include "plan.h"

namespace tppo {

constexpr int kScanThreads = 1024;
constexpr int kFillThreads = 256, kFillTpt = kTileTokens / kFillThreads;
constexpr int kFillMaxGroups = 2048;

struct Sums { int win, keep, val, tiles; };     // window / kept / value tokens, tiles of the compact output

__device__ __forceinline__ Sums add4(Sums a, Sums b) {
    return {a.win + b.win, a.keep + b.keep, a.val + b.val, a.tiles + b.tiles};
}

__device__ __forceinline__ Sums shfl_up4(Sums a, int off) {
    return {__shfl_up(a.win, off), __shfl_up(a.keep, off), __shfl_up(a.val, off), __shfl_up(a.tiles, off)};
}

__device__ __forceinline__ Sums shfl_xor4(Sums a, int off) {
    return {__shfl_xor(a.win, off), __shfl_xor(a.keep, off), __shfl_xor(a.val, off), __shfl_xor(a.tiles, off)};
}

static inline int64_t select_max_tiles(int64_t capacity, int64_t B) { return capacity / kTileTokens + B + 1; }

// window / keep lengths of sequence i (a bad layout counts as an empty window and sets the status bit)
__device__ __forceinline__ Sums lengths_of(const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ ctx_len,
                                           const int32_t* __restrict__ done, int i, int n_tok, int tail_drop,
                                           int32_t* status) {
    const int lo = cu_seqlens[i], hi = cu_seqlens[i + 1], ctx = ctx_len[i];
    int win = hi - lo - ctx;
    if (ctx < 1 || win < 0 || lo < 0 || hi > n_tok) {
        if (status) set_status(status, TPPO_STATUS_BAD_LAYOUT);
        win = 0;
    }
    const bool fin = done[i] != 0;
    const int keep = fin ? win : max(win - tail_drop, 0);
    return {win, keep, fin ? win : 0, tiles_of(keep)};
}

// `parts` workgroups share the sequences (one up to a few thousand of them): workgroup g owns a contiguous
// range and, inside it, thread t a contiguous block, so there is one workgroup-wide prefix sum whatever B is:
// pass A adds up the block, the scan gives the block's starting offsets, pass B re-reads the (cache-resident)
// metadata and writes the per-sequence outputs and tile descriptors.  Where its range starts a workgroup
// finds out by adding up, by itself, the lengths of all sequences before the range.
__global__ __launch_bounds__(kScanThreads) void select_scan_kernel(
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ ctx_len,
    const int32_t* __restrict__ done, int B, int n_tok, int tail_drop, int parts,
    int32_t* __restrict__ resp_off, int32_t* __restrict__ sel_off,
    int32_t* __restrict__ keep_len, int64_t* __restrict__ counts, Tile* __restrict__ tiles,
    int tile_cap, int32_t* __restrict__ n_tiles, int32_t* status) {
    __shared__ Sums wave_tot[2][kScanThreads / kWave];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int part = blockIdx.x;
    const int range = (B + parts - 1) / parts;
    const int p_begin = min(part * range, B), p_end = min(p_begin + range, B);
    const int per = (p_end - p_begin + kScanThreads - 1) / kScanThreads;
    const int i_begin = min(p_begin + tid * per, p_end), i_end = min(i_begin + per, p_end);
    Sums mine = {0, 0, 0, 0}, ahead = {0, 0, 0, 0};
    for (int i = tid; i < p_begin; i += kScanThreads)
        ahead = add4(ahead, lengths_of(cu_seqlens, ctx_len, done, i, n_tok, tail_drop, nullptr));
    for (int i = i_begin; i < i_end; ++i) mine = add4(mine, lengths_of(cu_seqlens, ctx_len, done, i, n_tok, tail_drop, status));
    Sums inc = mine;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const Sums y = shfl_up4(inc, off);
        if (lane >= off) inc = add4(inc, y);
        ahead = add4(ahead, shfl_xor4(ahead, off));
    }
    if (lane == kWave - 1) wave_tot[0][wave] = inc;
    if (lane == 0) wave_tot[1][wave] = ahead;
    __syncthreads();
    Sums run = {inc.win - mine.win, inc.keep - mine.keep, inc.val - mine.val, inc.tiles - mine.tiles};
    Sums total = {0, 0, 0, 0};
    for (int w = 0; w < kScanThreads / kWave; ++w) {
        if (w < wave) run = add4(run, wave_tot[0][w]);
        run = add4(run, wave_tot[1][w]);
        total = add4(total, add4(wave_tot[0][w], wave_tot[1][w]));
    }
    if (part == 0 && tid == 0) {
        resp_off[0] = 0;
        sel_off[0] = 0;
    }
    for (int i = i_begin; i < i_end; ++i) {
        const Sums x = lengths_of(cu_seqlens, ctx_len, done, i, n_tok, tail_drop, nullptr);
        keep_len[i] = x.keep;
        if (tiles) emit_tiles(tiles, tile_cap, run.tiles, i, run.keep, x.keep);       // compact domain
        run = add4(run, x);
        resp_off[i + 1] = run.win;
        sel_off[i + 1] = run.keep;
    }
    if (part == parts - 1 && tid == 0) {                // the last range ends where the batch ends
        counts[0] = total.keep;
        counts[1] = total.win;
        counts[2] = total.val;
        if (n_tiles) n_tiles[0] = min(total.tiles, tile_cap);
    }
}

__global__ __launch_bounds__(kFillThreads) void select_fill_kernel(
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ ctx_len,
    const int32_t* __restrict__ input_ids, int n_tok, const int32_t* __restrict__ resp_off,
    const Tile* __restrict__ tiles, const int32_t* __restrict__ n_tiles,
    int32_t* __restrict__ sel_rows, int32_t* __restrict__ sel_targets,
    int32_t* __restrict__ sel_resp_idx, int64_t capacity, int32_t* status) {
    const int count = *n_tiles;
    const int tid = threadIdx.x;
    for (int w = blockIdx.x; w < count; w += gridDim.x) {
        const Tile t = tiles[w];
        const int i = t.seg, len = t.len(), t0 = t.number() * kTileTokens;
        const int first_pos = cu_seqlens[i] + ctx_len[i] + t0;      // packed position of the tile's first token
        const int first_resp = resp_off[i] + t0;
#pragma unroll
        for (int q = 0; q < kFillTpt; ++q) {
            const int k = q * kFillThreads + tid;                    // lane-consecutive: coalesced stores
            const int64_t m = (int64_t)t.start + k;
            if (k < len) {
                if (m >= capacity) {
                    if (m == capacity) set_status(status, TPPO_STATUS_CAPACITY);
                } else {
                    const int pos = first_pos + k;
                    if (sel_rows) sel_rows[m] = pos - 1;
                    if (sel_targets) sel_targets[m] = (pos >= 0 && pos < n_tok) ? input_ids[pos] : -1;
                    if (sel_resp_idx) sel_resp_idx[m] = first_resp + k;
                }
            }
        }
    }
}

}  // namespace tppo

extern "C" size_t tppo_select_workspace_bytes(int64_t B, int64_t capacity) {
    if (B < 0 || capacity < 0) return 256;
    return tppo::round_up((size_t)tppo::select_max_tiles(capacity, B) * sizeof(tppo::Tile), 256) + 256;
}

extern "C" int tppo_select(const int32_t* cu_seqlens, const int32_t* ctx_len, const int32_t* done,
                           const int32_t* input_ids, int64_t B, int64_t n_tok, int32_t tail_drop,
                           int32_t* resp_off, int32_t* sel_off, int32_t* keep_len,
                           int32_t* sel_rows, int32_t* sel_targets, int32_t* sel_resp_idx,
                           int64_t capacity, int64_t* counts, void* workspace, size_t workspace_bytes,
                           void* plan, size_t plan_bytes, int32_t* status, void* stream) {
    using namespace tppo;
    if (B < 0 || n_tok < 0 || capacity < 0 || B > INT32_MAX / 4 || n_tok > INT32_MAX) return TPPO_ERR_SIZE;
    if (tail_drop < 0) return TPPO_ERR_PARAM;
    if (!cu_seqlens || !resp_off || !sel_off || !counts) return TPPO_ERR_NULL;
    if (B > 0 && (!ctx_len || !done || !keep_len)) return TPPO_ERR_NULL;
    if (sel_targets && !input_ids) return TPPO_ERR_NULL;
    const bool want_fill = (sel_rows || sel_targets || sel_resp_idx) && B > 0 && capacity > 0;
    // the list covers every kept token, also those beyond `capacity` (they are reported, not written)
    const int64_t list_tokens = capacity < n_tok ? n_tok : capacity;
    const int64_t cap64 = select_max_tiles(list_tokens, B);
    if (cap64 > INT32_MAX / 4) return TPPO_ERR_SIZE;
    if (want_fill && (!workspace || !is_aligned(workspace, 256) ||
                      workspace_bytes < tppo_select_workspace_bytes(B, list_tokens)))
        return TPPO_ERR_WORKSPACE;
    // a plan is sized for the largest response-packed domain this batch can have: n_resp <= n_tok
    const int64_t plan_cap = plan_max_tiles(n_tok, B);
    if (plan && (!is_aligned(plan, 256) || plan_bytes < plan_bytes_for(plan_cap) || plan_cap > INT32_MAX / 8))
        return TPPO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Tile* tiles = want_fill ? static_cast<Tile*>(workspace) : nullptr;
    int32_t* n_tiles = want_fill ? reinterpret_cast<int32_t*>(static_cast<char*>(workspace) +
                                                              round_up((size_t)cap64 * sizeof(Tile), 256))
                                 : nullptr;
    const int parts = build_parts(B);
    hipLaunchKernelGGL(select_scan_kernel, dim3(parts), dim3(kScanThreads), 0, s, cu_seqlens, ctx_len,
                       done, (int)B, (int)n_tok, (int)tail_drop, parts, resp_off, sel_off, keep_len, counts,
                       tiles, (int)cap64, n_tiles, status);
    if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
    // n_resp is known on the device only: the builder reads it from the offsets
    if (plan && launch_plan_build(resp_off, keep_len, done, B, -1, plan_cap, plan, status, s) != TPPO_OK)
        return TPPO_ERR_LAUNCH;
    if (want_fill) {
        const int groups = (int)(cap64 < kFillMaxGroups ? cap64 : kFillMaxGroups);
        hipLaunchKernelGGL(select_fill_kernel, dim3(groups), dim3(kFillThreads), 0, s, cu_seqlens,
                           ctx_len, input_ids, (int)n_tok, resp_off, tiles, n_tiles, sel_rows,
                           sel_targets, sel_resp_idx, capacity, status);
        if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
    }
    return TPPO_OK;
}
