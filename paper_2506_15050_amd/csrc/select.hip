// tppo_select: token filter of Sec. 3.2 as a segmented compaction.
//   kernel 1 (one workgroup): per-sequence window / keep lengths and their
//            prefix sums (resp_off, sel_off), counts;
//   kernel 2: one thread per compact slot m: locate its sequence in sel_off
//            and emit (row, target id, response-packed index).
#include "common.h"

namespace tppo {

constexpr int kScanThreads = 1024;

struct Triple { int win, keep, val; };

__device__ __forceinline__ Triple add3(Triple a, Triple b) {
    return {a.win + b.win, a.keep + b.keep, a.val + b.val};
}

__global__ __launch_bounds__(kScanThreads) void select_scan_kernel(
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ ctx_len,
    const int32_t* __restrict__ done, int B, int n_tok, int tail_drop,
    int32_t* __restrict__ resp_off, int32_t* __restrict__ sel_off,
    int32_t* __restrict__ keep_len, int64_t* __restrict__ counts, int32_t* status) {
    __shared__ Triple wave_tot[kScanThreads / kWave];
    __shared__ Triple carry_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) {
        carry_s = {0, 0, 0};
        resp_off[0] = 0;
        sel_off[0] = 0;
    }
    __syncthreads();
    for (int base = 0; base < B; base += kScanThreads) {
        const int i = base + tid;
        Triple x = {0, 0, 0};
        if (i < B) {
            const int lo = cu_seqlens[i], hi = cu_seqlens[i + 1], ctx = ctx_len[i];
            int win = hi - lo - ctx;
            if (ctx < 1 || win < 0 || lo < 0 || hi > n_tok) {
                set_status(status, TPPO_STATUS_BAD_LAYOUT);
                win = 0;
            }
            const bool fin = done[i] != 0;
            const int keep = fin ? win : max(win - tail_drop, 0);
            keep_len[i] = keep;
            x = {win, keep, fin ? win : 0};
        }
        // inclusive scan inside the wave
        Triple inc = x;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            Triple y = {__shfl_up(inc.win, off), __shfl_up(inc.keep, off), __shfl_up(inc.val, off)};
            if (lane >= off) inc = add3(inc, y);
        }
        if (lane == kWave - 1) wave_tot[wave] = inc;
        __syncthreads();
        Triple pre = carry_s;
        for (int w = 0; w < wave; ++w) pre = add3(pre, wave_tot[w]);
        inc = add3(inc, pre);
        if (i < B) {
            resp_off[i + 1] = inc.win;
            sel_off[i + 1] = inc.keep;
        }
        __syncthreads();
        if (tid == kScanThreads - 1) carry_s = inc;
        __syncthreads();
    }
    if (tid == 0) {
        counts[0] = carry_s.keep;
        counts[1] = carry_s.win;
        counts[2] = carry_s.val;
    }
}

__global__ __launch_bounds__(256) void select_fill_kernel(
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ ctx_len,
    const int32_t* __restrict__ input_ids, int B, int n_tok,
    const int32_t* __restrict__ resp_off, const int32_t* __restrict__ sel_off,
    int32_t* __restrict__ sel_rows, int32_t* __restrict__ sel_targets,
    int32_t* __restrict__ sel_resp_idx, int64_t capacity, int32_t* status) {
    const int64_t m = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int M = sel_off[B];
    if (m >= M) return;
    if (m >= capacity) {
        if (m == capacity) set_status(status, TPPO_STATUS_CAPACITY);
        return;
    }
    const int i = find_segment(sel_off, 0, B - 1, (int)m);
    const int t = (int)m - sel_off[i];
    const int pos = cu_seqlens[i] + ctx_len[i] + t;
    if (sel_rows) sel_rows[m] = pos - 1;
    if (sel_targets) sel_targets[m] = (pos >= 0 && pos < n_tok) ? input_ids[pos] : -1;
    if (sel_resp_idx) sel_resp_idx[m] = resp_off[i] + t;
}

}  // namespace tppo

extern "C" int tppo_select(const int32_t* cu_seqlens, const int32_t* ctx_len, const int32_t* done,
                           const int32_t* input_ids, int64_t B, int64_t n_tok, int32_t tail_drop,
                           int32_t* resp_off, int32_t* sel_off, int32_t* keep_len,
                           int32_t* sel_rows, int32_t* sel_targets, int32_t* sel_resp_idx,
                           int64_t capacity, int64_t* counts, int32_t* status, void* stream) {
    using namespace tppo;
    if (B < 0 || n_tok < 0 || capacity < 0 || B > INT32_MAX - 1 || n_tok > INT32_MAX) return TPPO_ERR_SIZE;
    if (tail_drop < 0) return TPPO_ERR_PARAM;
    if (!cu_seqlens || !resp_off || !sel_off || !counts) return TPPO_ERR_NULL;
    if (B > 0 && (!ctx_len || !done || !keep_len)) return TPPO_ERR_NULL;
    if (sel_targets && !input_ids) return TPPO_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(select_scan_kernel, dim3(1), dim3(kScanThreads), 0, s, cu_seqlens, ctx_len,
                       done, (int)B, (int)n_tok, (int)tail_drop, resp_off, sel_off, keep_len, counts,
                       status);
    if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
    const bool want_fill = sel_rows || sel_targets || sel_resp_idx;
    const int64_t slots = capacity < n_tok ? capacity + 1 : n_tok;   // +1: lets the overflow be reported
    if (want_fill && B > 0 && slots > 0) {
        const int64_t blocks = (slots + 255) / 256;
        hipLaunchKernelGGL(select_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, s, cu_seqlens,
                           ctx_len, input_ids, (int)B, (int)n_tok, resp_off, sel_off, sel_rows,
                           sel_targets, sel_resp_idx, capacity, status);
        if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
    }
    return TPPO_OK;
}
