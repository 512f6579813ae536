// tppo_ppo_losses: clipped surrogate (Eq. (ppoloss)) and clipped value loss
// (Eqs. (valueclip), (valueloss)) as masked streaming reductions over the
// response-packed arrays.  Token sets follow Sec. 3.2: policy tokens are the
// first keep_len[i] window tokens of each sequence, value tokens all window
// tokens of finished sequences.  No token depends on another, so the pass walks
// the arrays in aligned frames of 1024 tokens (plan.h), four consecutive tokens
// per thread: a frame's descriptor names the sequence of its first token, and
// a thread whose four tokens lie inside that sequence (all threads of most
// frames) knows its share of both sets from two comparisons.  Only a thread at
// or beyond a sequence boundary inside the frame looks into the offset arrays.
// No mask array is read, and a thread with no member of a set issues no loads
// for that set.
//
// One launch per call.  A persistent grid walks the frames; a thread issues all loads of its share of a
// frame at once (non-temporal 16-byte accesses, consecutive lanes on consecutive 16 bytes, no branch and no wait
// between them), and the many co-resident wavefronts cover each other's memory latency: there is deliberately
// no software pipeline, whose second register set would halve the wavefronts per CU while the compiler, unable
// to count loads issued under a predicate, waits for all of them anyway.  Sums are token-level (Sec. 4.1.1): a
// term is fp32, every sum of terms fp64, in a fixed order, no float atomics -> bit-identical reruns.
// Each workgroup publishes its partial sums as tagged words (plan.h); the
// workgroup with the highest id -- dispatched last -- waits for all of them
// (bounded), adds them up in a fixed order and writes the result, which saves
// the second launch a separate finalisation kernel would cost.
#include <stdlib.h>

#include "plan.h"

namespace tppo {

#ifndef TPPO_LOSS_THREADS
#define TPPO_LOSS_THREADS 256
#endif
constexpr int kLossThreads = TPPO_LOSS_THREADS;
constexpr int kLossParts = kTileTokens / (4 * kLossThreads);      // a workgroup takes this fraction of a frame, four tokens per thread
static_assert(kLossParts >= 1 && kLossParts * 4 * kLossThreads == kTileTokens, "whole parts of a frame");
// Workgroups of the persistent grids, measured on 40 M tokens: the read-only pass is fastest with 8 per CU; the
// pass that also writes two arrays with 4 per CU (fewer accesses in flight at once, as for a bare elementwise
// pass of 6 reads and 2 writes).
constexpr int kLossGroups = 2048, kGradGroups = 1024;
constexpr int kFinishSpin = 1 << 20;
static_assert(kLossGroups <= kFinishGroups, "the plan holds partial sums for kFinishGroups workgroups");

struct LossParams {
    const float *logp_new, *logp_old, *adv, *v_new, *v_old, *ret;
    const int32_t *resp_off, *keep_len, *done;
    void* plan;
    int32_t* status;
    int B, n_resp;
    uint32_t tag;
    float ratio_lo, ratio_hi, xi_low, xi_high;
};

typedef float float4u __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access, 4-byte aligned

// exp for the probability ratio: one multiply and the hardware exp2 (relative error ~1e-7 (1 + |x|), far inside
// the tolerances; the library expf costs ~15 more instructions per token)
__device__ __forceinline__ float ratio_exp(float x) {
    return __builtin_amdgcn_exp2f(x * 1.4426950408889634f);
}

__device__ __forceinline__ float clampf(float x, float lo, float hi) {
    return fminf(fmaxf(x, lo), hi);
}

// fminf / fmaxf return the operand that IS a number, so a NaN input would be clipped away; inside a token set
// it must reach the result instead (the term of such a token is undefined), hence the explicit tests.
__device__ __forceinline__ float surrogate(float ln, float lo, float a, float rlo, float rhi) {
    const float rho = ratio_exp(ln - lo);
    const float u = rho * a;
    const float t = fminf(u, clampf(rho, rlo, rhi) * a);
    return u != u ? u : t;
}

__device__ __forceinline__ bool value_undefined(float d0, float d1, float vo) {
    return d0 != d0 || d1 != d1 || vo != vo;
}

__device__ __forceinline__ float value_term(float v, float vo, float r, float xl, float xh) {
    const float d0 = v - r;
    const float d1 = clampf(v, vo - xl, vo + xh) - r;
    return value_undefined(d0, d1, vo) ? __builtin_nanf("") : fmaxf(d0 * d0, d1 * d1);
}

__device__ __forceinline__ double block_sum(double x, double* s_red) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_down(x, off);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) s_red[wave] = x;
    __syncthreads();
    double t = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += s_red[w];
    return t;   // valid in thread 0
}

// Four consecutive results per access; `n` = how many of the four exist.
__device__ __forceinline__ void store4(float* __restrict__ dst, int first, const float (&x)[4], int n) {
    if (n >= 4) {
        float4u t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = x[e];
        __builtin_nontemporal_store(t, reinterpret_cast<float4u*>(dst + first));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (e < n) dst[first + e] = x[e];
    }
}

// What one thread holds of one frame: 16 bytes of each of the six arrays.
struct LossRegs {
    float4u ln, lo, a, v, vo, r;
};

// A thread's four consecutive tokens: the first one's index, how many of the four exist, and which are policy /
// value tokens (bit e: token first + e).
struct TokenSets {
    int first, n_tok, pol, val;
};

// The sets of the tokens at or beyond `end` of sequence `seg` (the last one the frame's descriptor knows):
// token by token, moving on to the sequence that holds the token -- normally the next one, whose four
// metadata words are asked for together; past empty sequences by bisection of the offsets, so the work is
// bounded whatever the layout.  Offsets that are not a layout (decreasing, beyond the arrays) put a token in
// no set; they cannot make an access leave the arrays.
__device__ __forceinline__ void walk_sets(const LossParams& p, int seg, int end, TokenSets& ts) {
    int pol_end = end;
    bool fin = false, inside = false;
    for (int e = 0; e < ts.n_tok; ++e) {
        const int q = ts.first + e;
        if (q < end && !inside) continue;                          // a token the descriptor covered
        if (q >= end) {                                            // find the sequence that holds q
            int nxt = seg + 1;
            if (nxt >= p.B) break;                                 // beyond the last sequence
            int lo = p.resp_off[nxt], hi = p.resp_off[nxt + 1], keep = p.keep_len[nxt], dn = p.done[nxt];
            if (hi <= q) {                                         // not the next one: the last sequence that begins at or before q
                int a = nxt + 1, b = p.B - 1;
                if (a > b) break;
                while (a < b) {
                    const int m = (a + b + 1) >> 1;
                    if (p.resp_off[m] <= q) a = m; else b = m - 1;
                }
                nxt = a;
                lo = p.resp_off[nxt]; hi = p.resp_off[nxt + 1]; keep = p.keep_len[nxt]; dn = p.done[nxt];
            }
            inside = q >= lo && q < hi;
            if (!inside) continue;                                 // no sequence holds q (seg, end unchanged: look again)
            seg = nxt;
            end = hi;
            pol_end = lo + min(max(keep, 0), hi - lo);
            fin = dn != 0;
        }
        ts.pol |= q < pol_end ? 1 << e : 0;
        ts.val |= fin ? 1 << e : 0;
    }
}

__device__ __forceinline__ TokenSets token_sets(const LossParams& p, const FrameDesc& d, int item, int tid,
                                                bool has_pol, bool has_val) {
    TokenSets ts;
    ts.first = item * (4 * kLossThreads) + 4 * tid;                // item: part item % kLossParts of frame item / kLossParts
    ts.n_tok = min(max(p.n_resp - ts.first, 0), 4);
    if (ts.first + 4 <= d.end) {                                   // all four in the frame's first sequence
        ts.pol = (1 << min(max(d.pol_end - ts.first, 0), 4)) - 1;
        ts.val = d.fin != 0 ? 0xF : 0;
    } else {                                                       // token by token: first sequence, second, or beyond
        ts.pol = ts.val = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int q = ts.first + e;
            const bool in1 = q < d.end, in2 = !in1 && q < d.end2;
            ts.pol |= ((in1 && q < d.pol_end) || (in2 && q < d.pol_end2)) ? 1 << e : 0;
            ts.val |= ((in1 && d.fin != 0) || (in2 && d.fin2 != 0)) ? 1 << e : 0;
        }
        if (ts.first + ts.n_tok > d.end2) walk_sets(p, d.seg2, d.end2, ts);
    }
    ts.pol = (has_pol && ts.n_tok > 0) ? ts.pol & ((1 << ts.n_tok) - 1) : 0;
    ts.val = (has_val && ts.n_tok > 0) ? ts.val & ((1 << ts.n_tok) - 1) : 0;
    return ts;
}

// A frame's descriptor, checked: a plan is caller-held memory.  Whatever it says, no access leaves the arrays
// (tokens are addressed by frame and thread, not through the descriptor); only `seg2` indexes the metadata.
__device__ __forceinline__ FrameDesc checked_frame(FrameDesc d, const LossParams& p, int tid) {
    if (d.seg < 0 || d.seg >= p.B || d.seg2 < 0 || d.seg2 >= p.B) {
        if (tid == 0) set_status(p.status, TPPO_STATUS_BAD_LAYOUT);
        d = FrameDesc{p.B - 1, 0, 0, 0, p.B - 1, 0, 0, 0};         // every token looks for its sequence itself and finds none
    }
    return d;
}

// Issue the loads of a thread's four tokens.  Consecutive lanes on consecutive 16 bytes (the access shape that
// streams at full rate), non-temporal.  Nothing is loaded for a set none of the four is in; with 1..3 members
// the 16 bytes are loaded whole -- the surplus elements are never used -- so that no branch and no wait
// separates the loads and all of them are in flight together; the one thread that would read past the END OF
// THE ARRAY reads the array's last 16 bytes instead (see unshift).  Needs n_resp >= 4.
__device__ __forceinline__ void loss_load(LossRegs& x, const LossParams& p, const TokenSets& ts) {
    const float4u zero = {0.f, 0.f, 0.f, 0.f};
    const int at = min(ts.first, p.n_resp - 4);
    x.ln = x.lo = x.a = x.v = x.vo = x.r = zero;
    if (ts.pol != 0) {
        x.ln = __builtin_nontemporal_load(reinterpret_cast<const float4u*>(p.logp_new + at));
        x.lo = __builtin_nontemporal_load(reinterpret_cast<const float4u*>(p.logp_old + at));
        x.a = __builtin_nontemporal_load(reinterpret_cast<const float4u*>(p.adv + at));
    }
    if (ts.val != 0) {
        x.v = __builtin_nontemporal_load(reinterpret_cast<const float4u*>(p.v_new + at));
        x.vo = __builtin_nontemporal_load(reinterpret_cast<const float4u*>(p.v_old + at));
        x.r = __builtin_nontemporal_load(reinterpret_cast<const float4u*>(p.ret + at));
    }
}

__device__ __forceinline__ float4u rotate_left(float4u t, int sh) {
    float4u o;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        o[e] = sh == 0 ? t[e] : sh == 1 ? t[(e + 1) & 3] : sh == 2 ? t[(e + 2) & 3] : t[(e + 3) & 3];
    return o;
}

// the array's last few tokens were loaded as part of its last 16 bytes: move them into place (only in the last
// frame, and there for at most one thread)
__device__ __forceinline__ void unshift(LossRegs& x, const TokenSets& ts, int item, int n_resp) {
    if (__builtin_expect((item + 1) * (4 * kLossThreads) <= n_resp, 1)) return;   // wave-uniform: not the array's end
    const int sh = ts.n_tok > 0 ? max(ts.first - (n_resp - 4), 0) : 0;
    x.ln = rotate_left(x.ln, sh); x.lo = rotate_left(x.lo, sh); x.a = rotate_left(x.a, sh);
    x.v = rotate_left(x.v, sh); x.vo = rotate_left(x.vo, sh); x.r = rotate_left(x.r, sh);
}

// The sums of all workgroups, collected by the one with the highest id.  Every thread adds up the workgroups
// tid, tid + blockDim, ... in that order, then the threads are added up in a fixed tree: deterministic.
// The words of kBatch workgroups are asked for together -- a thread's polls are round trips through the L2, and
// one after the other they would be the longest part of a call on a small batch; only a workgroup that has
// not published yet is polled again (bounded).  Returns false when a wait gave up.
template <int kSums, int kBatch>
__device__ __forceinline__ bool collect_sums(const unsigned long long* words, uint32_t tag, int groups,
                                             double (&tot)[kSums], double* s_red, int* s_flag) {
    constexpr int kWords = 2 * kSums;
    double acc[kSums];
#pragma unroll
    for (int q = 0; q < kSums; ++q) acc[q] = 0.0;
    bool ok = true;
    const int step = (int)blockDim.x;
    for (int g0 = threadIdx.x; g0 < groups; g0 += step * kBatch) {
        unsigned long long w[kBatch][kWords];
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const int g = min(g0 + b * step, groups - 1);          // (a clamped duplicate is read and not used)
#pragma unroll
            for (int q = 0; q < kWords; ++q)
                w[b][q] = __hip_atomic_load(words + (int64_t)g * kFinishWords + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const int g = g0 + b * step;
            if (g >= groups) break;
            bool ready = true;
#pragma unroll
            for (int q = 0; q < kWords; ++q) ready = ready && (uint32_t)(w[b][q] >> 32) == tag;
            for (int spin = 0; spin < kFinishSpin && !ready; ++spin) {
                __builtin_amdgcn_s_sleep(2);
                ready = true;
#pragma unroll
                for (int q = 0; q < kWords; ++q) {
                    w[b][q] = __hip_atomic_load(words + (int64_t)g * kFinishWords + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ready = ready && (uint32_t)(w[b][q] >> 32) == tag;
                }
            }
            ok = ok && ready;
#pragma unroll
            for (int q = 0; q < kSums; ++q)
                acc[q] += ready ? (double)__uint_as_float((unsigned)w[b][2 * q]) + (double)__uint_as_float((unsigned)w[b][2 * q + 1]) : 0.0;
        }
    }
    if (threadIdx.x == 0) *s_flag = 1;
    __syncthreads();
    if (!ok) *s_flag = 0;
#pragma unroll
    for (int q = 0; q < kSums; ++q) tot[q] = block_sum(acc[q], s_red);
    return *s_flag != 0;
}

__device__ __forceinline__ void write_losses(tppo_loss_out* out, double pol_terms, double val_terms, long long np,
                                             long long nv) {
    const double policy_sum = -pol_terms, value_sum = 0.5 * val_terms;   // policy_loss = -J_PPO
    out->policy_sum = (float)policy_sum;
    out->value_sum = (float)value_sum;
    out->policy_loss = np > 0 ? (float)(policy_sum / (double)np) : 0.f;
    out->value_loss = nv > 0 ? (float)(value_sum / (double)nv) : 0.f;
    out->n_policy = np;
    out->n_value = nv;
}

// what a call that could not compute leaves behind: not a number, so that nobody trains on it
__device__ __forceinline__ void write_invalid(tppo_loss_out* out) {
    out->policy_sum = out->value_sum = out->policy_loss = out->value_loss = __builtin_nanf("");
    out->n_policy = out->n_value = 0;
}

__global__ __launch_bounds__(kLossThreads, 8) void loss_kernel(LossParams p, tppo_loss_out* __restrict__ out) {
    __shared__ double s_red[kLossThreads / kWave];
    __shared__ int s_flag;
    const Plan pl = plan_open(p.plan);
    const int tid = threadIdx.x;
    const bool has_pol = p.logp_new != nullptr, has_val = p.v_new != nullptr;
    const bool plan_ok = pl.hdr->B == p.B && pl.hdr->n_resp == p.n_resp && pl.hdr->has_sets != 0 &&
                         pl.cap >= p.n_resp / kTileTokens + p.B + 1;
    if (!plan_ok) {                                                // not this batch's plan: touch nothing of it
        if (blockIdx.x == 0 && tid == 0) {
            set_status(p.status, TPPO_STATUS_BAD_LAYOUT);
            write_invalid(out);
        }
        return;
    }
    const int count = (p.n_resp + 4 * kLossThreads - 1) / (4 * kLossThreads);     // work items: parts of frames

    double pol_acc = 0.0, val_acc = 0.0;
    FrameDesc ahead = {};
    if ((int)blockIdx.x < count) ahead = load_frame(pl.frames + blockIdx.x / kLossParts);
    for (int f = blockIdx.x; f < count; f += gridDim.x) {
        const FrameDesc d = checked_frame(ahead, p, tid);
        if (f + (int)gridDim.x < count) ahead = load_frame(pl.frames + (f + gridDim.x) / kLossParts);     // the next item's, meanwhile
        const TokenSets ts = token_sets(p, d, f, tid, has_pol, has_val);
        LossRegs cur;
        loss_load(cur, p, ts);
        unshift(cur, ts, f, p.n_resp);
        float pol_t = 0.f, val_t = 0.f;                            // this thread's <= 8 terms of the frame
        if (ts.pol != 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = surrogate(cur.ln[e], cur.lo[e], cur.a[e], p.ratio_lo, p.ratio_hi);
                pol_t += (ts.pol >> e & 1) ? t : 0.f;              // select, never multiply by a mask
            }
        }
        if (ts.val != 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = value_term(cur.v[e], cur.vo[e], cur.r[e], p.xi_low, p.xi_high);
                val_t += (ts.val >> e & 1) ? t : 0.f;
            }
        }
        pol_acc += (double)pol_t;
        val_acc += (double)val_t;
    }
    const double ps = block_sum(pol_acc, s_red);
    const double vs = block_sum(val_acc, s_red);
    unsigned long long* mine = pl.finish_words + (int64_t)blockIdx.x * kFinishWords;
    if (tid == 0) {
        publish(mine, p.tag, ps);
        publish(mine + 2, p.tag, vs);
    }
    if (blockIdx.x != gridDim.x - 1) return;
    double tot[2];
    const bool ok = collect_sums<2, 4>(pl.finish_words, p.tag, (int)gridDim.x, tot, s_red, &s_flag);
    if (tid == 0) {
        if (!ok) {
            set_status(p.status, TPPO_STATUS_TIMEOUT);
            tot[0] = tot[1] = __builtin_nan("");
        }
        write_losses(out, tot[0], tot[1], has_pol ? pl.hdr->n_policy : 0,
                     has_val ? pl.hdr->n_value : 0);
    }
}

// nothing to sum (no tokens, or neither half asked for): both sets are empty
__global__ void loss_empty_kernel(tppo_loss_out* __restrict__ out, tppo_loss_stats* __restrict__ stats) {
    if (threadIdx.x != 0) return;
    if (out) write_losses(out, 0.0, 0.0, 0, 0);
    if (stats) {
        stats->ratio_mean = stats->policy_clip_frac = stats->value_clip_frac = stats->reserved = 0.f;
        stats->n_policy_clipped = stats->n_value_clipped = 0;
    }
}

// ---------------------------------------------------------------------------
// tppo_ppo_losses_backward: the same streaming pass, also writing the
// derivatives of the two losses with respect to logp_new and v_new and
// counting the tokens whose clip is active.
//   policy token: surrogate min(u, c), u = rho A, c = clip(rho) A.  Where
//     u <= c the unclipped branch is the minimum (inside the clip range both
//     are the same function) and d/dlogp_new = rho A; where c < u the clip is
//     saturated, c is constant, the derivative is 0.
//   value token: 1/2 max(d0^2, d1^2), d0 = V - R, d1 = V_clip - R.  Where
//     d0^2 >= d1^2 the derivative is d0; otherwise V is outside the clip
//     range, V_clip is constant and the derivative is 0.
//   a token with a NaN among its inputs: the derivative is NaN, and it counts
//     neither as clipped nor as unclipped.
// Token-level means: the set sizes are known from the metadata before the pass
// (the plan holds them), so each derivative is final when it is written; tokens
// outside a set get 0.
constexpr int kGradSums = 5;       // policy terms, value terms, ratios, clipped policy tokens, clipped value tokens
static_assert(2 * kGradSums <= kFinishWords, "a workgroup's sums must fit its tagged words");

struct GradParams {
    LossParams fwd;
    float* grad_logp;
    float* grad_v;
    float policy_scale, value_scale;
    long long policy_denominator, value_denominator;     // <= 0: the call's own token counts
};

__global__ __launch_bounds__(kLossThreads, 4) void loss_grad_kernel(GradParams gp, tppo_loss_out* __restrict__ out,
                                                                tppo_loss_stats* __restrict__ stats) {
    __shared__ double s_red[kLossThreads / kWave];
    __shared__ int s_flag;
    const LossParams& p = gp.fwd;
    const Plan pl = plan_open(p.plan);
    const int tid = threadIdx.x;
    const bool has_pol = p.logp_new != nullptr, has_val = p.v_new != nullptr;
    const bool plan_ok = pl.hdr->B == p.B && pl.hdr->n_resp == p.n_resp && pl.hdr->has_sets != 0 &&
                         pl.cap >= p.n_resp / kTileTokens + p.B + 1;
    if (!plan_ok) {                                                // not this batch's plan: touch nothing of it
        if (blockIdx.x == 0 && tid == 0) {
            set_status(p.status, TPPO_STATUS_BAD_LAYOUT);
            if (out) write_invalid(out);
        }
        return;
    }
    const int count = (p.n_resp + 4 * kLossThreads - 1) / (4 * kLossThreads);     // work items: parts of frames
    const long long np = has_pol ? pl.hdr->n_policy : 0, nv = has_val ? pl.hdr->n_value : 0;
    const long long den_p = gp.policy_denominator > 0 ? gp.policy_denominator : np;
    const long long den_v = gp.value_denominator > 0 ? gp.value_denominator : nv;
    const float pol_coef = den_p > 0 ? -gp.policy_scale / (float)den_p : 0.f;     // policy_loss = -J_PPO
    const float val_coef = den_v > 0 ? gp.value_scale / (float)den_v : 0.f;

    double pol_acc = 0.0, val_acc = 0.0, ratio_acc = 0.0;
    int pol_clipped = 0, val_clipped = 0;
    FrameDesc ahead = {};
    if ((int)blockIdx.x < count) ahead = load_frame(pl.frames + blockIdx.x / kLossParts);
    for (int f = blockIdx.x; f < count; f += gridDim.x) {
        const FrameDesc d = checked_frame(ahead, p, tid);
        if (f + (int)gridDim.x < count) ahead = load_frame(pl.frames + (f + gridDim.x) / kLossParts);     // the next item's, meanwhile
        const TokenSets ts = token_sets(p, d, f, tid, has_pol, has_val);
        LossRegs cur;
        loss_load(cur, p, ts);
        unshift(cur, ts, f, p.n_resp);
        float pol_t = 0.f, val_t = 0.f, ratio_t = 0.f;
        if (has_pol && ts.n_tok > 0) {
            float gl[4] = {0.f, 0.f, 0.f, 0.f};
            if (ts.pol != 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float rho = ratio_exp(cur.ln[e] - cur.lo[e]);
                    const float u = rho * cur.a[e];
                    const float c = clampf(rho, p.ratio_lo, p.ratio_hi) * cur.a[e];
                    const bool in_set = (ts.pol >> e & 1) != 0, unclipped = u <= c, undefined = u != u;
                    pol_t += in_set ? (undefined ? u : fminf(u, c)) : 0.f;     // select, never multiply by a mask
                    ratio_t += in_set ? rho : 0.f;
                    pol_clipped += (in_set && !unclipped && !undefined) ? 1 : 0;
                    gl[e] = in_set ? (undefined ? u : unclipped ? pol_coef * u : 0.f) : 0.f;
                }
            }
            store4(gp.grad_logp, ts.first, gl, ts.n_tok);
        }
        if (has_val && ts.n_tok > 0) {
            float gv[4] = {0.f, 0.f, 0.f, 0.f};
            if (ts.val != 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float d0 = cur.v[e] - cur.r[e];
                    const float d1 = clampf(cur.v[e], cur.vo[e] - p.xi_low, cur.vo[e] + p.xi_high) - cur.r[e];
                    const float q0 = d0 * d0, q1 = d1 * d1;
                    const bool in_set = (ts.val >> e & 1) != 0, unclipped = q0 >= q1;
                    const bool undefined = value_undefined(d0, d1, cur.vo[e]);
                    const float nan = __builtin_nanf("");
                    val_t += in_set ? (undefined ? nan : fmaxf(q0, q1)) : 0.f;
                    val_clipped += (in_set && !unclipped && !undefined) ? 1 : 0;
                    gv[e] = in_set ? (undefined ? nan : unclipped ? val_coef * d0 : 0.f) : 0.f;
                }
            }
            store4(gp.grad_v, ts.first, gv, ts.n_tok);
        }
        pol_acc += (double)pol_t;
        val_acc += (double)val_t;
        ratio_acc += (double)ratio_t;
    }
    const double sums[kGradSums] = {pol_acc, val_acc, ratio_acc, (double)pol_clipped, (double)val_clipped};
    unsigned long long* mine = pl.finish_words + (int64_t)blockIdx.x * kFinishWords;
#pragma unroll
    for (int q = 0; q < kGradSums; ++q) {
        const double t = block_sum(sums[q], s_red);
        if (tid == 0) publish(mine + 2 * q, p.tag, t);
    }
    if (blockIdx.x != gridDim.x - 1 || (!out && !stats)) return;
    double tot[kGradSums];
    const bool ok = collect_sums<kGradSums, 2>(pl.finish_words, p.tag, (int)gridDim.x, tot, s_red, &s_flag);
    if (tid == 0) {
        if (!ok) {
            set_status(p.status, TPPO_STATUS_TIMEOUT);
#pragma unroll
            for (int q = 0; q < kGradSums; ++q) tot[q] = __builtin_nan("");
        }
        if (out) write_losses(out, tot[0], tot[1], np, nv);
        if (stats) {
            stats->ratio_mean = np > 0 ? (float)(tot[2] / (double)np) : 0.f;
            stats->policy_clip_frac = np > 0 ? (float)(tot[3] / (double)np) : 0.f;
            stats->value_clip_frac = nv > 0 ? (float)(tot[4] / (double)nv) : 0.f;
            stats->reserved = 0.f;
            stats->n_policy_clipped = ok ? (long long)tot[3] : -1;
            stats->n_value_clipped = ok ? (long long)tot[4] : -1;
        }
    }
}

// Batches of fewer than four tokens (the streaming kernels' 16-byte accesses need four): one workgroup, one
// thread per sequence, token by token from the definitions.  kGrad also writes the derivatives.
template <bool kGrad>
__global__ __launch_bounds__(256) void loss_tiny_kernel(GradParams gp, const int32_t* __restrict__ resp_off,
                                                        tppo_loss_out* __restrict__ out,
                                                        tppo_loss_stats* __restrict__ stats) {
    __shared__ double s_red[256 / kWave];
    __shared__ double s_count[2];
    const LossParams& p = gp.fwd;
    const bool has_pol = p.logp_new != nullptr, has_val = p.v_new != nullptr;
    const int tid = threadIdx.x;
    double cnt_p = 0.0, cnt_v = 0.0;
    for (int i = tid; i < p.B; i += blockDim.x) {
        const int win = max(min(resp_off[i + 1], p.n_resp) - max(resp_off[i], 0), 0);
        if (has_pol) cnt_p += (double)min(max(p.keep_len[i], 0), win);
        if (has_val && p.done[i] != 0) cnt_v += (double)win;
    }
    const double tp_ = block_sum(cnt_p, s_red), tv_ = block_sum(cnt_v, s_red);
    if (tid == 0) {
        s_count[0] = tp_;
        s_count[1] = tv_;
    }
    __syncthreads();
    const long long np = (long long)s_count[0], nv = (long long)s_count[1];
    const long long den_p = gp.policy_denominator > 0 ? gp.policy_denominator : np;
    const long long den_v = gp.value_denominator > 0 ? gp.value_denominator : nv;
    const float pol_coef = den_p > 0 ? -gp.policy_scale / (float)den_p : 0.f;
    const float val_coef = den_v > 0 ? gp.value_scale / (float)den_v : 0.f;
    double sums[kGradSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int i = tid; i < p.B; i += blockDim.x) {
        const int lo = max(resp_off[i], 0), hi = min(resp_off[i + 1], p.n_resp);
        const int keep = min(max(p.keep_len[i], 0), max(hi - lo, 0));
        const bool fin = p.done[i] != 0;
        for (int t = lo; t < hi; ++t) {
            if (has_pol) {
                float g = 0.f;
                if (t - lo < keep) {
                    const float rho = ratio_exp(p.logp_new[t] - p.logp_old[t]);
                    const float u = rho * p.adv[t], c = clampf(rho, p.ratio_lo, p.ratio_hi) * p.adv[t];
                    const bool unclipped = u <= c, undefined = u != u;
                    sums[0] += (double)(undefined ? u : fminf(u, c));
                    sums[2] += (double)rho;
                    sums[3] += (!unclipped && !undefined) ? 1.0 : 0.0;
                    g = undefined ? u : unclipped ? pol_coef * u : 0.f;
                }
                if (kGrad) gp.grad_logp[t] = g;
            }
            if (has_val) {
                float g = 0.f;
                if (fin) {
                    const float d0 = p.v_new[t] - p.ret[t];
                    const float d1 = clampf(p.v_new[t], p.v_old[t] - p.xi_low, p.v_old[t] + p.xi_high) - p.ret[t];
                    const bool unclipped = d0 * d0 >= d1 * d1, undefined = value_undefined(d0, d1, p.v_old[t]);
                    sums[1] += (double)(undefined ? __builtin_nanf("") : fmaxf(d0 * d0, d1 * d1));
                    sums[4] += (!unclipped && !undefined) ? 1.0 : 0.0;
                    g = undefined ? __builtin_nanf("") : unclipped ? val_coef * d0 : 0.f;
                }
                if (kGrad) gp.grad_v[t] = g;
            }
        }
    }
    double tot[kGradSums];
#pragma unroll
    for (int q = 0; q < kGradSums; ++q) tot[q] = block_sum(sums[q], s_red);
    if (tid == 0) {
        if (out) write_losses(out, tot[0], tot[1], np, nv);
        if (stats) {
            stats->ratio_mean = np > 0 ? (float)(tot[2] / (double)np) : 0.f;
            stats->policy_clip_frac = np > 0 ? (float)(tot[3] / (double)np) : 0.f;
            stats->value_clip_frac = nv > 0 ? (float)(tot[4] / (double)nv) : 0.f;
            stats->reserved = 0.f;
            stats->n_policy_clipped = (long long)tot[3];
            stats->n_value_clipped = (long long)tot[4];
        }
    }
}

// Workgroups of the persistent grids.  Nothing depends on all of them being resident at once: only the
// workgroup dispatched last waits, and only for workgroups dispatched before it.
static int loss_groups(int64_t n_resp, bool grad) {
    const int64_t frames = (n_resp + 4 * kLossThreads - 1) / (4 * kLossThreads);    // work items
    int groups = grad ? kGradGroups : kLossGroups;
#ifdef TPPO_TUNING
    if (const char* e = getenv("TPPO_LOSS_GROUPS")) {
        const int forced = atoi(e);
        if (forced >= 1 && forced <= kFinishGroups) groups = forced;
    }
#endif
    return frames < groups ? (int)frames : groups;
}

// checks shared by the forward and the backward entry point; on TPPO_OK `plan` points at a plan of this layout
static int loss_prepare(int n_pol_ptr, int n_val_ptr, const int32_t* resp_off, const int32_t* keep_len,
                        const int32_t* done, int64_t B, int64_t n_resp, float eps_low, float eps_high, float xi_low,
                        float xi_high, void* workspace, size_t workspace_bytes, void*& plan, bool& empty,
                        int32_t* status, hipStream_t s) {
    if (B < 0 || n_resp < 0 || n_resp > INT32_MAX - kTileTokens || B > INT32_MAX / 4) return TPPO_ERR_SIZE;
    if (!(eps_low >= 0.f) || !(eps_high >= 0.f) || !(xi_low >= 0.f) || !(xi_high >= 0.f)) return TPPO_ERR_PARAM;
    if ((n_pol_ptr != 0 && n_pol_ptr != 3) || (n_val_ptr != 0 && n_val_ptr != 3)) return TPPO_ERR_NULL;
    if (B > 0 && (!resp_off || !keep_len || !done)) return TPPO_ERR_NULL;
    if (n_resp > 0 && B == 0) return TPPO_ERR_SIZE;
    if (plan_max_tiles(n_resp, B) > INT32_MAX / 8) return TPPO_ERR_SIZE;
    empty = n_resp == 0 || (n_pol_ptr == 0 && n_val_ptr == 0);
    if (plan) {
        if (!is_aligned(plan, 256)) return TPPO_ERR_WORKSPACE;
    } else {
        if (!workspace || !is_aligned(workspace, 256) ||
            workspace_bytes < plan_bytes_for(plan_max_tiles(n_resp, B)))
            return TPPO_ERR_WORKSPACE;
        if (!empty && n_resp >= 4 && launch_plan_build(resp_off, keep_len, done, B, n_resp, plan_max_tiles(n_resp, B), workspace, status, s) != TPPO_OK)
            return TPPO_ERR_LAUNCH;
        plan = workspace;
    }
    return TPPO_OK;
}

static void fill_params(LossParams& p, const float* logp_new, const float* logp_old, const float* adv,
                        const float* v_new, const float* v_old, const float* ret, const int32_t* resp_off,
                        const int32_t* keep_len, const int32_t* done, void* plan, int32_t* status, int64_t B, int64_t n_resp, float eps_low,
                        float eps_high, float xi_low, float xi_high) {
    p.logp_new = logp_new; p.logp_old = logp_old; p.adv = adv;
    p.v_new = v_new; p.v_old = v_old; p.ret = ret;
    p.resp_off = resp_off; p.keep_len = keep_len; p.done = done;
    p.plan = plan; p.status = status;
    p.B = (int)B; p.n_resp = (int)n_resp;
    p.tag = next_call_tag();
    p.ratio_lo = 1.f - eps_low; p.ratio_hi = 1.f + eps_high;
    p.xi_low = xi_low; p.xi_high = xi_high;
}

}  // namespace tppo

extern "C" size_t tppo_ppo_losses_workspace_bytes(int64_t n_resp, int64_t B) {
    if (n_resp < 0 || B < 0) return 256;
    return tppo::plan_bytes_for(tppo::plan_max_tiles(n_resp, B));
}

extern "C" int tppo_ppo_losses(const float* logp_new, const float* logp_old, const float* adv,
                               const float* v_new, const float* v_old, const float* ret,
                               const int32_t* resp_off, const int32_t* keep_len,
                               const int32_t* done, int64_t B, int64_t n_resp, float eps_low,
                               float eps_high, float xi_low, float xi_high, tppo_loss_out* out,
                               void* workspace, size_t workspace_bytes, void* plan, int32_t* status,
                               void* stream) {
    using namespace tppo;
    if (!out) return TPPO_ERR_NULL;
    const int n_pol_ptr = (logp_new != nullptr) + (logp_old != nullptr) + (adv != nullptr);
    const int n_val_ptr = (v_new != nullptr) + (v_old != nullptr) + (ret != nullptr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    bool empty = false;
    const int rc = loss_prepare(n_pol_ptr, n_val_ptr, resp_off, keep_len, done, B, n_resp, eps_low, eps_high, xi_low,
                                xi_high, workspace, workspace_bytes, plan, empty, status, s);
    if (rc != TPPO_OK) return rc;
    if (empty) {
        hipLaunchKernelGGL(loss_empty_kernel, dim3(1), dim3(64), 0, s, out, (tppo_loss_stats*)nullptr);
        return launch_result();
    }
    if (n_resp < 4) {
        GradParams gp = {};
        fill_params(gp.fwd, logp_new, logp_old, adv, v_new, v_old, ret, resp_off, keep_len, done, plan, status, B, n_resp,
                    eps_low, eps_high, xi_low, xi_high);
        hipLaunchKernelGGL(loss_tiny_kernel<false>, dim3(1), dim3(256), 0, s, gp, resp_off, out, (tppo_loss_stats*)nullptr);
        return launch_result();
    }
    LossParams p;
    fill_params(p, logp_new, logp_old, adv, v_new, v_old, ret, resp_off, keep_len, done, plan, status, B, n_resp, eps_low,
                eps_high, xi_low, xi_high);
    hipLaunchKernelGGL(loss_kernel, dim3(loss_groups(n_resp, false)), dim3(kLossThreads), 0, s, p, out);
    return launch_result();
}

extern "C" size_t tppo_ppo_losses_backward_workspace_bytes(int64_t n_resp, int64_t B) {
    return tppo_ppo_losses_workspace_bytes(n_resp, B);
}

extern "C" int tppo_ppo_losses_backward(const float* logp_new, const float* logp_old, const float* adv,
                                        const float* v_new, const float* v_old, const float* ret,
                                        const int32_t* resp_off, const int32_t* keep_len,
                                        const int32_t* done, int64_t B, int64_t n_resp, float eps_low,
                                        float eps_high, float xi_low, float xi_high, float policy_scale,
                                        float value_scale, int64_t policy_denominator,
                                        int64_t value_denominator, float* grad_logp, float* grad_v,
                                        tppo_loss_out* out, tppo_loss_stats* stats, void* workspace,
                                        size_t workspace_bytes, void* plan, int32_t* status, void* stream) {
    using namespace tppo;
    if (!(policy_scale == policy_scale) || !(value_scale == value_scale)) return TPPO_ERR_PARAM;
    const int n_pol_ptr = (logp_new != nullptr) + (logp_old != nullptr) + (adv != nullptr);
    const int n_val_ptr = (v_new != nullptr) + (v_old != nullptr) + (ret != nullptr);
    const bool halves_ok = (n_pol_ptr == 0 || n_pol_ptr == 3) && (n_val_ptr == 0 || n_val_ptr == 3);
    if (halves_ok && ((n_pol_ptr == 3) != (grad_logp != nullptr) || (n_val_ptr == 3) != (grad_v != nullptr)))
        return TPPO_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    bool empty = false;
    const int rc = loss_prepare(n_pol_ptr, n_val_ptr, resp_off, keep_len, done, B, n_resp, eps_low, eps_high, xi_low,
                                xi_high, workspace, workspace_bytes, plan, empty, status, s);
    if (rc != TPPO_OK) return rc;
    if (empty) {
        if (out || stats) hipLaunchKernelGGL(loss_empty_kernel, dim3(1), dim3(64), 0, s, out, stats);
        return launch_result();
    }
    GradParams gp;
    fill_params(gp.fwd, logp_new, logp_old, adv, v_new, v_old, ret, resp_off, keep_len, done, plan, status, B, n_resp, eps_low,
                eps_high, xi_low, xi_high);
    gp.grad_logp = grad_logp; gp.grad_v = grad_v;
    gp.policy_scale = policy_scale; gp.value_scale = value_scale;
    gp.policy_denominator = policy_denominator; gp.value_denominator = value_denominator;
    if (n_resp < 4) {
        hipLaunchKernelGGL(loss_tiny_kernel<true>, dim3(1), dim3(256), 0, s, gp, resp_off, out, stats);
        return launch_result();
    }
    hipLaunchKernelGGL(loss_grad_kernel, dim3(loss_groups(n_resp, true)), dim3(kLossThreads), 0, s, gp, out, stats);
    return launch_result();
}
