// tppo_ppo_losses: clipped surrogate (Eq. (ppoloss)) and clipped value loss
// (Eqs. (valueclip), (valueloss)) as masked streaming reductions over the
// response-packed arrays.  Token sets follow Sec. 3.2: policy tokens are the
// first keep_len[i] window tokens of each sequence, value tokens all window
// tokens of finished sequences.  The tokens are cut into chunks that never
// straddle two sequences (chunks.h), so set membership is one comparison per
// token for the policy set and one flag per chunk for the value set: no mask
// array is read, and a chunk outside a set issues no loads for that set.  Sums
// are token-level (Sec. 4.1.1): fp32 per thread over a few tokens, fp64 across
// threads and workgroups, fixed order, no atomics -> bit-identical reruns.
#include <stdlib.h>

#include "chunks.h"

namespace tppo {

constexpr int kLossMaxGroups = 2048;

struct LossWs {
    Chunk* chunks;        // [cap]
    double* partials;     // [kLossMaxGroups][2]
    long long* counts;    // [2]: tokens in the policy set, in the value set
    int32_t* n_chunks;    // [1]
};

static inline size_t loss_ws_bytes(int64_t cap) {
    return round_up((size_t)cap * sizeof(Chunk), 256) + (size_t)kLossMaxGroups * 2 * sizeof(double) + 256;
}

__host__ __device__ __forceinline__ LossWs loss_ws(void* ws, int64_t cap) {
    char* p = static_cast<char*>(ws);
    LossWs w;
    w.chunks = reinterpret_cast<Chunk*>(p);
    p += ((size_t)cap * sizeof(Chunk) + 255) / 256 * 256;
    w.partials = reinterpret_cast<double*>(p);
    p += (size_t)kLossMaxGroups * 2 * sizeof(double);
    w.counts = reinterpret_cast<long long*>(p);
    w.n_chunks = reinterpret_cast<int32_t*>(p + 2 * sizeof(long long));
    return w;
}

struct LossParams {
    const float *logp_new, *logp_old, *adv, *v_new, *v_old, *ret;
    const int32_t *keep_len, *done;
    int cap;
    float ratio_lo, ratio_hi, xi_low, xi_high;
};

// Sizes of the two token sets (Sec. 3.2), from the metadata alone; one workgroup, result valid in thread 0.
__device__ __forceinline__ void count_sets(const int32_t* __restrict__ resp_off, const int32_t* __restrict__ keep_len,
                                           const int32_t* __restrict__ done, int B, long long& n_pol, long long& n_val) {
    __shared__ long long s_cnt[2][kBuildThreads / kWave];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, waves = blockDim.x >> 6;
    long long np = 0, nv = 0;
    for (int i = tid; i < B; i += blockDim.x) {
        const int win = max(resp_off[i + 1] - resp_off[i], 0);
        np += min(max(keep_len[i], 0), win);
        nv += done[i] != 0 ? win : 0;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        np += __shfl_down(np, off);
        nv += __shfl_down(nv, off);
    }
    if (lane == 0) {
        s_cnt[0][wave] = np;
        s_cnt[1][wave] = nv;
    }
    __syncthreads();
    n_pol = n_val = 0;
    if (tid == 0)
        for (int w = 0; w < waves; ++w) {
            n_pol += s_cnt[0][w];
            n_val += s_cnt[1][w];
        }
}

// workgroups 0 .. parts-1 build the chunk list, workgroup `parts` counts the two sets meanwhile
__global__ __launch_bounds__(kBuildThreads) void loss_init_kernel(const int32_t* __restrict__ resp_off,
                                                                  const int32_t* __restrict__ keep_len,
                                                                  const int32_t* __restrict__ done, int B,
                                                                  int n_resp, int cap, int parts, void* ws_raw,
                                                                  int32_t* status) {
    LossWs ws = loss_ws(ws_raw, cap);
    if ((int)blockIdx.x < parts) {
        build_chunks(resp_off, B, n_resp, ws.chunks, cap, ws.n_chunks, status, blockIdx.x, parts);
    } else {
        long long np, nv;
        count_sets(resp_off, keep_len, done, B, np, nv);
        if (threadIdx.x == 0) {
            ws.counts[0] = np;
            ws.counts[1] = nv;
        }
    }
}

typedef float float4u __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access, 4-byte aligned

// exp for the probability ratio: one multiply and the hardware exp2 (relative error ~1e-7 (1 + |x|), far inside
// the tolerances; the library expf costs ~15 more instructions per token in a kernel that is half VALU-bound)
__device__ __forceinline__ float ratio_exp(float x) {
#ifdef TPPO_LIBM_EXP
    return expf(x);
#else
    return __builtin_amdgcn_exp2f(x * 1.4426950408889634f);
#endif
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

// Four consecutive tokens per access, consecutive lanes on consecutive 16 bytes
// (the access shape that streams at copy speed).  `n` = how many of the four are
// in the set; nothing is loaded for n = 0.
__device__ __forceinline__ void load4(float (&x)[4], const float* __restrict__ src, int first, int n) {
    if (n >= 4) {
        const float4u t = *reinterpret_cast<const float4u*>(src + first);
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = t[e];
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = e < n ? src[first + e] : 0.f;
    }
}

// What one thread holds of one chunk: kLossGroups 16-byte groups of each of the six arrays.
constexpr int kLossGroups = kChunkTokens / (4 * kChunkThreads);      // 2
struct LossRegs {
    float ln[kLossGroups][4], lo[kLossGroups][4], a[kLossGroups][4];
    float v[kLossGroups][4], vo[kLossGroups][4], r[kLossGroups][4];
    int n_pol[kLossGroups], n_val[kLossGroups];
};

// issue the loads of a chunk (nothing is loaded for groups that hold no member of a set)
__device__ __forceinline__ void loss_load(LossRegs& x, const LossParams& p, const Chunk& ch, int keep, int fin,
                                          bool has_pol, bool has_val, int tid) {
    const int start = ch.start, len = ch.len();
    const int pol_in_chunk = has_pol ? min(max(keep - ch.number() * kChunkTokens, 0), len) : 0;
    const int val_in_chunk = (has_val && fin != 0) ? len : 0;
#pragma unroll
    for (int g = 0; g < kLossGroups; ++g) {
        const int k0 = g * 4 * kChunkThreads + tid * 4;
        x.n_pol[g] = min(max(pol_in_chunk - k0, 0), 4);
        x.n_val[g] = min(max(val_in_chunk - k0, 0), 4);
        if (x.n_pol[g] > 0) {
            load4(x.ln[g], p.logp_new, start + k0, x.n_pol[g]);
            load4(x.lo[g], p.logp_old, start + k0, x.n_pol[g]);
            load4(x.a[g], p.adv, start + k0, x.n_pol[g]);
        }
        if (x.n_val[g] > 0) {
            load4(x.v[g], p.v_new, start + k0, x.n_val[g]);
            load4(x.vo[g], p.v_old, start + k0, x.n_val[g]);
            load4(x.r[g], p.ret, start + k0, x.n_val[g]);
        }
    }
}

__global__ __launch_bounds__(kChunkThreads) void loss_partial_kernel(LossParams p, void* ws_raw) {
    __shared__ double s_red[kChunkThreads / kWave];
    LossWs ws = loss_ws(ws_raw, p.cap);
    const int tid = threadIdx.x;
    const bool has_pol = p.logp_new != nullptr, has_val = p.v_new != nullptr;
    const int count = *ws.n_chunks;

    float pol_acc = 0.f, val_acc = 0.f;
    int w = blockIdx.x;
    // Software pipeline over the workgroup's chunks: the loads of chunk i+1 are in flight while chunk i is
    // summed, and the descriptor (with its sequence's keep_len / done) of chunk i+2 while chunk i+1 loads.
    LossRegs cur;
    Chunk d_next = {};
    int keep_next = 0, fin_next = 0;
    if (w < count) {
        const Chunk d = ws.chunks[w];
        loss_load(cur, p, d, p.keep_len[d.seg], p.done[d.seg], has_pol, has_val, tid);
        if (w + (int)gridDim.x < count) {
            d_next = ws.chunks[w + gridDim.x];
            keep_next = p.keep_len[d_next.seg];
            fin_next = p.done[d_next.seg];
        }
    }
    for (; w < count; w += gridDim.x) {
        const int w1 = w + gridDim.x, w2 = w1 + gridDim.x;
        LossRegs nxt;
        if (w1 < count) loss_load(nxt, p, d_next, keep_next, fin_next, has_pol, has_val, tid);
        if (w2 < count) {
            d_next = ws.chunks[w2];
            keep_next = p.keep_len[d_next.seg];
            fin_next = p.done[d_next.seg];
        }
#pragma unroll
        for (int g = 0; g < kLossGroups; ++g) {
            if (cur.n_pol[g] > 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float t = surrogate(cur.ln[g][e], cur.lo[g][e], cur.a[g][e], p.ratio_lo, p.ratio_hi);
                    pol_acc += e < cur.n_pol[g] ? t : 0.f;     // select, never multiply by a mask
                }
            }
            if (cur.n_val[g] > 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float t = value_term(cur.v[g][e], cur.vo[g][e], cur.r[g][e], p.xi_low, p.xi_high);
                    val_acc += e < cur.n_val[g] ? t : 0.f;
                }
            }
        }
        if (w1 < count) cur = nxt;
    }
    const double ps = block_sum((double)pol_acc, s_red);
    const double vs = block_sum((double)val_acc, s_red);
    if (tid == 0) {
        ws.partials[2 * blockIdx.x] = ps;
        ws.partials[2 * blockIdx.x + 1] = vs;
    }
}

// `counts`: the set sizes the list-building kernel left (NULL: that kernel did not run, both sets are empty)
__global__ __launch_bounds__(kChunkThreads) void loss_final_kernel(
    const double* __restrict__ partials, int groups, const long long* __restrict__ counts, int has_pol,
    int has_val, tppo_loss_out* __restrict__ out) {
    __shared__ double s_red[kChunkThreads / kWave];
    const int tid = threadIdx.x;
    double ps = 0.0, vs = 0.0;
    for (int g = tid; g < groups; g += kChunkThreads) {
        ps += partials[2 * g];
        vs += partials[2 * g + 1];
    }
    ps = block_sum(ps, s_red);
    vs = block_sum(vs, s_red);
    if (tid == 0) {
        const long long np = (counts && has_pol) ? counts[0] : 0, nv = (counts && has_val) ? counts[1] : 0;
        const double policy_sum = -ps, value_sum = 0.5 * vs;
        out->policy_sum = (float)policy_sum;
        out->value_sum = (float)value_sum;
        out->policy_loss = np > 0 ? (float)(policy_sum / (double)np) : 0.f;
        out->value_loss = nv > 0 ? (float)(value_sum / (double)nv) : 0.f;
        out->n_policy = np;
        out->n_value = nv;
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
// Token-level means: the set sizes are known from the metadata before the pass
// (the list-building kernel counts them), so each derivative is final when it
// is written; tokens outside a set get 0.
constexpr int kGradPartials = 5;       // policy sum, value sum, ratio sum, clipped policy, clipped value

struct GradWs {
    Chunk* chunks;        // [cap]
    double* partials;     // [kLossMaxGroups][kGradPartials]
    long long* counts;    // [2]: tokens in the policy set, in the value set
    int32_t* n_chunks;    // [1]
};

static inline size_t grad_ws_bytes(int64_t cap) {
    return round_up((size_t)cap * sizeof(Chunk), 256) + (size_t)kLossMaxGroups * kGradPartials * sizeof(double) + 256;
}

__host__ __device__ __forceinline__ GradWs grad_ws(void* ws, int64_t cap) {
    char* p = static_cast<char*>(ws);
    GradWs w;
    w.chunks = reinterpret_cast<Chunk*>(p);
    p += ((size_t)cap * sizeof(Chunk) + 255) / 256 * 256;
    w.partials = reinterpret_cast<double*>(p);
    p += (size_t)kLossMaxGroups * kGradPartials * sizeof(double);
    w.counts = reinterpret_cast<long long*>(p);
    w.n_chunks = reinterpret_cast<int32_t*>(p + 2 * sizeof(long long));
    return w;
}

struct GradParams {
    LossParams fwd;
    float* grad_logp;
    float* grad_v;
    float policy_scale, value_scale;
    long long policy_denominator, value_denominator;     // <= 0: the call's own token counts
};

// workgroups 0 .. parts-1 build the chunk list, workgroup `parts` counts the two sets meanwhile
__global__ __launch_bounds__(kBuildThreads) void loss_grad_init_kernel(
    const int32_t* __restrict__ resp_off, const int32_t* __restrict__ keep_len,
    const int32_t* __restrict__ done, int B, int n_resp, int cap, int parts, int has_pol, int has_val,
    void* ws_raw, int32_t* status) {
    GradWs ws = grad_ws(ws_raw, cap);
    if ((int)blockIdx.x < parts) {
        build_chunks(resp_off, B, n_resp, ws.chunks, cap, ws.n_chunks, status, blockIdx.x, parts);
    } else {
        long long np, nv;
        count_sets(resp_off, keep_len, done, B, np, nv);
        if (threadIdx.x == 0) {
            ws.counts[0] = has_pol ? np : 0;
            ws.counts[1] = has_val ? nv : 0;
        }
    }
}

// Four consecutive results per access; `n` = how many of the four exist.
__device__ __forceinline__ void store4(float* __restrict__ dst, int first, const float (&x)[4], int n) {
    if (n >= 4) {
        float4u t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = x[e];
        *reinterpret_cast<float4u*>(dst + first) = t;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (e < n) dst[first + e] = x[e];
    }
}

__global__ __launch_bounds__(kChunkThreads) void loss_grad_kernel(GradParams gp, void* ws_raw) {
    __shared__ double s_red[kChunkThreads / kWave];
    const LossParams& p = gp.fwd;
    GradWs ws = grad_ws(ws_raw, p.cap);
    const int tid = threadIdx.x;
    const bool has_pol = p.logp_new != nullptr, has_val = p.v_new != nullptr;
    const int count = *ws.n_chunks;
    constexpr int kGroups = kChunkTokens / (4 * kChunkThreads);      // 16-byte groups per thread: 2
    const long long den_p = gp.policy_denominator > 0 ? gp.policy_denominator : ws.counts[0];
    const long long den_v = gp.value_denominator > 0 ? gp.value_denominator : ws.counts[1];
    const float pol_coef = den_p > 0 ? -gp.policy_scale / (float)den_p : 0.f;     // policy_loss = -J_PPO
    const float val_coef = den_v > 0 ? gp.value_scale / (float)den_v : 0.f;

    float pol_acc = 0.f, val_acc = 0.f, ratio_acc = 0.f;
    int pol_clipped = 0, val_clipped = 0;
    int w = blockIdx.x;
    Chunk cur = ws.chunks[w < count ? w : 0];
    int keep = 0, fin = 0;
    if (w < count) {
        keep = p.keep_len[cur.seg];
        fin = p.done[cur.seg];
    }
    for (; w < count; w += gridDim.x) {
        const int start = cur.start, len = cur.len();
        const int pol_in_chunk = has_pol ? min(max(keep - cur.number() * kChunkTokens, 0), len) : 0;
        const int val_in_chunk = (has_val && fin != 0) ? len : 0;
        const int w_next = w + gridDim.x;
        Chunk nxt = cur;
        int keep_n = 0, fin_n = 0;
        if (w_next < count) {
            nxt = ws.chunks[w_next];
            keep_n = p.keep_len[nxt.seg];
            fin_n = p.done[nxt.seg];
        }
        float ln[kGroups][4], lo[kGroups][4], a[kGroups][4], v[kGroups][4], vo[kGroups][4], r[kGroups][4];
        int n_pol[kGroups], n_val[kGroups], n_tok[kGroups];
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            const int k0 = g * 4 * kChunkThreads + tid * 4;
            n_tok[g] = min(max(len - k0, 0), 4);
            n_pol[g] = min(max(pol_in_chunk - k0, 0), 4);
            n_val[g] = min(max(val_in_chunk - k0, 0), 4);
            if (n_pol[g] > 0) {
                load4(ln[g], p.logp_new, start + k0, n_pol[g]);
                load4(lo[g], p.logp_old, start + k0, n_pol[g]);
                load4(a[g], p.adv, start + k0, n_pol[g]);
            }
            if (n_val[g] > 0) {
                load4(v[g], p.v_new, start + k0, n_val[g]);
                load4(vo[g], p.v_old, start + k0, n_val[g]);
                load4(r[g], p.ret, start + k0, n_val[g]);
            }
        }
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            const int k0 = g * 4 * kChunkThreads + tid * 4;
            if (has_pol && n_tok[g] > 0) {
                float gl[4] = {0.f, 0.f, 0.f, 0.f};
                if (n_pol[g] > 0) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float rho = ratio_exp(ln[g][e] - lo[g][e]);
                        const float u = rho * a[g][e];
                        const float c = clampf(rho, p.ratio_lo, p.ratio_hi) * a[g][e];
                        const bool in_set = e < n_pol[g], unclipped = u <= c, undefined = u != u;
                        pol_acc += in_set ? (undefined ? u : fminf(u, c)) : 0.f;     // select, never multiply by a mask
                        ratio_acc += in_set ? rho : 0.f;
                        pol_clipped += (in_set && !unclipped && !undefined) ? 1 : 0;
                        gl[e] = in_set ? (undefined ? u : unclipped ? pol_coef * u : 0.f) : 0.f;
                    }
                }
                store4(gp.grad_logp, start + k0, gl, n_tok[g]);
            }
            if (has_val && n_tok[g] > 0) {
                float gv[4] = {0.f, 0.f, 0.f, 0.f};
                if (n_val[g] > 0) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float d0 = v[g][e] - r[g][e];
                        const float d1 = clampf(v[g][e], vo[g][e] - p.xi_low, vo[g][e] + p.xi_high) - r[g][e];
                        const float q0 = d0 * d0, q1 = d1 * d1;
                        const bool in_set = e < n_val[g], unclipped = q0 >= q1;
                        const bool undefined = value_undefined(d0, d1, vo[g][e]);
                        const float nan = __builtin_nanf("");
                        val_acc += in_set ? (undefined ? nan : fmaxf(q0, q1)) : 0.f;
                        val_clipped += (in_set && !unclipped && !undefined) ? 1 : 0;
                        gv[e] = in_set ? (undefined ? nan : unclipped ? val_coef * d0 : 0.f) : 0.f;
                    }
                }
                store4(gp.grad_v, start + k0, gv, n_tok[g]);
            }
        }
        cur = nxt;
        keep = keep_n;
        fin = fin_n;
    }
    const double sums[kGradPartials] = {(double)pol_acc, (double)val_acc, (double)ratio_acc,
                                        (double)pol_clipped, (double)val_clipped};
#pragma unroll
    for (int q = 0; q < kGradPartials; ++q) {
        const double t = block_sum(sums[q], s_red);
        if (tid == 0) ws.partials[kGradPartials * blockIdx.x + q] = t;
    }
}

__global__ void loss_grad_zero_counts_kernel(void* ws_raw, int cap) {
    GradWs ws = grad_ws(ws_raw, cap);
    if (threadIdx.x < 2) ws.counts[threadIdx.x] = 0;
}

__global__ __launch_bounds__(kChunkThreads) void loss_grad_final_kernel(void* ws_raw, int cap, int groups,
                                                                       tppo_loss_out* __restrict__ out,
                                                                       tppo_loss_stats* __restrict__ stats) {
    __shared__ double s_red[kChunkThreads / kWave];
    GradWs ws = grad_ws(ws_raw, cap);
    const int tid = threadIdx.x;
    double acc[kGradPartials] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int g = tid; g < groups; g += kChunkThreads)
#pragma unroll
        for (int q = 0; q < kGradPartials; ++q) acc[q] += ws.partials[kGradPartials * g + q];
    double tot[kGradPartials];
#pragma unroll
    for (int q = 0; q < kGradPartials; ++q) tot[q] = block_sum(acc[q], s_red);
    if (tid == 0) {
        const long long np = ws.counts[0], nv = ws.counts[1];
        const double policy_sum = -tot[0], value_sum = 0.5 * tot[1];
        if (out) {
            out->policy_sum = (float)policy_sum;
            out->value_sum = (float)value_sum;
            out->policy_loss = np > 0 ? (float)(policy_sum / (double)np) : 0.f;
            out->value_loss = nv > 0 ? (float)(value_sum / (double)nv) : 0.f;
            out->n_policy = np;
            out->n_value = nv;
        }
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

}  // namespace tppo

namespace tppo {
// Grid of the persistent streaming kernels: as many workgroups as the device keeps resident at once (asked of
// the runtime once per device and kernel), so that every workgroup starts at time zero and none queues behind.
template <class Kernel>
static int resident_groups(Kernel kernel, int* cache) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return kLossMaxGroups;
    if (cache[dev] > 0) return cache[dev];
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kChunkThreads, 0) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || per_cu < 1)
        return kLossMaxGroups;
    const int n = per_cu * cus;
    cache[dev] = n < kLossMaxGroups ? n : kLossMaxGroups;
    if (const char* e = getenv("TPPO_LOSS_GROUPS")) {      // tuning override
        const int forced = atoi(e);
        if (forced >= 1 && forced <= kLossMaxGroups) cache[dev] = forced;
    }
    return cache[dev];
}
}  // namespace tppo

extern "C" size_t tppo_ppo_losses_workspace_bytes(int64_t n_resp, int64_t B) {
    if (n_resp < 0 || B < 0) return 256;
    return tppo::loss_ws_bytes(tppo::max_chunks(n_resp, B));
}

extern "C" int tppo_ppo_losses(const float* logp_new, const float* logp_old, const float* adv,
                               const float* v_new, const float* v_old, const float* ret,
                               const int32_t* resp_off, const int32_t* keep_len,
                               const int32_t* done, int64_t B, int64_t n_resp, float eps_low,
                               float eps_high, float xi_low, float xi_high, tppo_loss_out* out,
                               void* workspace, size_t workspace_bytes, int32_t* status,
                               void* stream) {
    using namespace tppo;
    if (B < 0 || n_resp < 0 || n_resp > INT32_MAX - kChunkTokens || B > INT32_MAX / 4) return TPPO_ERR_SIZE;
    if (!(eps_low >= 0.f) || !(eps_high >= 0.f) || !(xi_low >= 0.f) || !(xi_high >= 0.f))
        return TPPO_ERR_PARAM;
    if (!out) return TPPO_ERR_NULL;
    const int n_pol_ptr = (logp_new != nullptr) + (logp_old != nullptr) + (adv != nullptr);
    const int n_val_ptr = (v_new != nullptr) + (v_old != nullptr) + (ret != nullptr);
    if ((n_pol_ptr != 0 && n_pol_ptr != 3) || (n_val_ptr != 0 && n_val_ptr != 3)) return TPPO_ERR_NULL;
    if (B > 0 && (!resp_off || !keep_len || !done)) return TPPO_ERR_NULL;
    if (n_resp > 0 && B == 0) return TPPO_ERR_SIZE;
    if (!workspace || !is_aligned(workspace, 256) ||
        workspace_bytes < tppo_ppo_losses_workspace_bytes(n_resp, B))
        return TPPO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t cap64 = max_chunks(n_resp, B);
    if (cap64 > INT32_MAX / 4) return TPPO_ERR_SIZE;
    const int cap = (int)cap64;
    LossWs ws = loss_ws(workspace, cap);

    int groups = 0;
    if (n_resp > 0 && (n_pol_ptr || n_val_ptr)) {
        const int parts = build_parts(B);
        hipLaunchKernelGGL(loss_init_kernel, dim3(parts + 1), dim3(kBuildThreads), 0, s, resp_off, keep_len, done,
                           (int)B, (int)n_resp, cap, parts, workspace, status);
        if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
        LossParams p;
        p.logp_new = logp_new; p.logp_old = logp_old; p.adv = adv;
        p.v_new = v_new; p.v_old = v_old; p.ret = ret;
        p.keep_len = keep_len; p.done = done;
        p.cap = cap;
        p.ratio_lo = 1.f - eps_low; p.ratio_hi = 1.f + eps_high;
        p.xi_low = xi_low; p.xi_high = xi_high;
        static int cache[64] = {};
        const int resident = resident_groups(loss_partial_kernel, cache);
        groups = cap < resident ? cap : resident;
        hipLaunchKernelGGL(loss_partial_kernel, dim3(groups), dim3(kChunkThreads), 0, s, p, workspace);
        if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
    }
    hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(kChunkThreads), 0, s, ws.partials, groups,
                       groups > 0 ? ws.counts : nullptr, n_pol_ptr ? 1 : 0, n_val_ptr ? 1 : 0, out);
    return launch_result();
}

extern "C" size_t tppo_ppo_losses_backward_workspace_bytes(int64_t n_resp, int64_t B) {
    if (n_resp < 0 || B < 0) return 256;
    return tppo::grad_ws_bytes(tppo::max_chunks(n_resp, B));
}

extern "C" int tppo_ppo_losses_backward(const float* logp_new, const float* logp_old, const float* adv,
                                        const float* v_new, const float* v_old, const float* ret,
                                        const int32_t* resp_off, const int32_t* keep_len,
                                        const int32_t* done, int64_t B, int64_t n_resp, float eps_low,
                                        float eps_high, float xi_low, float xi_high, float policy_scale,
                                        float value_scale, int64_t policy_denominator,
                                        int64_t value_denominator, float* grad_logp, float* grad_v,
                                        tppo_loss_out* out, tppo_loss_stats* stats, void* workspace,
                                        size_t workspace_bytes, int32_t* status, void* stream) {
    using namespace tppo;
    if (B < 0 || n_resp < 0 || n_resp > INT32_MAX - kChunkTokens || B > INT32_MAX / 4) return TPPO_ERR_SIZE;
    if (!(eps_low >= 0.f) || !(eps_high >= 0.f) || !(xi_low >= 0.f) || !(xi_high >= 0.f))
        return TPPO_ERR_PARAM;
    if (!(policy_scale == policy_scale) || !(value_scale == value_scale)) return TPPO_ERR_PARAM;
    const int n_pol_ptr = (logp_new != nullptr) + (logp_old != nullptr) + (adv != nullptr);
    const int n_val_ptr = (v_new != nullptr) + (v_old != nullptr) + (ret != nullptr);
    if ((n_pol_ptr != 0 && n_pol_ptr != 3) || (n_val_ptr != 0 && n_val_ptr != 3)) return TPPO_ERR_NULL;
    if ((n_pol_ptr == 3) != (grad_logp != nullptr) || (n_val_ptr == 3) != (grad_v != nullptr)) return TPPO_ERR_NULL;
    if (B > 0 && (!resp_off || !keep_len || !done)) return TPPO_ERR_NULL;
    if (n_resp > 0 && B == 0) return TPPO_ERR_SIZE;
    if (!workspace || !is_aligned(workspace, 256) ||
        workspace_bytes < tppo_ppo_losses_backward_workspace_bytes(n_resp, B))
        return TPPO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t cap64 = max_chunks(n_resp, B);
    if (cap64 > INT32_MAX / 4) return TPPO_ERR_SIZE;
    const int cap = (int)cap64;

    // the list-building kernel also counts the two sets; it runs for an empty batch too (B = 0: zero counts)
    int groups = 0;
    if (B > 0) {
        const int parts = build_parts(B);
        hipLaunchKernelGGL(loss_grad_init_kernel, dim3(parts + 1), dim3(kBuildThreads), 0, s, resp_off, keep_len, done,
                           (int)B, (int)n_resp, cap, parts, n_pol_ptr ? 1 : 0, n_val_ptr ? 1 : 0, workspace, status);
        if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
        if (n_resp > 0 && (n_pol_ptr || n_val_ptr)) {
            GradParams gp;
            gp.fwd.logp_new = logp_new; gp.fwd.logp_old = logp_old; gp.fwd.adv = adv;
            gp.fwd.v_new = v_new; gp.fwd.v_old = v_old; gp.fwd.ret = ret;
            gp.fwd.keep_len = keep_len; gp.fwd.done = done;
            gp.fwd.cap = cap;
            gp.fwd.ratio_lo = 1.f - eps_low; gp.fwd.ratio_hi = 1.f + eps_high;
            gp.fwd.xi_low = xi_low; gp.fwd.xi_high = xi_high;
            gp.grad_logp = grad_logp; gp.grad_v = grad_v;
            gp.policy_scale = policy_scale; gp.value_scale = value_scale;
            gp.policy_denominator = policy_denominator; gp.value_denominator = value_denominator;
            static int cache[64] = {};
            const int resident = resident_groups(loss_grad_kernel, cache);
            groups = cap < resident ? cap : resident;
            hipLaunchKernelGGL(loss_grad_kernel, dim3(groups), dim3(kChunkThreads), 0, s, gp, workspace);
            if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
        }
    }
    if (out || stats) {
        if (B == 0) {       // no metadata kernel ran: counts are zero by definition
            hipLaunchKernelGGL(loss_grad_zero_counts_kernel, dim3(1), dim3(64), 0, s, workspace, cap);
            if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
        }
        hipLaunchKernelGGL(loss_grad_final_kernel, dim3(1), dim3(kChunkThreads), 0, s, workspace, cap, groups,
                           out, stats);
    }
    return launch_result();
}
