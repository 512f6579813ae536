// tppo_ppo_losses: clipped surrogate (Eq. (ppoloss)) and clipped value loss
// (Eqs. (valueclip), (valueloss)) as masked streaming reductions over the
// response-packed arrays.  Token sets follow Sec. 3.2: policy tokens are the
// first keep_len[i] window tokens of each sequence, value tokens all window
// tokens of finished sequences; membership is derived from the per-sequence
// metadata (held in LDS), so no mask array is read, and 16-byte groups with no
// member of a set are not loaded for that set.  Sums are token-level
// (Sec. 4.1.1): fp32 per thread over a few tokens, fp64 across threads and
// workgroups, fixed order, no atomics -> bit-identical reruns.
#include "common.h"

namespace tppo {

constexpr int kLossThreads = 256;
constexpr int kLossTpt = 4;
constexpr int kLossTile = kLossThreads * kLossTpt;
constexpr int kLossMaxGroups = 2048;
constexpr int kLossMaxLdsBytes = 60 * 1024;

struct LossParams {
    const float *logp_new, *logp_old, *adv, *v_new, *v_old, *ret;
    const int32_t *resp_off, *keep_len, *done;
    int B, n_resp, tiles;
    float ratio_lo, ratio_hi, xi_low, xi_high;
    int use_lds, vec;
};

__device__ __forceinline__ float clampf(float x, float lo, float hi) {
    return fminf(fmaxf(x, lo), hi);
}

__device__ __forceinline__ float surrogate(float ln, float lo, float a, float rlo, float rhi) {
    const float rho = expf(ln - lo);
    return fminf(rho * a, clampf(rho, rlo, rhi) * a);
}

__device__ __forceinline__ float value_term(float v, float vo, float r, float xl, float xh) {
    const float d0 = v - r;
    const float d1 = clampf(v, vo - xl, vo + xh) - r;
    return fmaxf(d0 * d0, d1 * d1);
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

__global__ __launch_bounds__(kLossThreads) void loss_partial_kernel(LossParams p,
                                                                    double* __restrict__ partials) {
    extern __shared__ int32_t s_meta[];                // [B+1] offsets, then [B] keep | done << 31
    __shared__ double s_red[kLossThreads / kWave];
    const int tid = threadIdx.x;
    const bool has_pol = p.logp_new != nullptr, has_val = p.v_new != nullptr;

    const int32_t* off = p.resp_off;
    if (p.use_lds) {
        for (int i = tid; i <= p.B; i += kLossThreads) s_meta[i] = p.resp_off[i];
        for (int i = tid; i < p.B; i += kLossThreads) {
            const unsigned keep = (unsigned)max(p.keep_len[i], 0);
            s_meta[p.B + 1 + i] = (int32_t)(keep | (p.done[i] != 0 ? 0x80000000u : 0u));
        }
        __syncthreads();
        off = s_meta;
    }

    float pol_acc = 0.f, val_acc = 0.f;
    for (int j = blockIdx.x; j < p.tiles; j += gridDim.x) {
        const int p0 = j * kLossTile + tid * kLossTpt;
        if (p0 >= p.n_resp) continue;
        int seg = find_segment(off, 0, p.B - 1, p0);
        int seg_lo = off[seg], seg_hi = off[seg + 1];
        bool in_pol[kLossTpt], in_val[kLossTpt];
        bool any_pol = false, any_val = false;
        unsigned kd = 0;
        bool have_kd = false;
#pragma unroll
        for (int k = 0; k < kLossTpt; ++k) {
            const int q = p0 + k;
            in_pol[k] = in_val[k] = false;
            if (q < p.n_resp) {
                while (q >= seg_hi && seg < p.B - 1) {
                    ++seg;
                    seg_lo = off[seg];
                    seg_hi = off[seg + 1];
                    have_kd = false;
                }
                if (q >= seg_lo && q < seg_hi) {
                    if (!have_kd) {
                        kd = p.use_lds ? (unsigned)s_meta[p.B + 1 + seg]
                                       : ((unsigned)max(p.keep_len[seg], 0) |
                                          (p.done[seg] != 0 ? 0x80000000u : 0u));
                        have_kd = true;
                    }
                    in_pol[k] = has_pol && (unsigned)(q - seg_lo) < (kd & 0x7fffffffu);
                    in_val[k] = has_val && (kd >> 31) != 0;
                    any_pol |= in_pol[k];
                    any_val |= in_val[k];
                }
            }
        }
        const bool full = p.vec && p0 + kLossTpt <= p.n_resp;
        if (any_pol) {
            float ln[kLossTpt], lo[kLossTpt], a[kLossTpt];
            if (full) {
                const float4 x = *reinterpret_cast<const float4*>(p.logp_new + p0);
                const float4 y = *reinterpret_cast<const float4*>(p.logp_old + p0);
                const float4 z = *reinterpret_cast<const float4*>(p.adv + p0);
                ln[0] = x.x; ln[1] = x.y; ln[2] = x.z; ln[3] = x.w;
                lo[0] = y.x; lo[1] = y.y; lo[2] = y.z; lo[3] = y.w;
                a[0] = z.x; a[1] = z.y; a[2] = z.z; a[3] = z.w;
            } else {
#pragma unroll
                for (int k = 0; k < kLossTpt; ++k) {
                    ln[k] = in_pol[k] ? p.logp_new[p0 + k] : 0.f;
                    lo[k] = in_pol[k] ? p.logp_old[p0 + k] : 0.f;
                    a[k] = in_pol[k] ? p.adv[p0 + k] : 0.f;
                }
            }
#pragma unroll
            for (int k = 0; k < kLossTpt; ++k) {
                const float t = surrogate(ln[k], lo[k], a[k], p.ratio_lo, p.ratio_hi);
                pol_acc += in_pol[k] ? t : 0.f;        // select, never multiply by a mask
            }
        }
        if (any_val) {
            float v[kLossTpt], vo[kLossTpt], r[kLossTpt];
            if (full) {
                const float4 x = *reinterpret_cast<const float4*>(p.v_new + p0);
                const float4 y = *reinterpret_cast<const float4*>(p.v_old + p0);
                const float4 z = *reinterpret_cast<const float4*>(p.ret + p0);
                v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
                vo[0] = y.x; vo[1] = y.y; vo[2] = y.z; vo[3] = y.w;
                r[0] = z.x; r[1] = z.y; r[2] = z.z; r[3] = z.w;
            } else {
#pragma unroll
                for (int k = 0; k < kLossTpt; ++k) {
                    v[k] = in_val[k] ? p.v_new[p0 + k] : 0.f;
                    vo[k] = in_val[k] ? p.v_old[p0 + k] : 0.f;
                    r[k] = in_val[k] ? p.ret[p0 + k] : 0.f;
                }
            }
#pragma unroll
            for (int k = 0; k < kLossTpt; ++k) {
                const float t = value_term(v[k], vo[k], r[k], p.xi_low, p.xi_high);
                val_acc += in_val[k] ? t : 0.f;
            }
        }
    }
    const double ps = block_sum((double)pol_acc, s_red);
    const double vs = block_sum((double)val_acc, s_red);
    if (tid == 0) {
        partials[2 * blockIdx.x] = ps;
        partials[2 * blockIdx.x + 1] = vs;
    }
}

__global__ __launch_bounds__(kLossThreads) void loss_final_kernel(
    const double* __restrict__ partials, int groups, const int32_t* __restrict__ resp_off,
    const int32_t* __restrict__ keep_len, const int32_t* __restrict__ done, int B, int has_pol,
    int has_val, tppo_loss_out* __restrict__ out) {
    __shared__ double s_red[kLossThreads / kWave];
    __shared__ long long s_cnt[2][kLossThreads / kWave];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double ps = 0.0, vs = 0.0;
    for (int g = tid; g < groups; g += kLossThreads) {
        ps += partials[2 * g];
        vs += partials[2 * g + 1];
    }
    ps = block_sum(ps, s_red);
    vs = block_sum(vs, s_red);
    long long np = 0, nv = 0;
    for (int i = tid; i < B; i += kLossThreads) {
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
    if (tid == 0) {
        np = nv = 0;
        for (int w = 0; w < kLossThreads / kWave; ++w) {
            np += s_cnt[0][w];
            nv += s_cnt[1][w];
        }
        if (!has_pol) np = 0;
        if (!has_val) nv = 0;
        const double policy_sum = -ps, value_sum = 0.5 * vs;
        out->policy_sum = (float)policy_sum;
        out->value_sum = (float)value_sum;
        out->policy_loss = np > 0 ? (float)(policy_sum / (double)np) : 0.f;
        out->value_loss = nv > 0 ? (float)(value_sum / (double)nv) : 0.f;
        out->n_policy = np;
        out->n_value = nv;
    }
}

}  // namespace tppo

extern "C" size_t tppo_ppo_losses_workspace_bytes(int64_t n_resp, int64_t B) {
    (void)n_resp;
    (void)B;
    return (size_t)tppo::kLossMaxGroups * 2 * sizeof(double);
}

extern "C" int tppo_ppo_losses(const float* logp_new, const float* logp_old, const float* adv,
                               const float* v_new, const float* v_old, const float* ret,
                               const int32_t* resp_off, const int32_t* keep_len,
                               const int32_t* done, int64_t B, int64_t n_resp, float eps_low,
                               float eps_high, float xi_low, float xi_high, tppo_loss_out* out,
                               void* workspace, size_t workspace_bytes, int32_t* status,
                               void* stream) {
    using namespace tppo;
    (void)status;
    if (B < 0 || n_resp < 0 || n_resp > INT32_MAX - kLossTile || B > INT32_MAX / 2 - 2) return TPPO_ERR_SIZE;
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
    double* partials = static_cast<double*>(workspace);

    LossParams p;
    p.logp_new = logp_new; p.logp_old = logp_old; p.adv = adv;
    p.v_new = v_new; p.v_old = v_old; p.ret = ret;
    p.resp_off = resp_off; p.keep_len = keep_len; p.done = done;
    p.B = (int)B; p.n_resp = (int)n_resp;
    p.tiles = (int)((n_resp + kLossTile - 1) / kLossTile);
    p.ratio_lo = 1.f - eps_low; p.ratio_hi = 1.f + eps_high;
    p.xi_low = xi_low; p.xi_high = xi_high;
    const size_t lds_bytes = (size_t)(2 * B + 1) * sizeof(int32_t);
    p.use_lds = lds_bytes <= (size_t)kLossMaxLdsBytes;
    p.vec = 1;
    const float* arrs[6] = {logp_new, logp_old, adv, v_new, v_old, ret};
    for (const float* a : arrs)
        if (a && !is_aligned(a, 16)) p.vec = 0;

    int groups = 0;
    if (p.tiles > 0 && (n_pol_ptr || n_val_ptr)) {
        groups = p.tiles < kLossMaxGroups ? p.tiles : kLossMaxGroups;
        hipLaunchKernelGGL(loss_partial_kernel, dim3(groups), dim3(kLossThreads),
                           p.use_lds ? lds_bytes : 0, s, p, partials);
        if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
    }
    hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(kLossThreads), 0, s, partials, groups,
                       resp_off, keep_len, done, (int)B, n_pol_ptr ? 1 : 0, n_val_ptr ? 1 : 0, out);
    return launch_result();
}
