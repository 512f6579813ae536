// tppo_egae: Extended GAE (Eq. (egae), Sec. 3.1) and returns R_t (Sec. 2.4) as
// one segmented reverse scan over the response-packed token array.
//
// Both recurrences are affine in the value carried in from the right:
//   A_t = delta_t + (gamma*lambda) A_{t+1},   R_t = r_t + gamma R_{t+1},
// and restart at the last token of every sequence (where the bootstrap value of
// Sec. 3.1 enters delta).  The tokens are cut into chunks of <= 2048 tokens that
// never straddle two sequences (chunks.h); a small kernel lists them in
// right-to-left processing order.  A persistent grid of workgroups then walks
// the list; for each chunk a workgroup
//   1. loads r, V (8 B/token; the loads of its NEXT chunk are already in flight
//      while it works on this one), composes its tokens' affine maps per
//      thread, across the wavefront with shuffles, across wavefronts via LDS;
//   2. publishes "value at my first token if nothing is carried in" for A and
//      R ({flag, float} words, two per quantity: hi + lo of an fp64);
//   3. if the sequence continues to its right, sums the published words of the
//      following chunks of the sequence, weighted by (gamma*lambda)^n resp.
//      gamma^n.  Those words depend on no other chunk, so there is no chain of
//      waits; the chunks to the right come earlier in the list, so they were
//      started earlier by a co-resident workgroup; the wait is bounded anyway;
//   4. replays its tokens with the carry and stores A, R (8 B/token).
// HBM traffic is the algorithmic 16 B/token plus 16 B per chunk of metadata.
//
// Arithmetic: inputs and outputs are fp32; the TD residuals, the affine maps and
// every partial sum are fp64.  With gamma*lambda close to 1 a sequence sums up
// to tens of thousands of residuals whose individual fp32 rounding errors would
// add up (random walk) beyond 1e-5; the kernel is bound by HBM, not by the ALUs,
// so fp64 costs nothing measurable.
#include <math.h>

#include "chunks.h"

namespace tppo {

constexpr int kSpinLimit = 1 << 22;

struct EgaeWs {
    Chunk* chunks;                    // [cap]
    unsigned long long* agg;          // [cap][4] {flag << 32 | float bits}: A hi, A lo, R hi, R lo
    int32_t* n_chunks;                // [1]
};

static inline size_t egae_ws_bytes(int64_t cap) {
    return round_up((size_t)cap * sizeof(Chunk), 256) + round_up((size_t)cap * 32, 256) + 256;
}

__host__ __device__ __forceinline__ EgaeWs egae_ws(void* ws, int64_t cap) {
    char* p = static_cast<char*>(ws);
    EgaeWs w;
    w.chunks = reinterpret_cast<Chunk*>(p);
    p += ((size_t)cap * sizeof(Chunk) + 255) / 256 * 256;
    w.agg = reinterpret_cast<unsigned long long*>(p);
    p += ((size_t)cap * 32 + 255) / 256 * 256;
    w.n_chunks = reinterpret_cast<int32_t*>(p);
    return w;
}

// the first `parts` workgroups build the chunk list; the others clear the published words
__global__ __launch_bounds__(kBuildThreads) void egae_init_kernel(const int32_t* __restrict__ resp_off,
                                                                  int B, int n_resp, int cap, int parts,
                                                                  void* ws_raw, int32_t* status) {
    EgaeWs ws = egae_ws(ws_raw, cap);
    if ((int)blockIdx.x < parts) {
        build_chunks(resp_off, B, n_resp, ws.chunks, cap, ws.n_chunks, status, blockIdx.x, parts);
    } else {
        const int64_t words = (int64_t)cap * 4;
        for (int64_t i = (int64_t)(blockIdx.x - parts) * kBuildThreads + threadIdx.x; i < words;
             i += (int64_t)(gridDim.x - parts) * kBuildThreads)
            ws.agg[i] = 0ull;
    }
}

struct Affine { double a, b; };   // x -> a*x + b

// f then g in scan order (f is the earlier token range): f(g(x))
__device__ __forceinline__ Affine compose(Affine f, Affine g) {
    return {f.a * g.a, fma(f.a, g.b, f.b)};
}

__device__ __forceinline__ Affine shfl_down(Affine f, int off) {
    return {__shfl_down(f.a, off), __shfl_down(f.b, off)};
}

__device__ __forceinline__ unsigned long long pack_word(float v) {
    return (1ull << 32) | (unsigned long long)__float_as_uint(v);
}

// a double travels as two fp32 words (hi + lo), each with its own flag
__device__ __forceinline__ void publish(unsigned long long* p, double x) {
    const float hi = (float)x, lo = (float)(x - (double)hi);
    __hip_atomic_store(p, pack_word(hi), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 1, pack_word(lo), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Bounded wait for the four words of one chunk (A hi, A lo, R hi, R lo).  All
// four loads of a poll are issued together, so a poll costs one memory round
// trip, not four.
__device__ __forceinline__ void wait_words(unsigned long long* p, double& a, double& r, int32_t* status) {
    for (int spin = 0; spin < kSpinLimit; ++spin) {
        const unsigned long long w0 = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long w1 = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long w2 = __hip_atomic_load(p + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long w3 = __hip_atomic_load(p + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((w0 >> 32) && (w1 >> 32) && (w2 >> 32) && (w3 >> 32)) {
            a = (double)__uint_as_float((unsigned)w0) + (double)__uint_as_float((unsigned)w1);
            r = (double)__uint_as_float((unsigned)w2) + (double)__uint_as_float((unsigned)w3);
            return;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    set_status(status, TPPO_STATUS_TIMEOUT);
    a = 0.0;
    r = 0.0;
}

typedef float float4u __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access, 4-byte aligned

constexpr int kEgaeThreads = 128;                       // 2 wavefronts, 16 tokens per thread:
constexpr int kTpt = kChunkTokens / kEgaeThreads;       // the per-wavefront scan is paid once per 1024 tokens
constexpr int kEgaeWaves = kEgaeThreads / kWave;
constexpr int kEgaeMaxGroups = 1536;                    // 6 workgroups per CU: all co-resident (<= 168 VGPRs)

struct TokenRegs { float r[kTpt], v[kTpt]; };

// Global memory is streamed with consecutive lanes on consecutive 16 bytes (the
// shape that runs at copy speed); the scan wants kTpt consecutive tokens per
// thread.  The two layouts are exchanged through LDS.  A thread's kTpt floats
// occupy 80 bytes there (64 + 16 of padding), which makes both the 16-byte
// writes in token order and the 16-byte reads in thread order conflict-free.
constexpr int kLdsRun = kTpt + 4;                          // floats per thread run, padded
constexpr int kLdsArray = kEgaeThreads * kLdsRun;          // floats per staged array
constexpr int kGroups = kChunkTokens / (4 * kEgaeThreads); // 16-byte groups per thread and array: 4

__device__ __forceinline__ int lds_slot(int token) { return (token / kTpt) * kLdsRun + (token % kTpt); }

struct Raw { float4u r[kGroups], v[kGroups]; float v_after; };

// issue the global loads of a chunk: group g of thread tid = tokens g*512 + tid*4 .. +3.
// kTerminal: there is no reward array; the only reward is terminal[seq] on the last token
// of a finished sequence (Sec. 2.1: the rule-based reward arrives with the end of the response).
template <bool kTerminal>
__device__ __forceinline__ void load_raw(Raw& x, const float* __restrict__ rewards,
                                         const float* __restrict__ values, const Chunk& ch,
                                         const int32_t* __restrict__ done, int tid) {
    const int start = ch.start, len = ch.len();
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
        const int k0 = g * 4 * kEgaeThreads + tid * 4;
        if (k0 + 4 <= len) {
            if (!kTerminal) x.r[g] = *reinterpret_cast<const float4u*>(rewards + start + k0);
            x.v[g] = *reinterpret_cast<const float4u*>(values + start + k0);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool ok = k0 + e < len;
                if (!kTerminal) x.r[g][e] = ok ? rewards[start + k0 + e] : 0.f;
                x.v[g][e] = ok ? values[start + k0 + e] : 0.f;
            }
        }
        if (kTerminal) {
#pragma unroll
            for (int e = 0; e < 4; ++e) x.r[g][e] = 0.f;
            const int last = len - 1 - k0;                          // the chunk's last token, if it is in this group
            if (ch.after == 0 && last >= 0 && last < 4 && done[ch.seg] != 0) {
                const float t = rewards[ch.seg];                    // `rewards` is terminal[B] in this mode
#pragma unroll
                for (int e = 0; e < 4; ++e) x.r[g][e] = e == last ? t : 0.f;
            }
        }
    }
}

// token order -> LDS (call, then __syncthreads, then read_runs)
__device__ __forceinline__ void stage_raw(const Raw& x, float* s_r, float* s_v, int tid) {
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
        const int slot = lds_slot(g * 4 * kEgaeThreads + tid * 4);
        *reinterpret_cast<float4*>(s_r + slot) = make_float4(x.r[g][0], x.r[g][1], x.r[g][2], x.r[g][3]);
        *reinterpret_cast<float4*>(s_v + slot) = make_float4(x.v[g][0], x.v[g][1], x.v[g][2], x.v[g][3]);
    }
}

__device__ __forceinline__ void read_runs(TokenRegs& t, const float* s_r, const float* s_v, int tid) {
#pragma unroll
    for (int q = 0; q < kTpt / 4; ++q) {
        const float4 rr = *reinterpret_cast<const float4*>(s_r + tid * kLdsRun + 4 * q);
        const float4 vv = *reinterpret_cast<const float4*>(s_v + tid * kLdsRun + 4 * q);
        t.r[4 * q] = rr.x; t.r[4 * q + 1] = rr.y; t.r[4 * q + 2] = rr.z; t.r[4 * q + 3] = rr.w;
        t.v[4 * q] = vv.x; t.v[4 * q + 1] = vv.y; t.v[4 * q + 2] = vv.z; t.v[4 * q + 3] = vv.w;
    }
}

// V(s_{t+1}) for a chunk's last token (held by the last thread only): the next
// chunk's first value, or the value of the state after the sequence -- 0 for a
// finished one, else the bootstrap value, by default V(s_{l-1}) (Sec. 3.1)
__device__ __forceinline__ float load_v_after(const Chunk& ch, const float* __restrict__ values,
                                              const int32_t* __restrict__ done,
                                              const float* __restrict__ bootstrap, int tid) {
    float v = 0.f;
    if (tid == kEgaeThreads - 1) {
        const int end = ch.start + ch.len();
        if (ch.after != 0) v = values[end];
        else if (done[ch.seg] == 0) v = bootstrap ? bootstrap[ch.seg] : values[end - 1];
    }
    return v;
}

// x^n for a small non-negative integer n (0^0 = 1)
__device__ __forceinline__ double powi(double x, int n) {
    double r = 1.0;
    while (n > 0) {
        if (n & 1) r *= x;
        x *= x;
        n >>= 1;
    }
    return r;
}

// One thread's tokens.  kFull: all kTpt tokens exist (no per-token guards).
//   pass 1 (kStore = false): the affine maps value-to-my-right -> value-at-my-first-token
//   pass 2 (kStore = true):  the values themselves, from the true value to my right
// The sequence's last token needs no special case: nothing follows it in its
// chunk, its map starts from a = 0 (set by the caller) and its V(s_{t+1}) is v_right.
template <bool kFull, bool kStore>
__device__ __forceinline__ void walk_tokens(const TokenRegs& tk, int n_mine, float v_right, double gamma,
                                            double c, Affine& fa, Affine& fr, float* out_a, float* out_r) {
    double v_next = (double)v_right;
#pragma unroll
    for (int k = kTpt - 1; k >= 0; --k) {
        if (kFull || k < n_mine) {
            const double vk = (double)tk.v[k], rk = (double)tk.r[k];
            const double delta = fma(gamma, v_next, rk) - vk;
            fa.b = fma(c, fa.b, delta);
            fr.b = fma(gamma, fr.b, rk);
            if (!kStore) {
                fa.a *= c;
                fr.a *= gamma;
            }
            v_next = vk;
        }
        if (kStore) {
            out_a[k] = (float)fa.b;
            out_r[k] = (float)fr.b;
        }
    }
}

template <bool kTerminal>
__global__ __launch_bounds__(kEgaeThreads, 3) void egae_scan_kernel(
    const float* __restrict__ rewards, const float* __restrict__ values,
    const int32_t* __restrict__ done, const float* __restrict__ bootstrap, int n_resp, int cap,
    double gamma, double c, double gamma_pow_chunk, double c_pow_chunk, float* __restrict__ adv,
    float* __restrict__ ret, void* ws_raw, int32_t* status) {
    __shared__ __attribute__((aligned(16))) float s_r[kLdsArray];      // rewards in, advantages out
    __shared__ __attribute__((aligned(16))) float s_v[kLdsArray];      // values in, returns out
    __shared__ float s_v0[kEgaeThreads + 1];
    __shared__ Affine s_wave[2][kEgaeWaves];
    __shared__ double s_carry[2];

    EgaeWs ws = egae_ws(ws_raw, cap);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int count = *ws.n_chunks;
    int w = blockIdx.x;
    if (w >= count) return;

    Chunk cur = ws.chunks[w];
    Raw raw;
    load_raw<kTerminal>(raw, rewards, values, cur, done, tid);
    raw.v_after = load_v_after(cur, values, done, bootstrap, tid);

    for (; w < count; w += gridDim.x) {
        const int start = cur.start, len = cur.len(), k0 = tid * kTpt;
        const int n_mine = min(max(len - k0, 0), kTpt);          // my tokens that exist
        // ---- this chunk's data: token order -> LDS -> kTpt consecutive tokens per thread
        stage_raw(raw, s_r, s_v, tid);
        if (tid == kEgaeThreads - 1) s_v0[kEgaeThreads] = raw.v_after;
        __syncthreads();
        TokenRegs tk;
        read_runs(tk, s_r, s_v, tid);
        // ---- start the next chunk's loads before working on this one
        const int w_next = w + gridDim.x;
        Chunk nxt = cur;
        if (w_next < count) {
            nxt = ws.chunks[w_next];
            load_raw<kTerminal>(raw, rewards, values, nxt, done, tid);
            raw.v_after = load_v_after(nxt, values, done, bootstrap, tid);
        }

        // ---- V(s_{t+1}) of my last token: my right neighbour's first value, or for
        // the owner of the chunk's last token the value after the chunk
        s_v0[tid] = tk.v[0];
        __syncthreads();
        const bool owns_last = n_mine > 0 && k0 + n_mine == len;
        const float v_right = owns_last ? s_v0[kEgaeThreads] : s_v0[tid + 1];

        // ---- pass 1: my tokens as one affine map of the value carried in from the right
        const double a0 = (owns_last && cur.after == 0) ? 0.0 : 1.0;   // nothing is carried past a sequence's end
        Affine fa = {a0, 0.0}, fr = {a0, 0.0};
        float* out_a = s_r + tid * kLdsRun;                      // my run in LDS: inputs are in registers by now
        float* out_r = s_v + tid * kLdsRun;
        if (len == kChunkTokens) walk_tokens<true, false>(tk, n_mine, v_right, gamma, c, fa, fr, out_a, out_r);
        else walk_tokens<false, false>(tk, n_mine, v_right, gamma, c, fa, fr, out_a, out_r);

        // ---- suffix composition across the wavefront (inclusive), then wavefronts
        Affine sa = fa, sr = fr;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const Affine ga = shfl_down(sa, off), gr = shfl_down(sr, off);
            if (lane + off < kWave) {
                sa = compose(sa, ga);
                sr = compose(sr, gr);
            }
        }
        if (lane == 0) {
            s_wave[0][wave] = sa;
            s_wave[1][wave] = sr;
        }
        Affine ea = shfl_down(sa, 1), er = shfl_down(sr, 1);      // exclusive: my right neighbour's inclusive
        if (lane == kWave - 1) {
            ea = {1.0, 0.0};
            er = {1.0, 0.0};
        }
        __syncthreads();
        for (int q = wave + 1; q < kEgaeWaves; ++q) {
            ea = compose(ea, s_wave[0][q]);
            er = compose(er, s_wave[1][q]);
        }

        // ---- publish the chunk's own contribution, then collect the carry
        if (wave == 0) {
            if (lane == 0 && cur.number() > 0) {                  // somebody to my left will ask for it
                Affine ta = s_wave[0][0], tr = s_wave[1][0];
                for (int q = 1; q < kEgaeWaves; ++q) {
                    ta = compose(ta, s_wave[0][q]);
                    tr = compose(tr, s_wave[1][q]);
                }
                publish(&ws.agg[4 * (int64_t)w], ta.b);
                publish(&ws.agg[4 * (int64_t)w + 2], tr.b);
            }
            double carry_a = 0.0, carry_r = 0.0;
            const int after = min(cur.after, w);                 // chunks to the right: list entries w-1 .. w-after
            for (int j0 = 1; j0 <= after; j0 += kWave) {
                const int j = j0 + lane;
                double ta = 0.0, tr = 0.0;
                if (j <= after) {
                    // j-1 full chunks lie in between
                    double ba, br;
                    wait_words(&ws.agg[4 * (int64_t)(w - j)], ba, br, status);
                    ta = powi(c_pow_chunk, j - 1) * ba;
                    tr = powi(gamma_pow_chunk, j - 1) * br;
                }
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) {
                    ta += __shfl_down(ta, off);
                    tr += __shfl_down(tr, off);
                }
                carry_a += ta;
                carry_r += tr;
            }
            if (lane == 0) {
                s_carry[0] = carry_a;
                s_carry[1] = carry_r;
            }
        }
        __syncthreads();

        // ---- pass 2: replay my tokens from the true value to my right and store
        Affine va = {0.0, fma(ea.a, s_carry[0], ea.b)}, vr = {0.0, fma(er.a, s_carry[1], er.b)};
        if (a0 == 0.0) {                                         // past a sequence's end there is nothing
            va.b = 0.0;
            vr.b = 0.0;
        }
        if (len == kChunkTokens) walk_tokens<true, true>(tk, n_mine, v_right, gamma, c, va, vr, out_a, out_r);
        else walk_tokens<false, true>(tk, n_mine, v_right, gamma, c, va, vr, out_a, out_r);
        // ---- results (written to my LDS run by pass 2): thread order -> token order -> global
        __syncthreads();
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            const int k0 = g * 4 * kEgaeThreads + tid * 4;
            const int slot = lds_slot(k0);
            const float4 oa = *reinterpret_cast<const float4*>(s_r + slot);
            const float4 orr = *reinterpret_cast<const float4*>(s_v + slot);
            if (k0 + 4 <= len) {
                float4u ua, ur;
                ua[0] = oa.x; ua[1] = oa.y; ua[2] = oa.z; ua[3] = oa.w;
                ur[0] = orr.x; ur[1] = orr.y; ur[2] = orr.z; ur[3] = orr.w;
                *reinterpret_cast<float4u*>(adv + start + k0) = ua;
                *reinterpret_cast<float4u*>(ret + start + k0) = ur;
            } else {
                const float ea_[4] = {oa.x, oa.y, oa.z, oa.w}, er_[4] = {orr.x, orr.y, orr.z, orr.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (k0 + e < len) {
                        adv[start + k0 + e] = ea_[e];
                        ret[start + k0 + e] = er_[e];
                    }
                }
            }
        }
        __syncthreads();                                        // s_r / s_v are refilled by the next chunk
        cur = nxt;
    }
}

}  // namespace tppo

extern "C" size_t tppo_egae_workspace_bytes(int64_t n_resp, int64_t B) {
    if (n_resp <= 0 || B <= 0) return 256;
    return tppo::egae_ws_bytes(tppo::max_chunks(n_resp, B));
}

namespace tppo {
// Workgroups of the scan that the current device keeps resident at the same time.  The look-back waits on
// chunks held by other workgroups, so the grid must never exceed this (else a waiting workgroup could keep
// the one it waits for from starting); asked of the runtime once per device.
static int egae_resident_groups() {
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] > 0) return cached[dev];
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, egae_scan_kernel<false>, kEgaeThreads, 0) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return 0;
    const int n = per_cu * cus;
    cached[dev] = n < kEgaeMaxGroups ? n : kEgaeMaxGroups;
    return cached[dev];
}
}  // namespace tppo

namespace tppo {
// `rewards` is the dense [n_resp] array, or with terminal_mode the per-sequence terminal[B] array
static int egae_launch(const float* rewards, bool terminal_mode, const float* values, const int32_t* resp_off,
                       const int32_t* done, const float* bootstrap, int64_t B, int64_t n_resp,
                       float gamma, float lambda, float* adv, float* ret, void* workspace,
                       size_t workspace_bytes, int32_t* status, void* stream) {
    if (B < 0 || n_resp < 0 || n_resp > INT32_MAX - kChunkTokens || B > INT32_MAX / 4) return TPPO_ERR_SIZE;
    if (!(gamma >= 0.f && gamma <= 1.f) || !(lambda >= 0.f && lambda <= 1.f)) return TPPO_ERR_PARAM;
    if (n_resp == 0) return TPPO_OK;
    if (B == 0) return TPPO_ERR_SIZE;
    if (!rewards || !values || !resp_off || !done || !adv || !ret) return TPPO_ERR_NULL;
    if (!workspace || !is_aligned(workspace, 256) ||
        workspace_bytes < tppo_egae_workspace_bytes(n_resp, B))
        return TPPO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t cap64 = max_chunks(n_resp, B);
    if (cap64 > INT32_MAX / 4) return TPPO_ERR_SIZE;
    const int cap = (int)cap64;
    const int clear_groups = (int)((cap64 * 4 + kBuildThreads * 8 - 1) / (kBuildThreads * 8));
    const int parts = build_parts(B);
    hipLaunchKernelGGL(egae_init_kernel, dim3(parts + (clear_groups < 1 ? 1 : clear_groups)), dim3(kBuildThreads),
                       0, s, resp_off, (int)B, (int)n_resp, cap, parts, workspace, status);
    if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
    const double g = (double)gamma, c = (double)gamma * (double)lambda;
    // weight of a whole chunk in the carry: (gamma*lambda)^2048 resp. gamma^2048
    const double gamma_pow_chunk = pow(g, (double)kChunkTokens), c_pow_chunk = pow(c, (double)kChunkTokens);
    const int resident = egae_resident_groups();
    if (resident < 1) return TPPO_ERR_LAUNCH;
    const int groups = cap < resident ? cap : resident;
    if (terminal_mode)
        hipLaunchKernelGGL(egae_scan_kernel<true>, dim3(groups), dim3(kEgaeThreads), 0, s, rewards, values, done,
                           bootstrap, (int)n_resp, cap, g, c, gamma_pow_chunk, c_pow_chunk, adv, ret, workspace, status);
    else
        hipLaunchKernelGGL(egae_scan_kernel<false>, dim3(groups), dim3(kEgaeThreads), 0, s, rewards, values, done,
                           bootstrap, (int)n_resp, cap, g, c, gamma_pow_chunk, c_pow_chunk, adv, ret, workspace, status);
    return launch_result();
}
}  // namespace tppo

extern "C" int tppo_egae(const float* rewards, const float* values, const int32_t* resp_off,
                         const int32_t* done, const float* bootstrap, int64_t B, int64_t n_resp,
                         float gamma, float lambda, float* adv, float* ret, void* workspace,
                         size_t workspace_bytes, int32_t* status, void* stream) {
    return tppo::egae_launch(rewards, false, values, resp_off, done, bootstrap, B, n_resp, gamma, lambda, adv,
                             ret, workspace, workspace_bytes, status, stream);
}

extern "C" int tppo_egae_terminal(const float* terminal_reward, const float* values, const int32_t* resp_off,
                                  const int32_t* done, const float* bootstrap, int64_t B, int64_t n_resp,
                                  float gamma, float lambda, float* adv, float* ret, void* workspace,
                                  size_t workspace_bytes, int32_t* status, void* stream) {
    return tppo::egae_launch(terminal_reward, true, values, resp_off, done, bootstrap, B, n_resp, gamma, lambda,
                             adv, ret, workspace, workspace_bytes, status, stream);
}
