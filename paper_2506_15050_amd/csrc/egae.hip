// tppo_egae: Extended GAE (Eq. (egae), Sec. 3.1) and returns R_t (Sec. 2.4) as
// one segmented reverse scan over the response-packed token array.
//
// Both recurrences are affine in the value carried in from the right:
//   A_t = delta_t + (gamma*lambda) A_{t+1},   R_t = r_t + gamma R_{t+1},
// and restart at the last token of every sequence (where the bootstrap value of
// Sec. 3.1 enters delta).  The array is cut into fixed tiles of kTile tokens,
// one workgroup each, independent of sequence boundaries.  A tile
//   1. loads r, V (8 B/token), composes its tokens' affine maps per thread,
//      then across the wavefront with shuffles and across wavefronts via LDS;
//   2. publishes "value at my first token if nothing is carried in" for A and
//      R as one 64-bit {flag, float} word each;
//   3. if its last token is not the end of a sequence, sums the published words
//      of the following tiles of that sequence, weighted by (gamma*lambda)^n
//      resp. gamma^n -- these words depend on no other tile, so there is no
//      chain of waits; tiles to the right have lower workgroup ids and were
//      dispatched earlier, and the wait is bounded;
//   4. replays its tokens with the carry and stores A, R (8 B/token).
// HBM traffic is the algorithmic 16 B/token plus O(tiles) metadata.
//
// Arithmetic: inputs and outputs are fp32; the TD residuals, the affine maps and
// every partial sum are fp64.  With gamma*lambda close to 1 a sequence sums up
// to tens of thousands of residuals whose individual fp32 rounding errors would
// add up (random walk) beyond 1e-5; the kernel is bound by HBM, not by the ALUs,
// so fp64 costs nothing measurable.
#include "common.h"

namespace tppo {

constexpr int kEgaeThreads = 256;
constexpr int kTpt = 8;                               // tokens per thread
constexpr int kTile = kEgaeThreads * kTpt;            // tokens per workgroup
constexpr int kSpinLimit = 1 << 22;

struct EgaeWs {
    int32_t* tile_seg;                // [tiles + 1] sequence that owns a tile's first token
    unsigned long long* agg;          // [tiles][4] {flag << 32 | float bits}: A hi, A lo, R hi, R lo
};

static inline size_t egae_ws_bytes(int64_t tiles) {
    return round_up((size_t)(tiles + 1) * 4, 256) + (size_t)tiles * 32;
}

__device__ __forceinline__ EgaeWs egae_ws(void* ws, int64_t tiles) {
    EgaeWs w;
    w.tile_seg = static_cast<int32_t*>(ws);
    w.agg = reinterpret_cast<unsigned long long*>(static_cast<char*>(ws) +
                                                  ((size_t)(tiles + 1) * 4 + 255) / 256 * 256);
    return w;
}

// Clears the published words and records, for every tile, the sequence that
// contains its first token (written by that sequence's thread: no search).
__global__ __launch_bounds__(256) void egae_init_kernel(const int32_t* __restrict__ resp_off, int B,
                                                        int n_resp, int tiles, void* ws_raw,
                                                        int32_t* status) {
    EgaeWs ws = egae_ws(ws_raw, tiles);
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < tiles) {
#pragma unroll
        for (int q = 0; q < 4; ++q) ws.agg[4 * i + q] = 0ull;
    }
    if (i == 0) {
        ws.tile_seg[tiles] = B - 1;
        if (resp_off[0] != 0 || resp_off[B] != n_resp) set_status(status, TPPO_STATUS_BAD_LAYOUT);
    }
    if (i < B) {
        const int lo = resp_off[i], hi = resp_off[i + 1];
        if (lo < 0 || hi < lo || hi > n_resp) {
            set_status(status, TPPO_STATUS_BAD_LAYOUT);
        } else if (hi > lo) {
            for (int j = (lo + kTile - 1) / kTile; j < tiles && (int64_t)j * kTile < hi; ++j)
                ws.tile_seg[j] = i;
        }
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

// bounded wait for a published word; returns its float payload
__device__ __forceinline__ float wait_word(unsigned long long* p, int32_t* status) {
    unsigned long long w = 0;
    for (int spin = 0; spin < kSpinLimit; ++spin) {
        w = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (w >> 32) return __uint_as_float((unsigned)w);
        __builtin_amdgcn_s_sleep(2);
    }
    set_status(status, TPPO_STATUS_TIMEOUT);
    return 0.f;
}

template <bool kVec>
__global__ __launch_bounds__(kEgaeThreads) void egae_scan_kernel(
    const float* __restrict__ rewards, const float* __restrict__ values,
    const int32_t* __restrict__ resp_off, const int32_t* __restrict__ done,
    const float* __restrict__ bootstrap, int B, int n_resp, int tiles, double gamma, double c,
    double log2_gamma, double log2_c, float* __restrict__ adv, float* __restrict__ ret,
    void* ws_raw, int32_t* status) {
    __shared__ float s_v0[kEgaeThreads + 1];
    __shared__ Affine s_wave[2][kEgaeThreads / kWave];
    __shared__ double s_carry[2];

    EgaeWs ws = egae_ws(ws_raw, tiles);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = tiles - 1 - (int)blockIdx.x;        // right-most tile first
    const int tile_start = j * kTile;
    const int tile_end = min(n_resp, tile_start + kTile);
    const int p0 = tile_start + tid * kTpt;

    // ---- loads (issued first; everything below overlaps their latency)
    float r[kTpt], v[kTpt];
    if (kVec && p0 + kTpt <= n_resp) {
#pragma unroll
        for (int q = 0; q < kTpt / 4; ++q) {
            const float4 rr = reinterpret_cast<const float4*>(rewards + p0)[q];
            const float4 vv = reinterpret_cast<const float4*>(values + p0)[q];
            r[4 * q] = rr.x; r[4 * q + 1] = rr.y; r[4 * q + 2] = rr.z; r[4 * q + 3] = rr.w;
            v[4 * q] = vv.x; v[4 * q + 1] = vv.y; v[4 * q + 2] = vv.z; v[4 * q + 3] = vv.w;
        }
    } else {
#pragma unroll
        for (int k = 0; k < kTpt; ++k) {
            const bool ok = p0 + k < n_resp;
            r[k] = ok ? rewards[p0 + k] : 0.f;
            v[k] = ok ? values[p0 + k] : 0.f;
        }
    }
    float v_after_tile = 0.f;                          // V of the token right of the tile
    if (tid == kEgaeThreads - 1 && tile_end < n_resp)
        v_after_tile = values[tile_end];

    // ---- which sequence owns each of my tokens; where sequences end
    int seg_first = ws.tile_seg[j];
    int seg_last = ws.tile_seg[j + 1];
    seg_first = min(max(seg_first, 0), B - 1);
    seg_last = min(max(seg_last, seg_first), B - 1);
    unsigned end_mask = 0;                             // bit k: token k is the last of its sequence
    float v_end[kTpt];                                 // V(s_l) to use at such a token
#pragma unroll
    for (int k = 0; k < kTpt; ++k) v_end[k] = 0.f;
    int seg = seg_first;
    if (p0 < tile_end) {
        seg = find_segment(resp_off, seg_first, seg_last, p0);
        int seg_end = resp_off[seg + 1];
        if (seg_end <= p0 || resp_off[seg] > p0) {     // metadata does not cover this token
            set_status(status, TPPO_STATUS_BAD_LAYOUT);
            seg_end = INT32_MAX;
        }
#pragma unroll
        for (int k = 0; k < kTpt; ++k) {
            const int p = p0 + k;
            if (p < tile_end) {
                while (p >= seg_end && seg < B - 1) {  // step over finished / empty sequences
                    ++seg;
                    seg_end = resp_off[seg + 1];
                }
                if (p == seg_end - 1) {
                    end_mask |= 1u << k;
                    v_end[k] = done[seg] != 0 ? 0.f : (bootstrap ? bootstrap[seg] : v[k]);
                }
            }
        }
    }

    // ---- V(s_{t+1}) of my last token comes from my right neighbour
    s_v0[tid] = v[0];
    if (tid == kEgaeThreads - 1) s_v0[kEgaeThreads] = v_after_tile;
    __syncthreads();
    const float v_right = s_v0[tid + 1];

    // ---- my tokens as one affine map of the value carried in from the right
    Affine fa = {1.0, 0.0}, fr = {1.0, 0.0};
#pragma unroll
    for (int k = kTpt - 1; k >= 0; --k) {
        if (p0 + k < tile_end) {
            const bool is_end = (end_mask >> k) & 1u;
            const float v_next = is_end ? v_end[k] : (k == kTpt - 1 ? v_right : v[k == kTpt - 1 ? k : k + 1]);
            const double delta = fma(gamma, (double)v_next, (double)r[k]) - (double)v[k];
            if (is_end) {
                fa = {0.0, delta};
                fr = {0.0, (double)r[k]};
            } else {
                fa = {c * fa.a, fma(c, fa.b, delta)};
                fr = {gamma * fr.a, fma(gamma, fr.b, (double)r[k])};
            }
        }
    }

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
    // exclusive suffix inside the wavefront: the inclusive one of my right neighbour
    Affine ea = shfl_down(sa, 1), er = shfl_down(sr, 1);
    if (lane == kWave - 1) {
        ea = {1.0, 0.0};
        er = {1.0, 0.0};
    }
    __syncthreads();
    constexpr int kWaves = kEgaeThreads / kWave;
    for (int w = wave + 1; w < kWaves; ++w) {
        ea = compose(ea, s_wave[0][w]);
        er = compose(er, s_wave[1][w]);
    }

    // ---- publish the tile's own contribution, then collect the carry
    if (wave == 0) {
        if (lane == 0) {
            Affine ta = s_wave[0][0], tr = s_wave[1][0];
            for (int w = 1; w < kWaves; ++w) {
                ta = compose(ta, s_wave[0][w]);
                tr = compose(tr, s_wave[1][w]);
            }
            publish(&ws.agg[4 * j], ta.b);
            publish(&ws.agg[4 * j + 2], tr.b);
        }
        // sequence of the tile's last token; does it run on into the next tile?
        const int s_last = find_segment(resp_off, seg_first, seg_last, tile_end - 1);
        const int s_end = resp_off[s_last + 1];
        double carry_a = 0.0, carry_r = 0.0;
        if (s_end > tile_end && s_end <= n_resp && j + 1 < tiles) {
            const int k_end = (s_end - 1) / kTile;     // tile holding the sequence's last token
            for (int k0 = j + 1; k0 <= k_end; k0 += kWave) {
                const int k = k0 + lane;
                double ta = 0.0, tr = 0.0;
                if (k <= k_end) {
                    const double n = (double)(k - j - 1) * (double)kTile;
                    // weight of the adjacent tile is 1 (also when the factor is 0)
                    const double wa = k == j + 1 ? 1.0 : exp2(n * log2_c);
                    const double wr = k == j + 1 ? 1.0 : exp2(n * log2_gamma);
                    const double ba = (double)wait_word(&ws.agg[4 * k], status) +
                                      (double)wait_word(&ws.agg[4 * k + 1], status);
                    const double br = (double)wait_word(&ws.agg[4 * k + 2], status) +
                                      (double)wait_word(&ws.agg[4 * k + 3], status);
                    ta = wa * ba;
                    tr = wr * br;
                }
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) {
                    ta += __shfl_down(ta, off);
                    tr += __shfl_down(tr, off);
                }
                carry_a += ta;
                carry_r += tr;
            }
        }
        if (lane == 0) {
            s_carry[0] = carry_a;
            s_carry[1] = carry_r;
        }
    }
    __syncthreads();

    // ---- replay my tokens with the true carry and store
    double a_next = fma(ea.a, s_carry[0], ea.b);
    double r_next = fma(er.a, s_carry[1], er.b);
    float out_a[kTpt], out_r[kTpt];
#pragma unroll
    for (int k = kTpt - 1; k >= 0; --k) {
        if (p0 + k < tile_end) {
            const bool is_end = (end_mask >> k) & 1u;
            const float v_next = is_end ? v_end[k] : (k == kTpt - 1 ? v_right : v[k == kTpt - 1 ? k : k + 1]);
            const double delta = fma(gamma, (double)v_next, (double)r[k]) - (double)v[k];
            a_next = is_end ? delta : fma(c, a_next, delta);
            r_next = is_end ? (double)r[k] : fma(gamma, r_next, (double)r[k]);
        }
        out_a[k] = (float)a_next;
        out_r[k] = (float)r_next;
    }
    if (kVec && p0 + kTpt <= n_resp) {
#pragma unroll
        for (int q = 0; q < kTpt / 4; ++q) {
            reinterpret_cast<float4*>(adv + p0)[q] =
                make_float4(out_a[4 * q], out_a[4 * q + 1], out_a[4 * q + 2], out_a[4 * q + 3]);
            reinterpret_cast<float4*>(ret + p0)[q] =
                make_float4(out_r[4 * q], out_r[4 * q + 1], out_r[4 * q + 2], out_r[4 * q + 3]);
        }
    } else {
#pragma unroll
        for (int k = 0; k < kTpt; ++k) {
            if (p0 + k < n_resp) {
                adv[p0 + k] = out_a[k];
                ret[p0 + k] = out_r[k];
            }
        }
    }
}

}  // namespace tppo

extern "C" size_t tppo_egae_workspace_bytes(int64_t n_resp, int64_t B) {
    (void)B;
    if (n_resp <= 0) return 256;
    const int64_t tiles = (n_resp + tppo::kTile - 1) / tppo::kTile;
    return tppo::egae_ws_bytes(tiles);
}

extern "C" int tppo_egae(const float* rewards, const float* values, const int32_t* resp_off,
                         const int32_t* done, const float* bootstrap, int64_t B, int64_t n_resp,
                         float gamma, float lambda, float* adv, float* ret, void* workspace,
                         size_t workspace_bytes, int32_t* status, void* stream) {
    using namespace tppo;
    if (B < 0 || n_resp < 0 || n_resp > INT32_MAX - kTile || B > INT32_MAX - 1) return TPPO_ERR_SIZE;
    if (!(gamma >= 0.f && gamma <= 1.f) || !(lambda >= 0.f && lambda <= 1.f)) return TPPO_ERR_PARAM;
    if (n_resp == 0) return TPPO_OK;
    if (B == 0) return TPPO_ERR_SIZE;
    if (!rewards || !values || !resp_off || !done || !adv || !ret) return TPPO_ERR_NULL;
    if (!workspace || !is_aligned(workspace, 256) ||
        workspace_bytes < tppo_egae_workspace_bytes(n_resp, B))
        return TPPO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int tiles = (int)((n_resp + kTile - 1) / kTile);
    const int init_threads = (int)(B > tiles ? B : tiles);
    hipLaunchKernelGGL(egae_init_kernel, dim3((init_threads + 255) / 256), dim3(256), 0, s, resp_off,
                       (int)B, (int)n_resp, tiles, workspace, status);
    if (launch_result() != TPPO_OK) return TPPO_ERR_LAUNCH;
    const double g = (double)gamma, c = (double)gamma * (double)lambda;
    // log2(0) = -inf makes every weight beyond the next tile exactly 0
    const double log2_gamma = log2(g), log2_c = log2(c);
    const bool vec = is_aligned(rewards, 16) && is_aligned(values, 16) && is_aligned(adv, 16) &&
                     is_aligned(ret, 16);
    if (vec)
        hipLaunchKernelGGL(egae_scan_kernel<true>, dim3(tiles), dim3(kEgaeThreads), 0, s, rewards,
                           values, resp_off, done, bootstrap, (int)B, (int)n_resp, tiles, g, c,
                           log2_gamma, log2_c, adv, ret, workspace, status);
    else
        hipLaunchKernelGGL(egae_scan_kernel<false>, dim3(tiles), dim3(kEgaeThreads), 0, s, rewards,
                           values, resp_off, done, bootstrap, (int)B, (int)n_resp, tiles, g, c,
                           log2_gamma, log2_c, adv, ret, workspace, status);
    return launch_result();
}
