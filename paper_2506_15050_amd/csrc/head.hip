// tppo_token_logprobs: log pi_theta(a_t|s_t) of the kept tokens -- the LM head
// W_head h fused with log-softmax and the gather of the sampled token's logit
// (the quantity inside the ratio of Eq. (ppoloss)); logits never reach memory.
//
// bf16 path (matrix cores).  The logits of a 256-token x 256-vocabulary tile
// are accumulated with v_mfma_f32_16x16x32_bf16 (or 32x32x16, see head_tile.h).
// The MFMA "row" operand is the W tile and the "column" operand the gathered
// hidden rows, so the accumulators a lane holds for one block all belong to ONE
// token (column lane % 16) and to different vocabulary entries: the running
// maximum, the running sum of exponentials and the target logit of a token
// live in that lane's registers across all vocabulary tiles of the sweep, with
// no cross-lane traffic until the very end.  The work is (token tiles) x
// (vocabulary splits), handed to a persistent grid (head_tile.h); each pair
// sweeps its share of vocabulary tiles and writes one (max, sumexp, target
// logit) triple per token; a small kernel merges the splits into logp and lse.
//
// Both operands are K-contiguous in memory ([V,H] and [rows,H]), which is the
// layout the MFMA wants for both, so tiles are staged into LDS as 16-byte
// chunks with an XOR swizzle of the chunk index (conflict-free ds_read_b128)
// and read back as operand fragments directly.
#include "head_tile.h"

namespace tppo {

// ------------------------------------------------------------------ generic
// One workgroup per kept token, one wavefront per vocabulary row at a time.
// fp32 FMA; serves TPPO_F32 and bf16 shapes the MFMA path does not take.
constexpr int kGenThreads = 256;
constexpr int kGenMaxH = 16320;               // the hidden row (fp32) and 48 bytes of partial results share 64 KiB of LDS

__device__ __forceinline__ float load_as_float(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float load_as_float(const uint16_t* p, int64_t i) {
    return __uint_as_float((unsigned)p[i] << 16);
}

template <typename T>
__global__ __launch_bounds__(kGenThreads) void head_generic_kernel(
    const T* __restrict__ hidden, int64_t n_rows, int H, int64_t ld_h, const T* __restrict__ w,
    int V, int64_t ld_w, const int32_t* __restrict__ sel_rows,
    const int32_t* __restrict__ sel_targets, int64_t M, const int64_t* __restrict__ m_actual,
    const int32_t* __restrict__ out_index, float* __restrict__ logp, float* __restrict__ lse,
    int32_t* status) {
    extern __shared__ float s_h[];
    __shared__ float s_part[3][kGenThreads / kWave];
    const int64_t m = blockIdx.x;
    const int64_t m_eff = m_actual ? min(M, *m_actual) : M;
    if (m >= m_eff) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = sel_rows[m];
    const int tgt = sel_targets[m];
    const int64_t o = out_index ? (int64_t)out_index[m] : m;
    const bool bad_row = row < 0 || row >= n_rows, bad_tgt = tgt < 0 || tgt >= V;
    if (bad_row || bad_tgt) {
        if (tid == 0) {
            set_status(status, bad_row ? TPPO_STATUS_BAD_ROW : TPPO_STATUS_BAD_TARGET);
            logp[o] = __builtin_nanf("");
            if (lse) lse[o] = __builtin_nanf("");
        }
        return;
    }
    for (int k = tid; k < H; k += kGenThreads) s_h[k] = load_as_float(hidden, row * ld_h + k);
    __syncthreads();
    float mx = -INFINITY, sum = 0.f, tz = 0.f;
    for (int v = wave; v < V; v += kGenThreads / kWave) {
        const T* wr = w + (int64_t)v * ld_w;
        float z = 0.f;
        for (int k = lane; k < H; k += kWave) z = fmaf(s_h[k], load_as_float(wr, k), z);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) z += __shfl_xor(z, off);
        const float mn = fmaxf(mx, z);
        sum = sum * expf(mx - mn) + expf(z - mn);
        mx = mn;
        if (v == tgt) tz = z;
    }
    if (lane == 0) {
        s_part[0][wave] = mx;
        s_part[1][wave] = sum;
        s_part[2][wave] = tz;
    }
    __syncthreads();
    if (tid == 0) {
        float gm = -INFINITY, gs = 0.f, gt = 0.f;
        for (int q = 0; q < kGenThreads / kWave; ++q) gm = fmaxf(gm, s_part[0][q]);
        for (int q = 0; q < kGenThreads / kWave; ++q) {
            if (s_part[1][q] > 0.f) gs += s_part[1][q] * expf(s_part[0][q] - gm);
            gt += s_part[2][q];
        }
        const float l = gm + logf(gs);
        logp[o] = gt - l;
        if (lse) lse[o] = l;
    }
}

// ------------------------------------------------------------------ MFMA path
// Per-lane running log-softmax state of the kTB token columns a lane owns, and
// the two steps that use it: folding a finished 256-wide vocabulary tile, and
// the final merge across lane halves / waves.
template <class C>
struct LaneSoftmax {
    float run_max[C::kTB], run_sum[C::kTB], tgt_logit[C::kTB];
    int tgt[C::kTB];

    __device__ __forceinline__ void init(const HeadParams& p, int64_t tok0, int64_t m_eff, int wt, int lane) {
#pragma unroll
        for (int tb = 0; tb < C::kTB; ++tb) {
            run_max[tb] = kNegBig;
            run_sum[tb] = 0.f;
            tgt_logit[tb] = 0.f;
            const int64_t t = tok0 + wt * C::kWaveT + tb * C::kMI + (lane % C::kMI);
            tgt[tb] = t < m_eff ? p.sel_targets[t] : -1;
        }
    }

    // acc holds logits: lane owns column lane%32 of block tb; entry e of block vb
    // is vocabulary id v_wave + vb*32 + (e/4)*8 + (lane/32)*4 + e%4.  Clears acc.
    __device__ __forceinline__ void fold(typename C::Acc (&acc)[C::kVB][C::kTB], const HeadParams& p, int64_t, int64_t,
                                         int vt, int wv, int, int lane) {
        constexpr int kVB = C::kVB, kTB = C::kTB, kE = C::kAccElems;
        const int grp = lane / C::kMI, V = p.V;
        const int v_wave = vt * C::kTileV + wv * C::kWaveV;
        if (vt * C::kTileV + C::kTileV > V) {                       // ragged last tile: mask ids >= V
#pragma unroll
            for (int vb = 0; vb < kVB; ++vb)
#pragma unroll
                for (int tb = 0; tb < kTB; ++tb)
#pragma unroll
                    for (int e = 0; e < kE; ++e)
                        if (v_wave + C::row_in_wave(vb, e, grp) >= V) acc[vb][tb][e] = -INFINITY;
        }
#pragma unroll
        for (int tb = 0; tb < kTB; ++tb) {
            float mx0 = -INFINITY, mx1 = -INFINITY;
#pragma unroll
            for (int vb = 0; vb < kVB; ++vb)
#pragma unroll
                for (int e = 0; e < kE; e += 2) {
                    mx0 = fmaxf(mx0, acc[vb][tb][e]);
                    mx1 = fmaxf(mx1, acc[vb][tb][e + 1]);
                }
            const float new_max = fmaxf(run_max[tb], fmaxf(mx0, mx1) * kLog2e);
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
            for (int vb = 0; vb < kVB; ++vb)
#pragma unroll
                for (int e = 0; e < kE; e += 4) {
                    s0 += __builtin_amdgcn_exp2f(fmaf(acc[vb][tb][e], kLog2e, -new_max));
                    s1 += __builtin_amdgcn_exp2f(fmaf(acc[vb][tb][e + 1], kLog2e, -new_max));
                    s2 += __builtin_amdgcn_exp2f(fmaf(acc[vb][tb][e + 2], kLog2e, -new_max));
                    s3 += __builtin_amdgcn_exp2f(fmaf(acc[vb][tb][e + 3], kLog2e, -new_max));
                }
            run_sum[tb] = fmaf(run_sum[tb], __builtin_amdgcn_exp2f(run_max[tb] - new_max), (s0 + s1) + (s2 + s3));
            run_max[tb] = new_max;
        }
        // target logit: rare (a lane owns kVB * kAccElems of V ids per tile), so only
        // waves in which some lane hits take the register-select path.  Row r of
        // a block belongs to lane group (r / 4) % kGroups, element (r / (4 kGroups)) * 4 + r % 4.
        bool hit = false;
#pragma unroll
        for (int tb = 0; tb < kTB; ++tb) {
            const int d = tgt[tb] - v_wave;
            hit |= d >= 0 && d < C::kWaveV && ((d >> 2) % C::kGroups) == grp;
        }
        if (__any(hit)) {
#pragma unroll
            for (int tb = 0; tb < kTB; ++tb) {
                const int d = tgt[tb] - v_wave;
                if (d >= 0 && d < C::kWaveV && ((d >> 2) % C::kGroups) == grp) {
                    const int vb_t = d / C::kMI, r = d % C::kMI;
                    const int e_t = (r / (4 * C::kGroups)) * 4 + (r & 3);
                    float z = 0.f;
#pragma unroll
                    for (int vb = 0; vb < kVB; ++vb)
#pragma unroll
                        for (int e = 0; e < kE; ++e) z = (vb == vb_t && e == e_t) ? acc[vb][tb][e] : z;
                    tgt_logit[tb] += z;
                }
            }
        }
#pragma unroll
        for (int vb = 0; vb < kVB; ++vb)
#pragma unroll
            for (int tb = 0; tb < kTB; ++tb)
#pragma unroll
                for (int e = 0; e < kE; ++e) acc[vb][tb][e] = 0.f;
    }

    // Merge the lane groups (same token, different vocabulary rows), then
    // the kWavesV waves that share a token, and write the split's triple.
    // s_merge: LDS scratch [kWavesV][3][kTileT] floats, idle at this point.
    __device__ __forceinline__ void finish(const HeadParams& p, float* s_merge, int64_t tok0, int64_t m_eff,
                                                int sp, int wv, int wt, int lane, int tid) {
        constexpr int kTileT = C::kTileT;
#pragma unroll
        for (int off = C::kMI; off < 64; off <<= 1) {            // butterfly over the 64 / kMI lane groups
#pragma unroll
            for (int tb = 0; tb < C::kTB; ++tb) {
                const float om = __shfl_xor(run_max[tb], off), os = __shfl_xor(run_sum[tb], off);
                const float ot = __shfl_xor(tgt_logit[tb], off);
                const float nm = fmaxf(run_max[tb], om);
                run_sum[tb] = run_sum[tb] * __builtin_amdgcn_exp2f(run_max[tb] - nm) + os * __builtin_amdgcn_exp2f(om - nm);
                run_max[tb] = nm;
                tgt_logit[tb] += ot;
            }
        }
        if (lane < C::kMI) {
#pragma unroll
            for (int tb = 0; tb < C::kTB; ++tb) {
                const int col = wt * C::kWaveT + tb * C::kMI + lane;
                s_merge[(wv * 3 + 0) * kTileT + col] = run_max[tb];
                s_merge[(wv * 3 + 1) * kTileT + col] = run_sum[tb];
                s_merge[(wv * 3 + 2) * kTileT + col] = tgt_logit[tb];
            }
        }
        __syncthreads();
        for (int col = tid; col < kTileT; col += C::kThreads) {
            const int64_t t = tok0 + col;
            if (t >= m_eff) continue;
            float gm = kNegBig, gs = 0.f, gt = 0.f;
#pragma unroll
            for (int q = 0; q < C::kWavesV; ++q) gm = fmaxf(gm, s_merge[(q * 3 + 0) * kTileT + col]);
#pragma unroll
            for (int q = 0; q < C::kWavesV; ++q) {
                gs += s_merge[(q * 3 + 1) * kTileT + col] * __builtin_amdgcn_exp2f(s_merge[(q * 3 + 0) * kTileT + col] - gm);
                gt += s_merge[(q * 3 + 2) * kTileT + col];
            }
            float* out = p.part + (int64_t)sp * p.M + t;
            out[0] = gm;
            out[(int64_t)p.splits * p.M] = gs;
            out[2 * (int64_t)p.splits * p.M] = gt;
        }
    }
};

__global__ __launch_bounds__(256) void head_combine_kernel(
    const float* __restrict__ part, int splits, int64_t M, const int64_t* __restrict__ m_actual,
    const int32_t* __restrict__ sel_rows, const int32_t* __restrict__ sel_targets, int64_t n_rows,
    int V, const int32_t* __restrict__ out_index, float* __restrict__ logp,
    float* __restrict__ lse, int32_t* status) {
    const int64_t m = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t m_eff = m_actual ? min(M, *m_actual) : M;
    if (m >= m_eff) return;
    const int64_t o = out_index ? (int64_t)out_index[m] : m;
    const int64_t row = sel_rows[m];
    const int tgt = sel_targets[m];
    const bool bad_row = row < 0 || row >= n_rows, bad_tgt = tgt < 0 || tgt >= V;
    if (bad_row || bad_tgt) {
        set_status(status, bad_row ? TPPO_STATUS_BAD_ROW : TPPO_STATUS_BAD_TARGET);
        logp[o] = __builtin_nanf("");
        if (lse) lse[o] = __builtin_nanf("");
        return;
    }
    const int64_t plane = (int64_t)splits * M;
    float gm = kNegBig;
    for (int s = 0; s < splits; ++s) gm = fmaxf(gm, part[(int64_t)s * M + m]);
    float gs = 0.f, gt = 0.f;
    for (int s = 0; s < splits; ++s) {
        gs += part[plane + (int64_t)s * M + m] * exp2f(part[(int64_t)s * M + m] - gm);
        gt += part[2 * plane + (int64_t)s * M + m];
    }
    const float l = (gm + log2f(gs)) * kLn2;
    logp[o] = gt - l;
    if (lse) lse[o] = l;
}

// Kernel variants (0 is what the library runs; a tuning build can select another through TPPO_HEAD_VARIANT).
using Cfg0 = HeadCfg<256, 256, 2, 4, 64, 2, 1, 32, 16, 8>;   // v_mfma_f32_16x16x32_bf16, one W block per MFMA step
using Cfg1 = HeadCfg<256, 256, 2, 4, 64, 2, 1, 16, 32>;      // v_mfma_f32_32x32x16_bf16
using Cfg2 = HeadCfg<256, 256, 2, 4, 64, 2, 1, 0, 32>;       // the same, transfers issued back to back
#ifdef TPPO_TUNING
// Two workgroups of 4 wavefronts per CU, 256 x 128 tiles, half-size stages: the two drift apart, so one's
// log-softmax fold and stage hand-overs fall into the other's MFMAs.  Measured: correct, and a third slower
// than variant 0 on every shape (0.34 / 0.38 / 0.38 of peak against 0.43 / 0.53 / 0.54 at H = 1024 / 3584 /
// 5120): half cache lines per transfer and 1.5x the L2 -> LDS bytes per flop cost more than the overlap gains.
using Cfg3 = HeadCfg<256, 128, 2, 2, 32, 2, 2, 24, 16, 8>;
#endif

template <class C>
constexpr HeadVariant make_variant() {
    return {head_mfma_kernel<C, LaneSoftmax>, C::kTileV, C::kTileT, C::kThreads, C::kLdsBytes, C::kWgsPerCu};
}
#ifdef TPPO_TUNING
static const HeadVariant kVariants[] = {make_variant<Cfg0>(), make_variant<Cfg1>(), make_variant<Cfg2>(), make_variant<Cfg3>()};
#else
static const HeadVariant kVariants[] = {make_variant<Cfg0>()};
#endif
[[maybe_unused]] [[maybe_unused]] constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

static const HeadVariant& pick_variant() {
    int id = 0;
#ifdef TPPO_TUNING
    if (const char* e = getenv("TPPO_HEAD_VARIANT")) id = atoi(e);       // tuning builds only
    if (id < 0 || id >= kNumVariants) id = 0;
#endif
    return kVariants[id];
}

static bool mfma_eligible(const void* hidden, int64_t H, int64_t ld_h, const void* w, int64_t ld_w,
                          tppo_dtype dt) {
    return dt == TPPO_BF16 && H >= 64 && H % 64 == 0 && ld_h % 8 == 0 && ld_w % 8 == 0 &&
           is_aligned(hidden, 16) && is_aligned(w, 16);
}

}  // namespace tppo

extern "C" size_t tppo_token_logprobs_workspace_bytes(int64_t M, int64_t H, int64_t V,
                                                      tppo_dtype dt) {
    using namespace tppo;
    (void)H;
    if (M <= 0 || V <= 0 || dt != TPPO_BF16) return 256;
    size_t need = 0;
    for (const HeadVariant& hv : kVariants) {
        const size_t n = (size_t)3 * (size_t)choose_splits(hv, M, V) * (size_t)M * sizeof(float);
        need = n > need ? n : need;
    }
    return round_up(need, 256) + arrivals_bytes(M);
}

extern "C" int tppo_token_logprobs(const void* hidden, int64_t n_rows, int64_t H, int64_t ld_hidden,
                                   const void* w_head, int64_t V, int64_t ld_w, tppo_dtype dt,
                                   const int32_t* sel_rows, const int32_t* sel_targets, int64_t M,
                                   const int64_t* m_actual, const int32_t* out_index, float* logp,
                                   float* lse, void* workspace, size_t workspace_bytes,
                                   int32_t* status, void* stream) {
    using namespace tppo;
    if (dt != TPPO_F32 && dt != TPPO_BF16) return TPPO_ERR_DTYPE;
    if (M < 0 || H < 0 || V < 0 || n_rows < 0 || M > INT32_MAX || V > INT32_MAX - 4096 ||
        H > INT32_MAX)
        return TPPO_ERR_SIZE;
    if (M == 0) return TPPO_OK;
    if (H == 0 || V == 0 || n_rows == 0 || ld_hidden < H || ld_w < H) return TPPO_ERR_SIZE;
    if (!hidden || !w_head || !sel_rows || !sel_targets || !logp) return TPPO_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);

    if (!mfma_eligible(hidden, H, ld_hidden, w_head, ld_w, dt)) {
        if (H > kGenMaxH) return TPPO_ERR_SIZE;
        const size_t lds = (size_t)H * sizeof(float);
        if (dt == TPPO_F32)
            hipLaunchKernelGGL(head_generic_kernel<float>, dim3((unsigned)M), dim3(kGenThreads), lds, s,
                               static_cast<const float*>(hidden), n_rows, (int)H, ld_hidden,
                               static_cast<const float*>(w_head), (int)V, ld_w, sel_rows, sel_targets, M,
                               m_actual, out_index, logp, lse, status);
        else
            hipLaunchKernelGGL(head_generic_kernel<uint16_t>, dim3((unsigned)M), dim3(kGenThreads), lds, s,
                               static_cast<const uint16_t*>(hidden), n_rows, (int)H, ld_hidden,
                               static_cast<const uint16_t*>(w_head), (int)V, ld_w, sel_rows,
                               sel_targets, M, m_actual, out_index, logp, lse, status);
        return launch_result();
    }

    const size_t workspace_bytes_needed = tppo_token_logprobs_workspace_bytes(M, H, V, dt);
    if (!workspace || !is_aligned(workspace, 256) || workspace_bytes < workspace_bytes_needed)
        return TPPO_ERR_WORKSPACE;
    HeadParams p = {};
    p.hidden = static_cast<const uint16_t*>(hidden);
    p.w = static_cast<const uint16_t*>(w_head);
    p.sel_rows = sel_rows;
    p.sel_targets = sel_targets;
    p.m_actual = m_actual;
    p.part = static_cast<float*>(workspace);
    p.n_rows = n_rows; p.ld_h = ld_hidden; p.ld_w = ld_w;
    p.H = (int)H;
    const HeadVariant& hv = pick_variant();
    plan_sweep(p, hv, M, V, static_cast<char*>(workspace) + workspace_bytes_needed - arrivals_bytes(M));
    if (launch_sweep(hv, p, s) != TPPO_OK) return TPPO_ERR_LAUNCH;
    hipLaunchKernelGGL(head_combine_kernel, dim3((unsigned)((M + 255) / 256)), dim3(256), 0, s, p.part,
                       p.splits, M, m_actual, sel_rows, sel_targets, n_rows, (int)V, out_index, logp,
                       lse, status);
    return launch_result();
}

extern "C" int tppo_version(void) { return TPPO_VERSION; }
