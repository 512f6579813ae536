// tppo_token_logprobs_backward: derivatives of the kept tokens' log-probs with
// respect to the hidden rows and the head matrix, without keeping logits from
// the forward pass.  With z = W h, logp = z[target] - lse:
//     dz[t, v] = g_t * ([v == target_t] - exp(z[t, v] - lse_t))
//     d/dh_t   = sum_v dz[t, v] W[v, :]          (dZ  . W)
//     d/dW_v   = sum_t dz[t, v] h_t              (dZ^T . Hid)
// The logits are recomputed tile by tile with the forward kernel's sweep, whose
// epilogue here turns each finished tile into dz and writes it as bf16 for a
// chunk of tokens at a time; the two products are the same sweep again with a
// plain store epilogue (both operands K-contiguous: W^T, dZ^T and the gathered
// Hid^T are made by a tiled transpose).
#include "head_tile.h"

namespace tppo {

__device__ __forceinline__ uint32_t bf16_rne_bits(float x) {
    uint32_t b = __float_as_uint(x);
    if (x != x) return 0x7FC0u;
    b += 0x7FFFu + ((b >> 16) & 1u);
    return b >> 16;
}

// Epilogue 1: a finished 256 (vocabulary) x 256 (token) tile of logits becomes
// dz; every lane owns one token column per block and writes each group of 4
// consecutive vocabulary entries it holds as one 8-byte store into row t of out[.., ld_out].
template <class C>
struct DzEpilogue {
    float lse2[C::kTB], g[C::kTB];
    int tgt[C::kTB];

    __device__ __forceinline__ void init(const HeadParams& p, int64_t tok0, int64_t m_eff, int wt, int lane) {
#pragma unroll
        for (int tb = 0; tb < C::kTB; ++tb) {
            const int64_t t = tok0 + wt * C::kWaveT + tb * C::kMI + (lane % C::kMI);
            lse2[tb] = 0.f;
            g[tb] = 0.f;
            tgt[tb] = -1;
            if (t < m_eff) {
                const int64_t i = p.aux_index ? (int64_t)p.aux_index[t] : t;
                lse2[tb] = p.aux0[i] * kLog2e;
                g[tb] = p.aux1[i];
                tgt[tb] = p.sel_targets[t];
            }
        }
    }

    __device__ __forceinline__ void fold(typename C::Acc (&acc)[C::kVB][C::kTB], const HeadParams& p, int64_t tok0,
                                         int64_t m_eff, int vt, int wv, int wt, int lane) {
        const int v_lane = vt * C::kTileV + wv * C::kWaveV + (lane / C::kMI) * 4;
        uint16_t* out = static_cast<uint16_t*>(p.out);
#pragma unroll
        for (int tb = 0; tb < C::kTB; ++tb) {
            const int64_t t = tok0 + wt * C::kWaveT + tb * C::kMI + (lane % C::kMI);
            if (t < m_eff) {
                uint16_t* row = out + t * p.ld_out;
#pragma unroll
                for (int vb = 0; vb < C::kVB; ++vb)
#pragma unroll
                    for (int q = 0; q < C::kQuads; ++q) {
                        const int v0 = v_lane + vb * C::kMI + q * (4 * C::kGroups);
                        if (v0 < p.out_cols) {
                            uint32_t h[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int v = v0 + j;
                                const float pz = __builtin_amdgcn_exp2f(fmaf(acc[vb][tb][q * 4 + j], kLog2e, -lse2[tb]));
                                float dz = (v == tgt[tb] ? g[tb] : 0.f) - g[tb] * pz;
                                dz = v < p.V ? dz : 0.f;                     // padding columns of the last tile
                                h[j] = bf16_rne_bits(dz);
                            }
                            uint2 packed;
                            packed.x = h[0] | (h[1] << 16);
                            packed.y = h[2] | (h[3] << 16);
                            *reinterpret_cast<uint2*>(row + v0) = packed;
                        }
                    }
            }
        }
#pragma unroll
        for (int vb = 0; vb < C::kVB; ++vb)
#pragma unroll
            for (int tb = 0; tb < C::kTB; ++tb)
#pragma unroll
                for (int e = 0; e < C::kAccElems; ++e) acc[vb][tb][e] = 0.f;
    }

    __device__ __forceinline__ void finish(const HeadParams&, float*, int64_t, int64_t, int, int, int, int, int) {}
};

// Epilogue 2: plain store of the fp32 tile, out[t, v] (+)= acc -- the sweep as an
// "NT" product out[T, V] = tokens[T, K] . w_role[V, K]^T.
template <class C>
struct StoreEpilogue {
    __device__ __forceinline__ void init(const HeadParams&, int64_t, int64_t, int, int) {}

    __device__ __forceinline__ void fold(typename C::Acc (&acc)[C::kVB][C::kTB], const HeadParams& p, int64_t tok0,
                                         int64_t m_eff, int vt, int wv, int wt, int lane) {
        const int v_lane = vt * C::kTileV + wv * C::kWaveV + (lane / C::kMI) * 4;
        float* out = static_cast<float*>(p.out);
#pragma unroll
        for (int tb = 0; tb < C::kTB; ++tb) {
            const int64_t t = tok0 + wt * C::kWaveT + tb * C::kMI + (lane % C::kMI);
            if (t < m_eff) {
                float* row = out + t * p.ld_out;
#pragma unroll
                for (int vb = 0; vb < C::kVB; ++vb)
#pragma unroll
                    for (int q = 0; q < C::kQuads; ++q) {
                        const int v0 = v_lane + vb * C::kMI + q * (4 * C::kGroups);
                        if (v0 < p.out_cols) {
                            float4 val = make_float4(acc[vb][tb][q * 4], acc[vb][tb][q * 4 + 1],
                                                     acc[vb][tb][q * 4 + 2], acc[vb][tb][q * 4 + 3]);
                            float4* dst = reinterpret_cast<float4*>(row + v0);
                            if (p.accumulate) {
                                const float4 old = *dst;
                                val.x += old.x; val.y += old.y; val.z += old.z; val.w += old.w;
                            }
                            *dst = val;
                        }
                    }
            }
        }
#pragma unroll
        for (int vb = 0; vb < C::kVB; ++vb)
#pragma unroll
            for (int tb = 0; tb < C::kTB; ++tb)
#pragma unroll
                for (int e = 0; e < C::kAccElems; ++e) acc[vb][tb][e] = 0.f;
    }

    __device__ __forceinline__ void finish(const HeadParams&, float*, int64_t, int64_t, int, int, int, int, int) {}
};

// dst[c, r] = src[index ? index[r] : r, c] for r < rows (0 for rows <= r < the
// next multiple of 64), c < cols; 2-byte elements, 64 x 64 tiles through LDS,
// 32-byte accesses on both sides.  cols % 64 == 0; rows of src and dst 16-byte aligned.
constexpr int kTrTile = 64, kTrThreads = 256;
__global__ __launch_bounds__(kTrThreads) void transpose_bf16_kernel(
    const uint16_t* __restrict__ src, int64_t rows, int64_t cols, int64_t ld_src,
    const int32_t* __restrict__ index, int64_t index_rows, uint16_t* __restrict__ dst, int64_t ld_dst) {
    __shared__ uint16_t tile[kTrTile][kTrTile + 2];
    const int64_t r0 = (int64_t)blockIdx.x * kTrTile, c0 = (int64_t)blockIdx.y * kTrTile;
    const int tid = threadIdx.x, i = tid >> 2, part = (tid & 3) * 16;
    {
        const int64_t r = r0 + i;
        uint4 a = make_uint4(0, 0, 0, 0), b = a;
        if (r < rows) {
            int64_t sr = index ? (int64_t)index[r] : r;
            sr = min(max(sr, (int64_t)0), index_rows - 1);
            const uint4* s = reinterpret_cast<const uint4*>(src + sr * ld_src + c0 + part);
            a = s[0];
            b = s[1];
        }
        const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            tile[i][part + 2 * j] = (uint16_t)(w[j] & 0xFFFFu);
            tile[i][part + 2 * j + 1] = (uint16_t)(w[j] >> 16);
        }
    }
    __syncthreads();
    {
        const int64_t c = c0 + i;                          // dst row
        uint32_t w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            w[j] = (uint32_t)tile[part + 2 * j][i] | ((uint32_t)tile[part + 2 * j + 1][i] << 16);
        if (c < cols) {
            uint4* d = reinterpret_cast<uint4*>(dst + c * ld_dst + r0 + part);
            d[0] = make_uint4(w[0], w[1], w[2], w[3]);
            d[1] = make_uint4(w[4], w[5], w[6], w[7]);
        }
    }
}

static int launch_transpose(const uint16_t* src, int64_t rows, int64_t cols, int64_t ld_src, const int32_t* index,
                            int64_t index_rows, uint16_t* dst, int64_t ld_dst, hipStream_t s) {
    const dim3 grid((unsigned)((rows + kTrTile - 1) / kTrTile), (unsigned)(cols / kTrTile));
    hipLaunchKernelGGL(transpose_bf16_kernel, grid, dim3(kTrThreads), 0, s, src, rows, cols, ld_src, index,
                       index_rows, dst, ld_dst);
    return launch_result();
}

using BwdCfg = HeadCfg<256, 256, 2, 4, 64, 2, 1, 32, 16, 8>;
static const HeadVariant kDzVariant = {head_mfma_kernel<BwdCfg, DzEpilogue>, BwdCfg::kTileV, BwdCfg::kTileT,
                                       BwdCfg::kThreads, BwdCfg::kLdsBytes, BwdCfg::kWgsPerCu};
// The products' tiles are deep (K = the vocabulary, or a chunk of tokens) and their splits need no merge, so a
// unit costs next to nothing besides its tiles: the schedule may cut the W-role rows into as many splits as
// there are tiles, which rounds the work to whole tiles per workgroup instead of to five at a time.  Units in
// row-major order, so that the XCDs share the long token-role rows (the operand that does not fit a cache).
static const HeadVariant kGemmVariant = {head_mfma_kernel<BwdCfg, StoreEpilogue>, BwdCfg::kTileV, BwdCfg::kTileT,
                                         BwdCfg::kThreads, BwdCfg::kLdsBytes, BwdCfg::kWgsPerCu, 0.02, 0};

constexpr int64_t kBwdChunkDefault = 98304, kBwdChunkMax = 98304;

struct BwdLayout {
    int64_t v_pad, chunk;              // vocabulary padded to 64; tokens per chunk (multiple of 256)
    size_t off_wt, off_dz, off_dzt, off_hidt, off_arrivals, total;
};

static BwdLayout bwd_layout(int64_t H, int64_t V, int64_t chunk) {
    BwdLayout L;
    L.v_pad = (V + 63) / 64 * 64;
    L.chunk = chunk;
    size_t o = 0;
    L.off_wt = o;       o += round_up((size_t)H * L.v_pad * 2, 256);           // W^T   [H, v_pad]
    L.off_dz = o;       o += round_up((size_t)chunk * L.v_pad * 2, 256);       // dZ    [chunk, v_pad]
    L.off_dzt = o;      o += round_up((size_t)L.v_pad * chunk * 2, 256);       // dZ^T  [v_pad, chunk]
    L.off_hidt = o;     o += round_up((size_t)H * chunk * 2, 256);             // Hid^T [H, chunk]
    L.off_arrivals = o; o += arrivals_bytes(chunk > V ? chunk : V);
    L.total = o;
    return L;
}

}  // namespace tppo

extern "C" size_t tppo_token_logprobs_backward_workspace_bytes(int64_t M, int64_t H, int64_t V, tppo_dtype dt) {
    using namespace tppo;
    if (M <= 0 || H <= 0 || V <= 0 || dt != TPPO_BF16) return 256;
    const int64_t m_round = (M + 255) / 256 * 256;
    return bwd_layout(H, V, m_round < kBwdChunkDefault ? m_round : kBwdChunkDefault).total;
}

extern "C" int tppo_token_logprobs_backward(const void* hidden, int64_t n_rows, int64_t H, int64_t ld_hidden,
                                            const void* w_head, int64_t V, int64_t ld_w, tppo_dtype dt,
                                            const int32_t* sel_rows, const int32_t* sel_targets, int64_t M,
                                            const float* lse, const float* grad_logp, const int32_t* in_index,
                                            float* grad_hidden, float* grad_w, int32_t accumulate_w,
                                            void* workspace, size_t workspace_bytes, int32_t* status,
                                            void* stream) {
    using namespace tppo;
    (void)status;
    if (dt != TPPO_BF16) return TPPO_ERR_DTYPE;
    if (M < 0 || H <= 0 || V <= 0 || n_rows <= 0 || M > INT32_MAX || V > INT32_MAX - 4096 || H > INT32_MAX)
        return TPPO_ERR_SIZE;
    if (ld_hidden < H || ld_w < H) return TPPO_ERR_SIZE;
    if (H % 64 != 0 || ld_hidden % 8 != 0 || ld_w % 8 != 0 || !is_aligned(hidden, 16) || !is_aligned(w_head, 16))
        return TPPO_ERR_PARAM;
    if (M == 0 || (!grad_hidden && !grad_w)) return TPPO_OK;
    if (!hidden || !w_head || !sel_rows || !sel_targets || !lse || !grad_logp) return TPPO_ERR_NULL;
    if ((grad_hidden && !is_aligned(grad_hidden, 16)) || (grad_w && !is_aligned(grad_w, 16))) return TPPO_ERR_PARAM;
    if (!workspace || !is_aligned(workspace, 256)) return TPPO_ERR_WORKSPACE;
    // the largest chunk (multiple of 256 tokens) the workspace holds
    const int64_t m_round = (M + 255) / 256 * 256;
    int64_t chunk = m_round < kBwdChunkMax ? m_round : kBwdChunkMax;
    while (chunk >= 256 && bwd_layout(H, V, chunk).total > workspace_bytes) chunk -= 256;
    if (chunk < 256) return TPPO_ERR_WORKSPACE;
    const BwdLayout L = bwd_layout(H, V, chunk);
    char* ws = static_cast<char*>(workspace);
    uint16_t* wt = reinterpret_cast<uint16_t*>(ws + L.off_wt);
    uint16_t* dz = reinterpret_cast<uint16_t*>(ws + L.off_dz);
    uint16_t* dzt = reinterpret_cast<uint16_t*>(ws + L.off_dzt);
    uint16_t* hidt = reinterpret_cast<uint16_t*>(ws + L.off_hidt);
    void* arrivals = ws + L.off_arrivals;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t* hid = static_cast<const uint16_t*>(hidden);
    const uint16_t* w = static_cast<const uint16_t*>(w_head);

    if (grad_hidden) {      // W^T [H, v_pad], K (= vocabulary) contiguous; padding columns are zero
        if (launch_transpose(w, V, H, ld_w, nullptr, V, wt, L.v_pad, s) != TPPO_OK) return TPPO_ERR_LAUNCH;
    }
    for (int64_t m0 = 0; m0 < M; m0 += chunk) {
        const int64_t mc = M - m0 < chunk ? M - m0 : chunk;
        const int64_t m_pad = (mc + 63) / 64 * 64;
        // 1. dZ[mc, v_pad] (bf16): logits recomputed, softmax derivative applied
        HeadParams p = {};
        p.hidden = hid; p.n_rows = n_rows; p.ld_h = ld_hidden;
        p.w = w; p.ld_w = ld_w; p.H = (int)H;
        p.sel_rows = sel_rows + m0;
        p.sel_targets = sel_targets + m0;
        p.aux0 = in_index ? lse : lse + m0;
        p.aux1 = in_index ? grad_logp : grad_logp + m0;
        p.aux_index = in_index ? in_index + m0 : nullptr;
        p.out = dz; p.ld_out = L.v_pad; p.out_cols = L.v_pad;
        plan_sweep(p, kDzVariant, mc, V, arrivals);
        if (launch_sweep(kDzVariant, p, s) != TPPO_OK) return TPPO_ERR_LAUNCH;
        // 2. grad_hidden[m0 + t, :] = dZ[t, :] . W   (token role: dZ rows; W role: rows of W^T; K = v_pad)
        if (grad_hidden) {
            HeadParams q = {};
            q.hidden = dz; q.n_rows = mc; q.ld_h = L.v_pad;
            q.w = wt; q.ld_w = L.v_pad; q.H = (int)L.v_pad;
            q.out = grad_hidden + m0 * H; q.ld_out = H; q.out_cols = H;
            plan_sweep(q, kGemmVariant, mc, H, arrivals, "TPPO_GH_SPLITS", "TPPO_GH_ORDER");
            if (launch_sweep(kGemmVariant, q, s) != TPPO_OK) return TPPO_ERR_LAUNCH;
        }
        // 3. grad_w[v, :] (+)= dZ^T[v, :] . Hid   (token role: rows of dZ^T; W role: rows of Hid^T; K = m_pad)
        if (grad_w) {
            if (launch_transpose(dz, mc, L.v_pad, L.v_pad, nullptr, mc, dzt, m_pad, s) != TPPO_OK) return TPPO_ERR_LAUNCH;
            if (launch_transpose(hid, mc, H, ld_hidden, sel_rows + m0, n_rows, hidt, m_pad, s) != TPPO_OK)
                return TPPO_ERR_LAUNCH;
            HeadParams q = {};
            q.hidden = dzt; q.n_rows = V; q.ld_h = m_pad;
            q.w = hidt; q.ld_w = m_pad; q.H = (int)m_pad;
            q.out = grad_w; q.ld_out = H; q.out_cols = H;
            q.accumulate = (m0 > 0 || accumulate_w) ? 1 : 0;
            plan_sweep(q, kGemmVariant, V, H, arrivals, "TPPO_GW_SPLITS", "TPPO_GW_ORDER");
            if (launch_sweep(kGemmVariant, q, s) != TPPO_OK) return TPPO_ERR_LAUNCH;
        }
    }
    return TPPO_OK;
}
