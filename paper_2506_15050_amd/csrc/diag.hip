// tppo_diag_mfma_rate: the matrix-core rate this chip sustains with operands in
// registers -- the inner loop of the LM-head kernel (8 wavefronts per
// workgroup, each a 128 x 64 tile of v_mfma_f32_16x16x32_bf16, one workgroup
// per CU) with no LDS, no global loads and no softmax.  A measuring stick for
// the benchmark's roofline line, not a step of the method.
#include "common.h"

namespace tppo {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 diag_bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float diag_f32x4;

constexpr int kDiagThreads = 512, kDiagGroups = 256;
constexpr int kDiagFragsPerLane = 8 + 4;                       // W-role and token-role fragments of one K step of 32
constexpr int kDiagOperandElems = 64 * kDiagFragsPerLane * 8;  // bf16 values the caller provides

__global__ __launch_bounds__(kDiagThreads, 2) void diag_mfma_rate_kernel(const uint16_t* __restrict__ operands,
                                                                        float* __restrict__ out, int iters) {
    const int lane = threadIdx.x & 63;
    diag_bf16x8 fa[8], fb[4];
    const diag_bf16x8* src = reinterpret_cast<const diag_bf16x8*>(operands) + lane * kDiagFragsPerLane;
#pragma unroll
    for (int i = 0; i < 8; ++i) fa[i] = src[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) fb[i] = src[8 + i];
    diag_f32x4 acc[8][4];
#pragma unroll
    for (int vb = 0; vb < 8; ++vb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[vb][tb][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int vb = 0; vb < 8; ++vb)
#pragma unroll
            for (int tb = 0; tb < 4; ++tb)
                acc[vb][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[vb], fb[tb], acc[vb][tb], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int vb = 0; vb < 8; ++vb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int e = 0; e < 4; ++e) sum += acc[vb][tb][e];
    out[blockIdx.x * kDiagThreads + threadIdx.x] = sum;
}

// Streaming measuring sticks: an elementwise pass over n_read input streams and n_write output streams
// (out = sum of the inputs), lanes on consecutive 16 bytes, grid-stride, nothing else.
constexpr int kStreamThreads = 256, kStreamGroups = 2048, kStreamMax = 8;

template <int NR, int NW>
__global__ __launch_bounds__(kStreamThreads) void diag_streams_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                                      int64_t stride16, int64_t n16, float* sink) {
    float acc = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * kStreamThreads + threadIdx.x; i < n16; i += (int64_t)gridDim.x * kStreamThreads) {
        float4 v[NR];
#pragma unroll
        for (int s = 0; s < NR; ++s) v[s] = src[s * stride16 + i];
        float4 t = v[0];
#pragma unroll
        for (int s = 1; s < NR; ++s) {
            t.x += v[s].x; t.y += v[s].y; t.z += v[s].z; t.w += v[s].w;
        }
#pragma unroll
        for (int s = 0; s < NW; ++s) dst[s * stride16 + i] = t;
        if (NW == 0) acc += (t.x + t.y) + (t.z + t.w);
    }
    if (NW == 0 && acc == 1.2345e-30f) sink[0] = acc;          // keeps the loads alive; practically never taken
}

template <int NR, int NW>
static int launch_streams(const void* src, void* dst, int64_t stride16, int64_t n16, hipStream_t s) {
    hipLaunchKernelGGL((diag_streams_kernel<NR, NW>), dim3(kStreamGroups), dim3(kStreamThreads), 0, s,
                       static_cast<const float4*>(src), static_cast<float4*>(dst), stride16, n16,
                       static_cast<float*>(const_cast<void*>(src)));
    return launch_result();
}

}  // namespace tppo

extern "C" int tppo_diag_streams(const void* src, void* dst, int64_t bytes_per_stream, int64_t stride_bytes,
                                 int32_t n_read, int32_t n_write, void* stream) {
    using namespace tppo;
    if (!src || (n_write > 0 && !dst)) return TPPO_ERR_NULL;
    if (bytes_per_stream < 16 || bytes_per_stream % 16 != 0 || stride_bytes % 16 != 0 || stride_bytes < bytes_per_stream)
        return TPPO_ERR_SIZE;
    if (!is_aligned(src, 16) || (dst && !is_aligned(dst, 16))) return TPPO_ERR_PARAM;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t n16 = bytes_per_stream / 16, st = stride_bytes / 16;
    const int shape = n_read * 10 + n_write;                // the shapes of this library's streaming kernels
    switch (shape) {
        case 10: return launch_streams<1, 0>(src, dst, st, n16, s);
        case 11: return launch_streams<1, 1>(src, dst, st, n16, s);
        case 22: return launch_streams<2, 2>(src, dst, st, n16, s);
        case 12: return launch_streams<1, 2>(src, dst, st, n16, s);
        case 60: return launch_streams<6, 0>(src, dst, st, n16, s);
        case 62: return launch_streams<6, 2>(src, dst, st, n16, s);
        default: return TPPO_ERR_PARAM;
    }
}

extern "C" int tppo_diag_mfma_rate(const void* operands, float* out, int64_t iters, double* flop,
                                   void* stream) {
    using namespace tppo;
    if (!operands || !out) return TPPO_ERR_NULL;
    if (iters < 0 || iters > (1 << 24)) return TPPO_ERR_SIZE;
    if (!is_aligned(operands, 16)) return TPPO_ERR_PARAM;
    hipLaunchKernelGGL(diag_mfma_rate_kernel, dim3(kDiagGroups), dim3(kDiagThreads), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(operands), out, (int)iters);
    if (flop) *flop = (double)kDiagGroups * (kDiagThreads / 64) * (double)iters * 32.0 * 16384.0;
    return launch_result();
}
