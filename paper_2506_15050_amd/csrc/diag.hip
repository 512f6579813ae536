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
// (out = sum of the inputs) and nothing else, in the shape that was measured fastest on this chip for each
// mix: lanes on consecutive 16 bytes, non-temporal loads and stores (every byte is touched once), ONE 16-byte
// element per thread and stream, small workgroups that come and go (the dispatcher keeps the chip full; a
// grid-stride loop of resident workgroups was measured 5-8 % slower with stores in the mix).
typedef float stream_vec __attribute__((ext_vector_type(4)));

template <int NR, int NW, int T>
__global__ __launch_bounds__(T) void diag_streams_kernel(const stream_vec* __restrict__ src, stream_vec* __restrict__ dst,
                                                         int64_t stride16, int64_t n16, float* sink) {
    const int64_t i = (int64_t)blockIdx.x * T + threadIdx.x;
    if (i >= n16) return;
    stream_vec v[NR];
#pragma unroll
    for (int s = 0; s < NR; ++s) v[s] = __builtin_nontemporal_load(src + s * stride16 + i);
    stream_vec t = v[0];
#pragma unroll
    for (int s = 1; s < NR; ++s) t += v[s];
#pragma unroll
    for (int s = 0; s < NW; ++s) __builtin_nontemporal_store(t, dst + s * stride16 + i);
    if (NW == 0 && (t[0] + t[1]) + (t[2] + t[3]) == 1.2345e-30f) sink[0] = t[0];   // keeps the loads alive
}

template <int NR, int NW, int T>
static int launch_streams(const void* src, void* dst, int64_t stride16, int64_t n16, hipStream_t s) {
    const int64_t groups = (n16 + T - 1) / T;
    if (groups > INT32_MAX) return TPPO_ERR_SIZE;
    hipLaunchKernelGGL((diag_streams_kernel<NR, NW, T>), dim3((unsigned)groups), dim3(T), 0, s,
                       static_cast<const stream_vec*>(src), static_cast<stream_vec*>(dst), stride16, n16,
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
        case 10: return launch_streams<1, 0, 64>(src, dst, st, n16, s);
        case 11: return launch_streams<1, 1, 64>(src, dst, st, n16, s);
        case 22: return launch_streams<2, 2, 64>(src, dst, st, n16, s);
        case 12: return launch_streams<1, 2, 64>(src, dst, st, n16, s);
        case 60: return launch_streams<6, 0, 128>(src, dst, st, n16, s);
        case 62: return launch_streams<6, 2, 128>(src, dst, st, n16, s);
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
