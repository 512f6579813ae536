// tppo_diag_mfma_rate: the matrix-core rate this chip sustains with operands in
// registers -- the inner loop of the LM-head kernel (8 wavefronts per
// workgroup, each a 128 x 64 tile of v_mfma_f32_32x32x16_bf16, one workgroup
// per CU) with no LDS, no global loads and no softmax.  A measuring stick for
// the benchmark's roofline line, not a step of the method.
#include "common.h"

namespace tppo {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 diag_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float diag_f32x16;

constexpr int kDiagThreads = 512, kDiagGroups = 256;
constexpr int kDiagFragsPerLane = 2 * (4 + 2);                 // two alternating operand sets
constexpr int kDiagOperandElems = 64 * kDiagFragsPerLane * 8;  // bf16 values the caller provides

__global__ __launch_bounds__(kDiagThreads, 2) void diag_mfma_rate_kernel(const uint16_t* __restrict__ operands,
                                                                        float* __restrict__ out, int iters) {
    const int lane = threadIdx.x & 63;
    diag_bf16x8 fa[2][4], fb[2][2];
    const diag_bf16x8* src = reinterpret_cast<const diag_bf16x8*>(operands) + lane * kDiagFragsPerLane;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < 4; ++i) fa[s][i] = src[s * 6 + i];
#pragma unroll
        for (int i = 0; i < 2; ++i) fb[s][i] = src[s * 6 + 4 + i];
    }
    diag_f32x16 acc[4][2];
#pragma unroll
    for (int vb = 0; vb < 4; ++vb)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[vb][tb][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int vb = 0; vb < 4; ++vb)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
                    acc[vb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s][vb], fb[s][tb], acc[vb][tb], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int vb = 0; vb < 4; ++vb)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int e = 0; e < 16; ++e) sum += acc[vb][tb][e];
    out[blockIdx.x * kDiagThreads + threadIdx.x] = sum;
}

}  // namespace tppo

extern "C" int tppo_diag_mfma_rate(const void* operands, float* out, int64_t iters, double* flop,
                                   void* stream) {
    using namespace tppo;
    if (!operands || !out) return TPPO_ERR_NULL;
    if (iters < 0 || iters > (1 << 24)) return TPPO_ERR_SIZE;
    if (!is_aligned(operands, 16)) return TPPO_ERR_PARAM;
    hipLaunchKernelGGL(diag_mfma_rate_kernel, dim3(kDiagGroups), dim3(kDiagThreads), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(operands), out, (int)iters);
    if (flop) *flop = (double)kDiagGroups * (kDiagThreads / 64) * (double)iters * 16.0 * 32768.0;
    return launch_result();
}
