// Measurement aid, no part of the attention path: how fast do the matrix cores of this device run
// v_mfma_f32_32x32x16_bf16 when nothing else is in the way?  With all-zero operands the answer is
// the nominal rate (one instruction per 32 clocks and SIMD at the boost clock); with operands like
// the ones attention feeds them (Gaussian values, a different operand pair for every instruction)
// the power limit lowers the clock, and that lower rate is what the pre-fill kernel competes with.
#include "skv_internal.h"

namespace skv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kOps = 8; // operand pairs held in registers

// One wave per SIMD; every wave issues iters x 32 MFMAs back to back on four independent
// accumulators, taking a different pair of its eight A and eight B operands each time.
__global__ __launch_bounds__(256) void calib_mfma_kernel(const u32x4 *__restrict__ operands,
                                                         float *__restrict__ sink, int iters) {
    const int lane = threadIdx.x & 63;
    bf16x8 a[kOps], b[kOps];
#pragma unroll
    for (int i = 0; i < kOps; ++i) {
        a[i] = __builtin_bit_cast(bf16x8, operands[(2 * i) * 64 + lane]);
        b[i] = __builtin_bit_cast(bf16x8, operands[(2 * i + 1) * 64 + lane]);
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[j][k] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kOps; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[(i + j) % kOps], acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int k = 0; k < 16; ++k) s += acc[j][k];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

} // namespace

hipError_t launch_calib_mfma(const void *operands, float *sink, int blocks, int iters, hipStream_t stream) {
    calib_mfma_kernel<<<dim3((unsigned)blocks), 256, 0, stream>>>((const u32x4 *)operands, sink, iters);
    return hipGetLastError();
}

} // namespace skv
