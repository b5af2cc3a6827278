// Measurement aid, no part of the attention path: how fast do the matrix cores of this device run
// v_mfma_f32_32x32x16_bf16 when nothing else is in the way?  With all-zero operands the answer is
// the nominal rate (one instruction per 32 clocks and SIMD at the boost clock); with operands like
// the ones attention feeds them (Gaussian values, a different operand pair for every instruction)
// the power limit lowers the clock, and that lower rate is what the pre-fill kernel competes with.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "skv_calib.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kOps = 8; // operand pairs held in registers

// One wave per SIMD; every wave issues iters x 32 MFMAs back to back on four independent
// accumulators, taking a different pair of its eight A and eight B operands each time.
// MIX adds, between the MFMAs, the other work a flash-attention tile does per MFMA, with no
// dependency on the MFMAs (so nothing waits: what changes is the power drawn, hence the clock):
//   bit 0: four vector instructions per MFMA (three fma and one exp2: scale, maximum, exponent,
//          row sum of one score per lane),
//   bit 1: LDS operand reads at the pre-fill kernel's rate, one 128-bit read (a K operand) and
//          two transposing 64-bit reads (a V^T operand) per four MFMAs.
template <int MIX>
__global__ __launch_bounds__(256) void calib_mfma_kernel(const u32x4 *__restrict__ operands,
                                                         float *__restrict__ sink, int iters) {
    __shared__ u32x4 lds[MIX & 2 ? 4096 : 1]; // 64 KiB of operand-like data
    const int lane = threadIdx.x & 63;
    if (MIX & 2) {
        for (int i = threadIdx.x; i < 4096; i += 256) lds[i] = operands[i & 1023];
        __syncthreads();
    }
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
    // side state: 16 values per lane that stay bounded under x <- c1 x + c2
    float x[16], y[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 16; ++k) x[k] = __builtin_bit_cast(float, operands[k * 64 + lane][0] & 0xffff0000u);
    const float c1 = -0.9990234375f, c2 = 0.01f;
    const uint32_t addr = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char *)lds) + lane * 16;
    u32x4 r0 = {0, 0, 0, 0};
    u32x2 t0 = {0, 0}, t1 = t0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kOps; ++i) {
            if (MIX & 2) {
                const uint32_t at = addr + ((it * kOps + i) & 15) * 4096;
                asm volatile("ds_read_b128 %0, %1" : "=v"(r0) : "v"(at));
                asm volatile("ds_read_b64_tr_b16 %0, %1 offset:1024" : "=v"(t0) : "v"(at));
                asm volatile("ds_read_b64_tr_b16 %0, %1 offset:2048" : "=v"(t1) : "v"(at));
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[(i + j) % kOps], acc[j], 0, 0, 0);
                if (MIX & 1) {
                    const int k = 4 * j;
                    asm volatile("v_fma_f32 %0, %0, %3, %4\n\tv_fma_f32 %1, %1, %3, %4\n\tv_fma_f32 %2, %2, %3, %4"
                                 : "+v"(x[k]), "+v"(x[k + 1]), "+v"(x[k + 2])
                                 : "v"(c1), "v"(c2));
                    asm volatile("v_exp_f32 %0, %1" : "=v"(y[j]) : "v"(x[k + 3]));
                }
            }
            if (MIX & 2) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                x[0] += __builtin_bit_cast(float, (r0[0] ^ t0[0] ^ t1[1]) & 0x007fffffu); // keeps the reads alive (a denormal)
            }
        }
    }
    float s = 0.f, side = y[0] + y[1] + y[2] + y[3];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int k = 0; k < 16; ++k) s += acc[j][k];
#pragma unroll
    for (int k = 0; k < 16; ++k) side += x[k];
    // the sink receives the MFMA result alone; the side work is kept alive by a store that does not happen
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = side == 123456.789f ? side : s;
}

hipError_t launch_calib_mfma(const void *operands, float *sink, int blocks, int iters, int mix, hipStream_t stream) {
    const dim3 grid((unsigned)blocks);
    const u32x4 *ops = (const u32x4 *)operands;
    switch (mix) {
    case 0: calib_mfma_kernel<0><<<grid, 256, 0, stream>>>(ops, sink, iters); break;
    case 1: calib_mfma_kernel<1><<<grid, 256, 0, stream>>>(ops, sink, iters); break;
    case 2: calib_mfma_kernel<2><<<grid, 256, 0, stream>>>(ops, sink, iters); break;
    case 3: calib_mfma_kernel<3><<<grid, 256, 0, stream>>>(ops, sink, iters); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace

extern "C" {

int32_t skv_calib_mfma_mix_bf16(const void *operands, float *sink, int32_t blocks, int32_t iters, int32_t mix,
                                void *stream) {
    if (!operands || !sink || blocks < 1 || iters < 1 || iters > (1 << 20) || mix < 0 || mix > 3) return 1;
    if (launch_calib_mfma(operands, sink, blocks, iters, mix, (hipStream_t)stream) != hipSuccess) {
        (void)hipGetLastError();
        return 7;
    }
    return 0;
}

int32_t skv_calib_mfma_bf16(const void *operands, float *sink, int32_t blocks, int32_t iters, void *stream) {
    return skv_calib_mfma_mix_bf16(operands, sink, blocks, iters, 0, stream);
}

} // extern "C"
