// Cache update of the inference loop (paper Alg. 2, "Update K_l, V_l" for layers in S; Sec. 3.1.1:
// new K/V rows are appended to the existing cache).  A pure copy: bits are never reinterpreted.
#include "skv_internal.h"

namespace skv {

// Work group = 4 waves x 64 lanes; wave y of block x moves rows 8 x + y and 8 x + y + 4, its lanes
// the 16-byte pieces of a row.  grid.y = {K, V}.  Row bookkeeping (sequence, length check,
// block-table lookup) is done once per row in 32-bit arithmetic; all loads of a wave are issued
// before its first store.  Every byte is touched once: loads and stores carry the non-temporal
// hint.  Measured on a prompt-sized append (4 x 8192 rows of 2 KiB, K and V: 128 MiB read, 128 MiB
// written): 16 rows per block without the hint 52.7 us, with it 49.5; 32 rows 53.5 / 51.4; 8 rows
// with the hint 45.4 us = 5.9 TB/s.
constexpr int kRowsPerBlock = 8;

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ uint4 load_piece(const uint4 *p) {
    return __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4 *)p));
}
__device__ __forceinline__ void store_piece(uint4 *p, uint4 v) {
    __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), (u32x4 *)p);
}

__global__ __launch_bounds__(256) void append_rows_kernel(SlotView c, const uint4 *__restrict__ k_new,
                                                           const uint4 *__restrict__ v_new,
                                                           const int32_t *__restrict__ start_pos,
                                                           const int32_t *__restrict__ new_lens,
                                                           int batch, int max_new, int pieces_per_row) {
    const int lane = threadIdx.x;
    const uint4 *src = blockIdx.y == 0 ? k_new : v_new;
    uint4 *dst = (uint4 *)(blockIdx.y == 0 ? c.k : c.v);
    const int64_t n_rows = (int64_t)batch * max_new;
    uint4 buf[kRowsPerBlock / 4][2];
    int64_t dst_off[kRowsPerBlock / 4];
#pragma unroll
    for (int k = 0; k < kRowsPerBlock / 4; ++k) {
        dst_off[k] = -1;
        const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.y + 4 * k;
        if (row >= n_rows) continue;
        const int b = (int)((uint32_t)row / (uint32_t)max_new); // the host keeps the row count below 2^32
        const int i = (int)(row - (int64_t)b * max_new);
        if (i >= new_lens[b]) continue;
        const int64_t pos = (int64_t)start_pos[b] + i;
        if (pos < 0 || pos >= c.max_ctx) {
            if (lane == 0) atomicOr(c.faults, (uint32_t)SKV_FAULT_APPEND_RANGE);
            continue;
        }
        const int64_t dst_row = slot_row(c, b, (int)pos);
        if (dst_row < 0) {
            if (lane == 0) atomicOr(c.faults, (uint32_t)SKV_FAULT_BLOCK_ID);
            continue;
        }
        dst_off[k] = dst_row * pieces_per_row;
        const uint4 *s = src + row * pieces_per_row;
        if (lane < pieces_per_row) buf[k][0] = load_piece(s + lane);
        if (lane + 64 < pieces_per_row) buf[k][1] = load_piece(s + lane + 64);
    }
#pragma unroll
    for (int k = 0; k < kRowsPerBlock / 4; ++k) {
        if (dst_off[k] < 0) continue;
        uint4 *d = dst + dst_off[k];
        if (lane < pieces_per_row) store_piece(d + lane, buf[k][0]);
        if (lane + 64 < pieces_per_row) store_piece(d + lane + 64, buf[k][1]);
        // rows wider than 2 KiB: the remaining pieces, two at a time
        const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.y + 4 * k;
        const uint4 *s = src + row * pieces_per_row;
        for (int p = lane + 128; p < pieces_per_row; p += 64) store_piece(d + p, load_piece(s + p));
    }
}

// ---- 8-bit slots: the update converts every (row, kv head) piece of head_dim 16-bit values to
// head_dim e4m3 codes and one exponent byte (see the top of skv.h): e = smallest integer with
// max|x| 2^-e <= 448, code = x 2^-e rounded to nearest even.  The scaling by a power of two is
// exact, so the stored bytes have one correct value.
//
// D / 8 lanes share a piece (16 bytes = 8 values each); the same lanes handle K and V of the piece
// so that the two exponent bytes leave as one 16-bit store.
template <bool BF16, int D>
__global__ __launch_bounds__(256) void append_quant_kernel(SlotView c, const uint4 *__restrict__ k_new,
                                                           const uint4 *__restrict__ v_new,
                                                           const int32_t *__restrict__ start_pos,
                                                           const int32_t *__restrict__ new_lens, int batch,
                                                           int max_new) {
    constexpr int LPH = D / 8;           // lanes per (row, head) piece
    constexpr int PPB = 256 / LPH;       // pieces per block
    const int hkv = c.n_kv_heads;
    const int64_t piece = (int64_t)blockIdx.x * PPB + threadIdx.x / LPH;
    const int li = threadIdx.x % LPH;
    const int64_t n_rows = (int64_t)batch * max_new;
    const int64_t row = piece / hkv;
    const int head = (int)(piece - row * hkv);
    // (the LPH lanes of a piece take every branch below together: the shuffles stay inside them)
    if (row >= n_rows) return;
    const int b = (int)((uint32_t)row / (uint32_t)max_new);
    const int i = (int)(row - (int64_t)b * max_new);
    if (i >= new_lens[b]) return;
    const int64_t pos = (int64_t)start_pos[b] + i;
    if (pos < 0 || pos >= c.max_ctx) {
        if (li == 0 && head == 0) atomicOr(c.faults, (uint32_t)SKV_FAULT_APPEND_RANGE);
        return;
    }
    const int64_t dst_row = slot_row(c, b, (int)pos);
    if (dst_row < 0) {
        if (li == 0 && head == 0) atomicOr(c.faults, (uint32_t)SKV_FAULT_BLOCK_ID);
        return;
    }
    const int64_t src_piece = (row * hkv + head) * LPH + li;
    const int64_t dst_head_row = kv8_head_row(c, dst_row, head); // the slot is head-major inside groups of rows
    const int64_t dst_piece = dst_head_row * LPH + li;           // 8 codes = 8 bytes per lane
    uint32_t ebytes = 0;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        const uint4 raw = load_piece((which == 0 ? k_new : v_new) + src_piece);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
        float x[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (BF16) {
                x[2 * j] = __builtin_bit_cast(float, w[j] << 16);
                x[2 * j + 1] = __builtin_bit_cast(float, w[j] & 0xffff0000u);
            } else {
                typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
                const f16x2 h = __builtin_bit_cast(f16x2, w[j]);
                x[2 * j] = (float)h[0];
                x[2 * j + 1] = (float)h[1];
            }
        }
        float amax = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(x[j]));
#pragma unroll
        for (int d = 1; d < LPH; d <<= 1) amax = fmaxf(amax, __shfl_xor(amax, d, LPH));
        // amax = f 2^k with 0.5 <= f < 1, 448 = 0.875 x 2^9: e = k - 9 if f <= 0.875, else k - 8
        const uint32_t bits = __builtin_bit_cast(uint32_t, amax);
        const int k = (int)(bits >> 23) - 126;
        int e = (bits & 0x7fffffu) <= 0x600000u ? k - 9 : k - 8;
        e = amax == 0.f ? 0 : max(e, -127);
        uint32_t lo = 0, hi = 0;
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(ldexpf(x[0], -e), ldexpf(x[1], -e), lo, false);
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(ldexpf(x[2], -e), ldexpf(x[3], -e), lo, true);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(ldexpf(x[4], -e), ldexpf(x[5], -e), hi, false);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(ldexpf(x[6], -e), ldexpf(x[7], -e), hi, true);
        uint2 *dst = (uint2 *)(which == 0 ? c.k : c.v) + dst_piece;
        *dst = make_uint2(lo, hi);
        ebytes |= (uint32_t)(e + 127) << (8 * which);
    }
    if (li == 0) ((uint16_t *)c.scales)[dst_head_row] = (uint16_t)ebytes;
}

hipError_t launch_append(const SlotView &slot, int dtype, const void *k_new, const void *v_new,
                         const int32_t *start_pos, const int32_t *new_lens, int batch, int max_new,
                         hipStream_t stream) {
    if (dtype_kv8(dtype)) {
        const int64_t rows = (int64_t)batch * max_new;
        const int per_block = 256 / (slot.head_dim / 8);
        const int64_t blocks = (rows * slot.n_kv_heads + per_block - 1) / per_block;
        if (blocks > 0x7fffffff || rows > 0xffffffffll || slot.scales == nullptr) return hipErrorInvalidValue;
        const dim3 grid((unsigned)blocks);
        const uint4 *k4 = (const uint4 *)k_new, *v4 = (const uint4 *)v_new;
        const bool bf = dtype_act(dtype) == SKV_BF16;
        if (slot.head_dim == 128) {
            if (bf) append_quant_kernel<true, 128><<<grid, 256, 0, stream>>>(slot, k4, v4, start_pos, new_lens, batch, max_new);
            else append_quant_kernel<false, 128><<<grid, 256, 0, stream>>>(slot, k4, v4, start_pos, new_lens, batch, max_new);
        } else if (slot.head_dim == 64) {
            if (bf) append_quant_kernel<true, 64><<<grid, 256, 0, stream>>>(slot, k4, v4, start_pos, new_lens, batch, max_new);
            else append_quant_kernel<false, 64><<<grid, 256, 0, stream>>>(slot, k4, v4, start_pos, new_lens, batch, max_new);
        } else {
            return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    const int row_bytes = slot.n_kv_heads * slot.head_dim * (dtype == SKV_F32 ? 4 : 2);
    const int pieces = row_bytes / 16; // head_dim is a multiple of 64, so rows are whole 16-byte pieces
    const int64_t rows = (int64_t)batch * max_new;
    const int64_t blocks = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
    if (blocks > 0x7fffffff || rows > 0xffffffffll) return hipErrorInvalidValue;
    append_rows_kernel<<<dim3((unsigned)blocks, 2), dim3(64, 4), 0, stream>>>(
        slot, (const uint4 *)k_new, (const uint4 *)v_new, start_pos, new_lens, batch, max_new, pieces);
    return hipGetLastError();
}

} // namespace skv
