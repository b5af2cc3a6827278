// Cache update of the inference loop (paper Alg. 2, "Update K_l, V_l" for layers in S; Sec. 3.1.1:
// new K/V rows are appended to the existing cache).  A pure copy: bits are never reinterpreted.
#include "skv_internal.h"

namespace skv {

// Work group = 4 waves x 64 lanes; wave y of block x moves rows 16 x + y, 16 x + y + 4, ... (16 rows
// per block), its lanes the 16-byte pieces of a row.  grid.y = {K, V}.  Row bookkeeping (sequence,
// length check, block-table lookup) is done once per row in 32-bit arithmetic; up to eight 16-byte
// loads per lane are in flight.
constexpr int kRowsPerBlock = 16;

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
        if (lane < pieces_per_row) buf[k][0] = s[lane];
        if (lane + 64 < pieces_per_row) buf[k][1] = s[lane + 64];
    }
#pragma unroll
    for (int k = 0; k < kRowsPerBlock / 4; ++k) {
        if (dst_off[k] < 0) continue;
        uint4 *d = dst + dst_off[k];
        if (lane < pieces_per_row) d[lane] = buf[k][0];
        if (lane + 64 < pieces_per_row) d[lane + 64] = buf[k][1];
        // rows wider than 2 KiB: the remaining pieces, two at a time
        const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.y + 4 * k;
        const uint4 *s = src + row * pieces_per_row;
        for (int p = lane + 128; p < pieces_per_row; p += 64) d[p] = s[p];
    }
}

hipError_t launch_append(const SlotView &slot, int dtype, const void *k_new, const void *v_new,
                         const int32_t *start_pos, const int32_t *new_lens, int batch, int max_new,
                         hipStream_t stream) {
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
