// Cache update of the inference loop (paper Alg. 2, "Update K_l, V_l" for layers in S; Sec. 3.1.1:
// new K/V rows are appended to the existing cache).  A pure copy: bits are never reinterpreted.
#include "skv_internal.h"

namespace skv {

// One thread moves 16 bytes.  grid.x covers (sequence, new row, 16-byte piece), grid.y = {K, V}.
__global__ __launch_bounds__(256) void append_rows_kernel(SlotView c, const uint4 *__restrict__ k_new,
                                                           const uint4 *__restrict__ v_new,
                                                           const int32_t *__restrict__ start_pos,
                                                           const int32_t *__restrict__ new_lens,
                                                           int batch, int max_new, int pieces_per_row) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)batch * max_new * pieces_per_row;
    if (t >= total) return;
    const int piece = (int)(t % pieces_per_row);
    const int64_t row = t / pieces_per_row;
    const int i = (int)(row % max_new);
    const int b = (int)(row / max_new);
    if (i >= new_lens[b]) return;
    const int64_t pos = (int64_t)start_pos[b] + i;
    if (pos < 0 || pos >= c.max_ctx) {
        if (piece == 0) atomicOr(c.faults, (uint32_t)SKV_FAULT_APPEND_RANGE);
        return;
    }
    const int64_t dst_row = slot_row(c, b, (int)pos);
    if (dst_row < 0) {
        if (piece == 0) atomicOr(c.faults, (uint32_t)SKV_FAULT_BLOCK_ID);
        return;
    }
    const uint4 *src = blockIdx.y == 0 ? k_new : v_new;
    uint4 *dst = (uint4 *)(blockIdx.y == 0 ? c.k : c.v);
    dst[dst_row * pieces_per_row + piece] = src[t];
}

hipError_t launch_append(const SlotView &slot, int dtype, const void *k_new, const void *v_new,
                         const int32_t *start_pos, const int32_t *new_lens, int batch, int max_new,
                         hipStream_t stream) {
    const int row_bytes = slot.n_kv_heads * slot.head_dim * (dtype == SKV_F32 ? 4 : 2);
    const int pieces = row_bytes / 16; // head_dim is a multiple of 64, so rows are whole 16-byte pieces
    const int64_t total = (int64_t)batch * max_new * pieces;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    append_rows_kernel<<<dim3((unsigned)blocks, 2), 256, 0, stream>>>(
        slot, (const uint4 *)k_new, (const uint4 *)v_new, start_pos, new_lens, batch, max_new, pieces);
    return hipGetLastError();
}

} // namespace skv
