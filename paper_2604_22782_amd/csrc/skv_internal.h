// Internal declarations shared by the translation units of libskv (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "skv.h"

namespace skv {

// Where the rows of one cache slot live.  Passed by value to every kernel.
struct SlotView {
    const void *k;              // base of the slot inside the K pool
    const void *v;              // base of the slot inside the V pool
    const uint16_t *scales;     // 8-bit slots only: per (row, kv head) the scale exponent bytes of K (low) and V (high)
    const int32_t *block_table; // nullptr = contiguous
    uint32_t *faults;           // device fault word of the cache
    int32_t max_blocks_per_seq; // paged
    int32_t block_shift;        // paged: log2(block_size)
    int32_t n_blocks;           // paged
    int32_t max_ctx;            // contiguous: positions per sequence; paged: max_blocks_per_seq << block_shift
    int32_t seq_rows;           // contiguous: rows the slot holds per sequence (max_ctx, rounded up to whole groups)
    int32_t group_shift;        // 8-bit slots: log2 of the rows of one kv head that lie together (0: row-major slot)
    int32_t n_kv_heads;
    int32_t head_dim;
};

// Row number (in units of one [n_kv_heads][head_dim] row) of logical (b, pos) inside the slot,
// or -1 if a paged lookup hits a block id outside the pool.  pos must be < max_ctx.
__device__ __forceinline__ int64_t slot_row(const SlotView &c, int b, int pos) {
    if (c.block_table == nullptr) return (int64_t)b * c.seq_rows + pos;
    const int blk = c.block_table[(int64_t)b * c.max_blocks_per_seq + (pos >> c.block_shift)];
    if ((unsigned)blk >= (unsigned)c.n_blocks) return -1;
    return ((int64_t)blk << c.block_shift) + (pos & ((1 << c.block_shift) - 1));
}

// 8-bit slots are head-major inside groups of R = 1 << group_shift consecutive rows (a group never
// straddles a sequence or a block): the head_dim codes of (row, kv head) start at element
// kv8_head_row(c, row, kvh) * head_dim of the slot, and the pair of exponent bytes is scale word
// kv8_head_row(c, row, kvh).  A reader of one kv head then streams R * head_dim contiguous bytes
// per group instead of head_dim bytes per row: strided 128-byte pieces cost 12-15 % of the HBM rate.
__device__ __forceinline__ int64_t kv8_head_row(const SlotView &c, int64_t row, int kvh) {
    const int gs = c.group_shift;
    return ((((row >> gs) * c.n_kv_heads) + kvh) << gs) + (row & ((1 << gs) - 1));
}

// Descriptor dtypes 3 and 4: 16-bit activations over slots of 8-bit codes with power-of-two scales.
__host__ __device__ constexpr bool dtype_kv8(int dtype) { return dtype == SKV_BF16_KV8 || dtype == SKV_F16_KV8; }
// dtype of q / out / new rows
__host__ __device__ constexpr int dtype_act(int dtype) {
    return dtype == SKV_BF16_KV8 ? SKV_BF16 : dtype == SKV_F16_KV8 ? SKV_F16 : dtype;
}

// fp32 value 2^(byte - 127) of a scale exponent byte (byte 0, the clamp of absurdly small rows, reads
// as the exponent field of a zero; the conversion instructions take the exponent field only).
__device__ __forceinline__ float scale_of_byte(uint32_t byte) { return __builtin_bit_cast(float, byte << 23); }

// One 16-byte piece of 16 e4m3 codes -> the 16 values code x 2^e in the 16-bit type, as two pieces.
template <bool BF16>
__device__ __forceinline__ void dequant_piece(uint4 codes, float scale, uint4 &lo, uint4 &hi) {
    const uint32_t w[4] = {codes.x, codes.y, codes.z, codes.w};
    uint32_t o[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (BF16) {
            o[2 * i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[i], scale, false));
            o[2 * i + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[i], scale, true));
        } else {
            o[2 * i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[i], scale, false));
            o[2 * i + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[i], scale, true));
        }
    }
    lo = make_uint4(o[0], o[1], o[2], o[3]);
    hi = make_uint4(o[4], o[5], o[6], o[7]);
}

struct AttnArgs {
    SlotView cache;
    const void *q;          // [rows][n_q_heads][head_dim]
    void *out;              // same
    const int32_t *q_lens;  // nullptr for decode (one row per sequence)
    const int32_t *kv_lens; // [batch]
    const int32_t *evict_sink;  // decode only, both or neither: positions [evict_sink[b], evict_first[b]) of
    const int32_t *evict_first; //   sequence b were evicted and are never read
    float *part_o;          // split partials [rows*n_q_heads][n_splits][head_dim]
    float *part_ml;         // [rows*n_q_heads][n_splits][2]  (max, sum)
    int32_t *work_counters; // one device word (256-byte block): next work item of the persistent launch shape
    int32_t batch;
    int32_t max_q;          // query rows per sequence in q/out (1 for decode)
    int32_t n_q_heads;
    int32_t max_kv_len;     // host bound on kv_lens
    int32_t keys_per_split; // chunk of the key axis one work item covers
    int32_t n_splits;       // ceil(max_kv_len / keys_per_split)
    int32_t slot_readers;   // layers routed to the slot being read (decode: picks the cache policy of the loads)
    float scale_log2e;      // softmax scale * log2(e)
    float *lse;             // pre-fill only, may be nullptr: [batch][n_q_heads][max_q] log-sum-exp of the scaled scores
};

// Keys sequence b attends to in a decode call.  Without eviction: positions 0 .. kv_lens[b] - 1.
// With it the positions [sink, first) are gone; the kernels walk the survivors as one compact range
// of sink + (kv_lens[b] - first) keys, key c sitting at position c (c < sink) or c + gap with
// gap = first - sink.  sink is a multiple of the 32-key tile and first a multiple of the block
// size, so a tile never straddles the gap.  Returns -1 for values the host promised not to pass.
__device__ __forceinline__ int decode_keys(const AttnArgs &a, int b, int &sink, int &gap) {
    const int len = a.kv_lens[b];
    sink = 0;
    gap = 0;
    if (a.evict_first != nullptr) {
        const int s = a.evict_sink[b], f = a.evict_first[b];
        if (s < 0 || (s & 31) || f < s || f > len || ((f - s) & ((1 << a.cache.group_shift) - 1))) return -1;
        sink = s;
        gap = f - s;
    }
    const int m = len - gap;
    return (len >= 1 && m >= 1 && m <= a.max_kv_len && len <= a.cache.max_ctx) ? m : -1;
}

// Launchers (each returns the hipError_t of its launch).
hipError_t launch_append(const SlotView &slot, int dtype, const void *k_new, const void *v_new,
                         const int32_t *start_pos, const int32_t *new_lens, int batch, int max_new,
                         hipStream_t stream);

// Generic vector-ALU attention (any dtype; used for fp32 and for shapes the MFMA kernels do not cover).
hipError_t launch_attn_valu(const AttnArgs &a, int dtype, int head_dim, int group, hipStream_t stream);
hipError_t launch_split_merge(const AttnArgs &a, int dtype, hipStream_t stream);

// 16-bit MFMA kernels.
bool decode_mfma_supported(int dtype, int head_dim, int group);
hipError_t launch_decode_mfma(const AttnArgs &a, int dtype, int head_dim, int group, hipStream_t stream);
bool prefill_mfma_supported(int dtype, int head_dim, int group);
hipError_t launch_prefill_mfma(const AttnArgs &a, int dtype, int head_dim, int group, hipStream_t stream);

// Software-pipelined pre-fill kernel (16-bit, head_dim 128, contiguous caches below 4 GiB per sequence).
bool prefill_pipe_supported(const AttnArgs &a, int dtype, int head_dim);
hipError_t launch_prefill_pipe(const AttnArgs &a, int dtype, int group, hipStream_t stream);

// Owner-layer K/V projection fused with the append (16-bit, head_dim 64 or 128, hidden % 64 == 0).
struct ProjArgs {
    SlotView slot;
    const void *x, *w_k, *w_v;
    const float *rope_cos, *rope_sin; // both nullptr: no rotation
    const float *k_norm_weight;       // nullptr: K heads are not normalised; else head_dim weights
    float k_norm_eps;
    const int32_t *start_pos, *new_lens;
    float *partial;                   // fp32 partial sums when the hidden axis is split
    int32_t batch, max_new, hidden, rope_positions;
};
bool project_append_supported(int dtype, int head_dim, int hidden);
int project_append_splits(int n_kv_heads, int head_dim, int64_t n_tokens, int hidden);
size_t project_append_workspace_bytes(int n_kv_heads, int head_dim, int64_t n_tokens, int hidden);
hipError_t launch_project_append(const ProjArgs &a, int dtype, int head_dim, int n_splits, hipStream_t stream);

// Training backward (16-bit, head_dim 64 or 128).  delta: [batch][n_q_heads][seq] scratch.
struct TrainBwdArgs {
    const void *q, *k, *v, *out, *d_out;
    const float *lse;
    void *dq;
    float *dk_accum, *dv_accum, *delta;
    const int32_t *seq_lens;
    uint32_t *faults;
    int32_t batch, seq, n_q_heads, n_kv_heads;
    float scale;
};
hipError_t launch_train_bwd(const TrainBwdArgs &a, int dtype, int head_dim, hipStream_t stream);

void set_last_kernel_name(const char *name);

// Developer knobs (see tuning() in skv_api.hip); all zero / false unless SKV_TUNING=1 is set.
struct Tuning {
    int decode_keys_per_split = 0; // 0 = chosen by the library
    int decode_loads = 0;          // 0 = chosen by the library, 1 = non-temporal, 2 = cached
    bool prefill_plain = false;
    bool project_wide = false;
    int project_splits = 0;
};
const Tuning &tuning();

} // namespace skv
