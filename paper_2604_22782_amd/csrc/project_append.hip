// Owner-layer K/V projection fused with the cache update (paper Sec. 4.3: the leader layer of a
// sharing group computes and stores K, V, the other layers skip their K/V projections; Alg. 2:
// "Update K_l, V_l" only for layers in S).  K = X W_k^T, V = X W_v^T on the matrix cores, an
// optional rotation of K by position, one rounding to the cache dtype, and the rows go straight
// into the slot: the projected K, V never exist as a tensor in HBM.
//
// Work group = 8 waves = 256 tokens x the head_dim features of ONE kv head of K or of V.  The
// product is formed transposed, out^T[feature][token] = W . X^T (v_mfma_f32_32x32x16: A = 32
// weight rows, B = 32 token rows, both read row-wise from LDS tiles of 64 hidden elements), so that
// a lane ends up owning one token and, over its registers, a quarter of that token's features of
// the head, its partner lane (l ^ 32) the others: the rotary pairs (i, i + d/2) sit in the same
// lane, and a token's row is written by two lanes.
#include "skv_internal.h"

namespace skv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct JBF16 {
    using vec8 = bf16x8;
    __device__ static f32x16 mfma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    __device__ static uint32_t pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        bf16x2 v = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
};
struct JF16 {
    using vec8 = f16x8;
    __device__ static f32x16 mfma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    __device__ static uint32_t pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
        f16x2 v = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
};

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kTokens = 32 * kWaves; // tokens per work group
constexpr int kKT = 64;              // hidden elements per staged tile
constexpr int kStride = kKT * 2 + 16; // LDS row stride: 16 consecutive rows x 16 bytes hit 16 bank groups

template <typename M, int D>
__global__ __launch_bounds__(kThreads, 1) void project_append_kernel(ProjArgs a) {
    using vec8 = typename M::vec8;
    constexpr int NB = D / 32;                           // feature blocks of the head
    constexpr int NX = kTokens * (kKT / 8) / kThreads;   // x pieces per thread and tile (4)
    constexpr int NW = D * (kKT / 8) / kThreads;         // weight pieces per thread and tile (2 or 1)
    constexpr int kStage = (kTokens + D) * kStride;
    __shared__ __attribute__((aligned(16))) char lds[2 * kStage];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int c = lane & 31;
    const int hh = lane >> 5;
    const int hkv = a.slot.n_kv_heads;
    const bool is_v = (int)blockIdx.x >= hkv;
    const int head = blockIdx.x % hkv;
    const int64_t n_tok = (int64_t)a.batch * a.max_new;
    const int64_t tok0 = (int64_t)blockIdx.y * kTokens;

    const uint16_t *w = (const uint16_t *)(is_v ? a.w_v : a.w_k) + (int64_t)head * D * a.hidden;
    const uint16_t *x = (const uint16_t *)a.x;

    uint4 xr[NX], wr[NW];
    auto issue = [&](int kt) {
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int piece = tid + i * kThreads;
            const int64_t row = tok0 + piece / (kKT / 8);
            xr[i] = make_uint4(0, 0, 0, 0);
            if (row < n_tok) xr[i] = *(const uint4 *)(x + row * a.hidden + kt * kKT + (piece % (kKT / 8)) * 8);
        }
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int piece = tid + i * kThreads;
            wr[i] = *(const uint4 *)(w + (int64_t)(piece / (kKT / 8)) * a.hidden + kt * kKT + (piece % (kKT / 8)) * 8);
        }
    };
    auto park = [&](int stage) {
        char *xs = lds + stage * kStage;
        char *ws = xs + kTokens * kStride;
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int piece = tid + i * kThreads;
            *(uint4 *)(xs + (piece / (kKT / 8)) * kStride + (piece % (kKT / 8)) * 16) = xr[i];
        }
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int piece = tid + i * kThreads;
            *(uint4 *)(ws + (piece / (kKT / 8)) * kStride + (piece % (kKT / 8)) * 16) = wr[i];
        }
    };

    f32x16 acc[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

    const int n_kt = a.hidden / kKT;
    issue(0);
    park(0);
    if (n_kt > 1) issue(1);
    __syncthreads();
    for (int kt = 0; kt < n_kt; ++kt) {
        const char *xs = lds + (kt & 1) * kStage + (32 * wave + c) * kStride + hh * 16;
        const char *ws = lds + (kt & 1) * kStage + kTokens * kStride + c * kStride + hh * 16;
#pragma unroll
        for (int st = 0; st < kKT / 16; ++st) {
            const vec8 b = __builtin_bit_cast(vec8, *(const uint4 *)(xs + st * 32));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[nb] = M::mfma(__builtin_bit_cast(vec8, *(const uint4 *)(ws + nb * 32 * kStride + st * 32)), b, acc[nb]);
        }
        if (kt + 1 < n_kt) park((kt + 1) & 1);
        __syncthreads();
        if (kt + 2 < n_kt) issue(kt + 2);
    }

    // lane owns token tok0 + 32 wave + c; element r of block nb is feature 32 nb + 8 (r/4) + 4 hh + r%4
    const int64_t m = tok0 + 32 * wave + c;
    if (m >= n_tok) return;
    const int b = (int)(m / a.max_new);
    const int i = (int)(m - (int64_t)b * a.max_new);
    if (i >= a.new_lens[b]) return;
    const int64_t pos = (int64_t)a.start_pos[b] + i;
    const bool rotate = !is_v && a.rope_cos != nullptr;
    if (pos < 0 || pos >= a.slot.max_ctx || (rotate && pos >= a.rope_positions)) {
        if (hh == 0) atomicOr(a.slot.faults, (uint32_t)SKV_FAULT_APPEND_RANGE);
        return;
    }
    const int64_t dst_row = slot_row(a.slot, b, (int)pos);
    if (dst_row < 0) {
        if (hh == 0) atomicOr(a.slot.faults, (uint32_t)SKV_FAULT_BLOCK_ID);
        return;
    }
    if (rotate) { // feature f < d/2 pairs with f + d/2: blocks nb and nb + NB/2, same element
        const float *ct = a.rope_cos + pos * (D / 2) + 4 * hh;
        const float *st = a.rope_sin + pos * (D / 2) + 4 * hh;
#pragma unroll
        for (int nb = 0; nb < NB / 2; ++nb)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const float4 cv = *(const float4 *)(ct + 32 * nb + 8 * g4);
                const float4 sv = *(const float4 *)(st + 32 * nb + 8 * g4);
                const float cc[4] = {cv.x, cv.y, cv.z, cv.w}, ss[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float lo = acc[nb][4 * g4 + j], hi = acc[nb + NB / 2][4 * g4 + j];
                    acc[nb][4 * g4 + j] = lo * cc[j] - hi * ss[j];
                    acc[nb + NB / 2][4 * g4 + j] = hi * cc[j] + lo * ss[j];
                }
            }
    }
    uint16_t *dst = (uint16_t *)(is_v ? a.slot.v : a.slot.k) + (dst_row * hkv + head) * D + 4 * hh;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
            *(uint2 *)(dst + 32 * nb + 8 * g4) = make_uint2(M::pack2(acc[nb][4 * g4], acc[nb][4 * g4 + 1]),
                                                            M::pack2(acc[nb][4 * g4 + 2], acc[nb][4 * g4 + 3]));
}

template <typename M, int D> hipError_t launch_j(const ProjArgs &a, hipStream_t stream) {
    const int64_t n_tok = (int64_t)a.batch * a.max_new;
    const int64_t tiles = (n_tok + kTokens - 1) / kTokens;
    if (tiles > 65535 || 2 * a.slot.n_kv_heads > 65535) return hipErrorInvalidValue;
    project_append_kernel<M, D><<<dim3((unsigned)(2 * a.slot.n_kv_heads), (unsigned)tiles), kThreads, 0, stream>>>(a);
    return hipGetLastError();
}

} // namespace

bool project_append_supported(int dtype, int head_dim, int hidden) {
    return (dtype == SKV_BF16 || dtype == SKV_F16) && (head_dim == 64 || head_dim == 128) && hidden >= kKT &&
           hidden % kKT == 0;
}

hipError_t launch_project_append(const ProjArgs &a, int dtype, int head_dim, hipStream_t stream) {
    if (dtype == SKV_BF16)
        return head_dim == 128 ? launch_j<JBF16, 128>(a, stream) : launch_j<JBF16, 64>(a, stream);
    return head_dim == 128 ? launch_j<JF16, 128>(a, stream) : launch_j<JF16, 64>(a, stream);
}

} // namespace skv
