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

#include <cstdlib>

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

// Rotation, rounding and the store of one lane's share of a token row: acc[nb][r] is feature
// 32 nb + 8 (r/4) + 4 hh + r%4 of head `head` of K (or V) for the token at row m of x.
template <typename M, int D>
__device__ __forceinline__ void finish_token(const ProjArgs &a, f32x16 (&acc)[D / 32], int64_t m, int head, bool is_v,
                                             int hh) {
    constexpr int NB = D / 32;
    const int hkv = a.slot.n_kv_heads;
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
    if (!is_v && a.k_norm_weight != nullptr) { // the lane and its partner (l ^ 32) hold the head's d features of the token
        float ss = 0.f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) ss += acc[nb][r] * acc[nb][r];
        ss += __shfl_xor(ss, 32, 64);
        const float inv = rsqrtf(ss * (1.f / D) + a.k_norm_eps);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const float4 wv = *(const float4 *)(a.k_norm_weight + 32 * nb + 8 * g4 + 4 * hh);
                acc[nb][4 * g4] *= inv * wv.x;
                acc[nb][4 * g4 + 1] *= inv * wv.y;
                acc[nb][4 * g4 + 2] *= inv * wv.z;
                acc[nb][4 * g4 + 3] *= inv * wv.w;
            }
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

// grid = (2 n_kv_heads, token tiles, splits of the hidden axis).  With one split the work group
// finishes its rows itself; with more (few tokens: the launch would not fill the chip, and the
// weights have to stream from HBM at full rate) it stores its fp32 partial sums,
// partial[split][token][K or V][head][feature], and finish_kernel adds them up.
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

    // Loads run kDepth tiles ahead of the MFMAs, in a ring of register sets (one tile of MFMAs is far
    // shorter than a trip to HBM); the LDS stage of a tile is filled one tile ahead.
    constexpr int kDepth = 4;
    struct Slot {
        uint4 x[NX], w[NW];
    };
    Slot s0, s1, s2, s3;
    auto issue = [&](int kt, Slot &q) {
        uint4 *xq = q.x, *wq = q.w;
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int piece = tid + i * kThreads;
            const int64_t row = tok0 + piece / (kKT / 8);
            xq[i] = make_uint4(0, 0, 0, 0);
            if (row < n_tok) xq[i] = *(const uint4 *)(x + row * a.hidden + kt * kKT + (piece % (kKT / 8)) * 8);
        }
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int piece = tid + i * kThreads;
            wq[i] = *(const uint4 *)(w + (int64_t)(piece / (kKT / 8)) * a.hidden + kt * kKT + (piece % (kKT / 8)) * 8);
        }
    };
    auto park = [&](int stage, const Slot &q) {
        const uint4 *xq = q.x, *wq = q.w;
        char *xs = lds + stage * kStage;
        char *ws = xs + kTokens * kStride;
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int piece = tid + i * kThreads;
            *(uint4 *)(xs + (piece / (kKT / 8)) * kStride + (piece % (kKT / 8)) * 16) = xq[i];
        }
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int piece = tid + i * kThreads;
            *(uint4 *)(ws + (piece / (kKT / 8)) * kStride + (piece % (kKT / 8)) * 16) = wq[i];
        }
    };

    f32x16 acc[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

    const int n_kt = a.hidden / kKT / (int)gridDim.z;   // tiles of this split
    const int kt0 = (int)blockIdx.z * n_kt;
    static_assert(kDepth == 4, "the ring is spelled out below");
    issue(kt0, s0);
    if (1 < n_kt) issue(kt0 + 1, s1);
    if (2 < n_kt) issue(kt0 + 2, s2);
    if (3 < n_kt) issue(kt0 + 3, s3);
    park(0, s0);
    __syncthreads();
    auto step = [&](int kt, Slot &mine, const Slot &next) {
        const char *xs = lds + (kt & 1) * kStage + (32 * wave + c) * kStride + hh * 16;
        const char *ws = lds + (kt & 1) * kStage + kTokens * kStride + c * kStride + hh * 16;
#pragma unroll
        for (int st = 0; st < kKT / 16; ++st) {
            const vec8 b = __builtin_bit_cast(vec8, *(const uint4 *)(xs + st * 32));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[nb] = M::mfma(__builtin_bit_cast(vec8, *(const uint4 *)(ws + nb * 32 * kStride + st * 32)), b, acc[nb]);
        }
        if (kt + 1 < n_kt) park((kt + 1) & 1, next);         // the next tile's registers landed long ago
        __syncthreads();
        if (kt + kDepth < n_kt) issue(kt0 + kt + kDepth, mine); // this tile's registers are free again
    };
    for (int base = 0; base < n_kt; base += kDepth) { // ring slots named explicitly: fixed registers
        step(base, s0, s1);
        if (base + 1 < n_kt) step(base + 1, s1, s2);
        if (base + 2 < n_kt) step(base + 2, s2, s3);
        if (base + 3 < n_kt) step(base + 3, s3, s0);
    }

    // lane owns token tok0 + 32 wave + c; element r of block nb is feature 32 nb + 8 (r/4) + 4 hh + r%4
    const int64_t m = tok0 + 32 * wave + c;
    if (m >= n_tok) return;
    if (gridDim.z == 1) {
        finish_token<M, D>(a, acc, m, head, is_v, hh);
        return;
    }
    float *part = a.partial + (((int64_t)blockIdx.z * n_tok + m) * 2 * hkv + blockIdx.x) * D + 4 * hh;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
            *(float4 *)(part + 32 * nb + 8 * g4) =
                make_float4(acc[nb][4 * g4], acc[nb][4 * g4 + 1], acc[nb][4 * g4 + 2], acc[nb][4 * g4 + 3]);
}

// The prompt-sized launch (one split): work group = 256 tokens x TWO heads (2 d features), wave =
// 64 tokens x one head, so that a weight operand read from LDS feeds two MFMAs and a token tile is
// staged once per two heads: 0.75 LDS operand reads per MFMA instead of 1.25.
template <typename M, int D>
__global__ __launch_bounds__(kThreads, 1) void project_append_wide_kernel(ProjArgs a) {
    using vec8 = typename M::vec8;
    constexpr int NB = D / 32;
    constexpr int kF = 2 * D;                            // features per work group
    constexpr int NX = kTokens * (kKT / 8) / kThreads;   // x pieces per thread and tile
    constexpr int NW = kF * (kKT / 8) / kThreads;        // weight pieces per thread and tile
    constexpr int kStage = (kTokens + kF) * kStride;
    __shared__ __attribute__((aligned(16))) char lds[2 * kStage];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int tg = wave & 3, hs = wave >> 2;             // token group of 64, head of the pair
    const int c = lane & 31;
    const int hh = lane >> 5;
    const int hkv = a.slot.n_kv_heads;
    const int64_t n_tok = (int64_t)a.batch * a.max_new;
    const int64_t tok0 = (int64_t)blockIdx.y * kTokens;
    const uint16_t *x = (const uint16_t *)a.x;
    // feature row f of the work group: head 2 blockIdx.x + f / D of the list [K heads, V heads]
    auto weight_row = [&](int f) {
        const int kh = 2 * (int)blockIdx.x + f / D;
        return (const uint16_t *)(kh >= hkv ? a.w_v : a.w_k) + ((int64_t)(kh % hkv) * D + f % D) * a.hidden;
    };

    struct Slot {
        uint4 x[NX], w[NW];
    };
    Slot s0, s1; // two tiles in flight: with 128 accumulator registers a third does not fit
    auto issue = [&](int kt, Slot &q) {
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int piece = tid + i * kThreads;
            const int64_t row = tok0 + piece / (kKT / 8);
            q.x[i] = make_uint4(0, 0, 0, 0);
            if (row < n_tok) q.x[i] = *(const uint4 *)(x + row * a.hidden + kt * kKT + (piece % (kKT / 8)) * 8);
        }
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int piece = tid + i * kThreads;
            q.w[i] = *(const uint4 *)(weight_row(piece / (kKT / 8)) + kt * kKT + (piece % (kKT / 8)) * 8);
        }
    };
    auto park = [&](int stage, const Slot &q) {
        char *xs = lds + stage * kStage;
        char *ws = xs + kTokens * kStride;
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int piece = tid + i * kThreads;
            *(uint4 *)(xs + (piece / (kKT / 8)) * kStride + (piece % (kKT / 8)) * 16) = q.x[i];
        }
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int piece = tid + i * kThreads;
            *(uint4 *)(ws + (piece / (kKT / 8)) * kStride + (piece % (kKT / 8)) * 16) = q.w[i];
        }
    };

    f32x16 acc[2][NB];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][i][r] = 0.f;

    const int n_kt = a.hidden / kKT;
    issue(0, s0);
    if (1 < n_kt) issue(1, s1);
    park(0, s0);
    __syncthreads();
    auto step = [&](int kt, Slot &mine, const Slot &next) {
        const char *xs = lds + (kt & 1) * kStage + (64 * tg + c) * kStride + hh * 16;
        const char *ws = lds + (kt & 1) * kStage + kTokens * kStride + (hs * D + c) * kStride + hh * 16;
#pragma unroll
        for (int st = 0; st < kKT / 16; ++st) {
            const vec8 b0 = __builtin_bit_cast(vec8, *(const uint4 *)(xs + st * 32));
            const vec8 b1 = __builtin_bit_cast(vec8, *(const uint4 *)(xs + 32 * kStride + st * 32));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const vec8 wa = __builtin_bit_cast(vec8, *(const uint4 *)(ws + nb * 32 * kStride + st * 32));
                acc[0][nb] = M::mfma(wa, b0, acc[0][nb]);
                acc[1][nb] = M::mfma(wa, b1, acc[1][nb]);
            }
            if (st & 1) __builtin_amdgcn_sched_barrier(0); // two steps' operands in flight, not four
        }
        if (kt + 1 < n_kt) park((kt + 1) & 1, next);
        __syncthreads();
        if (kt + 2 < n_kt) issue(kt + 2, mine);
    };
    for (int base = 0; base < n_kt; base += 2) { // ring slots named explicitly: fixed registers
        step(base, s0, s1);
        if (base + 1 < n_kt) step(base + 1, s1, s0);
    }

    const int kh = 2 * (int)blockIdx.x + hs;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int64_t m = tok0 + 64 * tg + 32 * t + c;
        if (m < n_tok) finish_token<M, D>(a, acc[t], m, kh % hkv, kh >= hkv, hh);
    }
}

// The prompt-sized launch for shapes whose [K heads, V heads] list divides into tiles of 256 features:
// work group = 4 waves (one per SIMD) = 256 tokens x 256 features, wave = 128 x 128 (16 accumulator
// blocks: an operand read from LDS feeds four MFMAs, 0.5 reads per MFMA).  The hidden axis moves
// in slots of 64 elements through all 160 KiB of LDS: three slots of token rows, two of weight rows;
// the rows go from memory straight into LDS (buffer loads with the lds bit: no staging registers,
// no LDS store instructions).
// A load instruction fills 1 KiB = 8 rows x 128 bytes (whole cache lines: with 64-byte row pieces
// the L2 saw twice the requests and delivered a third less); inside it lane L = 8 g + s writes 16
// bytes at 16 L and fetches row g, piece s ^ (r / 2) with r = the row's index among its 16: eight
// neighbouring lanes fetch the 128 contiguous bytes of one row (one access of the vector cache;
// with a row per lane the loads ran at a lane per clock), and the exclusive-or puts the 16 rows of
// one piece into 16 different bank groups for the 128-bit operand reads (no bank conflicts).
// The barrier at the start of slot t publishes it (each wave has waited for its own loads) and
// releases slot t - 1; during slot t the weight rows of slot t + 1 and then the token rows of slot
// t + 2 are requested, one load after every four MFMAs; the MFMAs of the last step of slot t - 1
// run after the barrier, over the first operand reads of slot t.
// grid = (token tiles x feature tiles, splits of the hidden axis).  With one split the work group
// finishes its rows itself (normalisation, rotation, rounding, store into the slot); with more
// (prompts too short to give every compute unit a tile) it stores fp32 partial sums like the
// one-head kernel, and project_finish_kernel completes them.
constexpr int kGT = 256;                    // tokens = features per work group
constexpr int kSub = 64;                    // hidden elements per ring slot
constexpr int kRingX = 3, kRingW = 2;       // slots of token rows, slots of weight rows
constexpr int kHalfSlot = kGT * kSub * 2;   // bytes of the token rows (or of the weight rows) of a slot
// s_waitcnt operands that wait for the vector memory counter alone (bits 3:0 and 15:14; the other counters at their maxima)
constexpr int kVmcnt0 = 0x0f70;

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ uint32_t uni(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }

// Raw buffer descriptor: 48-bit base, stride 0, byte count, 32-bit untyped data.
__device__ __forceinline__ u32x4 make_srd(const void *base, uint32_t bytes) {
    const uint64_t p = (uint64_t)base;
    u32x4 r;
    r[0] = uni((uint32_t)p);
    r[1] = uni((uint32_t)(p >> 32) & 0xffffu);
    r[2] = uni(bytes);
    r[3] = 0x00020000u;
    return r;
}

// 64 lanes x 16 bytes from srd + voff + soff to LDS bytes lds_dst + 16 lane.  Written as an
// instruction of its own, not through the compiler's builtin: the compiler would wait for ALL
// outstanding loads of this kind before any later LDS read, and the ring lives on loads that stay
// in flight across two barriers.  The kernel counts them itself (s_waitcnt vmcnt).
// (M0, which carries the LDS address, is named as clobbered; the compiler notes that it does not
// save it, and this kernel has no other use of it.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_chunk_to_lds(u32x4 srd, uint32_t lds_dst, int voff, int soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_dst), "v"(voff), "s"(srd), "s"(soff)
                 : "memory", "m0");
}
#pragma clang diagnostic pop

template <typename M, int D>
__global__ __launch_bounds__(256, 1) void project_append_tile_kernel(ProjArgs a) {
    using vec8 = typename M::vec8;
    constexpr int NB = D / 32;
    constexpr int HW = 128 / D;                          // heads per wave
    __shared__ __attribute__((aligned(1024))) char lds[(kRingX + kRingW) * kHalfSlot]; // all 160 KiB

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tg = wave & 1, fg = wave >> 1;             // token half, feature half of the work group's tile
    const int c = lane & 31;
    const int hh = lane >> 5;
    const int hkv = a.slot.n_kv_heads;
    const int64_t n_tok = (int64_t)a.batch * a.max_new;
    // work groups that share a token tile run on one XCD (ids are dealt to the 8 XCDs in turn)
    const int n_ft = 2 * hkv * D / kGT;
    const int64_t id = blockIdx.x, n_tt = gridDim.x / n_ft;
    const bool by_xcd = n_tt % 8 == 0;
    const int ft = (int)((by_xcd ? id >> 3 : id) % n_ft);
    const int64_t tt = by_xcd ? ((id >> 3) / n_ft) * 8 + (id & 7) : id / n_ft;
    const int64_t tok0 = tt * kGT;

    // the 64 weight rows this wave stages: features 64 wave .. + 63 of the tile, inside one head
    const int kh_w = (ft * kGT + 64 * wave) / D;
    const uint16_t *w_rows = (const uint16_t *)(kh_w >= hkv ? a.w_v : a.w_k) +
                             ((int64_t)(kh_w % hkv) * D + (ft * kGT + 64 * wave) % D) * a.hidden;
    const int64_t rows_left = n_tok - tok0 - 64 * wave;  // token rows this wave stages: 64 wave .. + 63 of the tile
    const uint32_t x_bytes = rows_left <= 0 ? 0u : (uint32_t)((rows_left < 64 ? rows_left : 64) * a.hidden * 2);
    const u32x4 x_srd = make_srd((const uint16_t *)a.x + (rows_left > 0 ? (tok0 + 64 * wave) * a.hidden : 0), x_bytes);
    const u32x4 w_srd = make_srd(w_rows, 64u * a.hidden * 2u);
    const uint32_t lds_base = uni((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds);
    // even chunks of a slot hold rows 0..7 of a group of 16, odd chunks rows 8..15 (r / 2 = 4 + g / 2)
    const int voff = ((lane >> 3) * a.hidden + ((lane & 7) ^ (lane >> 4)) * 8) * 2;
    const int row8 = 8 * a.hidden * 2;                   // bytes between the first rows of two chunks
    const int n_sub = a.hidden / kSub / (int)gridDim.y;  // slots of this split of the hidden axis
    const int sub0 = (int)blockIdx.y * n_sub;
    // chunk c (of 8) of the wave's token rows / weight rows of slot `sub`
    auto request_x = [&](int sub, int c) {
        load_chunk_to_lds(x_srd, lds_base + (sub % kRingX) * kHalfSlot + (8 * wave + c) * 1024, voff ^ ((c & 1) * 64),
                          uni(c * row8 + (sub0 + sub) * kSub * 2));
    };
    auto request_w = [&](int sub, int c) {
        load_chunk_to_lds(w_srd, lds_base + (kRingX + (sub & 1)) * kHalfSlot + (8 * wave + c) * 1024,
                          voff ^ ((c & 1) * 64), uni(c * row8 + (sub0 + sub) * kSub * 2));
    };

    f32x16 acc[4][4]; // [token block][feature block of the wave]
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][i][r] = 0.f;

    // operand address of row c of a 32-row block, k-step 0 of a slot; k-step j is the same address ^ 32 j
    const int rd0 = 128 * c + 16 * (hh ^ ((c >> 1) & 7));
    const int x_rd = 16 * tg * 1024 + rd0, w_rd = kRingX * kHalfSlot + 16 * fg * 1024 + rd0;
    uint4 xa[4], wa[4], xb[4], wb[4];
    // Operands of k-step `step` of slot `sub`, one block at a time: parts 0..3 = token blocks (all
    // four are needed by the first MFMAs of the step), parts 4..7 = weight blocks.
    auto fetch_part = [&](int sub, int step, int part, uint4 (&xo)[4], uint4 (&wo)[4]) {
        const char *xs = lds + (sub % kRingX) * kHalfSlot, *ws = lds + (sub & 1) * kHalfSlot;
        const int flip = step * 32;
        if (part < 4) xo[part] = *(const uint4 *)(xs + ((x_rd ^ flip) + part * 4096));
        else wo[part - 4] = *(const uint4 *)(ws + ((w_rd ^ flip) + (part - 4) * 4096));
    };
    // 16 MFMAs; after every two of them `between(j)`, j = 0..7, reads one block of the next step's
    // operands and, on odd j, may send a load out.  All loads of a slot at once would hold the wave
    // at the memory pipeline (16 cycles per load, four waves) while the matrix cores idle: measured,
    // the two phases simply added up; operand reads in a burst of eight cost 2.5 % against two at a time.
    auto multiply = [&](const uint4 (&xo)[4], const uint4 (&wo)[4], auto between) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                acc[t][i] = M::mfma(__builtin_bit_cast(vec8, wo[i]), __builtin_bit_cast(vec8, xo[t]), acc[t][i]);
                if (t & 1) {
                    between(2 * i + (t >> 1));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };
    auto nothing = [](int) {};

#pragma unroll
    for (int c = 0; c < 8; ++c) request_x(0, c);
#pragma unroll
    for (int c = 0; c < 8; ++c) request_w(0, c);
    if (1 < n_sub) {
#pragma unroll
        for (int c = 0; c < 8; ++c) request_x(1, c);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) xb[i] = wb[i] = make_uint4(0, 0, 0, 0); // the first turn multiplies zeros
    for (int sub = 0; sub < n_sub; ++sub) {
        // own loads of this slot; the eight token loads of the next slot, issued after them, may still fly
        if (sub + 1 < n_sub) __builtin_amdgcn_s_waitcnt(kVmcnt0 | 8);
        else __builtin_amdgcn_s_waitcnt(kVmcnt0);
        __syncthreads();
        const bool more_w = sub + 1 < n_sub, more_x = sub + 2 < n_sub;
        multiply(xb, wb, [&](int j) { // last step of the slot before; step 0 of this slot is read meanwhile
            fetch_part(sub, 0, j, xa, wa);
            if (more_w && (j & 1)) request_w(sub + 1, j >> 1);
        });
        multiply(xa, wa, [&](int j) {
            fetch_part(sub, 1, j, xb, wb);
            if (more_w && (j & 1)) request_w(sub + 1, 4 + (j >> 1));
        });
        multiply(xb, wb, [&](int j) {
            fetch_part(sub, 2, j, xa, wa);
            if (more_x && (j & 1)) request_x(sub + 2, j >> 1);
        });
        multiply(xa, wa, [&](int j) {
            fetch_part(sub, 3, j, xb, wb);
            if (more_x && (j & 1)) request_x(sub + 2, 4 + (j >> 1));
        });
    }
    multiply(xb, wb, nothing);

#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int64_t m = tok0 + 128 * tg + 32 * t + c;
#pragma unroll
        for (int h = 0; h < HW; ++h) {
            const int kh = (ft * kGT + 128 * fg) / D + h;
            f32x16(&part)[NB] = *(f32x16(*)[NB]) & acc[t][h * NB];
            if (m >= n_tok) continue;
            if (gridDim.y == 1) {
                finish_token<M, D>(a, part, m, kh % hkv, kh >= hkv, hh);
                continue;
            }
            // a split of the hidden axis: fp32 partial sums, partial[split][token][K or V head][feature]
            float *dst = a.partial + (((int64_t)blockIdx.y * n_tok + m) * 2 * hkv + kh) * D + 4 * hh;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4)
                    *(float4 *)(dst + 32 * nb + 8 * g4) =
                        make_float4(part[nb][4 * g4], part[nb][4 * g4 + 1], part[nb][4 * g4 + 2], part[nb][4 * g4 + 3]);
        }
    }
}

// Few token rows (one decode token per sequence: at most 64 rows, where the launch is a stream of
// the weights and nothing else).  Every wave is a work group of its own: wave (fb, s) forms the 32
// features of feature block fb of the [K heads, V heads] list for all token rows (two blocks of 32)
// over the hidden columns of split s.  No LDS and no barrier: both MFMA operands come straight from
// memory in operand layout -- lane (c, hh) owns row c (a weight row / a token row) and, of every 64
// columns, the 32 contiguous ones 32 hh .. 32 hh + 31 (the order of the contraction is free as long
// as both operands use it), i.e. 64 contiguous bytes per row and tile, two lanes per 128-byte line.
// Loads run three tiles ahead in a register ring.  The fp32 partial sums of a split go to the
// workspace in the layout project_finish_kernel reads.  Four splits at hidden 4096 and 8 kv heads of
// 128 (256 waves, one per compute unit): 4 MiB of partial traffic beside the 17 MiB of weights and
// rows, where the one-head kernel above needed sixteen splits (16 MiB) to fill the chip.
constexpr int kSmallTokens = 64;
template <typename M, int D>
__global__ __launch_bounds__(64) void project_small_kernel(ProjArgs a, int n_splits) {
    using vec8 = typename M::vec8;
    constexpr int NB = D / 32;
    const int lane = threadIdx.x, c = lane & 31, hh = lane >> 5;
    const int hkv = a.slot.n_kv_heads;
    const int kh = (int)blockIdx.x / NB, nb = (int)blockIdx.x % NB; // head in the [K, V] list, feature block of it
    const bool is_v = kh >= hkv;
    const int head = is_v ? kh - hkv : kh;
    const int n_tok = a.batch * a.max_new;                           // <= kSmallTokens (checked by the launcher)
    const int cols = a.hidden / n_splits;
    const int64_t col0 = (int64_t)blockIdx.y * cols + 32 * hh;
    const uint16_t *w = (const uint16_t *)(is_v ? a.w_v : a.w_k) + ((int64_t)head * D + 32 * nb + c) * a.hidden + col0;
    // token rows past the last one repeat it (their results are not stored)
    const uint16_t *x0 = (const uint16_t *)a.x + (int64_t)min(c, n_tok - 1) * a.hidden + col0;
    const uint16_t *x1 = (const uint16_t *)a.x + (int64_t)min(32 + c, n_tok - 1) * a.hidden + col0;
    const bool two = n_tok > 32;

    struct Slot {
        uint4 w[4], x0[4], x1[4];
    };
    auto issue = [&](int kt, Slot &q) {
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            q.w[st] = *(const uint4 *)(w + kt * 64 + 8 * st);
            q.x0[st] = *(const uint4 *)(x0 + kt * 64 + 8 * st);
            if (two) q.x1[st] = *(const uint4 *)(x1 + kt * 64 + 8 * st);
        }
    };
    f32x16 acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc0[r] = acc1[r] = 0.f;
    auto compute = [&](const Slot &q) {
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            const vec8 wa = __builtin_bit_cast(vec8, q.w[st]);
            acc0 = M::mfma(wa, __builtin_bit_cast(vec8, q.x0[st]), acc0);
            if (two) acc1 = M::mfma(wa, __builtin_bit_cast(vec8, q.x1[st]), acc1);
        }
    };
    const int n_kt = cols / 64;
    Slot s0, s1, s2;
#pragma unroll
    for (int st = 0; st < 4; ++st) s0.x1[st] = s1.x1[st] = s2.x1[st] = make_uint4(0, 0, 0, 0);
    issue(0, s0);
    if (1 < n_kt) issue(1, s1);
    if (2 < n_kt) issue(2, s2);
    for (int base = 0; base < n_kt; base += 3) { // ring slots named explicitly: fixed registers
        compute(s0);
        if (base + 3 < n_kt) issue(base + 3, s0);
        if (base + 1 < n_kt) {
            compute(s1);
            if (base + 4 < n_kt) issue(base + 4, s1);
        }
        if (base + 2 < n_kt) {
            compute(s2);
            if (base + 5 < n_kt) issue(base + 5, s2);
        }
    }
    // lane owns token c (acc0) and 32 + c (acc1); element r is feature 32 nb + 8 (r/4) + 4 hh + r%4 of the head
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const int m = 32 * tb + c;
        if (m >= n_tok) continue;
        const f32x16 &acc = tb == 0 ? acc0 : acc1;
        float *part = a.partial + (((int64_t)blockIdx.y * n_tok + m) * 2 * hkv + kh) * D + 32 * nb + 4 * hh;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
            *(float4 *)(part + 8 * g4) = make_float4(acc[4 * g4], acc[4 * g4 + 1], acc[4 * g4 + 2], acc[4 * g4 + 3]);
    }
}


// Adds up the partial sums of the splits.  One thread per (token, K or V head, half hh, feature
// block nb < NB/2, group g4): the four features 32 nb + 8 g4 + 4 hh .. + 3 of the head and their
// rotary partners d/2 further on, i.e. what finish_token needs together.
template <typename M, int D>
__global__ __launch_bounds__(256) void project_finish_kernel(ProjArgs a, int n_splits) {
    constexpr int NB = D / 32;
    const int hkv = a.slot.n_kv_heads;
    const int64_t n_tok = (int64_t)a.batch * a.max_new;
    int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int g4 = (int)(t & 3);
    t >>= 2;
    const int nb = (int)(t % (NB / 2));
    t /= NB / 2;
    const int hh = (int)(t & 1);
    t >>= 1;
    const int kh = (int)(t % (2 * hkv));
    const int64_t m = t / (2 * hkv);
    if (m >= n_tok) return;
    const int f_lo = 32 * nb + 8 * g4 + 4 * hh, f_hi = f_lo + D / 2;
    float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
    const float *part0 = a.partial + (m * 2 * hkv + kh) * D;
    const int64_t split_stride = n_tok * 2 * hkv * D;
    int s = 0;
    for (; s + 4 <= n_splits; s += 4) { // eight loads in flight (the split counts are powers of two); summed in split order
        float4 u[4], v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            u[j] = *(const float4 *)(part0 + (s + j) * split_stride + f_lo);
            v[j] = *(const float4 *)(part0 + (s + j) * split_stride + f_hi);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            lo.x += u[j].x; lo.y += u[j].y; lo.z += u[j].z; lo.w += u[j].w;
            hi.x += v[j].x; hi.y += v[j].y; hi.z += v[j].z; hi.w += v[j].w;
        }
    }
    for (; s < n_splits; ++s) {
        const float4 u = *(const float4 *)(part0 + s * split_stride + f_lo), v = *(const float4 *)(part0 + s * split_stride + f_hi);
        lo.x += u.x; lo.y += u.y; lo.z += u.z; lo.w += u.w;
        hi.x += v.x; hi.y += v.y; hi.z += v.z; hi.w += v.w;
    }
    const int head = kh % hkv;
    const bool is_v = kh >= hkv;
    if (!is_v && a.k_norm_weight != nullptr) {
        // the 4 (D / 64) 2 threads of this (token, head) are neighbours in the wave and hold its d features
        float ss = lo.x * lo.x + lo.y * lo.y + lo.z * lo.z + lo.w * lo.w + hi.x * hi.x + hi.y * hi.y + hi.z * hi.z + hi.w * hi.w;
#pragma unroll
        for (int d = 1; d < 4 * (NB / 2) * 2; d <<= 1) ss += __shfl_xor(ss, d, 64);
        const float inv = rsqrtf(ss * (1.f / D) + a.k_norm_eps);
        const float4 wl = *(const float4 *)(a.k_norm_weight + f_lo), wh = *(const float4 *)(a.k_norm_weight + f_hi);
        lo = make_float4(lo.x * inv * wl.x, lo.y * inv * wl.y, lo.z * inv * wl.z, lo.w * inv * wl.w);
        hi = make_float4(hi.x * inv * wh.x, hi.y * inv * wh.y, hi.z * inv * wh.z, hi.w * inv * wh.w);
    }
    const int b = (int)(m / a.max_new);
    const int i = (int)(m - (int64_t)b * a.max_new);
    if (i >= a.new_lens[b]) return;
    const int64_t pos = (int64_t)a.start_pos[b] + i;
    const bool rotate = !is_v && a.rope_cos != nullptr;
    const bool first = hh == 0 && nb == 0 && g4 == 0;
    if (pos < 0 || pos >= a.slot.max_ctx || (rotate && pos >= a.rope_positions)) {
        if (first) atomicOr(a.slot.faults, (uint32_t)SKV_FAULT_APPEND_RANGE);
        return;
    }
    const int64_t dst_row = slot_row(a.slot, b, (int)pos);
    if (dst_row < 0) {
        if (first) atomicOr(a.slot.faults, (uint32_t)SKV_FAULT_BLOCK_ID);
        return;
    }
    if (rotate) {
        const float4 cv = *(const float4 *)(a.rope_cos + pos * (D / 2) + f_lo);
        const float4 sv = *(const float4 *)(a.rope_sin + pos * (D / 2) + f_lo);
        const float4 l = lo, h = hi;
        lo = make_float4(l.x * cv.x - h.x * sv.x, l.y * cv.y - h.y * sv.y, l.z * cv.z - h.z * sv.z, l.w * cv.w - h.w * sv.w);
        hi = make_float4(h.x * cv.x + l.x * sv.x, h.y * cv.y + l.y * sv.y, h.z * cv.z + l.z * sv.z, h.w * cv.w + l.w * sv.w);
    }
    uint16_t *dst = (uint16_t *)(is_v ? a.slot.v : a.slot.k) + (dst_row * hkv + head) * D;
    *(uint2 *)(dst + f_lo) = make_uint2(M::pack2(lo.x, lo.y), M::pack2(lo.z, lo.w));
    *(uint2 *)(dst + f_hi) = make_uint2(M::pack2(hi.x, hi.y), M::pack2(hi.z, hi.w));
}

// The tile kernel takes the launches whose (head, 256-token tile) grid the one-head kernel would
// run unsplit, on shapes whose [K heads, V heads] list divides into tiles of 256 features.
// The few-rows kernel takes launches of at most 64 token rows (it always leaves fp32 partial sums
// for project_finish_kernel, also with a single split).
bool small_kernel_takes(int64_t n_tokens, int hidden) {
    return n_tokens >= 1 && n_tokens <= kSmallTokens && hidden % 64 == 0 && !tuning().project_wide;
}

bool tile_kernel_takes(int n_kv_heads, int head_dim, int64_t n_tokens, int hidden) {
    const int64_t tiles = (n_tokens + kTokens - 1) / kTokens;
    return 2 * (int64_t)n_kv_heads * tiles >= 128 && (2 * n_kv_heads * head_dim) % kGT == 0 && hidden % kSub == 0 &&
           hidden <= (1 << 20) && !tuning().project_wide;
}

template <typename M, int D> hipError_t launch_j(const ProjArgs &a, int n_splits, hipStream_t stream) {
    const int64_t n_tok = (int64_t)a.batch * a.max_new;
    const int64_t tiles = (n_tok + kTokens - 1) / kTokens;
    if (tiles > 65535 || 2 * a.slot.n_kv_heads > 65535) return hipErrorInvalidValue;
    hipError_t e = hipSuccess;
    if (small_kernel_takes(n_tok, a.hidden)) {
        const dim3 grid((unsigned)(2 * a.slot.n_kv_heads * (D / 32)), (unsigned)n_splits);
        project_small_kernel<M, D><<<grid, 64, 0, stream>>>(a, n_splits);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        const int64_t threads = n_tok * 2 * a.slot.n_kv_heads * 2 * (D / 64) * 4;
        project_finish_kernel<M, D><<<dim3((unsigned)((threads + 255) / 256)), 256, 0, stream>>>(a, n_splits);
        return hipGetLastError();
    }
    if (tile_kernel_takes(a.slot.n_kv_heads, D, n_tok, a.hidden)) {
        const int64_t groups = ((n_tok + kGT - 1) / kGT) * (2 * a.slot.n_kv_heads * D / kGT);
        if (groups > 0x7fffffff) return hipErrorInvalidValue;
        project_append_tile_kernel<M, D><<<dim3((unsigned)groups, (unsigned)n_splits), 256, 0, stream>>>(a);
        e = hipGetLastError();
    } else if (n_splits == 1) {
        project_append_wide_kernel<M, D><<<dim3((unsigned)a.slot.n_kv_heads, (unsigned)tiles), kThreads, 0, stream>>>(a);
        return hipGetLastError();
    } else {
        const dim3 grid((unsigned)(2 * a.slot.n_kv_heads), (unsigned)tiles, (unsigned)n_splits);
        project_append_kernel<M, D><<<grid, kThreads, 0, stream>>>(a);
        e = hipGetLastError();
    }
    if (e != hipSuccess || n_splits == 1) return e;
    const int64_t threads = n_tok * 2 * a.slot.n_kv_heads * 2 * (D / 64) * 4;
    project_finish_kernel<M, D><<<dim3((unsigned)((threads + 255) / 256)), 256, 0, stream>>>(a, n_splits);
    return hipGetLastError();
}

} // namespace

bool project_append_supported(int dtype, int head_dim, int hidden) {
    return (dtype == SKV_BF16 || dtype == SKV_F16) && (head_dim == 64 || head_dim == 128) && hidden >= kKT &&
           hidden % kKT == 0;
}

// Splits of the hidden axis.  Tile kernel (prompts): one while its 256 x 256 tiles alone give
// about a work group per compute unit (8192 tokens at 8 kv heads of 128); below that as many as get
// there, each at least 512 wide -- a prompt of 2048 tokens would otherwise occupy a quarter of the
// chip.  One-head kernel (few tokens): as many as bring the launch to about one work group per
// compute unit, each at least 128 wide.
int project_append_splits(int n_kv_heads, int head_dim, int64_t n_tokens, int hidden) {
    const int want = tuning().project_splits; // developer knob: a power of two that divides the tiles of the hidden axis
    if (want >= 1 && (want & (want - 1)) == 0 && hidden / kKT % want == 0) return want;
    int splits = 1;
    if (small_kernel_takes(n_tokens, hidden)) { // one wave per (32 features, split): about one per compute unit, splits at least 256 wide
        const int64_t waves = 2 * (int64_t)n_kv_heads * (head_dim / 32);
        while (waves * splits < 256 && hidden / 64 % (2 * splits) == 0 && hidden / (2 * splits) >= 256) splits *= 2;
        return splits;
    }
    if (tile_kernel_takes(n_kv_heads, head_dim, n_tokens, hidden)) {
        const int64_t groups = ((n_tokens + kGT - 1) / kGT) * (2 * n_kv_heads * head_dim / kGT);
        while (groups * splits < 192 && hidden / kSub % (2 * splits) == 0 && hidden / (2 * splits) >= 512) splits *= 2;
        return splits;
    }
    const int64_t tiles = (n_tokens + kTokens - 1) / kTokens;
    const int64_t groups = 2 * (int64_t)n_kv_heads * tiles;
    if (groups >= 128) return 1;
    while (groups * splits < 256 && hidden / kKT % (2 * splits) == 0 && hidden / (2 * splits) >= 128) splits *= 2;
    return splits;
}

size_t project_append_workspace_bytes(int n_kv_heads, int head_dim, int64_t n_tokens, int hidden) {
    const int splits = project_append_splits(n_kv_heads, head_dim, n_tokens, hidden);
    if (small_kernel_takes(n_tokens, hidden)) // partial sums also with a single split
        return (size_t)splits * (size_t)n_tokens * 2 * n_kv_heads * head_dim * sizeof(float);
    return splits == 1 ? 0 : (size_t)splits * (size_t)n_tokens * 2 * n_kv_heads * head_dim * sizeof(float);
}

hipError_t launch_project_append(const ProjArgs &a, int dtype, int head_dim, int n_splits, hipStream_t stream) {
    if (dtype == SKV_BF16)
        return head_dim == 128 ? launch_j<JBF16, 128>(a, n_splits, stream) : launch_j<JBF16, 64>(a, n_splits, stream);
    return head_dim == 128 ? launch_j<JF16, 128>(a, n_splits, stream) : launch_j<JF16, 64>(a, n_splits, stream);
}

} // namespace skv
