// Gradient of the training-time routed attention (paper Sec. 3.2: layer l attends to the K, V of a
// sampled layer l' <= l; Eq. (3.1) over whole sequences with a causal mask).  With P = softmax(S),
// S = scale Q K^T and delta_i = <dO_i, O_i>:
//     dV = P^T dO,   dP = dO V^T,   dS = P o (dP - delta),   dQ = scale dS K,   dK = scale dS^T Q.
// P is recomputed from the forward's log-sum-exp, tile by tile, on the matrix cores
// (v_mfma_f32_32x32x16); nothing of size seq x seq is ever stored.  Three launches, no atomics:
//   delta_kernel   one float per (row, head);
//   dkdv_kernel    a wave owns 32 keys of one kv head (K^T, V^T and the dK^T, dV^T accumulators
//                  stay in its registers) and walks over the query heads of the group and the
//                  query rows at or below its keys; the owner ADDS its result to the fp32 buffers
//                  of the source layer, which several reader layers share;
//   dq_kernel      a wave owns 32 query rows (Q^T, dO^T, dQ^T in registers) and walks over the
//                  keys at or before them, like the forward.
// Tiles of the streamed operand (Q and dO rows, or K and V rows) are staged in LDS twice where both
// a row-wise (A operand of S / dP) and a transposed (A operand of the d x row products, through
// ds_read_b64_tr_b16) view is needed, each with the row stride that keeps its reads conflict-free.
// As in the forward, the order of the contraction index inside a 16-wide MFMA step is permuted so
// that exponentiated accumulators, rounded to 16 bits, are directly the next product's B operand.
#include <type_traits>

#include "skv_internal.h"

namespace skv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

struct TBF16 {
    using vec8 = bf16x8;
    __device__ static f32x16 mfma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    __device__ static uint32_t pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        bf16x2 v = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
    __device__ static float widen(uint16_t x) { return __builtin_bit_cast(float, (uint32_t)x << 16); }
};
struct TF16 {
    using vec8 = f16x8;
    __device__ static f32x16 mfma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    __device__ static uint32_t pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
        f16x2 v = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
    __device__ static float widen(uint16_t x) { return (float)__builtin_bit_cast(_Float16, x); }
};

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kTile = 64;            // rows of the streamed operand per LDS stage
constexpr int kOwned = 32 * kWaves;  // rows (dq) / keys (dk, dv) a work group owns
constexpr float kLog2e = 1.4426950408889634f;

template <int D> struct Geo {
    static constexpr int LPR = D / 8;                 // 16-byte pieces per row
    static constexpr int NL = kTile * LPR / kThreads; // loads per thread, tile and tensor
    static constexpr int R_STRIDE = D * 2 + 16;       // row-wise view: 16 rows x 16 bytes hit 16 bank groups
    static constexpr int T_STRIDE = D * 2 + 64;       // transposed view: 4 rows x 64 bytes hit all banks
    static constexpr int R_BYTES = kTile * R_STRIDE;
    static constexpr int T_BYTES = kTile * T_STRIDE;
    static_assert(NL >= 1, "tile too small for the work group");
};

__device__ __forceinline__ s16x4 lds_read_tr16(const char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(p));
}

// A operand (32 x 16, rows = the feature index d of block db, contraction = rows 16 x .. 16 x + 15
// of the staged tile in the permuted order of the packed accumulators) through transposing reads.
template <typename M, int T_STRIDE>
__device__ __forceinline__ typename M::vec8 read_transposed(const char *lane_base, int x, int db) {
    const char *p = lane_base + 16 * x * T_STRIDE + db * 64;
    const s16x4 lo = lds_read_tr16(p);
    const s16x4 hi = lds_read_tr16(p + 8 * T_STRIDE);
    const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(typename M::vec8, both);
}

// Elements 8 x .. 8 x + 7 of an accumulator block, rounded to 16 bits: B operand of step x.
template <typename M> __device__ __forceinline__ typename M::vec8 pack_step(const float *e) {
    const uint4 raw = make_uint4(M::pack2(e[0], e[1]), M::pack2(e[2], e[3]), M::pack2(e[4], e[5]), M::pack2(e[6], e[7]));
    return __builtin_bit_cast(typename M::vec8, raw);
}

// ---- delta_i = <dO_i, O_i> ---------------------------------------------------------------------
template <typename M, int D>
__global__ __launch_bounds__(256) void delta_kernel(TrainBwdArgs a) {
    constexpr int LPR = D / 8;
    const int64_t n_rh = (int64_t)a.batch * a.seq * a.n_q_heads;
    const int64_t rh = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPR; // (b, row, head) flattened as in out
    const int piece = threadIdx.x % LPR;
    float s = 0.f;
    int b = 0, row = 0, head = 0;
    bool ok = rh < n_rh;
    if (ok) {
        head = (int)(rh % a.n_q_heads);
        const int64_t br = rh / a.n_q_heads;
        row = (int)(br % a.seq);
        b = (int)(br / a.seq);
        ok = row < a.seq_lens[b];
    }
    if (ok) {
        const uint4 o = *(const uint4 *)((const uint16_t *)a.out + rh * D + piece * 8);
        const uint4 g = *(const uint4 *)((const uint16_t *)a.d_out + rh * D + piece * 8);
        const uint32_t ow[4] = {o.x, o.y, o.z, o.w}, gw[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s += M::widen((uint16_t)ow[i]) * M::widen((uint16_t)gw[i]);
            s += M::widen((uint16_t)(ow[i] >> 16)) * M::widen((uint16_t)(gw[i] >> 16));
        }
    }
#pragma unroll
    for (int d = 1; d < LPR; d <<= 1) s += __shfl_xor(s, d, 64);
    if (ok && piece == 0) a.delta[((int64_t)b * a.n_q_heads + head) * a.seq + row] = s;
}

// ---- dK, dV --------------------------------------------------------------------------------------
template <typename M, int D>
__global__ __launch_bounds__(kThreads, 1) void dkdv_kernel(TrainBwdArgs a, int n_kt) {
    using Ge = Geo<D>;
    using vec8 = typename M::vec8;
    constexpr int NL = Ge::NL, LPR = Ge::LPR;
    // per stage: Q row-wise, Q transposed view, dO row-wise, dO transposed view, lse (log2), delta
    constexpr int kStage = 2 * Ge::R_BYTES + 2 * Ge::T_BYTES + 2 * kTile * 4;
    __shared__ __attribute__((aligned(16))) char lds[2 * kStage];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int c = lane & 31;
    const int hh = lane >> 5;
    const int hkv = a.n_kv_heads, hq = a.n_q_heads;
    const int G = hq / hkv;

    // heavy key tiles (the first ones: every later row reads them) first, for the whole launch
    const int pairs = a.batch * hkv;
    const int kt = blockIdx.x / pairs;
    const int kvh = (blockIdx.x % pairs) % hkv;
    const int b = (blockIdx.x % pairs) / hkv;
    const int n = a.seq_lens[b];
    if (n < 1 || n > a.seq) {
        if (tid == 0 && kt == 0 && kvh == 0) atomicOr(a.faults, (uint32_t)SKV_FAULT_KV_LEN);
        return;
    }
    const int k0 = kt * kOwned;
    if (k0 >= n) return;
    const int kb0 = k0 + 32 * wave; // first key of this wave
    const int my_key = kb0 + c;

    // K^T, V^T as B operands: lane (key c, k-group hh), step s holds K[key][16 s + 8 hh .. + 8)
    vec8 kB[D / 16], vB[D / 16];
    {
        const int64_t off = (((int64_t)b * a.seq + my_key) * hkv + kvh) * D + 8 * hh;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            uint4 rk = make_uint4(0, 0, 0, 0), rv = rk;
            if (my_key < n) {
                rk = *(const uint4 *)((const uint16_t *)a.k + off + 16 * s);
                rv = *(const uint4 *)((const uint16_t *)a.v + off + 16 * s);
            }
            kB[s] = __builtin_bit_cast(vec8, rk);
            vB[s] = __builtin_bit_cast(vec8, rv);
        }
    }

    const int qt0 = k0 / kTile;                    // first row tile that sees keys of this work group
    const int n_qt = (n - 1) / kTile - qt0 + 1;    // row tiles per head
    const int n_it = G * n_qt;

    // staging: thread t moves pieces t, t + 256, ... of the Q and dO tiles; rows beyond n are zero
    uint4 qr[NL], gr[NL];
    float aux = 0.f; // threads 0..63: lse of row tid (in log2 units), 64..127: delta of row tid - 64
    auto issue = [&](int it) {
        const int head = kvh * G + it / n_qt;
        const int r_first = (qt0 + it % n_qt) * kTile;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int piece = tid + i * kThreads;
            const int row = r_first + piece / LPR;
            qr[i] = gr[i] = make_uint4(0, 0, 0, 0);
            if (row < n) {
                const int64_t off = (((int64_t)b * a.seq + row) * hq + head) * D + (piece % LPR) * 8;
                qr[i] = *(const uint4 *)((const uint16_t *)a.q + off);
                gr[i] = *(const uint4 *)((const uint16_t *)a.d_out + off);
            }
        }
        if (tid < 2 * kTile) {
            const int row = r_first + (tid & (kTile - 1));
            const int64_t off = ((int64_t)b * hq + head) * a.seq + row;
            if (tid < kTile)
                aux = row < n ? a.lse[off] * kLog2e : INFINITY; // +inf: the row's weights become 0
            else
                aux = row < n ? a.delta[off] : 0.f;
        }
    };
    auto park = [&](int stage) {
        char *qs = lds + stage * kStage;
        char *qt_ = qs + Ge::R_BYTES;
        char *gs = qt_ + Ge::T_BYTES;
        char *gt = gs + Ge::R_BYTES;
        float *ax = (float *)(gt + Ge::T_BYTES);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int piece = tid + i * kThreads;
            const int r = piece / LPR, p = (piece % LPR) * 16;
            *(uint4 *)(qs + r * Ge::R_STRIDE + p) = qr[i];
            *(uint4 *)(qt_ + r * Ge::T_STRIDE + p) = qr[i];
            *(uint4 *)(gs + r * Ge::R_STRIDE + p) = gr[i];
            *(uint4 *)(gt + r * Ge::T_STRIDE + p) = gr[i];
        }
        if (tid < 2 * kTile) ax[tid] = aux;
    };

    f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) dk[i][r] = dv[i][r] = 0.f;

    const float cs = a.scale * kLog2e;
    const int sl = lane & 15;
    const int t_lane_off = (4 * hh + (sl >> 2)) * Ge::T_STRIDE + ((lane >> 4) & 1) * 32 + (sl & 3) * 8;

    // one block of 32 rows against this wave's 32 keys
    auto compute_block = [&](const char *stage, int rb, int r0, auto masked) {
        const char *qs = stage;
        const char *qt_ = qs + Ge::R_BYTES;
        const char *gs = qt_ + Ge::T_BYTES;
        const char *gt = gs + Ge::R_BYTES;
        const float *ax = (const float *)(gt + Ge::T_BYTES);
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
        // S = Q K^T and dP = dO V^T: rows x keys, lane = key column, element r = row 8 (r/4) + 4 hh + r%4
        const char *qa = qs + (32 * rb + c) * Ge::R_STRIDE + hh * 16;
        const char *ga = gs + (32 * rb + c) * Ge::R_STRIDE + hh * 16;
#pragma unroll
        for (int st = 0; st < D / 16; ++st) {
            s = M::mfma(__builtin_bit_cast(vec8, *(const uint4 *)(qa + st * 32)), kB[st], s);
            dp = M::mfma(__builtin_bit_cast(vec8, *(const uint4 *)(ga + st * 32)), vB[st], dp);
        }
        float p[16], ds[16];
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const float4 l4 = *(const float4 *)(ax + 32 * rb + 8 * g4 + 4 * hh);
            const float4 d4 = *(const float4 *)(ax + kTile + 32 * rb + 8 * g4 + 4 * hh);
            const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = 4 * g4 + j;
                float w = __builtin_amdgcn_exp2f(fmaf(s[r], cs, -lv[j]));
                if constexpr (decltype(masked)::value) {
                    if (my_key > r0 + 8 * g4 + 4 * hh + j) w = 0.f; // the row does not see this key
                }
                p[r] = w;
                ds[r] = w * (dp[r] - dl[j]);
            }
        }
        // dV^T += dO^T P and dK^T += Q^T dS: feature x keys, contraction over the 32 rows
        const char *gtb = gt + 32 * rb * Ge::T_STRIDE + t_lane_off;
        const char *qtb = qt_ + 32 * rb * Ge::T_STRIDE + t_lane_off;
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const vec8 pB = pack_step<M>(p + 8 * x);
            const vec8 dsB = pack_step<M>(ds + 8 * x);
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                dv[db] = M::mfma(read_transposed<M, Ge::T_STRIDE>(gtb, x, db), pB, dv[db]);
                dk[db] = M::mfma(read_transposed<M, Ge::T_STRIDE>(qtb, x, db), dsB, dk[db]);
            }
        }
    };

    issue(0);
    park(0);
    if (n_it > 1) issue(1);
    __syncthreads();
    for (int it = 0; it < n_it; ++it) {
        const char *stage = lds + (it & 1) * kStage;
        const int r_first = (qt0 + it % n_qt) * kTile;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int r0 = r_first + 32 * rb;
            if (r0 + 31 < kb0 || r0 >= n || kb0 >= n) continue; // rows before the keys, or nothing valid
            if (r0 < kb0 + 31)
                compute_block(stage, rb, r0, std::true_type{});
            else
                compute_block(stage, rb, r0, std::false_type{});
        }
        if (it + 1 < n_it) park((it + 1) & 1);
        __syncthreads();
        if (it + 2 < n_it) issue(it + 2);
    }

    if (my_key >= n) return;
    // lane owns key my_key; element r of block db is feature 32 db + 8 (r/4) + 4 hh + r%4
    const int64_t off = (((int64_t)b * a.seq + my_key) * hkv + kvh) * D + 4 * hh;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            float4 *pk = (float4 *)(a.dk_accum + off + 32 * db + 8 * q4);
            float4 *pv = (float4 *)(a.dv_accum + off + 32 * db + 8 * q4);
            float4 ak = *pk, av = *pv;
            ak.x += a.scale * dk[db][4 * q4];
            ak.y += a.scale * dk[db][4 * q4 + 1];
            ak.z += a.scale * dk[db][4 * q4 + 2];
            ak.w += a.scale * dk[db][4 * q4 + 3];
            av.x += dv[db][4 * q4];
            av.y += dv[db][4 * q4 + 1];
            av.z += dv[db][4 * q4 + 2];
            av.w += dv[db][4 * q4 + 3];
            *pk = ak;
            *pv = av;
        }
}

// ---- dQ ------------------------------------------------------------------------------------------
// W waves of 32 rows per work group.  W = 8 keeps the wave below 256 registers (the 64 keys of a
// tile are processed as two blocks of 32), so two waves share a SIMD and cover each other's waits.
template <typename M, int D, int W>
__global__ __launch_bounds__(64 * W, 1) void dq_kernel(TrainBwdArgs a, int n_rt) {
    using Ge = Geo<D>;
    using vec8 = typename M::vec8;
    constexpr int LPR = Ge::LPR;
    constexpr int NT = 64 * W;                 // threads
    constexpr int NL = kTile * LPR / NT;       // loads per thread, tile and tensor
    static_assert(NL >= 1, "tile too small for the work group");
    constexpr int kRows = 32 * W;              // rows a work group owns
    // per stage: K row-wise, K transposed view, V row-wise
    constexpr int kStage = 2 * Ge::R_BYTES + Ge::T_BYTES;
    __shared__ __attribute__((aligned(16))) char lds[2 * kStage];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int c = lane & 31;
    const int hh = lane >> 5;
    const int hkv = a.n_kv_heads, hq = a.n_q_heads;
    const int G = hq / hkv;

    // heavy (late) row tiles first, for the whole launch; the heads of a group are neighbours
    const int pairs = a.batch * hq;
    const int rt = n_rt - 1 - blockIdx.x / pairs;
    const int head = (blockIdx.x % pairs) % hq;
    const int b = (blockIdx.x % pairs) / hq;
    const int kvh = head / G;
    const int n = a.seq_lens[b];
    if (n < 1 || n > a.seq) return; // reported by dkdv_kernel
    const int q_begin = rt * kRows;
    if (q_begin >= n) return;
    const int n_keys = min(q_begin + kRows, n); // keys the work group needs: 0 .. its last row
    const int n_tiles = (n_keys + kTile - 1) / kTile;

    const int r0 = q_begin + 32 * wave;
    const int my_row = r0 + c;
    const bool row_ok = my_row < n;
    const bool wave_ok = r0 < n;
    const int wave_last = min(r0 + 31, n - 1);

    // Q^T, dO^T as B operands: lane (row c, k-group hh), step s holds Q[row][16 s + 8 hh .. + 8)
    vec8 qB[D / 16], gB[D / 16];
    const int64_t row_off = (((int64_t)b * a.seq + my_row) * hq + head) * D;
    {
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            uint4 rq = make_uint4(0, 0, 0, 0), rg = rq;
            if (row_ok) {
                rq = *(const uint4 *)((const uint16_t *)a.q + row_off + 8 * hh + 16 * s);
                rg = *(const uint4 *)((const uint16_t *)a.d_out + row_off + 8 * hh + 16 * s);
            }
            qB[s] = __builtin_bit_cast(vec8, rq);
            gB[s] = __builtin_bit_cast(vec8, rg);
        }
    }
    float lse2 = INFINITY, delta = 0.f; // a row beyond the length gets weights 0
    if (row_ok) {
        const int64_t off = ((int64_t)b * hq + head) * a.seq + my_row;
        lse2 = a.lse[off] * kLog2e;
        delta = a.delta[off];
    }

    uint4 kr[NL], vr[NL];
    auto issue = [&](int t) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int piece = tid + i * NT;
            const int key = t * kTile + piece / LPR;
            kr[i] = vr[i] = make_uint4(0, 0, 0, 0);
            if (key < n_keys) {
                const int64_t off = (((int64_t)b * a.seq + key) * hkv + kvh) * D + (piece % LPR) * 8;
                kr[i] = *(const uint4 *)((const uint16_t *)a.k + off);
                vr[i] = *(const uint4 *)((const uint16_t *)a.v + off);
            }
        }
    };
    auto park = [&](int stage) {
        char *ks = lds + stage * kStage;
        char *ktv = ks + Ge::R_BYTES;
        char *vs = ktv + Ge::T_BYTES;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int piece = tid + i * NT;
            const int r = piece / LPR, p = (piece % LPR) * 16;
            *(uint4 *)(ks + r * Ge::R_STRIDE + p) = kr[i];
            *(uint4 *)(ktv + r * Ge::T_STRIDE + p) = kr[i];
            *(uint4 *)(vs + r * Ge::R_STRIDE + p) = vr[i];
        }
    };

    f32x16 dq[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[i][r] = 0.f;

    const float cs = a.scale * kLog2e;
    const int sl = lane & 15;
    const int t_lane_off = (4 * hh + (sl >> 2)) * Ge::T_STRIDE + ((lane >> 4) & 1) * 32 + (sl & 3) * 8;

    // one block of 32 keys (kb = 0, 1 of the staged tile) against this wave's 32 rows
    auto compute_block = [&](const char *stage, int j0, int kb, auto masked) {
        const char *ks = stage;
        const char *ktv = ks + Ge::R_BYTES;
        const char *vs = ktv + Ge::T_BYTES;
        // S^T = K Q^T and dP^T = V dO^T: keys x rows, lane = row column
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
        const char *ka = ks + (32 * kb + c) * Ge::R_STRIDE + hh * 16;
        const char *va = vs + (32 * kb + c) * Ge::R_STRIDE + hh * 16;
#pragma unroll
        for (int st = 0; st < D / 16; ++st) {
            s = M::mfma(__builtin_bit_cast(vec8, *(const uint4 *)(ka + st * 32)), qB[st], s);
            dp = M::mfma(__builtin_bit_cast(vec8, *(const uint4 *)(va + st * 32)), gB[st], dp);
        }
        // element r is key j0 + 32 kb + 8 (r/4) + 4 hh + r%4
        float ds[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float w = __builtin_amdgcn_exp2f(fmaf(s[r], cs, -lse2));
            if constexpr (decltype(masked)::value) {
                const int key = j0 + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
                if (key > my_row) w = 0.f;
            }
            ds[r] = w * (dp[r] - delta);
        }
        // dQ^T += K^T dS^T: feature x rows, contraction over the 32 keys
        const char *kt_ = ktv + 32 * kb * Ge::T_STRIDE + t_lane_off;
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const vec8 dsB = pack_step<M>(ds + 8 * x);
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
                dq[db] = M::mfma(read_transposed<M, Ge::T_STRIDE>(kt_, x, db), dsB, dq[db]);
        }
    };

    issue(0);
    park(0);
    if (n_tiles > 1) issue(1);
    __syncthreads();
    for (int t = 0; t < n_tiles; ++t) {
        const int j0 = t * kTile;
        const char *stage = lds + (t & 1) * kStage;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const int jb = j0 + 32 * kb;
            if (!wave_ok || jb > wave_last) continue;
            if (jb + 31 > r0)
                compute_block(stage, j0, kb, std::true_type{});
            else
                compute_block(stage, j0, kb, std::false_type{});
        }
        if (t + 1 < n_tiles) park((t + 1) & 1);
        __syncthreads();
        if (t + 2 < n_tiles) issue(t + 2);
    }

    if (!row_ok) return;
    // lane owns row my_row; element r of block db is feature 32 db + 8 (r/4) + 4 hh + r%4
    uint16_t *op = (uint16_t *)a.dq + row_off + 4 * hh;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const uint2 w = make_uint2(M::pack2(a.scale * dq[db][4 * q4], a.scale * dq[db][4 * q4 + 1]),
                                       M::pack2(a.scale * dq[db][4 * q4 + 2], a.scale * dq[db][4 * q4 + 3]));
            *(uint2 *)(op + 32 * db + 8 * q4) = w;
        }
}

constexpr int kDqWaves = 8;

template <typename M, int D> hipError_t launch_b(const TrainBwdArgs &a, hipStream_t stream) {
    const int64_t n_rh = (int64_t)a.batch * a.seq * a.n_q_heads;
    const int64_t delta_blocks = (n_rh * (D / 8) + 255) / 256;
    const int n_kt = (a.seq + kOwned - 1) / kOwned;
    const int64_t kv_blocks = (int64_t)a.batch * a.n_kv_heads * n_kt;
    const int n_rt = (a.seq + 32 * kDqWaves - 1) / (32 * kDqWaves);
    const int64_t q_blocks = (int64_t)a.batch * a.n_q_heads * n_rt;
    if (delta_blocks > 0x7fffffff || kv_blocks > 0x7fffffff || q_blocks > 0x7fffffff) return hipErrorInvalidValue;
    delta_kernel<M, D><<<dim3((unsigned)delta_blocks), 256, 0, stream>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dkdv_kernel<M, D><<<dim3((unsigned)kv_blocks), kThreads, 0, stream>>>(a, n_kt);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    dq_kernel<M, D, kDqWaves><<<dim3((unsigned)q_blocks), 64 * kDqWaves, 0, stream>>>(a, n_rt);
    set_last_kernel_name("dkdv_kernel");
    return hipGetLastError();
}

} // namespace

hipError_t launch_train_bwd(const TrainBwdArgs &a, int dtype, int head_dim, hipStream_t stream) {
    if (dtype == SKV_BF16)
        return head_dim == 128 ? launch_b<TBF16, 128>(a, stream) : launch_b<TBF16, 64>(a, stream);
    return head_dim == 128 ? launch_b<TF16, 128>(a, stream) : launch_b<TF16, 64>(a, stream);
}

} // namespace skv
