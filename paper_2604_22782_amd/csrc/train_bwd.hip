// Gradient of the training-time routed attention (paper Sec. 3.2: layer l attends to the K, V of a
// sampled layer l' <= l; Eq. (3.1) over whole sequences with a causal mask).  With P = softmax(S),
// S = scale Q K^T and delta_i = <dO_i, O_i>:
//     dV = P^T dO,   dP = dO V^T,   dS = P o (dP - delta),   dQ = scale dS K,   dK = scale dS^T Q.
// P is recomputed from the forward's log-sum-exp, tile by tile, on the matrix cores
// (v_mfma_f32_32x32x16); nothing of size seq x seq is ever stored.  Three launches, no atomics:
//   delta_kernel   one float per (row, head);
//   dkdv_kernel    a work group owns 128 keys of one kv head (their K, V rows stay in LDS, the
//                  dK^T, dV^T accumulators in registers) and walks over the query heads of the
//                  group and the query rows at or below its keys; it ADDS its result to the fp32
//                  buffers of the source layer, which several reader layers share;
//   dq_kernel      a wave owns 32 query rows (Q^T, dO^T, dQ^T in registers) and walks over the
//                  keys at or before them, like the forward.
// Both run 8 waves per work group, two per SIMD, below 256 registers per lane: the instruction
// order is the compiler's, and the second wave is what covers its waits.
// The streamed tiles (Q and dO rows, or K and V rows) are read from LDS both row-wise (A operand
// of S / dP) and transposed (A operand of the feature x row products, ds_read_b64_tr_b16).
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

constexpr int kTile = 64;            // rows of the streamed operand per LDS stage
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ s16x4 lds_read_tr16(const char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(p));
}

// LDS layout of every tile (resident K, V block, staged Q, dO, K, V tiles): chunks of 4 rows
// (4 x 2D bytes + 64 bytes of padding); inside a chunk the 16-byte piece p of row r sits at
// 64 p + 16 r.  Row-wise operand reads (16 lanes = 16 consecutive rows, one piece) and transposing
// reads (16 lanes = 4 rows x 32 bytes) both touch every bank exactly once, so one copy serves both.
template <int D> struct Chunked {
    static constexpr int CH = 8 * D + 64;
    static constexpr int BLOCK32 = 8 * CH;  // 32 rows
    static constexpr int TILE = 16 * CH;    // 64 rows
    __device__ static int piece(int r, int p) { return (r >> 2) * CH + 64 * p + 16 * (r & 3); }
    // Staging order: 16 consecutive threads take 4 rows x 4 consecutive pieces of a chunk.  Their
    // 16-byte LDS stores then fall into 16 different bank groups (pieces of one row lie 64 bytes
    // apart: a thread per piece of one row would hit every bank four times), and each quad of
    // threads still loads 64 contiguous bytes of one row from memory.  q-th piece -> (row, piece)
    __device__ static int staged_row(int q) { return 4 * (q / (4 * (D / 8))) + ((q & 15) >> 2); }
    __device__ static int staged_piece(int q) { return 4 * ((q % (4 * (D / 8))) >> 4) + (q & 3); }
    // lane part of a row-wise read of row c of a 32-row block: pieces 2 s + hh (+ 128 s per step)
    __device__ static int row_lane(int c, int hh) { return (c >> 2) * CH + 16 * (c & 3) + 64 * hh; }
    // lane part of a transposing read: rows 4 hh + sl / 4 of a 16-row step (+ 4 CH per step, + 2 CH
    // for its second half), 8 bytes at byte 32 a + 8 (sl % 4) of the 64-byte feature block (+ 256 per block)
    __device__ static int tr_lane(int lane) {
        const int sl = lane & 15, a = (lane >> 4) & 1, hh = lane >> 5;
        return hh * CH + 128 * a + 64 * ((sl & 3) >> 1) + 16 * (sl >> 2) + 8 * (sl & 1);
    }
};

template <typename M, int D>
__device__ __forceinline__ typename M::vec8 read_transposed_chunked(const char *lane_base, int x, int db) {
    using C = Chunked<D>;
    const char *p = lane_base + x * 4 * C::CH + db * 256;
    const s16x4 lo = lds_read_tr16(p);
    const s16x4 hi = lds_read_tr16(p + 2 * C::CH);
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
constexpr int kKvWaves = 8;             // 4 key blocks of 32 x the 2 row blocks of a 64-row tile
constexpr int kKvThreads = 64 * kKvWaves;
constexpr int kKvKeys = 128;            // keys a work group owns

// A work group owns 128 keys of one kv head; their K and V rows stay in LDS (B operands of S and
// dP).  Wave (kblk, rb) handles key block kblk against row block rb of every staged 64-row tile of
// Q and dO, so two waves per SIMD cover each other's waits; the two waves of a key block add their
// accumulators through LDS at the end.
template <typename M, int D>
__global__ __launch_bounds__(kKvThreads, 1) void dkdv_kernel(TrainBwdArgs a, int n_kt) {
    using C = Chunked<D>;
    using vec8 = typename M::vec8;
    constexpr int LPR = D / 8;
    constexpr int NL = kTile * LPR / kKvThreads;          // staged pieces per thread, tile and tensor
    constexpr int NKV = kKvKeys * LPR / kKvThreads;       // resident pieces per thread and tensor
    static_assert(NL >= 1 && NKV >= 1, "work group too large for the tile");
    constexpr int kResident = 2 * 4 * C::BLOCK32;         // K then V of the 128 keys
    constexpr int kStage = 2 * C::TILE + 2 * kTile * 4;   // Q, dO, lse (log2 units), delta
    constexpr int kReduce = 4 * (D / 32) * 16 * 64 * 4;   // one tensor's accumulators of four waves
    constexpr int kLds = kResident + 2 * kStage > kReduce ? kResident + 2 * kStage : kReduce;
    __shared__ __attribute__((aligned(16))) char lds[kLds];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int kblk = wave & 3, rb = wave >> 2;
    const int c = lane & 31;
    const int hh = lane >> 5;
    const int hkv = a.n_kv_heads, hq = a.n_q_heads;
    const int G = hq / hkv;

    // heavy key tiles (the first ones: every later row reads them) first, for the whole launch.
    // (Sending all key tiles of a (sequence, kv head) pair to one XCD, as dq_kernel does with its row
    // tiles, raises the HBM traffic here from 4.6 to 5.5-7.3 GiB per launch: the tiles of a pair run at
    // different rows of Q and dO, more of them than one L2 holds.)
    const int pairs = a.batch * hkv;
    const int kt = blockIdx.x / pairs;
    const int kvh = (blockIdx.x % pairs) % hkv;
    const int b = (blockIdx.x % pairs) / hkv;
    const int n = a.seq_lens[b];
    if (n < 1 || n > a.seq) {
        if (tid == 0 && kt == 0 && kvh == 0) atomicOr(a.faults, (uint32_t)SKV_FAULT_KV_LEN);
        return;
    }
    const int k0 = kt * kKvKeys;
    if (k0 >= n) return;
    const int kb0 = k0 + 32 * kblk; // first key of this wave
    const int my_key = kb0 + c;

    char *k_res = lds, *v_res = lds + 4 * C::BLOCK32;
    {   // resident K, V rows; keys beyond the length are zero
#pragma unroll
        for (int i = 0; i < NKV; ++i) {
            const int piece = tid + i * kKvThreads;
            const int r = C::staged_row(piece), p = C::staged_piece(piece);
            uint4 rk = make_uint4(0, 0, 0, 0), rv = rk;
            if (k0 + r < n) {
                const int64_t off = (((int64_t)b * a.seq + k0 + r) * hkv + kvh) * D + p * 8;
                rk = *(const uint4 *)((const uint16_t *)a.k + off);
                rv = *(const uint4 *)((const uint16_t *)a.v + off);
            }
            *(uint4 *)(k_res + C::piece(r, p)) = rk;
            *(uint4 *)(v_res + C::piece(r, p)) = rv;
        }
    }

    const int qt0 = k0 / kTile;                    // first row tile that sees keys of this work group
    const int n_qt = (n - 1) / kTile - qt0 + 1;    // row tiles per head
    const int n_it = G * n_qt;

    // staging: thread t moves pieces t, t + 512, ... of the Q and dO tiles; rows beyond n are zero
    uint4 qr[NL], gr[NL];
    float aux = 0.f; // threads 0..63: lse of row tid (in log2 units), 64..127: delta of row tid - 64
    auto issue = [&](int it) {
        const int head = kvh * G + it / n_qt;
        const int r_first = (qt0 + it % n_qt) * kTile;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int piece = tid + i * kKvThreads;
            const int row = r_first + C::staged_row(piece);
            qr[i] = gr[i] = make_uint4(0, 0, 0, 0);
            if (row < n) {
                const int64_t off = (((int64_t)b * a.seq + row) * hq + head) * D + C::staged_piece(piece) * 8;
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
        char *qs = lds + kResident + stage * kStage;
        char *gs = qs + C::TILE;
        float *ax = (float *)(gs + C::TILE);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int piece = tid + i * kKvThreads;
            const int off = C::piece(C::staged_row(piece), C::staged_piece(piece));
            *(uint4 *)(qs + off) = qr[i];
            *(uint4 *)(gs + off) = gr[i];
        }
        if (tid < 2 * kTile) ax[tid] = aux;
    };

    f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) dk[i][r] = dv[i][r] = 0.f;

    const float cs = a.scale * kLog2e;
    const int row_lane = C::row_lane(c, hh);
    const int tr_lane = C::tr_lane(lane);
    const char *kb_ = k_res + kblk * C::BLOCK32 + row_lane; // B operands: this wave's keys
    const char *vb_ = v_res + kblk * C::BLOCK32 + row_lane;

    // this wave's block of 32 rows against its 32 keys
    auto compute_block = [&](const char *stage, int r0, auto masked) {
        const char *qs = stage + rb * C::BLOCK32;
        const char *gs = qs + C::TILE;
        const float *ax = (const float *)(stage + 2 * C::TILE);
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
        // S = Q K^T and dP = dO V^T: rows x keys, lane = key column, element r = row 8 (r/4) + 4 hh + r%4.
        // Four steps' operands at a time: fetching all eight at once does not fit the register budget.
#pragma unroll
        for (int half = 0; half < D / 64; ++half) {
#pragma unroll
            for (int st = 4 * half; st < 4 * half + 4; ++st) {
                s = M::mfma(__builtin_bit_cast(vec8, *(const uint4 *)(qs + row_lane + st * 128)),
                            __builtin_bit_cast(vec8, *(const uint4 *)(kb_ + st * 128)), s);
                dp = M::mfma(__builtin_bit_cast(vec8, *(const uint4 *)(gs + row_lane + st * 128)),
                             __builtin_bit_cast(vec8, *(const uint4 *)(vb_ + st * 128)), dp);
            }
            __builtin_amdgcn_sched_barrier(0);
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
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const vec8 pB = pack_step<M>(p + 8 * x);
            const vec8 dsB = pack_step<M>(ds + 8 * x);
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                dv[db] = M::mfma(read_transposed_chunked<M, D>(gs + tr_lane, x, db), pB, dv[db]);
                dk[db] = M::mfma(read_transposed_chunked<M, D>(qs + tr_lane, x, db), dsB, dk[db]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    issue(0);
    park(0);
    if (n_it > 1) issue(1);
    __syncthreads();
    for (int it = 0; it < n_it; ++it) {
        const char *stage = lds + kResident + (it & 1) * kStage;
        const int r0 = (qt0 + it % n_qt) * kTile + 32 * rb;
        if (!(r0 + 31 < kb0 || r0 >= n || kb0 >= n)) { // else: rows before the keys, or nothing valid
            if (r0 < kb0 + 31)
                compute_block(stage, r0, std::true_type{});
            else
                compute_block(stage, r0, std::false_type{});
        }
        if (it + 1 < n_it) park((it + 1) & 1);
        __syncthreads();
        if (it + 2 < n_it) issue(it + 2);
    }

    // The waves of the second row block hand their sums to their partners through LDS (all tiles
    // are done: the staging area is free), one tensor at a time; the partners add and write out.
    // lane owns key my_key; element r of block db is feature 32 db + 8 (r/4) + 4 hh + r%4
    float *red = (float *)lds + (size_t)kblk * (D / 32) * 16 * 64 + lane;
    const int64_t off = (((int64_t)b * a.seq + my_key) * hkv + kvh) * D + 4 * hh;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        __syncthreads();
        if (rb == 1) {
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) red[(db * 16 + r) * 64] = which == 0 ? dk[db][r] : dv[db][r];
        }
        __syncthreads();
        if (rb == 0 && my_key < n) {
            float *dst = (which == 0 ? a.dk_accum : a.dv_accum) + off;
            const float f = which == 0 ? a.scale : 1.f;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    float4 *pd = (float4 *)(dst + 32 * db + 8 * q4);
                    float4 acc = *pd;
                    const f32x16 &mine = which == 0 ? dk[db] : dv[db];
                    acc.x += f * (mine[4 * q4] + red[(db * 16 + 4 * q4) * 64]);
                    acc.y += f * (mine[4 * q4 + 1] + red[(db * 16 + 4 * q4 + 1) * 64]);
                    acc.z += f * (mine[4 * q4 + 2] + red[(db * 16 + 4 * q4 + 2) * 64]);
                    acc.w += f * (mine[4 * q4 + 3] + red[(db * 16 + 4 * q4 + 3) * 64]);
                    *pd = acc;
                }
        }
    }
}

// ---- dQ ------------------------------------------------------------------------------------------
// W waves of 32 rows per work group.  W = 8 keeps the wave below 256 registers (the 64 keys of a
// tile are processed as two blocks of 32), so two waves share a SIMD and cover each other's waits.
template <typename M, int D, int W>
__global__ __launch_bounds__(64 * W, 1) void dq_kernel(TrainBwdArgs a, int n_rt) {
    using C = Chunked<D>;
    using vec8 = typename M::vec8;
    constexpr int LPR = D / 8;
    constexpr int NT = 64 * W;                 // threads
    constexpr int NL = kTile * LPR / NT;       // loads per thread, tile and tensor
    static_assert(NL >= 1, "tile too small for the work group");
    constexpr int kRows = 32 * W;              // rows a work group owns
    constexpr int kStage = 2 * C::TILE;        // K, V
    __shared__ __attribute__((aligned(16))) char lds[2 * kStage];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int c = lane & 31;
    const int hh = lane >> 5;
    const int hkv = a.n_kv_heads, hq = a.n_q_heads;
    const int G = hq / hkv;

    // block -> (sequence, head, row tile).  Work groups are dealt round-robin to the 8 XCDs, each with
    // an L2 of its own: when the (sequence, kv head) pairs divide by 8, the G heads and all row tiles
    // of a pair go to one XCD (they read the same K, V rows: HBM traffic 5.3 -> 0.8 GiB per launch);
    // heavy (late) row tiles first
    const int pairs = a.batch * hkv;
    int pair, rem;
    if (pairs % 8 == 0) {
        const int k = blockIdx.x >> 3;
        pair = (blockIdx.x & 7) + 8 * (k / (G * n_rt));
        rem = k % (G * n_rt);
    } else {
        pair = blockIdx.x % pairs;
        rem = blockIdx.x / pairs;
    }
    const int rt = n_rt - 1 - rem / G;
    const int kvh = pair % hkv;
    const int head = kvh * G + rem % G;
    const int b = pair / hkv;
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
            const int key = t * kTile + C::staged_row(piece);
            kr[i] = vr[i] = make_uint4(0, 0, 0, 0);
            if (key < n_keys) {
                const int64_t off = (((int64_t)b * a.seq + key) * hkv + kvh) * D + C::staged_piece(piece) * 8;
                kr[i] = *(const uint4 *)((const uint16_t *)a.k + off);
                vr[i] = *(const uint4 *)((const uint16_t *)a.v + off);
            }
        }
    };
    auto park = [&](int stage) {
        char *ks = lds + stage * kStage;
        char *vs = ks + C::TILE;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int piece = tid + i * NT;
            const int off = C::piece(C::staged_row(piece), C::staged_piece(piece));
            *(uint4 *)(ks + off) = kr[i];
            *(uint4 *)(vs + off) = vr[i];
        }
    };

    f32x16 dq[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[i][r] = 0.f;

    const float cs = a.scale * kLog2e;
    const int row_lane = C::row_lane(c, hh);
    const int tr_lane = C::tr_lane(lane);

    // one block of 32 keys (kb = 0, 1 of the staged tile) against this wave's 32 rows
    auto compute_block = [&](const char *stage, int j0, int kb, auto masked) {
        const char *ks = stage + kb * C::BLOCK32;
        const char *vs = ks + C::TILE;
        // S^T = K Q^T and dP^T = V dO^T: keys x rows, lane = row column
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
        // four steps' operands at a time: fetching all eight at once does not fit the register budget
#pragma unroll
        for (int half = 0; half < D / 64; ++half) {
#pragma unroll
            for (int st = 4 * half; st < 4 * half + 4; ++st) {
                s = M::mfma(__builtin_bit_cast(vec8, *(const uint4 *)(ks + row_lane + st * 128)), qB[st], s);
                dp = M::mfma(__builtin_bit_cast(vec8, *(const uint4 *)(vs + row_lane + st * 128)), gB[st], dp);
            }
            __builtin_amdgcn_sched_barrier(0);
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
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const vec8 dsB = pack_step<M>(ds + 8 * x);
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
                dq[db] = M::mfma(read_transposed_chunked<M, D>(ks + tr_lane, x, db), dsB, dq[db]);
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
    const int n_kt = (a.seq + kKvKeys - 1) / kKvKeys;
    const int64_t kv_blocks = (int64_t)a.batch * a.n_kv_heads * n_kt;
    const int n_rt = (a.seq + 32 * kDqWaves - 1) / (32 * kDqWaves);
    const int64_t q_blocks = (int64_t)a.batch * a.n_q_heads * n_rt;
    if (delta_blocks > 0x7fffffff || kv_blocks > 0x7fffffff || q_blocks > 0x7fffffff) return hipErrorInvalidValue;
    delta_kernel<M, D><<<dim3((unsigned)delta_blocks), 256, 0, stream>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dkdv_kernel<M, D><<<dim3((unsigned)kv_blocks), kKvThreads, 0, stream>>>(a, n_kt);
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
