// Pre-fill-phase routed attention for 16-bit caches (paper Sec. 3.1.1 "Pre-fill": the prompt's
// tokens are processed in parallel; Eq. (3.1): the keys and values come from the slot of the
// layer's source layer).  A tiled causal flash-attention kernel on the gfx950 matrix cores.
//
// Work group = 8 waves = 256 consecutive query rows of one (sequence, query head); wave w owns
// rows 32w..32w+31.  The key axis is walked in tiles of 64 keys staged in LDS (double buffered,
// filled by all 512 threads with coalesced 128-bit loads issued one tile ahead).  Per tile a wave
//   S^T[key][row] = K . Q^T      v_mfma_f32_32x32x16, Q^T lives in registers for the whole kernel;
//   online softmax down the columns: a lane owns one query row (column) and 32 of the 64 keys,
//       its partner lane (l ^ 32) the other 32;
//   O^T[d][row] += V^T . P^T     V^T comes from LDS through ds_read_b64_tr_b16, and the key order
//       inside the contraction is permuted so that the S^T accumulators are, after exponentiation
//       and rounding to 16 bits, directly the B operand: the weights never leave the registers.
// Row i of a sequence with n cached positions and q query rows sits at position n - q + i and
// sees keys 0..that position; tiles entirely above a wave's diagonal are skipped, only tiles that
// touch it are masked.
#include <type_traits>

#include "skv_internal.h"

namespace skv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

struct PBF16 {
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
struct PF16 {
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
constexpr int kBM = 32 * kWaves; // query rows per work group
constexpr int kBN = 64;          // keys per tile

template <int D> struct Geo {
    static constexpr int LPR = D / 8;                  // 16-byte pieces per row
    static constexpr int PIECES = kBN * LPR;           // pieces per tile and tensor
    static constexpr int NL = PIECES / (64 * kWaves);  // loads per thread, tile and tensor
    static constexpr int K_STRIDE = D * 2 + 16;
    static constexpr int V_STRIDE = D * 2 + 64;
    static constexpr int K_BYTES = kBN * K_STRIDE;
    static constexpr int V_BYTES = kBN * V_STRIDE;
    static constexpr int STAGE_BYTES = K_BYTES + V_BYTES;
    static_assert(NL >= 1, "tile too small for the work group");
};

__device__ __forceinline__ s16x4 lds_read_tr16(const char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(p));
}

// KV8: the slot holds 8-bit codes with a power-of-two scale per (row, kv head); a thread then moves
// one 16-byte piece of 16 codes per tile and tensor and parks it as two pieces of 16-bit values
// (code x 2^e, exact), so everything behind the LDS tile is the same for both kinds of slot.
template <typename M, int D, bool KV8>
__global__ __launch_bounds__(64 * kWaves, 1) void prefill_mfma_kernel(AttnArgs a, int G, int n_qt, int xcd_map) {
    using Ge = Geo<D>;
    using vec8 = typename M::vec8;
    constexpr int LPR = KV8 ? D / 16 : Ge::LPR;                // 16-byte pieces per slot row
    constexpr int NL = KV8 ? 1 : Ge::NL;                       // loads per thread, tile and tensor
    constexpr int EB = KV8 ? 1 : 2;                            // bytes per slot element
    constexpr bool kAllLoad = kBN * LPR >= 64 * kWaves;        // 8-bit slots of head_dim 64: half the threads load
    __shared__ __attribute__((aligned(16))) char lds[2 * Ge::STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int c = lane & 31;  // MFMA column: query row of the wave (B, C) / row of the A operand
    const int hh = lane >> 5; // MFMA k-group
    const int hkv = a.cache.n_kv_heads;

    // block -> (query tile, head, sequence).  Heavy (late) query tiles first; with xcd_map the
    // G heads of a kv head and neighbouring query tiles land on one XCD (ids are dealt round-robin
    // to the 8 XCDs) so that they share K/V tiles in that XCD's L2.
    int qt, head, b;
    {
        const int id = blockIdx.x;
        int pair, rem;
        if (xcd_map) {
            const int per_pair = G * n_qt;
            const int k = id >> 3;
            pair = (id & 7) + 8 * (k / per_pair);
            rem = k % per_pair;
        } else {
            pair = id / (G * n_qt);
            rem = id % (G * n_qt);
        }
        qt = n_qt - 1 - rem / G;
        head = (pair % hkv) * G + rem % G;
        b = pair / hkv;
    }
    const int kvh = head / G;

    const int nq = a.q_lens[b];
    const int n = a.kv_lens[b];
    if (nq < 0 || nq > a.max_q || n < 1 || n > a.max_kv_len || nq > n) {
        if (tid == 0 && qt == 0 && head == 0) atomicOr(a.cache.faults, (uint32_t)SKV_FAULT_KV_LEN);
        return; // nothing is written for a sequence with impossible lengths
    }
    const int q_begin = qt * kBM;
    if (q_begin >= nq) return;
    const int offset = n - nq;
    const int q_last = min(q_begin + kBM, nq) - 1;  // last valid row of the work group
    const int n_keys = offset + q_last + 1;         // keys the work group needs
    const int n_tiles = (n_keys + kBN - 1) / kBN;

    const int r0 = q_begin + 32 * wave;
    const int my_row = r0 + c;
    const bool row_ok = my_row < nq;
    const int my_pos = offset + my_row;
    const bool wave_ok = r0 < nq;
    const int wave_last_pos = offset + min(r0 + 31, nq - 1);

    // Q^T as B operand: lane (row c, k-group hh), k-step s holds Q[row][16 s + 8 hh .. + 8)
    vec8 qB[D / 16];
    {
        const uint16_t *qp =
            (const uint16_t *)a.q + (((int64_t)b * a.max_q + my_row) * a.n_q_heads + head) * D + 8 * hh;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (row_ok) raw = *(const uint4 *)(qp + 16 * s);
            qB[s] = __builtin_bit_cast(vec8, raw);
        }
    }

    // cooperative tile loads: thread t moves pieces t, t + 512, ... (16 lanes per row => coalesced)
    // 16-bit slots are row-major; 8-bit slots keep the rows of a kv head together (kv8_head_row)
    const char *kp = (const char *)a.cache.k + (KV8 ? 0 : (int64_t)kvh * D * EB);
    const char *vp = (const char *)a.cache.v + (KV8 ? 0 : (int64_t)kvh * D * EB);
    const int64_t row_bytes = KV8 ? (int64_t)D : (int64_t)hkv * D * EB;
    const bool loader = kAllLoad || tid < kBN * LPR;
    auto rows_of = [&](int j0, int32_t *rows) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            if (!loader) { rows[i] = -1; continue; }
            // keys past the last needed one repeat it: they are masked anyway, and a real row keeps
            // the V operand finite (0 x NaN from never-written cache memory would poison the sum)
            const int key = min(j0 + (tid + i * 64 * kWaves) / LPR, n_keys - 1);
            const int64_t r = slot_row(a.cache, b, key);
            if (r < 0 && (tid % LPR) == 0) atomicOr(a.cache.faults, (uint32_t)SKV_FAULT_BLOCK_ID);
            rows[i] = (int32_t)r;
        }
    };
    uint16_t sr[NL]; // 8-bit slots: exponent bytes (K low, V high) of the row of each piece
#pragma unroll
    for (int i = 0; i < NL; ++i) sr[i] = 0x7f7f;
    auto issue = [&](const int32_t *rows, uint4 *kr, uint4 *vr) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            if (rows[i] >= 0) { // a bad block id keeps the previous (finite) piece
                const int64_t hr = KV8 ? kv8_head_row(a.cache, rows[i], kvh) : rows[i];
                const int64_t off = hr * row_bytes + (tid % LPR) * 16;
                kr[i] = *(const uint4 *)(kp + off);
                vr[i] = *(const uint4 *)(vp + off);
                if constexpr (KV8) sr[i] = a.cache.scales[hr];
            }
        }
    };
    auto park = [&](int stage, const uint4 *kr, const uint4 *vr) {
        char *ks = lds + stage * Ge::STAGE_BYTES;
        char *vs = ks + Ge::K_BYTES;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int piece = tid + i * 64 * kWaves;
            if constexpr (KV8) {
                if (!loader) continue;
                constexpr bool bf = std::is_same<M, PBF16>::value;
                uint4 lo, hi;
                dequant_piece<bf>(kr[i], scale_of_byte(sr[i] & 0xffu), lo, hi);
                *(uint4 *)(ks + (piece / LPR) * Ge::K_STRIDE + (piece % LPR) * 32) = lo;
                *(uint4 *)(ks + (piece / LPR) * Ge::K_STRIDE + (piece % LPR) * 32 + 16) = hi;
                dequant_piece<bf>(vr[i], scale_of_byte(sr[i] >> 8), lo, hi);
                *(uint4 *)(vs + (piece / LPR) * Ge::V_STRIDE + (piece % LPR) * 32) = lo;
                *(uint4 *)(vs + (piece / LPR) * Ge::V_STRIDE + (piece % LPR) * 32 + 16) = hi;
            } else {
                *(uint4 *)(ks + (piece / LPR) * Ge::K_STRIDE + (piece % LPR) * 16) = kr[i];
                *(uint4 *)(vs + (piece / LPR) * Ge::V_STRIDE + (piece % LPR) * 16) = vr[i];
            }
        }
    };

    float m_run = -INFINITY, l_part = 0.f;
    f32x16 o[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] = 0.f;

    uint4 kr[NL], vr[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) kr[i] = vr[i] = make_uint4(0, 0, 0, 0);
    int32_t rows[NL];
    rows_of(0, rows);
    issue(rows, kr, vr);
    park(0, kr, vr);
    if (n_tiles > 1) {
        rows_of(kBN, rows);
        issue(rows, kr, vr);
        if (n_tiles > 2) rows_of(2 * kBN, rows);
    }
    __syncthreads();

    const float cs = a.scale_log2e; // > 0 (checked by the host): maxima can be taken on raw scores
    const int sl = lane & 15;
    const int v_lane_off = (4 * hh + (sl >> 2)) * Ge::V_STRIDE + ((lane >> 4) & 1) * 32 + (sl & 3) * 8;

    // One 64-key tile for this wave.  `masked` is a compile-time tag: only tiles that touch the
    // wave's diagonal pay for the causal mask.
    auto compute_tile = [&](const char *ks, const char *vs, int j0, auto masked) {
        // S^T = K Q^T: key blocks [j0, j0+32) and [j0+32, j0+64), two independent accumulator chains
        f32x16 s0, s1;
#pragma unroll
        for (int r = 0; r < 16; ++r) s0[r] = s1[r] = 0.f;
        const char *k0 = ks + c * Ge::K_STRIDE + hh * 16;
        const char *k1 = k0 + 32 * Ge::K_STRIDE;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            const vec8 a0 = __builtin_bit_cast(vec8, *(const uint4 *)(k0 + s * 32));
            const vec8 a1 = __builtin_bit_cast(vec8, *(const uint4 *)(k1 + s * 32));
            s0 = M::mfma(a0, qB[s], s0);
            s1 = M::mfma(a1, qB[s], s1);
        }
        // element r of block kb is key j0 + 32 kb + 8 (r / 4) + 4 hh + (r % 4)
        float sc[32];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            sc[r] = s0[r];
            sc[16 + r] = s1[r];
        }
        if constexpr (decltype(masked)::value) {
#pragma unroll
            for (int r = 0; r < 32; ++r) {
                const int key = j0 + 32 * (r >> 4) + 8 * ((r & 15) >> 2) + 4 * hh + (r & 3);
                if (key > my_pos) sc[r] = -INFINITY;
            }
        }
        float mt = sc[0];
#pragma unroll
        for (int r = 1; r < 32; ++r) mt = fmaxf(mt, sc[r]);
        mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
        const float m_new = fmaxf(m_run, mt); // raw-score units; finite from the first tile on
        // Lazy reference: the accumulators are rescaled only when some row's maximum grew by more
        // than 2^8 in weight; until then weights may reach 256 instead of 1, which fp32 sums and
        // 16-bit weights hold without loss, and the final division by the row sum is unaffected.
        if (__any((m_new - m_run) * cs > 8.f)) {
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * cs);
            l_part *= alpha;
#pragma unroll
            for (int i = 0; i < D / 32; ++i) o[i] *= alpha;
            m_run = m_new;
        }
        const float neg_mc = -m_run * cs;
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 32; ++r) { // weights 2^(cs (s - m)); masked scores are -inf -> 0
            sc[r] = __builtin_amdgcn_exp2f(fmaf(sc[r], cs, neg_mc));
            psum += sc[r];
        }
        l_part += psum;
        // P^T as B operands: MFMA step x = 2 kb + u takes accumulator elements 8u .. 8u+7 of block kb:
        // k-slot (hh, j) = key 16 x + 4 hh + j (j < 4) or 16 x + 8 + 4 hh + (j - 4)
        vec8 pB[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const uint4 raw = make_uint4(M::pack2(sc[8 * x], sc[8 * x + 1]), M::pack2(sc[8 * x + 2], sc[8 * x + 3]),
                                         M::pack2(sc[8 * x + 4], sc[8 * x + 5]), M::pack2(sc[8 * x + 6], sc[8 * x + 7]));
            pB[x] = __builtin_bit_cast(vec8, raw);
        }
        // O^T[d][row] += V^T P^T.  A 16-lane block reads 4 keys x 16 d transposed:
        // lanes 0-15 / 16-31 are the low / high 16 d of the 32-d block, hh picks the key group.
        const char *vbase = vs + v_lane_off;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const char *vx = vbase + 16 * x * Ge::V_STRIDE;
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const s16x4 lo = lds_read_tr16(vx + db * 64);
                const s16x4 hi = lds_read_tr16(vx + 8 * Ge::V_STRIDE + db * 64);
                const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                o[db] = M::mfma(__builtin_bit_cast(vec8, both), pB[x], o[db]);
            }
        }
    };

    for (int t = 0; t < n_tiles; ++t) {
        const int j0 = t * kBN;
        const char *ks = lds + (t & 1) * Ge::STAGE_BYTES;
        const char *vs = ks + Ge::K_BYTES;

        if (wave_ok && j0 <= wave_last_pos) {
            if (j0 + kBN - 1 > offset + r0) // the tile touches the diagonal of this wave
                compute_tile(ks, vs, j0, std::true_type{});
            else
                compute_tile(ks, vs, j0, std::false_type{});
        }

        // stage the next tile (its loads were issued a tile ago), then fetch the one after
        if (t + 1 < n_tiles) park((t + 1) & 1, kr, vr);
        __syncthreads();
        if (t + 2 < n_tiles) {
            issue(rows, kr, vr);
            if (t + 3 < n_tiles) rows_of((t + 3) * kBN, rows);
        }
    }

    if (!row_ok) return;
    const float l_tot = l_part + __shfl_xor(l_part, 32, 64);
    const float inv = 1.f / l_tot;
    if (a.lse != nullptr && hh == 0) // natural log of sum_j exp(scale s_j) = ln 2 (cs m + log2 l)
        a.lse[((int64_t)b * a.n_q_heads + head) * a.max_q + my_row] =
            0.6931471805599453f * (m_run * cs + __builtin_amdgcn_logf(l_tot));
    // O^T accumulators: lane owns row my_row; element r of block db is d = 32 db + 8 (r/4) + 4 hh + (r%4)
    uint16_t *op = (uint16_t *)a.out + (((int64_t)b * a.max_q + my_row) * a.n_q_heads + head) * D + 4 * hh;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const uint2 w = make_uint2(M::pack2(o[db][4 * q4] * inv, o[db][4 * q4 + 1] * inv),
                                       M::pack2(o[db][4 * q4 + 2] * inv, o[db][4 * q4 + 3] * inv));
            *(uint2 *)(op + 32 * db + 8 * q4) = w;
        }
}

template <typename M, int D, bool KV8>
hipError_t launch_p(const AttnArgs &a, int group, hipStream_t stream) {
    const int n_qt = (a.max_q + kBM - 1) / kBM;
    const int pairs = a.batch * a.cache.n_kv_heads;
    const int64_t blocks = (int64_t)pairs * group * n_qt;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    const int xcd_map = (pairs % 8) == 0;
    prefill_mfma_kernel<M, D, KV8><<<dim3((unsigned)blocks), 64 * kWaves, 0, stream>>>(a, group, n_qt, xcd_map);
    set_last_kernel_name("prefill_mfma_kernel");
    return hipGetLastError();
}

} // namespace

bool prefill_mfma_supported(int dtype, int head_dim, int group) {
    (void)group;
    const int act = dtype_act(dtype);
    return (act == SKV_BF16 || act == SKV_F16) && (head_dim == 64 || head_dim == 128);
}

hipError_t launch_prefill_mfma(const AttnArgs &a, int dtype, int head_dim, int group, hipStream_t stream) {
    if (dtype_kv8(dtype)) {
        if (a.cache.scales == nullptr) return hipErrorInvalidValue;
        if (dtype_act(dtype) == SKV_BF16)
            return head_dim == 128 ? launch_p<PBF16, 128, true>(a, group, stream) : launch_p<PBF16, 64, true>(a, group, stream);
        return head_dim == 128 ? launch_p<PF16, 128, true>(a, group, stream) : launch_p<PF16, 64, true>(a, group, stream);
    }
    if (dtype == SKV_BF16) {
        return head_dim == 128 ? launch_p<PBF16, 128, false>(a, group, stream) : launch_p<PBF16, 64, false>(a, group, stream);
    }
    return head_dim == 128 ? launch_p<PF16, 128, false>(a, group, stream) : launch_p<PF16, 64, false>(a, group, stream);
}

} // namespace skv
