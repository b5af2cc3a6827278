// Sampling-phase routed attention for 16-bit caches (paper Eq. (3.1) with one query token per
// sequence, Sec. 3.1.1 "Sampling"): a split-K flash-decoding kernel for gfx950.
//
// The kernel is bound by streaming K and V rows from HBM exactly once.  Work group = 4 waves =
// one (sequence, kv head, key-axis split); the waves take 32-key tiles round-robin.  Per tile a
// wave
//   1. has the tile's K and V rows in registers from coalesced 128-bit buffer loads issued two
//      tiles ahead (16 lanes cover one 256-byte row, a wave-wide load covers 4 whole rows),
//   2. parks them in its private LDS region and at once issues the loads of the tile after next,
//   3. S^T[key][head] = K . Q^T on the matrix cores (v_mfma_f32_16x16x32): the G <= 16 query heads
//      of the GQA group are the 16 columns, so a K/V tile is read once for the whole group and
//      16-bit data feeds the MFMA without unpacking,
//   4. online softmax in registers: a lane holds one head (column) and 8 keys; the maximum over
//      the 32 keys needs two cross-lane steps (lanes l, l^16, l^32, l^48 share a column),
//   5. O^T[d][head] += V^T . P^T, with V^T read from LDS through the transposing read
//      ds_read_b64_tr_b16.  The key order inside the contraction is permuted so that the
//      accumulator layout of step 3 is directly the B-operand layout of this product: the
//      weights never leave the registers.
// The four waves merge through LDS.  A sequence that fits one split gets its normalised output
// at once; otherwise every split writes (max, sum, unnormalised out) in fp32 for the merge launch.
// (Merging in the same launch by the last work group to finish was measured and rejected: making
// the partials visible across the per-XCD L2s costs each work group either an L2 write-back or
// the round trip of write-through stores, which is more than the small merge launch.)
#include <type_traits>

#include "skv_internal.h"

namespace skv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

struct MBF16 {
    using vec8 = bf16x8;
    __device__ static f32x4 mfma(vec8 a, vec8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    __device__ static uint32_t pack2(float lo, float hi) { // round to nearest even
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        bf16x2 v = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
};
struct MF16 {
    using vec8 = f16x8;
    __device__ static f32x4 mfma(vec8 a, vec8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
    __device__ static uint32_t pack2(float lo, float hi) {
        typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
        f16x2 v = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
};

constexpr int kTile = 32; // keys per wave tile
// A launch on a slot that several layers read, whose K/V slice is at most this large, uses cached
// loads: the memory-side cache of the device (256 MiB) then serves the other layers of the sharing
// group.  Measured per call, first / later reader of a group: 128 MiB slice 36.5 / 29.5 us cached
// against 33.6 / 31.7 us streaming; 256 MiB 60.9 / 48.1 against 56.7 / 54.1; 512 MiB 111.6 / 108.9
// against 101.7 / 98.1 (streaming wins: nothing is left on chip for the next reader).
constexpr int64_t kOnChipBytes = (int64_t)256 << 20;

// KV8: the slot holds 8-bit codes (16 per 16-byte piece) that are converted to the 16-bit type on
// their way into LDS; everything behind the LDS tile is the same for both kinds of slot.
template <int D, bool KV8> struct Geo {
    static constexpr int LPR = KV8 ? D / 16 : D / 8; // lanes per row (16 bytes each)
    static constexpr int RPL = 64 / LPR;         // rows per wave-wide load
    static constexpr int NL = kTile / RPL;       // loads per tile and tensor
    static constexpr int K_STRIDE = D * 2 + 16;  // LDS row strides in bytes: chosen so that the 16 rows
    static constexpr int V_STRIDE = D * 2 + 32;  //   one MFMA operand read touches fall in distinct banks
    static constexpr int K_BYTES = kTile * K_STRIDE;
    static constexpr int V_BYTES = kTile * V_STRIDE;
    static constexpr int WAVE_BYTES = K_BYTES + V_BYTES;
};

__device__ __forceinline__ s16x4 lds_read_tr16(const char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(p));
}

// A tile is fetched with BUFFER loads: the descriptor (wave-uniform base, byte count) bounds every lane,
// so rows beyond the end of the range read as zero without a branch.  Every tile therefore issues
// the same number of load instructions whatever its length, and the wait before a tile is parked
// counts exactly the loads issued after it: the loads of the following tile stay in flight across
// it.  (With predicated loads the count of later loads has no lower bound and the wait drains them all.)
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t uniform_rsrc(const void *base, uint32_t bytes) {
    const uint64_t p = (uint64_t)base;
    // (the builtin returns a signed int: widen each half as unsigned, or bit 31 of the low half smears over the high one)
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)p);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
    const uint64_t u = ((uint64_t)hi << 32) | (uint64_t)lo;
    // stride 0 (raw), byte count, 32-bit untyped data
    return __builtin_amdgcn_make_buffer_rsrc((void *)u, 0, (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}
template <bool kStream> __device__ __forceinline__ uint4 buffer_load_16(__amdgpu_buffer_rsrc_t r, uint32_t off) {
    return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, kStream ? 2 : 0)); // 2: non-temporal
}
template <bool kStream> __device__ __forceinline__ uint16_t buffer_load_2(__amdgpu_buffer_rsrc_t r, uint32_t off) {
    return (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)off, 0, kStream ? 2 : 0);
}

// kStream: the K/V loads carry the non-temporal hint (every byte is used once: stream it past the
// caches).  Without it the rows are cached as usual, which is what lets the next layer of a sharing
// group find a small slot slice on chip.
template <typename M, int D, int kWaves, bool kStream, bool KV8>
__global__ __launch_bounds__(64 * kWaves, 2) void decode_mfma_kernel(AttnArgs a, int G, int persistent) {
    using Ge = Geo<D, KV8>;
    using vec8 = typename M::vec8;
    constexpr int NL = Ge::NL, LPR = Ge::LPR, RPL = Ge::RPL;
    __shared__ __attribute__((aligned(16))) char lds[kWaves * Ge::WAVE_BYTES];
    __shared__ int s_item, s_n_rem;
    extern __shared__ int s_prefix[]; // persistent mode: batch + 1 running counts of full splits, then batch uint16

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform on purpose (scalar loads below)
    const int n = lane & 15; // MFMA column: query head of the group (B, C operands) / row (A operand)
    const int g = lane >> 4; // MFMA k-group
    const int hkv = a.cache.n_kv_heads;

    auto keys_of = [&](int bb, int &sink, int &gap) -> int { return decode_keys(a, bb, sink, gap); };

    // One work item = (sequence, kv head, key split).
    auto process_item = [&](const int b, const int kvh, const int split) {
    const int head0 = kvh * G;
    int sink, gap;
    const int kv_end = keys_of(b, sink, gap);
    if (kv_end < 1) { // lengths the host promised not to pass
        if (threadIdx.x == 0 && split == 0 && kvh == 0) atomicOr(a.cache.faults, (uint32_t)SKV_FAULT_KV_LEN);
        if (split == 0)
            for (int e = threadIdx.x; e < G * D; e += blockDim.x)
                ((uint16_t *)a.out)[((int64_t)b * a.n_q_heads + head0) * D + e] = 0;
        return;
    }
    const int k_begin = split * a.keys_per_split;
    const int k_end = min(kv_end, k_begin + a.keys_per_split);
    if (k_begin >= k_end) return; // uniform over the work group
    const int ns = (kv_end + a.keys_per_split - 1) / a.keys_per_split; // splits that hold keys of this sequence

    // Q^T as B operand: lane (n, g), k-step s holds Q[head n][32 s + 8 g .. + 8); heads >= G are zero.
    vec8 qB[D / 32];
    {
        const uint16_t *qp = (const uint16_t *)a.q + ((int64_t)b * a.n_q_heads + head0 + n) * D + 8 * g;
#pragma unroll
        for (int s = 0; s < D / 32; ++s) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (n < G) raw = *(const uint4 *)(qp + 32 * s);
            qB[s] = __builtin_bit_cast(vec8, raw);
        }
    }

    char *ks = lds + wave * Ge::WAVE_BYTES;
    char *vs = ks + Ge::K_BYTES;
    const int lrow = lane / LPR;   // row inside one wave-wide load
    const int lcol = lane % LPR;   // 16-byte piece inside the row
    constexpr int EB = KV8 ? 1 : 2; // bytes per slot element
    // 16-bit slots are row-major ([row][kv head][d]): the lane's part of an address is its row inside
    // the load times the row size plus its piece.  8-bit slots keep the rows of a kv head together
    // (kv8_head_row): the RPL rows of a load are contiguous and the lane's part is 16 x lane.
    const char *kp = (const char *)a.cache.k + (KV8 ? 0 : ((int64_t)kvh * D) * EB); // uniform; the lane's part is lane_off
    const char *vp = (const char *)a.cache.v + (KV8 ? 0 : ((int64_t)kvh * D) * EB);
    const int64_t row_bytes = KV8 ? (int64_t)D : (int64_t)hkv * D * EB; // distance of consecutive rows of this kv head inside a load
    const uint16_t *sp = KV8 ? a.cache.scales : nullptr; // 8-bit slots: exponent bytes of K (low) and V (high) per (row, kv head)

    // Paged caches: the (at most four) block ids a 32-key tile touches are fetched with SCALAR loads
    // one tile ahead.  They have a counter of their own, so waiting for them never drains the
    // vector loads of the K/V tiles that are still in flight.  (The table is not written while the
    // kernel runs: reading it through the constant address space is what makes the loads scalar even
    // after the stores of an earlier work item.)
    const bool paged = a.cache.block_table != nullptr;
    const int shift = a.cache.block_shift;
    auto blocks_of = [&](int j0, int32_t *blk) {
        if (paged) {
            typedef const __attribute__((address_space(4))) int32_t table_word;
            table_word *row = (table_word *)(uintptr_t)(a.cache.block_table + (int64_t)b * a.cache.max_blocks_per_seq);
            const int first = (j0 + (j0 >= sink ? gap : 0)) >> shift;
#pragma unroll
            for (int u = 0; u < 4; ++u) blk[u] = row[min(first + u, a.cache.max_blocks_per_seq - 1)];
        }
    };
    // Load t of the tile at j0 covers RPL consecutive keys, which lie inside one block (blocks hold at
    // least RPL positions and tiles start on block boundaries): its first row is WAVE-UNIFORM, so the
    // address of a lane is a scalar base (slot + first row of the load) plus a 32-bit lane offset that
    // never changes (row inside the load, piece inside the row).  The address arithmetic of the 2 x NL
    // loads of a tile is then scalar work, and the bound against k_end is the byte count of the
    // load's buffer descriptor: nothing is left to do per lane.
    const uint32_t lane_off = (uint32_t)(lrow * (int)row_bytes + lcol * 16);
    auto first_row_of = [&](int j0, const int32_t *blk, int t) -> int64_t { // -1: nothing to load
        const int c0 = j0 + RPL * t;                  // first key of the load, uniform
        if (c0 >= k_end) return -1;
        const int skip = j0 >= sink ? gap : 0;        // the whole tile lies on one side of the gap
        const int p0 = c0 + skip;                     // its position
        if (!paged) return (int64_t)b * a.cache.seq_rows + p0;
        const int u = (p0 >> shift) - ((j0 + skip) >> shift); // 0..3 (0 when a block holds 32 keys or more)
        const int32_t id = u == 0 ? blk[0] : u == 1 ? blk[1] : u == 2 ? blk[2] : blk[3];
        if ((uint32_t)id >= (uint32_t)a.cache.n_blocks) {
            if (lane == 0) atomicOr(a.cache.faults, (uint32_t)SKV_FAULT_BLOCK_ID);
            return -1;
        }
        return ((int64_t)id << shift) + (p0 & ((1 << shift) - 1));
    };
    const uint32_t lane_soff = (uint32_t)(lrow * 2); // 8-bit slots: the lane's row inside the load's exponent byte pairs
    auto issue = [&](int j0, const int32_t *blk, uint4 *kr, uint4 *vr, uint16_t *sr) {
#pragma unroll
        for (int t = 0; t < NL; ++t) {
            const int64_t r0 = first_row_of(j0, blk, t);
            const int rows = r0 < 0 ? 0 : min(RPL, k_end - (j0 + RPL * t)); // rows of the load inside the range
            const int64_t rr = r0 < 0 ? 0 : r0;                             // a valid base in any case
            // first row of the load, in rows of this kv head (8-bit slots: the load never leaves its group)
            const int64_t hr = KV8 ? kv8_head_row(a.cache, rr, kvh) : rr;
            const uint32_t bytes = (uint32_t)(rows * (int)row_bytes);
            const __amdgpu_buffer_rsrc_t rk = uniform_rsrc(kp + hr * row_bytes, bytes);
            const __amdgpu_buffer_rsrc_t rv = uniform_rsrc(vp + hr * row_bytes, bytes);
            kr[t] = buffer_load_16<kStream>(rk, lane_off);
            vr[t] = buffer_load_16<kStream>(rv, lane_off);
            if constexpr (KV8) // rows that are not loaded read as codes 0 with exponent byte 0: zeros
                sr[t] = buffer_load_2<kStream>(uniform_rsrc(sp + hr, (uint32_t)(rows * 2)), lane_soff);
        }
    };

    float m_run = -INFINITY, l_part = 0.f;
    f32x4 o[D / 16];
#pragma unroll
    for (int i = 0; i < D / 16; ++i) o[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Tiles of the split are dealt round-robin to the waves.  The walk starts at a tile that
    // differs from work group to work group (softmax does not care about key order): work groups
    // that run side by side then sit at unrelated offsets of their ranges instead of marching
    // through the HBM channels in lockstep.
    const int n_tiles = (k_end - k_begin + kTile - 1) / kTile;
    const int start = (split * 7 + kvh * 3 + b * 5) % n_tiles;
    auto tile_j0 = [&](int tt) {
        int t2 = tt + start;
        if (t2 >= n_tiles) t2 -= n_tiles;
        return k_begin + t2 * kTile;
    };

    // Two tiles per wave are in flight from HBM (register sets A, B) while another is computed from
    // LDS; the block ids run one more tile ahead.
    int32_t blk[4] = {0, 0, 0, 0};
    int tt_issue = wave; // next tile of this wave to request
    // Always issues a tile's worth of loads: past the last tile they carry an empty descriptor (no
    // memory access, no address arithmetic), which keeps the number of loads in flight behind any
    // tile a constant.
    auto issue_next = [&](uint4 *kr, uint4 *vr, uint16_t *sr) {
        if (tt_issue < n_tiles) {
            issue(tile_j0(tt_issue), blk, kr, vr, sr);
        } else {
            const __amdgpu_buffer_rsrc_t none = uniform_rsrc(kp, 0);
#pragma unroll
            for (int t = 0; t < NL; ++t) {
                kr[t] = buffer_load_16<kStream>(none, lane_off);
                vr[t] = buffer_load_16<kStream>(none, lane_off);
                if constexpr (KV8) sr[t] = buffer_load_2<kStream>(none, lane_soff);
            }
        }
        tt_issue += kWaves;
        if (tt_issue < n_tiles) blocks_of(tile_j0(tt_issue), blk);
    };
    uint4 krA[NL], vrA[NL], krB[NL], vrB[NL];
    uint16_t srA[KV8 ? NL : 1], srB[KV8 ? NL : 1];
    if (wave < n_tiles) blocks_of(tile_j0(wave), blk);
    issue_next(krA, vrA, srA);
    issue_next(krB, vrB, srB);

    auto process = [&](int tt, uint4 *kr, uint4 *vr, uint16_t *sr) {
        const int j0 = tile_j0(tt);
        // park the tile in LDS: row-major, 16-byte pieces, padded row stride
#pragma unroll
        for (int t = 0; t < NL; ++t) {
            if constexpr (KV8) { // 16 codes x 2^e -> two pieces of eight 16-bit values, exactly
                constexpr bool bf = std::is_same<M, MBF16>::value;
                uint4 lo, hi;
                dequant_piece<bf>(kr[t], scale_of_byte(sr[t] & 0xffu), lo, hi);
                *(uint4 *)(ks + (RPL * t + lrow) * Ge::K_STRIDE + lcol * 32) = lo;
                *(uint4 *)(ks + (RPL * t + lrow) * Ge::K_STRIDE + lcol * 32 + 16) = hi;
                dequant_piece<bf>(vr[t], scale_of_byte(sr[t] >> 8), lo, hi);
                *(uint4 *)(vs + (RPL * t + lrow) * Ge::V_STRIDE + lcol * 32) = lo;
                *(uint4 *)(vs + (RPL * t + lrow) * Ge::V_STRIDE + lcol * 32 + 16) = hi;
            } else {
                *(uint4 *)(ks + (RPL * t + lrow) * Ge::K_STRIDE + lcol * 16) = kr[t];
                *(uint4 *)(vs + (RPL * t + lrow) * Ge::V_STRIDE + lcol * 16) = vr[t];
            }
        }
        // the tile is exchanged between the lanes of this wave only: order the LDS traffic for the
        // compiler (the hardware runs one wave's LDS operations in order)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        issue_next(kr, vr, sr); // the freed register set requests the tile after the one in flight

        // S^T = K Q^T for keys [j0, j0+16) and [j0+16, j0+32)
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < D / 32; ++s) {
            const vec8 a0 = __builtin_bit_cast(vec8, *(const uint4 *)(ks + n * Ge::K_STRIDE + (4 * s + g) * 16));
            const vec8 a1 = __builtin_bit_cast(vec8, *(const uint4 *)(ks + (16 + n) * Ge::K_STRIDE + (4 * s + g) * 16));
            s0 = M::mfma(a0, qB[s], s0);
            s1 = M::mfma(a1, qB[s], s1);
        }
        // lane (head n, group g) holds keys j0 + 4g + r (s0) and j0 + 16 + 4g + r (s1); log2 units
        float sc[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            sc[r] = s0[r] * a.scale_log2e;
            sc[4 + r] = s1[r] * a.scale_log2e;
        }
        if (j0 + kTile > k_end) { // ragged tail
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (j0 + 4 * g + r >= k_end) sc[r] = -INFINITY;
                if (j0 + 16 + 4 * g + r >= k_end) sc[4 + r] = -INFINITY;
            }
        }
        float mt = sc[0];
#pragma unroll
        for (int r = 1; r < 8; ++r) mt = fmaxf(mt, sc[r]);
        mt = fmaxf(mt, __shfl_xor(mt, 16, 64));
        mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
        const float m_new = fmaxf(m_run, mt); // finite: every tile holds at least one key
        const float alpha = exp2f(m_run - m_new);
        m_run = m_new;
        float p[8], psum = 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            p[r] = exp2f(sc[r] - m_new);
            psum += p[r];
        }
        l_part = l_part * alpha + psum;
        if (__any(alpha != 1.f)) { // the running maximum settles quickly; skip the rescale when it did
#pragma unroll
            for (int i = 0; i < D / 16; ++i) o[i] *= alpha;
        }
        const uint4 praw = make_uint4(M::pack2(p[0], p[1]), M::pack2(p[2], p[3]), M::pack2(p[4], p[5]),
                                      M::pack2(p[6], p[7]));
        const vec8 pB = __builtin_bit_cast(vec8, praw);
        // O^T[d][head] += V^T P^T; k-slot (g, j) is key 4g + j for j < 4 and 16 + 4g + (j - 4) otherwise
        const char *v_lo = vs + (4 * g + (n >> 2)) * Ge::V_STRIDE + (n & 3) * 8;
        const char *v_hi = v_lo + 16 * Ge::V_STRIDE;
#pragma unroll
        for (int i = 0; i < D / 16; ++i) {
            const s16x4 lo = lds_read_tr16(v_lo + i * 32);
            const s16x4 hi = lds_read_tr16(v_hi + i * 32);
            const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            o[i] = M::mfma(__builtin_bit_cast(vec8, both), pB, o[i]);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); // reads of this tile before the next tile's writes
        __builtin_amdgcn_wave_barrier();
    };
    int tt = wave;
    for (; tt + kWaves < n_tiles; tt += 2 * kWaves) { // both tiles exist: no load of the loop body is conditional
        process(tt, krA, vrA, srA);
        process(tt + kWaves, krB, vrB, srB);
    }
    if (tt < n_tiles) process(tt, krA, vrA, srA);

    // ---- merge the four waves through LDS --------------------------------------------------
    float l_tot = l_part + __shfl_xor(l_part, 16, 64);
    l_tot += __shfl_xor(l_tot, 32, 64);
    __syncthreads(); // every wave is done with its tile region
    float *mo = (float *)lds;                 // [wave][G][D]
    float *mml = mo + kWaves * 16 * D;        // [wave][16][2]
    if (n < G) {
#pragma unroll
        for (int i = 0; i < D / 16; ++i)
            *(f32x4 *)(mo + ((wave * G + n) * D + 16 * i + 4 * g)) = o[i];
        if (g == 0) {
            mml[(wave * 16 + n) * 2] = m_run;
            mml[(wave * 16 + n) * 2 + 1] = l_tot;
        }
    }
    __syncthreads();
    for (int w = threadIdx.x; w < G * (D / 4); w += blockDim.x) {
        const int h = w / (D / 4), d4 = (w % (D / 4)) * 4;
        float m = -INFINITY;
#pragma unroll
        for (int v = 0; v < kWaves; ++v) m = fmaxf(m, mml[(v * 16 + h) * 2]);
        float l = 0.f;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int v = 0; v < kWaves; ++v) {
            const float mv = mml[(v * 16 + h) * 2];
            const float wv = mv == -INFINITY ? 0.f : exp2f(mv - m);
            l += mml[(v * 16 + h) * 2 + 1] * wv;
            acc += *(const f32x4 *)(mo + ((v * G + h) * D + d4)) * wv;
        }
        const int64_t rh = (int64_t)b * a.n_q_heads + head0 + h;
        if (ns == 1) {
            const float inv = 1.f / l;
            *(uint2 *)((uint16_t *)a.out + rh * D + d4) =
                make_uint2(M::pack2(acc[0] * inv, acc[1] * inv), M::pack2(acc[2] * inv, acc[3] * inv));
        } else {
            const int64_t pidx = rh * a.n_splits + split;
            *(f32x4 *)(a.part_o + pidx * D + d4) = acc;
            if (d4 == 0) {
                a.part_ml[pidx * 2] = m;
                a.part_ml[pidx * 2 + 1] = l;
            }
        }
    }
    }; // process_item

    if (!persistent) {
        process_item(blockIdx.z, blockIdx.y, blockIdx.x);
        return;
    }
    // Persistent mode: when the sequences have very different lengths, a (split, head, sequence) grid
    // is mostly work groups with nothing to do, each costing a slot and a memory round trip under
    // load.  Instead a fixed number of work groups (two per compute unit) pull items from a counter.
    // Order of the items: first every FULL split of every sequence (all keys_per_split long), then
    // the last, partial split of each sequence, the longest first.  The launch ends when the last
    // item ends, and with short items last the work groups finish close together (items in sequence
    // order left the tail to chance: half an item per work group, 8 % of a launch of six items each).
    // prefix[b] = number of full splits of the sequences before b; order[r] = sequence of the r-th
    // partial split (a sequence with an impossible length has one, of size 0, which zero-fills its
    // output and raises the fault word).
    const int kps = a.keys_per_split;
    unsigned short *s_order = (unsigned short *)(s_prefix + a.batch + 1);
    int *s_rem = (int *)lds;                 // set-up scratch in the tile area: partial size, -1 = none
    int *s_tmp = s_rem + a.batch;
    if (wave == 0) {
        const int per = (a.batch + 63) / 64;
        int cnt_full = 0, cnt_rem = 0;
        for (int i = 0; i < per; ++i) {
            const int bb = lane * per + i;
            if (bb < a.batch) {
                int sk, gp;
                const int len = keys_of(bb, sk, gp);
                const bool valid = len >= 1;
                const int rem = valid ? len % kps : 0;
                const bool has = !valid || rem > 0;
                cnt_full += valid ? len / kps : 0;
                cnt_rem += has;
                s_rem[bb] = has ? rem : -1;
            }
        }
        int incl_f = cnt_full, incl_r = cnt_rem;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int uf = __shfl_up(incl_f, d, 64), ur = __shfl_up(incl_r, d, 64);
            if (lane >= d) {
                incl_f += uf;
                incl_r += ur;
            }
        }
        int run_f = incl_f - cnt_full, run_r = incl_r - cnt_rem;
        if (lane == 0) s_prefix[0] = 0;
        if (lane == 63) s_n_rem = incl_r;
        for (int i = 0; i < per; ++i) {
            const int bb = lane * per + i;
            if (bb < a.batch) {
                int sk, gp;
                const int len = keys_of(bb, sk, gp);
                run_f += len >= 1 ? len / kps : 0;
                s_prefix[bb + 1] = run_f;
                if (s_rem[bb] >= 0) s_order[run_r++] = (unsigned short)bb;
            }
        }
    }
    __syncthreads();
    const int n_rem = s_n_rem;
    if (a.batch <= (int)blockDim.x) { // rank by counting: one partial split per thread
        int rank = -1, mine = 0;
        if ((int)threadIdx.x < n_rem) {
            mine = s_order[threadIdx.x];
            const int r = s_rem[mine];
            rank = 0;
            for (int u = 0; u < n_rem; ++u) {
                const int other = s_order[u], ro = s_rem[other];
                rank += (ro > r) || (ro == r && other < mine);
            }
            s_tmp[rank] = mine;
        }
        __syncthreads();
        if ((int)threadIdx.x < n_rem) s_order[threadIdx.x] = (unsigned short)s_tmp[threadIdx.x];
        __syncthreads();
    }
    const int total_full = s_prefix[a.batch];
    const int total = (total_full + n_rem) * hkv;
    int32_t *counter = a.work_counters; // zero when the launch starts (cleared by the launcher)
    int next = blockIdx.x; // the first item needs no ticket; tickets count on from the grid size
    for (;;) {
        if (threadIdx.x == 0) s_item = next;
        __syncthreads();
        const int item = s_item;
        __syncthreads(); // every thread has read the item; also fences the previous item's LDS use
        if (item >= total) break;
        // take the next ticket now: its round trip hides behind this item's work
        if (threadIdx.x == 0)
            next = (int)gridDim.x + __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int kvh = item % hkv;
        const int j = item / hkv;
        int seq, split;
        if (j < total_full) {
            int lo = 0, hi = a.batch; // largest b with prefix[b] <= j
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_prefix[mid] <= j) lo = mid;
                else hi = mid;
            }
            seq = lo;
            split = j - s_prefix[lo];
        } else {
            seq = s_order[j - total_full];
            int sk, gp;
            const int len = keys_of(seq, sk, gp);
            split = len >= 1 ? len / kps : 0; // the partial split is the last one
        }
        // all lanes hold the same values; say so to the compiler (scalar registers, scalar loads)
        process_item(__builtin_amdgcn_readfirstlane(seq), __builtin_amdgcn_readfirstlane(kvh),
                     __builtin_amdgcn_readfirstlane(split));
    }
}

// Clears the work counter of the persistent launch shape (a kernel, not a memset: the call may be
// recorded into a HIP graph).
__global__ void clear_counter_kernel(int32_t *counter) {
    if (threadIdx.x < 2) counter[threadIdx.x] = 0;
}

template <typename M, int D, bool KV8>
hipError_t launch_d(const AttnArgs &a, int group, hipStream_t stream) {
    static const int n_cu = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        return cus;
    }();
    // Items are pulled from a counter by two resident work groups per compute unit when the grid
    // could hold many empty splits (more than two splits per sequence); a batch too large for the
    // split-count table in LDS, or a launch with few items, uses the plain grid.
    const int64_t max_items = (int64_t)a.n_splits * a.cache.n_kv_heads * a.batch;
    // Cache policy of the K/V loads: stream past the caches unless everything the launch can read
    // (sequences x longest length x K and V rows) is small enough to stay on chip until the next
    // layer of the sharing group reads it again.
    const int64_t slice_bytes = (int64_t)a.batch * a.max_kv_len * a.cache.n_kv_heads * D * 2 * (KV8 ? 1 : 2);
    const int forced = tuning().decode_loads;
    const bool stream_loads = forced ? forced == 1 : (a.slot_readers < 2 || slice_bytes > kOnChipBytes);
    if (a.n_splits > 2 && a.batch <= 1024 && a.work_counters != nullptr && max_items > 2 * n_cu) {
        const size_t dyn = sizeof(int) * (size_t)(a.batch + 1) + sizeof(unsigned short) * (size_t)a.batch;
        clear_counter_kernel<<<1, 64, 0, stream>>>(a.work_counters);
        if (stream_loads) decode_mfma_kernel<M, D, 4, true, KV8><<<dim3(2 * n_cu), 256, dyn, stream>>>(a, group, 1);
        else decode_mfma_kernel<M, D, 4, false, KV8><<<dim3(2 * n_cu), 256, dyn, stream>>>(a, group, 1);
    } else {
        const dim3 grid((unsigned)a.n_splits, (unsigned)a.cache.n_kv_heads, (unsigned)a.batch);
        if (stream_loads) decode_mfma_kernel<M, D, 4, true, KV8><<<grid, 256, 0, stream>>>(a, group, 0);
        else decode_mfma_kernel<M, D, 4, false, KV8><<<grid, 256, 0, stream>>>(a, group, 0);
    }
    set_last_kernel_name("decode_mfma_kernel");
    return hipGetLastError();
}

} // namespace

bool decode_mfma_supported(int dtype, int head_dim, int group) {
    const int act = dtype_act(dtype);
    return (act == SKV_BF16 || act == SKV_F16) && (head_dim == 64 || head_dim == 128) && group <= 16;
}

hipError_t launch_decode_mfma(const AttnArgs &a, int dtype, int head_dim, int group, hipStream_t stream) {
    if (a.batch > 65535 || a.cache.n_kv_heads > 65535) return hipErrorInvalidValue;
    if (dtype_kv8(dtype)) {
        if (a.cache.scales == nullptr) return hipErrorInvalidValue;
        if (dtype_act(dtype) == SKV_BF16)
            return head_dim == 128 ? launch_d<MBF16, 128, true>(a, group, stream) : launch_d<MBF16, 64, true>(a, group, stream);
        return head_dim == 128 ? launch_d<MF16, 128, true>(a, group, stream) : launch_d<MF16, 64, true>(a, group, stream);
    }
    if (dtype == SKV_BF16) {
        return head_dim == 128 ? launch_d<MBF16, 128, false>(a, group, stream) : launch_d<MBF16, 64, false>(a, group, stream);
    }
    return head_dim == 128 ? launch_d<MF16, 128, false>(a, group, stream) : launch_d<MF16, 64, false>(a, group, stream);
}

} // namespace skv
