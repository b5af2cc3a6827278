// Pre-fill-phase routed attention (paper Sec. 3.1.1 "Pre-fill", Eq. (3.1)) for 16-bit contiguous
// caches with head_dim 128: the software-pipelined kernel.
//
// Work group = 4 waves, each owning 64 query rows of one query head as two blocks of 32, so that
// every K / V^T operand read from LDS feeds two MFMAs.  The waves share the K/V tiles of one kv head:
// with a GQA group of 4 (or a multiple) they are the SAME 64 rows of four query heads of the group --
// all four reach their diagonal in the same tile, where 256 consecutive rows of one head reach it one
// tile after the other and leave SIMDs idle for 1.5 tiles per work group (2.3 % of a launch at 8192
// positions); a group of 2 gives two heads x 128 rows, a single head 256 consecutive rows.
// One wave per SIMD holds ~400 registers: O^T and Q^T in AGPRs, two S^T and two P^T buffers in
// VGPRs.  K/V tiles of 64 keys travel from HBM straight into a ring of four LDS stages
// (buffer_load ... lds), requested almost two tiles before their first use.  The instruction
// stream of the loop (which MFMA, which vector instruction, which LDS read goes where) is written
// by gen_prefill_pipe.py and included below; this file only prepares its scalar operands.
//
// Buffer loads with a per-(slot, sequence, kv head) resource descriptor fetch K and V: the
// hardware clamps any offset outside the sequence's region to a zero read, so even a wrong offset
// cannot touch foreign memory.  Offsets are 32-bit, hence the 4 GiB limit in pipe_supported().
#include "skv_internal.h"

#include "prefill_pipe_body_nq2.inc"
#include "prefill_pipe_body_nq2_paged.inc"

namespace skv {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kD = 128;

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

template <bool BF16, int NQ, bool PAGED>
__global__ __launch_bounds__(512 / NQ, 1) void prefill_pipe_kernel(AttnArgs a, int G, int gh, int n_qt, int n_pairs, int xcd_map) {
    static_assert(SKV_PIPE2_THREADS == 256 && SKV_PIPE2P_THREADS == 256 && SKV_PIPE2P_LDS_BYTES == SKV_PIPE2_LDS_BYTES);
    __shared__ __attribute__((aligned(16))) char lds[SKV_PIPE2_LDS_BYTES];
    constexpr int kRowsPerWave = 32 * NQ;

    const int hkv = a.cache.n_kv_heads;
    // A work group takes gh heads of the group (gh = 4, 2 or 1 divides G) x 256 / gh rows: wave w owns
    // head w % gh of them and the 64 rows of row block w / gh.
    // A work group walks PAIRS of query tiles one after the other, tile u from the end and tile u from
    // the start: under the causal mask their key tiles add up to the same number for every u, so all
    // work groups of a launch are equally long, and starting a work group costs a compute unit about
    // 1.6 us.  n_pairs pairs per work group: u = u0, u0 + n_half / n_pairs, ...
    // block -> (pair of query tiles, heads, sequence); with xcd_map the heads of a kv head and
    // neighbouring query tiles land on one XCD and share its L2
    const int wave = (int)uni(threadIdx.x >> 6);
    const int rows_per_group = 256 / gh;
    const int hg = G / gh; // sets of gh heads per kv head
    const int n_half = (n_qt + 1) / 2;
    const int n_u0 = n_half / n_pairs; // n_pairs divides n_half (launcher)
    int u0, hset, kvh, b;
    {
        const int id = blockIdx.x;
        int pair, rem;
        if (xcd_map) {
            const int per_pair = hg * n_u0;
            const int k = id >> 3;
            pair = (id & 7) + 8 * (k / per_pair);
            rem = k % per_pair;
        } else {
            pair = id / (hg * n_u0);
            rem = id % (hg * n_u0);
        }
        u0 = rem / hg;
        hset = rem % hg;
        kvh = pair % hkv;
        b = pair / hkv;
    }
    const int head = kvh * G + hset * gh + wave % gh;

    const int nq = a.q_lens[b];
    const int n = a.kv_lens[b];
    if (nq < 0 || nq > a.max_q || n < 1 || n > a.max_kv_len || nq > n) {
        if (threadIdx.x == 0 && u0 == 0 && kvh == 0 && hset == 0) atomicOr(a.cache.faults, (uint32_t)SKV_FAULT_KV_LEN);
        return; // nothing is written for a sequence with impossible lengths
    }
    bool first = true;
    for (int pass = 0; pass < 2 * n_pairs; ++pass) {
    const int u = u0 + (pass >> 1) * n_u0;
    const int qt = (pass & 1) == 0 ? n_qt - 1 - u : u;
    if ((pass & 1) == 1 && u >= n_qt - 1 - u) continue; // an odd count: the middle tile was the pass before
    const int q_begin = qt * rows_per_group;
    if (q_begin >= nq) continue;
    if (!first) __syncthreads(); // every wave has left the last tile's LDS stages (its K/V requests have landed; output stores may still be on their way)
    first = false;
    const int offset = n - nq;
    const int q_last = min(q_begin + rows_per_group, nq) - 1;
    const int n_keys = offset + q_last + 1; // keys the work group needs
    const int n_tiles = (n_keys + 63) >> 6;

    const int r0 = q_begin + kRowsPerWave * (wave / gh);
    const int rows_valid = nq - r0;
    const bool active = rows_valid > 0;
    const int p0 = offset + r0;
    const int p1 = offset + min(r0 + kRowsPerWave - 1, nq - 1);
    const int tw_last = active ? (p1 >> 6) : -1; // last tile this wave computes on
    const int t_mask = active ? ((p0 + 1) >> 6) : 0; // first tile that touches its diagonal

    const int64_t row_bytes = (int64_t)hkv * kD * 2;
    // contiguous: the descriptor covers this sequence's region of the slot; paged: the whole slot
    // (rows are found through the block table), from this kv head's first byte on
    const int64_t seq_rows = PAGED ? 0 : (int64_t)b * a.cache.max_ctx;
    const int64_t rows_covered = PAGED ? ((int64_t)a.cache.n_blocks << a.cache.block_shift) : a.cache.max_ctx;
    const char *kbase = (const char *)a.cache.k + (seq_rows * hkv + kvh) * (kD * 2);
    const char *vbase = (const char *)a.cache.v + (seq_rows * hkv + kvh) * (kD * 2);
    const uint32_t span = (uint32_t)(rows_covered * row_bytes - (int64_t)kvh * (kD * 2));
    const int32_t *tbl = PAGED ? a.cache.block_table + (int64_t)b * a.cache.max_blocks_per_seq : nullptr;
    const u32x4 srdk = make_srd(kbase, span);
    const u32x4 srdv = make_srd(vbase, span);

    const int q_row = active ? r0 : q_begin; // an idle wave still loads (and ignores) valid rows
    const int64_t qo = (((int64_t)b * a.max_q + q_row) * a.n_q_heads + head) * kD * 2;
    const char *qp = (const char *)a.q + qo;
    char *op = (char *)a.out + qo;
    const float *lsep = a.lse != nullptr ? a.lse + ((int64_t)b * a.n_q_heads + head) * a.max_q + q_row : nullptr;
    const uint32_t q_row_stride = (uint32_t)a.n_q_heads * kD * 2;
    const uint32_t rv_clamp = active ? (uint32_t)min(rows_valid, kRowsPerWave) : 1u;
    const float cs = a.scale_log2e;
    const float thr = fminf(8.0f / cs, 3.0e38f); // finite: the first tile (maximum -inf so far) must pass it

    const uint32_t lds_base = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char *)lds);
    const uint32_t tid = threadIdx.x;

#define SKV_PIPE_OPERANDS                                                                              \
    [srdk] "s"(srdk), [srdv] "s"(srdv), [qp] "s"(qp), [op] "s"(op), [lsep] "s"(lsep), [lds] "s"(uni(lds_base)),         \
        [qrs] "s"(uni(q_row_stride)), [rv] "s"(uni(rv_clamp)), [rvs] "s"(uni((uint32_t)rows_valid)),   \
        [krb] "s"(uni((uint32_t)row_bytes)), [nk1] "s"(uni((uint32_t)(n_keys - 1))),                   \
        [nt] "s"(uni((uint32_t)n_tiles)), [tms] "s"(uni((uint32_t)t_mask)),                            \
        [twl] "s"(uni((uint32_t)tw_last)), [p0] "s"(uni((uint32_t)p0)),                                \
        [cs] "s"(uni(__builtin_bit_cast(uint32_t, cs))), [thr] "s"(uni(__builtin_bit_cast(uint32_t, thr))), \
        [wv] "s"(uni((uint32_t)wave)), [tid] "v"(tid), [tbl] "s"(tbl), [flt] "s"(a.cache.faults),                \
        [shift] "s"(uni((uint32_t)a.cache.block_shift)), [bsm1] "s"(uni((1u << a.cache.block_shift) - 1u)),           \
        [nblk] "s"(uni((uint32_t)a.cache.n_blocks))

#define SKV_PIPE_RUN(TAG)                                                                              \
    if constexpr (BF16) {                                                                              \
        asm volatile(SKV_PIPE##TAG##_ASM_BF16 : : SKV_PIPE_OPERANDS : SKV_PIPE##TAG##_CLOBBERS);      \
    } else {                                                                                           \
        asm volatile(SKV_PIPE##TAG##_ASM_F16 : : SKV_PIPE_OPERANDS : SKV_PIPE##TAG##_CLOBBERS);       \
    }
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
    static_assert(NQ == 2);
    if constexpr (!PAGED) {
        SKV_PIPE_RUN(2)
    } else {
        SKV_PIPE_RUN(2P)
    }
#pragma clang diagnostic pop
#undef SKV_PIPE_RUN
#undef SKV_PIPE_OPERANDS
    } // pass
}

} // namespace

bool prefill_pipe_supported(const AttnArgs &a, int dtype, int head_dim) {
    if (!(dtype == SKV_BF16 || dtype == SKV_F16) || head_dim != kD) return false;
    // 32-bit byte offsets inside one sequence's region of the slot (paged: inside the whole slot, plus
    // one block, the offset an invalid block id is turned into), 24-bit multiplier operands
    const int64_t row_bytes = (int64_t)a.cache.n_kv_heads * kD * 2;
    if (row_bytes >= (1 << 24) || a.cache.max_ctx >= (1 << 24)) return false;
    if (a.cache.block_table != nullptr) {
        // a wave stages 16 (8) consecutive positions per tile: they must lie in one block
        if (a.cache.block_shift < 4) return false;
        const int64_t rows = ((int64_t)a.cache.n_blocks + 1) << a.cache.block_shift;
        return rows < (1 << 24) && rows * row_bytes < ((int64_t)1 << 32) && (int64_t)a.n_q_heads * kD * 2 < (1 << 24);
    }
    if ((int64_t)a.cache.max_ctx * row_bytes >= ((int64_t)1 << 32)) return false;
    if ((int64_t)a.n_q_heads * kD * 2 >= (1 << 24)) return false;
    return true;
}

hipError_t launch_prefill_pipe(const AttnArgs &a, int dtype, int group, hipStream_t stream) {
    const int gh = group % 4 == 0 ? 4 : group % 2 == 0 ? 2 : 1; // heads of the group that share a work group
    const int rows_per_group = 256 / gh;
    const int n_qt = (a.max_q + rows_per_group - 1) / rows_per_group;
    const int pairs = a.batch * a.cache.n_kv_heads;
    // pairs of query tiles per work group: as many as leave four work groups per compute unit
    const int n_half = (n_qt + 1) / 2;
    int n_pairs = 1;
#ifdef SKV_PIPE_PAIRS
    n_pairs = SKV_PIPE_PAIRS;
#else
    while (n_half % (2 * n_pairs) == 0 && (int64_t)pairs * (group / gh) * (n_half / (2 * n_pairs)) >= 4 * 256) n_pairs *= 2;
#endif
    const int64_t blocks = (int64_t)pairs * (group / gh) * (n_half / n_pairs);
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    const int xcd_map = (pairs % 8) == 0;
    const dim3 grid((unsigned)blocks);
    const bool paged = a.cache.block_table != nullptr;
#define SKV_PIPE_LAUNCH(BF, NQ_, PG) prefill_pipe_kernel<BF, NQ_, PG><<<grid, 512 / NQ_, 0, stream>>>(a, group, gh, n_qt, n_pairs, xcd_map)
    if (dtype == SKV_BF16) { if (paged) SKV_PIPE_LAUNCH(true, 2, true); else SKV_PIPE_LAUNCH(true, 2, false); }
    else { if (paged) SKV_PIPE_LAUNCH(false, 2, true); else SKV_PIPE_LAUNCH(false, 2, false); }
#undef SKV_PIPE_LAUNCH
    set_last_kernel_name("prefill_pipe_kernel");
    return hipGetLastError();
}

} // namespace skv
