// Routed attention on the vector ALUs (paper Eq. (3.1): Output_l = Attn(Q_l, K_l', V_l')),
// for any dtype.  It is the fp32 path and covers the shapes the MFMA kernels do not.
//
// One wavefront owns one work item = (query row, kv head, key-axis split) and serves all G query
// heads of the kv head from a single read of each K/V row.  A key row of D elements is spread
// over LPR = D*sizeof(T)/16 lanes, 16 bytes per lane, so one wave-wide load fetches 64/LPR whole
// rows with fully coalesced 128-bit accesses.  Every group of LPR lanes runs its own online
// softmax over the keys it sees; the groups (and, in a second launch, the splits) are merged
// with the usual max / rescale / sum rule.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "skv_internal.h"

namespace skv {

namespace {

struct F32 { using storage = float; static constexpr int kBytes = 4; };
struct F16 { using storage = uint16_t; static constexpr int kBytes = 2; };
struct BF16 { using storage = uint16_t; static constexpr int kBytes = 2; };

template <typename T> struct Conv;
template <> struct Conv<F32> {
    static constexpr int EPL = 4; // elements per 16-byte piece
    __device__ static void unpack(const uint4 &r, float *f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
    __device__ static uint4 pack(const float *f) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
};
template <> struct Conv<BF16> {
    static constexpr int EPL = 8;
    __device__ static void unpack(const uint4 &r, float *f) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static uint32_t rne(float x) { // float -> bf16 bits, round to nearest even
        uint32_t u = __float_as_uint(x);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u; // NaN stays NaN
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    __device__ static uint4 pack(const float *f) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = rne(f[2 * i]) | (rne(f[2 * i + 1]) << 16);
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};
template <> struct Conv<F16> {
    static constexpr int EPL = 8;
    __device__ static void unpack(const uint4 &r, float *f) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __half2float(__ushort_as_half((unsigned short)(w[i] & 0xffffu)));
            f[2 * i + 1] = __half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
        }
    }
    __device__ static uint4 pack(const float *f) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = (uint32_t)__half_as_ushort(__float2half_rn(f[2 * i])) |
                   ((uint32_t)__half_as_ushort(__float2half_rn(f[2 * i + 1])) << 16);
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};

constexpr int kWavesPerBlock = 4;

template <typename T, int D, int G>
__global__ __launch_bounds__(64 * kWavesPerBlock) void attn_valu_kernel(AttnArgs a) {
    constexpr int EPL = Conv<T>::EPL;
    constexpr int LPR = D / EPL;  // lanes per key row
    constexpr int KPW = 64 / LPR; // key rows per wave-wide load
    static_assert(LPR >= 1 && LPR <= 64 && (LPR & (LPR - 1)) == 0, "row must fit a wave");

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int hkv = a.cache.n_kv_heads;
    const int64_t item = (int64_t)blockIdx.x * kWavesPerBlock + wave;
    const int64_t n_items = (int64_t)a.batch * a.max_q * hkv * a.n_splits;
    if (item >= n_items) return;
    const int split = (int)(item % a.n_splits);
    const int kvh = (int)((item / a.n_splits) % hkv);
    const int64_t row = item / ((int64_t)a.n_splits * hkv); // (b, i)
    const int i = (int)(row % a.max_q);
    const int b = (int)(row / a.max_q);

    int kv_end = a.kv_lens[b];
    bool bad = kv_end < 1 || kv_end > a.max_kv_len;
    if (a.q_lens != nullptr) {
        const int nq = a.q_lens[b];
        if (nq < 0 || nq > a.max_q || nq > kv_end) bad = true;
        if (!bad && i >= nq) return; // padding row: neither read nor written
        kv_end = kv_end - nq + i + 1;
    }
    const int grp = lane / LPR;
    const int li = lane % LPR;
    const int e0 = li * EPL;
    const int head0 = kvh * G;
    const int64_t q_base = (row * a.n_q_heads + head0) * D + e0;

    if (bad) { // lengths the host promised not to pass: define the output, record the fault
        if (lane == 0 && split == 0 && kvh == 0) atomicOr(a.cache.faults, (uint32_t)SKV_FAULT_KV_LEN);
        // decode: the sequence's output row is zeroed; pre-fill: nothing is written (as in the MFMA kernels)
        if (split == 0 && grp == 0 && a.q_lens == nullptr) {
            float z[EPL] = {};
#pragma unroll
            for (int h = 0; h < G; ++h)
                *(uint4 *)((typename T::storage *)a.out + q_base + (int64_t)h * D) = Conv<T>::pack(z);
        }
        return;
    }

    const int k_begin = split * a.keys_per_split;
    const int k_end = min(kv_end, k_begin + a.keys_per_split);
    if (k_begin >= k_end) return; // this split holds no key of this row; the merge never reads it

    float qf[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const uint4 raw = *(const uint4 *)((const typename T::storage *)a.q + q_base + (int64_t)h * D);
        Conv<T>::unpack(raw, qf[h]);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qf[h][e] *= a.scale_log2e;
    }

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = -INFINITY;
        l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;
    }

    const typename T::storage *kp = (const typename T::storage *)a.cache.k;
    const typename T::storage *vp = (const typename T::storage *)a.cache.v;
    const int64_t head_off = (int64_t)kvh * D + e0;
    const int64_t row_elems = (int64_t)hkv * D;

    for (int j0 = k_begin; j0 < k_end; j0 += KPW) {
        const int j = j0 + grp;
        bool valid = j < k_end;
        int64_t r = valid ? slot_row(a.cache, b, j) : 0;
        if (r < 0) { // block id outside the pool: the key is skipped and the fault recorded
            if (li == 0) atomicOr(a.cache.faults, (uint32_t)SKV_FAULT_BLOCK_ID);
            valid = false;
            r = 0;
        }
        uint4 kraw = make_uint4(0, 0, 0, 0), vraw = make_uint4(0, 0, 0, 0);
        if (valid) {
            kraw = *(const uint4 *)(kp + r * row_elems + head_off);
            vraw = *(const uint4 *)(vp + r * row_elems + head_off);
        }
        float kf[EPL], vf[EPL];
        Conv<T>::unpack(kraw, kf);
        Conv<T>::unpack(vraw, vf);
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) s = fmaf(qf[h][e], kf[e], s);
#pragma unroll
            for (int mask = 1; mask < LPR; mask <<= 1) s += __shfl_xor(s, mask, 64);
            if (valid) { // s is in log2 units: weights are 2^(s - m)
                const float m_new = fmaxf(m[h], s);
                const float alpha = exp2f(m[h] - m_new); // 0 on the first key (m = -inf)
                const float p = exp2f(s - m_new);
                l[h] = l[h] * alpha + p;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[h][e] = fmaf(acc[h][e], alpha, p * vf[e]);
                m[h] = m_new;
            }
        }
    }

    // merge the KPW lane groups of the wave
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
        for (int mask = LPR; mask < 64; mask <<= 1) {
            const float m_o = __shfl_xor(m[h], mask, 64);
            const float l_o = __shfl_xor(l[h], mask, 64);
            const float m_new = fmaxf(m[h], m_o);
            const float sa = m[h] == -INFINITY ? 0.f : exp2f(m[h] - m_new);
            const float sb = m_o == -INFINITY ? 0.f : exp2f(m_o - m_new);
            l[h] = l[h] * sa + l_o * sb;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float a_o = __shfl_xor(acc[h][e], mask, 64);
                acc[h][e] = acc[h][e] * sa + a_o * sb;
            }
            m[h] = m_new;
        }
    }

    if (grp != 0) return;
    if ((kv_end + a.keys_per_split - 1) / a.keys_per_split == 1) { // the row fits one split: final result
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float inv = 1.f / l[h];
            float o[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[e] = acc[h][e] * inv;
            *(uint4 *)((typename T::storage *)a.out + q_base + (int64_t)h * D) = Conv<T>::pack(o);
        }
    } else {
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const int64_t p = (row * a.n_q_heads + head0 + h) * a.n_splits + split;
            float *po = a.part_o + p * D + e0;
#pragma unroll
            for (int e = 0; e < EPL; e += 4)
                *(float4 *)(po + e) = make_float4(acc[h][e], acc[h][e + 1], acc[h][e + 2], acc[h][e + 3]);
            if (li == 0) {
                a.part_ml[p * 2] = m[h];
                a.part_ml[p * 2 + 1] = l[h];
            }
        }
    }
}

// Split merge: out = sum_s o_s 2^(m_s - m) / sum_s l_s 2^(m_s - m), m = max_s m_s, over the
// splits that hold at least one key of the row.  One work group per (row, head): D / 4 lanes cover
// the output, the 256 / (D / 4) lane groups share the splits (a sequence of 32768 keys has up to
// 128 of them: one thread walking them all made this launch as long as the attention launch of a
// single sequence) and add up through LDS.
template <typename T>
__global__ __launch_bounds__(256) void split_merge_kernel(AttnArgs a, int D) {
    __shared__ float s_m[16], s_l[16];
    __shared__ __attribute__((aligned(16))) float s_o[1024];
    const int quads = D / 4;            // 16, 32 or 64 lanes per group
    const int ng = 256 / quads;         // 16, 8 or 4 groups
    const int qd = threadIdx.x % quads, sg = threadIdx.x / quads;
    const int64_t rh = blockIdx.x;      // row * n_q_heads + head   (decode: row = sequence)
    const int b = (int)(rh / a.n_q_heads);
    int sink, gap;
    const int kv_end = a.max_q == 1 ? decode_keys(a, b, sink, gap) : a.kv_lens[b];
    if (kv_end < 1 || kv_end > a.max_kv_len) return; // the attention kernel wrote zeros
    const int ns = (kv_end + a.keys_per_split - 1) / a.keys_per_split;
    if (ns == 1) return; // the attention kernel already wrote the final result
    const float *ml = a.part_ml + rh * a.n_splits * 2;
    float m = -INFINITY;
    for (int s = sg; s < ns; s += ng) m = fmaxf(m, ml[2 * s]);
    if (qd == 0) s_m[sg] = m;
    __syncthreads();
    m = s_m[0];
    for (int g = 1; g < ng; ++g) m = fmaxf(m, s_m[g]);
    float l = 0.f, o[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s = sg; s < ns; s += ng) {
        const float w = exp2f(ml[2 * s] - m);
        l += ml[2 * s + 1] * w;
        const float4 p = *(const float4 *)(a.part_o + (rh * a.n_splits + s) * D + qd * 4);
        o[0] += p.x * w; o[1] += p.y * w; o[2] += p.z * w; o[3] += p.w * w;
    }
    if (qd == 0) s_l[sg] = l;
    *(float4 *)(s_o + sg * D + qd * 4) = make_float4(o[0], o[1], o[2], o[3]);
    __syncthreads();
    if (sg != 0) return;
    for (int g = 1; g < ng; ++g) { // fixed order: the result does not depend on timing
        l += s_l[g];
        const float4 p = *(const float4 *)(s_o + g * D + qd * 4);
        o[0] += p.x; o[1] += p.y; o[2] += p.z; o[3] += p.w;
    }
    const float inv = 1.f / l;
    typename T::storage *dst = (typename T::storage *)a.out + rh * D + qd * 4;
    if constexpr (T::kBytes == 4) {
        *(float4 *)dst = make_float4(o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv);
    } else {
        float f[8] = {o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv, 0.f, 0.f, 0.f, 0.f};
        const uint4 w = Conv<T>::pack(f);
        *(uint2 *)dst = make_uint2(w.x, w.y);
    }
}

template <typename T, int D>
hipError_t launch_valu_dg(const AttnArgs &a, int group, hipStream_t stream) {
    const int64_t items = (int64_t)a.batch * a.max_q * a.cache.n_kv_heads * a.n_splits;
    const int64_t blocks = (items + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(64 * kWavesPerBlock);
    switch (group) {
    case 1: attn_valu_kernel<T, D, 1><<<grid, block, 0, stream>>>(a); break;
    case 2: attn_valu_kernel<T, D, 2><<<grid, block, 0, stream>>>(a); break;
    case 4: attn_valu_kernel<T, D, 4><<<grid, block, 0, stream>>>(a); break;
    case 8: attn_valu_kernel<T, D, 8><<<grid, block, 0, stream>>>(a); break;
    case 16: attn_valu_kernel<T, D, 16><<<grid, block, 0, stream>>>(a); break;
    default: return hipErrorInvalidValue;
    }
    set_last_kernel_name("attn_valu_kernel");
    return hipGetLastError();
}

template <typename T>
hipError_t launch_valu_d(const AttnArgs &a, int head_dim, int group, hipStream_t stream) {
    switch (head_dim) {
    case 64: return launch_valu_dg<T, 64>(a, group, stream);
    case 128: return launch_valu_dg<T, 128>(a, group, stream);
    case 256: return launch_valu_dg<T, 256>(a, group, stream);
    default: return hipErrorInvalidValue;
    }
}

} // namespace

hipError_t launch_attn_valu(const AttnArgs &a, int dtype, int head_dim, int group, hipStream_t stream) {
    switch (dtype) {
    case SKV_F32: return launch_valu_d<F32>(a, head_dim, group, stream);
    case SKV_F16: return launch_valu_d<F16>(a, head_dim, group, stream);
    case SKV_BF16: return launch_valu_d<BF16>(a, head_dim, group, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_split_merge(const AttnArgs &a, int dtype, hipStream_t stream) {
    const int D = a.cache.head_dim;
    const int64_t total = (int64_t)a.batch * a.max_q * a.n_q_heads; // one work group per (row, head)
    if (total > 0x7fffffff || !(D == 64 || D == 128 || D == 256)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)total), block(256);
    switch (dtype) {
    case SKV_F32: split_merge_kernel<F32><<<grid, block, 0, stream>>>(a, D); break;
    case SKV_F16: split_merge_kernel<F16><<<grid, block, 0, stream>>>(a, D); break;
    case SKV_BF16: split_merge_kernel<BF16><<<grid, block, 0, stream>>>(a, D); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace skv
