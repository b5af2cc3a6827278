// C ABI of libskv: validation, route -> slot map, sizing, launch configuration.
// Every entry point is documented in include/skv.h; nothing here computes attention on the host.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "skv_internal.h"

struct skv_cache {
    skv_cache_desc_t d;          // route pointer inside is not used after alloc
    std::vector<int32_t> route;  // host copy
    std::vector<int32_t> slot;   // slot_of_layer
    int32_t n_slots = 0;
    void *k_pool = nullptr, *v_pool = nullptr, *scale_pool = nullptr;
    bool owns_pools = false;
    size_t pool_bytes_each = 0;
    size_t scale_pool_bytes = 0; // 8-bit slots: uint16 per (row, kv head), all slots
    size_t slot_bytes = 0;       // bytes of one slot inside a pool
    const int32_t *block_table = nullptr;
    const int32_t *evict_sink = nullptr, *evict_first = nullptr; // borrowed device arrays, both or neither
    int32_t max_blocks_per_seq = 0;
    int32_t block_shift = 0;
    uint32_t *faults = nullptr;  // device word
};

namespace {

thread_local int32_t g_last_hip_error = 0;
thread_local const char *g_last_kernel = "";

skv_status_t hip_fail(hipError_t e) {
    g_last_hip_error = (int32_t)e;
    (void)hipGetLastError(); // clear the sticky per-thread error
    return e == hipErrorOutOfMemory ? SKV_ERR_OOM : SKV_ERR_HIP;
}

// Pre-fill kernel choice: pipelined -> plain MFMA -> vector ALU.
skv_status_t launch_prefill(const skv::AttnArgs &a, int dtype, int head_dim, int g, hipStream_t stream) {
    hipError_t e;
    if (skv::dtype_kv8(dtype)) // 8-bit slots: the kernel that stages tiles through registers converts on the way
        e = skv::launch_prefill_mfma(a, dtype, head_dim, g, stream);
    else if (!skv::tuning().prefill_plain && skv::prefill_pipe_supported(a, dtype, head_dim))
        e = skv::launch_prefill_pipe(a, dtype, g, stream);
    else if (skv::prefill_mfma_supported(dtype, head_dim, g))
        e = skv::launch_prefill_mfma(a, dtype, head_dim, g, stream);
    else
        e = skv::launch_attn_valu(a, dtype, head_dim, g, stream);
    return e == hipSuccess ? SKV_OK : hip_fail(e);
}

int elem_bytes(int dtype) { return dtype == SKV_F32 ? 4 : skv::dtype_kv8(dtype) ? 1 : 2; } // of a slot element

int ilog2_exact(int v) {
    for (int s = 0; s < 31; ++s)
        if ((1 << s) == v) return s;
    return -1;
}

skv_status_t check_desc(const skv_cache_desc_t *d, int32_t *n_slots, std::vector<int32_t> *slot) {
    if (!d || !d->route) return SKV_ERR_INVALID_ARG;
    if (d->n_layers <= 0 || d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->batch <= 0 || d->max_ctx <= 0)
        return SKV_ERR_INVALID_ARG;
    if (d->dtype < SKV_F32 || d->dtype > SKV_F16_KV8) return SKV_ERR_UNSUPPORTED;
    if (d->head_dim != 64 && d->head_dim != 128 && d->head_dim != 256) return SKV_ERR_UNSUPPORTED;
    if (skv::dtype_kv8(d->dtype) && d->head_dim == 256) return SKV_ERR_UNSUPPORTED;
    if (d->n_q_heads % d->n_kv_heads) return SKV_ERR_UNSUPPORTED;
    const int g = d->n_q_heads / d->n_kv_heads;
    if (g != 1 && g != 2 && g != 4 && g != 8 && g != 16) return SKV_ERR_UNSUPPORTED;
    if (d->block_size < 0) return SKV_ERR_INVALID_ARG;
    if (d->block_size > 0) {
        if (ilog2_exact(d->block_size) < 3 || d->block_size > 256) return SKV_ERR_UNSUPPORTED;
        if (skv::dtype_kv8(d->dtype) && d->block_size < 16) return SKV_ERR_UNSUPPORTED; // a wave-wide load of codes covers 16 rows of 64
        if (d->n_blocks <= 0) return SKV_ERR_INVALID_ARG;
    }
    if ((d->k_pool == nullptr) != (d->v_pool == nullptr)) return SKV_ERR_INVALID_ARG;
    if (skv::dtype_kv8(d->dtype) && (d->k_pool == nullptr) != (d->scale_pool == nullptr)) return SKV_ERR_INVALID_ARG;
    std::vector<int32_t> tmp((size_t)d->n_layers);
    int32_t ns = 0;
    skv_status_t st = skv_route_validate(d->route, d->n_layers, tmp.data(), &ns);
    if (st != SKV_OK) return st;
    if (n_slots) *n_slots = ns;
    if (slot) slot->swap(tmp);
    return SKV_OK;
}

// 8-bit slots keep the rows of one kv head together in groups of this many consecutive rows: the
// four 32-key tiles the waves of a decode work group take side by side, or a whole block where
// blocks are smaller; 1 = row-major slot.  (Decode over the Llama-3-8B-shaped workload: groups of
// 32 / 64 / 128 rows = runs of 4 / 8 / 16 KiB per kv head: 97 / 94 / 92 us per call; row-major: 106-111.)
constexpr int kGroupRows = 128;
int group_rows_of(const skv_cache_desc_t *d) {
    if (!skv::dtype_kv8(d->dtype)) return 1;
    return d->block_size > 0 ? std::min(d->block_size, kGroupRows) : kGroupRows;
}

// rows a contiguous slot holds per sequence: whole groups
size_t seq_rows_of(const skv_cache_desc_t *d) {
    const size_t g = (size_t)group_rows_of(d);
    return ((size_t)d->max_ctx + g - 1) / g * g;
}

size_t slot_rows_of(const skv_cache_desc_t *d) {
    return d->block_size > 0 ? (size_t)d->n_blocks * d->block_size : (size_t)d->batch * seq_rows_of(d);
}

size_t slot_bytes_of(const skv_cache_desc_t *d) {
    return slot_rows_of(d) * (size_t)d->n_kv_heads * d->head_dim * elem_bytes(d->dtype);
}

// 8-bit slots: the exponent bytes of one slot (uint16 per row and kv head)
size_t slot_scale_bytes_of(const skv_cache_desc_t *d) {
    return skv::dtype_kv8(d->dtype) ? slot_rows_of(d) * (size_t)d->n_kv_heads * sizeof(uint16_t) : 0;
}

skv::SlotView view_of(const skv_cache *c, int slot) {
    skv::SlotView v;
    v.k = (const char *)c->k_pool + (size_t)slot * c->slot_bytes;
    v.v = (const char *)c->v_pool + (size_t)slot * c->slot_bytes;
    v.scales = c->scale_pool ? (const uint16_t *)((const char *)c->scale_pool + (size_t)slot * slot_scale_bytes_of(&c->d)) : nullptr;
    v.block_table = c->block_table;
    v.faults = c->faults;
    v.max_blocks_per_seq = c->max_blocks_per_seq;
    v.block_shift = c->block_shift;
    v.n_blocks = c->d.n_blocks;
    v.max_ctx = c->d.block_size > 0
                    ? (int32_t)std::min<int64_t>((int64_t)c->max_blocks_per_seq << c->block_shift, INT32_MAX)
                    : c->d.max_ctx;
    v.seq_rows = (int32_t)seq_rows_of(&c->d);
    v.group_shift = ilog2_exact(group_rows_of(&c->d));
    v.n_kv_heads = c->d.n_kv_heads;
    v.head_dim = c->d.head_dim;
    return v;
}

// Key-axis chunk covered by one work item of the decode kernels.  Deterministic in
// (batch, n_kv_heads, max_kv_len) so that the workspace size and the launch agree.
constexpr int64_t kMaxKeysPerSplit = 4096;
// Distance of a library-owned V pool from its K pool, modulo 1 KiB (see skv_cache_alloc).
constexpr size_t kPoolSkew = 384;
// The workspace of a decode call starts with the work counters of the persistent launch shape.
constexpr size_t kCounterBytes = 256;

int32_t decode_keys_per_split(const skv_cache *c, int32_t n_seqs, int32_t max_kv_len) {
    if (const int forced = skv::tuning().decode_keys_per_split) return forced;
    // About one work group per compute unit (256) when every sequence is max_kv_len long, within
    // 256..2048 keys.  Measured on the Llama-3-8B decode shape (4096 keys, 8 kv heads): with two
    // tiles per wave in flight the kernel gains from long splits (fewer pipeline fills, partial
    // results and merges); for 4..32 sequences 256 work groups beat 512 and 1024 by 10-40 %, and
    // from 64 sequences on the 2048-key cap (1024 equal work groups, four per CU) is the optimum.
    const int64_t units = (int64_t)n_seqs * c->d.n_kv_heads;
    int64_t kps = (int64_t)max_kv_len * units / 256;
    kps = ((kps + 255) / 256) * 256;
    // A 4096-key split only where it covers the whole sequence (one work item per sequence and
    // kv head, no partial results, no merge launch: +1 % on 64 x 4096 keys); with longer or ragged
    // sequences 2048-key items balance better (paged ragged batch: 5.85 vs 5.6 TB/s).
    const int64_t cap = max_kv_len <= kMaxKeysPerSplit ? kMaxKeysPerSplit : kMaxKeysPerSplit / 2;
    return (int32_t)std::min<int64_t>(cap, std::max<int64_t>(256, kps));
}

bool paged_ready(const skv_cache *c) { return c->d.block_size == 0 || c->block_table != nullptr; }

} // namespace

namespace skv {
void set_last_kernel_name(const char *name) { g_last_kernel = name; }

// Developer knobs for A/B timing.  The environment is read ONCE, at the first call that asks, and
// only if it holds SKV_TUNING=1; without that the defaults below are what runs.
//   SKV_DECODE_KEYS_PER_SPLIT=<multiple of 128>  key-axis chunk of the decode kernel
//   SKV_DECODE_LOADS=nt|cached                   cache policy of the decode kernel's K/V loads
//   SKV_PREFILL_KERNEL=plain                     keep the pipelined pre-fill kernel out
//   SKV_PROJECT_KERNEL=wide                      keep the tile projection kernel out
//   SKV_PROJECT_SPLITS=<power of two>            hidden-axis splits of the projection
const Tuning &tuning() {
    static const Tuning t = [] {
        Tuning r;
        const char *on = getenv("SKV_TUNING");
        if (on == nullptr || strcmp(on, "1") != 0) return r;
        if (const char *e = getenv("SKV_DECODE_KEYS_PER_SPLIT")) {
            const int v = atoi(e);
            if (v > 0 && v % 128 == 0) r.decode_keys_per_split = v;
        }
        if (const char *e = getenv("SKV_DECODE_LOADS")) r.decode_loads = strcmp(e, "nt") == 0 ? 1 : strcmp(e, "cached") == 0 ? 2 : 0;
        if (const char *e = getenv("SKV_PREFILL_KERNEL")) r.prefill_plain = strcmp(e, "plain") == 0;
        if (const char *e = getenv("SKV_PROJECT_KERNEL")) r.project_wide = strcmp(e, "wide") == 0;
        if (const char *e = getenv("SKV_PROJECT_SPLITS")) r.project_splits = atoi(e);
        return r;
    }();
    return t;
}
} // namespace skv

extern "C" {

skv_status_t skv_route_from_strategy(const int32_t *owners, int32_t n_owners, int32_t n_layers,
                                     int32_t *route_out) {
    if (!owners || !route_out || n_layers <= 0 || n_owners <= 0) return SKV_ERR_INVALID_ARG;
    std::vector<char> is_owner((size_t)n_layers, 0);
    for (int i = 0; i < n_owners; ++i) {
        if (owners[i] < 0 || owners[i] >= n_layers || is_owner[owners[i]]) return SKV_ERR_BAD_ROUTE;
        is_owner[owners[i]] = 1;
    }
    if (!is_owner[0]) return SKV_ERR_BAD_ROUTE;
    int32_t last = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (is_owner[l]) last = l;
        route_out[l] = last;
    }
    return SKV_OK;
}

skv_status_t skv_route_validate(const int32_t *route, int32_t n_layers, int32_t *slot_of_layer,
                                int32_t *n_slots) {
    if (!route || n_layers <= 0) return SKV_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l) {
        const int32_t r = route[l];
        if (r < 0 || r > l) return SKV_ERR_BAD_ROUTE;
        if (route[r] != r) return SKV_ERR_BAD_ROUTE;
    }
    std::vector<int32_t> rank((size_t)n_layers, -1);
    int32_t ns = 0;
    for (int l = 0; l < n_layers; ++l)
        if (route[l] == l) rank[l] = ns++;
    if (slot_of_layer)
        for (int l = 0; l < n_layers; ++l) slot_of_layer[l] = rank[route[l]];
    if (n_slots) *n_slots = ns;
    return SKV_OK;
}

skv_status_t skv_cache_bytes(const skv_cache_desc_t *desc, size_t *total_bytes) {
    if (!total_bytes) return SKV_ERR_INVALID_ARG;
    int32_t ns = 0;
    skv_status_t st = check_desc(desc, &ns, nullptr);
    if (st != SKV_OK) return st;
    *total_bytes = (size_t)ns * (2 * slot_bytes_of(desc) + slot_scale_bytes_of(desc));
    return SKV_OK;
}

skv_status_t skv_cache_pool_bytes(const skv_cache_desc_t *desc, size_t *kv_pool_bytes, size_t *scale_pool_bytes) {
    int32_t ns = 0;
    skv_status_t st = check_desc(desc, &ns, nullptr);
    if (st != SKV_OK) return st;
    if (kv_pool_bytes) *kv_pool_bytes = (size_t)ns * slot_bytes_of(desc);
    if (scale_pool_bytes) *scale_pool_bytes = (size_t)ns * slot_scale_bytes_of(desc);
    return SKV_OK;
}

skv_status_t skv_cache_alloc(const skv_cache_desc_t *desc, skv_cache_t **out) {
    if (!out) return SKV_ERR_INVALID_ARG;
    int32_t ns = 0;
    std::vector<int32_t> slot;
    skv_status_t st = check_desc(desc, &ns, &slot);
    if (st != SKV_OK) return st;
    const size_t each = (size_t)ns * slot_bytes_of(desc);
    const size_t scale_bytes = (size_t)ns * slot_scale_bytes_of(desc);
    if (desc->k_pool && desc->pool_bytes < each) return SKV_ERR_CAPACITY;
    if (desc->k_pool && desc->scale_pool_bytes < scale_bytes) return SKV_ERR_CAPACITY;

    skv_cache *c = new (std::nothrow) skv_cache();
    if (!c) return SKV_ERR_OOM;
    c->d = *desc;
    c->route.assign(desc->route, desc->route + desc->n_layers);
    c->d.route = nullptr;
    c->slot.swap(slot);
    c->n_slots = ns;
    c->pool_bytes_each = each;
    c->scale_pool_bytes = scale_bytes;
    c->slot_bytes = slot_bytes_of(desc);
    c->block_shift = desc->block_size > 0 ? ilog2_exact(desc->block_size) : 0;

    hipError_t e = hipMalloc((void **)&c->faults, 256);
    if (e == hipSuccess) e = hipMemset(c->faults, 0, 256);
    if (e != hipSuccess) {
        if (c->faults) (void)hipFree(c->faults);
        delete c;
        return hip_fail(e);
    }
    if (desc->k_pool) {
        c->k_pool = desc->k_pool;
        c->v_pool = desc->v_pool;
        c->scale_pool = scale_bytes ? desc->scale_pool : nullptr;
    } else {
        c->owns_pools = true;
        // One allocation, the V pool kPoolSkew bytes past a multiple of 1 KiB behind the start of the K pool.
        // The decode kernel streams the K and the V rows of the same positions at the same time; when the
        // two pools are a multiple of 1 KiB apart (separate allocations are: both start on a 2 MiB boundary)
        // the two streams meet in the same memory channels.  Measured on 64 sequences x 4096 positions, 8
        // kv heads x 128, bf16: 173 us per call at distance = 0 mod 1 KiB, 161 us at 256 or 384 (171 at 128,
        // 166 at 512, 209 at 64: rows off the 128-byte lines); 32 kv heads and paged pools gain 1-1.5 % at
        // 384, 8-bit slots are indifferent.
        const size_t v_off = (each + 1023) / 1024 * 1024 + kPoolSkew;
        e = hipMalloc(&c->k_pool, v_off + each);
        if (e == hipSuccess) c->v_pool = (char *)c->k_pool + v_off;
        if (e == hipSuccess && scale_bytes) e = hipMalloc(&c->scale_pool, scale_bytes);
        if (e == hipSuccess) e = hipMemset(c->k_pool, 0, each);
        if (e == hipSuccess) e = hipMemset(c->v_pool, 0, each);
        // exponent byte 127 = scale 1: never-written rows read as zeros, not as 0 x 2^-127
        if (e == hipSuccess && scale_bytes) e = hipMemset(c->scale_pool, 127, scale_bytes);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) {
            if (c->k_pool) (void)hipFree(c->k_pool); // the V pool is part of this allocation
            if (c->scale_pool) (void)hipFree(c->scale_pool);
            (void)hipFree(c->faults);
            delete c;
            return hip_fail(e);
        }
    }
    *out = c;
    return SKV_OK;
}

skv_status_t skv_cache_free(skv_cache_t *c) {
    if (!c) return SKV_OK;
    skv_status_t st = SKV_OK;
    if (c->owns_pools) {
        hipError_t e1 = hipFree(c->k_pool); // K and V pools are one allocation
        hipError_t e3 = c->scale_pool ? hipFree(c->scale_pool) : hipSuccess;
        if (e1 != hipSuccess) st = hip_fail(e1);
        if (e3 != hipSuccess) st = hip_fail(e3);
    }
    hipError_t e = hipFree(c->faults);
    if (e != hipSuccess) st = hip_fail(e);
    delete c;
    return st;
}

skv_status_t skv_cache_info(const skv_cache_t *c, int32_t *n_slots, void **k_pool, void **v_pool,
                            size_t *pool_bytes_each) {
    if (!c) return SKV_ERR_INVALID_ARG;
    if (n_slots) *n_slots = c->n_slots;
    if (k_pool) *k_pool = c->k_pool;
    if (v_pool) *v_pool = c->v_pool;
    if (pool_bytes_each) *pool_bytes_each = c->pool_bytes_each;
    return SKV_OK;
}

skv_status_t skv_cache_scale_info(const skv_cache_t *c, void **scale_pool, size_t *scale_pool_bytes) {
    if (!c) return SKV_ERR_INVALID_ARG;
    if (scale_pool) *scale_pool = c->scale_pool;
    if (scale_pool_bytes) *scale_pool_bytes = c->scale_pool_bytes;
    return SKV_OK;
}

skv_status_t skv_cache_slot_of_layer(const skv_cache_t *c, int32_t layer, int32_t *slot, int32_t *is_owner) {
    if (!c || layer < 0 || layer >= c->d.n_layers) return SKV_ERR_INVALID_ARG;
    if (slot) *slot = c->slot[layer];
    if (is_owner) *is_owner = c->route[layer] == layer;
    return SKV_OK;
}

skv_status_t skv_cache_set_block_table(skv_cache_t *c, const int32_t *table, int32_t max_blocks_per_seq) {
    if (!c || !table || max_blocks_per_seq <= 0) return SKV_ERR_INVALID_ARG;
    if (c->d.block_size == 0) return SKV_ERR_UNSUPPORTED;
    c->block_table = table;
    c->max_blocks_per_seq = max_blocks_per_seq;
    return SKV_OK;
}

skv_status_t skv_cache_set_eviction(skv_cache_t *c, const int32_t *sink_len, const int32_t *first_pos) {
    if (!c || (sink_len == nullptr) != (first_pos == nullptr)) return SKV_ERR_INVALID_ARG;
    c->evict_sink = sink_len;
    c->evict_first = first_pos;
    return SKV_OK;
}

skv_status_t skv_cache_device_faults(skv_cache_t *c, uint32_t *faults) {
    if (!c || !faults) return SKV_ERR_INVALID_ARG;
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(faults, c->faults, sizeof(uint32_t), hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemset(c->faults, 0, sizeof(uint32_t));
    if (e != hipSuccess) return hip_fail(e);
    return SKV_OK;
}

skv_status_t skv_kv_append(skv_cache_t *c, int32_t layer, const void *k_new, const void *v_new,
                           const int32_t *start_pos, const int32_t *new_lens, int32_t max_new,
                           void *stream) {
    if (!c || !k_new || !v_new || !start_pos || !new_lens) return SKV_ERR_INVALID_ARG;
    if (layer < 0 || layer >= c->d.n_layers || max_new < 0) return SKV_ERR_INVALID_ARG;
    if (c->route[layer] != layer) return SKV_ERR_NOT_OWNER;
    if (!paged_ready(c)) return SKV_ERR_INVALID_ARG;
    if (max_new == 0) return SKV_OK;
    hipError_t e = skv::launch_append(view_of(c, c->slot[layer]), c->d.dtype, k_new, v_new, start_pos,
                                      new_lens, c->d.batch, max_new, (hipStream_t)stream);
    return e == hipSuccess ? SKV_OK : hip_fail(e);
}

skv_status_t skv_decode_range_workspace_bytes(const skv_cache_t *c, int32_t seq_count, int32_t max_kv_len,
                                              size_t *bytes) {
    if (!c || !bytes || max_kv_len <= 0 || seq_count <= 0 || seq_count > c->d.batch) return SKV_ERR_INVALID_ARG;
    // The split count of a launch is not monotone in its length hint (the split length is rounded to
    // 256 keys), so size for the most splits any hint up to max_kv_len can produce: splits are at
    // least 256 keys long, and either about 256 / (sequences x kv heads) per sequence or capped at
    // 2048 keys and more.
    const int64_t units = (int64_t)seq_count * c->d.n_kv_heads;
    const int64_t by_len = ((int64_t)max_kv_len + 255) / 256;
    const int64_t by_units = 256 / units + 2;
    const int64_t capped = ((int64_t)max_kv_len + kMaxKeysPerSplit / 2 - 1) / (kMaxKeysPerSplit / 2);
    const int32_t kps = decode_keys_per_split(c, seq_count, max_kv_len); // exact for this hint (covers the tuning knob)
    const int64_t exact = ((int64_t)max_kv_len + kps - 1) / kps;
    const size_t n_splits = (size_t)std::max({exact, capped, std::min(by_len, by_units)});
    *bytes = kCounterBytes + (size_t)seq_count * c->d.n_q_heads * n_splits * (c->d.head_dim + 2) * sizeof(float);
    return SKV_OK;
}

skv_status_t skv_kv_project_workspace_bytes(const skv_cache_t *c, int32_t max_new, int32_t hidden, size_t *bytes) {
    if (!c || !bytes || max_new < 0 || hidden < 1) return SKV_ERR_INVALID_ARG;
    if (!skv::project_append_supported(c->d.dtype, c->d.head_dim, hidden)) return SKV_ERR_UNSUPPORTED;
    *bytes = skv::project_append_workspace_bytes(c->d.n_kv_heads, c->d.head_dim, (int64_t)c->d.batch * max_new, hidden);
    return SKV_OK;
}

skv_status_t skv_kv_project_append(skv_cache_t *c, int32_t layer, const void *x, const void *w_k, const void *w_v,
                                   const float *rope_cos, const float *rope_sin, int32_t rope_positions,
                                   const float *k_norm_weight, float k_norm_eps, const int32_t *start_pos,
                                   const int32_t *new_lens, int32_t max_new, int32_t hidden, void *workspace,
                                   size_t workspace_bytes, void *stream) {
    if (!c || !x || !w_k || !w_v || !start_pos || !new_lens) return SKV_ERR_INVALID_ARG;
    if (layer < 0 || layer >= c->d.n_layers || max_new < 0 || hidden < 1) return SKV_ERR_INVALID_ARG;
    if ((rope_cos == nullptr) != (rope_sin == nullptr)) return SKV_ERR_INVALID_ARG;
    if (rope_cos != nullptr && rope_positions < 1) return SKV_ERR_INVALID_ARG;
    if (k_norm_weight != nullptr && !(k_norm_eps >= 0.f)) return SKV_ERR_INVALID_ARG;
    if (c->route[layer] != layer) return SKV_ERR_NOT_OWNER;
    if (!paged_ready(c)) return SKV_ERR_INVALID_ARG;
    if (!skv::project_append_supported(c->d.dtype, c->d.head_dim, hidden)) return SKV_ERR_UNSUPPORTED;
    if (max_new == 0) return SKV_OK;
    const int64_t n_tokens = (int64_t)c->d.batch * max_new;
    const int n_splits = skv::project_append_splits(c->d.n_kv_heads, c->d.head_dim, n_tokens, hidden);
    const size_t need = skv::project_append_workspace_bytes(c->d.n_kv_heads, c->d.head_dim, n_tokens, hidden);
    if (need > 0 && (!workspace || workspace_bytes < need)) return SKV_ERR_INVALID_ARG;
    skv::ProjArgs a;
    a.partial = (float *)workspace;
    a.slot = view_of(c, c->slot[layer]);
    a.x = x;
    a.w_k = w_k;
    a.w_v = w_v;
    a.rope_cos = rope_cos;
    a.rope_sin = rope_sin;
    a.k_norm_weight = k_norm_weight;
    a.k_norm_eps = k_norm_eps;
    a.start_pos = start_pos;
    a.new_lens = new_lens;
    a.batch = c->d.batch;
    a.max_new = max_new;
    a.hidden = hidden;
    a.rope_positions = rope_positions;
    const hipError_t e = skv::launch_project_append(a, c->d.dtype, c->d.head_dim, n_splits, (hipStream_t)stream);
    return e == hipSuccess ? SKV_OK : hip_fail(e);
}

skv_status_t skv_decode_workspace_bytes(const skv_cache_t *c, int32_t max_kv_len, size_t *bytes) {
    if (!c) return SKV_ERR_INVALID_ARG;
    return skv_decode_range_workspace_bytes(c, c->d.batch, max_kv_len, bytes);
}

skv_status_t skv_attn_decode_range(skv_cache_t *c, int32_t layer, int32_t seq_begin, int32_t seq_count,
                                   const void *q, void *out, const int32_t *kv_lens, int32_t max_kv_len,
                                   float scale, void *workspace, size_t workspace_bytes, void *stream) {
    if (!c || !q || !out || !kv_lens) return SKV_ERR_INVALID_ARG;
    if (layer < 0 || layer >= c->d.n_layers || max_kv_len <= 0) return SKV_ERR_INVALID_ARG;
    if (seq_begin < 0 || seq_count <= 0 || seq_begin > c->d.batch - seq_count) return SKV_ERR_INVALID_ARG;
    if (!(scale > 0.f)) return SKV_ERR_INVALID_ARG;
    if (!paged_ready(c)) return SKV_ERR_INVALID_ARG;
    skv::SlotView view = view_of(c, c->slot[layer]);
    if (max_kv_len > view.max_ctx) return SKV_ERR_CAPACITY;
    size_t need = 0;
    skv_decode_range_workspace_bytes(c, seq_count, max_kv_len, &need);
    if (!workspace || workspace_bytes < need) return SKV_ERR_INVALID_ARG;

    // The kernels number sequences from 0: move the view to the first sequence of the range.
    if (view.block_table != nullptr) {
        view.block_table += (size_t)seq_begin * view.max_blocks_per_seq;
    } else {
        const size_t seq_bytes = (size_t)view.seq_rows * c->d.n_kv_heads * c->d.head_dim * elem_bytes(c->d.dtype);
        view.k = (const char *)view.k + (size_t)seq_begin * seq_bytes;
        view.v = (const char *)view.v + (size_t)seq_begin * seq_bytes;
        if (view.scales != nullptr) view.scales += (size_t)seq_begin * view.seq_rows * c->d.n_kv_heads;
    }

    const int g = c->d.n_q_heads / c->d.n_kv_heads;
    const bool mfma = skv::decode_mfma_supported(c->d.dtype, c->d.head_dim, g);
    if (c->evict_first != nullptr && !mfma) return SKV_ERR_UNSUPPORTED; // eviction: 16-bit and 8-bit slots only
    skv::AttnArgs a;
    a.lse = nullptr;
    a.cache = view;
    a.q = q;
    a.out = out;
    a.q_lens = nullptr;
    a.kv_lens = kv_lens;
    a.evict_sink = c->evict_sink ? c->evict_sink + seq_begin : nullptr;
    a.evict_first = c->evict_first ? c->evict_first + seq_begin : nullptr;
    a.batch = seq_count;
    a.max_q = 1;
    a.n_q_heads = c->d.n_q_heads;
    a.max_kv_len = max_kv_len;
    a.keys_per_split = decode_keys_per_split(c, seq_count, max_kv_len);
    a.n_splits = (max_kv_len + a.keys_per_split - 1) / a.keys_per_split;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.slot_readers = (int32_t)std::count(c->slot.begin(), c->slot.end(), c->slot[layer]);
    a.work_counters = (int32_t *)workspace; // cleared by the launcher whenever the kernel uses them
    a.part_o = (float *)((char *)workspace + kCounterBytes);
    a.part_ml = a.part_o + (size_t)seq_count * c->d.n_q_heads * a.n_splits * c->d.head_dim;

    hipError_t e;
    if (mfma)
        e = skv::launch_decode_mfma(a, c->d.dtype, c->d.head_dim, g, (hipStream_t)stream);
    else
        e = skv::launch_attn_valu(a, c->d.dtype, c->d.head_dim, g, (hipStream_t)stream);
    if (e == hipSuccess && a.n_splits > 1) e = skv::launch_split_merge(a, skv::dtype_act(c->d.dtype), (hipStream_t)stream);
    return e == hipSuccess ? SKV_OK : hip_fail(e);
}

skv_status_t skv_attn_decode(skv_cache_t *c, int32_t layer, const void *q, void *out,
                             const int32_t *kv_lens, int32_t max_kv_len, float scale, void *workspace,
                             size_t workspace_bytes, void *stream) {
    if (!c) return SKV_ERR_INVALID_ARG;
    return skv_attn_decode_range(c, layer, 0, c->d.batch, q, out, kv_lens, max_kv_len, scale, workspace,
                                 workspace_bytes, stream);
}

namespace {
// Scratch of skv_attn_decode_static: device memory that exists from the moment the library is loaded
// (one copy per device, held until the process ends).  In host code the array's name is only a
// stand-in; its device address comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
__device__ __attribute__((aligned(256))) unsigned char scratch[kStaticScratchBytes];

skv_status_t static_scratch(void **out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *ptr[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return SKV_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (ptr[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return SKV_OK;
}
} // namespace

skv_status_t skv_static_scratch_bytes(size_t *bytes) {
    if (!bytes) return SKV_ERR_INVALID_ARG;
    *bytes = kStaticScratchBytes;
    return SKV_OK;
}

skv_status_t skv_attn_decode_static(skv_cache_t *c, int32_t layer, const void *q, void *out, const int32_t *kv_lens,
                                    int32_t max_kv_len, float scale, void *stream) {
    if (!c || max_kv_len <= 0) return SKV_ERR_INVALID_ARG;
    size_t need = 0;
    if (skv_status_t st = skv_decode_workspace_bytes(c, max_kv_len, &need); st != SKV_OK) return st;
    if (need > kStaticScratchBytes) return SKV_ERR_CAPACITY;
    void *ws = nullptr;
    if (skv_status_t st = static_scratch(&ws); st != SKV_OK) return st;
    // the kernels take the scratch as they take a caller's workspace; the work counter at its start is
    // cleared in-stream by the launcher, every split partial is written before the merge reads it
    return skv_attn_decode_range(c, layer, 0, c->d.batch, q, out, kv_lens, max_kv_len, scale, ws, need, stream);
}

skv_status_t skv_attn_prefill(skv_cache_t *c, int32_t layer, const void *q, void *out,
                              const int32_t *q_lens, const int32_t *kv_lens, int32_t max_q,
                              int32_t max_kv_len, float scale, void *stream) {
    if (!c || !q || !out || !q_lens || !kv_lens) return SKV_ERR_INVALID_ARG;
    if (layer < 0 || layer >= c->d.n_layers || max_q <= 0 || max_kv_len <= 0) return SKV_ERR_INVALID_ARG;
    if (!(scale > 0.f)) return SKV_ERR_INVALID_ARG;
    if (!paged_ready(c)) return SKV_ERR_INVALID_ARG;
    if (c->evict_first != nullptr) return SKV_ERR_UNSUPPORTED; // pre-fill over an evicted cache is not built
    const skv::SlotView view = view_of(c, c->slot[layer]);
    if (max_kv_len > view.max_ctx) return SKV_ERR_CAPACITY;

    skv::AttnArgs a;
    a.evict_sink = a.evict_first = nullptr;
    a.lse = nullptr;
    a.cache = view;
    a.q = q;
    a.out = out;
    a.q_lens = q_lens;
    a.kv_lens = kv_lens;
    a.batch = c->d.batch;
    a.max_q = max_q;
    a.n_q_heads = c->d.n_q_heads;
    a.max_kv_len = max_kv_len;
    a.slot_readers = 1;
    a.keys_per_split = max_kv_len; // a prefill row is never split along the key axis
    a.n_splits = 1;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.part_o = nullptr;
    a.part_ml = nullptr;
    a.work_counters = nullptr;

    return launch_prefill(a, c->d.dtype, c->d.head_dim, c->d.n_q_heads / c->d.n_kv_heads, (hipStream_t)stream);
}

/* ---- training-time routed attention ------------------------------------------------------- */

skv_status_t skv_train_sample_route(int32_t scheme, int32_t n_layers, int32_t k, double p, uint64_t seed,
                                    uint64_t step, int32_t *route) {
    if (!route || n_layers < 1) return SKV_ERR_INVALID_ARG;
    const bool random = scheme == SKV_TRAIN_RCLA || scheme == SKV_TRAIN_RDCLA_K;
    const bool grouped = scheme == SKV_TRAIN_CLA_K || scheme == SKV_TRAIN_RDCLA_K;
    if (!random && !grouped) return SKV_ERR_INVALID_ARG;
    if (grouped && k < 1) return SKV_ERR_INVALID_ARG;
    if (random && !(p >= 0.0 && p <= 1.0)) return SKV_ERR_INVALID_ARG;
    // SplitMix64 output function: the value a generator whose state is x returns on its next step
    auto mix = [](uint64_t x) {
        x += 0x9E3779B97F4A7C15ull;
        x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
        x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
        return x ^ (x >> 31);
    };
    const uint64_t pass = mix(mix(seed) ^ step);
    auto draw = [&](int32_t layer, int which) { return mix(pass ^ (uint64_t)(256 * (int64_t)layer + which)); };
    auto decide = [&](int32_t layer) { return (double)(draw(layer, 0) >> 11) * 0x1.0p-53 < p; };
    for (int32_t l = 0; l < n_layers; ++l) {
        const int32_t fixed = grouped ? k * (l / k) : l;
        if (scheme == SKV_TRAIN_CLA_K)
            route[l] = fixed;
        else if (scheme == SKV_TRAIN_RDCLA_K)
            route[l] = decide(l) ? l : fixed;
        else if (l == 0 || decide(l))
            route[l] = l;
        else
            route[l] = (int32_t)(((draw(l, 1) >> 32) * (uint64_t)l) >> 32);
    }
    return SKV_OK;
}

namespace {
// Fault word of the training calls: a device variable of the library (zero from load time on), so
// that no compute call allocates.  Every device holds its own copy at its own address.
__device__ __attribute__((aligned(256))) uint32_t g_train_faults[64];

skv_status_t train_fault_word(uint32_t **out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static uint32_t *word[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return SKV_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (word[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_train_faults));
        if (e != hipSuccess) return hip_fail(e);
        word[dev] = (uint32_t *)p;
    }
    *out = word[dev];
    return SKV_OK;
}

bool train_shape_ok(int32_t batch, int32_t seq, int32_t hq, int32_t hkv) {
    return batch >= 1 && seq >= 1 && hq >= 1 && hkv >= 1 && hq % hkv == 0;
}
} // namespace

skv_status_t skv_train_attn_fwd(const void *q, const void *k, const void *v, void *out, float *lse,
                                const int32_t *seq_lens, int32_t batch, int32_t seq, int32_t n_q_heads,
                                int32_t n_kv_heads, int32_t head_dim, int32_t dtype, float scale, void *stream) {
    if (!q || !k || !v || !out || !lse || !seq_lens) return SKV_ERR_INVALID_ARG;
    if (!train_shape_ok(batch, seq, n_q_heads, n_kv_heads) || !(scale > 0.f)) return SKV_ERR_INVALID_ARG;
    if (!(dtype == SKV_BF16 || dtype == SKV_F16) || !(head_dim == 64 || head_dim == 128)) return SKV_ERR_UNSUPPORTED;
    uint32_t *faults = nullptr;
    if (skv_status_t st = train_fault_word(&faults); st != SKV_OK) return st;
    // the source layer's activations are laid out exactly like one contiguous cache slot of
    // capacity seq, so the pre-fill kernels run on them unchanged
    skv::AttnArgs a;
    a.evict_sink = a.evict_first = nullptr;
    a.cache.k = k;
    a.cache.v = v;
    a.cache.scales = nullptr;
    a.cache.block_table = nullptr;
    a.cache.faults = faults;
    a.cache.max_blocks_per_seq = 0;
    a.cache.block_shift = 0;
    a.cache.n_blocks = 0;
    a.cache.max_ctx = seq;
    a.cache.seq_rows = seq;
    a.cache.group_shift = 0;
    a.cache.n_kv_heads = n_kv_heads;
    a.cache.head_dim = head_dim;
    a.q = q;
    a.out = out;
    a.q_lens = seq_lens;
    a.kv_lens = seq_lens;
    a.part_o = nullptr;
    a.part_ml = nullptr;
    a.work_counters = nullptr;
    a.batch = batch;
    a.max_q = seq;
    a.n_q_heads = n_q_heads;
    a.max_kv_len = seq;
    a.keys_per_split = seq;
    a.slot_readers = 1;
    a.n_splits = 1;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.lse = lse;
    return launch_prefill(a, dtype, head_dim, n_q_heads / n_kv_heads, (hipStream_t)stream);
}

skv_status_t skv_train_bwd_workspace_bytes(int32_t batch, int32_t seq, int32_t n_q_heads, size_t *bytes) {
    if (!bytes || batch < 1 || seq < 1 || n_q_heads < 1) return SKV_ERR_INVALID_ARG;
    *bytes = (size_t)batch * (size_t)seq * (size_t)n_q_heads * sizeof(float);
    return SKV_OK;
}

skv_status_t skv_train_attn_bwd(const void *q, const void *k, const void *v, const void *out, const float *lse,
                                const void *d_out, void *dq, float *dk_accum, float *dv_accum,
                                const int32_t *seq_lens, int32_t batch, int32_t seq, int32_t n_q_heads,
                                int32_t n_kv_heads, int32_t head_dim, int32_t dtype, float scale, void *workspace,
                                size_t workspace_bytes, void *stream) {
    if (!q || !k || !v || !out || !lse || !d_out || !dq || !dk_accum || !dv_accum || !seq_lens || !workspace)
        return SKV_ERR_INVALID_ARG;
    if (!train_shape_ok(batch, seq, n_q_heads, n_kv_heads) || !(scale > 0.f)) return SKV_ERR_INVALID_ARG;
    if (!(dtype == SKV_BF16 || dtype == SKV_F16) || !(head_dim == 64 || head_dim == 128)) return SKV_ERR_UNSUPPORTED;
    size_t need = 0;
    skv_train_bwd_workspace_bytes(batch, seq, n_q_heads, &need);
    if (workspace_bytes < need) return SKV_ERR_INVALID_ARG;
    uint32_t *faults = nullptr;
    if (skv_status_t st = train_fault_word(&faults); st != SKV_OK) return st;
    skv::TrainBwdArgs a;
    a.q = q; a.k = k; a.v = v; a.out = out; a.d_out = d_out;
    a.lse = lse;
    a.dq = dq;
    a.dk_accum = dk_accum; a.dv_accum = dv_accum;
    a.delta = (float *)workspace;
    a.seq_lens = seq_lens;
    a.faults = faults;
    a.batch = batch; a.seq = seq; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads;
    a.scale = scale;
    const hipError_t e = skv::launch_train_bwd(a, dtype, head_dim, (hipStream_t)stream);
    return e == hipSuccess ? SKV_OK : hip_fail(e);
}

skv_status_t skv_train_device_faults(uint32_t *faults) {
    if (!faults) return SKV_ERR_INVALID_ARG;
    uint32_t *word = nullptr;
    if (skv_status_t st = train_fault_word(&word); st != SKV_OK) return st;
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return hip_fail(e);
    e = hipMemcpy(faults, word, sizeof(uint32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e);
    if (*faults != 0) {
        e = hipMemset(word, 0, sizeof(uint32_t));
        if (e != hipSuccess) return hip_fail(e);
    }
    return SKV_OK;
}

const char *skv_status_str(skv_status_t s) {
    switch (s) {
    case SKV_OK: return "SKV_OK";
    case SKV_ERR_INVALID_ARG: return "SKV_ERR_INVALID_ARG";
    case SKV_ERR_BAD_ROUTE: return "SKV_ERR_BAD_ROUTE";
    case SKV_ERR_NOT_OWNER: return "SKV_ERR_NOT_OWNER";
    case SKV_ERR_CAPACITY: return "SKV_ERR_CAPACITY";
    case SKV_ERR_OOM: return "SKV_ERR_OOM";
    case SKV_ERR_UNSUPPORTED: return "SKV_ERR_UNSUPPORTED";
    case SKV_ERR_HIP: return "SKV_ERR_HIP";
    }
    return "SKV_ERR_UNKNOWN";
}

int32_t skv_last_hip_error(void) { return g_last_hip_error; }
const char *skv_last_kernel_name(void) { return g_last_kernel; }

} // extern "C"
