/*
 * skv -- routed grouped-query attention over a depth-shared KV cache, for AMD MI355X (gfx950).
 *
 * Layer l of a decoder reads the K/V cache of a source layer route[l] <= l (cross-layer
 * attention, paper Eq. (3.1)); only layers with route[l] == l ("owners", the cache-sharing
 * strategy S of Sec. 3.1.3) hold a cache slot, so cache memory is proportional to the number
 * of distinct slots instead of the number of layers.  This library holds the slot cache and
 * runs the three operations of the paper's inference loop (Alg. 2): the cache update for owner
 * layers, attention of one new token against the routed slot (sampling phase, Sec. 3.1.1) and
 * causal attention of many tokens against it (pre-fill phase).
 *
 * Conventions
 *   - C linkage, plain pointers and sizes only.  "host" / "device" on every pointer says where
 *     the memory lives.  Device pointers are ordinary HIP allocations (for example the storage
 *     of a PyTorch-ROCm tensor).  `stream` is a hipStream_t passed as void* (NULL = default).
 *   - Every compute call only ENQUEUES work on `stream`: no synchronisation, no allocation.
 *     Caller-owned buffers must stay alive until that work has run.  Calls that share a workspace
 *     must not overlap in time: enqueue them on one stream, or order the streams.
 *   - Layers, heads, positions and slots are 0-based (the paper counts layers from 1).
 *   - Query head h reads kv head h / (n_q_heads / n_kv_heads).
 *   - The query at absolute position p sees cached positions 0..p.
 *   - Every function returns a status; on any status other than SKV_OK nothing was enqueued
 *     and the cache is unchanged.  There is no CPU compute path: without a usable HIP device
 *     the compute calls return SKV_ERR_HIP.
 *   - Lengths and positions live on the device and cannot be checked by the host without a
 *     synchronisation.  Kernels never touch memory outside the cache: a position beyond the
 *     capacity, or a block id outside [0, n_blocks), is skipped and recorded in a per-cache
 *     fault word (skv_cache_device_faults).
 *
 * Cache layout (element type = dtype of the descriptor)
 *   contiguous (block_size == 0):  K and V pools are [n_slots][batch][max_ctx][n_kv_heads][head_dim]
 *   paged      (block_size  > 0):  K and V pools are [n_slots][n_blocks][block_size][n_kv_heads][head_dim];
 *       logical (b, pos) lives in physical block table[b][pos / block_size] at offset
 *       pos % block_size.  One table serves every slot.
 *
 * 8-bit slots (dtype SKV_BF16_KV8 / SKV_F16_KV8).  The paper leaves the composition of depth-wise
 * sharing with KV quantisation open (Sec. 5, Limitations); this library's reading: the head_dim
 * values x of one (position, kv head) of K (and likewise of V) are stored as head_dim e4m3 codes
 * (the 8-bit float of the OCP 8-bit floating point specification: 4 exponent bits of bias 7, 3
 * mantissa bits, largest value 448) and one exponent byte:
 *     e = the smallest integer with max|x| * 2^-e <= 448, clamped to [-127, 127] (0 if all x are 0),
 *     code_i = x_i * 2^-e rounded to the nearest e4m3 number, ties to the even code; byte = e + 127.
 * skv_kv_append does this conversion; attention reads code * 2^e, which is exact in bf16 / fp16,
 * so Eq. (3.1) is evaluated on the stored values exactly as on a 16-bit cache.
 * Layout of 8-bit slots: 1-byte elements, and the rows of one kv head lie together in groups of
 * R consecutive rows, so that a reader of one kv head streams R * head_dim contiguous bytes
 * (strided 64- or 128-byte pieces cost a good part of the HBM rate):
 *   contiguous:  K and V pools are [n_slots][batch][ceil(max_ctx / 128)][n_kv_heads][128][head_dim]   (R = 128)
 *   paged:       K and V pools are [n_slots][n_blocks][block_size / R][n_kv_heads][R][head_dim],
 *                R = min(block_size, 128); block_size must be at least 16
 * and a third pool holds the exponent bytes as uint16 in the same order without the last axis
 * ([...][n_kv_heads][R]; low byte: K, high byte: V).  head_dim must be 64 or 128.
 */
#ifndef SKV_H
#define SKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct skv_cache skv_cache_t; /* opaque, owned by the library */

typedef enum {
    SKV_OK = 0,
    SKV_ERR_INVALID_ARG = 1, /* null pointer, negative size, layer out of range, small workspace */
    SKV_ERR_BAD_ROUTE = 2,   /* route violates 0 <= route[l] <= l or route[route[l]] == route[l] */
    SKV_ERR_NOT_OWNER = 3,   /* cache update asked for a layer that owns no slot */
    SKV_ERR_CAPACITY = 4,    /* a host-side length exceeds the cache capacity */
    SKV_ERR_OOM = 5,         /* device or host allocation failed */
    SKV_ERR_UNSUPPORTED = 6, /* head_dim / dtype / head grouping / block size not supported */
    SKV_ERR_HIP = 7          /* a HIP call failed; see skv_last_hip_error */
} skv_status_t;

/* SKV_F32 / SKV_F16 / SKV_BF16: slots, queries, new rows and outputs all have this type.
 * SKV_BF16_KV8 / SKV_F16_KV8: queries, new rows and outputs are bf16 / fp16, the slots hold 8-bit
 * codes (see "8-bit slots" below). */
typedef enum { SKV_F32 = 0, SKV_F16 = 1, SKV_BF16 = 2, SKV_BF16_KV8 = 3, SKV_F16_KV8 = 4 } skv_dtype_t;

/* Bits of the per-cache device fault word. */
enum {
    SKV_FAULT_APPEND_RANGE = 1, /* an append row fell outside the capacity and was dropped */
    SKV_FAULT_BLOCK_ID = 2,     /* a block-table entry was outside [0, n_blocks) */
    SKV_FAULT_KV_LEN = 4        /* a kv length was < 1, above the hint/capacity, or < q length */
};

typedef struct {
    int32_t n_layers;
    int32_t n_q_heads;
    int32_t n_kv_heads;  /* must divide n_q_heads; group size n_q_heads / n_kv_heads in {1,2,4,8,16} */
    int32_t head_dim;    /* 64, 128 or 256 */
    int32_t batch;       /* number of sequences */
    int32_t max_ctx;     /* capacity in positions per sequence (contiguous: pool extent;
                            paged: max_blocks_per_seq * block_size is the effective bound) */
    int32_t dtype;       /* skv_dtype_t */
    int32_t block_size;  /* 0 = contiguous, else tokens per physical block (power of two, 8..256; 8-bit slots: 16..256) */
    int32_t n_blocks;    /* paged: physical blocks per slot pool; ignored when contiguous */
    const int32_t *route; /* host, n_layers entries, copied by skv_cache_alloc */
    void *k_pool;        /* device, optional caller-owned storage for K; NULL = library allocates */
    void *v_pool;        /* device, same for V; both or neither */
    size_t pool_bytes;   /* size of EACH caller pool; must be >= the K pool's bytes (skv_cache_pool_bytes) */
    void *scale_pool;    /* device, 8-bit slots with caller pools only: storage of the exponent bytes */
    size_t scale_pool_bytes; /* its size; must be >= the scale pool's bytes (skv_cache_pool_bytes) */
} skv_cache_desc_t;

/* ---- routing (host only, no device needed) ------------------------------------------------ */

/* Eq. (3.2): route[l] = l if l is in the strategy, else the largest strategy layer below l.
 * owners: host, n_owners distinct layers in any order.  route_out: host, n_layers.
 * SKV_ERR_BAD_ROUTE if layer 0 is not an owner (the map is undefined for the layers before the
 * first owner), or an owner is outside [0, n_layers) or repeated. */
skv_status_t skv_route_from_strategy(const int32_t *owners, int32_t n_owners, int32_t n_layers,
                                     int32_t *route_out);

/* Checks a route (any l' <= l that owns a slot is allowed, Eq. (3.1)) and derives the slot map:
 * slot_of_layer[l] = rank of route[l] among the owners in ascending order.
 * slot_of_layer (host, n_layers) and n_slots may be NULL. */
skv_status_t skv_route_validate(const int32_t *route, int32_t n_layers, int32_t *slot_of_layer,
                                int32_t *n_slots);

/* Total bytes of the K and V pools together:
 * 2 * n_slots * batch * max_ctx * n_kv_heads * head_dim * sizeof(dtype)   (contiguous)
 * 2 * n_slots * n_blocks * block_size * n_kv_heads * head_dim * sizeof(dtype)   (paged)
 * i.e. the footprint M = L x (T + t) x S of Sec. 3.1.1 with L replaced by |S|.  8-bit slots: one byte
 * per element plus the pool of exponent bytes, and a contiguous slot holds max_ctx rounded up to a
 * multiple of 128 rows per sequence (see "8-bit slots" above). */
skv_status_t skv_cache_bytes(const skv_cache_desc_t *desc, size_t *total_bytes);

/* The parts of skv_cache_bytes: bytes of the K pool (the V pool has the same size) and of the pool
 * of exponent bytes (0 unless the slots are 8-bit): total = 2 * kv_pool_bytes + scale_pool_bytes,
 * i.e. per cached position and kv head 2 * head_dim * sizeof(element) (+ 2 for 8-bit slots).
 * Either out pointer may be NULL. */
skv_status_t skv_cache_pool_bytes(const skv_cache_desc_t *desc, size_t *kv_pool_bytes, size_t *scale_pool_bytes);

/* ---- cache object --------------------------------------------------------------------------- */

/* The cache of Sec. 3.1.1 under a sharing strategy (Sec. 3.1.3): one K and one V slot per owner
 * layer instead of per layer, sized as skv_cache_bytes says.  Validates the descriptor, copies the
 * route, allocates the pools unless the caller gave them, and zero-fills library-allocated pools.
 * *out is set only on SKV_OK.  Synchronous.  Ownership: the handle and library-allocated pools
 * belong to the library until skv_cache_free; caller pools and the block table are only borrowed.
 * Placement: library-allocated K and V pools are one allocation (up to 1407 bytes more than
 * skv_cache_bytes says), the V pool 384 bytes past a multiple of 1 KiB behind the start of the K pool.
 * The decode call reads the K and the V rows of the same positions at the same time, and pools that lie
 * a multiple of 1 KiB apart (two separate device allocations do) send both streams to the same memory
 * channels: 7 % slower on 8 kv heads x 128 in bf16, 1-1.5 % on 32 kv heads or paged pools.  A caller
 * that brings its own pools should place them likewise (any distance of 256 or 384 modulo 1 KiB; keep
 * both on 128-byte boundaries). */
skv_status_t skv_cache_alloc(const skv_cache_desc_t *desc, skv_cache_t **out);

/* Ends the life of a cache made by skv_cache_alloc (Sec. 3.1.1: the cache lives for one generation
 * request).  Frees the handle and library-allocated pools (never caller pools).  NULL is accepted.
 * The caller must have synchronised all streams that still use the cache. */
skv_status_t skv_cache_free(skv_cache_t *cache);

/* Introspection (host values).  Any out pointer may be NULL. */
skv_status_t skv_cache_info(const skv_cache_t *cache, int32_t *n_slots, void **k_pool_device,
                            void **v_pool_device, size_t *pool_bytes_each);
skv_status_t skv_cache_slot_of_layer(const skv_cache_t *cache, int32_t layer, int32_t *slot,
                                     int32_t *is_owner);
/* 8-bit slots: the pool of exponent bytes (device pointer, bytes); NULL / 0 for other caches. */
skv_status_t skv_cache_scale_info(const skv_cache_t *cache, void **scale_pool_device, size_t *scale_pool_bytes);

/* Paged caches: borrow the block table, device int32 [batch][max_blocks_per_seq].  Must be set
 * before the first append / attention call and stay alive while the cache is used. */
skv_status_t skv_cache_set_block_table(skv_cache_t *cache, const int32_t *table_device,
                                       int32_t max_blocks_per_seq);

/* Temporal eviction (the paper's Sec. 5 names the composition of depth-wise sharing with "temporal
 * eviction methods" as open; this library's reading is a sliding window with sinks): of the
 * kv_lens[b] cached positions of sequence b only [0, sink_len[b]) and [first_pos[b], kv_lens[b])
 * survive; the positions between were dropped from EVERY slot (one dropped block frees its rows in
 * |S| slots instead of L), their rows and, for a paged cache, their block-table entries are never
 * read again and may hold anything.  sink_len, first_pos: device int32[batch], borrowed until they
 * are replaced; both NULL switches eviction off.  sink_len[b] must be a multiple of 32 and
 * 0 <= sink_len[b] <= first_pos[b] <= kv_lens[b]; over 8-bit slots the number of dropped positions
 * first_pos[b] - sink_len[b] must be a multiple of the group size R of the slot (whole groups are
 * dropped); other values set SKV_FAULT_KV_LEN and zero the sequence's output.  A paged cache that wants
 * its dropped blocks back drops whole blocks (first_pos[b] a multiple of the block size); the kernels
 * do not ask for it.
 * While eviction is on, skv_attn_decode / _range / _static attend over the surviving positions
 * only, and their max_kv_len bounds the number of SURVIVING positions per sequence (kv_lens[b]
 * itself is bounded by the capacity); skv_attn_prefill returns SKV_ERR_UNSUPPORTED, and so does
 * decode on a float32 cache or with head_dim 256.  Appends are unaffected. */
skv_status_t skv_cache_set_eviction(skv_cache_t *cache, const int32_t *sink_len, const int32_t *first_pos);

/* Reads and clears the device fault word (synchronises the device). */
skv_status_t skv_cache_device_faults(skv_cache_t *cache, uint32_t *faults);

/* ---- the three operations of the inference loop (Alg. 2) ----------------------------------- */

/* "Update K_l, V_l", allowed only if layer owns a slot (else SKV_ERR_NOT_OWNER, cache untouched).
 * k_new, v_new: device [batch][max_new][n_kv_heads][head_dim]; row i < new_lens[b] of sequence b
 * is written, bit for bit, to position start_pos[b] + i of the layer's slot; other rows are
 * ignored.  start_pos, new_lens: device int32[batch].  8-bit slots: k_new, v_new are bf16 / fp16 and
 * every (row, kv head) piece is converted to codes and an exponent byte as stated at the top (the
 * conversion is deterministic: the stored bytes have exactly one correct value). */
skv_status_t skv_kv_append(skv_cache_t *cache, int32_t layer, const void *k_new, const void *v_new,
                           const int32_t *start_pos, const int32_t *new_lens, int32_t max_new,
                           void *stream);

/* The same update with the projection in front of it (Sec. 4.3: the leader layer of a sharing
 * group computes and stores K, V; every other layer skips its K/V projections, which is where the
 * paper's throughput gain comes from): K = x w_k^T, V = x w_v^T with fp32 accumulation, K
 * optionally rotated by position, rounded once to the cache dtype and written to the slot as
 * skv_kv_append would; the projected rows never exist in memory outside the cache.
 * x: device [batch][max_new][hidden], cache dtype; w_k, w_v: device
 * [n_kv_heads * head_dim][hidden] (one row per output feature).  rope_cos, rope_sin: device float
 * [rope_positions][head_dim / 2], or both NULL for no rotation; feature i < head_dim / 2 of a head
 * pairs with i + head_dim / 2:  k'_i = k_i cos - k_(i+d/2) sin,  k'_(i+d/2) = k_(i+d/2) cos +
 * k_i sin, with the table row of the token's position start_pos[b] + i (a position beyond the
 * table drops the row and sets SKV_FAULT_APPEND_RANGE).  V is never rotated.
 * k_norm_weight: device float[head_dim] or NULL.  Not NULL: every head's key vector is normalised
 * before the rotation, k <- k / sqrt(mean_d(k^2) + k_norm_eps) * k_norm_weight[d] (the per-head key
 * normalisation of the Qwen3 family); V is never normalised.
 * workspace: device scratch of skv_kv_project_workspace_bytes(cache, max_new, hidden) bytes (0 for
 * large prompts: launches too small to fill the chip -- one decode token per sequence, or a prompt
 * of a few thousand tokens -- split the hidden axis over work groups and keep fp32 partial sums
 * there; launches of at most 64 token rows always do); may be NULL when that is 0.
 * SKV_ERR_NOT_OWNER for a layer without a slot (nothing is computed: that is the saving);
 * SKV_ERR_UNSUPPORTED unless the cache is 16-bit, head_dim 64 or 128 and hidden a multiple of 64. */
skv_status_t skv_kv_project_workspace_bytes(const skv_cache_t *cache, int32_t max_new, int32_t hidden,
                                            size_t *bytes);
skv_status_t skv_kv_project_append(skv_cache_t *cache, int32_t layer, const void *x, const void *w_k,
                                   const void *w_v, const float *rope_cos, const float *rope_sin,
                                   int32_t rope_positions, const float *k_norm_weight, float k_norm_eps,
                                   const int32_t *start_pos,
                                   const int32_t *new_lens, int32_t max_new, int32_t hidden,
                                   void *workspace, size_t workspace_bytes, void *stream);

/* Scratch bytes skv_attn_decode needs for sequences of up to max_kv_len positions: enough for
 * every call whose max_kv_len hint is at most this one.  The scratch holds what the sampling-phase
 * attention of Eq. (3.1) keeps between its two launches when the key axis is split: per (sequence,
 * query head, split) the running maximum, the sum of weights and the unnormalised output in fp32,
 * plus 256 bytes of work counters. */
skv_status_t skv_decode_workspace_bytes(const skv_cache_t *cache, int32_t max_kv_len, size_t *bytes);

/* Sampling-phase attention, Eq. (3.1) for one query token per sequence:
 *   out[b][h] = sum_j softmax_j(scale * <q[b][h], K[j]>) V[j],  j < kv_lens[b],
 * over the slot of route[layer].  q, out: device [batch][n_q_heads][head_dim], dtype of the
 * cache; fp32 accumulation; out rounded to nearest even.  scale must be > 0 (else
 * SKV_ERR_INVALID_ARG; the same holds for skv_attn_prefill).  kv_lens: device int32[batch], each in
 * [1, max_kv_len]; max_kv_len (host) only sizes the launch and must be >= every kv_lens[b]
 * (positions beyond it are not read).  workspace: device, >= skv_decode_workspace_bytes. */
skv_status_t skv_attn_decode(skv_cache_t *cache, int32_t layer, const void *q, void *out,
                             const int32_t *kv_lens, int32_t max_kv_len, float scale,
                             void *workspace, size_t workspace_bytes, void *stream);

/* Sampling-phase attention for the sequences [seq_begin, seq_begin + seq_count) of the cache only.
 * q, out and kv_lens describe just those sequences (q, out: device [seq_count][n_q_heads][head_dim];
 * kv_lens: device int32[seq_count]); everything else is as in skv_attn_decode, which is the range
 * [0, batch).  The workspace must hold skv_decode_range_workspace_bytes(cache, seq_count, max_kv_len).
 * Purpose: the layers of one sharing group read the same slot, and the paper's closing remark on
 * inference efficiency (Sec. 4.3, last paragraph) is that a backend could keep the shared K,V
 * on chip across consecutive layers.  A caller that runs the group's layers back to back on one
 * chunk of sequences whose slice of the slot fits the on-chip caches (256 MiB of Infinity Cache on
 * MI355X), chunk by chunk, reads the slot from HBM once per group instead of once per layer.
 * SKV_ERR_INVALID_ARG if the range is empty or leaves [0, batch). */
skv_status_t skv_decode_range_workspace_bytes(const skv_cache_t *cache, int32_t seq_count,
                                              int32_t max_kv_len, size_t *bytes);
skv_status_t skv_attn_decode_range(skv_cache_t *cache, int32_t layer, int32_t seq_begin, int32_t seq_count,
                                   const void *q, void *out, const int32_t *kv_lens, int32_t max_kv_len,
                                   float scale, void *workspace, size_t workspace_bytes, void *stream);

/* skv_attn_decode for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as skv_attn_decode, but the split partials and the work counter live
 * in a scratch array that is part of the library's device image (skv_static_scratch_bytes: 64 MiB per
 * device, present from load time until the process ends); the call allocates and frees nothing.
 * SKV_ERR_CAPACITY if skv_decode_workspace_bytes(cache, max_kv_len) exceeds that size (nothing is
 * enqueued).  Every call on one device shares that device's scratch: two calls that overlap in
 * time on one device race (keep them on one stream or order the streams), whatever their caches.
 * The first call on a device looks the array's address up (no allocation); make it outside a
 * stream capture. */
skv_status_t skv_static_scratch_bytes(size_t *bytes);
skv_status_t skv_attn_decode_static(skv_cache_t *cache, int32_t layer, const void *q, void *out,
                                    const int32_t *kv_lens, int32_t max_kv_len, float scale, void *stream);

/* Pre-fill-phase attention: q_lens[b] query rows per sequence; row i sits at absolute position
 * kv_lens[b] - q_lens[b] + i and sees cached positions 0..that position of the routed slot.
 * q, out: device [batch][max_q][n_q_heads][head_dim]; rows i >= q_lens[b] are neither read nor
 * written.  q_lens, kv_lens: device int32[batch], 0 <= q_lens[b] <= min(max_q, kv_lens[b]),
 * kv_lens[b] <= max_kv_len.  A sequence whose lengths break these rules sets SKV_FAULT_KV_LEN and
 * nothing is written for it, whatever the dtype (skv_attn_decode zero-fills the output row of such a
 * sequence instead). */
skv_status_t skv_attn_prefill(skv_cache_t *cache, int32_t layer, const void *q, void *out,
                              const int32_t *q_lens, const int32_t *kv_lens, int32_t max_q,
                              int32_t max_kv_len, float scale, void *stream);

/* ---- diagnostics ---------------------------------------------------------------------------- */
const char *skv_status_str(skv_status_t status);
/* Code of the last failing HIP call seen by this thread's skv_* calls (0 = none). */
int32_t skv_last_hip_error(void);
/* Name of the kernel the last successful skv_attn_* call on this thread launched (static string),
 * for profiling scripts that have to find it in a trace. */
const char *skv_last_kernel_name(void);


/* ---- training-time routed attention (Sec. 3.2, Sec. 4.2.3) ---------------------------------- */
/* During training every layer computes its own K, V and attends, in each forward pass, either to
 * them or to those of an earlier layer.  The library draws the per-pass source layers and runs
 * the attention over whole sequences with its gradient; the caller owns the activations. */

typedef enum {
    SKV_TRAIN_RCLA = 0,    /* Sec. 3.2: d ~ Bernoulli(p); d = 1 self, d = 0 a uniformly drawn earlier layer */
    SKV_TRAIN_CLA_K = 1,   /* Sec. 4.2.3 CLA@k: groups of k layers attend to the group's first layer */
    SKV_TRAIN_RDCLA_K = 2  /* Sec. 4.2.3 RD-CLA@k: per layer and pass a coin, d ~ Bernoulli(p);
                              d = 1 the layer's own K, V, d = 0 the fixed layer of CLA@k */
} skv_train_scheme_t;

/* Source layers of one forward pass (host only): route[l] = layer whose K, V layer l attends to,
 * 0-based, route[l] <= l, route[0] = 0.  Counter-based, so a pass can be replayed (backward,
 * recomputation, another rank): r(layer, which) = mix(mix(mix(seed) ^ step) ^ (256 layer + which))
 * with mix the SplitMix64 output function; the decision is d = 1 iff (r(l, 0) >> 11) 2^-53 < p,
 * the R-CLA source is ((r(l, 1) >> 32) * l) >> 32.  k is used by the two @k schemes only (k >= 1),
 * p by the two random ones (0 <= p <= 1).  SKV_ERR_INVALID_ARG otherwise. */
skv_status_t skv_train_sample_route(int32_t scheme, int32_t n_layers, int32_t k, double p,
                                    uint64_t seed, uint64_t step, int32_t *route);

/* Forward, Eq. (3.1) over whole sequences with a causal mask: row i of sequence b attends to
 * rows 0..i of k, v (the activations of the source layer), i < seq_lens[b].
 * q, out: device [batch][seq][n_q_heads][head_dim]; k, v: device [batch][seq][n_kv_heads][head_dim];
 * dtype SKV_BF16 or SKV_F16, head_dim 64 or 128 (else SKV_ERR_UNSUPPORTED); fp32 accumulation.
 * lse: device float [batch][n_q_heads][seq], receives log sum_j exp(scale <q_i, k_j>) (natural
 * log), which the backward needs.  seq_lens: device int32[batch], each in [1, seq]; rows at or
 * beyond a sequence's length are neither read nor written.  Asynchronous on `stream`; allocates
 * nothing (the fault word of the training calls, see skv_train_device_faults, is a device variable
 * of the library). */
skv_status_t skv_train_attn_fwd(const void *q, const void *k, const void *v, void *out, float *lse,
                                const int32_t *seq_lens, int32_t batch, int32_t seq,
                                int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                int32_t dtype, float scale, void *stream);

/* Scratch bytes of skv_train_attn_bwd (one float per query row and head). */
skv_status_t skv_train_bwd_workspace_bytes(int32_t batch, int32_t seq, int32_t n_q_heads, size_t *bytes);

/* Backward of skv_train_attn_fwd for the loss whose gradient with respect to out is d_out
 * (device, layout and dtype of out); q, k, v, out, lse as in / from the forward.
 * dq: device, layout and dtype of q, written (rows beyond a sequence's length untouched).
 * dk_accum, dv_accum: device FLOAT [batch][seq][n_kv_heads][head_dim]; the gradients with
 * respect to k and v are ADDED to them: a layer read by several layers in one pass (and by the
 * heads of a group) collects all of them in one fp32 buffer, which the caller zeroes before the
 * pass and rounds afterwards.  Calls that add into the same buffers must be ordered on one
 * stream.  Deterministic (no atomics).  Asynchronous on `stream`. */
skv_status_t skv_train_attn_bwd(const void *q, const void *k, const void *v, const void *out,
                                const float *lse, const void *d_out, void *dq, float *dk_accum,
                                float *dv_accum, const int32_t *seq_lens, int32_t batch, int32_t seq,
                                int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t dtype,
                                float scale, void *workspace, size_t workspace_bytes, void *stream);

/* Reads and clears the fault word of the training calls (a sequence length outside [1, seq] sets
 * SKV_FAULT_KV_LEN and nothing is computed for that sequence).  Synchronises the device. */
skv_status_t skv_train_device_faults(uint32_t *faults);

#ifdef __cplusplus
}
#endif
#endif /* SKV_H */
