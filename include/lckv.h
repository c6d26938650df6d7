/*
 * lckv.h - C ABI of the MI355X (gfx950) decode-attention library for the Layer-Condensed KV Cache model
 * (Wu & Tu, "Layer-Condensed KV Cache for Efficient Inference of Large Language Models").
 *
 * One decode step of that model (Section 2.1, Figure 1b): the queries of every non-warmup ("condensed")
 * layer attend to ONE shared KV cache that holds only the top layer's keys and values, with the diagonal
 * masked (the token being decoded is not visible to itself); the few warmup layers keep standard attention
 * over caches of their own (themselves included); the step stores the new token's K/V of every producing
 * layer.  A "slot" is one layer's worth of K and V cache.
 *
 * Conventions
 *   - Every function returns LCKV_OK (0) or a negative LCKV_ERR_* code; nothing throws, nothing aborts.
 *   - "device" pointers are HIP device memory on the current device, "host" pointers are ordinary memory.
 *   - The caller owns every buffer and the stream.  The library owns only the handle and a few small device
 *     tables.  Unless stated, a call only enqueues work on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and does not synchronise; it performs no allocation after
 *     lckv_cache_alloc, so it may be captured into a HIP graph.
 *   - Tensors are dense, row-major, in the cache's element type (bf16 or fp32), 16-byte aligned.
 *   - Sequence lengths live on the device (int32[B]): t_b = tokens already cached for sequence b.
 *   - On a host without a GPU lckv_cache_alloc still returns a handle: the pairing table, the planners and every
 *     argument check work on it, and each call that would enqueue work returns LCKV_ERR_HIP after its checks.
 *   - Measurement and tuning hooks (kernel timing, read probe, forced split size, load policy, prefill tile) are
 *     declared in lckv_tools.h, not here.
 *
 * Physical cache layout (private to the library, stated so that storage can be sized and reasoned about):
 * a slot is an array of "page pairs"; a page pair holds 16 consecutive positions of one kv head, first the K
 * page then the V page, each 16*D*elem bytes, stored in the register order of the matrix instructions that
 * consume them (bf16) or row-major [16][D] (fp32).  Contiguous caches index page pairs as
 * [b][kv_head][page]; paged caches as [physical_block][kv_head] with physical_block = table[b][page].
 * Only lckv_append_kv / lckv_cache_load_dense write it and lckv_cache_read reads it back logically.
 */
#ifndef LCKV_H
#define LCKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LCKV_OK 0
#define LCKV_ERR_NULL (-1)          /* a required pointer is NULL */
#define LCKV_ERR_CONFIG (-2)        /* unsupported or inconsistent lckv_config field */
#define LCKV_ERR_LAYER (-3)         /* layer or slot index out of range */
#define LCKV_ERR_NOT_PRODUCER (-4)  /* lckv_append_kv on a layer whose K/V no slot stores */
#define LCKV_ERR_BATCH (-5)         /* B < 1 or B > B_max */
#define LCKV_ERR_LENGTH (-6)        /* max_len_hint (+1 new token) exceeds the cache capacity */
#define LCKV_ERR_WORKSPACE (-7)     /* workspace NULL, misaligned or smaller than lckv_workspace_bytes */
#define LCKV_ERR_ALIGN (-8)         /* a device pointer is not aligned as required */
#define LCKV_ERR_BLOCK_TABLE (-9)   /* paged cache used before lckv_cache_set_block_table, or bad table */
#define LCKV_ERR_HIP (-10)          /* a HIP runtime call failed (launch, copy, event) */
#define LCKV_ERR_MASK (-11)         /* warmup_mask passed to a call differs from the cache's */
#define LCKV_ERR_STORAGE (-12)      /* kv_storage smaller than lckv_cache_bytes */
#define LCKV_ERR_RANGE (-13)        /* position / count out of range in a cache accessor */

#define LCKV_BF16 0
#define LCKV_F32 1

/* Which layer produces the shared slot (the paper says "the top layer", Section 2.1, and leaves open what
 * that means when the topmost layers are warmup layers):
 *   TOP_OF_CONDENSED (default): the topmost non-warmup layer; every warmup layer has a slot of its own,
 *                               so there are w + 1 slots for 0 < w < L.
 *   LAST_LAYER: layer L-1 even when it is a warmup layer (it then reads that slot with itself visible). */
#define LCKV_PAIR_TOP_OF_CONDENSED 0
#define LCKV_PAIR_LAST_LAYER 1

/* Sticky device-side error bits reported by lckv_last_device_error. */
#define LCKV_DEV_ERR_CAPACITY 1     /* a sequence length reached the capacity; the access was skipped/clamped */
#define LCKV_DEV_ERR_BLOCK 2        /* a block-table entry was outside [0, num_blocks); the page was skipped */
#define LCKV_DEV_ERR_BARRIER 4      /* lckv_step_one_launch: a wait at the device-wide barrier between two layers ran
                                       into its time bound; the workgroups left the kernel, the step is incomplete */

/* Size of the library's own scratch array (device memory inside the loaded library, one copy per GPU), used by
 * lckv_step_static_scratch. */
#define LCKV_STATIC_SCRATCH_BYTES (32u << 20)

typedef struct lckv_cache lckv_cache; /* opaque */

typedef struct lckv_config {
    int32_t L;            /* layers, 1..1024 */
    int32_t Hq;           /* query heads */
    int32_t Hkv;          /* kv heads; Hq % Hkv == 0 and Hq / Hkv <= 16; query head h reads kv head h / (Hq/Hkv) */
    int32_t D;            /* head dimension: 64 or 128 */
    int32_t dtype;        /* LCKV_BF16 (bf16 storage, fp32 accumulation) or LCKV_F32 */
    int32_t B_max;        /* sequences the cache can hold (contiguous layout); upper bound on B in every call */
    int32_t T_max;        /* contiguous layout: positions per sequence (rounded up to a multiple of 16) */
    int32_t page_size;    /* 0 = contiguous, 16 = paged with a block table */
    int64_t num_blocks;   /* paged only: physical 16-token blocks per slot */
    const uint8_t *warmup_mask; /* host, L bytes, 1 = warmup layer (Section 2.1); copied */
    int32_t pairing_rule; /* LCKV_PAIR_* */
    float scale;          /* softmax scale; 0 means 1/sqrt(D) (the paper does not state it) */
    /* Sink + window policy (Section 3.3, integration with StreamingLLM: only the K/V of the first few tokens and
     * of the recent tokens are kept).  window_tokens = 0: off.  Otherwise every slot keeps the first sink_tokens
     * positions and a ring of the last window_tokens positions (position t >= sink lives in entry
     * sink + (t - sink) % window), sequences may grow without bound, a condensed layer attends to the sinks and
     * the last `window` previous tokens, a warmup layer to the sinks and the last `window` tokens including the
     * one being decoded.  Needs sink_tokens + window_tokens <= the layout's capacity (T_max, or 16 * blocks per
     * sequence).  RoPE re-indexing inside the window is outside this library: K arrives position-encoded. */
    int32_t sink_tokens;
    int32_t window_tokens;
} lckv_config;

/* Bytes of device storage a cache with this config needs (all slots).  Host only. */
int lckv_cache_bytes(const lckv_config *cfg, size_t *bytes);

/* Footprint planner: the largest number of sequences of cfg->T_max positions (contiguous layout; cfg->B_max is
 * ignored) whose caches fit in budget_bytes.  The cache size is slots * B * T * 2 * Hkv * D * elem, so the gain
 * over a standard transformer (all layers warmup) is L / slots - the memory side of the paper's batch-size
 * claims (Section 3.1, Table 1).  Host only. */
int lckv_plan_max_batch(const lckv_config *cfg, size_t budget_bytes, int32_t *max_batch);

/* Build the pairing table of Section 2.1 from cfg->warmup_mask and bind the caller's device storage
 * (kv_storage, 256-byte aligned, at least lckv_cache_bytes; NOT cleared, NOT freed by the library).
 * Allocates the handle and small device tables.  All config errors are found before any GPU call. */
int lckv_cache_alloc(const lckv_config *cfg, void *kv_storage, size_t kv_bytes, lckv_cache **out);
int lckv_cache_free(lckv_cache *cache);

/* Paged caches: device table int32[B_max][max_blocks_per_seq]; entry [b][p] is the physical block holding
 * positions 16p..16p+15 of sequence b in EVERY slot (one table serves all slots).  Borrowed, not copied: it
 * must stay valid, and may be updated by the caller between calls.  Capacity per sequence becomes
 * 16 * max_blocks_per_seq; with the sink + window policy a row must hold sink_tokens + window_tokens positions
 * (LCKV_ERR_BLOCK_TABLE otherwise, here and in every call that would index such a row). */
int lckv_cache_set_block_table(lckv_cache *cache, const int32_t *dev_table, int32_t max_blocks_per_seq);

/* Pairing table (Section 2.1): number of slots; the slot layer `layer` reads and whether the token being
 * decoded is visible to it (1 for warmup layers, 0 for condensed layers: diagonal mask); the layer whose new
 * K/V go to `slot`.  Slots are numbered by ascending producer layer.  Host only. */
int lckv_n_slots(const lckv_cache *cache, int32_t *n_slots);
int lckv_kv_slot(const lckv_cache *cache, int32_t layer, int32_t *slot, int32_t *self_visible);
int lckv_slot_producer(const lckv_cache *cache, int32_t slot, int32_t *layer);

/* Store the new token's K/V of a producing layer (Section 2.1: only the K/V of the top layer - and of the warmup
 * layers, which keep standard attention - are computed and cached; Section 3.3 for where the new token goes and
 * when under the sink + window policy): for every b < B,
 *   K[slot(layer)][b][t_b] = k_new[b], V[...] = v_new[b]      (bits copied unchanged)
 * k_new, v_new: device [B][Hkv][D].  dev_seq_lens: device int32[B], read, not changed.
 * A sequence already at capacity is skipped and LCKV_DEV_ERR_CAPACITY is raised on the device (never with the
 * sink + window policy, where the entry of the oldest recent token is overwritten).  With that policy the new
 * K/V of the shared slot must be appended AFTER the condensed layers of the step have attended (lckv_step does
 * so): before, it would overwrite a token they still see.  Warmup layers append before their own attention. */
int lckv_append_kv(lckv_cache *cache, int32_t layer, const void *k_new, const void *v_new,
                   const int32_t *dev_seq_lens, int32_t B, void *hip_stream);

/* Attention of one layer's queries for one decode step (Section 2.1):
 *   out[b][h] = softmax_j(scale * <q[b][h], K[slot][b][j][h/G]>) . V[slot][b][j][h/G],   j < n_b,
 * n_b = t_b for a condensed layer (diagonal masked), t_b + 1 for a warmup layer (the caller has appended
 * this layer's new K/V first).  n_b = 0 gives the zero vector (the paper's zero dummy K/V for the first
 * token).  q, out: device [B][Hq][D].  warmup_mask: optional host array of L bytes; if not NULL it must
 * equal the cache's mask (LCKV_ERR_MASK otherwise).  max_len_hint: host-side upper bound on every t_b
 * (lengths above it are clamped and raise LCKV_DEV_ERR_CAPACITY); it fixes the split of the key range.
 * workspace: device scratch for split partials, 256-byte aligned, at least lckv_workspace_bytes. */
int lckv_decode_attention(lckv_cache *cache, int32_t layer, const void *q, void *out,
                          const int32_t *dev_seq_lens, const uint8_t *warmup_mask, int32_t B,
                          int32_t max_len_hint, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Attention of all prompt tokens of one layer in one pass, for the parallel computation of Section 2.2 and the
 * iterative prompt encoding of Section 2.3 (m + b iterations over the whole prompt, each pairing the condensed
 * layers with the top layer's K/V of the previous iteration, zeros before the first):
 *   out[b][i][h] = softmax_j(scale * <q[b][i][h], K[slot][b][j][h/G]>) . V[slot][b][j][h/G]
 * over j < i for a condensed layer (diagonal masked; token 0 sees nothing: zero vector) and j <= i for a warmup
 * layer, for i < prompt_len_b; rows i >= prompt_len_b are written as zeros.  The K/V are read from the cache:
 * the caller first imports them with lckv_cache_load_dense - a warmup layer's own K/V of this iteration before
 * its attention, the top layer's K/V into the shared slot at the END of an iteration - so after the last
 * iteration the cache holds the prompt and decoding can start.  q, out: device [B][S][Hq][D]; dev_prompt_lens:
 * device int32[B], each <= S; S <= capacity.  Not available with the sink + window policy.  Only enqueues.
 * The bf16 kernel's workgroup-to-task map is laid out for MI355X's 8 XCDs with round-robin dispatch of
 * workgroups (all row chunks of a head on one XCD, sharing its L2); on another partitioning the results are the
 * same and only the cache reuse changes. */
int lckv_prefill_attention(lckv_cache *cache, int32_t layer, const void *q, void *out,
                           const int32_t *dev_prompt_lens, int32_t B, int32_t S, void *hip_stream);

/* The projections either side of the attention for one decode step of `layer` (Section 2.1: every layer maps
 * the hidden state to queries, but only a layer that produces a cache slot - a warmup layer, or the condensed
 * layer that owns the shared cache - computes keys and values; the other layers have no W_K, W_V):
 *   q_out[b] = rot_{t_b}(x[b] . w_q^T)                                    every layer
 *   K[slot][b][t_b] = rot_{t_b}(x[b] . w_k^T),  V[slot][b][t_b] = x[b] . w_v^T    producing layers only
 * i.e. for a producing layer the call also performs lckv_append_kv of the new token, straight from the product -
 * unless k_out and v_out (device [B][Hkv][D], both or neither) are given: then the rotated keys and the values go
 * there instead, the cache is not touched, and the caller stores them with lckv_append_kv when the time has come.
 * That is how the condensed producing layer is driven under the sink + window policy (Section 3.3), where its new
 * K/V may only replace a ring entry after the layer's own attention; storing at once is refused there
 * (LCKV_ERR_CONFIG).
 * rot_t is the rotary position embedding in the Llama convention (the paper trains Llama models and does not
 * restate it): within a head, channel i < D/2 is paired with channel i + D/2 and the pair is turned by the
 * angle t * rope_base^(-2i/D); rope_base <= 0 means no rotation.  Products are accumulated in fp32 (bf16 caches:
 * one launch; the hidden dimension is cut in four whose sums are added in a fixed order, so results do not vary
 * from run to run) or in fp64 (fp32 caches, the parity mode: two launches), rotated in fp32 and rounded once to
 * the element type.
 * x: device [B][hidden] in the cache's element type; w_q (Hq*D rows), w_k, w_v (Hkv*D rows): device, PACKED by
 * lckv_pack_projection_weight, 16-byte aligned; bf16 needs hidden % 256 == 0.  w_k and w_v must both be given
 * for a producing layer (LCKV_ERR_NULL) and must both be NULL for any other (LCKV_ERR_NOT_PRODUCER: such
 * parameters do not exist).  q_out: device [B][Hq][D].  dev_seq_lens: read, not changed.  workspace: device,
 * 256-byte aligned, at least lckv_project_workspace_bytes (0 for bf16 caches: then it may be NULL); its contents
 * need not be kept between calls.
 * k_out / v_out on a layer that produces no slot: LCKV_ERR_NOT_PRODUCER.  Only enqueues. */
int lckv_project_qkv(lckv_cache *cache, int32_t layer, const void *x, int32_t hidden, const void *w_q,
                     const void *w_k, const void *w_v, void *q_out, void *k_out, void *v_out,
                     const int32_t *dev_seq_lens, int32_t B, float rope_base, void *workspace,
                     size_t workspace_bytes, void *hip_stream);
int lckv_project_workspace_bytes(const lckv_cache *cache, int32_t B, int32_t hidden, size_t *bytes);
/* Weights are handed to lckv_project_qkv in the order the matrix instructions take them (made once, when the
 * model is loaded).  w: device [n_rows][hidden] row-major ("out features x in features"), n_rows a multiple of the
 * head dimension D (whole heads); w_packed: device, same size, must not overlap w.  bf16: tiles of 16 rows, each
 * tile [hidden/32 steps][4 channel octets kb][16 rows r][8 channels] (lane kb*16 + r of a wave holds channels
 * 32*step + 8*kb .. +7 of the tile's row r), a tile's image contiguous; tile t holds, of head t / (D/16), the
 * rows of 8 rotary pairs: r < 8: channel 8 (t % (D/16)) + r, r >= 8: its partner D/2 further on - so the
 * rotation needs nothing outside one wave.  fp32: a plain copy.  Only enqueues. */
int lckv_pack_projection_weight(const lckv_cache *cache, const void *w, void *w_packed, int32_t n_rows,
                                int32_t hidden, void *hip_stream);

/* The whole decode step of Section 2.1 (Figure 1b) for one new token per sequence: layers in index order (layer
 * l+1 starts after layer l has finished: in the model its query depends on layer l's output, the "bottom-up
 * computation" of that section); a warmup layer's K/V are appended just before its attention (it sees itself),
 * the shared slot's new K/V just after the attention of the condensed layer that produces them (the diagonal is
 * masked, so no condensed layer sees them in this step); at the end every t_b is incremented on the device.
 * With the sink + window policy max_len_hint may exceed the capacity.
 *   q_all, out_all: device [L][B][Hq][D];  k_new_all, v_new_all: device [n_slots][B][Hkv][D], slot order. */
int lckv_step(lckv_cache *cache, const void *q_all, const void *k_new_all, const void *v_new_all, void *out_all,
              int32_t *dev_seq_lens, int32_t B, int32_t max_len_hint, void *workspace, size_t workspace_bytes,
              void *hip_stream);

/* The same step in ONE kernel launch (bf16 caches; LCKV_ERR_CONFIG otherwise), for slots so small that a layer's pass
 * over its slot lasts about as long as a kernel launch (the TinyLlama-shaped workload: 22 layers of 128 MiB).  A
 * grid that is resident all at once walks the layers in index order; a device-wide barrier ends every layer's
 * attention, so layer l+1 still starts only when layer l's results are complete; the merge of layer l's split
 * partials and the shared slot's append run right after that barrier.  Same units of work and same arithmetic
 * as lckv_step: the results are the same bit for bit.  workspace: at least lckv_step_one_launch_workspace_bytes
 * (two sets of split partials, used in turn).  The barrier's waits are bounded (a few seconds by default,
 * lckv_set_barrier_wait_ms in lckv_tools.h): if one expires, LCKV_DEV_ERR_BARRIER is raised and every workgroup
 * leaves the kernel.  A cooperative launch: do not capture it in a HIP graph, and enqueue at most one such step
 * per cache at a time (all launches of a cache share two barrier counters, used in turn). */
int lckv_step_one_launch(lckv_cache *cache, const void *q_all, const void *k_new_all, const void *v_new_all,
                         void *out_all, int32_t *dev_seq_lens, int32_t B, int32_t max_len_hint, void *workspace,
                         size_t workspace_bytes, void *hip_stream);
int lckv_step_one_launch_workspace_bytes(const lckv_cache *cache, int32_t B, int32_t max_len_hint, size_t *bytes);

/* lckv_step for callers that cannot allocate device memory and so have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace,
 * same kernels, same results bit for bit; the split partials go to the library's own scratch array of
 * LCKV_STATIC_SCRATCH_BYTES (part of the loaded library, one copy per GPU, held until the process ends).  The
 * call allocates nothing.  LCKV_ERR_WORKSPACE if lckv_workspace_bytes for this B and max_len_hint exceeds
 * LCKV_STATIC_SCRATCH_BYTES.  Nothing in the array has to start at zero (every split writes its partial before
 * the merge reads it), and it keeps the last call's contents.  All handles and all calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU (two streams, two threads) race - serialise them. */
int lckv_step_static_scratch(lckv_cache *cache, const void *q_all, const void *k_new_all, const void *v_new_all,
                             void *out_all, int32_t *dev_seq_lens, int32_t B, int32_t max_len_hint,
                             void *hip_stream);

/* Bytes of workspace lckv_decode_attention / lckv_step need for this B and max_len_hint.  Host only. */
int lckv_workspace_bytes(const lckv_cache *cache, int32_t B, int32_t max_len_hint, size_t *bytes);

/* Bulk import (e.g. after prompt encoding): positions [0, min(T, t_b)) of every sequence b < B of `slot` are
 * written from dense device tensors k, v of shape [B][T][Hkv][D]; dev_seq_lens (device int32[B]) may be NULL,
 * then all T positions are written.  Bits copied unchanged.  This is the store of Section 2.3's prompt encoding:
 * each of its m + b iterations imports a producing layer's K/V of all prompt tokens before the next reads them. */
int lckv_cache_load_dense(lckv_cache *cache, int32_t slot, const void *k, const void *v,
                          const int32_t *dev_seq_lens, int32_t B, int32_t T, void *hip_stream);

/* Logical read-back for tests and snapshots: positions [pos, pos + n_pos) of sequence b in `slot` are copied
 * to host_k, host_v as [n_pos][Hkv][D].  Allocates a temporary and SYNCHRONISES the device. */
int lckv_cache_read(lckv_cache *cache, int32_t slot, int32_t b, int32_t pos, int32_t n_pos, void *host_k,
                    void *host_v);

/* Read and clear the sticky device error bits (LCKV_DEV_ERR_*).  SYNCHRONISES the device. */
int lckv_last_device_error(lckv_cache *cache, int32_t *bits);

const char *lckv_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* LCKV_H */
