// Host side of liblckv: argument checks, the pairing table of Section 2.1, split planning and kernel launches.
#include <math.h>
#include <string.h>

#include <mutex>
#include <new>

#include "lckv_internal.h"

using namespace lckv;

// Scratch of lckv_step_static_scratch, the entry point for callers that cannot allocate: device memory that is
// part of the loaded library, one copy per GPU, held until the process ends.  The name is a host-side stand-in,
// never a device address: host code uses the pointer hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[LCKV_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // per device: where that GPU's copy of `scratch` lives

// The current device's copy of `scratch`; asked of the runtime once per device, with that device current.
int static_scratch_of_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LCKV_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LCKV_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return LCKV_OK;
}

constexpr uint64_t kMagic = 0x4c434b5643414348ull;  // "LCKVCACH"
constexpr size_t kProfilePairs = 4096;
constexpr int kTargetWorkgroups = 2048;  // 8 per compute unit: enough to hide the tail of the last wave of groups
constexpr int kMinSplitTokens = 256;
constexpr int kMinSplitBytes = 256 * 1024;  // K/V bytes of one kv head a split should at least stream: below that
                                            // a workgroup is over before its loads are up to speed, and the
                                            // merge of the partial results costs more than the split gains
constexpr double kLastLevelCacheBytes = 256.0 * 1024 * 1024;  // MI355X Infinity Cache

bool valid(const lckv_cache *c) { return c && c->magic == kMagic; }

int elem_bytes(int dtype) { return dtype == LCKV_BF16 ? 2 : 4; }

int check_config(const lckv_config *cfg) {
    if (!cfg) return LCKV_ERR_NULL;
    if (!cfg->warmup_mask) return LCKV_ERR_NULL;
    if (cfg->L < 1 || cfg->L > 1024) return LCKV_ERR_CONFIG;
    if (cfg->Hq < 1 || cfg->Hkv < 1 || cfg->Hq % cfg->Hkv != 0) return LCKV_ERR_CONFIG;
    if (cfg->Hq / cfg->Hkv > kMaxGroup) return LCKV_ERR_CONFIG;
    if (cfg->Hq > 65535) return LCKV_ERR_CONFIG;
    if (cfg->D != 64 && cfg->D != 128) return LCKV_ERR_CONFIG;
    if (cfg->dtype != LCKV_BF16 && cfg->dtype != LCKV_F32) return LCKV_ERR_CONFIG;
    if (cfg->B_max < 1 || cfg->B_max > 65535) return LCKV_ERR_CONFIG;
    // one thread per output element in the small kernels: a launch holds fewer than 2^32 threads
    if ((int64_t)cfg->B_max * cfg->Hq * cfg->D >= ((int64_t)1 << 31)) return LCKV_ERR_CONFIG;
    if (cfg->page_size != 0 && cfg->page_size != kPage) return LCKV_ERR_CONFIG;
    if (cfg->page_size == 0 && (cfg->T_max < 1 || cfg->T_max > (1 << 24))) return LCKV_ERR_CONFIG;
    if (cfg->page_size == kPage && (cfg->num_blocks < 1 || cfg->num_blocks > (int64_t)1 << 31)) return LCKV_ERR_CONFIG;
    if (cfg->pairing_rule != LCKV_PAIR_TOP_OF_CONDENSED && cfg->pairing_rule != LCKV_PAIR_LAST_LAYER)
        return LCKV_ERR_CONFIG;
    if (!(cfg->scale >= 0.f) || isinf(cfg->scale)) return LCKV_ERR_CONFIG;
    if (cfg->sink_tokens < 0 || cfg->window_tokens < 0) return LCKV_ERR_CONFIG;
    if (cfg->window_tokens == 0 && cfg->sink_tokens != 0) return LCKV_ERR_CONFIG;
    if ((int64_t)cfg->sink_tokens + cfg->window_tokens > (1 << 24)) return LCKV_ERR_CONFIG;
    if (cfg->page_size == 0 && cfg->window_tokens > 0 &&
        cfg->sink_tokens + cfg->window_tokens > (cfg->T_max + kPage - 1) / kPage * kPage)
        return LCKV_ERR_CONFIG;
    for (int l = 0; l < cfg->L; ++l)
        if (cfg->warmup_mask[l] > 1) return LCKV_ERR_CONFIG;
    return LCKV_OK;
}

// Section 2.1: warmup layers keep standard attention on caches of their own; all other layers read the one
// cache of "the top layer" with the diagonal masked.  Slots are numbered by ascending producer layer.
void build_pairing(const lckv_config &cfg, std::vector<int32_t> &kv_slot, std::vector<int32_t> &self_visible,
                   std::vector<int32_t> &producer) {
    const int L = cfg.L;
    const uint8_t *warm = cfg.warmup_mask;
    int shared_from = -1;
    for (int l = L - 1; l >= 0; --l)
        if (!warm[l]) {
            shared_from = cfg.pairing_rule == LCKV_PAIR_LAST_LAYER ? L - 1 : l;
            break;
        }
    std::vector<int32_t> slot_of(L, -1);
    producer.clear();
    for (int l = 0; l < L; ++l)
        if (warm[l] || l == shared_from) {
            slot_of[l] = (int32_t)producer.size();
            producer.push_back(l);
        }
    kv_slot.assign(L, 0);
    self_visible.assign(L, 0);
    for (int l = 0; l < L; ++l) {
        kv_slot[l] = warm[l] ? slot_of[l] : slot_of[shared_from];
        self_visible[l] = warm[l] ? 1 : 0;
    }
}

struct Geometry {
    int32_t n_slots, pages_per_seq, page_bytes;
    size_t slot_bytes;
};

Geometry geometry(const lckv_config &cfg) {
    std::vector<int32_t> a, b, prod;
    build_pairing(cfg, a, b, prod);
    Geometry g;
    g.n_slots = (int32_t)prod.size();
    g.page_bytes = kPage * cfg.D * elem_bytes(cfg.dtype);
    g.pages_per_seq = cfg.page_size ? 0 : (cfg.T_max + kPage - 1) / kPage;
    size_t pairs = cfg.page_size ? (size_t)cfg.num_blocks * cfg.Hkv
                                 : (size_t)cfg.B_max * cfg.Hkv * (size_t)g.pages_per_seq;
    g.slot_bytes = pairs * 2 * (size_t)g.page_bytes;
    return g;
}

// Positions a sequence can hold at once: the layout's capacity, or sink + window under that policy.
int kept_capacity(const lckv_cache *c) {
    return c->cfg.window_tokens > 0 ? c->cfg.sink_tokens + c->cfg.window_tokens : c->capacity;
}

// Upper bound on the keys a query with `hint` cached tokens (+ itself if `self`) attends to.
int visible_bound(const lckv_cache *c, int hint, int self) {
    int64_t n = (int64_t)hint + self;
    if (c->cfg.window_tokens > 0 && n > kept_capacity(c)) n = kept_capacity(c);
    return (int)n;
}

SlotView slot_view(const lckv_cache *c, int slot) {
    SlotView v;
    v.base = c->storage + (size_t)slot * c->slot_bytes;
    v.table = c->table;
    v.max_blocks = c->max_blocks;
    v.num_blocks = c->cfg.num_blocks;
    v.pages_per_seq = c->pages_per_seq;
    v.Hkv = c->cfg.Hkv;
    v.page_bytes = c->page_bytes;
    v.capacity = kept_capacity(c);
    v.ring_sink = c->cfg.sink_tokens;
    v.ring_window = c->cfg.window_tokens;
    return v;
}

struct SplitPlan {
    int32_t tokens, n_splits;
    int32_t waves;  // per workgroup: 4, or 8 / 16 where one wide workgroup replaces 2 / 3-4 splits (bf16 only)
};

// Keys per split: fixed by B, Hkv and the length bound only, never by an individual sequence's length, so a
// sequence's result does not depend on which other sequences share the batch.
SplitPlan plan_splits(const lckv_cache *c, int B, int max_n, bool allow_wide = true) {
    SplitPlan p;
    p.waves = 4;
    if (max_n < 1) max_n = 1;
    if (c->forced_split_tokens > 0) {
        p.tokens = c->forced_split_tokens;
    } else {
        int64_t units = (int64_t)B * c->cfg.Hkv;
        int64_t want = (kTargetWorkgroups + units - 1) / units;
        int64_t min_tokens = kMinSplitBytes / (2 * (int64_t)c->cfg.D * elem_bytes(c->cfg.dtype));
        if (min_tokens < kMinSplitTokens) min_tokens = kMinSplitTokens;
        int64_t most = max_n / min_tokens;
        if (most < 1) most = 1;
        if (want > most) want = most;
        if (want < 1) want = 1;
        int64_t t = (max_n + want - 1) / want;
        p.tokens = (int32_t)((t + 63) / 64 * 64);
    }
    p.n_splits = (max_n + p.tokens - 1) / p.tokens;
    if (allow_wide && c->cfg.dtype == LCKV_BF16) {
        // A few splits only: the waves of those splits go into ONE workgroup instead, which merges them through
        // LDS - the same number of waves stream the same keys, but no partial results go through memory and no
        // merge kernel follows (for small slots that kernel and its launch are a fifth of a layer's time).  The
        // merge buffer in LDS bounds the width: 16 waves at D = 64, 8 at D = 128.
        const int widest = c->cfg.D == 64 ? 16 : 8;
        int waves = 4;
        if (c->forced_waves > 0)
            waves = c->forced_waves <= widest ? c->forced_waves : widest;
        else if (c->forced_split_tokens == 0 && p.n_splits == 2)
            waves = 8;
        else if (c->forced_split_tokens == 0 && (p.n_splits == 3 || p.n_splits == 4) && widest == 16)
            waves = 16;
        if (waves > 4 && c->forced_waves == 0) {
            p.tokens = (max_n + 63) / 64 * 64;
            p.n_splits = 1;
        }
        p.waves = waves;
    }
    return p;
}

size_t workspace_need(const lckv_cache *c, int B, int n_splits) {
    if (n_splits <= 1) return 0;
    size_t rows = (size_t)n_splits * B * c->cfg.Hq;
    size_t o = rows * c->cfg.D * sizeof(float);
    size_t ml = rows * sizeof(float2);
    return (o + 255) / 256 * 256 + (ml + 255) / 256 * 256;
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

int attention_impl(lckv_cache *c, int layer, const void *q, void *out, const int32_t *lens, int B, int max_len_hint,
                   void *workspace, size_t workspace_bytes, hipStream_t stream) {
    const lckv_config &cfg = c->cfg;
    const int self = c->self_visible[layer];
    const int max_n = visible_bound(c, max_len_hint, self);
    SplitPlan sp = plan_splits(c, B, max_n);
    size_t need = workspace_need(c, B, sp.n_splits);
    if (need > 0) {
        if (!workspace || !aligned(workspace, 256) || workspace_bytes < need) return LCKV_ERR_WORKSPACE;
    }
    if (c->host_only) return LCKV_ERR_HIP;
    AttnParams p;
    p.slot = slot_view(c, c->kv_slot[layer]);
    p.q = q;
    p.out = out;
    p.seq_lens = lens;
    size_t rows = (size_t)sp.n_splits * B * cfg.Hq;
    p.part_o = (float *)workspace;
    p.part_ml = need ? (float2 *)((char *)workspace + (rows * cfg.D * sizeof(float) + 255) / 256 * 256) : nullptr;
    p.dev_err = c->dev_err;
    p.B = B;
    p.Hq = cfg.Hq;
    p.Hkv = cfg.Hkv;
    p.G = cfg.Hq / cfg.Hkv;
    p.self_visible = self;
    p.max_n = max_n;
    p.clamp_is_policy = cfg.window_tokens > 0 && max_n == kept_capacity(c);
    p.split_tokens = sp.tokens;
    p.n_splits = sp.n_splits;
    p.waves = sp.waves;
    p.scale_log2e = c->scale * 1.4426950408889634f;
    // K/V of one layer's pass: B * n * 2 * Hkv * D * elem bytes.  Past the size of the last-level cache nothing
    // of it survives until the next layer reads the slot again, and the nontemporal hint makes the stream faster.
    const double pass_bytes = (double)B * max_n * 2.0 * cfg.Hkv * cfg.D * elem_bytes(cfg.dtype);
    p.unit_mul = 1;
    for (int prime : {2731, 1571, 7919, 104729})  // the first that does not divide the number of units
        if (((int64_t)B * cfg.Hkv) % prime != 0) {
            p.unit_mul = prime;
            break;
        }
    p.nontemporal = c->load_policy == LCKV_LOAD_NONTEMPORAL ||
                    (c->load_policy == LCKV_LOAD_AUTO && pass_bytes > kLastLevelCacheBytes);

    const bool timed = c->profiling && c->ev_used + 2 <= c->ev.size();
    if (timed && hipEventRecord(c->ev[c->ev_used], stream) != hipSuccess) return LCKV_ERR_HIP;
    hipError_t e = cfg.dtype == LCKV_BF16 ? launch_attn_bf16(p, cfg.D, stream) : launch_attn_f32(p, cfg.D, stream);
    if (e != hipSuccess) return LCKV_ERR_HIP;
    if (timed) {
        if (hipEventRecord(c->ev[c->ev_used + 1], stream) != hipSuccess) return LCKV_ERR_HIP;
        c->ev_used += 2;
    }
    if (sp.n_splits > 1 && launch_combine(p, cfg.D, cfg.dtype, stream) != hipSuccess) return LCKV_ERR_HIP;
    return LCKV_OK;
}

// What every call that touches a slot checks first: the batch fits, a paged cache has its table, and under the
// sink + window policy the kept positions fit the layout (a ring entry maps to page entry / 16 of the
// sequence's table row: a row shorter than sink + window would be indexed past its end).
int check_slot_access(const lckv_cache *c, int B) {
    if (B < 1 || B > c->cfg.B_max) return LCKV_ERR_BATCH;
    if (c->cfg.page_size && !c->table) return LCKV_ERR_BLOCK_TABLE;
    if (c->cfg.window_tokens > 0 && kept_capacity(c) > c->capacity) return LCKV_ERR_BLOCK_TABLE;
    return LCKV_OK;
}

int check_call(const lckv_cache *c, int B, int max_len_hint, int extra) {
    int rc = check_slot_access(c, B);
    if (rc != LCKV_OK) return rc;
    if (max_len_hint < 0) return LCKV_ERR_LENGTH;
    if (c->cfg.window_tokens == 0 && (int64_t)max_len_hint + extra > c->capacity) return LCKV_ERR_LENGTH;
    return LCKV_OK;
}

// Per layer, for the one-launch step: the slot it reads, whether it sees itself, the slot it produces and when that
// slot's new K/V may be stored.  A warmup layer's private slot (read by nobody else): at the start of the step.  A
// slot that other layers read too: by a producer that sees itself, right before its own attention (the layers
// below have read the slot by then); by a condensed producer, after its own attention (no condensed layer sees the
// token being decoded, and under the sink + window policy the entry it replaces is still read until then).
int upload_layer_table(lckv_cache *c) {
    const int L = c->cfg.L;
    std::vector<int32_t> t(4 * (size_t)L);
    for (int l = 0; l < L; ++l) {
        int produced = -1;
        for (int s = 0; s < c->n_slots; ++s)
            if (c->producer[s] == l) produced = s;
        int when = kAppendNone;
        if (produced >= 0) {
            bool shared = false;
            for (int k = 0; k < L; ++k)
                if (k != l && c->kv_slot[k] == produced) shared = true;
            when = !c->self_visible[l] ? kAppendAfterOwnAttention : shared ? kAppendBeforeOwnAttention : kAppendAtStart;
        }
        t[4 * l] = c->kv_slot[l];
        t[4 * l + 1] = c->self_visible[l];
        t[4 * l + 2] = produced;
        t[4 * l + 3] = when;
    }
    if (hipMalloc((void **)&c->dev_layer_table, t.size() * sizeof(int32_t)) != hipSuccess) return LCKV_ERR_HIP;
    if (hipMemcpy(c->dev_layer_table, t.data(), t.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess)
        return LCKV_ERR_HIP;
    return LCKV_OK;
}

// The slot whose K/V `layer` produces, or -1.
int produced_slot(const lckv_cache *c, int layer) {
    for (int s = 0; s < c->n_slots; ++s)
        if (c->producer[s] == layer) return s;
    return -1;
}

}  // namespace

extern "C" {

int lckv_cache_bytes(const lckv_config *cfg, size_t *bytes) {
    if (!bytes) return LCKV_ERR_NULL;
    int rc = check_config(cfg);
    if (rc != LCKV_OK) return rc;
    Geometry g = geometry(*cfg);
    *bytes = g.slot_bytes * (size_t)g.n_slots;
    return LCKV_OK;
}

int lckv_plan_max_batch(const lckv_config *cfg, size_t budget_bytes, int32_t *max_batch) {
    if (!max_batch) return LCKV_ERR_NULL;
    if (!cfg) return LCKV_ERR_NULL;
    lckv_config one = *cfg;
    one.B_max = 1;
    int rc = check_config(&one);
    if (rc != LCKV_OK) return rc;
    if (one.page_size != 0) return LCKV_ERR_CONFIG;
    Geometry g = geometry(one);
    size_t per_sequence = g.slot_bytes * (size_t)g.n_slots;
    size_t n = budget_bytes / per_sequence;
    *max_batch = n > 65535 ? 65535 : (int32_t)n;
    return LCKV_OK;
}

int lckv_cache_alloc(const lckv_config *cfg, void *kv_storage, size_t kv_bytes, lckv_cache **out) {
    if (!out) return LCKV_ERR_NULL;
    *out = nullptr;
    int rc = check_config(cfg);
    if (rc != LCKV_OK) return rc;
    if (!kv_storage) return LCKV_ERR_NULL;
    if (!aligned(kv_storage, 256)) return LCKV_ERR_ALIGN;
    Geometry g = geometry(*cfg);
    if (kv_bytes < g.slot_bytes * (size_t)g.n_slots) return LCKV_ERR_STORAGE;

    lckv_cache *c = new (std::nothrow) lckv_cache();
    if (!c) return LCKV_ERR_HIP;
    c->magic = kMagic;
    c->cfg = *cfg;
    c->warm.assign(cfg->warmup_mask, cfg->warmup_mask + cfg->L);
    c->cfg.warmup_mask = c->warm.data();
    build_pairing(c->cfg, c->kv_slot, c->self_visible, c->producer);
    c->n_slots = g.n_slots;
    c->storage = (char *)kv_storage;
    c->slot_bytes = g.slot_bytes;
    c->pages_per_seq = g.pages_per_seq;
    c->page_bytes = g.page_bytes;
    c->table = nullptr;
    c->max_blocks = 0;
    c->capacity = cfg->page_size ? 0 : g.pages_per_seq * kPage;
    c->forced_split_tokens = 0;
    c->forced_waves = 0;
    c->load_policy = LCKV_LOAD_AUTO;
    c->prefill_query_blocks = 0;  // 0: chosen per head dimension at launch
    c->scale = cfg->scale > 0.f ? cfg->scale : 1.0f / sqrtf((float)cfg->D);
    c->profiling = false;
    c->ev_used = 0;
    c->dev_err = nullptr;
    c->dev_layer_table = nullptr;
    c->step_launches = 0;
    c->barrier_wait_ms = 2000.0;
    c->scratch = nullptr;
    // A host without a GPU still gets a handle: the pairing table, the planners and every argument check work
    // on it, and each call that would enqueue work returns LCKV_ERR_HIP after its checks.
    int n_dev = 0;
    c->host_only = hipGetDeviceCount(&n_dev) != hipSuccess || n_dev < 1;
    if (c->host_only) {
        (void)hipGetLastError();
    } else if (hipMalloc((void **)&c->dev_err, 256) != hipSuccess || hipMemset(c->dev_err, 0, 256) != hipSuccess ||
               static_scratch_of_current_device(&c->scratch) != LCKV_OK || upload_layer_table(c) != LCKV_OK) {
        if (c->dev_err) (void)hipFree(c->dev_err);
        if (c->dev_layer_table) (void)hipFree(c->dev_layer_table);
        c->magic = 0;
        delete c;
        return LCKV_ERR_HIP;
    }
    *out = c;
    return LCKV_OK;
}

int lckv_cache_free(lckv_cache *c) {
    if (!valid(c)) return LCKV_ERR_NULL;
    for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
    if (c->dev_err) (void)hipFree(c->dev_err);
    if (c->dev_layer_table) (void)hipFree(c->dev_layer_table);
    c->magic = 0;
    delete c;
    return LCKV_OK;
}

int lckv_cache_set_block_table(lckv_cache *c, const int32_t *dev_table, int32_t max_blocks_per_seq) {
    if (!valid(c) || !dev_table) return LCKV_ERR_NULL;
    if (!c->cfg.page_size) return LCKV_ERR_BLOCK_TABLE;
    if (max_blocks_per_seq < 1 || max_blocks_per_seq > (1 << 24) / kPage) return LCKV_ERR_BLOCK_TABLE;
    if (!aligned(dev_table, 4)) return LCKV_ERR_ALIGN;
    if (c->cfg.window_tokens > 0 && kept_capacity(c) > max_blocks_per_seq * kPage) return LCKV_ERR_BLOCK_TABLE;
    c->table = dev_table;
    c->max_blocks = max_blocks_per_seq;
    c->capacity = max_blocks_per_seq * kPage;
    return LCKV_OK;
}

int lckv_n_slots(const lckv_cache *c, int32_t *n_slots) {
    if (!valid(c) || !n_slots) return LCKV_ERR_NULL;
    *n_slots = c->n_slots;
    return LCKV_OK;
}

int lckv_kv_slot(const lckv_cache *c, int32_t layer, int32_t *slot, int32_t *self_visible) {
    if (!valid(c) || !slot || !self_visible) return LCKV_ERR_NULL;
    if (layer < 0 || layer >= c->cfg.L) return LCKV_ERR_LAYER;
    *slot = c->kv_slot[layer];
    *self_visible = c->self_visible[layer];
    return LCKV_OK;
}

int lckv_slot_producer(const lckv_cache *c, int32_t slot, int32_t *layer) {
    if (!valid(c) || !layer) return LCKV_ERR_NULL;
    if (slot < 0 || slot >= c->n_slots) return LCKV_ERR_LAYER;
    *layer = c->producer[slot];
    return LCKV_OK;
}

int lckv_append_kv(lckv_cache *c, int32_t layer, const void *k_new, const void *v_new, const int32_t *dev_seq_lens,
                   int32_t B, void *hip_stream) {
    if (!valid(c) || !k_new || !v_new || !dev_seq_lens) return LCKV_ERR_NULL;
    if (layer < 0 || layer >= c->cfg.L) return LCKV_ERR_LAYER;
    const int slot = produced_slot(c, layer);
    if (slot < 0) return LCKV_ERR_NOT_PRODUCER;
    int rc = check_slot_access(c, B);
    if (rc != LCKV_OK) return rc;
    if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(dev_seq_lens, 4)) return LCKV_ERR_ALIGN;
    if (c->host_only) return LCKV_ERR_HIP;
    hipError_t e = launch_append(slot_view(c, slot), k_new, v_new, dev_seq_lens, B, c->cfg.D, c->cfg.dtype,
                                 c->dev_err, (hipStream_t)hip_stream);
    return e == hipSuccess ? LCKV_OK : LCKV_ERR_HIP;
}

int lckv_decode_attention(lckv_cache *c, int32_t layer, const void *q, void *out, const int32_t *dev_seq_lens,
                          const uint8_t *warmup_mask, int32_t B, int32_t max_len_hint, void *workspace,
                          size_t workspace_bytes, void *hip_stream) {
    if (!valid(c) || !q || !out || !dev_seq_lens) return LCKV_ERR_NULL;
    if (layer < 0 || layer >= c->cfg.L) return LCKV_ERR_LAYER;
    if (warmup_mask && memcmp(warmup_mask, c->warm.data(), (size_t)c->cfg.L) != 0) return LCKV_ERR_MASK;
    int rc = check_call(c, B, max_len_hint, c->self_visible[layer]);
    if (rc != LCKV_OK) return rc;
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(dev_seq_lens, 4)) return LCKV_ERR_ALIGN;
    return attention_impl(c, layer, q, out, dev_seq_lens, B, max_len_hint, workspace, workspace_bytes,
                          (hipStream_t)hip_stream);
}

int lckv_prefill_attention(lckv_cache *c, int32_t layer, const void *q, void *out, const int32_t *dev_prompt_lens,
                           int32_t B, int32_t S, void *hip_stream) {
    if (!valid(c) || !q || !out || !dev_prompt_lens) return LCKV_ERR_NULL;
    if (layer < 0 || layer >= c->cfg.L) return LCKV_ERR_LAYER;
    if (c->cfg.window_tokens > 0) return LCKV_ERR_CONFIG;  // prompts are encoded into a cache that keeps everything
    if (B < 1 || B > c->cfg.B_max) return LCKV_ERR_BATCH;
    if (c->cfg.page_size && !c->table) return LCKV_ERR_BLOCK_TABLE;
    if (S < 1 || S > c->capacity) return LCKV_ERR_LENGTH;
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(dev_prompt_lens, 4)) return LCKV_ERR_ALIGN;
    if (c->host_only) return LCKV_ERR_HIP;
    const lckv_config &cfg = c->cfg;
    AttnParams p;
    p.slot = slot_view(c, c->kv_slot[layer]);
    p.q = q;
    p.out = out;
    p.seq_lens = dev_prompt_lens;
    p.part_o = nullptr;
    p.part_ml = nullptr;
    p.dev_err = c->dev_err;
    p.B = B;
    p.Hq = cfg.Hq;
    p.Hkv = cfg.Hkv;
    p.G = cfg.Hq / cfg.Hkv;
    p.self_visible = c->self_visible[layer];
    p.max_n = S;
    p.clamp_is_policy = 0;
    p.split_tokens = (S + 63) / 64 * 64;
    p.n_splits = 1;
    p.scale_log2e = c->scale * 1.4426950408889634f;
    p.nontemporal = 0;
    p.unit_mul = 1;
    hipError_t e = cfg.dtype == LCKV_BF16
                       ? launch_prefill_bf16(p, S, cfg.D, c->prefill_query_blocks, (hipStream_t)hip_stream)
                       : launch_prefill_f32(p, S, cfg.D, (hipStream_t)hip_stream);
    return e == hipSuccess ? LCKV_OK : LCKV_ERR_HIP;
}

int lckv_set_prefill_tile(lckv_cache *c, int32_t query_blocks_per_wave) {
    if (!valid(c)) return LCKV_ERR_NULL;
    if (query_blocks_per_wave != 0 && query_blocks_per_wave != 2 && query_blocks_per_wave != 4) return LCKV_ERR_CONFIG;
    c->prefill_query_blocks = query_blocks_per_wave;
    return LCKV_OK;
}

// Both forms of the whole step: argument checks, then the layers in index order on one stream.
static int step_impl(lckv_cache *c, const void *q_all, const void *k_new_all, const void *v_new_all, void *out_all,
                     int32_t *dev_seq_lens, int32_t B, int32_t max_len_hint, void *workspace, size_t workspace_bytes,
                     bool static_scratch, void *hip_stream) {
    if (!valid(c) || !q_all || !k_new_all || !v_new_all || !out_all || !dev_seq_lens) return LCKV_ERR_NULL;
    int rc = check_call(c, B, max_len_hint, 1);  // the new token must fit
    if (rc != LCKV_OK) return rc;
    if (!aligned(q_all, 16) || !aligned(out_all, 16) || !aligned(k_new_all, 16) || !aligned(v_new_all, 16) ||
        !aligned(dev_seq_lens, 4))
        return LCKV_ERR_ALIGN;
    size_t need = 0;
    rc = lckv_workspace_bytes(c, B, max_len_hint, &need);
    if (rc != LCKV_OK) return rc;
    if (static_scratch) {
        if (need > (size_t)LCKV_STATIC_SCRATCH_BYTES) return LCKV_ERR_WORKSPACE;
        if (c->host_only) return LCKV_ERR_HIP;
        if ((rc = static_scratch_of_current_device(&workspace)) != LCKV_OK) return rc;
        workspace_bytes = LCKV_STATIC_SCRATCH_BYTES;
    } else if (need > 0 && (!workspace || !aligned(workspace, 256) || workspace_bytes < need)) {
        return LCKV_ERR_WORKSPACE;
    }
    if (c->host_only) return LCKV_ERR_HIP;

    const lckv_config &cfg = c->cfg;
    const size_t eb = (size_t)elem_bytes(cfg.dtype);
    const size_t q_layer = (size_t)B * cfg.Hq * cfg.D * eb;
    const size_t kv_slot_sz = (size_t)B * cfg.Hkv * cfg.D * eb;
    hipStream_t stream = (hipStream_t)hip_stream;
    auto append_slots_of = [&](int l) -> int {
        for (int s = 0; s < c->n_slots; ++s) {
            if (c->producer[s] != l) continue;
            hipError_t e = launch_append(slot_view(c, s), (const char *)k_new_all + s * kv_slot_sz,
                                         (const char *)v_new_all + s * kv_slot_sz, dev_seq_lens, B, cfg.D, cfg.dtype,
                                         c->dev_err, stream);
            if (e != hipSuccess) return LCKV_ERR_HIP;
        }
        return LCKV_OK;
    };
    for (int l = 0; l < cfg.L; ++l) {
        // A warmup layer sees the token being decoded: its K/V go in first.  The shared slot's new K/V are
        // invisible to every condensed layer of this step (diagonal mask) and, under the sink + window policy,
        // replace an entry those layers still read: they go in after the producing layer's attention.
        const bool before = c->self_visible[l] != 0;
        if (before && (rc = append_slots_of(l)) != LCKV_OK) return rc;
        rc = attention_impl(c, l, (const char *)q_all + l * q_layer, (char *)out_all + l * q_layer, dev_seq_lens, B,
                            max_len_hint, workspace, workspace_bytes, stream);
        if (rc != LCKV_OK) return rc;
        if (!before && (rc = append_slots_of(l)) != LCKV_OK) return rc;
    }
    return launch_bump(dev_seq_lens, B, stream) == hipSuccess ? LCKV_OK : LCKV_ERR_HIP;
}

int lckv_step(lckv_cache *c, const void *q_all, const void *k_new_all, const void *v_new_all, void *out_all,
              int32_t *dev_seq_lens, int32_t B, int32_t max_len_hint, void *workspace, size_t workspace_bytes,
              void *hip_stream) {
    return step_impl(c, q_all, k_new_all, v_new_all, out_all, dev_seq_lens, B, max_len_hint, workspace,
                     workspace_bytes, false, hip_stream);
}

// Split partials of the larger of the two plans (with and without the new token visible).
int partials_bytes(const lckv_cache *c, int32_t B, int32_t max_len_hint, bool allow_wide, size_t *bytes) {
    if (!valid(c) || !bytes) return LCKV_ERR_NULL;
    if (B < 1 || B > c->cfg.B_max) return LCKV_ERR_BATCH;
    if (max_len_hint < 0) return LCKV_ERR_LENGTH;
    size_t a = workspace_need(c, B, plan_splits(c, B, visible_bound(c, max_len_hint, 0), allow_wide).n_splits);
    size_t b = workspace_need(c, B, plan_splits(c, B, visible_bound(c, max_len_hint, 1), allow_wide).n_splits);
    *bytes = a > b ? a : b;
    return LCKV_OK;
}

int lckv_step_one_launch_workspace_bytes(const lckv_cache *c, int32_t B, int32_t max_len_hint, size_t *bytes) {
    int rc = partials_bytes(c, B, max_len_hint, false, bytes);
    if (rc == LCKV_OK) *bytes *= 2;  // two sets of split partials, taken in turn by layer parity
    return rc;
}

int lckv_step_one_launch(lckv_cache *c, const void *q_all, const void *k_new_all, const void *v_new_all,
                         void *out_all, int32_t *dev_seq_lens, int32_t B, int32_t max_len_hint, void *workspace,
                         size_t workspace_bytes, void *hip_stream) {
    if (!valid(c) || !q_all || !k_new_all || !v_new_all || !out_all || !dev_seq_lens) return LCKV_ERR_NULL;
    if (c->cfg.dtype != LCKV_BF16) return LCKV_ERR_CONFIG;
    int rc = check_call(c, B, max_len_hint, 1);  // the new token must fit
    if (rc != LCKV_OK) return rc;
    if (!aligned(q_all, 16) || !aligned(out_all, 16) || !aligned(k_new_all, 16) || !aligned(v_new_all, 16) ||
        !aligned(dev_seq_lens, 4))
        return LCKV_ERR_ALIGN;
    size_t one = 0;
    rc = partials_bytes(c, B, max_len_hint, false, &one);
    if (rc != LCKV_OK) return rc;
    if (one > 0 && (!workspace || !aligned(workspace, 256) || workspace_bytes < 2 * one)) return LCKV_ERR_WORKSPACE;
    if (c->host_only) return LCKV_ERR_HIP;

    const lckv_config &cfg = c->cfg;
    StepParams sp{};
    sp.a.slot = slot_view(c, 0);
    sp.a.seq_lens = dev_seq_lens;
    sp.a.dev_err = c->dev_err;
    sp.a.B = B;
    sp.a.Hq = cfg.Hq;
    sp.a.Hkv = cfg.Hkv;
    sp.a.G = cfg.Hq / cfg.Hkv;
    sp.a.scale_log2e = c->scale * 1.4426950408889634f;
    sp.a.waves = 4;
    sp.a.unit_mul = 1;
    for (int prime : {2731, 1571, 7919, 104729})  // as in the per-layer launch
        if (((int64_t)B * cfg.Hkv) % prime != 0) {
            sp.a.unit_mul = prime;
            break;
        }
    int max_units = 1;
    for (int vis = 0; vis < 2; ++vis) {
        const int max_n = visible_bound(c, max_len_hint, vis);
        const SplitPlan plan = plan_splits(c, B, max_n, false);  // this kernel's workgroups have four waves
        sp.max_n[vis] = max_n;
        sp.split_tokens[vis] = plan.tokens;
        sp.n_splits[vis] = plan.n_splits;
        const double pass_bytes = (double)B * max_n * 2.0 * cfg.Hkv * cfg.D * elem_bytes(cfg.dtype);
        sp.nontemporal[vis] = c->load_policy == LCKV_LOAD_NONTEMPORAL ||
                              (c->load_policy == LCKV_LOAD_AUTO && pass_bytes > kLastLevelCacheBytes);
        const int64_t units = (int64_t)plan.n_splits * cfg.Hkv * B;
        if (units > max_units) max_units = (int)(units > (1 << 30) ? (1 << 30) : units);
    }
    sp.a.clamp_is_policy = cfg.window_tokens > 0 && sp.max_n[0] == kept_capacity(c);
    {   // two sets of partials; in each, the (m, l) pairs lie past the partial outputs of the plan with more splits
        const int ns = sp.n_splits[0] > sp.n_splits[1] ? sp.n_splits[0] : sp.n_splits[1];
        const size_t rows = (size_t)ns * B * cfg.Hq;
        const size_t o_bytes = (rows * cfg.D * sizeof(float) + 255) / 256 * 256;
        for (int k = 0; k < 2; ++k) {
            sp.part_o[k] = one ? (float *)((char *)workspace + k * one) : nullptr;
            sp.part_ml[k] = one ? (float2 *)((char *)workspace + k * one + o_bytes) : nullptr;
        }
    }
    sp.q_all = (const char *)q_all;
    sp.out_all = (char *)out_all;
    sp.k_new_all = (const char *)k_new_all;
    sp.v_new_all = (const char *)v_new_all;
    sp.storage = c->storage;
    sp.slot_bytes = (int64_t)c->slot_bytes;
    sp.layer_table = c->dev_layer_table;
    sp.L = cfg.L;
    sp.seq_lens_rw = dev_seq_lens;
    // two sets of 1 + kBarrierGroups counters in the handle's device block (words 8.. and 32.., zero at first)
    static_assert(8 + 1 + kBarrierGroups <= 32 && 32 + 1 + kBarrierGroups <= 64, "the device block has 64 words");
    uint32_t *counters = (uint32_t *)c->dev_err;
    sp.barrier = counters + ((c->step_launches & 1u) ? 32 : 8);
    sp.barrier_next = counters + ((c->step_launches & 1u) ? 8 : 32);
    sp.wait_ticks = (int64_t)(c->barrier_wait_ms * 1e5);  // the wall clock ticks at 100 MHz
    c->step_launches += 1;
    hipError_t e = launch_step_bf16(sp, cfg.D, max_units, (hipStream_t)hip_stream);
    return e == hipSuccess ? LCKV_OK : LCKV_ERR_HIP;
}

int lckv_step_static_scratch(lckv_cache *c, const void *q_all, const void *k_new_all, const void *v_new_all,
                             void *out_all, int32_t *dev_seq_lens, int32_t B, int32_t max_len_hint,
                             void *hip_stream) {
    return step_impl(c, q_all, k_new_all, v_new_all, out_all, dev_seq_lens, B, max_len_hint, nullptr, 0, true,
                     hip_stream);
}

int lckv_workspace_bytes(const lckv_cache *c, int32_t B, int32_t max_len_hint, size_t *bytes) {
    return partials_bytes(c, B, max_len_hint, true, bytes);
}

// Workspace of lckv_project_qkv: none for bf16 caches (one launch, sums stay on chip); fp32 caches (parity mode):
// the products [B][(Hq + 2 Hkv) D] in fp32 between the two launches.
static size_t project_acc_bytes(const lckv_cache *c, int B, int hidden) {
    (void)hidden;
    if (c->cfg.dtype == LCKV_BF16) return 0;
    size_t n = ((size_t)c->cfg.Hq + 2 * (size_t)c->cfg.Hkv) * c->cfg.D * (size_t)B * sizeof(float);
    return (n + 255) / 256 * 256;
}

int lckv_pack_projection_weight(const lckv_cache *c, const void *w, void *w_packed, int32_t n_rows, int32_t hidden,
                                void *hip_stream) {
    if (!valid(c) || !w || !w_packed) return LCKV_ERR_NULL;
    if (n_rows < 16 || n_rows % c->cfg.D != 0 || hidden < 1 || (int64_t)n_rows * hidden > ((int64_t)1 << 40))
        return LCKV_ERR_CONFIG;  // whole heads: the packed order keeps the rotary pairs of a head together
    if (c->cfg.dtype == LCKV_BF16 && hidden % 256 != 0) return LCKV_ERR_CONFIG;
    if (!aligned(w, 16) || !aligned(w_packed, 16)) return LCKV_ERR_ALIGN;
    if (w == w_packed) return LCKV_ERR_CONFIG;
    if (c->host_only) return LCKV_ERR_HIP;
    hipError_t e = launch_pack_weight(w, w_packed, n_rows, hidden, c->cfg.D, c->cfg.dtype, (hipStream_t)hip_stream);
    return e == hipSuccess ? LCKV_OK : LCKV_ERR_HIP;
}

int lckv_project_workspace_bytes(const lckv_cache *c, int32_t B, int32_t hidden, size_t *bytes) {
    if (!valid(c) || !bytes) return LCKV_ERR_NULL;
    if (B < 1 || B > c->cfg.B_max) return LCKV_ERR_BATCH;
    if (hidden < 1 || (c->cfg.dtype == LCKV_BF16 && hidden % 256 != 0)) return LCKV_ERR_CONFIG;
    *bytes = project_acc_bytes(c, B, hidden);
    return LCKV_OK;
}

int lckv_project_qkv(lckv_cache *c, int32_t layer, const void *x, int32_t hidden, const void *w_q, const void *w_k,
                     const void *w_v, void *q_out, void *k_out, void *v_out, const int32_t *dev_seq_lens, int32_t B,
                     float rope_base, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!valid(c) || !x || !w_q || !q_out || !dev_seq_lens) return LCKV_ERR_NULL;
    if (layer < 0 || layer >= c->cfg.L) return LCKV_ERR_LAYER;
    const int slot = produced_slot(c, layer);
    if (slot < 0 && (w_k || w_v || k_out || v_out)) return LCKV_ERR_NOT_PRODUCER;
    if (slot >= 0 && (!w_k || !w_v)) return LCKV_ERR_NULL;
    if ((k_out == nullptr) != (v_out == nullptr)) return LCKV_ERR_NULL;
    const bool deferred = k_out != nullptr;
    if (B < 1 || B > c->cfg.B_max) return LCKV_ERR_BATCH;
    if (hidden < 1 || (int64_t)hidden * B > ((int64_t)1 << 40)) return LCKV_ERR_CONFIG;
    if (c->cfg.dtype == LCKV_BF16 && hidden % 256 != 0) return LCKV_ERR_CONFIG;
    // Under the sink + window policy the shared slot's new K/V replace an entry the producing layer's own
    // attention still reads: they cannot be stored by this call, only handed back.
    if (slot >= 0 && !deferred && c->cfg.window_tokens > 0 && !c->self_visible[layer]) return LCKV_ERR_CONFIG;
    if (slot >= 0 && !deferred) {
        int rc = check_slot_access(c, B);
        if (rc != LCKV_OK) return rc;
    }
    if (!aligned(x, 16) || !aligned(w_q, 16) || !aligned(q_out, 16) || !aligned(dev_seq_lens, 4) ||
        (w_k && !aligned(w_k, 16)) || (w_v && !aligned(w_v, 16)) || (deferred && (!aligned(k_out, 16) || !aligned(v_out, 16))))
        return LCKV_ERR_ALIGN;
    size_t need = 0;
    lckv_project_workspace_bytes(c, B, hidden, &need);
    if (need > 0 && (!workspace || !aligned(workspace, 256) || workspace_bytes < need)) return LCKV_ERR_WORKSPACE;
    if (c->host_only) return LCKV_ERR_HIP;
    float *acc = (float *)workspace;
    hipError_t e = launch_project(x, hidden, w_q, w_k, w_v, q_out, k_out, v_out, slot_view(c, slot >= 0 ? slot : 0),
                                  dev_seq_lens, B, c->cfg.Hq, c->cfg.Hkv, c->cfg.D, c->cfg.dtype, rope_base, acc,
                                  c->dev_err, (hipStream_t)hip_stream);
    return e == hipSuccess ? LCKV_OK : LCKV_ERR_HIP;
}

int lckv_set_workgroup_waves(lckv_cache *c, int32_t waves) {
    if (!valid(c)) return LCKV_ERR_NULL;
    if (waves != 0 && waves != 4 && waves != 8 && waves != 16) return LCKV_ERR_CONFIG;
    c->forced_waves = waves;
    return LCKV_OK;
}

int lckv_set_split_tokens(lckv_cache *c, int32_t tokens) {
    if (!valid(c)) return LCKV_ERR_NULL;
    if (tokens < 0 || tokens % kPage != 0) return LCKV_ERR_CONFIG;
    c->forced_split_tokens = tokens;
    return LCKV_OK;
}

int lckv_set_barrier_wait_ms(lckv_cache *c, double ms) {
    if (!valid(c)) return LCKV_ERR_NULL;
    if (!(ms >= 0.0) || ms > 60000.0) return LCKV_ERR_CONFIG;
    c->barrier_wait_ms = ms;
    return LCKV_OK;
}

int lckv_set_load_policy(lckv_cache *c, int32_t policy) {
    if (!valid(c)) return LCKV_ERR_NULL;
    if (policy != LCKV_LOAD_AUTO && policy != LCKV_LOAD_TEMPORAL && policy != LCKV_LOAD_NONTEMPORAL)
        return LCKV_ERR_CONFIG;
    c->load_policy = policy;
    return LCKV_OK;
}

int lckv_cache_load_dense(lckv_cache *c, int32_t slot, const void *k, const void *v, const int32_t *dev_seq_lens,
                          int32_t B, int32_t T, void *hip_stream) {
    if (!valid(c) || !k || !v) return LCKV_ERR_NULL;
    if (slot < 0 || slot >= c->n_slots) return LCKV_ERR_LAYER;
    int rc = check_slot_access(c, B);
    if (rc != LCKV_OK) return rc;
    if (T < 0 || T > kept_capacity(c)) return LCKV_ERR_LENGTH;
    if (!aligned(k, 16) || !aligned(v, 16) || (dev_seq_lens && !aligned(dev_seq_lens, 4))) return LCKV_ERR_ALIGN;
    if (c->host_only) return LCKV_ERR_HIP;
    hipError_t e = launch_load_dense(slot_view(c, slot), k, v, dev_seq_lens, B, T, c->cfg.D, c->cfg.dtype,
                                     c->dev_err, (hipStream_t)hip_stream);
    return e == hipSuccess ? LCKV_OK : LCKV_ERR_HIP;
}

int lckv_cache_read(lckv_cache *c, int32_t slot, int32_t b, int32_t pos, int32_t n_pos, void *host_k, void *host_v) {
    if (!valid(c) || !host_k || !host_v) return LCKV_ERR_NULL;
    if (slot < 0 || slot >= c->n_slots) return LCKV_ERR_LAYER;
    if (b < 0 || b >= c->cfg.B_max) return LCKV_ERR_BATCH;
    if (c->cfg.page_size && !c->table) return LCKV_ERR_BLOCK_TABLE;
    // under the sink + window policy `pos` is a logical position of any size; the caller asks only for
    // positions that are still kept
    if (pos < 0 || n_pos < 1 || n_pos > kept_capacity(c) || kept_capacity(c) > c->capacity) return LCKV_ERR_RANGE;
    if (c->cfg.window_tokens == 0 && (int64_t)pos + n_pos > c->capacity) return LCKV_ERR_RANGE;
    if ((int64_t)n_pos * c->cfg.Hkv * c->cfg.D >= ((int64_t)1 << 31)) return LCKV_ERR_RANGE;
    if (c->host_only) return LCKV_ERR_HIP;
    size_t bytes = (size_t)n_pos * c->cfg.Hkv * c->cfg.D * elem_bytes(c->cfg.dtype);
    char *tmp = nullptr;
    if (hipMalloc((void **)&tmp, 2 * bytes) != hipSuccess) return LCKV_ERR_HIP;
    int rc = LCKV_OK;
    if (launch_gather(slot_view(c, slot), b, pos, n_pos, c->cfg.D, c->cfg.dtype, tmp, tmp + bytes, c->dev_err,
                      nullptr) != hipSuccess ||
        hipDeviceSynchronize() != hipSuccess || hipMemcpy(host_k, tmp, bytes, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(host_v, tmp + bytes, bytes, hipMemcpyDeviceToHost) != hipSuccess)
        rc = LCKV_ERR_HIP;
    (void)hipFree(tmp);
    return rc;
}

int lckv_last_device_error(lckv_cache *c, int32_t *bits) {
    if (!valid(c) || !bits) return LCKV_ERR_NULL;
    if (c->host_only) return LCKV_ERR_HIP;
    if (hipDeviceSynchronize() != hipSuccess) return LCKV_ERR_HIP;
    if (hipMemcpy(bits, c->dev_err, sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess) return LCKV_ERR_HIP;
    if (*bits && hipMemset(c->dev_err, 0, sizeof(int32_t)) != hipSuccess) return LCKV_ERR_HIP;
    return LCKV_OK;
}

int lckv_profile_enable(lckv_cache *c, int32_t enable) {
    if (!valid(c)) return LCKV_ERR_NULL;
    if (c->host_only) return LCKV_ERR_HIP;
    if (enable && c->ev.empty()) {
        c->ev.reserve(2 * kProfilePairs);
        for (size_t i = 0; i < 2 * kProfilePairs; ++i) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return LCKV_ERR_HIP;
            c->ev.push_back(e);
        }
    }
    c->profiling = enable != 0;
    return LCKV_OK;
}

int lckv_profile_launch_ms(lckv_cache *c, float *ms, int32_t capacity, int32_t *n_launches) {
    if (!valid(c) || !ms || !n_launches) return LCKV_ERR_NULL;
    if (capacity < 0) return LCKV_ERR_RANGE;
    if (c->host_only) return LCKV_ERR_HIP;
    if (hipDeviceSynchronize() != hipSuccess) return LCKV_ERR_HIP;
    int32_t n = 0;
    for (size_t i = 0; i + 1 < c->ev_used && n < capacity; i += 2, ++n)
        if (hipEventElapsedTime(&ms[n], c->ev[i], c->ev[i + 1]) != hipSuccess) return LCKV_ERR_HIP;
    *n_launches = n;
    return LCKV_OK;
}

int lckv_profile_read(lckv_cache *c, int32_t *n_launches, double *total_ms) {
    if (!valid(c) || !n_launches || !total_ms) return LCKV_ERR_NULL;
    if (c->host_only) return LCKV_ERR_HIP;
    if (hipDeviceSynchronize() != hipSuccess) return LCKV_ERR_HIP;
    double sum = 0.0;
    for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->ev[i], c->ev[i + 1]) != hipSuccess) return LCKV_ERR_HIP;
        sum += ms;
    }
    *n_launches = (int32_t)(c->ev_used / 2);
    *total_ms = sum;
    c->ev_used = 0;
    return LCKV_OK;
}

int lckv_hbm_read_probe(lckv_cache *c, const void *dev_buf, size_t bytes, int32_t nontemporal, void *hip_stream) {
    if (!valid(c) || !dev_buf) return LCKV_ERR_NULL;
    if (!aligned(dev_buf, 16)) return LCKV_ERR_ALIGN;
    if (c->host_only) return LCKV_ERR_HIP;
    hipError_t e = launch_stream_probe(dev_buf, bytes, nontemporal, c->dev_err + 1, (hipStream_t)hip_stream);
    return e == hipSuccess ? LCKV_OK : LCKV_ERR_HIP;
}

const char *lckv_strerror(int code) {
    switch (code) {
        case LCKV_OK: return "ok";
        case LCKV_ERR_NULL: return "required pointer is NULL or handle is not a live lckv_cache";
        case LCKV_ERR_CONFIG: return "unsupported or inconsistent configuration";
        case LCKV_ERR_LAYER: return "layer or slot index out of range";
        case LCKV_ERR_NOT_PRODUCER: return "no slot stores this layer's K/V";
        case LCKV_ERR_BATCH: return "batch size or sequence index out of range";
        case LCKV_ERR_LENGTH: return "length exceeds the cache capacity";
        case LCKV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case LCKV_ERR_ALIGN: return "device pointer misaligned";
        case LCKV_ERR_BLOCK_TABLE: return "block table missing or invalid";
        case LCKV_ERR_HIP: return "HIP runtime call failed";
        case LCKV_ERR_MASK: return "warmup mask differs from the cache's";
        case LCKV_ERR_STORAGE: return "kv storage too small";
        case LCKV_ERR_RANGE: return "position range outside the cache";
        default: return "unknown lckv error";
    }
}

}  // extern "C"
