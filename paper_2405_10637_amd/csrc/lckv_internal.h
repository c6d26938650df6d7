// Internal declarations shared by the host API and the gfx950 kernels of liblckv.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/lckv.h"
#include "../../include/lckv_tools.h"

namespace lckv {

constexpr int kPage = 16;        // positions per page
constexpr int kMaxGroup = 16;    // query heads per kv head that fit one 16-column matrix tile

// What a kernel needs to find a page pair of one slot.
struct SlotView {
    char *base;                 // first byte of the slot
    const int32_t *table;       // paged: device block table [B_max][max_blocks], else nullptr
    int32_t max_blocks;         // paged: table row length
    int64_t num_blocks;         // paged: physical blocks per slot
    int32_t pages_per_seq;      // contiguous: pages per (b, kv head)
    int32_t Hkv;
    int32_t page_bytes;         // bytes of one K (or V) page = 16 * D * elem
    int32_t capacity;           // positions a sequence can hold (sink + window with the sink + window policy)
    int32_t ring_sink;          // sink + window policy: positions below this stay where they are
    int32_t ring_window;        // ... and later positions live in a ring of this many entries; 0 = policy off
};

// Entry of a slot that holds logical position t: identity, or with the sink + window policy the ring entry
// (Section 3.3 of the LCKV paper: the first few and the recent tokens are kept).
__device__ __forceinline__ int entry_of_position(const SlotView &v, int t) {
    if (v.ring_window > 0 && t >= v.ring_sink + v.ring_window)
        return v.ring_sink + (t - v.ring_sink) % v.ring_window;
    return t;
}

// Index of the page pair holding page p of (b, kv head g); -1 if the block table entry is invalid.
__device__ __forceinline__ int64_t page_pair_index(const SlotView &v, int b, int g, int p) {
    if (v.table) {
        int32_t blk = v.table[(int64_t)b * v.max_blocks + p];
        if (blk < 0 || (int64_t)blk >= v.num_blocks) return -1;
        return (int64_t)blk * v.Hkv + g;
    }
    return ((int64_t)b * v.Hkv + g) * v.pages_per_seq + p;
}

// Element offsets inside a page (in elements, not bytes) for position j (0..15) and channel d.  bf16 pages are
// stored in matrix-operand order: the 16 bytes lane l of a wave feeds to the matrix instruction sit at byte
// l*16 of a 1 KiB tile, so a wave's load is one contiguous, lane-ordered KiB.
//
// bf16 K page: [D/32 tiles][4 channel octets kb][16 positions j][8 channels]: tile ks is the 16x32 A operand of
// the QK instruction for channels 32ks..32ks+31; lane kb*16 + j holds channels 32ks + 8kb .. +8 of position j.
__host__ __device__ __forceinline__ int k_elem_offset_bf16(int j, int d) {
    return (((d >> 5) * 4 + ((d & 31) >> 3)) * kPage + j) * 8 + (d & 7);
}
// bf16 V page: [D/32 tiles][4 position quads kb][16 channels r][2 channel blocks][4 positions]: lane kb*16 + r
// holds positions 4kb..4kb+3 of channels (2dp)*16 + r and (2dp+1)*16 + r, the A operands of two 16x16x16 PV
// instructions.
__host__ __device__ __forceinline__ int v_elem_offset_bf16(int j, int d) {
    int dblk = d >> 4, r = d & 15, dp = dblk >> 1, dsel = dblk & 1, kb = j >> 2, kq = j & 3;
    return ((((dp * 4 + kb) * 16 + r) * 2 + dsel) * 4) + kq;
}
// fp32 pages are row-major [16][D].
__host__ __device__ __forceinline__ int kv_elem_offset_f32(int j, int d, int D) { return j * D + d; }

// ---- element-wise pieces shared by the stand-alone kernels and the persistent step kernel --------------------

template <typename E>
__device__ __forceinline__ int k_off(int j, int d, int D);
template <>
__device__ __forceinline__ int k_off<uint16_t>(int j, int d, int) { return k_elem_offset_bf16(j, d); }
template <>
__device__ __forceinline__ int k_off<uint32_t>(int j, int d, int D) { return kv_elem_offset_f32(j, d, D); }
template <typename E>
__device__ __forceinline__ int v_off(int j, int d, int D);
template <>
__device__ __forceinline__ int v_off<uint16_t>(int j, int d, int) { return v_elem_offset_bf16(j, d); }
template <>
__device__ __forceinline__ int v_off<uint32_t>(int j, int d, int D) { return kv_elem_offset_f32(j, d, D); }

// Element i of [B][Hkv][D] of the new token's K and V into the slot at position t_b (bits copied unchanged).
template <typename E>
__device__ __forceinline__ void append_element(const SlotView &sv, const E *k_new, const E *v_new,
                                               const int32_t *seq_lens, int D, int32_t *dev_err, int64_t i) {
    int d = (int)(i % D);
    int g = (int)((i / D) % sv.Hkv);
    int b = (int)(i / ((int64_t)D * sv.Hkv));
    int t = seq_lens[b];
    if (t >= 0) t = entry_of_position(sv, t);  // identity, or the ring entry under the sink + window policy
    if (t < 0 || t >= sv.capacity) {
        if (d == 0) atomicOr(dev_err, LCKV_DEV_ERR_CAPACITY);
        return;
    }
    int64_t idx = page_pair_index(sv, b, g, t / kPage);
    if (idx < 0) {
        if (d == 0) atomicOr(dev_err, LCKV_DEV_ERR_BLOCK);
        return;
    }
    E *kpage = (E *)(sv.base + idx * (2 * (int64_t)sv.page_bytes));
    E *vpage = (E *)((char *)kpage + sv.page_bytes);
    int j = t % kPage;
    kpage[k_off<E>(j, d, D)] = k_new[i];
    vpage[v_off<E>(j, d, D)] = v_new[i];
}

__device__ __forceinline__ void store_out(float *o, float v) { *o = v; }
__device__ __forceinline__ void store_out(uint16_t *o, float v) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    typedef __attribute__((ext_vector_type(2))) float floatx2_t;
    floatx2_t f = {v, 0.f};
    bf16x2_t h = __builtin_convertvector(f, bf16x2_t);  // round to nearest even
    *o = (uint16_t)(__builtin_bit_cast(uint32_t, h) & 0xffffu);
}

// Output element i of the merge of split partials: with (m_s, l_s, o_s) the running maximum (log2 units),
// denominator and unnormalised output of split s,  out = sum_s 2^(m_s - M) o_s / sum_s 2^(m_s - M) l_s,
// M = max_s m_s.  Splits without a visible key carry m_s = -inf and are skipped; no visible key at all gives zero.
// DEVICE_SCOPE_LOADS: the partials were written by other workgroups of the SAME launch (and released at device
// scope): read them past this compute unit's caches.
template <typename O, bool DEVICE_SCOPE_LOADS = false>
__device__ __forceinline__ void combine_element(const float *part_o, const float2 *part_ml, O *out, int64_t rows,
                                                int D, int S, int64_t i) {
    auto ld = [](const float *p) {
        return DEVICE_SCOPE_LOADS ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *p;
    };
    const float neg_inf = -__builtin_huge_valf();
    int64_t row = i / D;
    int d = (int)(i % D);
    float M = neg_inf;
    for (int s = 0; s < S; ++s) M = fmaxf(M, ld(&part_ml[(int64_t)s * rows + row].x));
    float num = 0.f, den = 0.f;
    for (int s = 0; s < S; ++s) {
        const float2 *pml = &part_ml[(int64_t)s * rows + row];
        float2 ml = {ld(&pml->x), ld(&pml->y)};
        if (ml.x == neg_inf) continue;
        float f = exp2f(ml.x - M);
        den += f * ml.y;
        num += f * ld(&part_o[((int64_t)s * rows + row) * D + d]);
    }
    store_out(out + i, den > 0.f ? num / den : 0.f);
}

struct AttnParams {
    SlotView slot;
    const void *q;              // [B][Hq][D]
    void *out;                  // [B][Hq][D]
    const int32_t *seq_lens;    // [B]
    float *part_o;              // [S][B][Hq][D] unnormalised partial outputs (S > 1)
    float2 *part_ml;            // [S][B][Hq] (running max in log2 units, partial denominator)
    int32_t *dev_err;
    int32_t B, Hq, Hkv, G;
    int32_t self_visible;       // 1: n_b = t_b + 1
    int32_t max_n;              // clamp for n_b
    int32_t clamp_is_policy;    // 1: n_b > max_n is the sink + window policy at work, not an error
    int32_t split_tokens;       // keys per split (multiple of 16)
    int32_t n_splits;
    int32_t waves;              // bf16 kernel: waves per workgroup (4, 8 or 16)
    float scale_log2e;          // scale * log2(e)
    int32_t nontemporal;        // 1: read K/V with the nontemporal hint (stream larger than the caches)
    int32_t unit_mul;           // launch order -> (sequence, kv head): unit = (id * unit_mul) mod (B * Hkv), coprime
};

// Everything the one-launch decode step needs: the attention parameters that are the same for every layer, the
// per-layer table, both split plans (a warmup layer sees one key more, which can move the split), the counters of
// the device-wide barrier.
struct StepParams {
    AttnParams a;                  // B, heads, scale, dev_err, seq_lens, block table ...; per-layer fields are filled in
    const char *q_all;             // [L][B][Hq][D]
    char *out_all;
    const char *k_new_all, *v_new_all;  // [n_slots][B][Hkv][D]
    char *storage;
    int64_t slot_bytes;
    const int32_t *layer_table;    // device [L][4]: slot read, self visible, slot produced (-1: none), when to append
    int32_t L;
    int32_t max_n[2], split_tokens[2], n_splits[2], nontemporal[2];  // by self_visible
    float *part_o[2];              // split partials, two sets taken in turn by layer parity
    float2 *part_ml[2];
    int32_t *seq_lens_rw;
    uint32_t *barrier;             // device counters of this launch (start at zero): [0] groups arrived, [1 + g] group g
    uint32_t *barrier_next;        // the next launch's counters, zeroed by this one
    int64_t wait_ticks;            // bound on a barrier wait, in ticks of the 100 MHz wall clock
};
constexpr int kBarrierGroups = 16;  // arrival counters per barrier (plus the top one)
// when to append a layer's new K/V in the one-launch step
constexpr int kAppendNone = 0, kAppendAtStart = 1, kAppendBeforeOwnAttention = 2, kAppendAfterOwnAttention = 3;

hipError_t launch_attn_bf16(const AttnParams &p, int D, hipStream_t s);
hipError_t launch_step_bf16(const StepParams &sp, int D, int max_units, hipStream_t s);
hipError_t launch_attn_f32(const AttnParams &p, int D, hipStream_t s);
hipError_t launch_prefill_f32(const AttnParams &p, int S, int D, hipStream_t s);
hipError_t launch_prefill_bf16(const AttnParams &p, int S, int D, int query_blocks, hipStream_t s);
hipError_t launch_combine(const AttnParams &p, int D, int dtype, hipStream_t s);
hipError_t launch_append(const SlotView &v, const void *k_new, const void *v_new, const int32_t *seq_lens,
                         int B, int D, int dtype, int32_t *dev_err, hipStream_t s);
hipError_t launch_bump(int32_t *seq_lens, int B, hipStream_t s);
hipError_t launch_load_dense(const SlotView &v, const void *k, const void *vv, const int32_t *lens, int B, int T,
                             int D, int dtype,
                             int32_t *dev_err, hipStream_t s);
hipError_t launch_pack_weight(const void *src, void *dst, int N, int hidden, int D, int dtype, hipStream_t s);
hipError_t launch_project(const void *x, int hidden, const void *w_q, const void *w_k, const void *w_v, void *q_out,
                          void *k_out, void *v_out, const SlotView &slot, const int32_t *seq_lens, int B, int Hq, int Hkv, int D, int dtype,
                          float rope_base, float *acc, int32_t *dev_err, hipStream_t s);
hipError_t launch_stream_probe(const void *buf, size_t bytes, int nontemporal, int32_t *sink, hipStream_t s);
hipError_t launch_gather(const SlotView &v, int b, int pos, int n_pos, int D, int dtype, void *dev_k, void *dev_v,
                         int32_t *dev_err, hipStream_t s);

}  // namespace lckv

struct lckv_cache {
    uint64_t magic;
    lckv_config cfg;
    std::vector<uint8_t> warm;
    std::vector<int32_t> kv_slot, self_visible, producer;  // pairing table
    int32_t n_slots;
    char *storage;
    size_t slot_bytes;
    int32_t pages_per_seq;
    int32_t page_bytes;
    const int32_t *table;
    int32_t max_blocks;
    int32_t capacity;
    int32_t forced_split_tokens;
    int32_t forced_waves;         // 0: the planner chooses the workgroup width
    int32_t load_policy;          // LCKV_LOAD_*
    int32_t prefill_query_blocks; // 16-position blocks per wave in the bf16 prefill kernel (2 or 4)
    int32_t *dev_err;
    int32_t *dev_layer_table;     // [L][4] for the one-launch step
    uint32_t step_launches;       // one-launch steps enqueued so far (picks the barrier counter)
    double barrier_wait_ms;       // bound on a device-wide barrier wait
    void *scratch;                // this device's copy of the library's static scratch array
    bool host_only;               // made on a host without a GPU: argument checks and planners only
    float scale;
    // kernel timing
    bool profiling;
    std::vector<hipEvent_t> ev;   // pairs (start, stop)
    size_t ev_used;
};
