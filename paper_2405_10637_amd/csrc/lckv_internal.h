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
    float scale_log2e;          // scale * log2(e)
    int32_t nontemporal;        // 1: read K/V with the nontemporal hint (stream larger than the caches)
    int32_t unit_mul;           // launch order -> (sequence, kv head): unit = (id * unit_mul) mod (B * Hkv), coprime
};

hipError_t launch_attn_bf16(const AttnParams &p, int D, hipStream_t s);
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
    int32_t load_policy;          // LCKV_LOAD_*
    int32_t prefill_query_blocks; // 16-position blocks per wave in the bf16 prefill kernel (2 or 4)
    int32_t *dev_err;
    void *scratch;                // this device's copy of the library's static scratch array
    bool host_only;               // made on a host without a GPU: argument checks and planners only
    float scale;
    // kernel timing
    bool profiling;
    std::vector<hipEvent_t> ev;   // pairs (start, stop)
    size_t ev_used;
};
