// Split-KV decode attention for bf16 caches on gfx950 (Section 2.1 of the LCKV paper: one query token per
// sequence attends to the slot its layer is paired with).
//
// One workgroup (4 waves) handles one (split, kv head, sequence).  All G = Hq/Hkv query heads of the kv head
// ride in the 16 columns of the matrix tiles, so K and V are read from HBM once per kv head:
//   S^T[key][query]  = K_page[16 keys x D]   . Q^T[D x 16 queries]      v_mfma_f32_16x16x32_bf16, D/32 steps
//   O^T[d][query]   += V_page^T[16 d x 16 keys] . P^T[16 keys x 16 queries]   v_mfma_f32_16x16x16_bf16, D/16 tiles
// The accumulator layout of the first product (lane (kb, c) holds keys 4kb..4kb+3 of query c) is exactly the
// B-operand layout of the second, so probabilities never leave registers.  Pages are stored in operand order:
// every global load is 16 bytes per lane, lane l at byte 16*l of a contiguous KiB.  Each wave keeps a running
// (max, sum, O) per query (online softmax, fp32); waves are merged through LDS at the end.
//
// The loads of a tile never sit under a branch: a page past the end of the split (or with a bad block-table
// entry) is redirected to a page that is certainly mapped and its contribution is dropped, so the compiler can
// keep the next tile's loads in flight while the current tile is consumed.
#include "bf16_mfma_common.h"

namespace lckv {

template <int D, int NP>
struct Tile {
    u32x4 k[NP][D / 32];
    u32x4 v[NP][D / 32];
    int page[NP];  // wave-uniform: page number, or -1 if what was loaded must be ignored
};

// The pages of a split, pg_begin .. pg_begin + n_pages - 1, are visited in rotated order: visit number `it` reads
// page pg_begin + (it + rot) mod n_pages.  `it`, `rot`, `n_pages` are wave-uniform, 0 <= rot < n_pages.
struct PageWalk {
    int pg_begin, n_pages, rot;
};

template <int D, int NP, bool PAGED, bool NT>
__device__ __forceinline__ void load_tile(Tile<D, NP> &t, const SlotView &sv, int b, int g, int it,
                                          const PageWalk &walk, int lane_off, int32_t *dev_err) {
    constexpr int64_t kPair = 2 * kPage * D * 2;  // bytes of a K page + V page
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        bool live = it + i < walk.n_pages;
        int rel = (live ? it + i : 0) + walk.rot;  // a visit past the end re-reads a page that certainly exists
        if (rel >= walk.n_pages) rel -= walk.n_pages;
        const int pgi = walk.pg_begin + rel;
        const int src = pgi;
        int64_t idx;
        if (PAGED) {
            int32_t blk = sv.table[(int64_t)b * sv.max_blocks + src];
            bool ok = blk >= 0 && (int64_t)blk < sv.num_blocks;
            if (!ok) {
                if (live && lane_off == 0) atomicOr(dev_err, LCKV_DEV_ERR_BLOCK);
                live = false;
                blk = 0;
            }
            idx = (int64_t)blk * sv.Hkv + g;
        } else {
            idx = ((int64_t)b * sv.Hkv + g) * sv.pages_per_seq + src;
        }
        t.page[i] = live ? pgi : -1;
        const char *base = sv.base + idx * kPair + lane_off;
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) t.k[i][ks] = load16<NT>(base + ks * 1024);
#pragma unroll
        for (int dp = 0; dp < D / 32; ++dp) t.v[i][dp] = load16<NT>(base + kPair / 2 + dp * 1024);
    }
}

template <int D, int NP>
__device__ __forceinline__ void consume_tile(Tile<D, NP> &t, const bf16x8 (&qb)[D / 32], floatx4 (&acc)[D / 16],
                                             float &m, float &l, int k_end, int kb, float c) {
    bool any = false;
#pragma unroll
    for (int i = 0; i < NP; ++i) any |= t.page[i] >= 0;
    if (!any) return;  // nothing usable in this tile (only possible with a bad block table)
    floatx4 s[NP];
    float smax = kNegInf;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        if (t.page[i] < 0) {  // wave-uniform
            s[i] = floatx4{kNegInf, kNegInf, kNegInf, kNegInf};
            continue;
        }
        floatx4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks)
            z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, t.k[i][ks]), qb[ks], z, 0, 0, 0);
        int key0 = t.page[i] * kPage + 4 * kb;
        if ((t.page[i] + 1) * kPage > k_end) {  // last, partly filled page: mask scores, clear stale values
            int nv = k_end - key0;              // valid keys among this lane's four
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (e >= nv) z[e] = kNegInf;
            uint32_t m01 = nv >= 2 ? 0xffffffffu : (nv == 1 ? 0x0000ffffu : 0u);
            uint32_t m23 = nv >= 4 ? 0xffffffffu : (nv == 3 ? 0x0000ffffu : 0u);
#pragma unroll
            for (int dp = 0; dp < D / 32; ++dp) {
                t.v[i][dp][0] &= m01;
                t.v[i][dp][1] &= m23;
                t.v[i][dp][2] &= m01;
                t.v[i][dp][3] &= m23;
            }
        }
        s[i] = z;
        smax = fmaxf(smax, fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])));
    }
    // the four lanes (kb = 0..3) of a query column share one running maximum
    smax = column_max4(smax);
    float m_new = fmaxf(m, smax);  // finite: a page that is used always holds a visible key
    float mb = m_new * c;
    float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
    const bool grew = __builtin_amdgcn_ballot_w64(m_new > m) != 0;  // wave-uniform
    m = m_new;
    float psum = 0.f;
    shortx4 pb[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i][0], c, -mb));
        float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i][1], c, -mb));
        float p2 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i][2], c, -mb));
        float p3 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i][3], c, -mb));
        psum += (p0 + p1) + (p2 + p3);
        u32x2 pk = {pack_bf16(p0, p1), pack_bf16(p2, p3)};
        pb[i] = __builtin_bit_cast(shortx4, pk);
    }
    if (grew) {  // some column's maximum moved: rescale what was accumulated under the old one
        l *= alpha;
#pragma unroll
        for (int j = 0; j < D / 16; ++j) acc[j] *= alpha;
    }
    l += psum;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        if (t.page[i] < 0) continue;
#pragma unroll
        for (int dp = 0; dp < D / 32; ++dp) {
            u32x2 lo = {t.v[i][dp][0], t.v[i][dp][1]};
            u32x2 hi = {t.v[i][dp][2], t.v[i][dp][3]};
            acc[2 * dp] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, lo), pb[i],
                                                                    acc[2 * dp], 0, 0, 0);
            acc[2 * dp + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, hi), pb[i],
                                                                        acc[2 * dp + 1], 0, 0, 0);
        }
    }
}

// One (split, kv head, sequence) unit of a layer's attention, by one workgroup of W waves; NP pages (of 16 keys)
// per wave and tile.  `launch_unit` is the unit's place in launch order (sequence-major, kv head minor): the order
// is scattered over the units by a multiplier coprime to their number.  Workgroups that run at the same time then
// read streams that lie far apart and at unrelated distances, instead of neighbours at one fixed distance whose
// addresses can fall on the same HBM channels; together with the rotated page walk below this makes the
// bandwidth independent of the cache capacity chosen (measured: 6.6-7.0 TB/s depending on the capacity without
// it).  Uses LDS; a workgroup that takes several units in a row synchronises between them.
template <int D, int NP, int W, bool PAGED, bool NT>
__device__ __forceinline__ void attn_bf16_unit(const AttnParams &p, int split, int launch_unit) {
    const int unit = (int)(((int64_t)launch_unit * p.unit_mul) % ((int64_t)p.B * p.Hkv));
    const int g = unit % p.Hkv, b = unit / p.Hkv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: page numbers stay uniform
    const int c = lane & 15, kb = lane >> 4;  // query column / key quad
    const int G = p.G;
    const int h = g * G + c;                  // query head of this lane's column (valid if c < G)

    const int64_t row = (int64_t)b * p.Hq + h;

    // Q^T operands: lane (kb, c) holds channels ks*32 + 8kb .. +8 of query head h; columns >= G are zero.  Asked
    // for before the sequence's length is looked at, so that the two round trips to memory overlap (with small
    // slots a workgroup's whole stream lasts only some twenty microseconds).
    bf16x8 qb[D / 32];
    {
        const char *qp = (const char *)p.q + (row * D + kb * 8) * 2;
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (c < G) v = *(const u32x4 *)(qp + ks * 64);
            qb[ks] = __builtin_bit_cast(bf16x8, v);
        }
    }

    int n = p.seq_lens[b] + p.self_visible;
    if (n > p.max_n) {
        n = p.max_n;
        if (tid == 0 && !p.clamp_is_policy) atomicOr(p.dev_err, LCKV_DEV_ERR_CAPACITY);
    }
    if (n < 0) n = 0;
    const int k_begin = split * p.split_tokens;
    const int k_end = min(n, k_begin + p.split_tokens);

    if (k_begin >= k_end) {  // nothing visible in this split
        if (p.n_splits == 1) {
            // no visible key at all: the zero vector (zero dummy K/V of the first token, Section 2.1)
            uint16_t *o = (uint16_t *)p.out + ((int64_t)b * p.Hq + (int64_t)g * G) * D;
            for (int i = tid; i < G * D; i += W * 64) o[i] = 0;
        } else if (tid < G) {
            p.part_ml[((int64_t)split * p.B + b) * p.Hq + g * G + tid] = float2{kNegInf, 0.f};
        }
        return;
    }

    floatx4 acc[D / 16];
#pragma unroll
    for (int j = 0; j < D / 16; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
    float m = kNegInf, l = 0.f;
    const float cs = p.scale_log2e;
    const int lane_off = lane * 16;
    constexpr int kStride = W * NP;

    // Each kv head starts at a different place of its page range (and wraps around).  Workgroups launched
    // together advance in lockstep, and with an unlucky distance between their streams they would all press on
    // the same HBM channels at the same time (measured: up to 12 % of the bandwidth for some strides); the
    // order of the keys does not matter to softmax attention.  The rotation depends on the head only, so a
    // sequence's result still does not depend on the rest of the batch.
    PageWalk walk;
    walk.pg_begin = k_begin / kPage;
    walk.n_pages = (k_end + kPage - 1) / kPage - walk.pg_begin;
    walk.rot = (int)(((int64_t)g * walk.n_pages) / p.Hkv);

    // two tiles in flight per wave: the loads of the next tile are issued before the current one is used
    int it = wave * NP;
    Tile<D, NP> ta, tb;
    // (The last tile is consumed in a branch of its own rather than after a conditional prefetch: a wait placed
    // after a branch that may or may not have issued loads would have to wait for all of them.)
    if (it < walk.n_pages) {
        load_tile<D, NP, PAGED, NT>(ta, p.slot, b, g, it, walk, lane_off, p.dev_err);
        for (;;) {
            if (it + kStride < walk.n_pages) {
                load_tile<D, NP, PAGED, NT>(tb, p.slot, b, g, it + kStride, walk, lane_off, p.dev_err);
                consume_tile<D, NP>(ta, qb, acc, m, l, k_end, kb, cs);
            } else {
                consume_tile<D, NP>(ta, qb, acc, m, l, k_end, kb, cs);
                break;
            }
            it += kStride;
            if (it + kStride < walk.n_pages) {
                load_tile<D, NP, PAGED, NT>(ta, p.slot, b, g, it + kStride, walk, lane_off, p.dev_err);
                consume_tile<D, NP>(tb, qb, acc, m, l, k_end, kb, cs);
            } else {
                consume_tile<D, NP>(tb, qb, acc, m, l, k_end, kb, cs);
                break;
            }
            it += kStride;
        }
    }

    // denominators were kept per lane: add the four key quads of each column
    l = column_sum4(l);

    // merge the W waves: (m, l, O) per query column through LDS
    __shared__ float sm_m[W][16];
    __shared__ float sm_l[W][16];
    __shared__ floatx4 sm_acc[W][D / 16][64];
    if (kb == 0) {
        sm_m[wave][c] = m * cs;  // log2 units; -inf for a wave that saw no page
        sm_l[wave][c] = l;
    }
#pragma unroll
    for (int j = 0; j < D / 16; ++j) sm_acc[wave][j][lane] = acc[j];
    __syncthreads();

    float M = kNegInf;
#pragma unroll
    for (int w = 0; w < W; ++w) M = fmaxf(M, sm_m[w][c]);
    float f[W], L = 0.f;
#pragma unroll
    for (int w = 0; w < W; ++w) {
        float mw = sm_m[w][c];
        f[w] = (mw == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(mw - M);
        L += f[w] * sm_l[w][c];
    }
    // wave w finishes channel tiles w, w + W, ...
    for (int j = wave; j < D / 16; j += W) {
        floatx4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < W; ++w)
            if (f[w] != 0.f) o += f[w] * sm_acc[w][j][lane];
        if (c < G) {
            int d0 = j * 16 + 4 * kb;  // this lane holds channels d0..d0+3 of query head h
            if (p.n_splits == 1) {
                float inv = L > 0.f ? 1.f / L : 0.f;
                u32x2 pk = {pack_bf16(o[0] * inv, o[1] * inv), pack_bf16(o[2] * inv, o[3] * inv)};
                *(u32x2 *)((uint16_t *)p.out + row * D + d0) = pk;
            } else {
                *(floatx4 *)(p.part_o + (((int64_t)split * p.B + b) * p.Hq + h) * D + d0) = o;
            }
        }
    }
    if (p.n_splits > 1 && wave == 0 && kb == 0 && c < G)
        p.part_ml[((int64_t)split * p.B + b) * p.Hq + h] = float2{M, L};
}

template <int D, int NP, int W, bool PAGED, bool NT>
__global__ __launch_bounds__(W * 64) void attn_bf16_kernel(AttnParams p) {
    attn_bf16_unit<D, NP, W, PAGED, NT>(p, blockIdx.x, blockIdx.z * p.Hkv + blockIdx.y);
}

template <int D, int NP, int W>
static hipError_t launch_variant(const AttnParams &p, hipStream_t s) {
    dim3 grid(p.n_splits, p.Hkv, p.B), block(W * 64);
    if (p.slot.table) {
        if (p.nontemporal)
            hipLaunchKernelGGL((attn_bf16_kernel<D, NP, W, true, true>), grid, block, 0, s, p);
        else
            hipLaunchKernelGGL((attn_bf16_kernel<D, NP, W, true, false>), grid, block, 0, s, p);
    } else {
        if (p.nontemporal)
            hipLaunchKernelGGL((attn_bf16_kernel<D, NP, W, false, true>), grid, block, 0, s, p);
        else
            hipLaunchKernelGGL((attn_bf16_kernel<D, NP, W, false, false>), grid, block, 0, s, p);
    }
    return hipGetLastError();
}

hipError_t launch_attn_bf16(const AttnParams &p, int D, hipStream_t s) {
    // One page per wave and tile: measured fastest on MI355X for the Llama-7B shape (two- and four-page tiles were
    // 1-2 % slower).  At D = 128 the kernel takes 185 registers, i.e. two waves per SIMD; cut to the 168 that three
    // waves would allow it spills inside the loop and the step takes 47.9 instead of 39.9 ms.  Workgroups of 8 or 16 waves stand in for
    // two or up to four splits (the host's plan): the merge of the waves through LDS is then the whole merge.
    if (p.waves != 4 && p.waves != 8 && !(p.waves == 16 && D == 64)) return hipErrorInvalidValue;
    if (D == 128) return p.waves == 8 ? launch_variant<128, 1, 8>(p, s) : launch_variant<128, 1, 4>(p, s);
    if (p.waves == 16) return launch_variant<64, 1, 16>(p, s);
    return p.waves == 8 ? launch_variant<64, 1, 8>(p, s) : launch_variant<64, 1, 4>(p, s);
}

// The whole decode step in ONE launch, for slots so small that a layer's pass lasts about as long as a kernel
// launch (TinyLlama shape: 128 MiB, 17 us at the HBM peak): a grid that is resident all at once walks the layers in
// index order; a device-wide barrier ends every layer's attention, so layer l + 1 starts only when layer l's
// partial results are complete (in the model its query depends on layer l's output, Section 2.1).  After the
// barrier the workgroups first merge layer l's split partials (two sets of partials, taken in turn, so that the
// next layer's can be written meanwhile) and store the shared slot's new K/V if layer l produces them, then go on
// with layer l + 1.  The units of a layer - (split, kv head, sequence), the same as the per-layer launch's, so the
// results are the same bit for bit - are dealt round-robin to the workgroups.
// The barrier is an arrival counter in device memory: one thread per workgroup publishes the workgroup's stores
// (release fence at device scope), counts itself in and polls until all have arrived, then an acquire fence.  The
// wait is bounded: when the bound expires the thread raises LCKV_DEV_ERR_BARRIER and its workgroup leaves the
// kernel, and so does every other workgroup when its own bound expires - nothing waits for ever.
template <int D, bool PAGED, bool NT>
__global__ __launch_bounds__(256) void step_bf16_kernel(StepParams sp) {
    __shared__ int sm_failed;
    const int tid = threadIdx.x;
    const int64_t kv_elems = (int64_t)sp.a.B * sp.a.Hkv * D;
    const int64_t layer_bytes = (int64_t)sp.a.B * sp.a.Hq * D * 2;
    uint32_t arrivals = 0;
    // `acquire`: also drop what this compute unit and its L2 may hold of other workgroups' data from BEFORE the
    // barrier.  Needed only where plain loads after the barrier read addresses that were read earlier in this
    // launch and written since; an invalidation of the L2 by every workgroup at every barrier was measured to cost
    // more than the attention itself.  The merge reads the partials with device-scope loads instead, which need none.
    auto barrier = [&](bool acquire) -> bool {
        ++arrivals;
        __syncthreads();  // every wave of this workgroup has finished the phase
        if (tid == 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");  // the workgroup's stores, out of this XCD's L2
            // arrivals are counted in kBarrierGroups groups and the groups in a top counter: read-modify-writes on
            // one address are served one after the other, and several hundred of them per barrier took longer
            // than a layer's attention
            const uint32_t n_groups = min((uint32_t)kBarrierGroups, gridDim.x);
            const uint32_t gi = blockIdx.x % n_groups;
            const uint32_t group_size = (gridDim.x - gi + n_groups - 1) / n_groups;
            if (atomicAdd(sp.barrier + 1 + gi, 1u) + 1u == arrivals * group_size) atomicAdd(sp.barrier, 1u);
            const uint32_t target = arrivals * n_groups;
            const long long t0 = wall_clock64();
            int failed = 0;
            while (__hip_atomic_load(sp.barrier, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                if (wall_clock64() - t0 > sp.wait_ticks) {
                    atomicOr(sp.a.dev_err, LCKV_DEV_ERR_BARRIER);
                    failed = 1;
                    break;
                }
                __builtin_amdgcn_s_sleep(32);  // about 1 us between polls
            }
            if (acquire) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            sm_failed = failed;
        }
        __syncthreads();
        return sm_failed == 0;
    };
    auto slot_view_of = [&](int slot) {
        SlotView sv = sp.a.slot;
        sv.base = sp.storage + (int64_t)slot * sp.slot_bytes;
        return sv;
    };
    auto append_slot = [&](int slot) {
        const SlotView sv = slot_view_of(slot);
        const uint16_t *k = (const uint16_t *)sp.k_new_all + slot * kv_elems, *v = (const uint16_t *)sp.v_new_all + slot * kv_elems;
        for (int64_t i = (int64_t)blockIdx.x * 256 + tid; i < kv_elems; i += (int64_t)gridDim.x * 256)
            append_element<uint16_t>(sv, k, v, sp.a.seq_lens, D, sp.a.dev_err, i);
    };
    if (blockIdx.x == 0 && tid <= kBarrierGroups) sp.barrier_next[tid] = 0u;

    // warmup layers' new K/V into their private slots (read by nobody else): all at the start, one barrier
    bool any = false;
    for (int l = 0; l < sp.L; ++l)
        if (sp.layer_table[4 * l + 3] == kAppendAtStart) {
            append_slot(sp.layer_table[4 * l + 2]);
            any = true;
        }
    if (any && !barrier(false)) return;  // nothing of these slots has been read in this launch yet

    for (int l = 0; l < sp.L; ++l) {
        const int slot = sp.layer_table[4 * l], vis = sp.layer_table[4 * l + 1];
        const int produced = sp.layer_table[4 * l + 2], when = sp.layer_table[4 * l + 3];
        if (when == kAppendBeforeOwnAttention) {  // a slot other layers read too: only now, and a barrier of its own
            append_slot(produced);
            if (!barrier(true)) return;  // the layers below have read this slot's last page in this launch
        }
        AttnParams p = sp.a;
        p.slot = slot_view_of(slot);
        p.q = sp.q_all + l * layer_bytes;
        p.out = sp.out_all + l * layer_bytes;
        p.self_visible = vis;
        p.max_n = sp.max_n[vis];
        p.split_tokens = sp.split_tokens[vis];
        p.n_splits = sp.n_splits[vis];
        p.part_o = sp.part_o[l & 1];
        p.part_ml = sp.part_ml[l & 1];
        const int n_units = p.n_splits * sp.a.Hkv * sp.a.B;
        for (int u = blockIdx.x; u < n_units; u += gridDim.x) {
            attn_bf16_unit<D, 1, 4, PAGED, NT>(p, u % p.n_splits, u / p.n_splits);
            __syncthreads();  // the unit's LDS is free again
        }
        if (!barrier(false)) return;
        if (p.n_splits > 1) {
            const int64_t rows = (int64_t)sp.a.B * sp.a.Hq;
            for (int64_t i = (int64_t)blockIdx.x * 256 + tid; i < rows * D; i += (int64_t)gridDim.x * 256)
                combine_element<uint16_t, true>(p.part_o, p.part_ml, (uint16_t *)p.out, rows, D, p.n_splits, i);
        }
        if (when == kAppendAfterOwnAttention) append_slot(produced);
    }
    // the lengths are read by the appends: one more barrier if the last layer appended after its attention
    if (sp.layer_table[4 * (sp.L - 1) + 3] == kAppendAfterOwnAttention && !barrier(false)) return;
    if (blockIdx.x == 0)
        for (int i = tid; i < sp.a.B; i += 256) sp.seq_lens_rw[i] += 1;
}

template <int D, bool PAGED, bool NT>
static hipError_t launch_step_variant(const StepParams &sp, int max_units, hipStream_t s) {
    static int resident = 0;  // workgroups of this kernel the device holds at once (asked once)
    if (resident == 0) {
        int per_cu = 0, dev = 0;
        hipDeviceProp_t prop;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, step_bf16_kernel<D, PAGED, NT>, 256, 0) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess || per_cu < 1)
            return hipErrorInvalidValue;
        resident = per_cu * prop.multiProcessorCount;
    }
    int grid = max_units < resident ? max_units : resident;
    if (grid < 1) grid = 1;
    StepParams copy = sp;
    void *args[] = {&copy};
    return hipLaunchCooperativeKernel((const void *)step_bf16_kernel<D, PAGED, NT>, dim3(grid), dim3(256), args, 0, s);
}

hipError_t launch_step_bf16(const StepParams &sp, int D, int max_units, hipStream_t s) {
    // one load policy for the whole launch (the condensed layers'; the policy never changes a result)
    const bool paged = sp.a.slot.table != nullptr, nt = sp.nontemporal[0] != 0;
#define LCKV_STEP_LAUNCH(DD)                                                                             \
    (paged ? (nt ? launch_step_variant<DD, true, true>(sp, max_units, s) : launch_step_variant<DD, true, false>(sp, max_units, s)) \
           : (nt ? launch_step_variant<DD, false, true>(sp, max_units, s) : launch_step_variant<DD, false, false>(sp, max_units, s)))
    return D == 128 ? LCKV_STEP_LAUNCH(128) : LCKV_STEP_LAUNCH(64);
#undef LCKV_STEP_LAUNCH
}

// Measurement aid: stream `bytes` of device memory through the same access pattern the attention kernel uses
// (16 bytes per lane, a contiguous KiB per wave load, 16 KiB per wave in flight twice) and do nothing with it.
// Gives the read bandwidth a kernel of this shape can reach on the device at hand.
template <bool NT>
__global__ __launch_bounds__(256) void stream_probe_kernel(const char *buf, size_t bytes, int32_t *sink) {
    constexpr size_t kChunk = 2u << 20;  // bytes per workgroup visit
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    u32x4 x = {0u, 0u, 0u, 0u};
    for (size_t at = (size_t)blockIdx.x * kChunk; at + kChunk <= bytes; at += (size_t)gridDim.x * kChunk) {
        const char *base = buf + at + lane * 16;
        for (int t = wave * 16; t < (int)(kChunk / 1024); t += 64) {
            u32x4 r[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) r[i] = load16<NT>(base + (size_t)(t + i) * 1024);
#pragma unroll
            for (int i = 0; i < 16; ++i) x ^= r[i];
        }
    }
    if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == 0x9e3779b9u) *sink = 1;  // data-dependent, all but never true: keeps the loads alive
}

hipError_t launch_stream_probe(const void *buf, size_t bytes, int nontemporal, int32_t *sink, hipStream_t s) {
    size_t chunks = bytes / (2u << 20);
    unsigned blocks = (unsigned)(chunks < 8192 ? chunks : 8192);
    if (blocks == 0) return hipSuccess;
    if (nontemporal)
        hipLaunchKernelGGL(stream_probe_kernel<true>, dim3(blocks), dim3(256), 0, s, (const char *)buf, bytes, sink);
    else
        hipLaunchKernelGGL(stream_probe_kernel<false>, dim3(blocks), dim3(256), 0, s, (const char *)buf, bytes, sink);
    return hipGetLastError();
}

}  // namespace lckv
