// Attention of all prompt tokens of one layer in one pass, bf16 caches, gfx950 matrix cores (the parallel
// computation graph of Section 2.2 and the iterative prompt encoding of Section 2.3 of the LCKV paper): token i
// of a sequence attends to positions j < i of the slot its layer is paired with (condensed layer: diagonal
// masked, the slot holds the top layer's K/V of the previous iteration) or j <= i (warmup layer, the slot holds
// this iteration's own K/V).
//
// Same matrix tiles and page layout as the decode kernel, but the 16 columns of a tile are 16 consecutive query
// positions of one head instead of the heads of a group, and each column has its own number of visible keys:
//   S^T[key][pos] = K_page . Q^T       (v_mfma_f32_16x16x32_bf16)
//   O^T[d][pos]  += V_pages^T . P^T    (v_mfma_f32_16x16x32_bf16 over two pages = 32 keys at a time)
// A workgroup of 4 waves owns 4 * QB blocks of 16 positions of one head (QB per wave) and walks the key pages
// 0 .. diagonal once.  Pages are brought into LDS by direct global-to-LDS loads (global_load_lds_dwordx4; the
// cache stores pages in operand order, so the LDS image needs no rearrangement and every wave reads its operands
// with conflict-free ds_read_b128), ST tiles of NPG pages in flight, and every page feeds all 64 * QB queries of
// the workgroup.  No merge between waves.  Compute-bound; the K/V of a head (S * D * 4 bytes) stay in the L2 of
// the XCD that runs all row chunks of that head.
#include "bf16_mfma_common.h"

namespace lckv {

namespace {

typedef __attribute__((address_space(3))) void *LdsPtr;
typedef __attribute__((address_space(4))) const int32_t *ConstTablePtr;

template <int D, int QB, int NPG, int ST, bool PAGED>
__global__ __launch_bounds__(256, (QB <= 2 ? 3 : D * QB > 384 ? 1 : 2)) void prefill_bf16_kernel(AttnParams p, int S, int heads_per_group) {
    // (waves per SIMD the register budget is cut for: within a wave the score products, the softmax and the P.V
    //  products run one after the other, so it is the other waves of the SIMD that keep the matrix core busy
    //  meanwhile - 3 waves at 2 query blocks per wave measured faster than 2 waves with more registers each; the
    //  128-channel, 4-block shape needs 128 registers for its accumulators alone)
    constexpr int kRows = 16 * QB;                 // query positions per wave
    constexpr int kPair = 2 * kPage * D * 2;       // bytes of a K page + V page
    constexpr int kLoadsPerPage = kPair / 1024;    // 1 KiB per wave-wide load
    constexpr int kLoadsPerWave = NPG * kLoadsPerPage / 4;
    static_assert(NPG * kLoadsPerPage % 4 == 0, "a tile's loads must divide among the four waves");
    static_assert(NPG % 2 == 0, "pages are consumed in pairs");
    constexpr float kLazy = 8.f;
    static_assert(ST >= 2 && ST <= 4, "tiles in flight");
    __shared__ __attribute__((aligned(16))) char lds[ST][NPG * kPair];

    // Which (sequence, head, row chunk) this workgroup takes.  Workgroups are handed to the 8 XCDs round-robin
    // by their launch index, and every XCD has an L2 of its own: the launch index is unfolded so that each XCD
    // gets a contiguous range of tasks, i.e. all row chunks of a head (and the heads of one kv group) run on one
    // XCD at about the same time and share that head's K/V pages in its L2.
    // Inside an XCD the heads are taken in groups of `heads_per_group`, and within a group the row chunks with
    // the most keys come first, for all its heads, before the shorter ones: the longest tasks of the whole list
    // are then not the last ones to start (list scheduling of the triangle: 91 % of the ideal makespan with one
    // head per group, 98 % with eight), while a group's K/V are still few enough to live in the L2.
    constexpr int kXcd = 8;
    const int n_chunks = (S + 4 * kRows - 1) / (4 * kRows);
    const int units = p.Hq * p.B;  // (sequence, head) pairs
    const int units_per_xcd = (units + kXcd - 1) / kXcd;
    const int xcd = blockIdx.x % kXcd, idx = blockIdx.x / kXcd;
    const int group = idx / (heads_per_group * n_chunks), rest = idx % (heads_per_group * n_chunks);
    const int unit = xcd * units_per_xcd + group * heads_per_group + rest % heads_per_group;
    if (unit >= min((xcd + 1) * units_per_xcd, units)) return;
    const int chunk = n_chunks - 1 - rest / heads_per_group;  // rows with the most keys first
    const int h = unit % p.Hq, b = unit / p.Hq;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, kb = lane >> 4;  // query position within a block / key quad
    const int g = h / p.G;
    const int i_wg = chunk * 4 * kRows;       // first row of the workgroup
    const int i_lo = i_wg + wave * kRows;     // first row of this wave

    // Q^T operands first: their addresses need nothing that is loaded, so they travel while the prompt length
    // and the first tiles are fetched (rows past the prompt are read too - they exist - and not used); they are
    // waited for just before the loop.
    bf16x8 qb[QB][D / 32];
#pragma unroll
    for (int x = 0; x < QB; ++x) {
        const int i = i_lo + 16 * x + c;
        const char *qp = (const char *)p.q + ((((int64_t)b * S + i) * p.Hq + h) * D + kb * 8) * 2;
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (i < S) v = *(const u32x4 *)(qp + ks * 64);
            qb[x][ks] = __builtin_bit_cast(bf16x8, v);
        }
    }
    int len = ((ConstTablePtr)p.seq_lens)[b];  // a scalar load (the lengths are not written while the kernel runs)
    if (len > p.max_n) {
        len = p.max_n;
        if (tid == 0) atomicOr(p.dev_err, LCKV_DEV_ERR_CAPACITY);
    }
    if (len < 0) len = 0;
    uint16_t *out = (uint16_t *)p.out;
    const int self = p.self_visible;
    const bool active = i_lo < len;           // wave-uniform: this wave has rows inside the prompt

    if (!active) {  // rows past the prompt are zero
        for (int r = 0; r < kRows && i_lo + r < S; ++r) {
            uint32_t *o = (uint32_t *)(out + (((int64_t)b * S + i_lo + r) * p.Hq + h) * D);
            for (int e = lane; e < D / 2; e += 64) o[e] = 0u;
        }
    }
    if (i_wg >= len) return;  // uniform over the workgroup: nothing to attend

    int n_col[QB];          // the number of keys each column sees
#pragma unroll
    for (int x = 0; x < QB; ++x) n_col[x] = min(i_lo + 16 * x + c + self, len);
    floatx4 acc[QB][D / 16];
    float m[QB], l[QB];
#pragma unroll
    for (int x = 0; x < QB; ++x) {
        m[x] = kNegInf;
        l[x] = 0.f;
#pragma unroll
        for (int j = 0; j < D / 16; ++j) acc[x][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    const float cs = p.scale_log2e;
    const int lane_off = lane * 16;
    // pages needed by the workgroup (its last row) and by this wave
    const int n_pages_wg = (min(i_wg + 4 * kRows - 1 + self, len) + kPage - 1) / kPage;
    const int n_pages = active ? (min(i_lo + kRows - 1 + self, len) + kPage - 1) / kPage : 0;
    const int n_tiles = (n_pages_wg + NPG - 1) / NPG;

    // This wave's share of the loads of tile t: 1 KiB pieces wave, wave + 4, ... of the tile's NPG page pairs.
    auto issue_tile = [&](int t) {
#pragma unroll
        for (int r = 0; r < kLoadsPerWave; ++r) {
            const int piece = wave + 4 * r;
            int pg = t * NPG + piece / kLoadsPerPage;
            if (pg >= n_pages_wg) pg = n_pages_wg - 1;  // past the end: any mapped page, it is not used
            int64_t idx;
            if (PAGED) {
                // read through the constant address space: a scalar load, which does not queue behind the tile
                // loads in flight as a vector load would (the table is not written while the kernel runs)
                int32_t blk = ((ConstTablePtr)p.slot.table)[(int64_t)b * p.slot.max_blocks + pg];
                if (blk < 0 || (int64_t)blk >= p.slot.num_blocks) {
                    if (lane == 0) atomicOr(p.dev_err, LCKV_DEV_ERR_BLOCK);
                    blk = 0;  // read something that exists; this sequence's result is undefined, the error is raised
                }
                idx = (int64_t)blk * p.slot.Hkv + g;
            } else {
                idx = ((int64_t)b * p.slot.Hkv + g) * p.slot.pages_per_seq + pg;
            }
            const char *src = p.slot.base + idx * kPair + (piece % kLoadsPerPage) * 1024 + lane_off;
            // global_load_lds_dwordx4: lane l's 16 bytes land at LDS address M0 + 16 * l.  Issued as assembly, not
            // through the compiler's builtin: the compiler cannot tell which LDS reads such a load may alias and
            // makes every LDS read after one wait for ALL loads in flight, which forfeits the prefetch.  The
            // waits are placed by hand below.
            const uint32_t dst = (uint32_t)(uintptr_t)(LdsPtr)(&lds[t % ST][piece * 1024]);
            uint32_t m0_saved;  // M0 carries the LDS address; whatever the compiler keeps there is put back
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\t"
                         "s_mov_b32 m0, %0"
                         : "=&s"(m0_saved)
                         : "s"(dst), "v"(src)
                         : "memory");
        }
    };

    // Two consecutive pages (32 keys) at a time: one softmax update per 32 keys, and the P.V product runs on the
    // full-rate 16x16x32 instruction - its 8 keys per lane are this lane's 4 keys of the first page and its 4
    // keys of the second, which is how the two score tiles and the two V operands already sit in registers.
    // `second` (wave-uniform) is false when the pair's second page lies above this wave's diagonal.
    // In three phases (scores of all QB blocks, softmax, P.V of all blocks) so that the K operands and the V
    // operands are not live in registers at the same time.
    auto consume_pair = [&](const char *page0, int pg, bool second) {
        const char *page1 = page0 + kPair;
        floatx4 z0[QB], z1[QB];
        bool live[QB];  // wave-uniform: the block sees at least one key of the pair
        {
            u32x4 kr[D / 32];
#pragma unroll
            for (int ks = 0; ks < D / 32; ++ks) kr[ks] = *(const u32x4 *)(page0 + ks * 1024 + lane_off);
#pragma unroll
            for (int x = 0; x < QB; ++x) {
                const int n_hi = min(i_lo + 16 * x + 15 + self, len);  // keys the last column of the block sees
                live[x] = pg * kPage < n_hi;
                z0[x] = floatx4{0.f, 0.f, 0.f, 0.f};
                z1[x] = floatx4{kNegInf, kNegInf, kNegInf, kNegInf};
                if (!live[x]) continue;
#pragma unroll
                for (int ks = 0; ks < D / 32; ++ks)
                    z0[x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kr[ks]), qb[x][ks],
                                                                    z0[x], 0, 0, 0);
            }
            if (second) {
#pragma unroll
                for (int ks = 0; ks < D / 32; ++ks) kr[ks] = *(const u32x4 *)(page1 + ks * 1024 + lane_off);
#pragma unroll
                for (int x = 0; x < QB; ++x) {
                    const int n_hi = min(i_lo + 16 * x + 15 + self, len);
                    if ((pg + 1) * kPage >= n_hi) continue;  // the second page lies above this block's diagonal
                    z1[x] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < D / 32; ++ks)
                        z1[x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kr[ks]), qb[x][ks],
                                                                        z1[x], 0, 0, 0);
                }
            }
        }
        bf16x8 pb[QB];
#pragma unroll
        for (int x = 0; x < QB; ++x) {
            if (!live[x]) continue;
            const int n_lo = min(i_lo + 16 * x + self, len);  // keys the first column of the block sees
            if ((pg + 2) * kPage > n_lo) {                    // the diagonal crosses this pair: mask per column
                const int key0 = pg * kPage + 4 * kb;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (key0 + e >= n_col[x]) z0[x][e] = kNegInf;
                    if (key0 + kPage + e >= n_col[x]) z1[x][e] = kNegInf;
                }
            }
            float smax = fmaxf(fmaxf(fmaxf(z0[x][0], z0[x][1]), fmaxf(z0[x][2], z0[x][3])),
                               fmaxf(fmaxf(z1[x][0], z1[x][1]), fmaxf(z1[x][2], z1[x][3])));
            smax = column_max4(smax);
            // The running reference m[x] follows the true maximum lazily: the accumulators are rescaled only when
            // some column's maximum has outgrown its reference by more than 2^kLazy (or has no reference yet), so
            // the weights stay <= 2^kLazy - harmless in fp32 sums and at bf16's relative precision - and the result
            // O / l is the same quotient.  (Both -inf: the comparison is false, nothing has been seen.)
            if (__builtin_amdgcn_ballot_w64((smax - m[x]) * cs > kLazy) != 0) {
                const float m_new = fmaxf(m[x], smax);
                const float alpha = __builtin_amdgcn_exp2f((m[x] - (m_new == kNegInf ? 0.f : m_new)) * cs);
                m[x] = m_new;
                l[x] *= alpha;
#pragma unroll
                for (int j = 0; j < D / 16; ++j) acc[x][j] *= alpha;
            }
            const float mb = (m[x] == kNegInf ? 0.f : m[x]) * cs;
            float pr[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pr[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(z0[x][e], cs, -mb));
                pr[4 + e] = __builtin_amdgcn_exp2f(__builtin_fmaf(z1[x][e], cs, -mb));
            }
            const u32x4 pk = {pack_bf16(pr[0], pr[1]), pack_bf16(pr[2], pr[3]), pack_bf16(pr[4], pr[5]),
                              pack_bf16(pr[6], pr[7])};
            pb[x] = __builtin_bit_cast(bf16x8, pk);
            l[x] += ((pr[0] + pr[1]) + (pr[2] + pr[3])) + ((pr[4] + pr[5]) + (pr[6] + pr[7]));
        }
        uint32_t a01 = 0xffffffffu, a23 = 0xffffffffu, b01 = 0xffffffffu, b23 = 0xffffffffu;
        if ((pg + 2) * kPage > len) {  // the prompt ends inside this pair: clear stale values (0 * NaN)
            const int nv0 = len - (pg * kPage + 4 * kb), nv1 = nv0 - kPage;
            a01 = nv0 >= 2 ? 0xffffffffu : (nv0 == 1 ? 0x0000ffffu : 0u);
            a23 = nv0 >= 4 ? 0xffffffffu : (nv0 == 3 ? 0x0000ffffu : 0u);
            b01 = nv1 >= 2 ? 0xffffffffu : (nv1 == 1 ? 0x0000ffffu : 0u);
            b23 = nv1 >= 4 ? 0xffffffffu : (nv1 == 3 ? 0x0000ffffu : 0u);
        }
        if (!second) b01 = b23 = 0u;  // that LDS page holds nothing of this wave's
        const bool clear_stale = (pg + 2) * kPage > len || !second;
#pragma unroll
        for (int dp = 0; dp < D / 32; ++dp) {
            const u32x4 v0 = *(const u32x4 *)(page0 + kPair / 2 + dp * 1024 + lane_off);
            const u32x4 v1 = *(const u32x4 *)(page1 + kPair / 2 + dp * 1024 + lane_off);
            u32x4 lo = {v0[0], v0[1], v1[0], v1[1]};  // channel block 2dp, 8 keys
            u32x4 hi = {v0[2], v0[3], v1[2], v1[3]};  // channel block 2dp + 1
            if (clear_stale) {                        // wave-uniform, true only for a wave's last pairs
                const u32x4 keep = {a01, a23, b01, b23};
                lo &= keep;
                hi &= keep;
            }
#pragma unroll
            for (int x = 0; x < QB; ++x) {
                if (!live[x]) continue;
                acc[x][2 * dp] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, lo), pb[x],
                                                                         acc[x][2 * dp], 0, 0, 0);
                acc[x][2 * dp + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, hi), pb[x],
                                                                             acc[x][2 * dp + 1], 0, 0, 0);
            }
        }
    };

    // Tile t is consumed while tiles t+1 .. t+ST-1 are on their way (a page that misses the L2 takes longer to
    // arrive than a tile takes to consume).  One barrier per tile: past it, every wave's share of tile t has
    // landed (each waited for its own loads first: they complete in order, so "at most as many outstanding as the
    // later tiles have" means tile t is there) and every wave has finished reading tile t-1, whose buffer the
    // loads of tile t+ST-1 then overwrite.
    for (int t = 0; t < ST - 1 && t < n_tiles; ++t) issue_tile(t);
    // The Q^T operands are waited for here, before the loop: a wait for them inside the loop would be a wait for
    // all loads in flight.
#pragma unroll
    for (int x = 0; x < QB; ++x)
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) asm volatile("" ::"v"(qb[x][ks]));  // a use: the compiler waits here
    for (int t = 0; t < n_tiles; ++t) {
        const int later = min(ST - 2, n_tiles - 1 - t);  // tiles issued after tile t
        if (later <= 0)
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (later == 1)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerWave) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kLoadsPerWave) : "memory");
        // the bare barrier instruction: __syncthreads() comes with a fence that waits for ALL outstanding loads
        asm volatile("s_barrier" ::: "memory");
        if (t + ST - 1 < n_tiles) issue_tile(t + ST - 1);
#pragma unroll
        for (int j = 0; j < NPG; j += 2) {
            const int pg = t * NPG + j;
            if (pg < n_pages) consume_pair(&lds[t % ST][j * kPair], pg, pg + 1 < n_pages);
        }
    }
    if (!active) return;

#pragma unroll
    for (int x = 0; x < QB; ++x) {
        const float L = column_sum4(l[x]);
        const int i = i_lo + 16 * x + c;
        if (i >= S) continue;
        const float inv = (i < len && L > 0.f) ? 1.f / L : 0.f;  // rows past the prompt, and a token that sees
                                                                 // nothing (zero dummy K/V), are zero
        uint16_t *o = out + (((int64_t)b * S + i) * p.Hq + h) * D + 4 * kb;
#pragma unroll
        for (int j = 0; j < D / 16; ++j) {
            const floatx4 a = acc[x][j];
            u32x2 pk = {pack_bf16(a[0] * inv, a[1] * inv), pack_bf16(a[2] * inv, a[3] * inv)};
            *(u32x2 *)(o + j * 16) = pk;
        }
    }
}

template <int D, int QB, int NPG, int ST = 3>
hipError_t launch_qb(const AttnParams &p, int S, hipStream_t s) {
    const int rows_per_group = 4 * 16 * QB;
    const int n_chunks = (S + rows_per_group - 1) / rows_per_group;
    const int64_t units = (int64_t)p.Hq * p.B, units_per_xcd = (units + 7) / 8;
    const int heads_per_group = 8;  // measured on the Llama-7B shape: 1: 648, 2: 671, 4: 685, 8: 693, 16: 670 TFLOP/s
    const int64_t per_xcd = (units_per_xcd + heads_per_group - 1) / heads_per_group * heads_per_group * n_chunks;
    if (per_xcd * 8 > (int64_t)1 << 30) return hipErrorInvalidValue;
    dim3 grid((unsigned)(per_xcd * 8)), block(256);  // one task per workgroup, the same number for each of the 8 XCDs
    if (p.slot.table)
        hipLaunchKernelGGL((prefill_bf16_kernel<D, QB, NPG, ST, true>), grid, block, 0, s, p, S, heads_per_group);
    else
        hipLaunchKernelGGL((prefill_bf16_kernel<D, QB, NPG, ST, false>), grid, block, 0, s, p, S, heads_per_group);
    return hipGetLastError();
}

}  // namespace

// p: seq_lens = prompt lengths, max_n = min(S, capacity), self_visible, scale; no splits.
hipError_t launch_prefill_bf16(const AttnParams &p, int S, int D, int qb, hipStream_t s) {
    if (qb == 0) qb = 2;  // measured: 643 vs 284 TFLOP/s at D=128 (Llama-7B shape), 543 vs 509 at D=64 (TinyLlama shape)
    if (D == 128) return qb == 2 ? launch_qb<128, 2, 2>(p, S, s) : launch_qb<128, 4, 2>(p, S, s);
    return qb == 2 ? launch_qb<64, 2, 4>(p, S, s) : launch_qb<64, 4, 4>(p, S, s);
}

}  // namespace lckv
