// Attention of all prompt tokens of one layer in one pass, bf16 caches, gfx950 matrix cores (the parallel
// computation graph of Section 2.2 and the iterative prompt encoding of Section 2.3 of the LCKV paper): token i
// of a sequence attends to positions j < i of the slot its layer is paired with (condensed layer: diagonal
// masked, the slot holds the top layer's K/V of the previous iteration) or j <= i (warmup layer, the slot holds
// this iteration's own K/V).
//
// Same page layout as the decode kernel, but here the columns of a matrix tile are 32 consecutive query positions
// of one head, each with its own number of visible keys, and the tiles are 32 x 32:
//   S^T[32 keys][32 queries]  = K_pair[32 keys x D] . Q^T[D x 32 queries]       v_mfma_f32_32x32x16_bf16, D/16 steps
//   O^T[32 d][32 queries]    += V_page^T[32 d x 16 keys] . P^T[16 keys x 32 queries]   same instruction, per page
// With the 32 x 32 accumulator layout a lane holds 16 scores of ONE query (and lane + 32 the other 16): the running
// maximum and the row sum need a single v_permlane32_swap, and the 8 probabilities a lane packs per page are
// exactly the B operand of the P.V instruction of that page.  The V operand of that instruction - for the lane of
// channel d and half h: positions 4h..4h+3 and 8+4h..8+4h+3 of the page - is two 8-byte pieces 512 bytes apart in
// the page as stored, one two-address LDS read, no register shuffling.
// A workgroup of 4 waves owns 4 * QT * 32 positions of one head (QT tiles of 32 per wave) and walks the key pages
// 0 .. diagonal once, two pages (32 keys) at a time.  Pages are brought into LDS by direct global-to-LDS loads
// (global_load_lds_dwordx4; the cache stores pages in operand order, so the LDS image needs no rearrangement and
// every operand read is conflict-free), ST tiles of NPG pages in flight, and every page feeds all queries of the
// workgroup.  A wave's tiles that lie wholly below its first row go through a loop without masks; only the tiles
// the diagonal (or the end of the prompt) crosses pay for masking, in a second loop that shares the accumulators.
// No merge between waves.  Compute-bound; the K/V of a head (S * D * 4 bytes) stay in the L2 of the XCD that runs
// all row chunks of that head.
#include <type_traits>

#include "bf16_mfma_common.h"

namespace lckv {

namespace {

typedef __attribute__((address_space(3))) void *LdsPtr;
typedef __attribute__((address_space(4))) const int32_t *ConstTablePtr;
typedef __attribute__((ext_vector_type(16))) float floatx16;

#ifndef LCKV_PF_OCC
#define LCKV_PF_OCC 3
#endif
template <int D, int QT, int NPG, int ST, bool PAGED>
__global__ __launch_bounds__(256, (D * QT <= 128 ? LCKV_PF_OCC : 1)) void prefill_bf16_kernel(
    AttnParams p, int S, int heads_per_group) {
    // (waves per SIMD the register budget is cut for: within a wave the score products, the softmax and the P.V
    //  products run one after the other, so it is the other waves of the SIMD that keep the matrix core busy
    //  meanwhile)
    constexpr int kRows = 32 * QT;                 // query positions per wave
    constexpr int kPair = 2 * kPage * D * 2;       // bytes of a K page + V page
    constexpr int kLoadsPerPage = kPair / 1024;    // 1 KiB per wave-wide load
    constexpr int kLoadsPerWave = NPG * kLoadsPerPage / 4;
    constexpr int kSteps = D / 16;                 // matrix instructions per score tile
    constexpr int kDT = D / 32;                    // 32-channel tiles of the output
    static_assert(NPG * kLoadsPerPage % 4 == 0, "a tile's loads must divide among the four waves");
    static_assert(NPG % 2 == 0, "pages are consumed in pairs");
    constexpr float kLazy = 8.f;
    static_assert(ST >= 3 && ST <= 4, "tiles in flight (the staging areas of the prologue and epilogue need a third buffer)");
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
    const int c = lane & 31, hf = lane >> 5;  // query position within a tile / which half of the key octets
    const int g = h / p.G;
    const int i_wg = chunk * 4 * kRows;       // first row of the workgroup
    const int i_lo = i_wg + wave * kRows;     // first row of this wave

    // The queries first: their addresses need nothing that is loaded, so they travel while the prompt length and
    // the first tiles are fetched.  They are fetched in 128-byte half rows, 8 rows per instruction (whole cache
    // lines; fetching them in operand order would take 32 bytes of 32 different rows per instruction, which
    // measured 11 us per workgroup), and turned into operand order through LDS further down.  Rows past the end
    // of the tensor read the last row and are never stored.
    constexpr int kHalves = D / 64;            // 128-byte pieces of a query row
    u32x4 qraw[QT][kHalves][4];
    bf16x8 qb[QT][kSteps];                     // the operands made of them before the loop
#pragma unroll
    for (int x = 0; x < QT; ++x)
#pragma unroll
        for (int hv = 0; hv < kHalves; ++hv)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = min(i_lo + 32 * x + 8 * k + (lane >> 3), S - 1);
                const char *qp = (const char *)p.q + ((((int64_t)b * S + i) * p.Hq + h) * D) * 2;
                qraw[x][hv][k] = *(const u32x4 *)(qp + hv * 128 + (lane & 7) * 16);
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

    int n_col[QT];          // the number of keys each column sees
#pragma unroll
    for (int x = 0; x < QT; ++x) n_col[x] = min(i_lo + 32 * x + c + self, len);
    floatx16 acc[QT][kDT];
    float m[QT], l[QT];
#pragma unroll
    for (int x = 0; x < QT; ++x) {
        m[x] = kNegInf;
        l[x] = 0.f;
#pragma unroll
        for (int j = 0; j < kDT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[x][j][e] = 0.f;
    }
    const float cs = p.scale_log2e;
    const int lane_off = lane * 16;
    // pages needed by the workgroup (its last row) and by this wave; keys every row of this wave sees
    const int n_pages_wg = (min(i_wg + 4 * kRows - 1 + self, len) + kPage - 1) / kPage;
    const int n_pages = active ? (min(i_lo + kRows - 1 + self, len) + kPage - 1) / kPage : 0;
    const int n_plain = active ? min(i_lo + self, len) : 0;  // keys [0, n_plain) are visible to all of the wave's rows
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

    // Where this lane's operands sit in a page pair held in LDS (bytes from the pair's first page).
    //   K operand of step s (channels 16 s .. 16 s + 15, A operand: lane (key, hf) holds channels 16 s + 8 hf .. + 7
    //   of key `key` of the 32): the K page stores 16-byte chunks [channel octet][position]; octet 2 s + hf of
    //   position c % 16 of page c / 16.
    //   V operand of channel tile dt for one page (A operand: lane (d, hf) holds 8 positions of channel 32 dt + d):
    //   positions 4 hf .. 4 hf + 3 at quad hf and 8 + 4 hf .. at quad hf + 2 of the V page's
    //   [channel pair][quad][16 channels][2][4 positions] order - 8 bytes each, 512 bytes apart.
    const int k_lane = (c >> 4) * kPair + (hf * kPage + (c & 15)) * 16;
    //   Which channel a lane's row of the tile stands for is free (the output rows are sorted out at the end): row c
    //   is channel 32 dt + 16 (c % 2) + c / 2, which makes the 8-byte pieces of lanes 0..31 (and of 32..63)
    //   contiguous in LDS - with row c = channel c, neighbouring lanes' pieces lie 16 bytes apart and the two-address
    //   reads were measured at half the rate (152 against 285 bytes per ns and compute unit).
    const int v_lane = kPair / 2 + (hf * 32 + c) * 8;

    // One pair of pages (32 keys) against the wave's QT tiles of 32 queries.  DIAG = false: every key of the pair
    // is visible to every row of the wave - no masks.  DIAG = true: the diagonal or the end of the prompt crosses
    // the pair: scores are masked per column, and values at positions past the prompt are cleared (they may hold
    // anything, 0 * NaN would poison the sum).
    auto consume_pair = [&](const char *pair, int pg, auto diag_tag) {
        constexpr bool DIAG = decltype(diag_tag)::value;
        floatx16 z[QT];
#pragma unroll
        for (int x = 0; x < QT; ++x)
#pragma unroll
            for (int e = 0; e < 16; ++e) z[x][e] = 0.f;
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            const u32x4 kr = *(const u32x4 *)(pair + k_lane + s * 512);
#pragma unroll
            for (int x = 0; x < QT; ++x)
                z[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kr), qb[x][s], z[x], 0, 0, 0);
        }
        bf16x8 pb[QT][2];
#pragma unroll
        for (int x = 0; x < QT; ++x) {
            // score register e of this lane: key pg * 16 + 8 (e / 4) + 4 hf + e % 4 of query column c
            if (DIAG) {
                const int key0 = pg * kPage + 4 * hf;
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (key0 + 8 * (e >> 2) + (e & 3) >= n_col[x]) z[x][e] = kNegInf;
            }
            float smax = fmaxf(fmaxf(z[x][0], z[x][1]), z[x][2]);
#pragma unroll
            for (int e = 3; e < 15; e += 2) smax = fmaxf(fmaxf(smax, z[x][e]), z[x][e + 1]);
            smax = fmaxf(smax, z[x][15]);
            {   // the two lanes of a column (c and c + 32) share one running maximum
                float a = smax, bb = smax;
                swap_halves32(a, bb);
                smax = fmaxf(a, bb);
            }
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
                for (int j = 0; j < kDT; ++j) acc[x][j] *= alpha;
            }
            const float mb = (m[x] == kNegInf ? 0.f : m[x]) * cs;
            float pr[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) pr[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(z[x][e], cs, -mb));
#pragma unroll
            for (int pgi = 0; pgi < 2; ++pgi) {
                const float *q8 = pr + 8 * pgi;
                const u32x4 pk = {pack_bf16(q8[0], q8[1]), pack_bf16(q8[2], q8[3]), pack_bf16(q8[4], q8[5]),
                                  pack_bf16(q8[6], q8[7])};
                pb[x][pgi] = __builtin_bit_cast(bf16x8, pk);
            }
            l[x] += (((pr[0] + pr[1]) + (pr[2] + pr[3])) + ((pr[4] + pr[5]) + (pr[6] + pr[7]))) +
                    (((pr[8] + pr[9]) + (pr[10] + pr[11])) + ((pr[12] + pr[13]) + (pr[14] + pr[15])));
        }
#pragma unroll
        for (int pgi = 0; pgi < 2; ++pgi) {
            uint32_t k01 = 0xffffffffu, k23 = 0xffffffffu, k45 = 0xffffffffu, k67 = 0xffffffffu;
            bool clear_stale = false;
            if (DIAG) {
                clear_stale = (pg + pgi + 1) * kPage > len;  // wave-uniform: the prompt ends inside this page
                if (clear_stale) {
                    const int nv0 = len - ((pg + pgi) * kPage + 4 * hf), nv1 = nv0 - 8;  // valid among each four
                    k01 = nv0 >= 2 ? 0xffffffffu : (nv0 == 1 ? 0x0000ffffu : 0u);
                    k23 = nv0 >= 4 ? 0xffffffffu : (nv0 == 3 ? 0x0000ffffu : 0u);
                    k45 = nv1 >= 2 ? 0xffffffffu : (nv1 == 1 ? 0x0000ffffu : 0u);
                    k67 = nv1 >= 4 ? 0xffffffffu : (nv1 == 3 ? 0x0000ffffu : 0u);
                }
            }
#pragma unroll
            for (int dt = 0; dt < kDT; ++dt) {
                const char *vp = pair + pgi * kPair + v_lane + dt * 1024;
                const u32x2 lo = *(const u32x2 *)vp;
                const u32x2 hi = *(const u32x2 *)(vp + 512);
                u32x4 vr = {lo[0], lo[1], hi[0], hi[1]};
                if (DIAG && clear_stale) {
                    const u32x4 keep = {k01, k23, k45, k67};
                    vr &= keep;
                }
#pragma unroll
                for (int x = 0; x < QT; ++x)
                    acc[x][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vr), pb[x][pgi],
                                                                         acc[x][dt], 0, 0, 0);
            }
        }
    };

    // Tile t is consumed while tiles t+1 .. t+ST-1 are on their way (a page that misses the L2 takes longer to
    // arrive than a tile takes to consume).  One barrier per tile: past it, every wave's share of tile t has
    // landed (each waited for its own loads first: they complete in order, so "at most as many outstanding as the
    // later tiles have" means tile t is there) and every wave has finished reading tile t-1, whose buffer the
    // loads of tile t+ST-1 then overwrite.
    for (int t = 0; t < ST - 1 && t < n_tiles; ++t) issue_tile(t);
    // Q^T operands: lane (c, hf) holds channels 16 s + 8 hf .. + 7 of query i_lo + 32 x + c.  Each wave turns its
    // half rows around in a 4 KiB piece of the last tile buffer, which no load targets before the first barrier:
    // 32 rows of 128 bytes, the 16-byte chunks of a row exchanged by the row number (chunk ^ row % 8) so that
    // neither the row-wise writes nor the column-wise reads pile up on a bank.  Wave-private, hence no barrier;
    // the reads are waited for here, before the loop (a wait inside the loop would be a wait for all loads in
    // flight).
    {
        static_assert(4 * 32 * 128 <= NPG * kPair, "the staging area is one tile buffer");
        char *stage = &lds[ST - 1][wave * 4096];
#pragma unroll
        for (int x = 0; x < QT; ++x)
#pragma unroll
            for (int hv = 0; hv < kHalves; ++hv) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int row = 8 * k + (lane >> 3);
                    *(u32x4 *)(stage + row * 128 + (((lane & 7) ^ (row & 7)) * 16)) = qraw[x][hv][k];
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4) {
                    const u32x4 v = *(const u32x4 *)(stage + c * 128 + (((2 * s4 + hf) ^ (c & 7)) * 16));
                    qb[x][hv * 4 + s4] = __builtin_bit_cast(bf16x8, v);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
    }
#pragma unroll
    for (int x = 0; x < QT; ++x)
#pragma unroll
        for (int s = 0; s < kSteps; ++s) asm volatile("" ::"v"(qb[x][s]));  // a use: the compiler waits here
    auto sync_tile = [&](int t) {
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
    };
    // Two loops over the tiles, one after the other, sharing the accumulators: first the tiles all of whose keys
    // every row of this wave sees (no masks), then the rest.  Every wave passes n_tiles barriers in all, wherever
    // its own first loop ends.  (One loop with the choice inside made the compiler copy all accumulators between
    // two register sets in every round.)
    const int t_plain = min(n_tiles, n_plain / (NPG * kPage));  // tiles 0 .. t_plain - 1 lie below the wave's first row
    int t = 0;
    for (; t < t_plain; ++t) {
        sync_tile(t);
#pragma unroll
        for (int j = 0; j < NPG; j += 2) consume_pair(&lds[t % ST][j * kPair], t * NPG + j, std::false_type{});
    }
    for (; t < n_tiles; ++t) {
        sync_tile(t);
#pragma unroll
        for (int j = 0; j < NPG; j += 2) {
            const int pg = t * NPG + j;
            if (pg < n_pages) consume_pair(&lds[t % ST][j * kPair], pg, std::true_type{});
        }
    }
    if (!active) return;

    // O^T accumulator register e of channel tile dt: row i = 8 (e / 4) + 4 hf + e % 4 of the tile, i.e. channel
    // 32 dt + 16 (i % 2) + i / 2, of query column c: registers 4 q .. 4 q + 3 are channels a, 16 + a, a + 1, 17 + a
    // with a = 4 q + 2 hf.
    // The rounded rows are turned around in LDS (a piece of the tile buffers that nobody reads any more: not the
    // last tile's, which a slower wave may still be consuming) so that they leave as whole 2 D-byte rows, several
    // rows per store instruction, instead of 8-byte pieces of 32 different rows.
    constexpr int kRowBytes = D * 2, kCpr = D / 8;          // 16-byte chunks per row
    constexpr int kStage = 32 * kRowBytes, kBuf = NPG * kPair;
    static_assert(kBuf % kStage == 0 && 4 * kStage <= 2 * kBuf, "staging areas of the four waves fit two buffers");
    char *stage = &lds[(n_tiles + (wave * kStage) / kBuf) % ST][(wave * kStage) % kBuf];
#pragma unroll
    for (int x = 0; x < QT; ++x) {
        float a = l[x], bb = l[x];
        swap_halves32(a, bb);
        const float L = a + bb;
        const int i = i_lo + 32 * x + c;
        const float inv = (i < len && L > 0.f) ? 1.f / L : 0.f;  // rows past the prompt, and a token that sees
                                                                 // nothing (zero dummy K/V), are zero
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const floatx16 &a16 = acc[x][dt];
                const uint32_t lo = pack_bf16(a16[4 * q4] * inv, a16[4 * q4 + 2] * inv);      // channels a, a + 1
                const uint32_t hi = pack_bf16(a16[4 * q4 + 1] * inv, a16[4 * q4 + 3] * inv);  // channels 16 + a, 17 + a
                const int a = 4 * q4 + 2 * hf;                                               // within the tile of 32
                const int chunk_lo = 4 * dt + (a >> 3), chunk_hi = chunk_lo + 2;             // 16-byte chunks of 8 channels
                char *row = stage + c * kRowBytes;
                *(uint32_t *)(row + ((chunk_lo ^ (c & (kCpr - 1))) * 16) + (a & 7) * 2) = lo;
                *(uint32_t *)(row + ((chunk_hi ^ (c & (kCpr - 1))) * 16) + (a & 7) * 2) = hi;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int k = 0; k < 32 * kCpr / 64; ++k) {
            const int row = k * (64 / kCpr) + lane / kCpr, chunk = lane % kCpr;
            const u32x4 v = *(const u32x4 *)(stage + row * kRowBytes + ((chunk ^ (row & (kCpr - 1))) * 16));
            const int i_row = i_lo + 32 * x + row;
            if (i_row < S) *(u32x4 *)(out + (((int64_t)b * S + i_row) * p.Hq + h) * D + chunk * 8) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

template <int D, int QT, int NPG, int ST = 3>
hipError_t launch_qt(const AttnParams &p, int S, hipStream_t s) {
    const int rows_per_group = 4 * 32 * QT;
    const int n_chunks = (S + rows_per_group - 1) / rows_per_group;
    const int64_t units = (int64_t)p.Hq * p.B, units_per_xcd = (units + 7) / 8;
    const int heads_per_group = 8;  // measured on the Llama-7B shape: 1: 648, 2: 671, 4: 685, 8: 693, 16: 670 TFLOP/s
    const int64_t per_xcd = (units_per_xcd + heads_per_group - 1) / heads_per_group * heads_per_group * n_chunks;
    if (per_xcd * 8 > (int64_t)1 << 30) return hipErrorInvalidValue;
    dim3 grid((unsigned)(per_xcd * 8)), block(256);  // one task per workgroup, the same number for each of the 8 XCDs
    if (p.slot.table)
        hipLaunchKernelGGL((prefill_bf16_kernel<D, QT, NPG, ST, true>), grid, block, 0, s, p, S, heads_per_group);
    else
        hipLaunchKernelGGL((prefill_bf16_kernel<D, QT, NPG, ST, false>), grid, block, 0, s, p, S, heads_per_group);
    return hipGetLastError();
}

}  // namespace

// p: seq_lens = prompt lengths, max_n = min(S, capacity), self_visible, scale; no splits.
// qb: 16-position query blocks per wave, 2 (one 32-query tile) or 4 (two); 0 = default.
hipError_t launch_prefill_bf16(const AttnParams &p, int S, int D, int qb, hipStream_t s) {
    if (qb == 0) qb = 2;
    if (D == 128) return qb == 2 ? launch_qt<128, 1, 2>(p, S, s) : launch_qt<128, 2, 2>(p, S, s);
    return qb == 2 ? launch_qt<64, 1, 4>(p, S, s) : launch_qt<64, 2, 4>(p, S, s);
}

}  // namespace lckv
