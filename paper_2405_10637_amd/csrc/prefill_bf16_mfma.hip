// Attention of all prompt tokens of one layer in one pass, bf16 caches, gfx950 matrix cores (the parallel
// computation graph of Section 2.2 and the iterative prompt encoding of Section 2.3 of the LCKV paper): token i
// of a sequence attends to positions j < i of the slot its layer is paired with (condensed layer: diagonal
// masked, the slot holds the top layer's K/V of the previous iteration) or j <= i (warmup layer, the slot holds
// this iteration's own K/V).
//
// Same matrix tiles and page layout as the decode kernel, but the 16 columns of a tile are 16 consecutive query
// positions of one head instead of the heads of a group, and each column has its own number of visible keys:
//   S^T[key][pos] = K_page . Q^T       (v_mfma_f32_16x16x32_bf16)
//   O^T[d][pos]  += V_page^T . P^T     (v_mfma_f32_16x16x16_bf16)
// A wave owns QB blocks of 16 positions, walks the key pages 0 .. diagonal once and applies every page to all its
// blocks (a page loaded once feeds 16*QB queries); pages come straight from the cache in operand order, there is
// no LDS and no merge between waves.  Compute-bound; K/V re-reads come from L2.
#include "bf16_mfma_common.h"

namespace lckv {

namespace {

template <int D>
struct PageRegs {
    u32x4 k[D / 32];
    u32x4 v[D / 32];
};

template <int D, bool PAGED>
__device__ __forceinline__ void load_page(PageRegs<D> &r, const SlotView &sv, int b, int g, int pg, int lane_off,
                                          int32_t *dev_err) {
    constexpr int64_t kPair = 2 * kPage * D * 2;
    int64_t idx;
    if (PAGED) {
        int32_t blk = sv.table[(int64_t)b * sv.max_blocks + pg];
        if (blk < 0 || (int64_t)blk >= sv.num_blocks) {
            if (lane_off == 0) atomicOr(dev_err, LCKV_DEV_ERR_BLOCK);
            blk = 0;  // read something that exists; the result of this sequence is undefined, the error is raised
        }
        idx = (int64_t)blk * sv.Hkv + g;
    } else {
        idx = ((int64_t)b * sv.Hkv + g) * sv.pages_per_seq + pg;
    }
    const char *base = sv.base + idx * kPair + lane_off;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) r.k[ks] = load16<false>(base + ks * 1024);
#pragma unroll
    for (int dp = 0; dp < D / 32; ++dp) r.v[dp] = load16<false>(base + kPair / 2 + dp * 1024);
}

template <int D, int QB, bool PAGED>
__global__ __launch_bounds__(256) void prefill_bf16_kernel(AttnParams p, int S) {
    constexpr int kRows = 16 * QB;  // query positions per wave
    const int h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, kb = lane >> 4;  // query position within a block / key quad
    const int g = h / p.G;
    const int chunk = gridDim.x - 1 - blockIdx.x;  // rows with the most keys first
    const int i_lo = (chunk * 4 + wave) * kRows;
    if (i_lo >= S) return;

    int len = p.seq_lens[b];
    if (len > p.max_n) {
        len = p.max_n;
        if (lane == 0) atomicOr(p.dev_err, LCKV_DEV_ERR_CAPACITY);
    }
    if (len < 0) len = 0;
    uint16_t *out = (uint16_t *)p.out;
    const int self = p.self_visible;

    if (i_lo >= len) {  // none of this wave's rows belongs to the prompt: zero rows
        for (int r = 0; r < kRows && i_lo + r < S; ++r) {
            uint32_t *o = (uint32_t *)(out + (((int64_t)b * S + i_lo + r) * p.Hq + h) * D);
            for (int e = lane; e < D / 2; e += 64) o[e] = 0u;
        }
        return;
    }

    // Q^T operands and the number of keys each column sees
    bf16x8 qb[QB][D / 32];
    int n_col[QB];
#pragma unroll
    for (int x = 0; x < QB; ++x) {
        const int i = i_lo + 16 * x + c;
        n_col[x] = min(i + self, len);
        const char *qp = (const char *)p.q + ((((int64_t)b * S + i) * p.Hq + h) * D + kb * 8) * 2;
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (i < S) v = *(const u32x4 *)(qp + ks * 64);
            qb[x][ks] = __builtin_bit_cast(bf16x8, v);
        }
    }

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
    const int n_most = min(i_lo + kRows - 1 + self, len);  // keys seen by the last column of this wave
    const int n_pages = (n_most + kPage - 1) / kPage;

    auto consume = [&](PageRegs<D> &r, int pg) {
        if ((pg + 1) * kPage > len) {  // last, partly filled page of the prompt: clear stale values (0 * NaN)
            int nv = len - (pg * kPage + 4 * kb);
            uint32_t m01 = nv >= 2 ? 0xffffffffu : (nv == 1 ? 0x0000ffffu : 0u);
            uint32_t m23 = nv >= 4 ? 0xffffffffu : (nv == 3 ? 0x0000ffffu : 0u);
#pragma unroll
            for (int dp = 0; dp < D / 32; ++dp) {
                r.v[dp][0] &= m01;
                r.v[dp][1] &= m23;
                r.v[dp][2] &= m01;
                r.v[dp][3] &= m23;
            }
        }
#pragma unroll
        for (int x = 0; x < QB; ++x) {
            const int n_lo = min(i_lo + 16 * x + self, len);       // keys the first column of the block sees
            const int n_hi = min(i_lo + 16 * x + 15 + self, len);  // ... and the last
            if (pg * kPage >= n_hi) continue;                      // the whole page lies above the diagonal
            floatx4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < D / 32; ++ks)
                z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, r.k[ks]), qb[x][ks], z, 0, 0, 0);
            if ((pg + 1) * kPage > n_lo) {  // the diagonal crosses this page: mask per column
                const int key0 = pg * kPage + 4 * kb;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (key0 + e >= n_col[x]) z[e] = kNegInf;
            }
            float smax = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
            smax = column_max4(smax);
            const float m_new = fmaxf(m[x], smax);
            const float m_use = m_new == kNegInf ? 0.f : m_new;  // a column that has seen no key yet
            const float mb = m_use * cs;
            const float alpha = __builtin_amdgcn_exp2f((m[x] - m_use) * cs);
            const bool grew = __builtin_amdgcn_ballot_w64(m_new > m[x]) != 0;
            m[x] = m_new;
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(z[0], cs, -mb));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(z[1], cs, -mb));
            const float p2 = __builtin_amdgcn_exp2f(__builtin_fmaf(z[2], cs, -mb));
            const float p3 = __builtin_amdgcn_exp2f(__builtin_fmaf(z[3], cs, -mb));
            u32x2 pk = {pack_bf16(p0, p1), pack_bf16(p2, p3)};
            const shortx4 pb = __builtin_bit_cast(shortx4, pk);
            if (grew) {
                l[x] *= alpha;
#pragma unroll
                for (int j = 0; j < D / 16; ++j) acc[x][j] *= alpha;
            }
            l[x] += (p0 + p1) + (p2 + p3);
#pragma unroll
            for (int dp = 0; dp < D / 32; ++dp) {
                u32x2 lo = {r.v[dp][0], r.v[dp][1]};
                u32x2 hi = {r.v[dp][2], r.v[dp][3]};
                acc[x][2 * dp] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, lo), pb,
                                                                           acc[x][2 * dp], 0, 0, 0);
                acc[x][2 * dp + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, hi), pb,
                                                                               acc[x][2 * dp + 1], 0, 0, 0);
            }
        }
    };

    // pages 0 .. n_pages-1 in order, the next page's loads in flight while the current one is used
    if (n_pages > 0) {
        PageRegs<D> ra, rb;
        int pg = 0;
        load_page<D, PAGED>(ra, p.slot, b, g, 0, lane_off, p.dev_err);
        for (;;) {
            if (pg + 1 < n_pages) {
                load_page<D, PAGED>(rb, p.slot, b, g, pg + 1, lane_off, p.dev_err);
                consume(ra, pg);
            } else {
                consume(ra, pg);
                break;
            }
            ++pg;
            if (pg + 1 < n_pages) {
                load_page<D, PAGED>(ra, p.slot, b, g, pg + 1, lane_off, p.dev_err);
                consume(rb, pg);
            } else {
                consume(rb, pg);
                break;
            }
            ++pg;
        }
    }

#pragma unroll
    for (int x = 0; x < QB; ++x) {
        float L = l[x];
        L = column_sum4(L);
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

template <int D, int QB>
hipError_t launch_qb(const AttnParams &p, int S, hipStream_t s) {
    const int rows_per_group = 4 * 16 * QB;
    dim3 grid((S + rows_per_group - 1) / rows_per_group, p.Hq, p.B), block(256);
    if (p.slot.table)
        hipLaunchKernelGGL((prefill_bf16_kernel<D, QB, true>), grid, block, 0, s, p, S);
    else
        hipLaunchKernelGGL((prefill_bf16_kernel<D, QB, false>), grid, block, 0, s, p, S);
    return hipGetLastError();
}

}  // namespace

// p: seq_lens = prompt lengths, max_n = min(S, capacity), self_visible, scale; no splits.
hipError_t launch_prefill_bf16(const AttnParams &p, int S, int D, int qb, hipStream_t s) {
    if (qb == 0) qb = D == 128 ? 2 : 4;  // what fits the register file without spilling
    if (D == 128) return qb == 2 ? launch_qb<128, 2>(p, S, s) : launch_qb<128, 4>(p, S, s);
    return qb == 2 ? launch_qb<64, 2>(p, S, s) : launch_qb<64, 4>(p, S, s);
}

}  // namespace lckv
