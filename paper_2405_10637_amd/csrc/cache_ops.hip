// Cache maintenance kernels of liblckv: append of the new token's K/V, bulk import, logical read-back, the
// length bump that ends a decode step, and the merge of split partials.  All of them move bits or do the
// final fp32 normalisation; none of them is on the bandwidth-critical path.
#include "lckv_internal.h"

namespace lckv {

namespace {

// K[slot][b][t_b] = k_new[b], V likewise (Section 2.1: the K/V of a producing layer are cached for later
// tokens).  One thread per (b, kv head, channel); E is the element's bit pattern type.
template <typename E>
__global__ void append_kernel(SlotView sv, const E *k_new, const E *v_new, const int32_t *seq_lens, int B, int D,
                              int32_t *dev_err) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (int64_t)B * sv.Hkv * D) append_element<E>(sv, k_new, v_new, seq_lens, D, dev_err, i);
}

// Dense [B][T][Hkv][D] -> cache, positions [0, min(T, lens[b])), any element type (used for fp32 caches, the
// parity mode).  One thread per 16-byte chunk of the dense tensors, grid-stride (a launch may not exceed 2^32 threads, and the big caches hold more elements than that).
template <typename E>
__global__ void load_dense_kernel(SlotView sv, const E *k, const E *v, const int32_t *lens, int B, int T, int D,
                                  int32_t *dev_err) {
    constexpr int C = 16 / (int)sizeof(E);  // elements per chunk
    const int chunks = D / C;
    const int64_t total = (int64_t)B * T * sv.Hkv * chunks;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        int dc = (int)(i % chunks);
        int g = (int)((i / chunks) % sv.Hkv);
        int t = (int)((i / ((int64_t)chunks * sv.Hkv)) % T);
        int b = (int)(i / ((int64_t)chunks * sv.Hkv * T));
        if (lens && t >= lens[b]) continue;
        int64_t idx = page_pair_index(sv, b, g, t / kPage);
        if (idx < 0) {
            if (dc == 0) atomicOr(dev_err, LCKV_DEV_ERR_BLOCK);
            continue;
        }
        E *kpage = (E *)(sv.base + idx * (2 * (int64_t)sv.page_bytes));
        E *vpage = (E *)((char *)kpage + sv.page_bytes);
        int j = t % kPage;
        const E *ks = k + i * C, *vs = v + i * C;
#pragma unroll
        for (int e = 0; e < C; ++e) {
            kpage[k_off<E>(j, dc * C + e, D)] = ks[e];
            vpage[v_off<E>(j, dc * C + e, D)] = vs[e];
        }
    }
}

// The same import for bf16 caches at speed (it is on the path of the prompt encoding of Section 2.3: each of
// its iterations stores a producing layer's K/V of all prompt tokens before the next iteration reads them).
// One wave per (sequence, page, kv head): it reads the 16 rows of the page from the dense tensors with 16 bytes
// per lane (a row of D channels is contiguous), and writes the K page and the V page in matrix-operand order.
// K: the operand order only permutes 16-byte chunks (8 channels of one position), so the loaded registers are
// stored as they are, each at its chunk's place.  V: four consecutive positions of one channel are contiguous
// there, a transposition of single elements, done through a wave-private LDS image of the 16 x D tile; the page is
// then written with lane-linear 16-byte stores, a contiguous KiB per instruction like every read of it later.
// Positions at or beyond min(T, t_b) are not written (partly filled last page: masked stores).
template <int D>
__global__ __launch_bounds__(256) void load_dense_bf16_kernel(SlotView sv, const uint16_t *k, const uint16_t *v,
                                                              const int32_t *lens, int B, int T, int32_t *dev_err) {
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    constexpr int kChunks = D / 8;              // 16-byte chunks per row
    constexpr int kRowsPerLoad = 64 / kChunks;  // rows one wave-wide load covers: 4 (D = 128) or 8 (D = 64)
    constexpr int kLoads = kPage / kRowsPerLoad;
    constexpr int kStride = D * 2 + 16;         // LDS row stride in bytes: rows 4 apart fall on different banks
    constexpr int kStores = kPage * D * 2 / 1024;  // KiB of a page = lane-linear stores per page
    __shared__ __attribute__((aligned(16))) char lds[4][kPage * kStride];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane % kChunks, pq = lane / kChunks;  // chunk within the row / row within the load
    const int n_pages = (T + kPage - 1) / kPage;
    const int head_groups = (sv.Hkv + 3) / 4;
    const int64_t total = (int64_t)B * n_pages * head_groups;
    for (int64_t task = blockIdx.x; task < total; task += gridDim.x) {  // uniform over the workgroup
        const int hg = (int)(task % head_groups);
        const int page = (int)((task / head_groups) % n_pages);
        const int b = (int)(task / ((int64_t)head_groups * n_pages));
        const int g = hg * 4 + wave;
        int limit = T;
        if (lens) limit = min(limit, lens[b]);
        const int n_valid = min(kPage, limit - page * kPage);  // rows of this page to write (may be <= 0)
        const bool work = g < sv.Hkv && n_valid > 0;            // wave-uniform
        int64_t idx = -1;
        if (work) {
            idx = page_pair_index(sv, b, g, page);
            if (idx < 0 && lane == 0) atomicOr(dev_err, LCKV_DEV_ERR_BLOCK);
        }
        const bool go = work && idx >= 0;
        char *kpage = sv.base + (go ? idx : 0) * (2 * (int64_t)sv.page_bytes);
        char *vpage = kpage + sv.page_bytes;
        char *tile = lds[wave];
        if (go) {
            u32x4 kr[kLoads], vr[kLoads];
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
                const int j = i * kRowsPerLoad + pq;
                const int t = min(page * kPage + j, T - 1);  // rows past the end: re-read the last one, not stored
                const int64_t at = (((int64_t)b * T + t) * sv.Hkv + g) * D + c * 8;
                kr[i] = __builtin_nontemporal_load((const u32x4 *)(k + at));
                vr[i] = __builtin_nontemporal_load((const u32x4 *)(v + at));
            }
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
                const int j = i * kRowsPerLoad + pq;
                // K page [D/32][4 octets][16 positions][8 channels]: chunk c of position j at 16 * (16 c + j)
                if (j < n_valid) *(u32x4 *)(kpage + (c * kPage + j) * 16) = kr[i];
                *(u32x4 *)(tile + j * kStride + c * 16) = vr[i];
            }
        }
        __syncthreads();
        if (go) {
            // V page [D/32 dp][4 quads kb][16 channels r][2 channel blocks][4 positions]: lane (kb, r) of store dp
            // writes channels 32 dp + r and 32 dp + 16 + r of positions 4 kb .. 4 kb + 3
            const int kb = lane >> 4, r = lane & 15;
#pragma unroll
            for (int dp = 0; dp < kStores; ++dp) {
                uint16_t e[8];
#pragma unroll
                for (int kq = 0; kq < 4; ++kq) {
                    const char *row = tile + (4 * kb + kq) * kStride;
                    e[kq] = *(const uint16_t *)(row + (32 * dp + r) * 2);
                    e[4 + kq] = *(const uint16_t *)(row + (32 * dp + 16 + r) * 2);
                }
                char *dst = vpage + dp * 1024 + lane * 16;
                if (4 * kb + 3 < n_valid) {
                    u32x4 o = {(uint32_t)e[0] | ((uint32_t)e[1] << 16), (uint32_t)e[2] | ((uint32_t)e[3] << 16),
                               (uint32_t)e[4] | ((uint32_t)e[5] << 16), (uint32_t)e[6] | ((uint32_t)e[7] << 16)};
                    *(u32x4 *)dst = o;
                } else {
#pragma unroll
                    for (int kq = 0; kq < 4; ++kq)
                        if (4 * kb + kq < n_valid) {
                            ((uint16_t *)dst)[kq] = e[kq];
                            ((uint16_t *)dst)[4 + kq] = e[4 + kq];
                        }
                }
            }
        }
        __syncthreads();
    }
}

// cache -> dense [n_pos][Hkv][D] for one sequence
template <typename E>
__global__ void gather_kernel(SlotView sv, int b, int pos, int n_pos, int D, E *out_k, E *out_v, int32_t *dev_err) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)n_pos * sv.Hkv * D;
    if (i >= total) return;
    int d = (int)(i % D);
    int g = (int)((i / D) % sv.Hkv);
    int t = entry_of_position(sv, pos + (int)(i / ((int64_t)D * sv.Hkv)));
    int64_t idx = page_pair_index(sv, b, g, t / kPage);
    if (idx < 0) {
        if (d == 0) atomicOr(dev_err, LCKV_DEV_ERR_BLOCK);
        out_k[i] = 0;
        out_v[i] = 0;
        return;
    }
    const E *kpage = (const E *)(sv.base + idx * (2 * (int64_t)sv.page_bytes));
    const E *vpage = (const E *)((const char *)kpage + sv.page_bytes);
    int j = t % kPage;
    out_k[i] = kpage[k_off<E>(j, d, D)];
    out_v[i] = vpage[v_off<E>(j, d, D)];
}

__global__ void bump_kernel(int32_t *seq_lens, int B) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B) seq_lens[i] += 1;
}

// Merge of split partials, one thread per output element.
template <typename O>
__global__ void combine_kernel(const float *part_o, const float2 *part_ml, O *out, int64_t rows, int D, int S) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows * D) combine_element<O>(part_o, part_ml, out, rows, D, S, i);
}

inline unsigned blocks_for(int64_t n, int bs) { return (unsigned)((n + bs - 1) / bs); }

}  // namespace

hipError_t launch_append(const SlotView &v, const void *k_new, const void *v_new, const int32_t *seq_lens, int B,
                         int D, int dtype, int32_t *dev_err, hipStream_t s) {
    int64_t total = (int64_t)B * v.Hkv * D;
    if (dtype == LCKV_BF16)
        hipLaunchKernelGGL(append_kernel<uint16_t>, dim3(blocks_for(total, 256)), dim3(256), 0, s, v,
                           (const uint16_t *)k_new, (const uint16_t *)v_new, seq_lens, B, D, dev_err);
    else
        hipLaunchKernelGGL(append_kernel<uint32_t>, dim3(blocks_for(total, 256)), dim3(256), 0, s, v,
                           (const uint32_t *)k_new, (const uint32_t *)v_new, seq_lens, B, D, dev_err);
    return hipGetLastError();
}

hipError_t launch_bump(int32_t *seq_lens, int B, hipStream_t s) {
    hipLaunchKernelGGL(bump_kernel, dim3(blocks_for(B, 256)), dim3(256), 0, s, seq_lens, B);
    return hipGetLastError();
}

hipError_t launch_load_dense(const SlotView &v, const void *k, const void *vv, const int32_t *lens, int B, int T,
                             int D, int dtype, int32_t *dev_err, hipStream_t s) {
    int64_t total = (int64_t)B * T * v.Hkv * (D * (dtype == LCKV_BF16 ? 2 : 4) / 16);
    if (total == 0) return hipSuccess;
    if (dtype == LCKV_BF16) {
        int64_t tasks = (int64_t)B * ((T + kPage - 1) / kPage) * ((v.Hkv + 3) / 4);
        unsigned grid = (unsigned)(tasks < (1 << 24) ? tasks : (1 << 24));
        if (D == 128)
            hipLaunchKernelGGL(load_dense_bf16_kernel<128>, dim3(grid), dim3(256), 0, s, v, (const uint16_t *)k,
                               (const uint16_t *)vv, lens, B, T, dev_err);
        else
            hipLaunchKernelGGL(load_dense_bf16_kernel<64>, dim3(grid), dim3(256), 0, s, v, (const uint16_t *)k,
                               (const uint16_t *)vv, lens, B, T, dev_err);
        return hipGetLastError();
    }
    int64_t nb = (total + 255) / 256;
    if (nb > (1 << 22)) nb = 1 << 22;  // grid-stride beyond this
    hipLaunchKernelGGL(load_dense_kernel<uint32_t>, dim3((unsigned)nb), dim3(256), 0, s, v,
                           (const uint32_t *)k, (const uint32_t *)vv, lens, B, T, D, dev_err);
    return hipGetLastError();
}

hipError_t launch_gather(const SlotView &v, int b, int pos, int n_pos, int D, int dtype, void *dev_k, void *dev_v,
                         int32_t *dev_err, hipStream_t s) {
    int64_t total = (int64_t)n_pos * v.Hkv * D;
    if (dtype == LCKV_BF16)
        hipLaunchKernelGGL(gather_kernel<uint16_t>, dim3(blocks_for(total, 256)), dim3(256), 0, s, v, b, pos, n_pos,
                           D, (uint16_t *)dev_k, (uint16_t *)dev_v, dev_err);
    else
        hipLaunchKernelGGL(gather_kernel<uint32_t>, dim3(blocks_for(total, 256)), dim3(256), 0, s, v, b, pos, n_pos,
                           D, (uint32_t *)dev_k, (uint32_t *)dev_v, dev_err);
    return hipGetLastError();
}

hipError_t launch_combine(const AttnParams &p, int D, int dtype, hipStream_t s) {
    int64_t rows = (int64_t)p.B * p.Hq;
    if (dtype == LCKV_BF16)
        hipLaunchKernelGGL(combine_kernel<uint16_t>, dim3(blocks_for(rows * D, 256)), dim3(256), 0, s, p.part_o,
                           p.part_ml, (uint16_t *)p.out, rows, D, p.n_splits);
    else
        hipLaunchKernelGGL(combine_kernel<float>, dim3(blocks_for(rows * D, 256)), dim3(256), 0, s, p.part_o,
                           p.part_ml, (float *)p.out, rows, D, p.n_splits);
    return hipGetLastError();
}

}  // namespace lckv
