// Cache maintenance kernels of liblckv: append of the new token's K/V, bulk import, logical read-back, the
// length bump that ends a decode step, and the merge of split partials.  All of them move bits or do the
// final fp32 normalisation; none of them is on the bandwidth-critical path.
#include "lckv_internal.h"

namespace lckv {

namespace {

constexpr float kNegInf = -__builtin_huge_valf();
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float floatx2;

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

// K[slot][b][t_b] = k_new[b], V likewise (Section 2.1: the K/V of a producing layer are cached for later
// tokens).  One thread per (b, kv head, channel); E is the element's bit pattern type.
template <typename E>
__global__ void append_kernel(SlotView sv, const E *k_new, const E *v_new, const int32_t *seq_lens, int B, int D,
                              int32_t *dev_err) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)B * sv.Hkv * D;
    if (i >= total) return;
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

// Dense [B][T][Hkv][D] -> cache, positions [0, min(T, lens[b])).  One thread per 16-byte chunk of the dense
// tensors, grid-stride (a launch may not exceed 2^32 threads, and the big caches hold more elements than that).
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

__device__ __forceinline__ void store_out(float *o, float v) { *o = v; }
__device__ __forceinline__ void store_out(uint16_t *o, float v) {
    floatx2 f = {v, 0.f};
    bf16x2 h = __builtin_convertvector(f, bf16x2);  // round to nearest even
    *o = (uint16_t)(__builtin_bit_cast(uint32_t, h) & 0xffffu);
}

// Merge of split partials: with (m_i, l_i, o_i) the running maximum (log2 units), denominator and
// unnormalised output of split i,  out = sum_i 2^(m_i - M) o_i / sum_i 2^(m_i - M) l_i,  M = max_i m_i.
// Splits without a visible key carry m_i = -inf and are skipped; no visible key at all gives zero.
template <typename O>
__global__ void combine_kernel(const float *part_o, const float2 *part_ml, O *out, int64_t rows, int D, int S) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * D) return;
    int64_t row = i / D;
    int d = (int)(i % D);
    float M = kNegInf;
    for (int s = 0; s < S; ++s) M = fmaxf(M, part_ml[(int64_t)s * rows + row].x);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < S; ++s) {
        float2 ml = part_ml[(int64_t)s * rows + row];
        if (ml.x == kNegInf) continue;
        float f = exp2f(ml.x - M);
        den += f * ml.y;
        num += f * part_o[((int64_t)s * rows + row) * D + d];
    }
    store_out(out + i, den > 0.f ? num / den : 0.f);
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
    int64_t nb = (total + 255) / 256;
    if (nb > (1 << 22)) nb = 1 << 22;  // grid-stride beyond this
    if (dtype == LCKV_BF16)
        hipLaunchKernelGGL(load_dense_kernel<uint16_t>, dim3((unsigned)nb), dim3(256), 0, s, v,
                           (const uint16_t *)k, (const uint16_t *)vv, lens, B, T, D, dev_err);
    else
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
