// Split-KV decode attention for fp32 caches (Section 2.1 of the LCKV paper), plain vector ALU, no matrix cores:
// the parity mode in which every product and sum is an fp32 FMA.
//
// One workgroup (4 waves) handles one (split, QUERY head, sequence).  A wave reads four keys at a time: the 16
// lanes of a row hold one key's D channels (float4 loads, a 256- or 512-byte row per 16 lanes), the dot
// product is finished with four DPP adds inside the row, and each row keeps its own running (max, sum, O) for
// the keys it sees - 16 independent online-softmax states per workgroup, merged through LDS at the end.
#include "lckv_internal.h"

namespace lckv {

namespace {

constexpr int kWaves = 4;
constexpr float kNegInf = -__builtin_huge_valf();

// x + (x from another lane of the same 16-lane row); ctrl: quad_perm / row_half_mirror / row_mirror
template <int kCtrl>
__device__ __forceinline__ float dpp_add(float x) {
    int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), kCtrl, 0xf, 0xf, true);
    return x + __builtin_bit_cast(float, y);
}
// sum over the 16 lanes of a row, result in every lane of the row
__device__ __forceinline__ float row_sum16(float x) {
    x = dpp_add<0xB1>(x);   // quad_perm [1,0,3,2]: lane ^ 1
    x = dpp_add<0x4E>(x);   // quad_perm [2,3,0,1]: lane ^ 2
    x = dpp_add<0x141>(x);  // row_half_mirror: quads 0<->1, 2<->3 (quad-uniform values)
    x = dpp_add<0x140>(x);  // row_mirror: halves 0<->1 (half-uniform values)
    return x;
}

// One workgroup's work: query row `row` of p.q / p.out (head h, reading kv head h / G of sequence b) over the keys
// [split * split_tokens, ...) of its n visible keys.
template <int D>
__device__ __forceinline__ void attend_row_f32(const AttnParams &p, int split, int h, int b, int n, int64_t row) {
    constexpr int NV = D / 64;  // float4 per lane per row
    const int g = h / p.G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kq = lane >> 4, r = lane & 15;  // which of the wave's 4 keys / 16-byte column of the row
    const int k_begin = split * p.split_tokens;
    const int k_end = min(n, k_begin + p.split_tokens);
    float *out = (float *)p.out + row * D;

    if (k_begin >= k_end) {
        if (p.n_splits == 1) {
            for (int i = tid; i < D; i += kWaves * 64) out[i] = 0.f;  // zero dummy K/V of the first token
        } else if (tid == 0) {
            p.part_ml[((int64_t)split * p.B + b) * p.Hq + h] = float2{kNegInf, 0.f};
        }
        return;
    }

    float4 qv[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) qv[i] = *(const float4 *)((const float *)p.q + row * D + i * 64 + r * 4);

    float4 acc[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) acc[i] = float4{0.f, 0.f, 0.f, 0.f};
    float m = kNegInf, l = 0.f;  // log2 units
    const float cs = p.scale_log2e;

    int cur_page = -1;
    const char *page_ptr = nullptr;
    for (int j = k_begin + wave * 4 + kq; j < k_end; j += kWaves * 4) {
        int pg = j / kPage;
        if (pg != cur_page) {
            cur_page = pg;
            int64_t idx = page_pair_index(p.slot, b, g, pg);
            page_ptr = idx >= 0 ? p.slot.base + idx * (2 * (int64_t)p.slot.page_bytes) : nullptr;
            if (idx < 0 && r == 0) atomicOr(p.dev_err, LCKV_DEV_ERR_BLOCK);
        }
        if (!page_ptr) continue;  // row-uniform
        const float *kp = (const float *)page_ptr + (j % kPage) * D + r * 4;
        const float *vp = (const float *)(page_ptr + p.slot.page_bytes) + (j % kPage) * D + r * 4;
        float4 kv[NV], vv[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            kv[i] = *(const float4 *)(kp + i * 64);
            vv[i] = *(const float4 *)(vp + i * 64);
        }
        float dot = 0.f;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            dot = __builtin_fmaf(qv[i].x, kv[i].x, dot);
            dot = __builtin_fmaf(qv[i].y, kv[i].y, dot);
            dot = __builtin_fmaf(qv[i].z, kv[i].z, dot);
            dot = __builtin_fmaf(qv[i].w, kv[i].w, dot);
        }
        // Rows whose j is past k_end have left the loop: their lanes are inactive, and row_sum16 only mixes
        // lanes of one row, so the active rows are complete.
        float s = row_sum16(dot) * cs;
        float m_new = fmaxf(m, s);
        float alpha = exp2f(m - m_new);  // m = -inf on the first key: 0
        float pj = exp2f(s - m_new);
        m = m_new;
        l = l * alpha + pj;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            acc[i].x = __builtin_fmaf(pj, vv[i].x, acc[i].x * alpha);
            acc[i].y = __builtin_fmaf(pj, vv[i].y, acc[i].y * alpha);
            acc[i].z = __builtin_fmaf(pj, vv[i].z, acc[i].z * alpha);
            acc[i].w = __builtin_fmaf(pj, vv[i].w, acc[i].w * alpha);
        }
    }

    // merge the 16 row states
    __shared__ float sm_m[kWaves * 4], sm_l[kWaves * 4];
    __shared__ float sm_acc[kWaves * 4][D];
    const int st = wave * 4 + kq;
    if (r == 0) {
        sm_m[st] = m;
        sm_l[st] = l;
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) *(float4 *)&sm_acc[st][i * 64 + r * 4] = acc[i];
    __syncthreads();
    if (tid < D) {
        float M = kNegInf;
        for (int i = 0; i < kWaves * 4; ++i) M = fmaxf(M, sm_m[i]);
        float L = 0.f, o = 0.f;
        for (int i = 0; i < kWaves * 4; ++i) {
            if (sm_m[i] == kNegInf) continue;
            float f = exp2f(sm_m[i] - M);
            L += f * sm_l[i];
            o += f * sm_acc[i][tid];
        }
        if (p.n_splits == 1) {
            out[tid] = L > 0.f ? o / L : 0.f;
        } else {
            p.part_o[(((int64_t)split * p.B + b) * p.Hq + h) * D + tid] = o;
            if (tid == 0) p.part_ml[((int64_t)split * p.B + b) * p.Hq + h] = float2{M, L};
        }
    }
}

// Decode: one query token per sequence.
template <int D>
__global__ __launch_bounds__(kWaves * 64) void attn_f32_kernel(AttnParams p) {
    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    int n = p.seq_lens[b] + p.self_visible;
    if (n > p.max_n) {
        n = p.max_n;
        if (threadIdx.x == 0 && !p.clamp_is_policy) atomicOr(p.dev_err, LCKV_DEV_ERR_CAPACITY);
    }
    if (n < 0) n = 0;
    attend_row_f32<D>(p, split, h, b, n, (int64_t)b * p.Hq + h);
}

// Prefill (all prompt tokens of a layer at once, Sections 2.2 and 2.3 of the LCKV paper): one workgroup per
// (token i, head, sequence); token i sees i keys, or i + 1 in a warmup layer; rows past the prompt are zero.
template <int D>
__global__ __launch_bounds__(kWaves * 64) void prefill_f32_kernel(AttnParams p, int S) {
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    int len = p.seq_lens[b];
    if (len > p.max_n) {
        len = p.max_n;
        if (threadIdx.x == 0) atomicOr(p.dev_err, LCKV_DEV_ERR_CAPACITY);
    }
    const int n = i < len ? i + p.self_visible : 0;  // n = 0 writes the zero vector
    attend_row_f32<D>(p, 0, h, b, n, ((int64_t)b * S + i) * p.Hq + h);
}

}  // namespace

hipError_t launch_attn_f32(const AttnParams &p, int D, hipStream_t s) {
    dim3 grid(p.n_splits, p.Hq, p.B), block(kWaves * 64);
    if (D == 128)
        hipLaunchKernelGGL((attn_f32_kernel<128>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((attn_f32_kernel<64>), grid, block, 0, s, p);
    return hipGetLastError();
}

// p: n_splits = 1, split_tokens >= S, max_n = min(S, capacity), seq_lens = prompt lengths.
hipError_t launch_prefill_f32(const AttnParams &p, int S, int D, hipStream_t s) {
    dim3 grid(S, p.Hq, p.B), block(kWaves * 64);
    if (D == 128)
        hipLaunchKernelGGL((prefill_f32_kernel<128>), grid, block, 0, s, p, S);
    else
        hipLaunchKernelGGL((prefill_f32_kernel<64>), grid, block, 0, s, p, S);
    return hipGetLastError();
}

}  // namespace lckv
