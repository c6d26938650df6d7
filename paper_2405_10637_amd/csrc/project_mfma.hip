// The projections either side of the attention, for one decode step of one layer (Section 2.1 of the LCKV paper:
// every layer maps the hidden state to queries; only a layer that PRODUCES a cache slot - a warmup layer, or the one
// condensed layer that owns the shared cache - maps it to keys and values, the others have no W_K, W_V at all):
//   y[b][n] = sum_c x[b][c] * W[n][c]        W = W_Q (and W_K, W_V stacked below it for a producing layer)
// then the rotary position embedding on queries and keys at position t_b (Llama convention: channel i < D/2 of a
// head is paired with channel i + D/2, angle t_b * base^(-2i/D)), the queries written to q_out, the keys and
// values stored straight into the slot at position t_b (the append of the decode step, fused).
//
// Three launches on the caller's stream:
//   1. prepare: clear the fp32 accumulator [B][N] in the workspace, tabulate cos/sin [B][D/2] (angles in double)
//   2. the matrix product, split over the hidden dimension, partial sums added with fp32 atomics
//   3. finish: rotate, round once, scatter into q_out / the cache pages
// The product streams each weight once from HBM (what bounds it: 2 * N * hidden bytes against 4 * B flops per
// weight) and is shaped for that.  A workgroup of 4 waves owns 128 output features x 256 hidden channels x up to
// 128 sequences: its x slice (64 KiB) is staged once in LDS in matrix-operand order and shared by the waves,
// each wave owns two 16-feature tiles whose weights it loads straight into registers (all 16 loads of 1 KiB
// issued before anything else, so 32 KiB per workgroup are in flight), and every LDS read of an x operand feeds
// two matrix instructions.  Features on the rows of the tiles (A operand = weights, rows of W are contiguous in
// memory), sequences on the columns.  The order of the contraction index inside a slice is permuted, the same way
// for both operands, so that each lane's eight 16-byte weight loads are 128 contiguous bytes.
#include "bf16_mfma_common.h"

namespace lckv {

namespace {

constexpr int kSliceC = 256;    // hidden channels per workgroup
constexpr int kSteps = 8;       // matrix instructions (32 channels each) per slice
constexpr int kTileRows = 128;  // output features per workgroup (8 tiles of 16, two per wave)

struct ProjParams {
    const void *x;              // [B][hidden]
    const void *w[3];           // W_Q [n_rows[0]][hidden], W_K, W_V (null: absent)
    int32_t n_rows[3];
    int32_t n_total;            // rows of the stacked matrix
    int32_t hidden, B;
    float *acc;                 // [B][n_total] fp32
    float2 *rope;               // [B][D/2] (cos, sin)
    const int32_t *seq_lens;
    void *q_out;                // [B][Hq][D]
    SlotView slot;              // where K/V go (producing layers)
    int32_t Hq, Hkv, D;
    double log2_base;           // log2(rope base); rotate = 0: no rotation
    int32_t rotate;
    int32_t *dev_err;
};

// Launch 1.
__global__ void project_prepare_kernel(ProjParams p) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t n_acc = (int64_t)p.B * p.n_total;
    if (i < n_acc) p.acc[i] = 0.f;
    const int half = p.D / 2;
    if (i < (int64_t)p.B * half) {
        const int b = (int)(i / half), k = (int)(i % half);
        float2 cs = {1.f, 0.f};
        if (p.rotate) {
            int t = p.seq_lens[b];
            if (t < 0) t = 0;
            const double angle = (double)t * exp2(-2.0 * k / p.D * p.log2_base);
            cs = float2{(float)cos(angle), (float)sin(angle)};
        }
        p.rope[i] = cs;
    }
}

// Row n of the stacked matrix -> pointer to that row's first element (rows never straddle: n_rows are multiples
// of 16 and a tile is 16 rows).
template <typename E>
__device__ __forceinline__ const E *stacked_row(const ProjParams &p, int n) {
    int m = 0;
    if (n >= p.n_rows[0]) {
        n -= p.n_rows[0];
        m = 1;
        if (n >= p.n_rows[1]) {
            n -= p.n_rows[1];
            m = 2;
        }
    }
    return (const E *)p.w[m] + (int64_t)n * p.hidden;
}

// Launch 2, bf16.  NB = 16-sequence blocks per pass (1, 2, 4 or 8).  grid (feature blocks, hidden slices,
// passes of 16 * NB sequences).
template <int NB>
__global__ __launch_bounds__(256, 2) void project_bf16_kernel(ProjParams p) {
    __shared__ __attribute__((aligned(16))) char lds[NB * kSteps * 1024];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, kb = lane >> 4;
    const int c0 = blockIdx.y * kSliceC;
    const int b0 = blockIdx.z * (16 * NB);

    // this wave's weights: two tiles x 8 steps, lane (kb, r) takes channels c0 + (kb*8 + s)*8 .. +7 of row r
    u32x4 wr[2][kSteps];
    bool have[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int n0 = blockIdx.x * kTileRows + (wave * 2 + nt) * 16;
        have[nt] = n0 < p.n_total;  // wave-uniform
        if (have[nt]) {
            const char *row = (const char *)(stacked_row<uint16_t>(p, n0 + r) + c0 + kb * 64);
#pragma unroll
            for (int s = 0; s < kSteps; ++s) wr[nt][s] = __builtin_nontemporal_load((const u32x4 *)(row + s * 16));
        } else {
#pragma unroll
            for (int s = 0; s < kSteps; ++s) wr[nt][s] = u32x4{0u, 0u, 0u, 0u};
        }
    }

    // the x slice into LDS, operand order: [sequence block][step s][lane (kb, b % 16)][8 channels]
    for (int i = tid; i < NB * 16 * 32; i += 256) {
        const int b = i >> 5, c8 = i & 31;  // 16-byte chunk c8 of row b: channels c0 + 8*c8 = c0 + (kb*8 + s)*8
        u32x4 v = {0u, 0u, 0u, 0u};
        if (b0 + b < p.B) v = *(const u32x4 *)((const uint16_t *)p.x + (int64_t)(b0 + b) * p.hidden + c0 + c8 * 8);
        const int ckb = c8 >> 3, s = c8 & 7;
        *(u32x4 *)(lds + ((((b >> 4) * kSteps + s) * 64) + ckb * 16 + (b & 15)) * 16) = v;
    }
    __syncthreads();

    floatx4 acc[2][NB];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[nt][j] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < kSteps; ++s)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const bf16x8 xb = __builtin_bit_cast(bf16x8, *(const u32x4 *)(lds + ((j * kSteps + s) * 64 + lane) * 16));
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                acc[nt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wr[nt][s]), xb,
                                                                     acc[nt][j], 0, 0, 0);
        }

    // lane (kb, c) holds features n0 + 4kb .. +3 of sequence b0 + 16j + c
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        if (!have[nt]) continue;
        const int n0 = blockIdx.x * kTileRows + (wave * 2 + nt) * 16;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int b = b0 + 16 * j + r;
            if (b >= p.B) continue;
            float *dst = p.acc + (int64_t)b * p.n_total + n0 + 4 * kb;
#pragma unroll
            for (int e = 0; e < 4; ++e) unsafeAtomicAdd(dst + e, acc[nt][j][e]);
        }
    }
}

// Launch 2, fp32 (parity mode, not tuned): one thread per output, products accumulated in double.
__global__ void project_f32_kernel(ProjParams p) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)p.B * p.n_total) return;
    const int b = (int)(i / p.n_total), n = (int)(i % p.n_total);
    const float *w = stacked_row<float>(p, n);
    const float *x = (const float *)p.x + (int64_t)b * p.hidden;
    double s = 0.0;
    for (int c = 0; c < p.hidden; ++c) s += (double)x[c] * (double)w[c];
    p.acc[i] = (float)s;
}

__device__ __forceinline__ uint16_t to_elem(float v, uint16_t) { return (uint16_t)(pack_bf16(v, 0.f) & 0xffffu); }
__device__ __forceinline__ uint32_t to_elem(float v, uint32_t) { return __builtin_bit_cast(uint32_t, v); }

// Launch 3.  One thread per (sequence, head of the stacked output, channel pair i < D/2).
template <typename E>
__global__ void project_finish_kernel(ProjParams p) {
    const int half = p.D / 2;
    const int heads = p.n_total / p.D;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)p.B * heads * half) return;
    const int i = (int)(idx % half);
    const int hg = (int)((idx / half) % heads);
    const int b = (int)(idx / ((int64_t)half * heads));
    const float *y = p.acc + (int64_t)b * p.n_total + (int64_t)hg * p.D;
    float lo = y[i], hi = y[i + half];
    const bool is_v = hg >= p.Hq + p.Hkv;
    if (!is_v) {
        const float2 cs = p.rope[(int64_t)b * half + i];
        const float rl = lo * cs.x - hi * cs.y, rh = hi * cs.x + lo * cs.y;
        lo = rl;
        hi = rh;
    }
    if (hg < p.Hq) {
        E *q = (E *)p.q_out + ((int64_t)b * p.Hq + hg) * p.D;
        q[i] = to_elem(lo, E{});
        q[i + half] = to_elem(hi, E{});
        return;
    }
    // a key or value head: into the slot at position t_b (the ring entry under the sink + window policy)
    const int g = is_v ? hg - p.Hq - p.Hkv : hg - p.Hq;
    int t = p.seq_lens[b];
    if (t >= 0) t = entry_of_position(p.slot, t);
    if (t < 0 || t >= p.slot.capacity) {
        if (i == 0) atomicOr(p.dev_err, LCKV_DEV_ERR_CAPACITY);
        return;
    }
    const int64_t pp = page_pair_index(p.slot, b, g, t / kPage);
    if (pp < 0) {
        if (i == 0) atomicOr(p.dev_err, LCKV_DEV_ERR_BLOCK);
        return;
    }
    E *page = (E *)(p.slot.base + pp * (2 * (int64_t)p.slot.page_bytes) + (is_v ? p.slot.page_bytes : 0));
    const int j = t % kPage;
    if (sizeof(E) == 2) {
        page[is_v ? v_elem_offset_bf16(j, i) : k_elem_offset_bf16(j, i)] = to_elem(lo, E{});
        page[is_v ? v_elem_offset_bf16(j, i + half) : k_elem_offset_bf16(j, i + half)] = to_elem(hi, E{});
    } else {
        page[kv_elem_offset_f32(j, i, p.D)] = to_elem(lo, E{});
        page[kv_elem_offset_f32(j, i + half, p.D)] = to_elem(hi, E{});
    }
}

}  // namespace

// x [B][hidden]; w_k / w_v null for a layer that produces no slot (then `slot` is not used).
hipError_t launch_project(const void *x, int hidden, const void *w_q, const void *w_k, const void *w_v, void *q_out,
                          const SlotView &slot, const int32_t *seq_lens, int B, int Hq, int Hkv, int D, int dtype,
                          float rope_base, float *acc, float2 *rope, int32_t *dev_err, hipStream_t s) {
    ProjParams p{};
    p.x = x;
    p.w[0] = w_q;
    p.w[1] = w_k;
    p.w[2] = w_v;
    p.n_rows[0] = Hq * D;
    p.n_rows[1] = w_k ? Hkv * D : 0;
    p.n_rows[2] = w_v ? Hkv * D : 0;
    p.n_total = p.n_rows[0] + p.n_rows[1] + p.n_rows[2];
    p.hidden = hidden;
    p.B = B;
    p.acc = acc;
    p.rope = rope;
    p.seq_lens = seq_lens;
    p.q_out = q_out;
    p.slot = slot;
    p.Hq = Hq;
    p.Hkv = Hkv;
    p.D = D;
    p.rotate = rope_base > 0.f;
    p.log2_base = p.rotate ? log2((double)rope_base) : 0.0;
    p.dev_err = dev_err;

    const int64_t n_acc = (int64_t)B * p.n_total;
    hipLaunchKernelGGL(project_prepare_kernel, dim3((unsigned)((n_acc + 255) / 256)), dim3(256), 0, s, p);
    if (dtype == LCKV_BF16) {
        const int per_pass = B > 64 ? 128 : B > 32 ? 64 : B > 16 ? 32 : 16;
        dim3 grid((p.n_total + kTileRows - 1) / kTileRows, hidden / kSliceC, (B + per_pass - 1) / per_pass);
        if (per_pass == 128)
            hipLaunchKernelGGL(project_bf16_kernel<8>, grid, dim3(256), 0, s, p);
        else if (per_pass == 64)
            hipLaunchKernelGGL(project_bf16_kernel<4>, grid, dim3(256), 0, s, p);
        else if (per_pass == 32)
            hipLaunchKernelGGL(project_bf16_kernel<2>, grid, dim3(256), 0, s, p);
        else
            hipLaunchKernelGGL(project_bf16_kernel<1>, grid, dim3(256), 0, s, p);
    } else {
        hipLaunchKernelGGL(project_f32_kernel, dim3((unsigned)((n_acc + 255) / 256)), dim3(256), 0, s, p);
    }
    const int64_t n_fin = n_acc / 2;
    if (dtype == LCKV_BF16)
        hipLaunchKernelGGL(project_finish_kernel<uint16_t>, dim3((unsigned)((n_fin + 255) / 256)), dim3(256), 0, s, p);
    else
        hipLaunchKernelGGL(project_finish_kernel<uint32_t>, dim3((unsigned)((n_fin + 255) / 256)), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace lckv
