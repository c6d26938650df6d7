// The projections either side of the attention, for one decode step of one layer (Section 2.1 of the LCKV paper:
// every layer maps the hidden state to queries; only a layer that PRODUCES a cache slot - a warmup layer, or the one
// condensed layer that owns the shared cache - maps it to keys and values, the others have no W_K, W_V at all):
//   y[b][n] = sum_c x[b][c] * W[n][c]        W = W_Q (and W_K, W_V stacked below it for a producing layer)
// then the rotary position embedding on queries and keys at position t_b (Llama convention: channel i < D/2 of a
// head is paired with channel i + D/2, angle t_b * base^(-2i/D)), the queries written to q_out, the keys and
// values stored straight into the slot at position t_b (the append of the decode step, fused).
//
// Two launches on the caller's stream:
//   1. the matrix product, split over the hidden dimension into slices; every slice writes its partial sums
//      [slice][B][N] in fp32 with plain stores (atomic adds from all XCDs onto one accumulator were measured:
//      they resolve outside the per-XCD L2 and took 35x the time of the weight stream)
//   2. finish: add the slices in a fixed order, rotate (angles formed in double), round once, scatter into
//      q_out / the cache pages
// The product streams each weight once from HBM (what bounds it: 2 * N * hidden bytes against 4 * B flops per
// weight) and is shaped for that.  A workgroup of 4 waves owns 128 output features x one slice of KSTEPS * 32
// hidden channels x up to 128 sequences (in two rounds of 64, both x slices in LDS from the start).  Each wave owns two 16-feature tiles whose weights it loads straight
// into registers, all of them issued before anything else (up to 128 KiB per workgroup in flight); meanwhile the
// x slice is staged in LDS in matrix-operand order, shared by the waves; after one barrier the wave runs its
// matrix instructions, each LDS read of an x operand feeding two of them.  Features on the rows of the tiles
// (A operand = weights), sequences on the columns.  The weights are taken in a packed image (made once, when
// the model is loaded, by the pack kernel below) whose tiles are in matrix-operand order, so that every load
// instruction is a contiguous KiB, as for the cache pages: with row-major weights an instruction touched 64
// bytes of 16 rows and the stream reached 2.0 TB/s at best.
#include "bf16_mfma_common.h"

namespace lckv {

namespace {

constexpr int kTileRows = 128;  // output features per workgroup (8 tiles of 16, two per wave)
typedef __attribute__((address_space(3))) void *LdsPtr;

struct ProjParams {
    const void *x;              // [B][hidden]
    const void *w[3];           // W_Q [n_rows[0]][hidden], W_K, W_V (null: absent)
    int32_t n_rows[3];
    int32_t n_total;            // rows of the stacked matrix
    int32_t hidden, B;
    float *acc;                 // [n_slices][B][n_total] fp32 partial sums
    int32_t n_slices;
    const int32_t *seq_lens;
    void *q_out;                // [B][Hq][D]
    void *k_out, *v_out;        // [B][Hkv][D]: if given, the new K/V go there instead of into the slot
    SlotView slot;              // where K/V go (producing layers)
    int32_t Hq, Hkv, D;
    double log2_base;           // log2(rope base); rotate = 0: no rotation
    int32_t rotate;
    int32_t *dev_err;
};

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

// Tile (16 rows) t of the stacked matrix -> its packed bf16 image: [hidden/32 steps][64 lanes][8 channels], lane
// (kb, r) of step s holding channels 32s + 8kb .. +7 of row r, i.e. the A operands of the tile in the order and
// lane layout the matrix instruction takes them; a tile's image is contiguous (hidden * 32 bytes).
__device__ __forceinline__ const char *stacked_tile(const ProjParams &p, int t) {
    int m = 0;
    if (t >= p.n_rows[0] / 16) {
        t -= p.n_rows[0] / 16;
        m = 1;
        if (t >= p.n_rows[1] / 16) {
            t -= p.n_rows[1] / 16;
            m = 2;
        }
    }
    return (const char *)p.w[m] + (int64_t)t * p.hidden * 32;
}

// Row-major [N][hidden] bf16 -> the packed image above.  One thread per 16-byte chunk.
__global__ void pack_weight_bf16_kernel(const uint16_t *src, uint16_t *dst, int N, int hidden) {
    const int chunks_per_row = hidden / 8;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)N * chunks_per_row) return;
    const int n = (int)(i / chunks_per_row), ch = (int)(i % chunks_per_row);
    const int t = n >> 4, r = n & 15, s = ch >> 2, kb = ch & 3;
    const u32x4 v = *(const u32x4 *)(src + (int64_t)n * hidden + ch * 8);
    *(u32x4 *)(dst + (((int64_t)t * (hidden / 32) + s) * 64 + kb * 16 + r) * 8) = v;
}

// Launch 1, bf16.  NB = 16-sequence blocks per pass (1, 2, 4 or 8), KSTEPS = matrix instructions (32 hidden
// channels each) per slice.  grid (feature blocks, slices, passes of 16 * NB sequences).
template <int NB, int KSTEPS, int ROUNDS>
__global__ __launch_bounds__(256, (ROUNDS == 1 ? 2 : 1)) void project_bf16_kernel(ProjParams p) {
    // The x slices in LDS, one buffer per round of 16 * NB sequences.  With 512-channel slices a sequence's slice
    // is 1 KiB = one fully coalesced load instruction, so it is kept row-major, rows 1 KiB + 16 bytes apart: lane
    // (kb, c) then reads its operand of step s at row c, byte 64s + 16kb, and the 16 lanes of a quarter wave fall
    // on 16 different bank quadruples.  With 256-channel slices the image is in operand order (each instruction
    // gathers 64 bytes of 16 sequences).
    constexpr bool kRowMajor = KSTEPS == 16;
    constexpr int kRowStride = KSTEPS * 64 + 16;
    constexpr int kRoundBytes = kRowMajor ? NB * 16 * kRowStride : NB * KSTEPS * 1024;
    constexpr int kDmaPerWave = kRowMajor ? 4 * NB : NB * KSTEPS / 4;  // load instructions per wave and round
    __shared__ __attribute__((aligned(16))) char lds[ROUNDS * kRoundBytes];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, kb = lane >> 4;
    const int c0 = blockIdx.y * (KSTEPS * 32);
    static_assert(NB * KSTEPS % 4 == 0, "tiles divide among the four waves");
    static_assert(2 * KSTEPS + (ROUNDS - 1) * kDmaPerWave < 64, "the wait below counts this many loads");

    // 1. The x slices of all rounds into LDS by direct global-to-LDS loads (issued as assembly: the compiler's
    //    builtin would make every LDS read below wait on each of them separately).  Rows past the batch: the last
    //    row, whose columns are never stored.
    auto dma = [&](const uint16_t *src, const char *dst_lds) {  // lane l's 16 bytes land at dst_lds + 16 l
        const uint32_t dst = (uint32_t)(uintptr_t)(LdsPtr)dst_lds;
        uint32_t m0_saved;  // M0 carries the LDS address; whatever the compiler keeps there is put back
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\t"
                     "s_mov_b32 m0, %0"
                     : "=&s"(m0_saved)
                     : "s"(dst), "v"(src)
                     : "memory");
    };
#pragma unroll
    for (int round = 0; round < ROUNDS; ++round) {
        const int b0 = (blockIdx.z * ROUNDS + round) * (16 * NB);
        const char *buf = lds + round * kRoundBytes;
        if (kRowMajor) {
#pragma unroll
            for (int k = 0; k < kDmaPerWave; ++k) {  // one instruction per sequence
                const int row = wave + 4 * k;
                dma((const uint16_t *)p.x + (int64_t)min(b0 + row, p.B - 1) * p.hidden + c0 + lane * 8,
                    buf + row * kRowStride);
            }
        } else {
#pragma unroll
            for (int k = 0; k < kDmaPerWave; ++k) {  // one instruction per (sequence block j, step st) operand
                const int tile = wave + 4 * k, j = tile / KSTEPS, st = tile % KSTEPS;
                dma((const uint16_t *)p.x + (int64_t)min(b0 + 16 * j + r, p.B - 1) * p.hidden + c0 + st * 32 + kb * 8,
                    buf + tile * 1024);
            }
        }
    }

    // 2. This wave's weights: two tiles x KSTEPS steps, from the packed image: every load instruction is one
    //    contiguous, lane-ordered KiB and the KSTEPS loads of a tile are consecutive KiBs.  (A tile past the end
    //    of the matrix reads the last tile instead, so that every wave has the same number of loads in flight.)
    u32x4 wr[2][KSTEPS];
    bool have[2];
    const int last_tile = p.n_total / 16 - 1;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int t = blockIdx.x * (kTileRows / 16) + wave * 2 + nt;
        have[nt] = t <= last_tile;  // wave-uniform
        const char *img = stacked_tile(p, min(t, last_tile)) + ((int64_t)(c0 / 32) * 64 + lane) * 16;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) wr[nt][s] = __builtin_nontemporal_load((const u32x4 *)(img + s * 1024));
    }

    // 3. The first round's x has landed when at most the later loads are outstanding (loads complete in order):
    //    the matrix instructions start on it while the weights are still streaming in - the compiler waits for
    //    each weight register where it is first used.
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * KSTEPS + (ROUNDS - 1) * kDmaPerWave) : "memory");
    float *part = p.acc + (int64_t)blockIdx.y * p.B * p.n_total;
#pragma unroll
    for (int round = 0; round < ROUNDS; ++round) {
        const int b0 = (blockIdx.z * ROUNDS + round) * (16 * NB);
        const char *buf = lds + round * kRoundBytes;
        if (round > 0) {
            if (b0 >= p.B) break;  // uniform
            asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");  // every wave's share of this round's x
        }
        floatx4 acc[2][NB];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int j = 0; j < NB; ++j) acc[nt][j] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s)
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const char *xp = kRowMajor ? buf + (16 * j + r) * kRowStride + (4 * s + kb) * 16
                                           : buf + ((j * KSTEPS + s) * 64 + lane) * 16;
                const bf16x8 xb = __builtin_bit_cast(bf16x8, *(const u32x4 *)xp);
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    acc[nt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wr[nt][s]), xb,
                                                                         acc[nt][j], 0, 0, 0);
            }

        // lane (kb, c) holds features n0 + 4kb .. +3 of sequence b0 + 16j + c: 16 bytes of this slice's partial sums
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            if (!have[nt]) continue;
            const int n0 = blockIdx.x * kTileRows + (wave * 2 + nt) * 16;
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int b = b0 + 16 * j + r;
                if (b < p.B) *(floatx4 *)(part + (int64_t)b * p.n_total + n0 + 4 * kb) = acc[nt][j];
            }
        }
    }
}

// Launch 1, fp32 (parity mode, not tuned): one thread per output, products accumulated in double.
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

template <typename E>
__device__ __forceinline__ void finish_pair(const ProjParams &p, float2 cs, int b, int hg, int i);

// Launch 2.  One thread per (sequence, head of the stacked output, channel pair i < D/2): adds the slices, forms
// the angle in double (position 32767 at the highest frequency is 32767 rad), rotates, stores.
template <typename E>
__global__ void project_finish_kernel(ProjParams p) {
    const int half = p.D / 2;
    const int heads = p.n_total / p.D;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)p.B * heads * half) return;
    const int i = (int)(idx % half);
    const int hg = (int)((idx / half) % heads);
    const int b = (int)(idx / ((int64_t)half * heads));
    float2 cs = {1.f, 0.f};
    if (p.rotate && hg < p.Hq + p.Hkv) {
        int t = p.seq_lens[b];
        if (t < 0) t = 0;
        const double angle = (double)t * exp2(-2.0 * i / p.D * p.log2_base);
        cs = float2{(float)cos(angle), (float)sin(angle)};
    }
    finish_pair<E>(p, cs, b, hg, i);
}

template <typename E>
__device__ __forceinline__ void finish_pair(const ProjParams &p, float2 cs, int b, int hg, int i) {
    const int half = p.D / 2;
    const float *y = p.acc + (int64_t)b * p.n_total + (int64_t)hg * p.D;
    float lo = 0.f, hi = 0.f;
#pragma unroll 8
    for (int sl = 0; sl < p.n_slices; ++sl) {  // fixed order: the result does not depend on the launch
        lo += y[(int64_t)sl * p.B * p.n_total + i];
        hi += y[(int64_t)sl * p.B * p.n_total + i + half];
    }
    const bool is_v = hg >= p.Hq + p.Hkv;
    if (!is_v) {
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
    const int g = is_v ? hg - p.Hq - p.Hkv : hg - p.Hq;
    if (p.k_out) {  // handed back to the caller, who appends them after the layer's attention
        E *o = (E *)(is_v ? p.v_out : p.k_out) + ((int64_t)b * p.Hkv + g) * p.D;
        o[i] = to_elem(lo, E{});
        o[i + half] = to_elem(hi, E{});
        return;
    }
    // a key or value head: into the slot at position t_b (the ring entry under the sink + window policy)
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

hipError_t launch_pack_weight(const void *src, void *dst, int N, int hidden, int dtype, hipStream_t s) {
    if (dtype == LCKV_BF16) {
        const int64_t chunks = (int64_t)N * (hidden / 8);
        hipLaunchKernelGGL(pack_weight_bf16_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s,
                           (const uint16_t *)src, (uint16_t *)dst, N, hidden);
        return hipGetLastError();
    }
    return hipMemcpyAsync(dst, src, (size_t)N * hidden * 4, hipMemcpyDeviceToDevice, s);  // fp32: row-major as is
}

// Hidden channels per slice for the bf16 product: 512 when that still gives every compute unit a workgroup, else
// 256 (more, thinner slices).  Needs hidden % 256 == 0.
int project_slice_channels(int n_total, int hidden) {
    const int64_t blocks = (n_total + kTileRows - 1) / kTileRows;
    return (hidden % 512 == 0 && blocks * (hidden / 512) >= 256) ? 512 : 256;
}

// x [B][hidden]; w_k / w_v null for a layer that produces no slot (then `slot` is not used).
hipError_t launch_project(const void *x, int hidden, const void *w_q, const void *w_k, const void *w_v, void *q_out,
                          void *k_out, void *v_out, const SlotView &slot, const int32_t *seq_lens, int B, int Hq, int Hkv, int D, int dtype,
                          float rope_base, float *acc, int32_t *dev_err, hipStream_t s) {
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
    p.seq_lens = seq_lens;
    p.q_out = q_out;
    p.k_out = k_out;
    p.v_out = v_out;
    p.slot = slot;
    p.Hq = Hq;
    p.Hkv = Hkv;
    p.D = D;
    p.rotate = rope_base > 0.f;
    p.log2_base = p.rotate ? log2((double)rope_base) : 0.0;
    p.dev_err = dev_err;

    const int64_t n_acc = (int64_t)B * p.n_total;
    if (dtype == LCKV_BF16) {
        // up to 64 sequences per round, up to two rounds per workgroup (the weights are read once per 128 sequences)
        const int per_round = B > 32 ? 64 : B > 16 ? 32 : 16;
        const int rounds = B > 64 ? 2 : 1;
        const int ksteps = project_slice_channels(p.n_total, hidden) / 32;
        p.n_slices = hidden / (ksteps * 32);
        dim3 grid((p.n_total + kTileRows - 1) / kTileRows, p.n_slices, (B + per_round * rounds - 1) / (per_round * rounds));
#define LCKV_PROJECT_LAUNCH(NB, ROUNDS)                                                   \
    if (ksteps == 16)                                                                     \
        hipLaunchKernelGGL((project_bf16_kernel<NB, 16, ROUNDS>), grid, dim3(256), 0, s, p); \
    else                                                                                  \
        hipLaunchKernelGGL((project_bf16_kernel<NB, 8, ROUNDS>), grid, dim3(256), 0, s, p)
        if (rounds == 2) {
            LCKV_PROJECT_LAUNCH(4, 2);
        } else if (per_round == 64) {
            LCKV_PROJECT_LAUNCH(4, 1);
        } else if (per_round == 32) {
            LCKV_PROJECT_LAUNCH(2, 1);
        } else {
            LCKV_PROJECT_LAUNCH(1, 1);
        }
#undef LCKV_PROJECT_LAUNCH
    } else {
        p.n_slices = 1;
        hipLaunchKernelGGL(project_f32_kernel, dim3((unsigned)((n_acc + 255) / 256)), dim3(256), 0, s, p);
    }
    if (dtype == LCKV_BF16)
        hipLaunchKernelGGL(project_finish_kernel<uint16_t>, dim3((unsigned)((n_acc / 2 + 255) / 256)), dim3(256), 0, s, p);
    else
        hipLaunchKernelGGL(project_finish_kernel<uint32_t>, dim3((unsigned)((n_acc / 2 + 255) / 256)), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace lckv
