// The projections either side of the attention, for one decode step of one layer (Section 2.1 of the LCKV paper:
// every layer maps the hidden state to queries; only a layer that PRODUCES a cache slot - a warmup layer, or the one
// condensed layer that owns the shared cache - maps it to keys and values, the others have no W_K, W_V at all):
//   y[b][n] = sum_c x[b][c] * W[n][c]        W = W_Q (and W_K, W_V stacked below it for a producing layer)
// then the rotary position embedding on queries and keys at position t_b (Llama convention: channel i < D/2 of a
// head is paired with channel i + D/2, angle t_b * base^(-2i/D)), the queries written to q_out, the keys and
// values stored straight into the slot at position t_b (the append of the decode step, fused).
//
// bf16: ONE launch.  A workgroup of 4 waves owns one or two tiles of 16 output features over the WHOLE hidden
// dimension and up to 64 sequences; the hidden dimension is cut among its four waves, which add their sums through
// LDS at the end - no partial sums travel through memory, and the rotation, the rounding and the scatter into
// q_out / the cache pages are the kernel's epilogue.  What makes the epilogue local is the order of the rows in the
// packed weight image (made once, when the model is loaded, by the pack kernel below): a tile holds the rows of
// 8 rotary pairs - channels i .. i+7 of a head and their partners i + D/2 .. - so a pair sits in two lanes of
// one wave, 32 lanes apart, and is exchanged with one v_permlane32_swap.  Each wave streams its tiles' weights
// straight into registers, a contiguous KiB per load, two chunks of the hidden dimension in flight; since no two
// waves need the same hidden channels, the x operands go straight to registers too (from the L2: x is small).
// Batches above 64 sequences are cut into parts that read the same weights at the same time on the same XCD,
// which fetches them from HBM once.  fp32 (parity mode): a plain product and a finish kernel, two launches.
// The product streams each weight once from HBM (what bounds it: 2 * N * hidden bytes against 4 * B flops per
// weight).
#include "bf16_mfma_common.h"

namespace lckv {

namespace {

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
    int32_t n_bparts;           // bf16: parts of 64 (or fewer) sequences the batch is cut into
    double rev_freq[64];        // bf16: base^(-2i/D) / (2 pi), i < D/2: turns per position of rotary pair i
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
// (kb, r) of step s holding channels 32s + 8kb .. +7 of the tile's row r, i.e. the A operands of the tile in the
// order and lane layout the matrix instruction takes them; a tile's image is contiguous (hidden * 32 bytes).
// Tile t of a matrix with heads of D channels holds, of head t / (D/16), the rows of 8 rotary pairs:
// rows r < 8 are channels 8 (t % (D/16)) + r, rows r >= 8 their partners D/2 further on.
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

// Row-major [N][hidden] bf16 -> the packed image above.  One thread per 16-byte chunk of the image.
__global__ void pack_weight_bf16_kernel(const uint16_t *src, uint16_t *dst, int N, int hidden, int D) {
    const int chunks_per_row = hidden / 8;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)N * chunks_per_row) return;
    // image order: [tile][step][kb][r]
    const int r = (int)(i & 15), kb = (int)((i >> 4) & 3);
    const int64_t ts = i >> 6;
    const int steps = hidden / 32, st = (int)(ts % steps), t = (int)(ts / steps);
    const int tph = D / 16, head = t / tph, ti = t % tph;
    const int row = head * D + 8 * ti + (r < 8 ? r : D / 2 + r - 8);
    const u32x4 v = *(const u32x4 *)(src + (int64_t)row * hidden + st * 32 + kb * 8);
    *(u32x4 *)(dst + i * 8) = v;
}

// The end of both bf16 kernels: the four waves' sums over their quarters of the hidden dimension are added in a
// fixed order (the result does not depend on the launch), rotated, rounded once and stored.
// `len_of` holds the cached lengths of the sequences this lane finishes (block wave + 4 k in entry k; -1 past the
// batch) and `freq` the table of turns per position in LDS: both were fetched when the kernel started, so that no
// round trip to memory is left between the last matrix instruction and the stores.
template <int TILES, int NB>
__device__ __forceinline__ void project_reduce_and_store(const ProjParams &p, char *lds, int slot_bytes,
                                                         const floatx4 (&acc)[TILES][NB], int tg, int b0, int wave,
                                                         int lane, const int (&len_of)[(NB + 3) / 4],
                                                         const double *freq) {
    // wave w's sums live in its own slot of the LDS (the one its x chunks went through): [tile][block][lane]
    auto red = [&](int w, int nt, int j) -> floatx4 & {
        return *(floatx4 *)(lds + w * slot_bytes + ((nt * NB + j) * 64 + lane) * 16);
    };
    const int c = lane & 15, kb = lane >> 4;
#pragma unroll
    for (int nt = 0; nt < TILES; ++nt)
#pragma unroll
        for (int j = 0; j < NB; ++j) red(wave, nt, j) = acc[nt][j];
    __syncthreads();
#pragma unroll
    for (int jk = 0; jk < (NB + 3) / 4; ++jk) {  // wave w finishes sequence blocks w, w + 4, ...
        const int j = wave + 4 * jk;
        if (j >= NB) break;
        const int b = b0 + 16 * j + c;
        const int t_pos = max(len_of[jk], 0);
#pragma unroll
        for (int nt = 0; nt < TILES; ++nt) {
            floatx4 y = red(0, nt, j);
#pragma unroll
            for (int w = 1; w < 4; ++w) y += red(w, nt, j);
            // lane (kb, c) holds rows 4 kb .. + 3 of the tile for sequence b: kb < 2: channels i0 + 4 kb + e of the
            // head, kb >= 2: their rotary partners.  a = the lower lane's value, b = the upper lane's, in both.
            const int t = tg * TILES + nt, tph = p.D / 16;
            const int hg = t / tph, i0 = 8 * (t % tph) + 4 * (kb & 1);
            const bool is_v = hg >= p.Hq + p.Hkv, upper = kb >= 2;
            float outv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float lo = y[e], hi = y[e];
                swap_halves32(lo, hi);
                float cs = 1.f, sn = 0.f;
                if (p.rotate && !is_v) {
                    const double turns = (double)t_pos * freq[i0 + e];
                    const float fr = (float)(turns - floor(turns));
                    sn = __builtin_amdgcn_sinf(fr);  // sine and cosine of 2 pi fr
                    cs = __builtin_amdgcn_cosf(fr);
                }
                outv[e] = upper ? hi * cs + lo * sn : lo * cs - hi * sn;
            }
            if (b >= p.B) continue;
            const int d0 = i0 + (upper ? p.D / 2 : 0);  // channels d0 .. d0 + 3 of head hg
            const u32x2 pk = {pack_bf16(outv[0], outv[1]), pack_bf16(outv[2], outv[3])};
            if (hg < p.Hq) {
                *(u32x2 *)((uint16_t *)p.q_out + ((int64_t)b * p.Hq + hg) * p.D + d0) = pk;
                continue;
            }
            const int g = is_v ? hg - p.Hq - p.Hkv : hg - p.Hq;
            if (p.k_out) {  // handed back to the caller, who appends them after the layer's attention
                *(u32x2 *)((uint16_t *)(is_v ? p.v_out : p.k_out) + ((int64_t)b * p.Hkv + g) * p.D + d0) = pk;
                continue;
            }
            // into the slot at position t_b (the ring entry under the sink + window policy)
            int entry = len_of[jk];
            if (entry >= 0) entry = entry_of_position(p.slot, entry);
            if (entry < 0 || entry >= p.slot.capacity) {
                if (d0 == 0) atomicOr(p.dev_err, LCKV_DEV_ERR_CAPACITY);
                continue;
            }
            const int64_t pp = page_pair_index(p.slot, b, g, entry / kPage);
            if (pp < 0) {
                if (d0 == 0) atomicOr(p.dev_err, LCKV_DEV_ERR_BLOCK);
                continue;
            }
            uint16_t *page = (uint16_t *)(p.slot.base + pp * (2 * (int64_t)p.slot.page_bytes) + (is_v ? p.slot.page_bytes : 0));
            const int jpos = entry % kPage;
            if (!is_v) {  // four channels of one octet: 8 contiguous bytes of the K page
                *(u32x2 *)(page + k_elem_offset_bf16(jpos, d0)) = pk;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) page[v_elem_offset_bf16(jpos, d0 + e)] = (uint16_t)(pack_bf16(outv[e], 0.f) & 0xffffu);
            }
        }
    }
}

// The bf16 projection.  TILES tiles of 16 features per workgroup, NB blocks of 16 sequences, KS steps of 32 hidden
// channels per chunk.  grid: feature groups x batch parts, laid out so that the parts of one group follow each other
// on one XCD.  Each wave streams the weights of its quarter of the hidden dimension into registers, a contiguous
// KiB per load, two chunks in flight.  The x operands of a matrix instruction are 64 bytes of 16 different rows;
// fetched like that (rows 2 * hidden bytes apart: one L2 channel at a time) they were measured three times slower
// than the weight stream, so each wave fetches its x chunk as whole rows (KS * 64 contiguous bytes per row),
// parks it in a wave-private piece of LDS with the 16-byte chunks of a row exchanged by the row number, and reads
// the operands from there without bank conflicts.  One chunk of x in registers on its way, one in LDS being
// used; no barrier before the final sum (nothing else is shared between waves).
template <int TILES, int NB, int KS>
__global__ __launch_bounds__(256) void project_staged_bf16_kernel(ProjParams p) {
    constexpr int kRowBytes = KS * 64, kLpr = kRowBytes / 16;   // bytes / lanes per row of a chunk
    constexpr int kRowsPerLoad = 64 / kLpr, kLoads = NB * 16 / kRowsPerLoad;
    constexpr int kStage = NB * 16 * kRowBytes;
    static_assert(kLoads >= 1 && kLpr <= 64, "a row of a chunk is at most one load instruction");
    // the sums of the four waves are exchanged through the same LDS once the x chunks are done with
    constexpr int kRed = TILES * NB * 64 * 16;
    constexpr int kSlot = kStage > kRed ? kStage : kRed;
    __shared__ __attribute__((aligned(16))) char xs[4][kSlot];
    __shared__ __attribute__((aligned(16))) double sm_freq[64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, kb = lane >> 4;
    const int n_groups = p.n_total / (16 * TILES);
    const int id = blockIdx.x;
    const int tg = (id / (8 * p.n_bparts)) * 8 + id % 8, bp = (id / 8) % p.n_bparts;
    if (tg >= n_groups) return;  // uniform
    const int b0 = bp * (16 * NB);
    // what the end of the kernel needs from memory, asked for now: the rotation table (read by the waves after
    // the barrier that precedes the final sum) and the lengths of the sequences this lane will finish
    if (tid < 64) sm_freq[tid] = p.rev_freq[tid];
    int len_of[(NB + 3) / 4];
#pragma unroll
    for (int jk = 0; jk < (NB + 3) / 4; ++jk) {
        const int b = b0 + 16 * (wave + 4 * jk) + c;
        len_of[jk] = (wave + 4 * jk < NB && b < p.B) ? p.seq_lens[b] : -1;
    }
    const int ks_w = p.hidden / 128;          // steps of 32 channels per wave; a multiple of KS (checked by the host)
    const int k_begin = wave * ks_w;
    const char *wimg[TILES];
#pragma unroll
    for (int nt = 0; nt < TILES; ++nt) wimg[nt] = stacked_tile(p, tg * TILES + nt) + ((int64_t)k_begin * 64 + lane) * 16;
    const char *xsrc[kLoads];  // load i: row i * kRowsPerLoad + lane / kLpr of the part, 16-byte chunk lane % kLpr
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int row = i * kRowsPerLoad + lane / kLpr;
        xsrc[i] = (const char *)p.x + ((int64_t)min(b0 + row, p.B - 1) * p.hidden + k_begin * 32) * 2 + (lane % kLpr) * 16;
    }
    char *stage = xs[wave];

    floatx4 acc[TILES][NB];
#pragma unroll
    for (int nt = 0; nt < TILES; ++nt)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[nt][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    u32x4 wa[TILES][KS], wb[TILES][KS], xraw[kLoads];
    auto load_w = [&](u32x4 (&w)[TILES][KS], int ch) {
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int nt = 0; nt < TILES; ++nt)
                w[nt][s] = __builtin_nontemporal_load((const u32x4 *)(wimg[nt] + (ch * KS + s) * 1024));
    };
    auto load_x = [&](int ch) {
#pragma unroll
        for (int i = 0; i < kLoads; ++i) xraw[i] = *(const u32x4 *)(xsrc[i] + ch * kRowBytes);
    };
    auto park_x = [&]() {
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            const int row = i * kRowsPerLoad + lane / kLpr;
            *(u32x4 *)(stage + row * kRowBytes + (((lane % kLpr) ^ (row & (kLpr - 1))) * 16)) = xraw[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    auto use_chunk = [&](const u32x4 (&w)[TILES][KS]) {
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int row = 16 * j + c;
                const u32x4 xb = *(const u32x4 *)(stage + row * kRowBytes + (((4 * s + kb) ^ (row & (kLpr - 1))) * 16));
#pragma unroll
                for (int nt = 0; nt < TILES; ++nt)
                    acc[nt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[nt][s]),
                                                                         __builtin_bit_cast(bf16x8, xb), acc[nt][j], 0, 0, 0);
            }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    const int n_chunks = ks_w / KS;
    load_x(0);
    load_w(wa, 0);
    park_x();
    for (int ch = 0; ch < n_chunks; ch += 2) {  // the weight registers take turns (no register copies)
        if (ch + 1 < n_chunks) {
            load_x(ch + 1);
            load_w(wb, ch + 1);
        }
        use_chunk(wa);
        if (ch + 1 >= n_chunks) break;
        park_x();
        if (ch + 2 < n_chunks) {
            load_x(ch + 2);
            load_w(wa, ch + 2);
        }
        use_chunk(wb);
        if (ch + 2 < n_chunks) park_x();
    }
    project_reduce_and_store<TILES, NB>(p, &xs[0][0], kSlot, acc, tg, b0, wave, lane, len_of, sm_freq);
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

hipError_t launch_pack_weight(const void *src, void *dst, int N, int hidden, int D, int dtype, hipStream_t s) {
    if (dtype == LCKV_BF16) {
        const int64_t chunks = (int64_t)N * (hidden / 8);
        hipLaunchKernelGGL(pack_weight_bf16_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s,
                           (const uint16_t *)src, (uint16_t *)dst, N, hidden, D);
        return hipGetLastError();
    }
    return hipMemcpyAsync(dst, src, (size_t)N * hidden * 4, hipMemcpyDeviceToDevice, s);  // fp32: row-major as is
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
        if (D / 2 > 64) return hipErrorInvalidValue;
        for (int i = 0; i < D / 2; ++i)
            p.rev_freq[i] = p.rotate ? pow((double)rope_base, -2.0 * i / D) / 6.283185307179586476925286766559 : 0.0;
        // Sequences and feature tiles per workgroup, measured on the Llama-7B shape (ms per step): B = 64: 32 x 2
        // tiles 0.49, 64 x 1 tile 0.54, 64 x 2 tiles 0.62; B = 128: 64 x 2 tiles 0.66, 32 x 4 tiles 0.70, 64 x 1 tile
        // 0.89.  (n_total is a multiple of 64: whole heads of at least 64 channels.)
        const int per_part = B > 64 ? 64 : B > 16 ? 32 : 16;
        const int tiles = B > 32 ? 2 : 1;
        p.n_bparts = (B + per_part - 1) / per_part;
        const int n_groups = p.n_total / (16 * tiles);
        dim3 grid((unsigned)((n_groups + 7) / 8 * 8 * p.n_bparts));
        // hidden channels per chunk: as many steps as divide a wave's quarter (hidden / 128 steps, an even number)
        // and as the registers of this batch shape hold
        const int ks_w = hidden / 128;
        const int ks_max = per_part == 64 ? 4 : per_part == 32 ? 8 : 16;
        int ks = 2;
        while (ks * 2 <= ks_max && ks_w % (ks * 2) == 0) ks *= 2;
#define LCKV_PROJECT_LAUNCH(T, NB, KS) \
    hipLaunchKernelGGL((project_staged_bf16_kernel<T, NB, KS>), grid, dim3(256), 0, s, p)
        if (per_part == 64) {
            if (ks == 4) LCKV_PROJECT_LAUNCH(2, 4, 4); else LCKV_PROJECT_LAUNCH(2, 4, 2);
        } else if (per_part == 32 && tiles == 2) {
            if (ks >= 4) LCKV_PROJECT_LAUNCH(2, 2, 4); else LCKV_PROJECT_LAUNCH(2, 2, 2);
        } else if (per_part == 32) {
            if (ks == 8) LCKV_PROJECT_LAUNCH(1, 2, 8); else if (ks == 4) LCKV_PROJECT_LAUNCH(1, 2, 4); else LCKV_PROJECT_LAUNCH(1, 2, 2);
        } else {
            if (ks == 16) LCKV_PROJECT_LAUNCH(1, 1, 16); else if (ks == 8) LCKV_PROJECT_LAUNCH(1, 1, 8);
            else if (ks == 4) LCKV_PROJECT_LAUNCH(1, 1, 4); else LCKV_PROJECT_LAUNCH(1, 1, 2);
        }
#undef LCKV_PROJECT_LAUNCH
        return hipGetLastError();
    }
    p.n_slices = 1;
    hipLaunchKernelGGL(project_f32_kernel, dim3((unsigned)((n_acc + 255) / 256)), dim3(256), 0, s, p);
    hipLaunchKernelGGL(project_finish_kernel<uint32_t>, dim3((unsigned)((n_acc / 2 + 255) / 256)), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace lckv
