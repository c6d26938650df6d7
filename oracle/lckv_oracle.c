/*
 * CPU oracle for one decode step of the Layer-Condensed KV Cache model
 * (Wu & Tu, "Layer-Condensed KV Cache for Efficient Inference of Large
 * Language Models", Section 2.1 and Figure 1b).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests, the smoke check
 * and the benchmark's CPU-baseline leg may call it.  It shares no code with
 * the GPU library and never calls it.
 *
 * What it computes is the plain definition, in double precision, on a cache
 * that has no layout tricks: K and V are dense arrays
 *     [slot][sequence b][position j][kv head g][d]        (float, row-major)
 * and every score, every exponential and every weighted sum is a scalar loop.
 * Inputs arrive as float (a bf16 value converts to float exactly); they are
 * widened to double before any arithmetic and the result stays in double.
 *
 * Pinned by tests/test_oracle_*.py: closed forms, reduction to standard causal
 * attention when every layer is a warmup layer (Section 4.2, caption of the
 * warmup-layer figure: w = L is exactly the standard transformer), a library
 * softmax/matmul evaluation, invariants.
 * The sink + window cache policy of Section 3.3 (StreamingLLM integration) is
 * an option of the step; it is written as a selection of logical positions
 * from the full history, not as a ring buffer.
 * lckv_oracle_project is the q / k / v projection with the rotary position
 * embedding, the step either side of the attention (which layers have K/V
 * projections at all is the pairing table's producer column).
 * lckv_oracle_footprint / lckv_oracle_max_batch are the memory side of the
 * method (Sections 1 and 3.1): bytes of K and V kept for a batch, counted
 * cache by cache from the pairing table, and the largest batch under a byte
 * budget found by trying batch sizes upward.
 * "Parity unpinned": the paper does not restate the rotary embedding, so the
 * pairing of channels (i with i + D/2) and the base are the Llama convention
 * taken as a reading; the formula under that reading is pinned.
 * "Parity unpinned": which layer owns the shared cache when the topmost
 * layers are warmup layers (pairing rule 1 vs rule 2 below) is not decided by
 * the paper; both are implemented, rule 1 is the default.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define LCKV_ORACLE_PAIR_TOP_OF_CONDENSED 0 /* rule 1 */
#define LCKV_ORACLE_PAIR_LAST_LAYER 1       /* rule 2 */

/*
 * Which cache each layer reads (Section 2.1).
 *
 *  - A warmup layer keeps standard attention: it owns a cache, appends its own
 *    new K/V, and its query sees positions 0..t (itself included).
 *  - Every other ("condensed") layer reads one shared cache that holds the
 *    K/V of "the top layer"; the diagonal is masked, so it sees 0..t-1 only.
 *
 * Rule 1: the shared cache is produced by the topmost condensed layer; warmup
 *         layers (also those above it) have caches of their own.
 * Rule 2: the shared cache is the cache of layer L-1 even if L-1 is a warmup
 *         layer (then L-1 reads it with itself visible, the condensed layers
 *         read it with the diagonal masked).
 *
 * Slots are numbered by ascending producer layer.  Outputs (all length L):
 *   kv_slot[l]       slot layer l reads
 *   self_visible[l]  1 if layer l sees the token being decoded, else 0
 *   producer[s]      for s < *n_slots, the layer whose new K/V go to slot s
 * Returns 0, or -1 on a bad argument.
 */
int lckv_oracle_pairing(int L, const uint8_t *warm, int rule, int32_t *kv_slot,
                        int32_t *self_visible, int32_t *producer,
                        int32_t *n_slots)
{
    if (L <= 0 || !warm || !kv_slot || !self_visible || !producer || !n_slots)
        return -1;
    if (rule != LCKV_ORACLE_PAIR_TOP_OF_CONDENSED &&
        rule != LCKV_ORACLE_PAIR_LAST_LAYER)
        return -1;

    int any_condensed = 0, top_condensed = -1;
    for (int l = 0; l < L; ++l)
        if (!warm[l]) { any_condensed = 1; top_condensed = l; }

    /* the layer whose K/V the condensed layers read */
    int shared_producer = -1;
    if (any_condensed)
        shared_producer = (rule == LCKV_ORACLE_PAIR_LAST_LAYER) ? L - 1
                                                                : top_condensed;

    /* producing layers in ascending order -> slot numbers */
    int ns = 0;
    int32_t *slot_of_layer = (int32_t *)malloc(sizeof(int32_t) * (size_t)L);
    if (!slot_of_layer) return -1;
    for (int l = 0; l < L; ++l) {
        int produces = warm[l] || l == shared_producer;
        slot_of_layer[l] = -1;
        if (produces) {
            slot_of_layer[l] = ns;
            producer[ns] = l;
            ++ns;
        }
    }
    for (int s = ns; s < L; ++s) producer[s] = -1;

    for (int l = 0; l < L; ++l) {
        if (warm[l]) {
            kv_slot[l] = slot_of_layer[l];
            self_visible[l] = 1;
        } else {
            kv_slot[l] = slot_of_layer[shared_producer];
            self_visible[l] = 0;
        }
    }
    *n_slots = ns;
    free(slot_of_layer);
    return 0;
}

/*
 * Attention of ONE query vector over n keys (Section 2.1; scaled dot-product
 * softmax attention, the scale being an argument):
 *     s_j = scale * <q, K_j>,   p = softmax(s),   out = sum_j p_j V_j.
 * n = 0 is the paper's "first token" case: with zero dummy K/V the result is
 * the zero vector.  K and V rows are `row_stride` floats apart.
 * `probs` (n doubles) may be NULL.
 */
void lckv_oracle_attend(const float *q, const float *K, const float *V,
                        int64_t n, int64_t row_stride, int D, double scale,
                        double *out, double *probs)
{
    for (int d = 0; d < D; ++d) out[d] = 0.0;
    if (n <= 0) return;

    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    if (!s) { for (int d = 0; d < D; ++d) out[d] = NAN; return; }

    double smax = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
        const float *k = K + j * row_stride;
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += (double)q[d] * (double)k[d];
        s[j] = scale * dot;
        if (s[j] > smax) smax = s[j];
    }
    double denom = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        s[j] = exp(s[j] - smax);
        denom += s[j];
    }
    for (int64_t j = 0; j < n; ++j) {
        double p = s[j] / denom;
        if (probs) probs[j] = p;
        const float *v = V + j * row_stride;
        for (int d = 0; d < D; ++d) out[d] += p * (double)v[d];
    }
    free(s);
}

/*
 * Many independent (query, key set) items, used for sampled checks of large
 * workloads: item i has q[i][D], K[i][T][D], V[i][T][D] (dense) and n_keys[i]
 * visible keys.  Items run in parallel on `threads` threads (0 = all cores).
 * Returns the number of threads used.
 */
int lckv_oracle_attend_many(int64_t n_items, const float *q, const float *K,
                            const float *V, const int64_t *n_keys, int64_t T,
                            int D, double scale, double *out, int threads)
{
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
    used = threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
    for (int64_t i = 0; i < n_items; ++i)
        lckv_oracle_attend(q + i * D, K + i * T * D, V + i * T * D, n_keys[i],
                           D, D, scale, out + i * D, NULL);
    return used;
}

/*
 * One decode step of the whole model's attention (Sections 2.1 and 2.2's
 * "decoding one token at a time"): layers in index order; a producing layer
 * first stores its new K/V at position t_b of its slot, then every layer's
 * queries attend to the slot the pairing assigns, over t_b keys (condensed)
 * or t_b + 1 keys (warmup).  Query head h reads kv head h / (Hq / Hkv).
 * Finally every t_b grows by one.
 *
 *   Kc, Vc   [n_slots][B][T_cap][Hkv][D] float, updated in place
 *   lens     [B] tokens cached before the step, incremented on return
 *   q        [L][B][Hq][D]
 *   k_new, v_new   [n_slots][B][Hkv][D], slot order
 *   out      [L][B][Hq][D] double
 * Returns the thread count used (>0), or a negative value on error
 * (-1 bad argument, -2 a sequence is already at capacity).
 *
 * Sink + window policy (Section 3.3, integration with StreamingLLM: only the
 * K/V of the first few tokens - four by default - and of the recent tokens are
 * kept): with window > 0, of a query's n candidate positions 0..n-1 only the
 * first `sink` and the last `window` are attended to.  The oracle keeps the
 * whole history in Kc, Vc and selects those positions by their logical index;
 * window = 0 switches the policy off.
 */
int lckv_oracle_step_streaming(int L, int Hq, int Hkv, int D, int B,
                               int64_t T_cap, const uint8_t *warm, int rule,
                               double scale, float *Kc, float *Vc,
                               int32_t *lens, const float *q,
                               const float *k_new, const float *v_new,
                               double *out, int64_t sink, int64_t window,
                               int threads)
{
    if (sink < 0 || window < 0) return -1;
    if (L <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || B <= 0 || T_cap <= 0 ||
        Hq % Hkv != 0)
        return -1;
    int32_t *kv_slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)L * 3);
    if (!kv_slot) return -1;
    int32_t *self_visible = kv_slot + L, *producer = kv_slot + 2 * L;
    int32_t n_slots = 0;
    if (lckv_oracle_pairing(L, warm, rule, kv_slot, self_visible, producer,
                            &n_slots) != 0) {
        free(kv_slot);
        return -1;
    }
    for (int b = 0; b < B; ++b)
        if (lens[b] < 0 || lens[b] >= T_cap) { free(kv_slot); return -2; }

    const int G = Hq / Hkv;
    const int64_t row = (int64_t)Hkv * D;      /* floats per cached position */
    const int64_t seq = T_cap * row;           /* floats per sequence        */
    const int64_t slot_sz = (int64_t)B * seq;  /* floats per slot            */
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
    used = threads;
#endif

    for (int l = 0; l < L; ++l) {
        /* append: bits copied unchanged */
        for (int s = 0; s < n_slots; ++s) {
            if (producer[s] != l) continue;
            for (int b = 0; b < B; ++b) {
                int64_t dst = s * slot_sz + b * seq + (int64_t)lens[b] * row;
                int64_t src = ((int64_t)s * B + b) * row;
                memcpy(Kc + dst, k_new + src, sizeof(float) * (size_t)row);
                memcpy(Vc + dst, v_new + src, sizeof(float) * (size_t)row);
            }
        }
        const int s = kv_slot[l];
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
        for (int bh = 0; bh < B * Hq; ++bh) {
            int b = bh / Hq, h = bh % Hq, g = h / G;
            int64_t n = (int64_t)lens[b] + (self_visible[l] ? 1 : 0);
            int64_t base = s * slot_sz + b * seq + (int64_t)g * D;
            int64_t qo = (((int64_t)l * B + b) * Hq + h) * D;
            if (window > 0 && n > sink + window) {
                /* kept set: positions [0, sink) and [n - window, n) */
                int64_t kept = sink + window;
                float *Kk = (float *)malloc(sizeof(float) * (size_t)(kept * D) * 2);
                float *Vk = Kk + kept * D;
                for (int64_t i = 0; i < kept; ++i) {
                    int64_t j = i < sink ? i : n - window + (i - sink);
                    memcpy(Kk + i * D, Kc + base + j * row, sizeof(float) * (size_t)D);
                    memcpy(Vk + i * D, Vc + base + j * row, sizeof(float) * (size_t)D);
                }
                lckv_oracle_attend(q + qo, Kk, Vk, kept, D, D, scale, out + qo, NULL);
                free(Kk);
                continue;
            }
            lckv_oracle_attend(q + qo, Kc + base, Vc + base, n, row, D, scale,
                               out + qo, NULL);
        }
    }
    for (int b = 0; b < B; ++b) lens[b] += 1;
    free(kv_slot);
    return used;
}

/* The step without the sink + window policy: every cached position is kept. */
int lckv_oracle_step(int L, int Hq, int Hkv, int D, int B, int64_t T_cap,
                     const uint8_t *warm, int rule, double scale, float *Kc,
                     float *Vc, int32_t *lens, const float *q,
                     const float *k_new, const float *v_new, double *out,
                     int threads)
{
    return lckv_oracle_step_streaming(L, Hq, Hkv, D, B, T_cap, warm, rule,
                                      scale, Kc, Vc, lens, q, k_new, v_new,
                                      out, 0, 0, threads);
}

/*
 * Attention of ALL prompt tokens of one layer in one pass, as used by the
 * parallel computation graph of Section 2.2 and by the iterative prompt
 * encoding of Section 2.3: token i of sequence b attends to the K/V at
 * positions j < i of the slot it is paired with (condensed layer: the
 * diagonal is masked, the K/V are the top layer's from the PREVIOUS iteration)
 * or j <= i (warmup layer: standard causal attention on this iteration's own
 * K/V).  Token 0 of a condensed layer has nothing to attend to: zero output
 * (zero dummy K/V).  Rows i >= lens[b] are zero.
 *
 *   Kc, Vc  one slot, [B][T_cap][Hkv][D] float, positions 0..lens[b]-1 filled
 *   q       [B][S][Hq][D],   out  [B][S][Hq][D] double
 * Returns the thread count used, or -1 on a bad argument.
 */
int lckv_oracle_prefill_attention(int Hq, int Hkv, int D, int B, int64_t S,
                                  int64_t T_cap, const float *Kc,
                                  const float *Vc, const int32_t *lens,
                                  int self_visible, double scale,
                                  const float *q, double *out, int threads)
{
    if (Hq <= 0 || Hkv <= 0 || D <= 0 || B <= 0 || S <= 0 || T_cap < S ||
        Hq % Hkv != 0)
        return -1;
    for (int b = 0; b < B; ++b)
        if (lens[b] < 0 || lens[b] > S) return -1;
    const int G = Hq / Hkv;
    const int64_t row = (int64_t)Hkv * D;
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
    used = threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
    for (int64_t bi = 0; bi < (int64_t)B * S; ++bi) {
        int b = (int)(bi / S);
        int64_t i = bi % S;
        for (int h = 0; h < Hq; ++h) {
            double *o = out + ((bi * Hq) + h) * D;
            if (i >= lens[b]) {
                for (int d = 0; d < D; ++d) o[d] = 0.0;
                continue;
            }
            int64_t n = i + (self_visible ? 1 : 0);
            int64_t base = (int64_t)b * T_cap * row + (int64_t)(h / G) * D;
            lckv_oracle_attend(q + ((bi * Hq) + h) * D, Kc + base, Vc + base,
                               n, row, D, scale, o, NULL);
        }
    }
    return used;
}

/*
 * The projections either side of the attention.  Section 2.1: a layer whose
 * K/V nobody reads does not compute them and has no W_K, W_V at all - only the
 * layers that PRODUCE a cache slot (warmup layers and the one condensed layer
 * that owns the shared cache, see lckv_oracle_pairing) map the hidden state to
 * keys and values; every layer maps it to queries.  This function is the map
 * itself, for one weight matrix:
 *     y[b][n] = sum_c x[b][c] * W[n][c]            (W is [N][hidden], N = n_heads*D)
 * followed, when pos != NULL (queries and keys; never values), by the rotary
 * position embedding in the convention of the Llama models the paper trains
 * (the paper itself does not restate it): within each head, channel i < D/2 is
 * paired with channel i + D/2 and the pair is rotated by the angle
 *     pos[b] * base^(-2i/D).
 *   x [B][hidden] float, W [N][hidden] float, pos [B] or NULL, out [B][N] double
 * Returns 0, or -1 on a bad argument.
 */
int lckv_oracle_project(int B, int hidden, int n_heads, int D, const float *x,
                        const float *W, const int64_t *pos, double rope_base,
                        double *out)
{
    if (B < 0 || hidden < 1 || n_heads < 1 || D < 2 || (D & 1) || !x || !W || !out)
        return -1;
    if (pos && !(rope_base > 0.0))
        return -1;
    const int64_t N = (int64_t)n_heads * D;
    for (int b = 0; b < B; ++b) {
        double *y = out + (int64_t)b * N;
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int c = 0; c < hidden; ++c)
                acc += (double)x[(int64_t)b * hidden + c] * (double)W[n * hidden + c];
            y[n] = acc;
        }
        if (!pos)
            continue;
        for (int h = 0; h < n_heads; ++h) {
            double *v = y + (int64_t)h * D;
            for (int i = 0; i < D / 2; ++i) {
                const double angle = (double)pos[b] * pow(rope_base, -2.0 * i / D);
                const double c = cos(angle), s = sin(angle);
                const double lo = v[i], hi = v[i + D / 2];
                v[i] = lo * c - hi * s;
                v[i + D / 2] = hi * c + lo * s;
            }
        }
    }
    return 0;
}

/*
 * Bytes of KV cache for B sequences of T positions (Section 1: the KV cache
 * grows with the sequence length and with the number of layers that keep
 * one; Section 2.1: here only the top layer and the warmup layers keep one).
 * Counted the long way: every cache named by the pairing table holds, per
 * sequence and position, one key and one value of D elements for each of its
 * Hkv heads.  Returns -1 on a bad argument.
 */
int64_t lckv_oracle_footprint(int L, const uint8_t *warm, int rule, int64_t B,
                              int64_t T, int Hkv, int D, int elem_bytes)
{
    if (L <= 0 || B < 0 || T < 0 || Hkv <= 0 || D <= 0 || elem_bytes <= 0)
        return -1;
    int32_t *kv_slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)L * 3);
    if (!kv_slot) return -1;
    int32_t n_slots = 0;
    if (lckv_oracle_pairing(L, warm, rule, kv_slot, kv_slot + L, kv_slot + 2 * L,
                            &n_slots) != 0) {
        free(kv_slot);
        return -1;
    }
    free(kv_slot);
    int64_t bytes = 0;
    for (int s = 0; s < n_slots; ++s)          /* every cache that is kept    */
        for (int64_t b = 0; b < B; ++b)        /* every sequence              */
            bytes += T * (int64_t)Hkv * D * elem_bytes   /* its keys          */
                   + T * (int64_t)Hkv * D * elem_bytes;  /* and its values    */
    return bytes;
}

/*
 * The largest batch whose caches fit in `budget` bytes (Section 3.1: the
 * maximum batch size is what the memory allows), found by trying batch sizes
 * upward; at most `limit` sequences.  Returns -1 on a bad argument.
 */
int64_t lckv_oracle_max_batch(int L, const uint8_t *warm, int rule, int64_t T,
                              int Hkv, int D, int elem_bytes, int64_t budget,
                              int64_t limit)
{
    if (budget < 0 || limit < 0) return -1;
    if (lckv_oracle_footprint(L, warm, rule, 0, T, Hkv, D, elem_bytes) < 0)
        return -1;
    int64_t B = 0;
    while (B < limit &&
           lckv_oracle_footprint(L, warm, rule, B + 1, T, Hkv, D, elem_bytes) <= budget)
        ++B;
    return B;
}

int lckv_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
