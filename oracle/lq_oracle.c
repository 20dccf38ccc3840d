/*
 * CPU oracle for the segmented multi-adapter LoRA update (the operation the paper's SMLM
 * kernel performs for one linear layer over one mixed batch, Section 3.3), its segment
 * metadata, and the gradient of that update.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, per-token fp64 implementation of the
 * definition and is only ever called by the tests, the smoke check and the benchmark's
 * CPU-baseline leg.  It shares no code with the GPU library and the GPU library never
 * calls it.
 *
 * What is computed (LoRA, cited in Section 1; batched over adapters as in Section 3.3):
 *   for every token t whose adapter a = token_adapter[t] is valid
 *       h[j]   = sum_k x[t,k] * A_a[j,k]                      j < r_a      (A_a is [r_a, d_in])
 *       y[t,n] = y0[t,n] + s_a * sum_j h[j] * B_a[j,n]        n < d_out    (B_a is [r_a, d_out])
 *   fine-tuning tokens additionally keep the unscaled h (what autograd would keep for the
 *   backward pass, Section 3.3); tokens without a valid adapter keep y0.
 *   Scale (Section 3.3 names two modes): the static per-adapter s_a above, or a dynamic scale
 *   "applied on a per-request basis during the forward pass".  The reading taken: an optional
 *   per-token array token_scale (all tokens of a request carry the request's value) that, when
 *   given, REPLACES s_a for every token:  y[t,n] = y0[t,n] + token_scale[t] * sum_j h[j] B_a[j,n].
 *
 * Pins (tests/test_oracle_pins.py): B = 0, single adapter vs. a dense fp64 matmul, rank-1
 * outer product, token-permutation invariance, exact rational brute force on tiny shapes,
 * linearity in the scale, central differences for the gradient, a hand-written expected
 * segment table and a library stable sort for the metadata; the per-token scale by the dense
 * form with a diagonal matrix, by row-wise linearity, by its agreement with the per-adapter
 * scale when the values coincide, and by exact differences; the row split / concatenation by
 * hand-built row sets; the dropout mask by its drop rates (overall, per row, per column), by the
 * absence of correlation between columns, rows and seeds, and by what it must leave untouched.
 * The individual BITS of the dropout mask have no outside reference (the paper fixes no
 * generator, the mask is a contract of this code base): for them, parity unpinned.  No other
 * function here is unpinned.
 *
 * Inputs are bfloat16 bit patterns (uint16) decoded here, independently of any other code.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { LQO_FINETUNE = 0, LQO_PREFILL = 1, LQO_DECODE = 2 };

static double bf16_decode(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static int token_is_live(int32_t adapter, uint8_t kind, int32_t n_adapters)
{
    return adapter >= 0 && adapter < n_adapters && kind <= LQO_DECODE;
}

/* ------------------------------------------------------------------------------------------
 * Segment metadata.  The batch is ordered fine-tune | prefill+evaluation | decode (Algorithm 1
 * computes its offsets from that order); inside a kind, tokens are grouped by adapter.  The
 * reading taken here: stable sort of the live token indices by (kind, adapter), one segment
 * per distinct key, h offsets = running sum of len * rank over fine-tune segments.
 * Written as a library sort of (key, token index) pairs, the index breaking ties.
 * ------------------------------------------------------------------------------------------ */
typedef struct { int64_t key; int32_t index; } lqo_item;

static int item_cmp(const void* pa, const void* pb)
{
    const lqo_item* a = (const lqo_item*)pa;
    const lqo_item* b = (const lqo_item*)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    return a->index < b->index ? -1 : (a->index > b->index ? 1 : 0); /* ties keep token order */
}

/* Outputs must hold: perm[n_tokens], seg_starts[n_tokens+1], seg_adapter[n_tokens],
 * seg_kind[n_tokens], h_offsets[n_tokens+1].  Returns the number of segments. */
int32_t lq_oracle_build_segments(const int32_t* token_adapter, const uint8_t* token_kind, int32_t n_tokens,
                                 const int32_t* ranks, int32_t n_adapters,
                                 int32_t* perm, int32_t* seg_starts, int32_t* seg_adapter, uint8_t* seg_kind,
                                 int64_t* h_offsets)
{
    lqo_item* items = (lqo_item*)malloc(sizeof(lqo_item) * (size_t)(n_tokens > 0 ? n_tokens : 1));
    int32_t n_live = 0;
    for (int32_t t = 0; t < n_tokens; ++t) {
        if (!token_is_live(token_adapter[t], token_kind[t], n_adapters)) continue;
        items[n_live].key = (int64_t)token_kind[t] * ((int64_t)1 << 32) + token_adapter[t];
        items[n_live].index = t;
        ++n_live;
    }
    qsort(items, (size_t)n_live, sizeof(lqo_item), item_cmp);

    int32_t n_seg = 0;
    int64_t h_off = 0;
    seg_starts[0] = 0;
    h_offsets[0] = 0;
    for (int32_t p = 0; p < n_live; ++p) {
        perm[p] = items[p].index;
        int last = (p + 1 == n_live) || (items[p + 1].key != items[p].key);
        if (last) {
            int32_t a = token_adapter[items[p].index];
            uint8_t kind = token_kind[items[p].index];
            int32_t len = p + 1 - seg_starts[n_seg];
            seg_adapter[n_seg] = a;
            seg_kind[n_seg] = kind;
            if (kind == LQO_FINETUNE) h_off += (int64_t)len * ranks[a];
            ++n_seg;
            seg_starts[n_seg] = p + 1;
            h_offsets[n_seg] = h_off;
        }
    }
    free(items);
    return n_seg;
}

/* ------------------------------------------------------------------------------------------
 * Forward.  y_ref is [n_tokens, d_out] fp64 (dense, leading dimension d_out); h_ref receives
 * the unscaled h rows of fine-tune tokens at the element offsets the metadata defines
 * (segment's h offset + row-in-segment * rank); token_h_offset[t] is that offset or -1 and
 * is computed by the caller from lq_oracle_build_segments.  The numerics never look at the
 * segment tables: each token is handled on its own from (adapter, kind).
 * ------------------------------------------------------------------------------------------ */
void lq_oracle_forward(const uint16_t* x, int64_t ldx, const uint16_t* y0, int64_t ldy,
                       int32_t n_tokens, int32_t d_in, int32_t d_out,
                       const uint16_t* const* A, const uint16_t* const* B,
                       const int32_t* ranks, const float* scales, int32_t n_adapters,
                       const int32_t* token_adapter, const uint8_t* token_kind,
                       const int64_t* token_h_offset, const float* token_scale /* NULL: per-adapter scales */,
                       double* y_ref, double* h_ref)
{
#pragma omp parallel
    {
        int32_t max_rank = 1;
        for (int32_t a = 0; a < n_adapters; ++a) if (ranks[a] > max_rank) max_rank = ranks[a];
        double* h = (double*)malloc(sizeof(double) * (size_t)max_rank);
#pragma omp for schedule(static)
        for (int32_t t = 0; t < n_tokens; ++t) {
            const uint16_t* xt = x + (int64_t)t * ldx;
            const uint16_t* y0t = y0 + (int64_t)t * ldy;
            double* yt = y_ref + (int64_t)t * d_out;
            int32_t a = token_adapter[t];
            if (!token_is_live(a, token_kind[t], n_adapters)) {
                for (int32_t n = 0; n < d_out; ++n) yt[n] = bf16_decode(y0t[n]);
                continue;
            }
            int32_t r = ranks[a];
            double s = token_scale ? (double)token_scale[t] : (double)scales[a];
            for (int32_t j = 0; j < r; ++j) {
                const uint16_t* Aj = A[a] + (int64_t)j * d_in;
                double acc = 0.0;
                for (int32_t k = 0; k < d_in; ++k) acc += bf16_decode(xt[k]) * bf16_decode(Aj[k]);
                h[j] = acc;
            }
            if (token_kind[t] == LQO_FINETUNE && token_h_offset && token_h_offset[t] >= 0 && h_ref)
                for (int32_t j = 0; j < r; ++j) h_ref[token_h_offset[t] + j] = h[j];
            for (int32_t n = 0; n < d_out; ++n) {
                double acc = 0.0;
                for (int32_t j = 0; j < r; ++j) acc += h[j] * bf16_decode(B[a][(int64_t)j * d_out + n]);
                yt[n] = bf16_decode(y0t[n]) + s * acc;
            }
        }
        free(h);
    }
}

/* ------------------------------------------------------------------------------------------
 * Backward of the update above for fine-tune tokens, i.e. the exact gradient of
 * L = sum_{t,n} dy[t,n] * y[t,n] with respect to B_a, A_a and x (what autograd computes for
 * the LoRA linears in the paper, Section 3.3 / Section 4.2):
 *     g[t,j]   = sum_n dy[t,n] * B_a[j,n]
 *     dB_a[j,n] += s_a * sum_t h[t,j] * dy[t,n]          (h recomputed here in fp64)
 *     dA_a[j,k] += s_a * sum_t g[t,j] * x[t,k]
 *     dx[t,k]   = dx0[t,k] + s_a * sum_j g[t,j] * A_a[j,k]
 * (with a per-token scale, s_a becomes token_scale[t] and moves inside the sums over t)
 * dA[a] is [r_a, d_in] fp64, dB[a] is [r_a, d_out] fp64, both accumulated into (caller zeroes);
 * dx_ref is [n_tokens, d_in] fp64 and receives dx0 (bf16) plus the update; rows of other
 * kinds receive dx0 unchanged.  g_ref (optional) receives g at the same offsets as h.
 * Each weight-gradient element sums its tokens in batch order, so the result is deterministic.
 * ------------------------------------------------------------------------------------------ */
void lq_oracle_backward(const uint16_t* x, int64_t ldx, const uint16_t* dy, int64_t lddy,
                        const uint16_t* dx0, int64_t lddx,
                        int32_t n_tokens, int32_t d_in, int32_t d_out,
                        const uint16_t* const* A, const uint16_t* const* B,
                        const int32_t* ranks, const float* scales, int32_t n_adapters,
                        const int32_t* token_adapter, const uint8_t* token_kind,
                        const int64_t* token_h_offset, const float* token_scale /* NULL: per-adapter scales */,
                        double* const* dA, double* const* dB, double* dx_ref, double* g_ref)
{
    int32_t max_rank = 1;
    for (int32_t a = 0; a < n_adapters; ++a) if (ranks[a] > max_rank) max_rank = ranks[a];
    size_t n_rows = (size_t)(n_tokens > 0 ? n_tokens : 1);
    double* h_all = (double*)calloc(n_rows * (size_t)max_rank, sizeof(double));
    double* g_all = (double*)calloc(n_rows * (size_t)max_rank, sizeof(double));

    /* per token: h, g and the dx row (tokens are independent here) */
#pragma omp parallel for schedule(static)
    for (int32_t t = 0; t < n_tokens; ++t) {
        const uint16_t* xt = x + (int64_t)t * ldx;
        const uint16_t* dyt = dy + (int64_t)t * lddy;
        double* dxt = dx_ref + (int64_t)t * d_in;
        double* h = h_all + (size_t)t * max_rank;
        double* g = g_all + (size_t)t * max_rank;
        for (int32_t k = 0; k < d_in; ++k) dxt[k] = dx0 ? bf16_decode(dx0[(int64_t)t * lddx + k]) : 0.0;
        int32_t a = token_adapter[t];
        if (!token_is_live(a, token_kind[t], n_adapters) || token_kind[t] != LQO_FINETUNE) continue;
        int32_t r = ranks[a];
        double s = token_scale ? (double)token_scale[t] : (double)scales[a];
        for (int32_t j = 0; j < r; ++j) {
            double acc_h = 0.0, acc_g = 0.0;
            for (int32_t k = 0; k < d_in; ++k) acc_h += bf16_decode(xt[k]) * bf16_decode(A[a][(int64_t)j * d_in + k]);
            for (int32_t n = 0; n < d_out; ++n) acc_g += bf16_decode(dyt[n]) * bf16_decode(B[a][(int64_t)j * d_out + n]);
            h[j] = acc_h;
            g[j] = acc_g;
        }
        if (g_ref && token_h_offset && token_h_offset[t] >= 0)
            for (int32_t j = 0; j < r; ++j) g_ref[token_h_offset[t] + j] = g[j];
        for (int32_t k = 0; k < d_in; ++k) {
            double acc = 0.0;
            for (int32_t j = 0; j < r; ++j) acc += g[j] * bf16_decode(A[a][(int64_t)j * d_in + k]);
            dxt[k] += s * acc;
        }
    }

    /* weight gradients: one row (a, j) at a time, tokens summed in their natural order */
    for (int32_t a = 0; a < n_adapters; ++a) {
        int32_t r = ranks[a];
#pragma omp parallel for schedule(static)
        for (int32_t j = 0; j < r; ++j) {
            double* dBj = dB[a] + (int64_t)j * d_out;
            double* dAj = dA[a] + (int64_t)j * d_in;
            for (int32_t t = 0; t < n_tokens; ++t) {
                if (token_adapter[t] != a || token_kind[t] != LQO_FINETUNE) continue;
                const uint16_t* xt = x + (int64_t)t * ldx;
                const uint16_t* dyt = dy + (int64_t)t * lddy;
                double s = token_scale ? (double)token_scale[t] : (double)scales[a];
                double hj = h_all[(size_t)t * max_rank + j];
                double gj = g_all[(size_t)t * max_rank + j];
                for (int32_t n = 0; n < d_out; ++n) dBj[n] += s * hj * bf16_decode(dyt[n]);
                for (int32_t k = 0; k < d_in; ++k) dAj[k] += s * gj * bf16_decode(xt[k]);
            }
        }
    }
    free(h_all);
    free(g_all);
}

int32_t lq_oracle_num_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------
 * LoRA dropout on the fine-tuning rows and the row split / concatenation of Algorithm 1.
 *
 * Dropout.  The paper's training configurations use LoRA dropout 0.05 (Appendix, LoRA
 * configuration tables): in the LoRA branch of a fine-tuning token the input x is replaced by
 * m * x / (1 - p), where the elements of m are independent and 1 with probability 1 - p.  The
 * paper fixes no generator, so the draw is a CONTRACT of this library (both sides implement
 * it): m[t,k] depends only on (seed, token row t, column k), through the 32-bit integer hash
 * of Jarzynski and Olano ("Hash Functions for GPU Rendering", JCGT 2020: one step of a linear
 * congruential generator followed by the PCG output permutation):
 *     hash(v)   = let s = v * 747796405 + 2891336453,
 *                     w = ((s >> ((s >> 28) + 4)) ^ s) * 277803737  in  (w >> 22) ^ w
 *     key(t)    = hash(seed ^ hash(t))
 *     word(t,q) = hash(key(t) + q)                 one word per pair of columns, q = k / 2
 *     field     = low 16 bits of word for even k, high 16 bits for odd k
 *     m[t,k]    = field >= threshold,   threshold = (uint32)(p * 65536 + 0.5) in fp32   (p in steps of 2^-16)
 * The factor 1 / (1 - p) is NOT applied to x (m * x is exact in bf16, x / (1 - p) is not): it
 * travels with the scale, s' = s / (1 - p) for the token (the per-token scale above), so the
 * saved h of a fine-tuning token is (m * x) A.  The gradient with respect to x through the LoRA
 * branch is m * (s' g A): the same mask applied to the rows of dx.
 * What the mathematics fixes, and the pins check: keep rate 1 - p, independence across
 * columns, rows and seeds; rows that are not fine-tuning rows are copied unchanged.
 * ------------------------------------------------------------------------------------------ */
static uint32_t lqo_hash(uint32_t v)
{
    uint32_t s = v * 747796405u + 2891336453u;
    uint32_t w = ((s >> ((s >> 28) + 4u)) ^ s) * 277803737u;
    return (w >> 22) ^ w;
}

int32_t lq_oracle_dropout_keep(uint32_t seed, int32_t t, int32_t k, uint32_t threshold)
{
    uint32_t key = lqo_hash(seed ^ lqo_hash((uint32_t)t));
    uint32_t word = lqo_hash(key + (uint32_t)(k >> 1));
    uint32_t field = (k & 1) ? (word >> 16) : (word & 0xffffu);
    return field >= threshold;
}

/* out[t,:] = m[t,:] * in[t,:] for live fine-tuning tokens, in[t,:] for every other token (bf16 bit patterns). */
void lq_oracle_dropout_rows(const uint16_t* in, int64_t ld_in, uint16_t* out, int64_t ld_out,
                            int32_t n_tokens, int32_t d, const int32_t* token_adapter, const uint8_t* token_kind,
                            int32_t n_adapters, uint32_t seed, uint32_t threshold)
{
    for (int32_t t = 0; t < n_tokens; ++t) {
        int ft = token_is_live(token_adapter[t], token_kind[t], n_adapters) && token_kind[t] == LQO_FINETUNE;
        for (int32_t k = 0; k < d; ++k) {
            uint16_t v = in[(int64_t)t * ld_in + k];
            out[(int64_t)t * ld_out + k] = (!ft || lq_oracle_dropout_keep(seed, t, k, threshold)) ? v : 0;
        }
    }
}

/* Row split of Algorithm 1: the attention layer takes the fine-tuning rows, the prefill (and
 * evaluation) rows and the decode rows out of Q, K, V by offsets that follow from the batch
 * order fine-tune | prefill | decode, runs a different attention implementation on each, and
 * concatenates the outputs again.  With the segment tables the rows of kind c are
 * perm[kind_offsets[c] .. kind_offsets[c+1]) (kind_offsets = where the segments of each kind
 * start in the segment order: Algorithm 1's Offset_p and Offset_d), so
 *     split :  part_c[i, :] = src[perm[kind_offsets[c] + i], :]
 *     concat:  dst[perm[kind_offsets[c] + i], :] = part_c[i, :]      (rows without adapter untouched)
 * kind_offsets has 4 entries; parts is the three parts back to back ([n_live, d]). */
void lq_oracle_kind_offsets(const int32_t* seg_starts, const uint8_t* seg_kind, int32_t n_segments, int32_t* kind_offsets)
{
    /* kind c starts at the first segment whose kind is >= c (the segments are ordered by kind), or at the end */
    for (int c = 0; c <= 3; ++c) {
        kind_offsets[c] = seg_starts[n_segments];
        for (int32_t s = n_segments - 1; s >= 0; --s)
            if (seg_kind[s] >= c) kind_offsets[c] = seg_starts[s];
    }
}

void lq_oracle_split_rows(const uint16_t* src, int64_t ld, int32_t d, const int32_t* perm, int32_t n_live, uint16_t* parts)
{
    for (int32_t i = 0; i < n_live; ++i)
        for (int32_t k = 0; k < d; ++k) parts[(int64_t)i * d + k] = src[(int64_t)perm[i] * ld + k];
}

void lq_oracle_concat_rows(const uint16_t* parts, int32_t d, const int32_t* perm, int32_t n_live, uint16_t* dst, int64_t ld)
{
    for (int32_t i = 0; i < n_live; ++i)
        for (int32_t k = 0; k < d; ++k) dst[(int64_t)perm[i] * ld + k] = parts[(int64_t)i * d + k];
}
