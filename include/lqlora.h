/*
 * lqlora — segmented multi-adapter LoRA forward/backward for AMD MI355X (gfx950), C ABI.
 *
 * The operation is the one the paper's SMLM kernel ("Segmented Multi-LoRA Multiplication",
 * Section 1 and Section 3.3) performs for ONE linear layer over ONE mixed batch: all
 * (token segment, adapter) LoRA products in one call, with fine-tuning, evaluation/prefill
 * and decode requests in the same batch, adapters kept as separate per-layer tensors
 * (never concatenated, so a pointer can be swapped at run time), and a run-time scale:
 *
 *     for every segment g with adapter a, rank r_a, scale s_a and token rows R_g:
 *         h[t, :]  = x[t, :] * A_a^T                     t in R_g      (A_a is [r_a, d_in])
 *         y[t, :] += s_a * h[t, :] * B_a                 t in R_g      (B_a is [r_a, d_out])
 *         fine-tune segments also store the unscaled h rows (fp32) for the backward pass.
 *
 * Conventions for every entry point
 *   - Every pointer is a DEVICE pointer (HBM) unless its name starts with host_.  The
 *     library never allocates, frees or synchronises: each call validates its host scalars,
 *     enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = the null stream)
 *     and returns.  The caller owns all buffers, including the workspace, and must keep
 *     them alive until the stream has passed the call.
 *   - bf16 tensors are row-major with an explicit leading dimension in ELEMENTS; base
 *     pointers must be 16-byte aligned and d_in, d_out and the leading dimensions must be
 *     multiples of 8 (else LQ_ERR_UNSUPPORTED).  Adapter matrices are dense row-major,
 *     16-byte aligned.  Ranks 1..LQ_MAX_RANK are supported, different per adapter.
 *   - Errors are return codes; nothing throws or aborts.  Host-side validation returns
 *     before anything is launched.  Metadata that only the device can see (adapter id out
 *     of range, rank out of range) never causes an out-of-bounds access: the segment is
 *     skipped and bit 0 of the int32 at workspace offset 0 is set (the caller may zero and
 *     read that word; the library only ever ORs into it).  Bit 1 reports that the fused
 *     variant's bounded device-wide wait timed out (its results are then incomplete).
 *   - x and y must not alias.  Rows of y that no segment covers are untouched bit for bit.
 *   - Calls on different streams that share a workspace race; give each stream its own.
 */
#ifndef LQLORA_H
#define LQLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LQ_OK = 0,
    LQ_ERR_INVALID_ARG = 1, /* null pointer, negative size, ld < d, unknown variant */
    LQ_ERR_UNSUPPORTED = 2, /* alignment / multiple-of-8 / rank or adapter-count limits */
    LQ_ERR_WORKSPACE = 3,   /* workspace missing or smaller than the *_workspace_bytes answer */
    LQ_ERR_HIP = 4          /* a HIP launch reported an error */
} lq_status;

/* Request kinds (Section 3.3: fine-tuning, evaluation, prefilling, decoding; evaluation is
 * structurally a prefill, so it shares LQ_SEG_PREFILL).  The numeric order is the batch
 * order of Algorithm 1: fine-tune | prefill+evaluation | decode. */
enum { LQ_SEG_FINETUNE = 0, LQ_SEG_PREFILL = 1, LQ_SEG_DECODE = 2 };

/* LQ_VARIANT_SPLIT: shrink kernel then expand kernel.  LQ_VARIANT_FUSED: one launch whose workgroups
 * meet at a device-wide barrier between the two phases: it needs all of them resident at once, so the
 * device must not be shared with other kernels while it runs (on another stream, say); if they are not,
 * the bounded wait times out, bit 1 of the workspace error word is set and y is incomplete.  The backward
 * call uses the same kind of launch for its first two steps.
 * LQ_VARIANT_SHRINK_ONLY / LQ_VARIANT_EXPAND_ONLY: the two halves of the split variant as separate
 * calls (same arguments, same workspace, shrink first), for callers that put other work between
 * them and for timing each kernel on its own.
 * LQ_VARIANT_SLAB: one launch in which every workgroup takes a slab of at most 32 rows of one segment
 * through both products, so that h stays on the compute unit: no partial-h traffic and no device-wide wait
 * (hence no residency requirement); every slab re-reads its adapter's matrices, which come from the L2 cache
 * when slabs of one segment run side by side.  The faster variant on batches whose segments are long compared
 * with the adapters' rank (fine-tuning and prefill rows); same results up to fp32 summation order.
 * LQ_VARIANT_AUTO: the library picks between the slab and the fused variant from the host arguments alone (a pure
 * function of max_rank and the output widths): slab for ranks up to 32 and up to 16384 output columns in all,
 * fused otherwise (wide outputs, where re-reading B per slab costs more than the partial-h round trip; and
 * larger ranks).  Where it picks fused, that variant's residency requirement applies. */
enum { LQ_VARIANT_SPLIT = 0, LQ_VARIANT_FUSED = 1, LQ_VARIANT_SHRINK_ONLY = 2, LQ_VARIANT_EXPAND_ONLY = 3,
       LQ_VARIANT_SLAB = 4, LQ_VARIANT_AUTO = 5 };

#define LQ_MAX_RANK 128
#define LQ_MAX_GROUP 4      /* linear layers per grouped call */
#define LQ_MAX_ADAPTERS 4096

const char* lora_status_string(lq_status status);

/* One size that serves every call of this header on a batch of these dimensions (the largest of
 * lora_build_workspace_bytes, lora_forward_workspace_bytes for every variant, and
 * lora_backward_workspace_bytes): a caller that keeps one workspace per stream needs nothing else.
 * The per-call sizers below give the exact requirement of each call. */
size_t lora_workspace_bytes(int32_t n_tokens, int32_t n_adapters, int32_t max_rank, int32_t d_in, int32_t d_out);

/* ---------------------------------------------------------------------------------------------
 * Segment metadata builder (integer only, deterministic, bit-exact).
 *
 * Turns per-token (adapter, kind) into the segment tables the forward consumes.  The paper only
 * fixes the batch order fine-tune | prefill+evaluation | decode (Algorithm 1 derives its offsets
 * from it); the tables are that order refined by adapter: a STABLE sort of token indices by
 * (kind, adapter), one segment per distinct key, ties in original token order.  Tokens whose
 * adapter id is outside [0, n_adapters) (use -1 for base-model-only requests) or whose kind is
 * not one of the three are left out of perm.
 *
 *   in   token_adapter int32[n_tokens], token_kind uint8[n_tokens], ranks int32[n_adapters]
 *   out  perm        int32[n_tokens]       token indices in segment order (first seg_starts[n_seg] valid)
 *        seg_starts  int32[max_segments+1] positions in perm; seg_starts[n_seg] = number of live tokens
 *        seg_adapter int32[max_segments]
 *        seg_kind    uint8[max_segments]
 *        h_offsets   int64[max_segments+1] element offset of each segment's saved h in h_out:
 *                                          running sum of len * rank over fine-tune segments
 *        n_segments  int32[1]              device scalar
 *   max_segments must be >= min(n_tokens, 3 * n_adapters).  n_tokens = 0 is valid (n_segments = 0).
 *   workspace: lora_build_workspace_bytes(n_tokens, n_adapters) bytes; its first 4096 bytes must be ZERO
 *            before the first call that uses it (batches of 2048 tokens and more are built by several
 *            workgroups that meet at a device-wide barrier, see LQ_VARIANT_FUSED for what that needs; its
 *            words are left at zero); the rest may hold anything.  May be NULL for up to 312 adapters:
 *            then one workgroup builds the tables, whatever the batch size.
 * ------------------------------------------------------------------------------------------- */
size_t lora_build_workspace_bytes(int32_t n_tokens, int32_t n_adapters);

lq_status lora_build_segments(const int32_t* token_adapter, const uint8_t* token_kind, int32_t n_tokens,
                              const int32_t* ranks, int32_t n_adapters,
                              int32_t* perm, int32_t* seg_starts, int32_t* seg_adapter, uint8_t* seg_kind,
                              int64_t* h_offsets, int32_t* n_segments, int32_t max_segments,
                              void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Forward (Section 3.3; formula above).
 *
 *   x        bf16 [n_tokens, d_in], leading dimension ldx          (read only)
 *   y        bf16 [n_tokens, d_out], leading dimension ldy         (read-modify-write, one rounding
 *                                                                   to nearest even per call)
 *   A_ptrs   [n_adapters] device array of device pointers to bf16 [r_a, d_in]
 *   B_ptrs   [n_adapters] device array of device pointers to bf16 [r_a, d_out]
 *   ranks    int32[n_adapters], scales float[n_adapters] (applied in fp32 to h * B before the add)
 *   token_scales  float[n_tokens] or NULL.  Section 3.3 names two scale modes: static (folded into the
 *            weights at load, or scales[a] here) and dynamic, "applied on a per-request basis during the
 *            forward pass".  When given, token_scales[t] REPLACES scales[adapter] for token row t (every
 *            token of a request carries the request's value; requests that share an adapter may differ);
 *            the saved h stays unscaled.  NULL: the per-adapter scales.
 *   max_rank host scalar >= every rank in use (sizes the h scratch); <= LQ_MAX_RANK
 *   perm     int32, row of x / y for each position of the segment order; NULL = identity
 *   seg_*    as produced by lora_build_segments (or by the caller); n_segments is a device scalar,
 *            max_segments the capacity of the tables (bounds the launch grid)
 *   h_out    float, receives the UNSCALED h rows of fine-tune segments, segment g at
 *            h_out + h_offsets[g], row-major [len_g, r_a]; h_out / h_offsets may be NULL, then
 *            nothing is saved (inference-only batches)
 *   variant  one of LQ_VARIANT_*; split, fused and slab give the same y and h_out up to fp32 summation
 *            order; h_out may be written by either half of the split variant
 *            (LQ_VARIANT_FUSED: LQ_ERR_UNSUPPORTED if the workspace's partial-h region would reach 2 GiB,
 *            i.e. beyond about 4 million tokens at rank 128)
 *   workspace lora_forward_workspace_bytes(...) bytes; its first 4096 bytes must be ZERO before the first
 *            call that uses it (error word, which the library only ORs into, and work counters that
 *            every launch leaves at zero); the rest may hold anything.  n_tokens = 0 returns LQ_OK
 *            with no launch.
 * ------------------------------------------------------------------------------------------- */
size_t lora_forward_workspace_bytes(int32_t n_tokens, int32_t max_rank, int32_t d_in, int32_t d_out,
                                    int32_t variant);

lq_status lora_segmented_forward(const void* x, int64_t ldx, void* y, int64_t ldy,
                                 int32_t d_in, int32_t d_out,
                                 const void* const* A_ptrs, const void* const* B_ptrs,
                                 const int32_t* ranks, const float* scales, const float* token_scales,
                                 int32_t n_adapters, int32_t max_rank,
                                 const int32_t* perm, int32_t n_tokens,
                                 const int32_t* seg_starts, const int32_t* seg_adapter, const uint8_t* seg_kind,
                                 const int32_t* n_segments, int32_t max_segments,
                                 float* h_out, const int64_t* h_offsets,
                                 int32_t variant, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Grouped forward: n_proj linear layers that read the SAME x in one call, each with its own y,
 * d_out, adapter tables and saved h.  Algorithm 1 computes Q, K and V from one X (and the MLP its
 * gate and up projections from one X); issued as one call they share the pass over x (workgroups
 * that share an L2 take the same rows of different layers side by side) and the launch.  The batch,
 * its tables, ranks, scales and token_scales are common to the layers; adapter a has the same rank in
 * every layer.  The result of every layer is what lora_segmented_forward gives for it alone.
 *
 *   host_y, host_ldy, host_d_out, host_A_ptrs, host_B_ptrs, host_h_out
 *            HOST arrays of n_proj entries (read during the call, not kept): per layer the device
 *            pointer y, its leading dimension, d_out, the device pointer tables A_ptrs / B_ptrs
 *            ([n_adapters] device pointers to bf16 [r_a, d_in] / [r_a, d_out]) and the device pointer
 *            h_out (host_h_out or any of its entries may be NULL: nothing saved)
 *   n_proj   1..LQ_MAX_GROUP; the y of two layers must differ
 *   workspace lora_forward_group_workspace_bytes(n_proj, n_tokens, max_rank) bytes, first 4096 zero
 *            as for the single call
 *   everything else as in lora_segmented_forward.
 * ------------------------------------------------------------------------------------------- */
size_t lora_forward_group_workspace_bytes(int32_t n_proj, int32_t n_tokens, int32_t max_rank);

lq_status lora_segmented_forward_group(const void* x, int64_t ldx, int32_t d_in, int32_t n_proj,
                                       void* const* host_y, const int64_t* host_ldy, const int32_t* host_d_out,
                                       const void* const* const* host_A_ptrs, const void* const* const* host_B_ptrs,
                                       float* const* host_h_out,
                                       const int32_t* ranks, const float* scales, const float* token_scales,
                                       int32_t n_adapters, int32_t max_rank,
                                       const int32_t* perm, int32_t n_tokens,
                                       const int32_t* seg_starts, const int32_t* seg_adapter, const uint8_t* seg_kind,
                                       const int32_t* n_segments, int32_t max_segments,
                                       const int64_t* h_offsets,
                                       int32_t variant, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * The forward for callers that CANNOT ALLOCATE device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * lora_segmented_forward, minus the workspace: the partial-h buffer and the counters live in a
 * device array that belongs to the library (LQ_STATIC_WORKSPACE_BYTES, held by every GPU the
 * library runs on until the process ends).  The call allocates nothing and enqueues only kernels
 * (one small fill kernel that clears the counters, then the forward's).
 *   variant     LQ_VARIANT_SPLIT, LQ_VARIANT_FUSED, LQ_VARIANT_SLAB or LQ_VARIANT_AUTO (else LQ_ERR_INVALID_ARG)
 *   error_word  device int32, may be NULL: receives (ORed in) the bits the workspace's word 0 would;
 *               with NULL those bits are not visible to the caller
 *   LQ_ERR_WORKSPACE if lora_forward_workspace_bytes(n_tokens, max_rank, d_in, d_out, variant) exceeds
 *   LQ_STATIC_WORKSPACE_BYTES (32 MiB of partial h: 8192 tokens at ranks up to 64, 65536 tokens at ranks
 *   up to 32 ...); use the call above with a workspace of your own then.
 *   All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 *   streams, or threads) race; calls on one stream are ordered and safe.
 * ------------------------------------------------------------------------------------------- */
#define LQ_STATIC_WORKSPACE_BYTES (4096 + (32 << 20))

lq_status lora_segmented_forward_static(const void* x, int64_t ldx, void* y, int64_t ldy,
                                        int32_t d_in, int32_t d_out,
                                        const void* const* A_ptrs, const void* const* B_ptrs,
                                        const int32_t* ranks, const float* scales, const float* token_scales,
                                        int32_t n_adapters, int32_t max_rank,
                                        const int32_t* perm, int32_t n_tokens,
                                        const int32_t* seg_starts, const int32_t* seg_adapter, const uint8_t* seg_kind,
                                        const int32_t* n_segments, int32_t max_segments,
                                        float* h_out, const int64_t* h_offsets,
                                        int32_t variant, int32_t* error_word, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Backward of the forward above for FINE-TUNE segments (other kinds are skipped).  The paper
 * leaves this to autograd, one call per LoRA linear, and names a dedicated kernel as future
 * work (Section 4.2, Appendix A).  Exact gradient of the forward as defined here, with
 * g = dy * B_a^T:
 *     dB_a += s_a * h^T dy        dA_a += s_a * g^T x        dx[t, :] += s_a * g[t, :] * A_a
 * (with token_scales, as in the forward, s_a becomes the row's own scale inside the sums over rows)
 *
 *   dy       bf16 [n_tokens, d_out] (rows of fine-tune tokens are read)
 *   dx       bf16 [n_tokens, d_in], read-modify-write on fine-tune rows only (one rounding per call);
 *            must not alias x or dy
 *   h_saved  float, the h_out written by the forward (same h_offsets)
 *   dA_ptrs / dB_ptrs  [n_adapters] device arrays of device pointers to float [r_a, d_in] / [r_a, d_out],
 *            accumulated into (caller zeroes); entries may be NULL (that gradient is skipped), and
 *            either table may be NULL; with both NULL only dx is computed
 *   variant  LQ_VARIANT_FUSED: g and dx in one launch (same residency requirement as the forward's fused
 *            variant; falls back to two launches where the partial-g region would reach 2 GiB);
 *            LQ_VARIANT_SPLIT: two launches, no device-wide wait; LQ_VARIANT_SLAB: g and dx in one launch of the
 *            forward's slab variant, no device-wide wait; LQ_VARIANT_AUTO: slab or fused by the forward's rule
 *            applied to this step (its outputs are the d_in columns of dx).  Other values: LQ_ERR_INVALID_ARG.
 *   workspace lora_backward_workspace_bytes(...) bytes; its first 4096 bytes zero as for the forward.
 *   Then the weight gradients: a fine-tune segment of up to 512 rows is accumulated straight into dA / dB;
 *   a longer one is cut into row chunks whose partial sums go to the workspace and are added in chunk
 *   order by one more launch (skipped for batches of up to 512 tokens).
 *   dA / dB are accumulated with fp32 additions in memory (plain device allocations, not fine-grained
 *   host-visible memory), one addition per element and fine-tune segment, and every other sum has a fixed
 *   order: results are reproducible run to run when every adapter has at most one fine-tune segment
 *   (always true of lora_build_segments' tables); two fine-tune segments of one adapter are both added,
 *   in either order.
 * ------------------------------------------------------------------------------------------- */
size_t lora_backward_workspace_bytes(int32_t n_tokens, int32_t n_adapters, int32_t max_rank, int32_t d_in,
                                     int32_t d_out);

lq_status lora_segmented_backward(const void* x, int64_t ldx, const void* dy, int64_t lddy, void* dx, int64_t lddx,
                                  int32_t d_in, int32_t d_out,
                                  const void* const* A_ptrs, const void* const* B_ptrs,
                                  float* const* dA_ptrs, float* const* dB_ptrs,
                                  const int32_t* ranks, const float* scales, const float* token_scales,
                                  int32_t n_adapters, int32_t max_rank,
                                  const int32_t* perm, int32_t n_tokens,
                                  const int32_t* seg_starts, const int32_t* seg_adapter, const uint8_t* seg_kind,
                                  const int32_t* n_segments, int32_t max_segments,
                                  const float* h_saved, const int64_t* h_offsets,
                                  int32_t variant, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * LoRA dropout on the fine-tuning rows.  The paper's training configurations use lora_dropout = 0.05
 * (Appendix, LoRA configuration tables): in the LoRA branch of a fine-tuning token x is replaced by
 * m * x / (1 - p), the elements of m independent and 1 with probability 1 - p.  This call computes
 *     out[t, :] = m[t, :] * in[t, :]   for live fine-tuning tokens t,   in[t, :] for every other token
 * (in == out is allowed: in place).  The factor 1 / (1 - p) is left to the caller's scale (pass
 * token_scales[t] = s / (1 - p) for those tokens to the forward and the backward): m * x is exact in bf16,
 * x / (1 - p) is not, so the saved h of a fine-tuning token is (m * x) A.  The same call applied to the
 * LoRA branch's dx gives the gradient with respect to x (the mask is the same function of seed, row, column).
 *
 * The paper fixes no generator; the mask is this library's CONTRACT: with the 32-bit hash of Jarzynski
 * and Olano (JCGT 2020)   hash(v): s = v * 747796405 + 2891336453;
 *                                   w = ((s >> ((s >> 28) + 4)) ^ s) * 277803737;  return (w >> 22) ^ w
 *   key(t) = hash(seed ^ hash(t)),  word(t, q) = hash(key(t) + q) for the column pair q = k / 2,
 *   field = low 16 bits of the word for even k, high 16 bits for odd k,
 *   m[t, k] = field >= (uint32)(p * 65536 + 0.5), computed in fp32   (so p acts in steps of 2^-16; p = 0 keeps everything)
 *   in / out  bf16 [n_tokens, d], leading dimensions ld_in / ld_out; d, ld multiples of 8, 16-byte aligned
 *   token_adapter, token_kind  as for lora_build_segments (a row is a fine-tuning row iff its adapter id
 *             lies in [0, n_adapters) and its kind is LQ_SEG_FINETUNE)
 *   p         in [0, 1), else LQ_ERR_INVALID_ARG
 * ------------------------------------------------------------------------------------------- */
lq_status lora_dropout_rows(const void* in, int64_t ld_in, void* out, int64_t ld_out, int32_t d,
                            const int32_t* token_adapter, const uint8_t* token_kind, int32_t n_tokens,
                            int32_t n_adapters, uint32_t seed, float p, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Row split by kind and concatenation (Algorithm 1).  The attention layer takes the fine-tuning,
 * the prefill (and evaluation) and the decode rows out of Q, K, V by offsets that follow from the
 * batch order fine-tune | prefill | decode, runs a different attention implementation on each part
 * and concatenates the outputs again.  With the segment tables the rows of kind c are
 * perm[kind_offsets[c] .. kind_offsets[c + 1]):
 *   lora_kind_offsets  kind_offsets int32[4] (device): where the fine-tune, prefill and decode rows start
 *                      in the segment order (Algorithm 1's Offset_p and Offset_d are entries 1 and 2), and
 *                      the number of live rows; a kind without rows starts where the next one starts
 *   lora_split_rows    parts[i, :] = src[perm[i], :] for the live positions i: the three kinds back to
 *                      back, dense [n_live, d] bf16 (capacity n_tokens rows); perm NULL = identity
 *   lora_concat_rows   dst[perm[i], :] = parts[i, :]; rows of dst without adapter are untouched
 *   d and ld multiples of 8, 16-byte aligned pointers; parts must not alias src / dst.
 * ------------------------------------------------------------------------------------------- */
lq_status lora_kind_offsets(const int32_t* seg_starts, const uint8_t* seg_kind, const int32_t* n_segments,
                            int32_t max_segments, int32_t* kind_offsets, void* stream);
lq_status lora_split_rows(const void* src, int64_t ld, int32_t d, const int32_t* perm, int32_t n_tokens,
                          const int32_t* seg_starts, const int32_t* n_segments, int32_t max_segments,
                          void* parts, void* stream);
lq_status lora_concat_rows(const void* parts, int32_t d, const int32_t* perm, int32_t n_tokens,
                           const int32_t* seg_starts, const int32_t* n_segments, int32_t max_segments,
                           void* dst, int64_t ld, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Timing of the library's own kernel launches, for benchmarks (not part of the paper's method).
 * While enabled, every launch gets a pair of events that receive the dispatch's start and end time
 * stamps, i.e. the duration a kernel trace reports, without the gaps between launches.
 *   lora_profile_enable(on)  on != 0 starts recording, 0 stops; both discard what was recorded.
 *   lora_profile_read(total_us, launches, n_kernels)  host arrays of n_kernels >= LQ_KERNEL_IDS entries,
 *       indexed by lq_kernel_id: summed duration in microseconds and number of launches since
 *       recording started; waits for the recorded launches to finish, then discards the records.
 * Host-side state shared by all threads of the process: call from one thread at a time.  At most
 * 65536 launches are recorded between reads; further ones run untimed.
 * ------------------------------------------------------------------------------------------- */
typedef enum {
    LQ_KERNEL_BUILD = 0, LQ_KERNEL_SHRINK = 1, LQ_KERNEL_EXPAND = 2, LQ_KERNEL_FUSED = 3,
    LQ_KERNEL_WGRAD = 4, LQ_KERNEL_WREDUCE = 5, LQ_KERNEL_SLAB = 6, LQ_KERNEL_IDS = 7
} lq_kernel_id;

lq_status lora_profile_enable(int32_t on);
lq_status lora_profile_read(double* total_us, int64_t* launches, int32_t n_kernels);

#ifdef __cplusplus
}
#endif
#endif /* LQLORA_H */
