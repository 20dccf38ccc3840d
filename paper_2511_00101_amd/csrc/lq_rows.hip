// Row operations next to the contraction: LoRA dropout on the fine-tuning rows (training configurations of the
// appendix: lora_dropout 0.05) and the row split by kind / concatenation of Algorithm 1.  Plain streaming kernels:
// 16-byte accesses, a workgroup walks whole rows, the grid strides over the rows.
#include "lq_internal.h"

namespace lq {
namespace {

constexpr int kRowThreads = 256;

// The dropout mask is a contract (include/lqlora.h): the 32-bit hash of Jarzynski and Olano (one step of a linear
// congruential generator and the PCG output permutation), keyed by (seed, row), one word per pair of columns.
__device__ __forceinline__ unsigned int hash32(unsigned int v)
{
    const unsigned int s = v * 747796405u + 2891336453u;
    const unsigned int w = ((s >> ((s >> 28) + 4u)) ^ s) * 277803737u;
    return (w >> 22) ^ w;
}

__global__ __launch_bounds__(kRowThreads) void dropout_rows_kernel(const u16* in, long long ld_in, u16* out, long long ld_out,
                                                                    int d, const int32_t* token_adapter,
                                                                    const uint8_t* token_kind, int n_tokens, int n_adapters,
                                                                    unsigned int seed, unsigned int threshold)
{
    for (int t = (int)blockIdx.x; t < n_tokens; t += (int)gridDim.x) {
        const int a = token_adapter[t], kind = token_kind[t];
        const bool ft = a >= 0 && a < n_adapters && kind == LQ_SEG_FINETUNE;  // workgroup uniform
        if (!ft && in == out) continue;                                        // in place: nothing to do for this row
        const unsigned int key = hash32(seed ^ hash32((unsigned int)t));
        const u16* src = in + (long long)t * ld_in;
        u16* dst = out + (long long)t * ld_out;
        for (int k = (int)threadIdx.x * 8; k < d; k += kRowThreads * 8) {
            u32x4 v = *reinterpret_cast<const u32x4*>(src + k);
            if (ft) {
                unsigned int w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {  // word i holds columns k + 2 i (low half) and k + 2 i + 1 (high half)
                    const unsigned int r = hash32(key + (unsigned int)((k >> 1) + i));
                    if ((r & 0xffffu) < threshold) w[i] &= 0xffff0000u;
                    if ((r >> 16) < threshold) w[i] &= 0x0000ffffu;
                }
                v = u32x4{w[0], w[1], w[2], w[3]};
            }
            *reinterpret_cast<u32x4*>(dst + k) = v;
        }
    }
}

// kind_offsets[c] = first position (in segment order) of a segment of kind >= c, or the number of live rows
__global__ void kind_offsets_kernel(const int32_t* seg_starts, const uint8_t* seg_kind, const int32_t* n_segments, int max_segments,
                                    int32_t* kind_offsets)
{
    const int c = (int)threadIdx.x;
    if (c > 3) return;
    const int n_seg = min(max(*n_segments, 0), max_segments);
    int off = seg_starts[n_seg];
    for (int s = n_seg - 1; s >= 0; --s)
        if (seg_kind[s] >= c) off = seg_starts[s];
    kind_offsets[c] = off;
}

// SPLIT: parts[i, :] = src[perm[i], :];  else: src[perm[i], :] = parts[i, :]   for the live positions i
template <bool SPLIT>
__global__ __launch_bounds__(kRowThreads) void move_rows_kernel(u16* src, long long ld, int d, const int32_t* perm, int n_tokens,
                                                                 const int32_t* seg_starts, const int32_t* n_segments,
                                                                 int max_segments, u16* parts)
{
    const int n_seg = min(max(*n_segments, 0), max_segments);
    const int n_live = min(max(seg_starts[n_seg], 0), n_tokens);
    for (int i = (int)blockIdx.x; i < n_live; i += (int)gridDim.x) {
        const int row = perm ? perm[i] : i;
        if (row < 0 || row >= n_tokens) continue;  // (a table written by a careless caller)
        u16* a = src + (long long)row * ld;
        u16* b = parts + (long long)i * d;
        for (int k = (int)threadIdx.x * 8; k < d; k += kRowThreads * 8) {
            if (SPLIT) *reinterpret_cast<u32x4*>(b + k) = *reinterpret_cast<const u32x4*>(a + k);
            else *reinterpret_cast<u32x4*>(a + k) = *reinterpret_cast<const u32x4*>(b + k);
        }
    }
}

int row_grid(int n_rows) { return n_rows < 1 ? 1 : n_rows < 4096 ? n_rows : 4096; }

}  // namespace
}  // namespace lq

extern "C" lq_status lora_dropout_rows(const void* in, int64_t ld_in, void* out, int64_t ld_out, int32_t d,
                                       const int32_t* token_adapter, const uint8_t* token_kind, int32_t n_tokens,
                                       int32_t n_adapters, uint32_t seed, float p, void* stream)
{
    using namespace lq;
    if (n_tokens < 0 || d <= 0 || n_adapters <= 0 || ld_in < d || ld_out < d) return LQ_ERR_INVALID_ARG;
    if (!(p >= 0.f && p < 1.f)) return LQ_ERR_INVALID_ARG;
    if (n_tokens > 0 && (!in || !out || !token_adapter || !token_kind)) return LQ_ERR_INVALID_ARG;
    if ((d % 8) || (ld_in % 8) || (ld_out % 8) || !aligned16(in) || !aligned16(out)) return LQ_ERR_UNSUPPORTED;
    if (n_tokens == 0) return LQ_OK;
    const unsigned int threshold = (unsigned int)(p * 65536.0f + 0.5f);
    hipLaunchKernelGGL(dropout_rows_kernel, dim3(row_grid(n_tokens)), dim3(kRowThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u16*>(in), (long long)ld_in, static_cast<u16*>(out), (long long)ld_out, d, token_adapter,
                       token_kind, n_tokens, n_adapters, seed, threshold);
    return hipGetLastError() == hipSuccess ? LQ_OK : LQ_ERR_HIP;
}

extern "C" lq_status lora_kind_offsets(const int32_t* seg_starts, const uint8_t* seg_kind, const int32_t* n_segments,
                                       int32_t max_segments, int32_t* kind_offsets, void* stream)
{
    if (!seg_starts || !seg_kind || !n_segments || !kind_offsets || max_segments < 0) return LQ_ERR_INVALID_ARG;
    hipLaunchKernelGGL(lq::kind_offsets_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), seg_starts, seg_kind,
                       n_segments, max_segments, kind_offsets);
    return hipGetLastError() == hipSuccess ? LQ_OK : LQ_ERR_HIP;
}

namespace lq {
namespace {
lq_status move_rows(bool split, void* rows, int64_t ld, int32_t d, const int32_t* perm, int32_t n_tokens,
                    const int32_t* seg_starts, const int32_t* n_segments, int32_t max_segments, void* parts, void* stream)
{
    if (n_tokens < 0 || d <= 0 || ld < d || max_segments < 0 || !seg_starts || !n_segments) return LQ_ERR_INVALID_ARG;
    if (n_tokens > 0 && (!rows || !parts)) return LQ_ERR_INVALID_ARG;
    if (rows && rows == parts) return LQ_ERR_INVALID_ARG;
    if ((d % 8) || (ld % 8) || !aligned16(rows) || !aligned16(parts)) return LQ_ERR_UNSUPPORTED;
    if (n_tokens == 0) return LQ_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (split)
        hipLaunchKernelGGL(move_rows_kernel<true>, dim3(row_grid(n_tokens)), dim3(kRowThreads), 0, st, static_cast<u16*>(rows),
                           (long long)ld, d, perm, n_tokens, seg_starts, n_segments, max_segments, static_cast<u16*>(parts));
    else
        hipLaunchKernelGGL(move_rows_kernel<false>, dim3(row_grid(n_tokens)), dim3(kRowThreads), 0, st, static_cast<u16*>(rows),
                           (long long)ld, d, perm, n_tokens, seg_starts, n_segments, max_segments, static_cast<u16*>(parts));
    return hipGetLastError() == hipSuccess ? LQ_OK : LQ_ERR_HIP;
}
}  // namespace
}  // namespace lq

extern "C" lq_status lora_split_rows(const void* src, int64_t ld, int32_t d, const int32_t* perm, int32_t n_tokens,
                                     const int32_t* seg_starts, const int32_t* n_segments, int32_t max_segments,
                                     void* parts, void* stream)
{
    return lq::move_rows(true, const_cast<void*>(src), ld, d, perm, n_tokens, seg_starts, n_segments, max_segments, parts, stream);
}

extern "C" lq_status lora_concat_rows(const void* parts, int32_t d, const int32_t* perm, int32_t n_tokens,
                                      const int32_t* seg_starts, const int32_t* n_segments, int32_t max_segments,
                                      void* dst, int64_t ld, void* stream)
{
    return lq::move_rows(false, dst, ld, d, perm, n_tokens, seg_starts, n_segments, max_segments, const_cast<void*>(parts), stream);
}
