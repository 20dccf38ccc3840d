// Segmented multi-adapter LoRA forward (Section 3.3): shrink (h = x A_a^T per segment), h-save for
// fine-tune segments, expand (y += s_a h B_a).
#include "lq_common.h"

namespace lq {
namespace {

// ------------------------------------------------------------------------------------------------
// Short-segment path (decode and other short segments): a chunk is up to 4 token rows of one
// segment.  The contraction over d_in is a per-lane 8-wide dot product on 16-byte bf16 loads
// followed by a wave-wide transpose-reduce; the contraction over the rank is a broadcast of h from
// one lane to the wave.  The work is bound by streaming A_a and B_a once per chunk.
// ------------------------------------------------------------------------------------------------
constexpr int kTT = 4;            // token rows per chunk
constexpr int kRJ = 16;           // rank rows per block (kTT * kRJ = 64 = one value per lane after the reduce)
constexpr int kSvThreads = 256;
constexpr int kSvWaves = kSvThreads / kWave;
constexpr int kKPerWaveIter = kWave * 8;  // d_in elements one wave covers per iteration
constexpr int kMaxKSplit = 16;

struct FwdParams {
    const u16* x; long long ldx;
    u16* y; long long ldy;
    int d_in, d_out;
    const void* const* A_ptrs; const void* const* B_ptrs;
    const int32_t* ranks; const float* scales; int n_adapters; int max_rank;
    const int32_t* perm; int n_tokens;
    const int32_t* seg_starts; const int32_t* seg_adapter; const uint8_t* seg_kind;
    const int32_t* n_segments; int max_segments;
    float* h_out; const long long* h_offsets;
    float* hpart;   // [ksplit][n_tokens][rstride] partial h, indexed by position in segment order
    int ksplit; int rstride;
    int* err;
};

// After the call, lane L holds the sum over all lanes of v[L].
template <int HALF>
__device__ __forceinline__ void transpose_reduce_step(float (&v)[64], int lane)
{
    const bool upper = (lane & HALF) != 0;
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
        const float send = upper ? v[i] : v[i + HALF];
        const float keep = upper ? v[i + HALF] : v[i];
        v[i] = keep + __shfl_xor(send, HALF, kWave);
    }
}
__device__ __forceinline__ float transpose_reduce64(float (&v)[64])
{
    const int lane = lane_id();
    transpose_reduce_step<32>(v, lane);
    transpose_reduce_step<16>(v, lane);
    transpose_reduce_step<8>(v, lane);
    transpose_reduce_step<4>(v, lane);
    transpose_reduce_step<2>(v, lane);
    transpose_reduce_step<1>(v, lane);
    return v[0];
}

struct SegInfo {
    int adapter, rank, kind;
    float scale;
    bool ok;
};

__device__ __forceinline__ SegInfo load_segment(const FwdParams& p, int seg)
{
    SegInfo s;
    s.adapter = p.seg_adapter[seg];
    s.kind = p.seg_kind[seg];
    s.ok = s.adapter >= 0 && s.adapter < p.n_adapters;
    s.rank = 0;
    s.scale = 0.f;
    if (s.ok) {
        s.rank = p.ranks[s.adapter];
        s.scale = p.scales[s.adapter];
        s.ok = s.rank >= 1 && s.rank <= p.max_rank;
    }
    if (!s.ok && lane_id() == 0) atomicOr(p.err, kErrBadSegment);
    return s;
}

// row of x / y for a position of the segment order; -1 if the table holds an invalid row
__device__ __forceinline__ int row_of(const FwdParams& p, int pos)
{
    const int row = p.perm ? p.perm[pos] : pos;
    return (row >= 0 && row < p.n_tokens) ? row : -1;
}

__global__ __launch_bounds__(kSvThreads) void shrink_short_kernel(FwdParams p)
{
    const int lane = lane_id(), w = (int)threadIdx.x / kWave;
    const int ks = (int)blockIdx.y * kSvWaves + w;
    if (ks >= p.ksplit) return;
    const int n_seg = min(*p.n_segments, p.max_segments);
    const Chunk c = find_chunk(p.seg_starts, n_seg, (int)blockIdx.x, kTT);
    if (c.seg < 0) return;
    const SegInfo s = load_segment(p, c.seg);
    if (!s.ok) return;
    const u16* __restrict__ A = static_cast<const u16*>(p.A_ptrs[s.adapter]);

    int row[kTT];
#pragma unroll
    for (int t = 0; t < kTT; ++t) row[t] = t < c.len ? row_of(p, c.pos + t) : -1;

    for (int jb = 0; jb < s.rank; jb += kRJ) {
        float acc[kTT * kRJ];
#pragma unroll
        for (int i = 0; i < kTT * kRJ; ++i) acc[i] = 0.f;

        for (int k = (ks * kWave + lane) * 8; k < p.d_in; k += p.ksplit * kKPerWaveIter) {
            float xf[kTT][8];
#pragma unroll
            for (int t = 0; t < kTT; ++t) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (row[t] >= 0) v = *reinterpret_cast<const u32x4*>(p.x + (long long)row[t] * p.ldx + k);
                unpack8(v, xf[t]);
            }
#pragma unroll
            for (int jj = 0; jj < kRJ; ++jj) {
                if (jb + jj < s.rank) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(A + (long long)(jb + jj) * p.d_in + k);
                    float af[8];
                    unpack8(v, af);
#pragma unroll
                    for (int t = 0; t < kTT; ++t)
#pragma unroll
                        for (int i = 0; i < 8; ++i) acc[t * kRJ + jj] = fmaf(xf[t][i], af[i], acc[t * kRJ + jj]);
                }
            }
        }
        const float total = transpose_reduce64(acc);
        const int t = lane / kRJ, jj = lane % kRJ;
        if (t < c.len && jb + jj < s.rank)
            p.hpart[((long long)ks * p.n_tokens + c.pos + t) * p.rstride + jb + jj] = total;
    }
}

__global__ __launch_bounds__(kSvThreads) void expand_short_kernel(FwdParams p)
{
    const int lane = lane_id(), w = (int)threadIdx.x / kWave;
    const int wave_id = (int)blockIdx.y * kSvWaves + w;
    const int n_waves = (int)gridDim.y * kSvWaves;
    const int n_seg = min(*p.n_segments, p.max_segments);
    const Chunk c = find_chunk(p.seg_starts, n_seg, (int)blockIdx.x, kTT);
    if (c.seg < 0) return;
    const SegInfo s = load_segment(p, c.seg);
    if (!s.ok) return;
    const u16* __restrict__ B = static_cast<const u16*>(p.B_ptrs[s.adapter]);

    // lane (t, jj) sums the split-K partials of h[t][b * 16 + jj] for every rank block b, saves the
    // unscaled value for fine-tune segments and leaves the scaled value in this wave's LDS slab as
    // hs[j][t], from where one 16-byte broadcast read fetches rank j of all four rows.
    __shared__ __attribute__((aligned(16))) float hs_all[kSvWaves][LQ_MAX_RANK][kTT];
    float (*hs)[kTT] = hs_all[w];
    const int t_l = lane / kRJ, jj_l = lane % kRJ;
    const bool save_h = s.kind == LQ_SEG_FINETUNE && p.h_out && p.h_offsets && wave_id == 0;
    const long long h_base = save_h ? p.h_offsets[c.seg] + (long long)(c.pos - c.first + t_l) * s.rank : 0;
    for (int jb = 0; jb < s.rank; jb += kRJ) {
        float sum = 0.f;
        const int j = jb + jj_l;
        if (t_l < c.len && j < s.rank) {
            for (int ks = 0; ks < p.ksplit; ++ks)
                sum += p.hpart[((long long)ks * p.n_tokens + c.pos + t_l) * p.rstride + j];
            if (save_h) p.h_out[h_base + j] = sum;
        }
        if (j < s.rank) hs[j][t_l] = sum * s.scale;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    int row[kTT];
#pragma unroll
    for (int t = 0; t < kTT; ++t) row[t] = t < c.len ? row_of(p, c.pos + t) : -1;

    for (int n = (wave_id * kWave + lane) * 8; n < p.d_out; n += n_waves * kKPerWaveIter) {
        float acc[kTT][8];
#pragma unroll
        for (int t = 0; t < kTT; ++t)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[t][i] = 0.f;
#pragma unroll 8
        for (int j = 0; j < s.rank; ++j) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(B + (long long)j * p.d_out + n);
            const f32x4 h4 = *reinterpret_cast<const f32x4*>(hs[j]);
            float bf[8];
            unpack8(v, bf);
            const float h[kTT] = {h4.x, h4.y, h4.z, h4.w};
#pragma unroll
            for (int t = 0; t < kTT; ++t)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[t][i] = fmaf(h[t], bf[i], acc[t][i]);
        }
#pragma unroll
        for (int t = 0; t < kTT; ++t) {
            if (row[t] >= 0) {
                u32x4* yp = reinterpret_cast<u32x4*>(p.y + (long long)row[t] * p.ldy + n);
                const u32x4 v = *yp;
                float yf[8];
                unpack8(v, yf);
                u32x4 o;
                o.x = pack_bf16x2(yf[0] + acc[t][0], yf[1] + acc[t][1]);
                o.y = pack_bf16x2(yf[2] + acc[t][2], yf[3] + acc[t][3]);
                o.z = pack_bf16x2(yf[4] + acc[t][4], yf[5] + acc[t][5]);
                o.w = pack_bf16x2(yf[6] + acc[t][6], yf[7] + acc[t][7]);
                *yp = o;
            }
        }
    }
}

int ksplit_for(int d_in)
{
    int ks = (d_in + kKPerWaveIter - 1) / kKPerWaveIter;
    return ks < 1 ? 1 : (ks > kMaxKSplit ? kMaxKSplit : ks);
}

int rstride_for(int max_rank) { return (max_rank + 3) / 4 * 4; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace lq

extern "C" size_t lora_forward_workspace_bytes(int32_t n_tokens, int32_t max_rank, int32_t d_in, int32_t d_out,
                                               int32_t variant)
{
    (void)d_out; (void)variant;
    if (n_tokens < 0 || max_rank < 1 || d_in < 1) return lq::kWsHeaderBytes;
    return (size_t)lq::kWsHeaderBytes +
           (size_t)lq::ksplit_for(d_in) * (size_t)n_tokens * (size_t)lq::rstride_for(max_rank) * sizeof(float);
}

extern "C" lq_status lora_segmented_forward(const void* x, int64_t ldx, void* y, int64_t ldy,
                                            int32_t d_in, int32_t d_out,
                                            const void* const* A_ptrs, const void* const* B_ptrs,
                                            const int32_t* ranks, const float* scales, int32_t n_adapters,
                                            int32_t max_rank,
                                            const int32_t* perm, int32_t n_tokens,
                                            const int32_t* seg_starts, const int32_t* seg_adapter,
                                            const uint8_t* seg_kind,
                                            const int32_t* n_segments, int32_t max_segments,
                                            float* h_out, const int64_t* h_offsets,
                                            int32_t variant, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace lq;
    if (n_tokens < 0 || d_in <= 0 || d_out <= 0 || n_adapters <= 0 || max_segments < 0 || max_rank < 1)
        return LQ_ERR_INVALID_ARG;
    if (variant != LQ_VARIANT_SPLIT && variant != LQ_VARIANT_FUSED) return LQ_ERR_INVALID_ARG;
    if (!A_ptrs || !B_ptrs || !ranks || !scales || !seg_starts || !seg_adapter || !seg_kind || !n_segments)
        return LQ_ERR_INVALID_ARG;
    if (n_tokens > 0 && (!x || !y)) return LQ_ERR_INVALID_ARG;
    if (ldx < d_in || ldy < d_out) return LQ_ERR_INVALID_ARG;
    if (x && x == y) return LQ_ERR_INVALID_ARG;
    if (max_rank > LQ_MAX_RANK || n_adapters > LQ_MAX_ADAPTERS) return LQ_ERR_UNSUPPORTED;
    if ((d_in % 8) || (d_out % 8) || (ldx % 8) || (ldy % 8) || !aligned16(x) || !aligned16(y)) return LQ_ERR_UNSUPPORTED;
    if (variant == LQ_VARIANT_FUSED) return LQ_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < lora_forward_workspace_bytes(n_tokens, max_rank, d_in, d_out, variant) ||
        !aligned16(workspace))
        return LQ_ERR_WORKSPACE;
    if (n_tokens == 0 || max_segments == 0) return LQ_OK;

    FwdParams p;
    p.x = static_cast<const u16*>(x); p.ldx = ldx;
    p.y = static_cast<u16*>(y); p.ldy = ldy;
    p.d_in = d_in; p.d_out = d_out;
    p.A_ptrs = A_ptrs; p.B_ptrs = B_ptrs; p.ranks = ranks; p.scales = scales;
    p.n_adapters = n_adapters; p.max_rank = max_rank;
    p.perm = perm; p.n_tokens = n_tokens;
    p.seg_starts = seg_starts; p.seg_adapter = seg_adapter; p.seg_kind = seg_kind;
    p.n_segments = n_segments; p.max_segments = max_segments;
    p.h_out = h_out; p.h_offsets = reinterpret_cast<const long long*>(h_offsets);
    p.err = static_cast<int*>(workspace);
    p.hpart = reinterpret_cast<float*>(static_cast<char*>(workspace) + kWsHeaderBytes);
    p.ksplit = ksplit_for(d_in);
    p.rstride = rstride_for(max_rank);

    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t seg_bound = max_segments;
    if (seg_bound > n_tokens) seg_bound = n_tokens;
    if (seg_bound > 3 * (int64_t)n_adapters) seg_bound = 3 * (int64_t)n_adapters;
    const int64_t chunk_bound = (n_tokens + kTT - 1) / kTT + seg_bound;
    if (chunk_bound > 0x7fffffff) return LQ_ERR_UNSUPPORTED;

    dim3 grid_s((unsigned)chunk_bound, (unsigned)((p.ksplit + kSvWaves - 1) / kSvWaves));
    hipLaunchKernelGGL(shrink_short_kernel, grid_s, dim3(kSvThreads), 0, st, p);
    int n_groups = (d_out + kSvWaves * kKPerWaveIter - 1) / (kSvWaves * kKPerWaveIter);
    if (n_groups > 8) n_groups = 8;
    dim3 grid_e((unsigned)chunk_bound, (unsigned)n_groups);
    hipLaunchKernelGGL(expand_short_kernel, grid_e, dim3(kSvThreads), 0, st, p);
    return hipGetLastError() == hipSuccess ? LQ_OK : LQ_ERR_HIP;
}
