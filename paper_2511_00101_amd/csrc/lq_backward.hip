// Backward of the segmented LoRA update for fine-tune segments.  The paper leaves this to autograd, one
// call per LoRA linear, and names a dedicated kernel as future work (Section 4.2, Appendix A); this is
// the exact gradient of the forward defined in lqlora.h, with g = dy B^T:
//     dx += s g A            dB += s h^T dy            dA += s g^T x
// g = dy B^T is the forward's shrink with the roles (x, A, d_in) := (dy, B, d_out), and dx += s g A is
// the forward's expand with (y, B, d_out) := (dx, A, d_in); both reuse those kernels, restricted to
// fine-tune segments.  The two weight gradients are contractions over the TOKEN axis, which is the
// strided axis of every operand, so they get a kernel of their own:
//   weight-gradient unit : 512 rows of a fine-tune segment x 512 columns of dy (for dB, with h) or of x
//                          (for dA, with g).  32 rows at a time are staged in LDS with coalesced loads
//                          (double buffered) and read back transposed into 16x16x32 bf16 MFMA
//                          fragments; h and g are split into bf16 high and low parts.  The unit stores
//                          its [rank x 512] partial to the workspace.
//   reduce unit          : one segment x 512 columns: adds the segment's partials in chunk order, applies
//                          the scale and accumulates into dA / dB.  Fixed order, so reproducible.
#include "lq_internal.h"

namespace lq {
namespace {

constexpr int kThreads = 512;
constexpr int kWgRows = 512;    // token rows per weight-gradient unit
constexpr int kWgCols = 512;    // columns per unit (8 waves x 64)
constexpr int kStepRows = 32;   // token rows per MFMA k step
constexpr int kBig = 0x7fffffff;

struct BwdParams {
    const u16* x; long long ldx;
    const u16* dy; long long lddy;
    int d_in, d_out;
    float* const* dA_ptrs; float* const* dB_ptrs;
    const void* const* A_ptrs; const void* const* B_ptrs;  // only for the table helpers
    const int32_t* ranks; const float* scales; int n_adapters; int max_rank;
    const int32_t* perm; int n_tokens;
    const int32_t* seg_starts; const int32_t* seg_adapter; const uint8_t* seg_kind;
    const int32_t* n_segments; int max_segments;
    const float* h_saved; const long long* h_offsets;
    const float* g;      // [ksplit][n_tokens][rstride] slices of g = dy B^T by position in segment order
    int ksplit; int rstride;
    float* wpart;        // [chunk][rstride][d_out + d_in] partial weight gradients
    int* err;
};

template <int NT>
struct WgCfg {
    static constexpr int YPITCH = kWgCols + 8;                 // u16 elements per staged activation row
    static constexpr int HPITCH = 16 * NT + 1;                 // floats per staged h / g row
    static constexpr size_t Y_BYTES = (size_t)kStepRows * YPITCH * sizeof(u16);
    static constexpr size_t H_BYTES = ((size_t)kStepRows * HPITCH * sizeof(float) + 15) / 16 * 16;
    static constexpr size_t BUF_BYTES = Y_BYTES + H_BYTES;
    static constexpr size_t LDS_BYTES = 2 * BUF_BYTES + kWgRows * sizeof(int);
};

__device__ __forceinline__ void split_hi_lo(const float (&v)[8], u32x4& hi, u32x4& lo)
{
    unsigned int h[8], l[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        h[i] = f32_to_bf16_bits(v[i]);
        l[i] = f32_to_bf16_bits(v[i] - __uint_as_float(h[i] << 16));
    }
    hi = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    lo = u32x4{l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)};
}

// D[rank][col] = sum_t H[t][rank] Y[t][col] over the unit's rows; H = h_saved (for dB, Y = dy) or g (for
// dA, Y = x).  MFMA: lane (c = lane % 16, kg = lane / 16) supplies H[8 kg ..][rank c] and Y[8 kg ..][col c]
// of a 32-row step and receives D[rank 4 kg + v][col c].
template <int NT>
__device__ __forceinline__ void wgrad_unit(const BwdParams& p, const Unit& u, int rank, int chunk_id, bool for_b,
                                           int col_block, unsigned char* lds)
{
    using C = WgCfg<NT>;
    const int lane = lane_id(), w = uniform((int)threadIdx.x / kWave), c = lane & 15, kg = lane >> 4;
    const u16* Y = for_b ? p.dy : p.x;
    const long long ldy = for_b ? p.lddy : p.ldx;
    const int d = for_b ? p.d_out : p.d_in;
    const int n0 = col_block * kWgCols;
    int* lds_row = reinterpret_cast<int*>(lds + 2 * C::BUF_BYTES);

    __syncthreads();  // the previous unit's LDS reads are done
    for (int i = (int)threadIdx.x; i < kWgRows; i += kThreads) lds_row[i] = i < u.len ? row_of(p, u.pos + i) : -1;
    __syncthreads();
    const int safe_row = max(lds_row[0], 0);

    // staging assignment.  Y: 16 threads cover 128 columns of one row per pass, 4 passes cover 512 columns.
    const int y_row = (int)threadIdx.x / 16, y_piece = (int)threadIdx.x % 16;
    const long long h_base = for_b ? p.h_offsets[u.seg] + (long long)(u.pos - u.first) * rank : 0;
    u32x4 gy[4];
    float gh[NT];
    auto stage_load = [&](int step) {
        const int i = step * kStepRows + y_row;
        const int row = lds_row[min(i, kWgRows - 1)];
        const u16* yrow = Y + (long long)(row >= 0 ? row : safe_row) * ldy;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = n0 + (y_piece + 16 * q) * 8;
            const u32x4 v = *reinterpret_cast<const u32x4*>(yrow + min(n, d - 8));
            gy[q] = (n < d && row >= 0) ? v : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            const int j = y_piece + 16 * q;
            float v = 0.f;
            if (i < u.len && j < rank) {
                if (for_b) {
                    v = p.h_saved[h_base + (long long)i * rank + j];
                } else {
                    for (int part = 0; part < p.ksplit; ++part)
                        v += p.g[((long long)part * p.n_tokens + u.pos + i) * p.rstride + j];
                }
            }
            gh[q] = v;
        }
    };
    auto stage_store = [&](int buf) {
        u16* ly = reinterpret_cast<u16*>(lds + buf * C::BUF_BYTES);
        float* lh = reinterpret_cast<float*>(lds + buf * C::BUF_BYTES + C::Y_BYTES);
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<u32x4*>(ly + y_row * C::YPITCH + (y_piece + 16 * q) * 8) = gy[q];
#pragma unroll
        for (int q = 0; q < NT; ++q) lh[y_row * C::HPITCH + y_piece + 16 * q] = gh[q];
    };

    f32x4 acc[NT][4];
#pragma unroll
    for (int jt = 0; jt < NT; ++jt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[jt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int n_steps = (u.len + kStepRows - 1) / kStepRows;
    stage_load(0);
    for (int step = 0; step < n_steps; ++step) {
        const int buf = step & 1;
        stage_store(buf);
        stage_load(min(step + 1, n_steps - 1));  // unconditional; the last one re-reads
        __syncthreads();  // one barrier per step: the buffer written now was last read two steps ago
        const u16* ly = reinterpret_cast<const u16*>(lds + buf * C::BUF_BYTES);
        const float* lh = reinterpret_cast<const float*>(lds + buf * C::BUF_BYTES + C::Y_BYTES);
        u32x4 yf[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const u16* col = ly + w * 64 + nt * 16 + c;
            unsigned int e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) e[i] = col[(8 * kg + i) * C::YPITCH];
            yf[nt] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
        }
#pragma unroll
        for (int jt = 0; jt < NT; ++jt) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = lh[(8 * kg + i) * C::HPITCH + jt * 16 + c];
            u32x4 hi, lo;
            split_hi_lo(v, hi, lo);
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                acc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(lo), as_bf16x8(yf[nt]), acc[jt][nt], 0, 0, 0);
                acc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(hi), as_bf16x8(yf[nt]), acc[jt][nt], 0, 0, 0);
            }
        }
    }

    const int dsum = p.d_out + p.d_in;
    float* out = p.wpart + (long long)chunk_id * p.rstride * dsum + (for_b ? 0 : p.d_out);
#pragma unroll
    for (int jt = 0; jt < NT; ++jt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int j = jt * 16 + 4 * kg + v, n = n0 + w * 64 + nt * 16 + c;
                if (j < rank && n < d) out[(long long)j * dsum + n] = acc[jt][nt][v];
            }
}

template <int NT>
__global__ __launch_bounds__(kThreads) void wgrad_kernel(BwdParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int n_seg = uniform(min(*p.n_segments, p.max_segments));
    const SegCache c0 = load_seg_cache(p, n_seg);
    const LenClass ft{1, kBig, 1 << LQ_SEG_FINETUNE};
    const int blocks_b = (p.d_out + kWgCols - 1) / kWgCols, blocks_a = (p.d_in + kWgCols - 1) / kWgCols;
    const int per_chunk = blocks_b + blocks_a;
    const int n_units = count_chunks(p, n_seg, c0, kWgRows, ft) * per_chunk;
    for (int id = (int)blockIdx.x; id < n_units; id += (int)gridDim.x) {
        Unit u;
        const int chunk_id = id / per_chunk, cb = id % per_chunk;
        if (!find_chunk(p, n_seg, c0, chunk_id, kWgRows, ft, u)) continue;
        if (u.ad < 0 || u.ad >= p.n_adapters) continue;  // flagged by the forward kernels already
        const int rank = p.ranks[u.ad];
        if (rank < 1 || rank > p.max_rank) continue;
        const bool for_b = cb < blocks_b;
        if (for_b ? (p.dB_ptrs == nullptr || p.dB_ptrs[u.ad] == nullptr) : (p.dA_ptrs == nullptr || p.dA_ptrs[u.ad] == nullptr))
            continue;
        wgrad_unit<NT>(p, u, rank, chunk_id, for_b, for_b ? cb : cb - blocks_b, lds_raw);
    }
}

// dA / dB += scale * (sum of the segment's chunk partials, in chunk order)
__global__ __launch_bounds__(kThreads) void wreduce_kernel(BwdParams p)
{
    const int n_seg = uniform(min(*p.n_segments, p.max_segments));
    const SegCache c0 = load_seg_cache(p, n_seg);
    const LenClass ft{1, kBig, 1 << LQ_SEG_FINETUNE};
    const int dsum = p.d_out + p.d_in;
    const int col_blocks = (dsum + kThreads - 1) / kThreads;
    const int n_units = count_chunks(p, n_seg, c0, kWgRows, ft) * col_blocks;
    for (int id = (int)blockIdx.x; id < n_units; id += (int)gridDim.x) {
        Unit u;
        const int chunk_id = id / col_blocks;
        if (!find_chunk(p, n_seg, c0, chunk_id, kWgRows, ft, u)) continue;
        if (u.pos != u.first) continue;  // only the segment's first chunk adds up the segment
        if (u.ad < 0 || u.ad >= p.n_adapters) continue;
        const int rank = p.ranks[u.ad];
        if (rank < 1 || rank > p.max_rank) continue;
        const float scale = p.scales[u.ad];
        const int n_chunks = (u.seg_len + kWgRows - 1) / kWgRows;
        const int col = (id % col_blocks) * kThreads + (int)threadIdx.x;
        if (col >= dsum) continue;
        const bool for_b = col < p.d_out;
        float* dst = for_b ? (p.dB_ptrs ? p.dB_ptrs[u.ad] : nullptr) : (p.dA_ptrs ? p.dA_ptrs[u.ad] : nullptr);
        if (!dst) continue;
        const int d = for_b ? p.d_out : p.d_in, n = for_b ? col : col - p.d_out;
        for (int j = 0; j < rank; ++j) {
            float sum = 0.f;
            for (int cc = 0; cc < n_chunks; ++cc)
                sum += p.wpart[((long long)(chunk_id + cc) * p.rstride + j) * dsum + col];
            dst[(long long)j * d + n] += scale * sum;
        }
    }
}

size_t wpart_bytes(int n_tokens, int n_adapters, int max_rank, int d_in, int d_out)
{
    const size_t chunks = (size_t)(n_tokens + kWgRows - 1) / kWgRows + (size_t)(n_tokens < n_adapters ? n_tokens : n_adapters);
    return chunks * (size_t)rstride_for(max_rank) * ((size_t)d_in + d_out) * sizeof(float);
}

template <int NT>
hipError_t launch_wgrad(const BwdParams& p, hipStream_t st)
{
    static int grid = 0;
    const size_t lds = WgCfg<NT>::LDS_BYTES;
    if (!grid) {
        int dev = 0, cus = 0, per_cu = 0;
        if (lds > 48 * 1024)
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(wgrad_kernel<NT>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipGetDevice(&dev);
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, wgrad_kernel<NT>, kThreads, lds) != hipSuccess || per_cu <= 0)
            per_cu = 1;
        grid = cus * per_cu;
    }
    hipLaunchKernelGGL(wgrad_kernel<NT>, dim3(grid), dim3(kThreads), lds, st, p);
    return hipGetLastError();
}

}  // namespace
}  // namespace lq

// workspace: [header 256 B][g slices: like the forward's partial h][partial weight gradients]
extern "C" size_t lora_backward_workspace_bytes(int32_t n_tokens, int32_t n_adapters, int32_t max_rank, int32_t d_in,
                                                int32_t d_out)
{
    if (n_tokens < 0 || n_adapters < 0 || max_rank < 1 || d_in < 0 || d_out < 0) return lq::kWsHeaderBytes;
    return (size_t)lq::kWsHeaderBytes + lq::h_slices_bytes(n_tokens, max_rank) +
           lq::wpart_bytes(n_tokens, n_adapters, max_rank, d_in, d_out);
}

extern "C" lq_status lora_segmented_backward(const void* x, int64_t ldx, const void* dy, int64_t lddy, void* dx,
                                             int64_t lddx, int32_t d_in, int32_t d_out,
                                             const void* const* A_ptrs, const void* const* B_ptrs,
                                             float* const* dA_ptrs, float* const* dB_ptrs,
                                             const int32_t* ranks, const float* scales, int32_t n_adapters,
                                             int32_t max_rank, const int32_t* perm, int32_t n_tokens,
                                             const int32_t* seg_starts, const int32_t* seg_adapter,
                                             const uint8_t* seg_kind, const int32_t* n_segments, int32_t max_segments,
                                             const float* h_saved, const int64_t* h_offsets,
                                             void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace lq;
    if (n_tokens < 0 || d_in <= 0 || d_out <= 0 || n_adapters <= 0 || max_segments < 0 || max_rank < 1)
        return LQ_ERR_INVALID_ARG;
    if (!A_ptrs || !B_ptrs || !ranks || !scales || !seg_starts || !seg_adapter || !seg_kind || !n_segments)
        return LQ_ERR_INVALID_ARG;
    if (n_tokens > 0 && (!x || !dy || !dx)) return LQ_ERR_INVALID_ARG;
    if ((dA_ptrs || dB_ptrs) && n_tokens > 0 && (!h_saved || !h_offsets)) return LQ_ERR_INVALID_ARG;
    if (ldx < d_in || lddx < d_in || lddy < d_out) return LQ_ERR_INVALID_ARG;
    if (x && (x == dx || dy == dx)) return LQ_ERR_INVALID_ARG;
    if (max_rank > LQ_MAX_RANK || n_adapters > LQ_MAX_ADAPTERS) return LQ_ERR_UNSUPPORTED;
    if ((d_in % 8) || (d_out % 8) || (ldx % 8) || (lddx % 8) || (lddy % 8) || !aligned16(x) || !aligned16(dy) || !aligned16(dx))
        return LQ_ERR_UNSUPPORTED;
    if (!workspace || !aligned16(workspace) ||
        workspace_bytes < lora_backward_workspace_bytes(n_tokens, n_adapters, max_rank, d_in, d_out))
        return LQ_ERR_WORKSPACE;
    if (n_tokens == 0 || max_segments == 0) return LQ_OK;

    int seg_bound = max_segments;
    if (seg_bound > n_tokens) seg_bound = n_tokens;
    if (seg_bound > n_adapters) seg_bound = n_adapters;  // fine-tune segments only
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);

    // 1. g = dy B^T on fine-tune rows: the forward's shrink over d_out against B
    FwdParams s1;
    s1.x = static_cast<const u16*>(dy); s1.ldx = lddy;
    s1.y = static_cast<u16*>(dx); s1.ldy = lddx;
    s1.d_in = d_out; s1.d_out = d_in;
    s1.A_ptrs = B_ptrs; s1.B_ptrs = A_ptrs; s1.ranks = ranks; s1.scales = scales;
    s1.n_adapters = n_adapters; s1.max_rank = max_rank;
    s1.perm = perm; s1.n_tokens = n_tokens;
    s1.seg_starts = seg_starts; s1.seg_adapter = seg_adapter; s1.seg_kind = seg_kind;
    s1.n_segments = n_segments; s1.max_segments = max_segments;
    s1.h_out = nullptr; s1.h_offsets = nullptr;
    s1.hpart = reinterpret_cast<float*>(ws + kWsHeaderBytes);
    s1.ksplit = 1; s1.rstride = rstride_for(max_rank);
    s1.err = reinterpret_cast<int*>(ws); s1.tickets = reinterpret_cast<int*>(ws) + 4;
    s1.ksplit_hint = 0; s1.kinds = kFinetuneOnly;
    if (run_shrink_expand(s1, LQ_VARIANT_SHRINK_ONLY, seg_bound, st) != hipSuccess) return LQ_ERR_HIP;

    // 2. partial weight gradients, then their reduction into dA / dB
    if (dA_ptrs || dB_ptrs) {
        BwdParams b;
        b.x = static_cast<const u16*>(x); b.ldx = ldx;
        b.dy = static_cast<const u16*>(dy); b.lddy = lddy;
        b.d_in = d_in; b.d_out = d_out;
        b.dA_ptrs = dA_ptrs; b.dB_ptrs = dB_ptrs; b.A_ptrs = A_ptrs; b.B_ptrs = B_ptrs;
        b.ranks = ranks; b.scales = scales; b.n_adapters = n_adapters; b.max_rank = max_rank;
        b.perm = perm; b.n_tokens = n_tokens;
        b.seg_starts = seg_starts; b.seg_adapter = seg_adapter; b.seg_kind = seg_kind;
        b.n_segments = n_segments; b.max_segments = max_segments;
        b.h_saved = h_saved; b.h_offsets = reinterpret_cast<const long long*>(h_offsets);
        b.g = s1.hpart; b.ksplit = s1.ksplit; b.rstride = s1.rstride;
        b.wpart = reinterpret_cast<float*>(ws + kWsHeaderBytes + h_slices_bytes(n_tokens, max_rank));
        b.err = reinterpret_cast<int*>(ws);
        const hipError_t e = max_rank <= 16 ? launch_wgrad<1>(b, st) : max_rank <= 32 ? launch_wgrad<2>(b, st)
                           : max_rank <= 64 ? launch_wgrad<4>(b, st) : launch_wgrad<8>(b, st);
        if (e != hipSuccess) return LQ_ERR_HIP;
        hipLaunchKernelGGL(wreduce_kernel, dim3(512), dim3(kThreads), 0, st, b);
        if (hipGetLastError() != hipSuccess) return LQ_ERR_HIP;
    }

    // 3. dx += s g A on fine-tune rows: the forward's expand over d_in against A, with the same k split
    s1.ksplit_hint = s1.ksplit;
    return run_shrink_expand(s1, LQ_VARIANT_EXPAND_ONLY, seg_bound, st) == hipSuccess ? LQ_OK : LQ_ERR_HIP;
}
