// Backward of the segmented LoRA update for fine-tune segments.  The paper leaves this to autograd, one
// call per LoRA linear, and names a dedicated kernel as future work (Section 4.2, Appendix A); this is
// the exact gradient of the forward defined in lqlora.h, with g = dy B^T:
//     dx += s g A            dB += s h^T dy            dA += s g^T x
// g = dy B^T is the forward's shrink with the roles (x, A, d_in) := (dy, B, d_out), and dx += s g A is
// the forward's expand with (y, B, d_out) := (dx, A, d_in); both reuse those kernels, restricted to
// fine-tune segments.  The two weight gradients are contractions over the TOKEN axis, which is the
// strided axis of every operand, so they get a kernel of their own:
//   weight-gradient unit : 512 rows of a fine-tune segment x 256 columns of dy (for dB, with h) or of x
//                          (for dA, with g).  32 rows at a time are staged in LDS with coalesced loads
//                          (four steps in flight in registers, two LDS buffers) and read back
//                          transposed into 16x16x32 bf16 MFMA fragments; h and g are split into bf16
//                          high and low parts.  A segment of up to 512 rows is one unit per column block,
//                          which adds its [rank x 256] result straight into dA / dB; a longer segment is
//                          cut into row chunks whose units store their partials to the workspace.
//   reduce unit          : one cut segment x 512 columns x 8 ranks: adds the segment's partials in chunk
//                          order, applies the scale and accumulates into dA / dB.  Fixed order, so
//                          reproducible.
// (Tried: the unit that stores the last partial of a (segment, column block) adds the partials up, so that no
// reduction launch is needed.  The partials then have to be stored and read with device-scope accesses, and
// every unit ends with a wait for its stores, an arrival and, for the last one, a round of loads: the
// weight-gradient launch went from 28 to 44 us on the layer stack, against 8 us for the reduction launch.)
#include "lq_internal.h"
#include <hip/amd_detail/amd_hip_unsafe_atomics.h>
#include <type_traits>
#include <utility>

namespace lq {
namespace {

constexpr int kWgRows = 512;    // token rows per weight-gradient unit
constexpr int kWgCols = 256;    // columns per unit (8 waves x 32)
constexpr int kWgTiles = kWgCols / (8 * 16);  // 16-column MFMA tiles per wave

constexpr int kStepRows = 32;   // token rows per MFMA k step
constexpr int kBig = 0x7fffffff;

struct BwdParams {
    const u16* x; long long ldx;
    const u16* dy; long long lddy;
    int d_in, d_out;
    float* const* dA_ptrs; float* const* dB_ptrs;
    const void* const* A_ptrs; const void* const* B_ptrs;  // only for the table helpers
    const int32_t* ranks; const float* scales; int n_adapters; int max_rank;
    const float* token_scales;  // per token row; when given it replaces scales[adapter] and moves inside the sums over tokens
    const int32_t* perm; int n_tokens;
    const int32_t* seg_starts; const int32_t* seg_adapter; const uint8_t* seg_kind;
    const int32_t* n_segments; int max_segments;
    const float* h_saved; const long long* h_offsets;
    const float* g;      // g = dy B^T of the fine-tune rows, laid out like h_saved
    int rstride;
    float* wpart;        // [chunk of a segment with more than 512 rows][rstride][d_out + d_in] partial weight gradients
    int* err;
};

template <int NT>
struct WgCfg {
    static constexpr int YPITCH = kWgCols + 8;                 // u16 elements per staged activation row
    static constexpr int HPITCH = 16 * NT + 8;                 // u16 elements per staged row of h / g (high or low parts)
    static constexpr size_t Y_BYTES = (size_t)kStepRows * YPITCH * sizeof(u16);
    static constexpr size_t H_BYTES = ((size_t)2 * kStepRows * HPITCH * sizeof(u16) + 15) / 16 * 16;  // high, then low
    static constexpr size_t BUF_BYTES = Y_BYTES + H_BYTES;
    static constexpr size_t LDS_BYTES = 2 * BUF_BYTES + kWgRows * sizeof(int);
};

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ...: a loop over register slots that have to be
// indexed with constants
template <int... Js, class F>
__device__ __forceinline__ void for_each_slot(std::integer_sequence<int, Js...>, F&& f)
{
    (f(std::integral_constant<int, Js>{}), ...);
}

// D[rank][col] = sum_t H[t][rank] Y[t][col] over the unit's rows; H = h_saved (for dB, Y = dy) or g (for
// dA, Y = x).  MFMA: lane (c = lane % 16, kg = lane / 16) supplies H[8 kg ..][rank c] and Y[8 kg ..][col c]
// of a 32-row step and receives D[rank 4 kg + v][col c].
// chunk_id < 0: the unit covers its whole segment and accumulates into dA / dB (times scale); else it stores its
// partial to slot chunk_id of wpart
template <int NT>
__device__ __forceinline__ void wgrad_unit(const BwdParams& p, const Unit& u, int rank, float scale, int chunk_id, bool for_b,
                                           int col_block, unsigned char* lds)
{
    using C = WgCfg<NT>;
    constexpr int YQ = kWgCols / 128;  // 16-byte pieces of a staged activation row per thread
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

    // staging assignment: 16 threads cover 128 columns (256 bytes) of one row per pass
    const int y_row = (int)threadIdx.x / 16, y_piece = (int)threadIdx.x % 16;
    // the unit's rows of h_saved (for dB) or of g (for dA); both are [row][rank] per segment
    const float* hsrc = (for_b ? p.h_saved : p.g) + p.h_offsets[u.seg] + (long long)(u.pos - u.first) * rank;
    constexpr int DEPTH = NT == 1 ? 4 : NT == 2 ? 3 : NT == 4 ? 2 : 1;  // steps in flight (as many as the registers allow)
    u32x4 gy[DEPTH][YQ];
    float gh[DEPTH][NT + 1];  // [NT]: the row's own scale (1 when the scale is the adapter's, applied by the reduction)
    // all loads are unconditional (clamped addresses), so the number in flight is static; what lies
    // outside the unit is zeroed when it is stored to LDS
    auto stage_load = [&](int step, u32x4 (&y)[YQ], float (&h)[NT + 1]) {
        const int i = step * kStepRows + y_row;
        const int row = lds_row[min(i, kWgRows - 1)];
        const u16* yrow = Y + (long long)(row >= 0 ? row : safe_row) * ldy;
#pragma unroll
        for (int q = 0; q < YQ; ++q) y[q] = *reinterpret_cast<const u32x4*>(yrow + min(n0 + (y_piece + 16 * q) * 8, d - 8));
        const float* hrow = hsrc + (long long)min(i, u.len - 1) * rank;
#pragma unroll
        for (int q = 0; q < NT; ++q) h[q] = hrow[min(y_piece + 16 * q, rank - 1)];
        h[NT] = p.token_scales ? p.token_scales[max(row, 0)] : 1.f;
    };
    auto stage_store = [&](int step, int buf, const u32x4 (&y)[YQ], const float (&h)[NT + 1]) {
        u16* ly = reinterpret_cast<u16*>(lds + buf * C::BUF_BYTES);
        u16* lh = reinterpret_cast<u16*>(lds + buf * C::BUF_BYTES + C::Y_BYTES);
        const int i = step * kStepRows + y_row;
        const bool row_live = i < u.len && lds_row[min(i, kWgRows - 1)] >= 0;
#pragma unroll
        for (int q = 0; q < YQ; ++q) {
            const bool live = row_live && n0 + (y_piece + 16 * q) * 8 < d;
            *reinterpret_cast<u32x4*>(ly + y_row * C::YPITCH + (y_piece + 16 * q) * 8) = live ? y[q] : u32x4{0u, 0u, 0u, 0u};
        }
        // h / g as bf16 high and low parts (together ~16 mantissa bits), split here once instead of in every wave
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            const float v = (i < u.len && y_piece + 16 * q < rank) ? h[q] * h[NT] : 0.f;
            const unsigned int hi = pack_bf16x2(v, 0.f) & 0xffffu;
            const unsigned int lo = pack_bf16x2(v - bf16_lo(hi), 0.f) & 0xffffu;
            lh[y_row * C::HPITCH + y_piece + 16 * q] = (u16)hi;
            lh[(kStepRows + y_row) * C::HPITCH + y_piece + 16 * q] = (u16)lo;
        }
    };

    f32x4 acc[NT][kWgTiles];
#pragma unroll
    for (int jt = 0; jt < NT; ++jt)
#pragma unroll
        for (int nt = 0; nt < kWgTiles; ++nt) acc[jt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int buf) {
        const u16* ly = reinterpret_cast<const u16*>(lds + buf * C::BUF_BYTES);
        const u16* lh = reinterpret_cast<const u16*>(lds + buf * C::BUF_BYTES + C::Y_BYTES);
        // the staged rows are the MFMA's k axis: both operands are read back transposed
        u32x4 yf[kWgTiles];
#pragma unroll
        for (int nt = 0; nt < kWgTiles; ++nt) yf[nt] = lds_read_transposed_16x32(ly + w * (16 * kWgTiles) + nt * 16, C::YPITCH);
#pragma unroll
        for (int jt = 0; jt < NT; ++jt) {
            const u32x4 hi = lds_read_transposed_16x32(lh + jt * 16, C::HPITCH);
            const u32x4 lo = lds_read_transposed_16x32(lh + kStepRows * C::HPITCH + jt * 16, C::HPITCH);
#pragma unroll
            for (int nt = 0; nt < kWgTiles; ++nt) {
                acc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(lo), as_bf16x8(yf[nt]), acc[jt][nt], 0, 0, 0);
                acc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(hi), as_bf16x8(yf[nt]), acc[jt][nt], 0, 0, 0);
            }
        }
    };

    // Pipeline: the loads of the next DEPTH steps are in flight in registers; a step is stored to one of
    // two LDS buffers (one barrier per step: the buffer written now was last read two steps ago), its
    // register slot is refilled with the step DEPTH ahead, and the step is multiplied out of LDS.
    const int n_steps = (u.len + kStepRows - 1) / kStepRows;
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd) stage_load(min(dd, n_steps - 1), gy[dd], gh[dd]);
    auto step_fn = [&](int step, auto slot) {
        constexpr int J = decltype(slot)::value;
        stage_store(step, step & 1, gy[J], gh[J]);
        stage_load(min(step + DEPTH, n_steps - 1), gy[J], gh[J]);  // unconditional; past the end it re-reads
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        compute(step & 1);
        __builtin_amdgcn_sched_barrier(0);
    };
    for (int step = 0; step < n_steps; step += DEPTH)
        for_each_slot(std::make_integer_sequence<int, DEPTH>{}, [&](auto slot) {
            if (step + decltype(slot)::value < n_steps) step_fn(step + decltype(slot)::value, slot);
        });

    if (chunk_id < 0) {
        // Accumulation with the hardware's fp32 addition in memory: every element receives exactly one addition per
        // segment, so the result does not depend on timing as long as an adapter has one fine-tune segment (always
        // true of the builder's tables); two segments of one adapter are both added, in either order.
        float* dst = for_b ? p.dB_ptrs[u.ad] : p.dA_ptrs[u.ad];
#pragma unroll
        for (int jt = 0; jt < NT; ++jt)
#pragma unroll
            for (int nt = 0; nt < kWgTiles; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int j = jt * 16 + 4 * kg + v, n = n0 + w * (16 * kWgTiles) + nt * 16 + c;
                    if (j < rank && n < d) unsafeAtomicAdd(dst + (long long)j * d + n, scale * acc[jt][nt][v]);
                }
        return;
    }
    const int dsum = p.d_out + p.d_in;
    float* out = p.wpart + (long long)chunk_id * p.rstride * dsum + (for_b ? 0 : p.d_out);
#pragma unroll
    for (int jt = 0; jt < NT; ++jt)
#pragma unroll
        for (int nt = 0; nt < kWgTiles; ++nt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int j = jt * 16 + 4 * kg + v, n = n0 + w * (16 * kWgTiles) + nt * 16 + c;
                if (j < rank && n < d) out[(long long)j * dsum + n] = acc[jt][nt][v];
            }
}

// (ranks up to 32: at most 128 registers, so that two workgroups share a compute unit and one's loads
// overlap the other's barriers)
// the fine-tune segments with more than 512 rows are cut into chunks (partials, then the reduction); the shorter
// ones are one unit per column block
__device__ __forceinline__ LenClass cut_class() { return LenClass{kWgRows + 1, kBig, 1 << LQ_SEG_FINETUNE}; }
__device__ __forceinline__ LenClass whole_class() { return LenClass{1, kWgRows + 1, 1 << LQ_SEG_FINETUNE}; }

template <int NT>
__global__ __launch_bounds__(kThreads, NT <= 2 ? 4 : 2) void wgrad_kernel(BwdParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    int n_seg;
    const SegCache c0 = load_seg_cache(p, n_seg);
    const LenClass cut = cut_class(), whole = whole_class();
    const int blocks_b = (p.d_out + kWgCols - 1) / kWgCols, blocks_a = (p.d_in + kWgCols - 1) / kWgCols;
    const int per_chunk = blocks_b + blocks_a;
    const int n_cut = count_chunks(p, n_seg, c0, kWgRows, cut) * per_chunk;  // the (larger) chunks first
    const int n_units = n_cut + count_chunks(p, n_seg, c0, kWgRows, whole) * per_chunk;
    for (int id = (int)blockIdx.x; id < n_units; id += (int)gridDim.x) {
        Unit u;
        const bool is_cut = id < n_cut;
        const int chunk_id = small_div(is_cut ? id : id - n_cut, per_chunk), cb = (is_cut ? id : id - n_cut) - chunk_id * per_chunk;
        if (!(is_cut ? find_chunk(p, n_seg, c0, chunk_id, kWgRows, cut, u) : find_chunk(p, n_seg, c0, chunk_id, kWgRows, whole, u)))
            continue;
        if (u.ad < 0 || u.ad >= p.n_adapters) continue;  // flagged by the forward kernels already
        const int rank = p.ranks[u.ad];
        if (rank < 1 || rank > p.max_rank) continue;
        const bool for_b = cb < blocks_b;
        if (for_b ? (p.dB_ptrs == nullptr || p.dB_ptrs[u.ad] == nullptr) : (p.dA_ptrs == nullptr || p.dA_ptrs[u.ad] == nullptr))
            continue;
        const float scale = p.token_scales ? 1.f : p.scales[u.ad];  // (per-token scales were applied row by row)
        wgrad_unit<NT>(p, u, rank, scale, is_cut ? chunk_id : -1, for_b, for_b ? cb : cb - blocks_b, lds_raw);
    }
}

// dA / dB += scale * (sum of a cut segment's chunk partials, in chunk order).  One unit = the first chunk of
// a segment x 512 columns of [dB | dA] x 8 ranks; a thread owns one column and keeps the 8 sums in
// registers, so the loads of a chunk's partials are independent of each other.  The accumulation is the
// hardware's fp32 addition in memory, one per element and segment (see wgrad_unit).
constexpr int kRedRanks = 8;
__global__ __launch_bounds__(kThreads) void wreduce_kernel(BwdParams p)
{
    int n_seg;
    const SegCache c0 = load_seg_cache(p, n_seg);
    const LenClass cut = cut_class();
    const int dsum = p.d_out + p.d_in;
    const int col_blocks = (dsum + kThreads - 1) / kThreads;
    const int rank_groups = (p.max_rank + kRedRanks - 1) / kRedRanks;
    const int per_chunk = col_blocks * rank_groups;
    const int n_units = count_chunks(p, n_seg, c0, kWgRows, cut) * per_chunk;
    for (int id = (int)blockIdx.x; id < n_units; id += (int)gridDim.x) {
        Unit u;
        const int chunk_id = small_div(id, per_chunk), sub = id - chunk_id * per_chunk;
        if (!find_chunk(p, n_seg, c0, chunk_id, kWgRows, cut, u)) continue;
        if (u.pos != u.first) continue;  // only the segment's first chunk adds up the segment
        if (u.ad < 0 || u.ad >= p.n_adapters) continue;
        const int n_chunks = (u.seg_len + kWgRows - 1) / kWgRows;
        const int j0 = (sub / col_blocks) * kRedRanks;
        const int col = (sub % col_blocks) * kThreads + (int)threadIdx.x;
        if (col >= dsum) continue;
        const float* __restrict__ part = p.wpart + ((long long)chunk_id * p.rstride + j0) * dsum + col;
        // Four chunks' partials are requested together (a chunk that does not exist re-reads the last one and is not
        // added): one round trip for the segments of the layer stack instead of one per chunk; the additions keep
        // the chunk order.  The first four go out before the adapter's rank, scale and pointer are asked for: where
        // the partials lie depends on the tables alone (rows beyond the rank lie inside the rstride rows of a partial).
        float v[4][kRedRanks];
        auto request = [&](int cc) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int jj = 0; jj < kRedRanks; ++jj) v[k][jj] = part[((long long)min(cc + k, n_chunks - 1) * p.rstride + jj) * dsum];
        };
        request(0);
        __builtin_amdgcn_sched_barrier(0);
        const int rank = p.ranks[u.ad];
        const float scale = p.token_scales ? 1.f : p.scales[u.ad];  // (per-token scales were applied row by row)
        const bool for_b = col < p.d_out;
        float* __restrict__ dst = for_b ? (p.dB_ptrs ? p.dB_ptrs[u.ad] : nullptr) : (p.dA_ptrs ? p.dA_ptrs[u.ad] : nullptr);
        if (rank < 1 || rank > p.max_rank || j0 >= rank || !dst) continue;
        const int d = for_b ? p.d_out : p.d_in, n = for_b ? col : col - p.d_out;
        float sum[kRedRanks];
#pragma unroll
        for (int jj = 0; jj < kRedRanks; ++jj) sum[jj] = 0.f;
        for (int cc = 0; cc < n_chunks; cc += 4) {
            if (cc > 0) request(cc);
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int jj = 0; jj < kRedRanks; ++jj) sum[jj] = cc + k < n_chunks ? sum[jj] + v[k][jj] : sum[jj];
        }
#pragma unroll
        for (int jj = 0; jj < kRedRanks; ++jj)
            if (j0 + jj < rank) unsafeAtomicAdd(dst + (long long)(j0 + jj) * d + n, scale * sum[jj]);
    }
}

// finished g of the fine-tune rows: at most n_tokens x max_rank floats (a multiple of 16 bytes)
size_t gsum_bytes(int n_tokens, int max_rank) { return ((size_t)n_tokens * (size_t)max_rank * sizeof(float) + 15) / 16 * 16; }

// Only segments with more than 512 rows keep partials: n such segments have at most n_tokens / 512 + n chunks
// and n <= n_tokens / 513, whatever tables the caller passes.
size_t wpart_bytes(int n_tokens, int max_rank, int d_in, int d_out)
{
    const size_t chunks = 2 * ((size_t)(n_tokens + kWgRows - 1) / kWgRows);
    return chunks * (size_t)rstride_for(max_rank) * ((size_t)d_in + d_out) * sizeof(float);
}

template <int NT>
hipError_t launch_wgrad(const BwdParams& p, hipStream_t st)
{
    static DeviceGrid cache;
    constexpr size_t lds = WgCfg<NT>::LDS_BYTES;
    const int grid = cache.get([] {
        int dev = 0, cus = 0, per_cu = 0;
        if (lds > 48 * 1024)
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(wgrad_kernel<NT>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipGetDevice(&dev);
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, wgrad_kernel<NT>, kThreads, lds) != hipSuccess || per_cu <= 0)
            per_cu = 1;
        return cus * per_cu;
    });
    return launch_kernel(kKernelWgrad, wgrad_kernel<NT>, dim3(grid), dim3(kThreads), lds, st, p);
}

}  // namespace
}  // namespace lq

// workspace: [header 4096 B][g slices: like the forward's partial h][finished g][partial weight gradients]
extern "C" size_t lora_backward_workspace_bytes(int32_t n_tokens, int32_t n_adapters, int32_t max_rank, int32_t d_in,
                                                int32_t d_out)
{
    (void)n_adapters;
    if (n_tokens < 0 || max_rank < 1 || d_in < 0 || d_out < 0) return lq::kWsHeaderBytes;
    return (size_t)lq::kWsHeaderBytes + lq::h_slices_bytes(n_tokens, max_rank) + lq::gsum_bytes(n_tokens, max_rank) +
           lq::wpart_bytes(n_tokens, max_rank, d_in, d_out);
}

extern "C" lq_status lora_segmented_backward(const void* x, int64_t ldx, const void* dy, int64_t lddy, void* dx,
                                             int64_t lddx, int32_t d_in, int32_t d_out,
                                             const void* const* A_ptrs, const void* const* B_ptrs,
                                             float* const* dA_ptrs, float* const* dB_ptrs,
                                             const int32_t* ranks, const float* scales, const float* token_scales,
                                             int32_t n_adapters, int32_t max_rank, const int32_t* perm, int32_t n_tokens,
                                             const int32_t* seg_starts, const int32_t* seg_adapter,
                                             const uint8_t* seg_kind, const int32_t* n_segments, int32_t max_segments,
                                             const float* h_saved, const int64_t* h_offsets,
                                             int32_t variant, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace lq;
    if (n_tokens < 0 || d_in <= 0 || d_out <= 0 || n_adapters <= 0 || max_segments < 0 || max_rank < 1)
        return LQ_ERR_INVALID_ARG;
    if (variant != LQ_VARIANT_SPLIT && variant != LQ_VARIANT_FUSED && variant != LQ_VARIANT_SLAB && variant != LQ_VARIANT_AUTO)
        return LQ_ERR_INVALID_ARG;
    if (variant == LQ_VARIANT_AUTO) variant = auto_variant(max_rank, d_in);  // (the step's outputs are dx's columns)
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

    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);

    // 1. g = dy B^T on fine-tune rows: the forward's shrink over d_out against B
    FwdParams s1;
    s1.x = static_cast<const u16*>(dy); s1.ldx = lddy;
    s1.d_in = d_out;
    Proj q;
    q.y = static_cast<u16*>(dx); q.ldy = lddx; q.d_out = d_in;
    q.A_ptrs = B_ptrs; q.B_ptrs = A_ptrs;
    s1.ranks = ranks; s1.scales = scales;
    s1.n_adapters = n_adapters; s1.max_rank = max_rank;
    s1.token_scales = token_scales;
    s1.perm = perm; s1.n_tokens = n_tokens;
    s1.seg_starts = seg_starts; s1.seg_adapter = seg_adapter; s1.seg_kind = seg_kind;
    s1.n_segments = n_segments; s1.max_segments = max_segments;
    // the finished g goes where the forward would save h: [segment offset + row x rank + j], for the weight gradients
    float* gsum = reinterpret_cast<float*>(ws + kWsHeaderBytes + h_slices_bytes(n_tokens, max_rank));
    const bool want_w = dA_ptrs || dB_ptrs;
    q.h_out = want_w ? gsum : nullptr; s1.h_offsets = want_w ? reinterpret_cast<const long long*>(h_offsets) : nullptr;
    s1.n_proj = 1;
    s1.proj0 = q;
    for (int k = 1; k < kMaxProj; ++k) s1.more[k - 1] = q;
    s1.hpart = reinterpret_cast<float*>(ws + kWsHeaderBytes);
    s1.hproj = 0;
    s1.ksplit = 1; s1.rstride = rstride_for(max_rank);
    s1.header = s1.err = reinterpret_cast<int*>(ws); s1.tickets = reinterpret_cast<int*>(ws) + 4;
    s1.ksplit_hint = 0; s1.kinds = kFinetuneOnly;
    // 2. dx += s g A on fine-tune rows: the forward's expand over d_in against A.  LQ_VARIANT_FUSED: both in a
    // single launch when its buffer descriptor can address the slices; else two launches with the same k split.
    // Whichever phase finishes g (the shrink without a split, the expand with one) also stores it to gsum.
    const bool one_launch = variant == LQ_VARIANT_FUSED && h_slices_bytes(n_tokens, max_rank) <= 0x7fffffffull;
    s1.coherent = one_launch; s1.hpart_bytes = one_launch ? (unsigned int)h_slices_bytes(n_tokens, max_rank) : 0;
    if (variant == LQ_VARIANT_SLAB) {
        if (run_slab(s1, st) != hipSuccess) return LQ_ERR_HIP;
    } else if (one_launch) {
        if (run_shrink_expand(s1, LQ_VARIANT_FUSED, st) != hipSuccess) return LQ_ERR_HIP;
    } else {
        if (run_shrink_expand(s1, LQ_VARIANT_SHRINK_ONLY, st) != hipSuccess) return LQ_ERR_HIP;
        s1.ksplit_hint = s1.ksplit;
        if (run_shrink_expand(s1, LQ_VARIANT_EXPAND_ONLY, st) != hipSuccess) return LQ_ERR_HIP;
    }

    // 3. partial weight gradients (from x, dy, the saved h and the finished g), then their reduction into dA / dB
    if (dA_ptrs || dB_ptrs) {
        BwdParams b;
        b.x = static_cast<const u16*>(x); b.ldx = ldx;
        b.dy = static_cast<const u16*>(dy); b.lddy = lddy;
        b.d_in = d_in; b.d_out = d_out;
        b.dA_ptrs = dA_ptrs; b.dB_ptrs = dB_ptrs; b.A_ptrs = A_ptrs; b.B_ptrs = B_ptrs;
        b.ranks = ranks; b.scales = scales; b.n_adapters = n_adapters; b.max_rank = max_rank;
        b.token_scales = token_scales;
        b.perm = perm; b.n_tokens = n_tokens;
        b.seg_starts = seg_starts; b.seg_adapter = seg_adapter; b.seg_kind = seg_kind;
        b.n_segments = n_segments; b.max_segments = max_segments;
        b.h_saved = h_saved; b.h_offsets = reinterpret_cast<const long long*>(h_offsets);
        b.g = gsum; b.rstride = s1.rstride;
        b.wpart = reinterpret_cast<float*>(ws + kWsHeaderBytes + h_slices_bytes(n_tokens, max_rank) + gsum_bytes(n_tokens, max_rank));
        b.err = reinterpret_cast<int*>(ws);
        const hipError_t e = max_rank <= 16 ? launch_wgrad<1>(b, st) : max_rank <= 32 ? launch_wgrad<2>(b, st)
                           : max_rank <= 64 ? launch_wgrad<4>(b, st) : launch_wgrad<8>(b, st);
        if (e != hipSuccess) return LQ_ERR_HIP;
        // (no segment of a batch of up to 512 tokens is cut into chunks: nothing to reduce)
        if (n_tokens > kWgRows && launch_kernel(kKernelWreduce, wreduce_kernel, dim3(512), dim3(kThreads), 0, st, b) != hipSuccess)
            return LQ_ERR_HIP;
    }
    return LQ_OK;
}
