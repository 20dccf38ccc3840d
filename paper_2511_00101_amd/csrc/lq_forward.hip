// Segmented multi-adapter LoRA forward (Section 3.3): shrink (h = x A_a^T per segment), h-save for
// fine-tune segments, expand (y += s_a h B_a).
//
// Every workgroup (8 waves) reads the segment tables itself, so the grids are a fixed number of
// resident workgroups that stride over "units"; no plan buffer or extra launch is needed.
//
//   shrink, tall unit  : up to 128 rows of a segment with more than 32 rows (longer segments are cut into
//                        even chunks) x one of `ksplit` slices of d_in.  A GEMM with a skinny output:
//                        each wave owns 16 rows and streams its x rows straight into MFMA fragments;
//                        the 256-wide k stage of A_a is staged in LDS once per workgroup (coalesced
//                        loads, double buffered) and shared by the 8 waves, so A_a crosses the L2->L1
//                        path once per chunk.
//   shrink, short unit : a segment of at most 32 rows x one slice of d_in.  GEMV-like: the 8 waves take
//                        alternate 64-wide k blocks of x and A_a and add their results through LDS in
//                        a fixed order.  The MFMA does the k reduction even when few rows are live.
//   (with ksplit > 1 every shrink unit stores the h of its slice and the expand kernel adds the slices
//    in order, so no workgroup waits for another and the sum does not depend on timing)
//   expand, long unit  : up to 512 rows (256 for ranks above 32) of a segment with >= 16 rows x a group of 512-column blocks of
//                        d_out.  The B_a block is staged in LDS and transposed into MFMA fragments
//                        that stay in registers; the unit's h rows are scaled, split into bf16 high and
//                        low parts and laid out as fragments in LDS once; then y streams by, 32 rows
//                        per step, read-modify-write.
//   expand, short unit : one wave: <= 4 rows of a segment with < 16 rows x 512 columns.  B_a rows are
//                        streamed with 16-byte loads, h is broadcast from LDS, plain FMAs.
// x and y are accessed with 16-byte loads/stores straight in the MFMA operand layout (16 rows x 64
// contiguous bytes per instruction); on MI355X that streams from HBM within a few percent of a
// row-contiguous pattern as long as nothing else competes for the address path, which is why A_a, B_a
// and h reach the MFMA through LDS instead.
#include "lq_internal.h"
#include <algorithm>
#include <mutex>
#include <type_traits>

namespace lq {
namespace {

constexpr int kTallMin = 33;     // shrink: segments with at least this many rows take the row-split path
constexpr int kTallRows = 128;   // shrink, tall unit: rows (8 waves x 16)
constexpr int kStageK = 256;     // shrink, tall unit: k elements of A staged per step
constexpr int kShortRows = 32;   // shrink, short unit: rows (two 16-row MFMA tiles)
constexpr int kBlockK = 64;      // shrink: k elements per wave step (two MFMA k steps)
constexpr int kLongMin = 16;     // expand: segments with at least this many rows take the MFMA path
constexpr int kTT = 4;           // expand, short unit: rows
constexpr int kShortN = 512;     // expand, short unit: columns (64 lanes x 8)
constexpr int kMaxKSplit = 8;
constexpr int kBig = 0x7fffffff;


// In the fused variant the h slices cross the barrier between workgroups on different XCDs, whose L2
// caches are not coherent with each other.  There they are written and read with device-scope accesses,
// which go past the L2's non-coherent lines, so that the barrier needs no cache write-back or
// invalidation (measured: those cost ~9 us per barrier with 256 workgroups).
__device__ __forceinline__ void h_store(float* ptr, float v, bool coherent)
{
    if (coherent) __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *ptr = v;
}
__device__ __forceinline__ float h_load(const float* ptr, bool coherent)
{
    return coherent ? __hip_atomic_load(const_cast<float*>(ptr), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *ptr;
}
// eight consecutive floats of hpart (16-byte aligned).  The device-scope form is a buffer load with the sc1
// cache policy: plain C++ has no 16-byte atomic load.
template <class PP>
__device__ __forceinline__ void h_load8(const PP& p, const float* ptr, f32x4& a, f32x4& b)
{
    if (!p.coherent) {
        a = *reinterpret_cast<const f32x4*>(ptr);
        b = *reinterpret_cast<const f32x4*>(ptr + 4);
    } else {
        constexpr int kRawBuffer = 0x00020000, kSc1 = 16;  // descriptor word 3 (raw 32-bit data); cache policy bit
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(p.hpart, 0, (int)p.hpart_bytes, kRawBuffer);
        const int off = (int)(reinterpret_cast<const char*>(ptr) - reinterpret_cast<const char*>(p.hpart));
        a = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, kSc1));
        b = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off + 16, 0, kSc1));
    }
}

// Where a shrink unit stores its h values: slice ks of the partial-h buffer.  With ksplit == 1 that is
// the finished h, and fine-tune segments store it to h_out as well; with ksplit > 1 the expand kernel
// adds the slices in order (and stores h_out), so no workgroup ever waits for another.
struct HDest { float* base; float* save; int save_ld; };
template <class PP>
__device__ __forceinline__ HDest h_dest(const PP& p, const Unit& u, const SegInfo& s, int ks, int nsplit)
{
    HDest d;
    d.base = p.hpart + u.pi * p.hproj + ((long long)ks * p.n_tokens + u.pos) * p.rstride;
    float* h_out = proj_of(p, u.pi).h_out;
    const bool save = nsplit == 1 && u.kd == LQ_SEG_FINETUNE && h_out && p.h_offsets;
    d.save = save ? h_out + p.h_offsets[u.seg] + (long long)(u.pos - u.first) * s.rank : nullptr;
    d.save_ld = s.rank;
    return d;
}

// finished h of one element: the slices added in order
template <class PP>
__device__ __forceinline__ float h_sum(const PP& p, int pi, long long pos, int j, int parts)
{
    // the first four slices are requested together (a slice that does not exist re-reads the last one and is
    // not added): one round trip instead of one per slice
    const long long slice = (long long)p.n_tokens * p.rstride;
    const float* at = p.hpart + pi * p.hproj + pos * p.rstride + j;
    float v[4];
#pragma unroll
    for (int part = 0; part < 4; ++part) v[part] = h_load(at + min(part, parts - 1) * slice, p.coherent);
    float sum = v[0];
#pragma unroll
    for (int part = 1; part < 4; ++part) sum += part < parts ? v[part] : 0.f;
    for (int part = 4; part < parts; ++part) sum += h_load(at + part * slice, p.coherent);
    return sum;
}

// =================================================================================================
// shrink, tall unit.  D[row][rank] = sum_k x[row][k] A[rank][k] with 16x16x32 bf16 MFMA: lane
// (c = lane % 16, kg = lane / 16) supplies x[row c][8 kg ..] and A[rank c][8 kg ..] of a 32-wide k step
// and receives D[row 4 kg + v][rank c].  d_in is cut into 256-wide stages; a slice is a run of
// consecutive stages.
// =================================================================================================
// ROWWISE: x is loaded row-wise (an instruction covers 2 rows x 512 contiguous bytes, which streams from HBM
// up to a quarter faster than the MFMA layout's 16 rows x 64 bytes when few units share a compute unit) and
// reaches the MFMA layout through a slab of LDS that belongs to the wave (`slabs`: 8 x 16 rows).
template <int NT, bool ROWWISE, class PP>  // 16-rank tiles: ranks up to 16 * NT
__device__ __forceinline__ void shrink_tall_unit(const PP& p, const Unit& u, const SegInfo& s, int ks, u16* lds,
                                                 u16* slabs)
{
    constexpr int PITCH = kStageK + 8;           // elements per staged A row or slab row (16-byte aligned, bank spread)
    constexpr int BUF = NT * 16 * PITCH;         // elements per stage buffer
    constexpr int NB = kStageK / kBlockK;        // x blocks per stage
    const int lane = lane_id(), w = uniform((int)threadIdx.x / kWave), c = lane & 15, kg = lane >> 4;
    const bool wave_live = w * 16 < u.len;

    const int i_row = w * 16 + c;
    const int row = i_row < u.len ? row_of(p, u.pos + i_row) : -1;
    const int safe_row = max(row_of(p, u.pos), 0);
    const u16* xrow = p.x + (long long)(row >= 0 ? row : safe_row) * p.ldx;
    // row-wise: instruction i of a stage covers rows 2 i and 2 i + 1 of the wave's 16, 32 lanes each
    const u16* xrw[ROWWISE ? 8 : 1];
    u16* slab = slabs + w * 16 * PITCH;
    if constexpr (ROWWISE) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = __shfl(row, 2 * i + (lane >> 5), kWave);  // lane c of the wave holds the wave's row c
            xrw[i] = p.x + (long long)(r >= 0 ? r : safe_row) * p.ldx + (lane & 31) * 8;
        }
    }

    // Stages of this slice, visited from a tile-dependent start with wrap-around: workgroups that run
    // side by side would otherwise sweep the same k range of different rows in step, which (with a
    // power-of-two row pitch) keeps hitting the same few HBM channels.
    const int n_stages = (p.d_in + kStageK - 1) / kStageK;
    const int n_per = (n_stages + p.ksplit - 1) >> p.ks_log2;  // slice ks = stages [ks n_per, (ks + 1) n_per)
    const int n_my = max(0, min(n_per, n_stages - ks * n_per));
    const int rot = n_my > 0 ? (int)(((unsigned)u.pos / kTallRows * 5u) % (unsigned)n_my) : 0;
    auto stage_of = [&](int i) {
        i += rot;
        if (i >= n_my) i -= n_my;
        return ks * n_per + i;
    };

    // staging assignment: 32 threads cover the 512 bytes of one A row, 16 rows per pass
    const int a_row = (int)threadIdx.x / 32, a_col = ((int)threadIdx.x % 32) * 8;
    auto stage_load = [&](int stage, u32x4 (&ga)[NT]) {
        const int k = stage * kStageK + a_col;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int j = nt * 16 + a_row;
            const u32x4 v = *(gconst_u32x4)(s.A + (long long)min(j, s.rank - 1) * p.d_in + min(k, p.d_in - 8));
            ga[nt] = (j < s.rank && k < p.d_in) ? v : u32x4{0u, 0u, 0u, 0u};  // zeros beyond the rank and beyond d_in
        }
    };
    auto stage_store = [&](int buf, const u32x4 (&ga)[NT]) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            *reinterpret_cast<u32x4*>(lds + buf * BUF + (nt * 16 + a_row) * PITCH + a_col) = ga[nt];
    };
    // x of a whole stage (4 blocks of 64 k) for this wave's 16 rows.  Past d_in the address is clamped
    // into the row; the staged A is zero there, so those products vanish.
    auto xload = [&](int stage, u32x4 (&xv)[NB][2]) {
        if constexpr (ROWWISE) {
            // (a lane's 8 columns lie wholly inside or wholly beyond d_in; beyond, it re-reads column 0)
            const int k0 = stage * kStageK + (lane & 31) * 8 < p.d_in ? stage * kStageK : -(lane & 31) * 8;
#pragma unroll
            for (int i = 0; i < 8; ++i) xv[i >> 1][i & 1] = *reinterpret_cast<const u32x4*>(xrw[i] + k0);
        } else {
            const int k0 = stage * kStageK + kg * 8;
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    xv[b][q] = *reinterpret_cast<const u32x4*>(xrow + min(k0 + b * kBlockK + 32 * q, p.d_in - 8));
        }
    };
    f32x4 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto mma = [&](const u32x4 (&xv)[NB][2], int buf) {
        if constexpr (ROWWISE) {  // the stage's x into the wave's slab as it was loaded: row 2 i + lane / 32
#pragma unroll
            for (int i = 0; i < 8; ++i)
                *reinterpret_cast<u32x4*>(slab + (2 * i + (lane >> 5)) * PITCH + (lane & 31) * 8) = xv[i >> 1][i & 1];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                u32x4 xf = xv[b][q];
                if constexpr (ROWWISE) xf = *reinterpret_cast<const u32x4*>(slab + c * PITCH + b * kBlockK + 32 * q + kg * 8);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const u32x4 af = *reinterpret_cast<const u32x4*>(lds + buf * BUF + (nt * 16 + c) * PITCH +
                                                                     b * kBlockK + 32 * q + kg * 8);
                    acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(xf), as_bf16x8(af), acc[nt], 0, 0, 0);
                }
            }
        if constexpr (ROWWISE) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();  // the slab is rewritten at the next stage
        }
    };

    // Pipeline: while stage i is multiplied out of LDS (A) and registers (x), the A piece of stage i + 1
    // is in flight to registers (stored to the other LDS buffer at the top of the next iteration), and so
    // is this wave's x of the next XB - 1 stages: two stages ahead where the registers allow it, which
    // doubles the bytes a compute unit keeps in flight.  A is requested before x in every iteration, so
    // the wait for A at the top of an iteration leaves the newest x stage in flight.  All loads are
    // unconditional (past the end they re-read the last stage), so the count in flight is static.
    constexpr int XB = NT <= 2 ? 3 : 2;
    u32x4 ga[NT], xr[XB][NB][2];
    if (n_my > 0) {
        stage_load(stage_of(0), ga);
#pragma unroll
        for (int b = 0; b < XB - 1; ++b) xload(stage_of(min(b, n_my - 1)), xr[b]);
    }
    auto step = [&](int i, auto slot) {
        constexpr int J = decltype(slot)::value;
        stage_store(i & 1, ga);
        stage_load(stage_of(min(i + 1, n_my - 1)), ga);
        xload(stage_of(min(i + XB - 1, n_my - 1)), xr[(J + XB - 1) % XB]);
        __syncthreads();  // one barrier per stage: the buffer written now was last read two stages ago
        __builtin_amdgcn_sched_barrier(0);
        if (wave_live) mma(xr[J], i & 1);
        __builtin_amdgcn_sched_barrier(0);
    };
    for (int i = 0; i < n_my; i += XB) {
        step(i, std::integral_constant<int, 0>{});
        if (i + 1 >= n_my) break;
        step(i + 1, std::integral_constant<int, 1>{});
        if constexpr (XB == 3) {
            if (i + 2 >= n_my) break;
            step(i + 2, std::integral_constant<int, 2>{});
        }
    }

    const HDest d = h_dest(p, u, s, ks, p.ksplit);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = w * 16 + kg * 4 + v, j = nt * 16 + c;
            if (i < u.len && j < s.rank) {
                h_store(d.base + (long long)i * p.rstride + j, acc[nt][v], p.coherent);
                if (d.save) d.save[(long long)i * d.save_ld + j] = acc[nt][v];
            }
        }
}

// =================================================================================================
// shrink, short unit: <= 32 rows; the 8 waves take alternate 64-wide k blocks (block b belongs to slice
// (b / 8) % ksplit and wave b % 8) and tree-reduce their accumulators through LDS in a fixed order.
// =================================================================================================
template <int NT, class PP>
__device__ __forceinline__ void shrink_short_unit(const PP& p, const Unit& u, const SegInfo& s, int ks, float* lds)
{
    constexpr int MT = kShortRows / 16;
    const int lane = lane_id(), w = uniform((int)threadIdx.x / kWave), c = lane & 15, kg = lane >> 4;

    // Rows and ranks beyond the live ones read a live row instead: MFMA rows and columns are independent,
    // and the results of such rows and columns are never stored.  So the loads need no branches.
    const int safe_row = max(row_of(p, u.pos), 0);
    const u16* xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int i = mt * 16 + c;
        const int row = i < u.len ? row_of(p, u.pos + i) : -1;
        xrow[mt] = p.x + (long long)(row >= 0 ? row : safe_row) * p.ldx + kg * 8;
    }
    gconst_u16 arow[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) arow[nt] = s.A + (long long)min(nt * 16 + c, s.rank - 1) * p.d_in + kg * 8;
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Workgroups that run side by side would otherwise sweep the same k range of different rows in step,
    // which (with a power-of-two row pitch) keeps hitting the same few HBM channels; so every tile starts
    // its sweep at a different block and wraps around.
    const int n_full = p.d_in / kBlockK;  // blocks that lie fully inside d_in; a shorter last block may follow
    const int rot = n_full > 0 ? (int)(((unsigned)u.pos * 37u) % (unsigned)n_full) : 0;  // same for all slices
    auto load = [&](int blk, u32x4 (&xv)[MT][2], u32x4 (&av)[NT][2]) {  // a block that lies fully inside d_in
        blk += rot;
        if (blk >= n_full) blk -= n_full;
        // A first: its addresses are known before the row indices (which x needs) have arrived
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) av[nt][q] = *(gconst_u32x4)(arow[nt] + blk * kBlockK + 32 * q);
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xv[mt][q] = *reinterpret_cast<const u32x4*>(xrow[mt] + blk * kBlockK + 32 * q);
    };
    auto mma = [&](const u32x4 (&xv)[MT][2], const u32x4 (&av)[NT][2]) {
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(xv[mt][q]), as_bf16x8(av[nt][q]),
                                                                          acc[mt][nt], 0, 0, 0);
    };

    const int stride = kWaves * p.ksplit;
    int blk = ks * kWaves + w;
    if constexpr (NT <= 4) {
        // Two blocks in flight per wave.  The prefetch is unconditional (past the end it re-reads the
        // current block) so that the number of loads in flight is static and the wait before the MFMAs
        // covers only the older block.
        u32x4 xa[MT][2], aa[NT][2], xb[MT][2], ab[NT][2];
        if (blk < n_full) {
            load(blk, xa, aa);
            while (true) {
                bool more = blk + stride < n_full;
                load(more ? blk + stride : blk, xb, ab);
                __builtin_amdgcn_sched_barrier(0);  // keep the prefetch ahead of the MFMAs
                mma(xa, aa);
                __builtin_amdgcn_sched_barrier(0);
                if (!more) break;
                blk += stride;
                more = blk + stride < n_full;
                load(more ? blk + stride : blk, xa, aa);
                __builtin_amdgcn_sched_barrier(0);
                mma(xb, ab);
                __builtin_amdgcn_sched_barrier(0);
                if (!more) break;
                blk += stride;
            }
        }
    } else {
        // ranks above 64: the fragments of one block already fill the register budget
        for (; blk < n_full; blk += stride) {
            u32x4 xa[MT][2], aa[NT][2];
            load(blk, xa, aa);
            mma(xa, aa);
        }
    }
    if (n_full * kBlockK < p.d_in && (n_full / kWaves) % p.ksplit == ks && n_full % kWaves == w) {
        // the last, shorter block: read inside the row and zero what lies beyond d_in
        u32x4 xa[MT][2], aa[NT][2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int k = n_full * kBlockK + 32 * q;
            const bool in = k + kg * 8 < p.d_in;
            const int kc = in ? k : 0;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const u32x4 v = *reinterpret_cast<const u32x4*>(xrow[mt] + kc);
                xa[mt][q] = in ? v : u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const u32x4 v = *(gconst_u32x4)(arow[nt] + kc);
                aa[nt][q] = in ? v : u32x4{0u, 0u, 0u, 0u};
            }
        }
        mma(xa, aa);
    }

    // Sum over the 8 waves in a fixed order: every wave parks its accumulators in LDS ([wave][register]
    // [lane]); after one barrier the 512 threads share the (register, lane) values, add the eight partial
    // sums as a balanced tree and store the result.
    constexpr int REGS = MT * NT * 4;
    {
        float* mine = lds + (size_t)w * REGS * kWave + lane;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) mine[((mt * NT + nt) * 4 + v) * kWave] = acc[mt][nt][v];
    }
    const HDest d = h_dest(p, u, s, ks, p.ksplit);
    __syncthreads();
#pragma unroll
    for (int e = (int)threadIdx.x; e < REGS * kWave; e += kThreads) {
        const int r = e / kWave, l = e % kWave;
        float t[kWaves];
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) t[ww] = lds[((size_t)ww * REGS + r) * kWave + l];
        const float sum = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
        const int v = r % 4, nt = (r / 4) % NT, mt = r / (4 * NT);
        const int i = mt * 16 + (l >> 4) * 4 + v, jj = nt * 16 + (l & 15);
        if (i < u.len && jj < s.rank) {
            h_store(d.base + (long long)i * p.rstride + jj, sum, p.coherent);
            if (d.save) d.save[(long long)i * d.save_ld + jj] = sum;
        }
    }
}

// =================================================================================================
// expand, long unit: D[col][row] = sum_j B[j][col] (s h[row][j]) with 16x16x32 bf16 MFMA, h split into
// a bf16 high and low part so that it keeps fp32 accuracy.  The output columns of two MFMA tiles are
// interleaved so that a lane ends up with 8 consecutive columns of one row: a 16-byte access to y.  For
// pair q and tile m, MFMA row rho maps to column 32 q + 8 (rho / 4) + 4 m + (rho % 4) of the wave's
// column range.
// =================================================================================================
__device__ __forceinline__ void split_bf16(const float (&v)[8], u32x4& hi, u32x4& lo)
{
    unsigned int h[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        h[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
        l[i] = pack_bf16x2(v[2 * i] - bf16_lo(h[i]), v[2 * i + 1] - bf16_hi(h[i]));
    }
    hi = u32x4{h[0], h[1], h[2], h[3]};
    lo = u32x4{l[0], l[1], l[2], l[3]};
}

template <int KSTEPS, int PAIRS>
struct ExpandCfg {
    static constexpr int WN = 32 * PAIRS;            // columns per wave
    static constexpr int UN = kWaves * WN;           // columns per block
    static constexpr int ROWS = 32 * KSTEPS;         // rank rows staged (ranks beyond the adapter's are zero)
    // token rows per unit, as many as the h fragments leave room for: every unit reads its block of B from HBM (y
    // streaming through the L2 leaves nothing of it for the next unit), so the B traffic of a launch is its row
    // chunks x the adapter's B (gate + up of the layer stack, 512 vs 256 rows: 166 -> 163 us, the step 10.95 -> 10.87 ms)
    static constexpr int CT = KSTEPS >= 4 ? 128 : KSTEPS == 1 ? 512 : 256;
    static constexpr int BPITCH = UN + 8;            // elements per staged B row
    static constexpr size_t B_BYTES = (size_t)ROWS * BPITCH * sizeof(u16);
    static constexpr size_t H_BYTES = (size_t)(CT / 16) * KSTEPS * 2 * kWave * 16;  // [tile][kstep][hi|lo][lane] x 16 B
    static constexpr size_t ROW_BYTES = (size_t)CT * sizeof(int);
    static constexpr size_t LDS_BYTES = B_BYTES + H_BYTES + ROW_BYTES;
};

// One unit = up to CT rows of one segment x the column blocks [nb_begin, nb_end).  The rows' h (and row
// indices) are prepared once and reused for every column block of the unit.
// A workgroup's first long unit and those of its loads that do not depend on h (its first block of B, its row
// indices): the fused kernel requests them while it waits at its barrier.
template <int KSTEPS, int PAIRS>
struct LongAhead {
    using C = ExpandCfg<KSTEPS, PAIRS>;
    bool live;  // workgroup uniform
    Unit u;
    SegInfo s;
    int nb_begin, nb_end;
    int row;    // row index of position u.pos + threadIdx.x
    u32x4 b[C::ROWS * (C::UN / 8) / kThreads];
};

template <int KSTEPS, int PAIRS, bool AHEAD, class PP>  // ranks up to 32 * KSTEPS; a wave covers 32 * PAIRS columns, a block 8 waves
__device__ __forceinline__ void expand_long_unit(const PP& p, const Unit& u, const SegInfo& s, int nb_begin,
                                                 int nb_end, unsigned char* lds, const LongAhead<KSTEPS, PAIRS>& pre)
{
    using C = ExpandCfg<KSTEPS, PAIRS>;
    constexpr int STAGE = C::ROWS * (C::UN / 8) / kThreads;  // 16-byte pieces of the B block per thread
    static_assert(C::ROWS * (C::UN / 8) % kThreads == 0, "staging loop assumes an even split");
    const Proj pj = proj_of(p, u.pi);  // this unit's linear layer: y, d_out (B comes with s)
    u16* lds_b = reinterpret_cast<u16*>(lds);
    u32x4* lds_h = reinterpret_cast<u32x4*>(lds + C::B_BYTES);
    int* lds_row = reinterpret_cast<int*>(lds + C::B_BYTES + C::H_BYTES);
    const int lane = lane_id(), w = uniform((int)threadIdx.x / kWave), c = lane & 15, g = lane >> 4;

    // The block of B of every column block: coalesced loads -> registers -> LDS -> transposed MFMA fragments
    // in registers.  The first block's loads go out before anything else; those of the next block are in
    // flight while a block's y streams by.
    u32x4 bstage[STAGE];
    auto b_load = [&](int n_block) {
#pragma unroll
        for (int i = 0; i < STAGE; ++i) {
            const int id = (int)threadIdx.x + i * kThreads;
            const int j = id / (C::UN / 8), n = n_block * C::UN + (id % (C::UN / 8)) * 8;
            bstage[i] = *(gconst_u32x4)(s.B + (long long)min(j, s.rank - 1) * pj.d_out + min(n, pj.d_out - 8));
        }
    };
    if constexpr (AHEAD) {
#pragma unroll
        for (int i = 0; i < STAGE; ++i) bstage[i] = pre.b[i];
    } else {
        b_load(nb_begin);
    }

    // 1. the unit's rows and their h: slices added, (fine-tune segments, first column block: stored to
    // h_out,) scaled, split into bf16 high/low, stored as ready-made fragments
    static_assert(C::CT <= kThreads, "one row index per thread");
    if constexpr (AHEAD) {
        if ((int)threadIdx.x < C::CT) lds_row[threadIdx.x] = pre.row;
    } else {
        if ((int)threadIdx.x < C::CT) lds_row[threadIdx.x] = (int)threadIdx.x < u.len ? row_of(p, u.pos + (int)threadIdx.x) : -1;
    }
    const int parts = p.ksplit;
    const bool save = u.kd == LQ_SEG_FINETUNE && pj.h_out && p.h_offsets && nb_begin == 0 && parts > 1;
    float* h_dst = save ? pj.h_out + p.h_offsets[u.seg] + (long long)(u.pos - u.first) * s.rank : nullptr;
    {
        // item = (row i, 8 ranks); a thread's items are loaded together, slice after slice
        constexpr int ITEMS = C::CT * (C::ROWS / 8) / kThreads;
        static_assert(C::CT * (C::ROWS / 8) % kThreads == 0, "h preparation assumes an even split");
        const int n_items = (u.len + 15) / 16 * 16 * (C::ROWS / 8);
        f32x4 h0[ITEMS], h1[ITEMS];
        const float* hp[ITEMS];
        float sc[ITEMS];  // the row's scale: the adapter's, or the token's own (dynamic scaling, Section 3.3)
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            if (it * kThreads >= n_items) break;  // workgroup uniform
            const int id = (int)threadIdx.x + it * kThreads;
            const int i = id / (C::ROWS / 8), jg = id % (C::ROWS / 8);
            sc[it] = s.scale;
            if (p.token_scales) {  // kernel uniform
                const int r = row_of(p, u.pos + min(i, u.len - 1));
                sc[it] = p.token_scales[max(r, 0)];
            }
            // (rank groups beyond the adapter's re-read its last one; they are zeroed below)
            hp[it] = p.hpart + u.pi * p.hproj + (long long)(u.pos + min(i, u.len - 1)) * p.rstride + 8 * min(jg, (s.rank - 1) >> 3);
            h_load8(p, hp[it], h0[it], h1[it]);
        }
        for (int part = 1; part < parts; ++part) {
            const long long off = (long long)part * p.n_tokens * p.rstride;
            f32x4 a0[ITEMS], a1[ITEMS];
#pragma unroll
            for (int it = 0; it < ITEMS; ++it) {
                if (it * kThreads >= n_items) break;
                h_load8(p, hp[it] + off, a0[it], a1[it]);
            }
#pragma unroll
            for (int it = 0; it < ITEMS; ++it) {
                if (it * kThreads >= n_items) break;
                h0[it] += a0[it];
                h1[it] += a1[it];
            }
        }
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const int id = (int)threadIdx.x + it * kThreads;
            if (id >= n_items) continue;
            const int i = id / (C::ROWS / 8), jg = id % (C::ROWS / 8);
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float raw = e < 4 ? h0[it][e & 3] : h1[it][e & 3];
                const bool live = i < u.len && 8 * jg + e < s.rank;
                if (save && live) h_dst[(long long)i * s.rank + 8 * jg + e] = raw;
                v[e] = live ? raw * sc[it] : 0.f;
            }
            u32x4 hi, lo;
            split_bf16(v, hi, lo);
            const int slot = ((i / 16) * KSTEPS + jg / 4) * 2;
            const int ln = (jg % 4) * 16 + (i % 16);
            lds_h[(slot + 0) * kWave + ln] = hi;
            lds_h[(slot + 1) * kWave + ln] = lo;
        }
    }
    // 2. per column block: stage B, then stream y
    for (int n_block = nb_begin; n_block < nb_end; ++n_block) {
    const int n_unit = n_block * C::UN;
    __syncthreads();  // the previous block's fragment reads are done; the unit's rows are in LDS
    // (row-wise layout) the first streaming step of y is requested here already: it arrives while B is staged
    int row_f[4];
    u32x4 y_f[4];
    if constexpr (PAIRS == 2) {
        const int n_ld = min(n_unit + w * C::WN + 8 * (lane & 7), pj.d_out - 8);
        const int safe = max(lds_row[0], 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            row_f[j] = lds_row[min(8 * j + (lane >> 3), C::CT - 1)];
            y_f[j] = *reinterpret_cast<const u32x4*>(pj.y + (long long)(row_f[j] >= 0 ? row_f[j] : safe) * pj.ldy + n_ld);
        }
    }
#pragma unroll
    for (int i = 0; i < STAGE; ++i) {
        const int id = (int)threadIdx.x + i * kThreads;
        const int j = id / (C::UN / 8), n = n_unit + (id % (C::UN / 8)) * 8;
        const bool live = j < s.rank && n < pj.d_out;
        *reinterpret_cast<u32x4*>(lds_b + j * C::BPITCH + (n - n_unit)) = live ? bstage[i] : u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();
    b_load(min(n_block + 1, nb_end - 1));  // unconditional: the last block is simply loaded again
    const int n_wave = n_unit + w * C::WN;
    u32x4 bfrag[PAIRS][2][KSTEPS];
#pragma unroll
    for (int q = 0; q < PAIRS; ++q)
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            // lane c: column 32 q + 8 (c / 4) + 4 m + c % 4 of the wave's range, rank rows 32 ks + 8 g .. + 7
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks)
                bfrag[q][m][ks] = lds_read_transposed_16x32(lds_b + 32 * ks * C::BPITCH + w * C::WN + 32 * q + 4 * m, C::BPITCH, 8);
        }
    if constexpr (PAIRS == 2) __syncthreads();  // every wave has its fragments: the B block's LDS becomes scratch
    if (n_wave >= pj.d_out) continue;

    const int n_steps = (u.len + 31) / 32;
    const int safe_row = max(lds_row[0], 0);
    if constexpr (PAIRS == 2) {
        // 3. stream y, 32 rows per step, the next step's loads in flight while this one is computed.  A wave
        // owns 64 columns = 128 bytes of a row, and y is accessed row-wise: an instruction covers 8 rows x
        // 128 contiguous bytes (measured 15 % faster from HBM than the MFMA layout's 16 rows x 64 bytes).
        // The products come out of the MFMA in that other layout, so every 16-row tile of them makes a round
        // trip through a 4 KB LDS slab of the wave (in the B block's space, free while y streams); the
        // 16-byte chunks of a slab row are XOR-swizzled with the row number against bank conflicts.
        // Loads are unconditional (dead rows and columns read a live address); only the stores are masked.
        float* slab = reinterpret_cast<float*>(lds_b) + w * (16 * 64);
        const int r8 = lane >> 3, piece = lane & 7;
        const int n_c = n_wave + 8 * piece, n_ld = min(n_c, pj.d_out - 8);
        int row_n[4];
        u32x4 y_n[4];
        auto fetch = [&](int step) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                row_n[j] = lds_row[min(step * 32 + 8 * j + r8, C::CT - 1)];
                y_n[j] = *reinterpret_cast<const u32x4*>(pj.y + (long long)(row_n[j] >= 0 ? row_n[j] : safe_row) * pj.ldy + n_ld);
            }
        };
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            row_n[j] = row_f[j];
            y_n[j] = y_f[j];
        }
        for (int step = 0; step < n_steps; ++step) {
            int row[4];
            u32x4 yv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                row[j] = row_n[j];
                yv[j] = y_n[j];
            }
            fetch(min(step + 1, n_steps - 1));  // unconditional, so the loads in flight are counted statically
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int tile = min(step * 2 + t, C::CT / 16 - 1);
                u32x4 h_hi[KSTEPS], h_lo[KSTEPS];
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) {
                    h_hi[ks] = lds_h[((tile * KSTEPS + ks) * 2 + 0) * kWave + lane];
                    h_lo[ks] = lds_h[((tile * KSTEPS + ks) * 2 + 1) * kWave + lane];
                }
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int m = 0; m < 2; ++m) {
                        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < KSTEPS; ++ks) {
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(bfrag[q][m][ks]), as_bf16x8(h_lo[ks]), acc, 0, 0, 0);
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(bfrag[q][m][ks]), as_bf16x8(h_hi[ks]), acc, 0, 0, 0);
                        }
                        // row c of the tile, columns 32 q + 8 g + 4 m .. + 4 = chunk 8 q + 2 g + m
                        *reinterpret_cast<f32x4*>(slab + c * 64 + (((8 * q + 2 * g + m) ^ c) & 15) * 4) = acc;
                    }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const int j = 2 * t + jj, rt = 8 * jj + r8;  // row of the step's instruction j = row rt of the tile
                    const f32x4 d0 = *reinterpret_cast<const f32x4*>(slab + rt * 64 + (((2 * piece) ^ rt) & 15) * 4);
                    const f32x4 d1 = *reinterpret_cast<const f32x4*>(slab + rt * 64 + (((2 * piece + 1) ^ rt) & 15) * 4);
                    if (row[j] >= 0 && step * 32 + 8 * j + r8 < u.len && n_c < pj.d_out) {
                        float yf[8];
                        unpack8(yv[j], yf);
                        u32x4 o;
                        o.x = pack_bf16x2(yf[0] + d0[0], yf[1] + d0[1]);
                        o.y = pack_bf16x2(yf[2] + d0[2], yf[3] + d0[3]);
                        o.z = pack_bf16x2(yf[4] + d1[0], yf[5] + d1[1]);
                        o.w = pack_bf16x2(yf[6] + d1[2], yf[7] + d1[3]);
                        *reinterpret_cast<u32x4*>(pj.y + (long long)row[j] * pj.ldy + n_c) = o;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();  // the slab is rewritten by the next tile
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {

        // 3. stream y: 32 rows per step, the next step's loads in flight while this one is computed.  Loads
        // are unconditional (dead rows and columns read a live address); only the stores are masked.
        const int n_lane = n_wave + 8 * g;  // + 32 q
        int n_ld[PAIRS];
    #pragma unroll
        for (int q = 0; q < PAIRS; ++q) n_ld[q] = min(n_lane + 32 * q, pj.d_out - 8);
        int row_n[2];
        u32x4 y_n[2][PAIRS];
        auto fetch = [&](int step) {
    #pragma unroll
            for (int t = 0; t < 2; ++t) {
                row_n[t] = lds_row[min(step * 32 + t * 16 + c, C::CT - 1)];
                const u16* yrow = pj.y + (long long)(row_n[t] >= 0 ? row_n[t] : safe_row) * pj.ldy;
    #pragma unroll
                for (int q = 0; q < PAIRS; ++q) y_n[t][q] = *reinterpret_cast<const u32x4*>(yrow + n_ld[q]);
            }
        };
        fetch(0);
        for (int step = 0; step < n_steps; ++step) {
            int row[2];
            u32x4 yv[2][PAIRS];
    #pragma unroll
            for (int t = 0; t < 2; ++t) {
                row[t] = row_n[t];
    #pragma unroll
                for (int q = 0; q < PAIRS; ++q) yv[t][q] = y_n[t][q];
            }
            fetch(min(step + 1, n_steps - 1));  // unconditional, so the loads in flight are counted statically
            __builtin_amdgcn_sched_barrier(0);
    #pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int tile = min(step * 2 + t, C::CT / 16 - 1);
                u32x4 h_hi[KSTEPS], h_lo[KSTEPS];
    #pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) {
                    h_hi[ks] = lds_h[((tile * KSTEPS + ks) * 2 + 0) * kWave + lane];
                    h_lo[ks] = lds_h[((tile * KSTEPS + ks) * 2 + 1) * kWave + lane];
                }
                f32x4 acc[PAIRS][2];
    #pragma unroll
                for (int q = 0; q < PAIRS; ++q)
    #pragma unroll
                    for (int m = 0; m < 2; ++m) {
                        acc[q][m] = f32x4{0.f, 0.f, 0.f, 0.f};
    #pragma unroll
                        for (int ks = 0; ks < KSTEPS; ++ks) {
                            acc[q][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(bfrag[q][m][ks]), as_bf16x8(h_lo[ks]),
                                                                                acc[q][m], 0, 0, 0);
                            acc[q][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(bfrag[q][m][ks]), as_bf16x8(h_hi[ks]),
                                                                                acc[q][m], 0, 0, 0);
                        }
                    }
                if (row[t] >= 0 && step * 32 + t * 16 + c < u.len) {
    #pragma unroll
                    for (int q = 0; q < PAIRS; ++q) {
                        if (n_lane + 32 * q < pj.d_out) {
                            float yf[8];
                            unpack8(yv[t][q], yf);
                            u32x4 o;
                            o.x = pack_bf16x2(yf[0] + acc[q][0][0], yf[1] + acc[q][0][1]);
                            o.y = pack_bf16x2(yf[2] + acc[q][0][2], yf[3] + acc[q][0][3]);
                            o.z = pack_bf16x2(yf[4] + acc[q][1][0], yf[5] + acc[q][1][1]);
                            o.w = pack_bf16x2(yf[6] + acc[q][1][2], yf[7] + acc[q][1][3]);
                            *reinterpret_cast<u32x4*>(pj.y + (long long)row[t] * pj.ldy + n_lane + 32 * q) = o;
                        }
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    }  // column blocks
}

// =================================================================================================
// expand, short unit: one wave per unit of <= 4 rows x 512 columns.  The wave puts the scaled h of its
// rows into its own LDS slab, then for every rank row j streams B[j][n .. n + 8) with one 16-byte load
// per lane and accumulates h[t][j] * B[j][n + i] for the four rows.
// =================================================================================================
struct ShortLds {
    __attribute__((aligned(16))) float hs[kWaves][LQ_MAX_RANK][kTT];  // per wave: hs[rank][row], scaled
};

constexpr int kShortGroup = 8;  // rank rows of B in flight per group

// A wave's first short unit and those of its loads that do not depend on h (row indices, y, the first 16
// rows of B): the fused kernel requests them while it waits at its barrier, so that only h is left to
// fetch behind it.
struct ShortAhead {
    bool live;  // wave uniform
    Unit u;
    SegInfo s;
    int n_block;
    int row[kTT];
    u32x4 y[kTT], b[2 * kShortGroup];
};

template <bool AHEAD, class PP>  // AHEAD: rows, y and the first 16 rows of B come from `pre`
__device__ __forceinline__ void expand_short_unit(const PP& p, const Unit& u, const SegInfo& s, int n_block,
                                                  ShortLds& sh, const ShortAhead& pre)
{
    constexpr int JG = kShortGroup;
    const int lane = lane_id(), w = uniform((int)threadIdx.x / kWave);
    const Proj pj = proj_of(p, u.pi);  // this unit's linear layer: y, d_out (B comes with s)
    float* hs = &sh.hs[w][0][0];  // hs[j][t] at j * kTT + t
    const int parts = p.ksplit;
    const bool save = u.kd == LQ_SEG_FINETUNE && pj.h_out && p.h_offsets && n_block == 0 && parts > 1;
    float* h_dst = save ? pj.h_out + p.h_offsets[u.seg] + (long long)(u.pos - u.first) * s.rank : nullptr;
    const int n = n_block * kShortN + lane * 8;
    const int n_ld = min(n, pj.d_out - 8);
    const int rank_up = (s.rank + JG - 1) / JG * JG;

    // The loads go out in the order rows, h, first group of B, y, so that each wait covers only what is
    // needed next.  Everything is loaded unconditionally from clamped addresses.
    int row[kTT];
#pragma unroll
    for (int t = 0; t < kTT; ++t) {
        if constexpr (AHEAD) row[t] = pre.row[t];
        else row[t] = t < u.len ? row_of(p, u.pos + t) : -1;
    }

    // the rows' scales: the adapter's, or the tokens' own (dynamic scaling, Section 3.3)
    float tsc[kTT];
#pragma unroll
    for (int t = 0; t < kTT; ++t) tsc[t] = p.token_scales ? p.token_scales[max(row[t], 0)] : s.scale;

    // item i = lane + 64 q is (row t = i % 4, rank j = i / 4); the first two per lane cover ranks up to 32
    static_assert(kTT == 4, "the scale of an item's row is picked by name");
    auto h_item = [&](int i) {
        const int t = i & (kTT - 1), j = i >> 2;
        const float h = h_sum(p, u.pi, u.pos + min(t, u.len - 1), min(j, s.rank - 1), parts);
        const bool live = t < u.len && j < s.rank;
        if (save && live) h_dst[(long long)t * s.rank + j] = h;
        const float scale = t == 0 ? tsc[0] : t == 1 ? tsc[1] : t == 2 ? tsc[2] : tsc[3];
        return live ? h * scale : 0.f;
    };
    const float h0 = h_item(lane), h1 = h_item(lane + kWave);

    // (AHEAD: the ring starts with the third group; the first two are in `pre`)
    constexpr int J_RING = AHEAD ? 2 * JG : 0;
    u32x4 bn[JG];
#pragma unroll
    for (int jj = 0; jj < JG; ++jj)
        bn[jj] = *(gconst_u32x4)(s.B + (long long)min(J_RING + jj, s.rank - 1) * pj.d_out + n_ld);
    const int safe_row = max(row[0], 0);
    u32x4 yv[kTT];
#pragma unroll
    for (int t = 0; t < kTT; ++t) {
        if constexpr (AHEAD) yv[t] = pre.y[t];
        else yv[t] = *reinterpret_cast<const u32x4*>(pj.y + (long long)(row[t] >= 0 ? row[t] : safe_row) * pj.ldy + n_ld);
    }

    hs[lane] = h0;
    hs[lane + kWave] = h1;
    for (int i = lane + 2 * kWave; i < rank_up * kTT; i += kWave) hs[i] = h_item(i);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    float acc[kTT][8];
#pragma unroll
    for (int t = 0; t < kTT; ++t)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[t][i] = 0.f;
    auto fma_group = [&](const u32x4* bc, int j0) {
#pragma unroll
        for (int jj = 0; jj < JG; ++jj) {
            const f32x4 h4 = *reinterpret_cast<const f32x4*>(hs + (j0 + jj) * kTT);  // zero beyond the rank
            float bf[8];
            unpack8(bc[jj], bf);
            const float h[kTT] = {h4.x, h4.y, h4.z, h4.w};
#pragma unroll
            for (int t = 0; t < kTT; ++t)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[t][i] = fmaf(h[t], bf[i], acc[t][i]);
        }
    };
    if constexpr (AHEAD) {
        fma_group(pre.b, 0);
        if (rank_up > JG) fma_group(pre.b + JG, JG);
    }
    for (int j0 = J_RING; j0 < rank_up; j0 += JG) {
        u32x4 bc[JG];
#pragma unroll
        for (int jj = 0; jj < JG; ++jj) bc[jj] = bn[jj];
#pragma unroll
        for (int jj = 0; jj < JG; ++jj)  // the next group (past the end: the last row again, unused)
            bn[jj] = *(gconst_u32x4)(s.B + (long long)min(j0 + JG + jj, s.rank - 1) * pj.d_out + n_ld);
        __builtin_amdgcn_sched_barrier(0);
        fma_group(bc, j0);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (n < pj.d_out) {
#pragma unroll
        for (int t = 0; t < kTT; ++t) {
            if (row[t] >= 0) {
                float yf[8];
                unpack8(yv[t], yf);
                u32x4 o;
                o.x = pack_bf16x2(yf[0] + acc[t][0], yf[1] + acc[t][1]);
                o.y = pack_bf16x2(yf[2] + acc[t][2], yf[3] + acc[t][3]);
                o.z = pack_bf16x2(yf[4] + acc[t][4], yf[5] + acc[t][5]);
                o.w = pack_bf16x2(yf[6] + acc[t][6], yf[7] + acc[t][7]);
                *reinterpret_cast<u32x4*>(pj.y + (long long)row[t] * pj.ldy + n) = o;
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the slab is rewritten by this wave's next unit
}

// =================================================================================================
// kernels
// =================================================================================================
template <int NT>
constexpr size_t shrink_lds_bytes()
{
    // two stage buffers of A, and (kernels for ranks up to 64) the eight waves' x slabs
    const size_t tall = (size_t)2 * NT * 16 * (kStageK + 8) * sizeof(u16) +
                        (NT <= 4 ? (size_t)kWaves * 16 * (kStageK + 8) * sizeof(u16) : 0);
    const size_t small = (size_t)kWaves * (kShortRows / 16) * NT * 4 * kWave * sizeof(float);
    return tall > small ? tall : small;
}

template <int NT, class PP>
__device__ __forceinline__ void shrink_phase(const PP& p, const Segs<PP>& sg, unsigned char* lds_raw,
                                             int* s_slot)
{
    // hand-out order, large units first so that a launch ends evenly: the even chunks (65 to 128 rows) of
    // the segments with more than 128 rows, the other tall segments (one chunk each), the short segments
    const LenClass tall{kTallRows + 1, kBig, p.kinds, true}, rest{kTallMin, kTallRows + 1, p.kinds}, small{1, kTallMin, p.kinds};
    const ClassScan ct = scan_class(p, sg, kTallRows, tall), cr = scan_class(p, sg, kTallRows, rest),
                    cm = scan_class(p, sg, kShortRows, small);
    const int n_full = ct.total << p.ks_log2, n_tall = n_full + (cr.total << p.ks_log2), n_small = cm.total << p.ks_log2;
    // A grouped call runs every unit once per projection.  Workgroups whose indices differ by 8 sit on the same XCD
    // and share its L2, so the projections of one unit are handed to such workgroups (ids r, r + 8, r + 16 ... of a
    // block of 8 n_proj ids): they run side by side and the x rows they all read cross the HBM interface once.
    const int n_per = n_tall + n_small, n_all = n_proj_of(p) == 1 ? n_per : ((n_per + 7) & ~7) * n_proj_of(p);
    for_each_unit(p.tickets + 0, n_all, s_slot, [&](int gid, int) {
        Unit u;
        SegInfo s;
        int id = gid;
        u.pi = 0;
        if (n_proj_of(p) > 1) {
            const int blk = small_div(gid, 8 * n_proj_of(p)), r = gid - blk * 8 * n_proj_of(p);
            u.pi = r >> 3;
            id = blk * 8 + (r & 7);
            if (id >= n_per) return;  // (padding of the last block)
        }
        const bool is_tall = id < n_tall;
        const int cid = id < n_full ? id : is_tall ? id - n_full : id - n_tall;
        const int chunk = cid >> p.ks_log2, ks = cid & (p.ksplit - 1);
        const bool ok = id < n_full ? find_unit(p, sg, ct, chunk, kTallRows, tall, u, s)
                        : is_tall   ? find_unit(p, sg, cr, chunk, kTallRows, rest, u, s)
                                    : find_unit(p, sg, cm, chunk, kShortRows, small, u, s);
        if (!ok) return;
        // the unit runs with as many 16-rank tiles as its adapter needs (at most NT, the launch's maximum)
        u16* lds_a = reinterpret_cast<u16*>(lds_raw);
        float* lds_r = reinterpret_cast<float*>(lds_raw);
        if (is_tall) {
            // row-wise x for ranks up to 32, in the kernels whose LDS has room for the slabs
            constexpr bool RW = NT <= 4;
            u16* slabs = lds_a + 2 * NT * 16 * (kStageK + 8);
            if (NT >= 8 && s.rank > 64) shrink_tall_unit<(NT >= 8 ? 8 : NT), false>(p, u, s, ks, lds_a, slabs);
            else if (NT >= 4 && s.rank > 32) shrink_tall_unit<(NT >= 4 ? 4 : NT), RW>(p, u, s, ks, lds_a, slabs);
            else if (NT >= 2 && s.rank > 16) shrink_tall_unit<(NT >= 2 ? 2 : NT), RW>(p, u, s, ks, lds_a, slabs);
            else shrink_tall_unit<1, RW>(p, u, s, ks, lds_a, slabs);
        } else {
            if (NT >= 8 && s.rank > 64) shrink_short_unit<(NT >= 8 ? 8 : NT)>(p, u, s, ks, lds_r);
            else if (NT >= 4 && s.rank > 32) shrink_short_unit<(NT >= 4 ? 4 : NT)>(p, u, s, ks, lds_r);
            else if (NT >= 2 && s.rank > 16) shrink_short_unit<(NT >= 2 ? 2 : NT)>(p, u, s, ks, lds_r);
            else shrink_short_unit<1>(p, u, s, ks, lds_r);
        }
    });
}

template <int NT, bool GROUP>
__global__ __launch_bounds__(kThreads) void shrink_kernel(KernelArg<GROUP> p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    __shared__ int s_slot[2];
    const auto sg = load_segs(p);
    shrink_phase<NT>(p, sg, lds_raw, s_slot);
}

// What the expand phase works out from the segment tables before it touches any data: the rows per long
// unit, the classes of units and their prefix sums, and per projection of a grouped call its column blocks and
// how they are grouped into units.  (The fused kernel does this before its barrier.)
struct ExpandPlan {
    int per, n_chunks, n_short;
    int long_blocks[kMaxProj], per_group[kMaxProj], groups[kMaxProj], short_blocks[kMaxProj];
    int sum_groups, sum_short_blocks;  // over the projections
    int n_full, n_big, n_long;         // long units: numbering of the classes
    LenClass shorts, full, big, little;
    ClassScan cf, cb, cl, cs;
};

// a[i] for a wave-uniform i (the arrays live in registers, which cannot be indexed)
__device__ __forceinline__ int pick(const int (&a)[kMaxProj], int i)
{
    static_assert(kMaxProj == 4, "the entries are picked by name");
    return i == 0 ? a[0] : i == 1 ? a[1] : i == 2 ? a[2] : a[3];
}
// index i into the concatenation of n ranges of lengths len[0 .. n): the range, and the index inside it
__device__ __forceinline__ int range_of(const int (&len)[kMaxProj], int n, int& i)
{
    int r = 0;
#pragma unroll
    for (int k = 0; k < kMaxProj - 1; ++k)
        if (r == k && k + 1 < n && i >= len[k]) {
            i -= len[k];
            r = k + 1;
        }
    return r;
}

template <int KSTEPS, int PAIRS, class PP>
__device__ __forceinline__ ExpandPlan plan_expand(const PP& p, const Segs<PP>& sg)
{
    using C = ExpandCfg<KSTEPS, PAIRS>;
    ExpandPlan e;
    const LenClass longs{kLongMin, kBig, p.kinds};
    e.shorts = LenClass{1, kLongMin, p.kinds};
    int sum_blocks = 0;
    e.sum_short_blocks = 0;
#pragma unroll
    for (int k = 0; k < kMaxProj; ++k) {
        const int d_out = k < n_proj_of(p) ? proj_of(p, k).d_out : 0;
        e.long_blocks[k] = (d_out + C::UN - 1) / C::UN;
        e.short_blocks[k] = (d_out + kShortN - 1) / kShortN;
        sum_blocks += e.long_blocks[k];
        e.sum_short_blocks += e.short_blocks[k];
    }

    // Rows per long unit: CT, halved (down to 64: the B block is staged once per unit) until the units fill two
    // rounds of the grid, or exactly one: so that a batch with few rows is still spread over the whole machine,
    // and so that equal units (a batch of long fine-tune segments only) do not leave half a round empty.
    int per = C::CT;
    if (sg.n_seg <= kCachedBatches * kWave) {  // (more segments than that: plenty of units anyway)
        const int grid = (int)gridDim.x;
        while (per > 64) {
            int chunks = 0;
#pragma unroll
            for (int b = 0; b < kCachedBatches; ++b) chunks += wave_sum(chunks_in(sg.c[b].en - sg.c[b].st, sg.c[b].kd, per, longs));
            const long long units = (long long)chunks * sum_blocks;
            if (units >= 2LL * grid || (units >= grid && units % grid == 0)) break;
            per >>= 1;
        }
    }
    e.per = per;
    e.full = LenClass{per + 1, kBig, p.kinds, true};
    e.big = LenClass{per / 2, per + 1, p.kinds};
    e.little = LenClass{kLongMin, per / 2, p.kinds};
    e.cf = scan_class(p, sg, per, e.full);
    e.cb = scan_class(p, sg, per, e.big);
    e.cl = scan_class(p, sg, per, e.little);
    e.n_chunks = e.cf.total + e.cb.total + e.cl.total;
    // Long units: a chunk of rows x a group of column blocks of one projection.  Groups are as large as possible
    // (the rows' h is prepared once per unit) while leaving about 4 units per workgroup.
    e.sum_groups = 0;
    const int groups_wanted = e.n_chunks > 0 ? small_div(4 * (int)gridDim.x + e.n_chunks - 1, e.n_chunks) : 1;  // per chunk, all projections
#pragma unroll
    for (int k = 0; k < kMaxProj; ++k) {
        const int blocks = e.long_blocks[k];
        // this projection's share of the groups, by its share of the column blocks
        const int wanted = blocks > 0 ? max(1, small_div(groups_wanted * blocks, max(1, sum_blocks))) : 1;
        e.per_group[k] = max(1, small_div(blocks, max(1, min(blocks, wanted))));
        e.groups[k] = small_div(blocks + e.per_group[k] - 1, e.per_group[k]);
        e.sum_groups += e.groups[k];
    }
    e.n_full = e.cf.total * e.sum_groups;
    e.n_big = e.n_full + e.cb.total * e.sum_groups;
    e.n_long = e.n_chunks * e.sum_groups;
    e.cs = scan_class(p, sg, kTT, e.shorts);
    e.n_short = e.cs.total * e.sum_short_blocks;
    return e;
}

// Short units: one per wave iteration.  Without long units they are dealt over the workgroups first (all
// compute units pull data); with long units they are packed eight to a workgroup, so that the other
// workgroups start streaming at once.
__device__ __forceinline__ int first_short_unit(const ExpandPlan& e)
{
    const int w = uniform((int)threadIdx.x / kWave);
    return e.n_chunks > 0 ? (int)blockIdx.x * kWaves + w : w * (int)gridDim.x + (int)blockIdx.x;
}
// short unit `id`: ids count through the row chunks, and for each chunk through the 512-column blocks of every projection
template <class PP>
__device__ __forceinline__ bool find_short_unit(const PP& p, const Segs<PP>& sg, const ExpandPlan& e, int id,
                                                Unit& u, SegInfo& s, int& n_block)
{
    const int chunk = small_div(id, e.sum_short_blocks);
    n_block = id - chunk * e.sum_short_blocks;
    u.pi = range_of(e.short_blocks, n_proj_of(p), n_block);
    return find_unit(p, sg, e.cs, chunk, kTT, e.shorts, u, s);
}

// requests the loads of this wave's first short unit that do not depend on h
template <class PP>
__device__ __forceinline__ ShortAhead short_request(const PP& p, const Segs<PP>& sg, const ExpandPlan& e)
{
    ShortAhead a;
    a.live = false;
    const int id = first_short_unit(e);
    if (id >= e.n_short) return a;
    a.live = find_short_unit(p, sg, e, id, a.u, a.s, a.n_block);
    if (!a.live) return a;
    const Proj q = proj_of(p, a.u.pi);
    const int n_ld = min(a.n_block * kShortN + lane_id() * 8, q.d_out - 8);
#pragma unroll
    for (int t = 0; t < kTT; ++t) a.row[t] = t < a.u.len ? row_of(p, a.u.pos + t) : -1;
#pragma unroll
    for (int jj = 0; jj < 2 * kShortGroup; ++jj)
        a.b[jj] = *(gconst_u32x4)(a.s.B + (long long)min(jj, a.s.rank - 1) * q.d_out + n_ld);
    const int safe_row = max(a.row[0], 0);
#pragma unroll
    for (int t = 0; t < kTT; ++t)
        a.y[t] = *reinterpret_cast<const u32x4*>(q.y + (long long)(a.row[t] >= 0 ? a.row[t] : safe_row) * q.ldy + n_ld);
    return a;
}

// long unit `id`: large ones first so that a launch ends evenly: the even chunks of the segments with more
// than `per` rows, the segments with per/2 to per rows, the smaller ones; within a class ids count through the
// row chunks, and for each chunk through the column groups of every projection
template <class PP>
__device__ __forceinline__ bool find_long_unit(const PP& p, const Segs<PP>& sg, const ExpandPlan& e, int id,
                                               Unit& u, SegInfo& s, int& nb_begin, int& nb_end)
{
    const int cid = id < e.n_full ? id : id < e.n_big ? id - e.n_full : id - e.n_big;
    const int chunk = small_div(cid, e.sum_groups);
    int g = cid - chunk * e.sum_groups;
    u.pi = range_of(e.groups, n_proj_of(p), g);
    const int per_group = pick(e.per_group, u.pi);
    nb_begin = g * per_group;
    nb_end = min(pick(e.long_blocks, u.pi), nb_begin + per_group);
    return id < e.n_full ? find_unit(p, sg, e.cf, chunk, e.per, e.full, u, s)
           : id < e.n_big ? find_unit(p, sg, e.cb, chunk, e.per, e.big, u, s)
                          : find_unit(p, sg, e.cl, chunk, e.per, e.little, u, s);
}

// requests the loads of this workgroup's first long unit that do not depend on h
template <int KSTEPS, int PAIRS, class PP>
__device__ __forceinline__ LongAhead<KSTEPS, PAIRS> long_request(const PP& p, const Segs<PP>& sg,
                                                                  const ExpandPlan& e)
{
    using C = ExpandCfg<KSTEPS, PAIRS>;
    constexpr int STAGE = C::ROWS * (C::UN / 8) / kThreads;
    LongAhead<KSTEPS, PAIRS> a;
    a.live = false;
    if ((int)blockIdx.x >= e.n_long) return a;
    a.live = find_long_unit(p, sg, e, (int)blockIdx.x, a.u, a.s, a.nb_begin, a.nb_end);
    if (!a.live) return a;
    const int d_out = proj_of(p, a.u.pi).d_out;
#pragma unroll
    for (int i = 0; i < STAGE; ++i) {
        const int id = (int)threadIdx.x + i * kThreads;
        const int j = id / (C::UN / 8), n = a.nb_begin * C::UN + (id % (C::UN / 8)) * 8;
        a.b[i] = *(gconst_u32x4)(a.s.B + (long long)min(j, a.s.rank - 1) * d_out + min(n, d_out - 8));
    }
    a.row = (int)threadIdx.x < a.u.len ? row_of(p, a.u.pos + (int)threadIdx.x) : -1;
    return a;
}

// AHEAD: this wave's first short unit and this workgroup's first long unit were requested into `ahead`, `lahead`
template <int KSTEPS, int PAIRS, bool AHEAD, class PP>
__device__ __forceinline__ void expand_phase(const PP& p, const Segs<PP>& sg, const ExpandPlan& e,
                                             unsigned char* lds_raw, ShortLds& sh, int* s_slot, const ShortAhead ahead,
                                             const LongAhead<KSTEPS, PAIRS> lahead)
{

    // short units first (their cost is mostly latency, which the start of a launch has to spare)
    {
        int first = first_short_unit(e);
        if constexpr (AHEAD) {  // this wave's first unit was requested ahead; the loop below takes the others
            if (first < e.n_short && ahead.live) expand_short_unit<true>(p, ahead.u, ahead.s, ahead.n_block, sh, ahead);
            first += kWaves * (int)gridDim.x;
        }
        if constexpr (AHEAD) {  // then the workgroup's first long unit (by now the short unit's registers are free)
            if (lahead.live)
                expand_long_unit<KSTEPS, PAIRS, true>(p, lahead.u, lahead.s, lahead.nb_begin, lahead.nb_end, lds_raw, lahead);
            __syncthreads();  // before the next long unit reuses the LDS
        }
        ShortAhead unused;
        unused.live = false;
        for (int id = first; id < e.n_short; id += kWaves * (int)gridDim.x) {
            Unit u;
            SegInfo s;
            int n_block;
            if (!find_short_unit(p, sg, e, id, u, s, n_block)) continue;
            expand_short_unit<false>(p, u, s, n_block, sh, unused);
        }
    }

    // long units, one per workgroup iteration
    if (e.n_chunks > 0) {
        LongAhead<KSTEPS, PAIRS> none;
        none.live = false;
        for_each_unit(p.tickets + 2, e.n_long, s_slot, [&](int id, int) {
            Unit u;
            SegInfo s;
            int nb_begin, nb_end;
            if (!find_long_unit(p, sg, e, id, u, s, nb_begin, nb_end)) return;
            expand_long_unit<KSTEPS, PAIRS, false>(p, u, s, nb_begin, nb_end, lds_raw, none);
        }, AHEAD ? 1 : 0);
    }
}

template <int KSTEPS, int PAIRS, bool GROUP>
__global__ __launch_bounds__(kThreads) void expand_kernel(KernelArg<GROUP> p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    __shared__ ShortLds sh;
    __shared__ int s_slot[2];
    const auto sg = load_segs(p);
    const ExpandPlan plan = plan_expand<KSTEPS, PAIRS>(p, sg);
    ShortAhead none;
    none.live = false;
    LongAhead<KSTEPS, PAIRS> lnone;
    lnone.live = false;
    expand_phase<KSTEPS, PAIRS, false>(p, sg, plan, lds_raw, sh, s_slot, none, lnone);
}

// =================================================================================================
// fused single launch: every workgroup runs its shrink units, all workgroups meet at a device-wide
// barrier (which also makes the h values visible across the XCDs' L2 caches), then every workgroup runs
// its expand units.  The grid is exactly the number of workgroups that are resident at once, so every
// workgroup reaches the barrier; the wait is bounded all the same, and a timeout is reported in the
// workspace error word instead of hanging.
//   (header words: see kBarGen, kBarTop, kBarSub)
// =================================================================================================
template <int NT, int KSTEPS, int PAIRS, bool GROUP>
__global__ __launch_bounds__(kThreads) void fused_kernel(KernelArg<GROUP> p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    __shared__ ShortLds sh;
    __shared__ int s_slot[2];
    const auto sg = load_segs(p);
    // The generation is read before this workgroup arrives, hence before the last arrival can change it;
    // and after the table loads, so that their results need not wait for this slower, uncached load.
    const int gen0 = __hip_atomic_load(p.header + kBarGen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    shrink_phase<NT>(p, sg, lds_raw, s_slot);
    // What the expand phase needs and h does not: worked out, and requested, while the workgroup waits: the plan
    // and, for every wave's first short unit, its row indices, y and the first rows of B.
    ExpandPlan plan;
    ShortAhead ahead;
    LongAhead<KSTEPS, PAIRS> lahead;
    const bool opened = grid_barrier(p.header, p.err, gen0, [&]() {
        plan = plan_expand<KSTEPS, PAIRS>(p, sg);
        ahead = short_request(p, sg, plan);
        lahead = long_request<KSTEPS, PAIRS>(p, sg, plan);
    });
    // The wait ran out (somewhere): h is incomplete, so y is left as it is; bit 1 of the error word says so.
    if (!opened) return;
    expand_phase<KSTEPS, PAIRS, true>(p, sg, plan, lds_raw, sh, s_slot, ahead, lahead);
}

int log2_of(int v)  // v is a power of two
{
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}
int ksplit_cap(int n_tokens) { return n_tokens <= 32768 ? kMaxKSplit : 1; }


// (the two instantiations of a kernel, for single and for grouped calls, use the same registers and LDS, hence the same grid)
template <int NT>
int shrink_grid()
{
    static DeviceGrid cache;
    return cache.get([] {
        return std::min(resident_grid(shrink_kernel<NT, false>, shrink_lds_bytes<NT>()),
                        resident_grid(shrink_kernel<NT, true>, shrink_lds_bytes<NT>()));
    });
}

// A 128-row shrink unit streams its rows at the rate of one compute unit, so a batch has to be cut into
// enough units for the launch to draw the full HBM rate and to end evenly: d_in is cut into slices (each
// at least four stages long) as long as that leaves less than one row chunk x slice per workgroup (more
// slices cost the expand kernel, which adds them up).  A pure function of host arguments.
int choose_ksplit(int n_tokens, int n_proj, int d_in, int grid)
{
    const long long chunks = (long long)((n_tokens + kTallRows - 1) / kTallRows) * n_proj;
    int ks = 1;
    while (ks < ksplit_cap(n_tokens) && chunks * ks * 2 < grid && d_in >= ks * 2 * 4 * kStageK) ks *= 2;
    return ks;
}

template <int NT>
hipError_t launch_shrink(const FwdParams& p, hipStream_t st)
{
    if (p.n_proj == 1)
        return launch_kernel(kKernelShrink, shrink_kernel<NT, false>, dim3(shrink_grid<NT>()), dim3(kThreads), shrink_lds_bytes<NT>(), st, static_cast<const FwdCore&>(p));
    return launch_kernel(kKernelShrink, shrink_kernel<NT, true>, dim3(shrink_grid<NT>()), dim3(kThreads), shrink_lds_bytes<NT>(), st, p);
}

template <int KSTEPS, int PAIRS>
hipError_t launch_expand(const FwdParams& p, hipStream_t st)
{
    static DeviceGrid cache;
    constexpr size_t lds = ExpandCfg<KSTEPS, PAIRS>::LDS_BYTES;
    const int grid = cache.get([] {
        return std::min(resident_grid(expand_kernel<KSTEPS, PAIRS, false>, lds), resident_grid(expand_kernel<KSTEPS, PAIRS, true>, lds));
    });
    if (p.n_proj == 1) return launch_kernel(kKernelExpand, expand_kernel<KSTEPS, PAIRS, false>, dim3(grid), dim3(kThreads), lds, st, static_cast<const FwdCore&>(p));
    return launch_kernel(kKernelExpand, expand_kernel<KSTEPS, PAIRS, true>, dim3(grid), dim3(kThreads), lds, st, p);
}

template <int NT, int KSTEPS, int PAIRS>
int fused_grid()
{
    static DeviceGrid cache;
    constexpr size_t lds = shrink_lds_bytes<NT>() > ExpandCfg<KSTEPS, PAIRS>::LDS_BYTES ? shrink_lds_bytes<NT>()
                                                                                       : ExpandCfg<KSTEPS, PAIRS>::LDS_BYTES;
    return cache.get([] {
        return std::min(resident_grid(fused_kernel<NT, KSTEPS, PAIRS, false>, lds), resident_grid(fused_kernel<NT, KSTEPS, PAIRS, true>, lds));
    });
}

template <int NT, int KSTEPS, int PAIRS>
hipError_t launch_fused(const FwdParams& p, hipStream_t st)
{
    const size_t lds = shrink_lds_bytes<NT>() > ExpandCfg<KSTEPS, PAIRS>::LDS_BYTES ? shrink_lds_bytes<NT>()
                                                                                   : ExpandCfg<KSTEPS, PAIRS>::LDS_BYTES;
    if (p.n_proj == 1)
        return launch_kernel(kKernelFused, fused_kernel<NT, KSTEPS, PAIRS, false>, dim3(fused_grid<NT, KSTEPS, PAIRS>()), dim3(kThreads), lds, st, static_cast<const FwdCore&>(p));
    return launch_kernel(kKernelFused, fused_kernel<NT, KSTEPS, PAIRS, true>, dim3(fused_grid<NT, KSTEPS, PAIRS>()), dim3(kThreads), lds, st, p);
}

}  // namespace

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// LQ_VARIANT_AUTO: slab or fused, from the host arguments alone.  Measured on the layer-stack shapes (5632 tokens,
// rank 32): slab wins up to 14336 output columns in all (q 40 vs 47 us, k 25 vs 30, q+k+v 64 vs 72, down 71 vs 76, gate
// 96 vs 101), fused beyond (gate+up 167 vs 178: a slab re-reads all of B for its 32 rows, the fused expand phase stages a
// block of B once per 512 rows) and for ranks above 32 (the Zipf batch with ranks up to 64: 125 vs 152 us).
int auto_variant(int max_rank, long long out_columns)
{
    return max_rank <= 32 && out_columns <= 16384 ? LQ_VARIANT_SLAB : LQ_VARIANT_FUSED;
}

int rstride_for(int max_rank) { return max_rank <= 32 ? 32 : max_rank <= 64 ? 64 : 128; }  // what the expand kernel reads per row

size_t h_slices_bytes(int n_tokens, int max_rank)
{
    return (size_t)ksplit_cap(n_tokens) * (size_t)n_tokens * (size_t)rstride_for(max_rank) * sizeof(float);
}

hipError_t run_shrink_expand(FwdParams& p, int variant, hipStream_t st)
{
    const int nt = nt_for(p.max_rank);
    hipError_t e = hipSuccess;
    if (variant == LQ_VARIANT_FUSED) {
        const int grid_f = nt == 1 ? fused_grid<1, 1, 2>() : nt == 2 ? fused_grid<2, 1, 2>()
                         : nt == 4 ? fused_grid<4, 2, 2>() : fused_grid<8, 4, 1>();
        p.ksplit = p.ksplit_hint > 0 ? p.ksplit_hint : choose_ksplit(p.n_tokens, p.n_proj, p.d_in, grid_f);
        p.ks_log2 = log2_of(p.ksplit);
        return nt == 1 ? launch_fused<1, 1, 2>(p, st) : nt == 2 ? launch_fused<2, 1, 2>(p, st)
             : nt == 4 ? launch_fused<4, 2, 2>(p, st) : launch_fused<8, 4, 1>(p, st);
    }
    const int grid_s = nt == 1 ? shrink_grid<1>() : nt == 2 ? shrink_grid<2>() : nt == 4 ? shrink_grid<4>() : shrink_grid<8>();
    p.ksplit = p.ksplit_hint > 0 ? p.ksplit_hint : choose_ksplit(p.n_tokens, p.n_proj, p.d_in, grid_s);
    p.ks_log2 = log2_of(p.ksplit);
    if (variant != LQ_VARIANT_EXPAND_ONLY) {
        e = nt == 1 ? launch_shrink<1>(p, st) : nt == 2 ? launch_shrink<2>(p, st)
          : nt == 4 ? launch_shrink<4>(p, st) : launch_shrink<8>(p, st);
        if (e != hipSuccess || variant == LQ_VARIANT_SHRINK_ONLY) return e;
    }
    return p.max_rank <= 32 ? launch_expand<1, 2>(p, st) : p.max_rank <= 64 ? launch_expand<2, 2>(p, st)
                                                                            : launch_expand<4, 1>(p, st);
}

}  // namespace lq

// workspace: [header 4096 B][hpart: cap x n_tokens x rstride floats]
extern "C" size_t lora_forward_workspace_bytes(int32_t n_tokens, int32_t max_rank, int32_t d_in, int32_t d_out,
                                               int32_t variant)
{
    (void)d_in; (void)d_out; (void)variant;
    if (n_tokens < 0 || max_rank < 1) return lq::kWsHeaderBytes;
    return (size_t)lq::kWsHeaderBytes + lq::h_slices_bytes(n_tokens, max_rank);
}

namespace lq {
namespace {

// Host-side checks and launch shared by the entry points below: n_proj linear layers that read the same x.
// err_word: where the kernels report device-side errors (NULL: word 0 of the workspace).
lq_status forward_checked(const void* x, int64_t ldx, int32_t d_in, int32_t n_proj, const Proj* projs,
                          const int32_t* ranks, const float* scales, const float* token_scales,
                          int32_t n_adapters, int32_t max_rank, const int32_t* perm, int32_t n_tokens,
                          const int32_t* seg_starts, const int32_t* seg_adapter, const uint8_t* seg_kind,
                          const int32_t* n_segments, int32_t max_segments, const int64_t* h_offsets,
                          int32_t variant, void* workspace, size_t workspace_bytes, int32_t* err_word, hipStream_t stream,
                          bool launch)
{
    if (n_proj < 1 || n_proj > kMaxProj || !projs) return LQ_ERR_INVALID_ARG;
    if (n_tokens < 0 || d_in <= 0 || n_adapters <= 0 || max_segments < 0 || max_rank < 1) return LQ_ERR_INVALID_ARG;
    if (variant < LQ_VARIANT_SPLIT || variant > LQ_VARIANT_AUTO) return LQ_ERR_INVALID_ARG;
    if (!ranks || !scales || !seg_starts || !seg_adapter || !seg_kind || !n_segments) return LQ_ERR_INVALID_ARG;
    if (n_tokens > 0 && !x) return LQ_ERR_INVALID_ARG;
    if (ldx < d_in) return LQ_ERR_INVALID_ARG;
    for (int k = 0; k < n_proj; ++k) {
        const Proj& q = projs[k];
        if (q.d_out <= 0 || !q.A_ptrs || !q.B_ptrs || q.ldy < q.d_out) return LQ_ERR_INVALID_ARG;
        if (n_tokens > 0 && !q.y) return LQ_ERR_INVALID_ARG;
        if (x && x == static_cast<const void*>(q.y)) return LQ_ERR_INVALID_ARG;
        for (int j = 0; j < k; ++j)
            if (q.y && q.y == projs[j].y) return LQ_ERR_INVALID_ARG;  // two layers cannot share their output
    }
    if (max_rank > LQ_MAX_RANK || n_adapters > LQ_MAX_ADAPTERS) return LQ_ERR_UNSUPPORTED;
    if ((d_in % 8) || (ldx % 8) || !aligned16(x)) return LQ_ERR_UNSUPPORTED;
    for (int k = 0; k < n_proj; ++k)
        if ((projs[k].d_out % 8) || (projs[k].ldy % 8) || !aligned16(projs[k].y)) return LQ_ERR_UNSUPPORTED;
    const size_t h_bytes = (size_t)n_proj * h_slices_bytes(n_tokens, max_rank);
    if (variant == LQ_VARIANT_AUTO) {
        long long columns = 0;
        for (int k = 0; k < n_proj; ++k) columns += projs[k].d_out;
        variant = auto_variant(max_rank, columns);
        if (variant == LQ_VARIANT_FUSED && h_bytes > 0x7fffffffull) variant = LQ_VARIANT_SLAB;  // (beyond the fused variant's reach)
    }
    if (!workspace || workspace_bytes < (size_t)kWsHeaderBytes + h_bytes || !aligned16(workspace)) return LQ_ERR_WORKSPACE;
    // the fused variant addresses the partial-h region through a buffer descriptor with 32-bit offsets
    if (variant == LQ_VARIANT_FUSED && h_bytes > 0x7fffffffull) return LQ_ERR_UNSUPPORTED;
    if (n_tokens == 0 || max_segments == 0 || !launch) return LQ_OK;

    FwdParams p;
    p.x = static_cast<const u16*>(x); p.ldx = ldx;
    p.d_in = d_in;
    p.n_proj = n_proj;
    p.proj0 = projs[0];
    for (int k = 1; k < kMaxProj; ++k) p.more[k - 1] = projs[k < n_proj ? k : 0];
    p.ranks = ranks; p.scales = scales;
    p.n_adapters = n_adapters; p.max_rank = max_rank;
    p.token_scales = token_scales;
    p.perm = perm; p.n_tokens = n_tokens;
    p.seg_starts = seg_starts; p.seg_adapter = seg_adapter; p.seg_kind = seg_kind;
    p.n_segments = n_segments; p.max_segments = max_segments;
    p.h_offsets = reinterpret_cast<const long long*>(h_offsets);
    p.rstride = rstride_for(max_rank);
    p.header = static_cast<int*>(workspace);
    p.err = err_word ? err_word : p.header;
    p.tickets = p.header + 4;
    p.hpart = reinterpret_cast<float*>(static_cast<char*>(workspace) + kWsHeaderBytes);
    p.hproj = (long long)(h_slices_bytes(n_tokens, max_rank) / sizeof(float));
    p.ksplit_hint = 0;
    p.kinds = kAllKinds;
    p.coherent = variant == LQ_VARIANT_FUSED;
    p.hpart_bytes = (unsigned int)h_bytes;
    if (variant == LQ_VARIANT_SLAB) {
        p.ksplit = 1; p.ks_log2 = 0;
        return run_slab(p, stream) == hipSuccess ? LQ_OK : LQ_ERR_HIP;
    }
    return run_shrink_expand(p, variant, stream) == hipSuccess ? LQ_OK : LQ_ERR_HIP;
}

Proj one_projection(void* y, int64_t ldy, int32_t d_out, const void* const* A_ptrs, const void* const* B_ptrs, float* h_out)
{
    Proj q;
    q.y = static_cast<u16*>(y); q.ldy = ldy; q.d_out = d_out;
    q.A_ptrs = A_ptrs; q.B_ptrs = B_ptrs; q.h_out = h_out;
    return q;
}

}  // namespace
}  // namespace lq

extern "C" size_t lora_forward_group_workspace_bytes(int32_t n_proj, int32_t n_tokens, int32_t max_rank)
{
    if (n_proj < 1 || n_tokens < 0 || max_rank < 1) return lq::kWsHeaderBytes;
    return (size_t)lq::kWsHeaderBytes + (size_t)n_proj * lq::h_slices_bytes(n_tokens, max_rank);
}

extern "C" lq_status lora_segmented_forward(const void* x, int64_t ldx, void* y, int64_t ldy,
                                            int32_t d_in, int32_t d_out,
                                            const void* const* A_ptrs, const void* const* B_ptrs,
                                            const int32_t* ranks, const float* scales, const float* token_scales,
                                            int32_t n_adapters, int32_t max_rank,
                                            const int32_t* perm, int32_t n_tokens,
                                            const int32_t* seg_starts, const int32_t* seg_adapter,
                                            const uint8_t* seg_kind,
                                            const int32_t* n_segments, int32_t max_segments,
                                            float* h_out, const int64_t* h_offsets,
                                            int32_t variant, void* workspace, size_t workspace_bytes, void* stream)
{
    const lq::Proj q = lq::one_projection(y, ldy, d_out, A_ptrs, B_ptrs, h_offsets ? h_out : nullptr);
    return lq::forward_checked(x, ldx, d_in, 1, &q, ranks, scales, token_scales, n_adapters, max_rank, perm, n_tokens,
                               seg_starts, seg_adapter, seg_kind, n_segments, max_segments, h_offsets, variant,
                               workspace, workspace_bytes, nullptr, static_cast<hipStream_t>(stream), true);
}

extern "C" lq_status lora_segmented_forward_group(const void* x, int64_t ldx, int32_t d_in, int32_t n_proj,
                                                  void* const* host_y, const int64_t* host_ldy, const int32_t* host_d_out,
                                                  const void* const* const* host_A_ptrs,
                                                  const void* const* const* host_B_ptrs, float* const* host_h_out,
                                                  const int32_t* ranks, const float* scales, const float* token_scales,
                                                  int32_t n_adapters, int32_t max_rank,
                                                  const int32_t* perm, int32_t n_tokens,
                                                  const int32_t* seg_starts, const int32_t* seg_adapter,
                                                  const uint8_t* seg_kind,
                                                  const int32_t* n_segments, int32_t max_segments,
                                                  const int64_t* h_offsets,
                                                  int32_t variant, void* workspace, size_t workspace_bytes, void* stream)
{
    if (n_proj < 1 || n_proj > LQ_MAX_GROUP) return LQ_ERR_INVALID_ARG;
    if (!host_y || !host_ldy || !host_d_out || !host_A_ptrs || !host_B_ptrs) return LQ_ERR_INVALID_ARG;
    lq::Proj projs[lq::kMaxProj];
    for (int k = 0; k < n_proj; ++k)
        projs[k] = lq::one_projection(host_y[k], host_ldy[k], host_d_out[k], host_A_ptrs[k], host_B_ptrs[k],
                                      host_h_out && h_offsets ? host_h_out[k] : nullptr);
    return lq::forward_checked(x, ldx, d_in, n_proj, projs, ranks, scales, token_scales, n_adapters, max_rank, perm, n_tokens,
                               seg_starts, seg_adapter, seg_kind, n_segments, max_segments, h_offsets, variant,
                               workspace, workspace_bytes, nullptr, static_cast<hipStream_t>(stream), true);
}

// ---------------------------------------------------------------------------------------------------------------
// The forward for callers that cannot allocate (code under HIP graph capture, tight serving loops): the workspace
// is a file-scope device array instead of a caller buffer.  Every GPU holds its own copy of the array at its own
// address, looked up once per device; host code only ever uses that looked-up address, never the array's name.
// ---------------------------------------------------------------------------------------------------------------
namespace lq {
namespace {

static __device__ __align__(256) unsigned char scratch[LQ_STATIC_WORKSPACE_BYTES];

void* g_scratch_ptr[kMaxDevices];  // per device: address of that device's copy of `scratch` (null: not looked up yet)
std::mutex g_scratch_mutex;

// address of the current device's scratch array (looked up on the first call on that device), or null
void* scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

// The header's counters must start at zero.  Every launch leaves them there, except one whose device-wide wait ran
// out; the previous call's partial h may stay.  A fill kernel rather than a memset node, so that the call can be
// captured into a graph.
__global__ __launch_bounds__(1024) void clear_header_kernel(int* header)
{
    header[threadIdx.x] = 0;
}

}  // namespace
}  // namespace lq

extern "C" lq_status lora_segmented_forward_static(const void* x, int64_t ldx, void* y, int64_t ldy,
                                                   int32_t d_in, int32_t d_out,
                                                   const void* const* A_ptrs, const void* const* B_ptrs,
                                                   const int32_t* ranks, const float* scales, const float* token_scales,
                                                   int32_t n_adapters, int32_t max_rank,
                                                   const int32_t* perm, int32_t n_tokens,
                                                   const int32_t* seg_starts, const int32_t* seg_adapter,
                                                   const uint8_t* seg_kind,
                                                   const int32_t* n_segments, int32_t max_segments,
                                                   float* h_out, const int64_t* h_offsets,
                                                   int32_t variant, int32_t* error_word, void* stream)
{
    using namespace lq;
    static_assert(kWsHeaderBytes == 1024 * sizeof(int), "clear_header_kernel clears one word per thread");
    if (variant != LQ_VARIANT_SPLIT && variant != LQ_VARIANT_FUSED && variant != LQ_VARIANT_SLAB && variant != LQ_VARIANT_AUTO)
        return LQ_ERR_INVALID_ARG;
    // (sizes first: a batch beyond the array's capacity is refused whatever else is wrong with the call)
    if (n_tokens > 0 && max_rank >= 1 && max_rank <= LQ_MAX_RANK &&
        lora_forward_workspace_bytes(n_tokens, max_rank, d_in, d_out, variant) > (size_t)LQ_STATIC_WORKSPACE_BYTES)
        return LQ_ERR_WORKSPACE;
    // host-side validation with a stand-in workspace address: nothing is launched, nothing is dereferenced
    void* const stand_in = reinterpret_cast<void*>(uintptr_t{256});
    const Proj q = one_projection(y, ldy, d_out, A_ptrs, B_ptrs, h_offsets ? h_out : nullptr);
    lq_status status = forward_checked(x, ldx, d_in, 1, &q, ranks, scales, token_scales, n_adapters, max_rank, perm,
                                       n_tokens, seg_starts, seg_adapter, seg_kind, n_segments, max_segments, h_offsets,
                                       variant, stand_in, (size_t)LQ_STATIC_WORKSPACE_BYTES, error_word, nullptr, false);
    if (status != LQ_OK || n_tokens == 0 || max_segments == 0) return status;
    void* ws = scratch_of_current_device();
    if (!ws) return LQ_ERR_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(clear_header_kernel, dim3(1), dim3(1024), 0, st, static_cast<int*>(ws));
    if (hipGetLastError() != hipSuccess) return LQ_ERR_HIP;
    return forward_checked(x, ldx, d_in, 1, &q, ranks, scales, token_scales, n_adapters, max_rank, perm, n_tokens,
                           seg_starts, seg_adapter, seg_kind, n_segments, max_segments, h_offsets, variant, ws,
                           (size_t)LQ_STATIC_WORKSPACE_BYTES, error_word, st, true);
}
