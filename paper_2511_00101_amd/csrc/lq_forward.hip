// Segmented multi-adapter LoRA forward (Section 3.3): shrink (h = x A_a^T per segment), h-save for
// fine-tune segments, expand (y += s_a h B_a).
//
// Work decomposition.  Every workgroup (8 waves) reads the segment tables itself (one wave scan per 64
// segments, cached in registers), so the grid is a fixed number of resident workgroups that stride
// over "units" and no plan buffer or extra launch is needed.
//   shrink unit        : 32 rows of one segment x one of `ksplit` interleaved slices of d_in.  16x16x32
//                        bf16 MFMA; the 8 waves take alternate 64-wide k blocks and tree-reduce through
//                        LDS (fixed order, so results are reproducible); the unit stores one partial h.
//                        Segments of any length take this path (the MFMA does the k reduction for free
//                        even when only a few of the 16 tile rows are live).
//   expand, long unit  : 64 rows of a segment with >= 16 rows x 512 columns of d_out.  The B_a block is
//                        staged once in LDS and transposed into MFMA fragments held in registers; y is
//                        streamed once (read-modify-write).
//   expand, short unit : one wave: <= 4 rows of a segment with < 16 rows x 512 columns.  B_a rows are
//                        streamed with 16-byte loads, h is broadcast from LDS, plain FMAs.
// x and y are accessed with 16-byte loads/stores straight in the MFMA operand layout (16 rows x 64
// contiguous bytes per instruction), which on MI355X streams within a few percent of a row-contiguous
// pattern, so neither goes through LDS.
#include "lq_common.h"

namespace lq {
namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kWave;
constexpr int kLongMin = 16;   // expand: segments with at least this many rows take the MFMA path
constexpr int kTT = 4;         // expand, short path: rows per unit
constexpr int kTileM = 32;     // shrink unit: rows (two 16-row MFMA tiles)
constexpr int kBlockK = 64;    // shrink: k elements per wave step (two MFMA k steps)
constexpr int kChunkT = 256;   // expand, long unit: rows (amortises staging the unit's block of B)
constexpr int kShortN = 512;   // expand, short unit: columns (64 lanes x 8)
constexpr int kMaxKSplit = 8;
constexpr int kXcds = 8;        // accelerator complex dies, each with its own L2

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
    float* hpart;    // [ksplit][n_tokens][rstride] partial h by position in segment order (unscaled)
    int ksplit;
    int rstride;     // multiple of 32
    int* err;
};

// ---- segment tables -----------------------------------------------------------------------------
struct SegLane { int st, en, ad, kd; };  // table entries of segment (batch * 64 + lane); empty beyond n_seg

__device__ __forceinline__ SegLane load_seg_lane(const FwdParams& p, int n_seg, int s)
{
    // the tables hold max_segments entries, so the loads can go out before n_seg has arrived
    const int sc = min(s, p.max_segments - 1);
    SegLane c;
    c.st = p.seg_starts[sc];
    c.en = p.seg_starts[sc + 1];
    c.ad = p.seg_adapter[sc];
    c.kd = p.seg_kind[sc];
    if (s >= n_seg) c.st = c.en = c.ad = c.kd = 0;
    return c;
}

struct Unit { int seg, pos, len, first, ad, kd; };

enum { kAll = 0, kLong = 1, kShort = 2 };  // which segments a chunk enumeration covers

__device__ __forceinline__ int chunks_in(int len, int per, int cls)
{
    const bool take = len > 0 && (cls == kAll || (len >= kLongMin) == (cls == kLong));
    return take ? (len + per - 1) / per : 0;
}

__device__ __forceinline__ int wave_sum(int v) { return uniform(__shfl(wave_inclusive_scan(v), kWave - 1, kWave)); }

// number of chunks of `per` rows over the segments of a class; wave uniform
__device__ __forceinline__ int count_chunks(const FwdParams& p, int n_seg, const SegLane& c0, int per, int cls)
{
    int total = wave_sum(chunks_in(c0.en - c0.st, per, cls));
    for (int s0 = kWave; s0 < n_seg; s0 += kWave) {
        const SegLane c = load_seg_lane(p, n_seg, s0 + lane_id());
        total += wave_sum(chunks_in(c.en - c.st, per, cls));
    }
    return total;
}

// the id-th chunk (ids count through the segments of the class in order); wave uniform result
__device__ __forceinline__ bool find_chunk(const FwdParams& p, int n_seg, const SegLane& c0, int id, int per,
                                           int cls, Unit& u)
{
    int base = 0;
    for (int s0 = 0; s0 < n_seg; s0 += kWave) {
        const SegLane c = s0 == 0 ? c0 : load_seg_lane(p, n_seg, s0 + lane_id());
        const int nch = chunks_in(c.en - c.st, per, cls);
        const int incl = wave_inclusive_scan(nch);
        const int total = uniform(__shfl(incl, kWave - 1, kWave));
        if (id < base + total) {
            const unsigned long long m = __ballot(base + incl > id);
            const int l = __ffsll((long long)m) - 1;
            const int local = id - base - uniform(__shfl(incl - nch, l, kWave));
            u.seg = s0 + l;
            u.first = uniform(__shfl(c.st, l, kWave));
            u.pos = u.first + local * per;
            u.len = min(per, uniform(__shfl(c.en, l, kWave)) - u.pos);
            u.ad = uniform(__shfl(c.ad, l, kWave));
            u.kd = uniform(__shfl(c.kd, l, kWave));
            return true;
        }
        base += total;
    }
    return false;
}

// Adapter matrices come from a pointer table, so the compiler cannot infer their address space; saying
// "global" turns flat loads into global loads.
typedef const __attribute__((address_space(1))) u16* gconst_u16;

struct SegInfo {
    gconst_u16 A; gconst_u16 B;
    int rank; float scale;
    bool ok;
};

__device__ __forceinline__ SegInfo load_adapter(const FwdParams& p, const Unit& u)
{
    SegInfo s;
    s.A = s.B = nullptr;
    s.rank = 0;
    s.scale = 0.f;
    s.ok = u.ad >= 0 && u.ad < p.n_adapters;
    if (s.ok) {
        s.rank = p.ranks[u.ad];
        s.scale = p.scales[u.ad];
        s.A = (gconst_u16)(p.A_ptrs[u.ad]);
        s.B = (gconst_u16)(p.B_ptrs[u.ad]);
        s.ok = s.rank >= 1 && s.rank <= p.max_rank && s.A && s.B;
    }
    if (!s.ok && threadIdx.x == 0) atomicOr(p.err, kErrBadSegment);
    return s;
}

// row of x / y for a position of the segment order; -1 if the table holds an invalid row
__device__ __forceinline__ int row_of(const FwdParams& p, int pos)
{
    // branch free: with perm == NULL a dummy entry is loaded and ignored
    const int32_t* tab = p.perm ? p.perm : p.seg_starts;
    const int v = tab[p.perm ? pos : 0];
    const int row = p.perm ? v : pos;
    return (row >= 0 && row < p.n_tokens) ? row : -1;
}

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& v) { return __builtin_bit_cast(bf16x8, v); }

// =================================================================================================
// shrink: D[row][rank] = sum_k x[row][k] A[rank][k] with 16x16x32 bf16 MFMA.
// Lane (c = lane % 16, kg = lane / 16) supplies x[row c][8 kg ..] and A[rank c][8 kg ..] of a 32-wide k
// step and receives D[row 4 kg + v][rank c].  d_in is cut into 64-wide blocks; block b belongs to
// slice (b / 8) % ksplit and to wave b % 8 of the workgroup that owns the slice.
// =================================================================================================
template <int NT>  // 16-rank tiles: ranks up to 16 * NT
__device__ __forceinline__ void shrink_unit(const FwdParams& p, const Unit& u, const SegInfo& s, int ks, float* lds)
{
    constexpr int MT = kTileM / 16;
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
    const int rot = n_full > 0 ? (int)(((unsigned)u.pos / kTileM * 37u) % (unsigned)n_full) : 0;  // same for all slices
    auto load = [&](int blk, u32x4 (&xv)[MT][2], u32x4 (&av)[NT][2]) {  // a block that lies fully inside d_in
        blk += rot;
        if (blk >= n_full) blk -= n_full;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int k = blk * kBlockK + 32 * q;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xv[mt][q] = *reinterpret_cast<const u32x4*>(xrow[mt] + k);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) av[nt][q] = *(const __attribute__((address_space(1))) u32x4*)(arow[nt] + k);
        }
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
                const u32x4 v = *(const __attribute__((address_space(1))) u32x4*)(arow[nt] + kc);
                aa[nt][q] = in ? v : u32x4{0u, 0u, 0u, 0u};
            }
        }
        mma(xa, aa);
    }

    // tree reduction over the 8 waves in a fixed order: slots[4][MT * NT * 4][64 lanes]
    constexpr int REGS = MT * NT * 4;
#pragma unroll
    for (int half = kWaves / 2; half >= 1; half >>= 1) {
        if (w >= half && w < 2 * half) {
            float* slot = lds + (size_t)(w - half) * REGS * kWave + lane;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) slot[((mt * NT + nt) * 4 + v) * kWave] = acc[mt][nt][v];
        }
        __syncthreads();
        if (w < half) {
            const float* slot = lds + (size_t)w * REGS * kWave + lane;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[mt][nt][v] += slot[((mt * NT + nt) * 4 + v) * kWave];
        }
        __syncthreads();
    }

    if (w == 0) {
        float* part = p.hpart + ((long long)ks * p.n_tokens + u.pos) * p.rstride;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int i = mt * 16 + kg * 4 + v, j = nt * 16 + c;
                    if (i < u.len && j < s.rank) part[(long long)i * p.rstride + j] = acc[mt][nt][v];
                }
    }
}

// =================================================================================================
// expand, long segments: D[col][row] = sum_j B[j][col] (s h[row][j]) with 16x16x32 bf16 MFMA, h split
// into a bf16 high and low part so that it keeps fp32 accuracy.  The output columns of two MFMA tiles
// are interleaved so that a lane ends up with 8 consecutive columns of one row: a 16-byte access to y.
// For pair q and tile m, MFMA row rho maps to column 32 q + 8 (rho / 4) + 4 m + (rho % 4) of the wave's
// column range.  The unit's block of B is staged in LDS with coalesced loads, transposed into
// fragments once and kept in registers while the rows stream by.
// =================================================================================================
__device__ __forceinline__ void split_bf16(const float (&v)[8], u32x4& hi, u32x4& lo)
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

template <int KSTEPS, int PAIRS, bool MULTI>  // ranks up to 32 * KSTEPS; a wave covers 32 * PAIRS columns, the unit
                                              // 8 waves; MULTI: h arrives as several partials (ksplit > 1)
__device__ __forceinline__ void expand_long_unit(const FwdParams& p, const Unit& u, const SegInfo& s, int n_block,
                                                 u16* lds_b)
{
    constexpr int WN = 32 * PAIRS, UN = kWaves * WN, ROWS = 32 * KSTEPS;
    constexpr int PITCH = UN + 8;  // elements; keeps rows 16-byte aligned and spreads them over banks
    constexpr int STAGE = ROWS * (UN / 8) / kThreads;  // 16-byte pieces of the B block per thread
    static_assert(ROWS * (UN / 8) % kThreads == 0, "staging loop assumes an even split");
    const int lane = lane_id(), w = uniform((int)threadIdx.x / kWave), c = lane & 15, g = lane >> 4;
    const int n_unit = n_block * UN;

    {
        u32x4 v[STAGE];
#pragma unroll
        for (int i = 0; i < STAGE; ++i) {
            const int id = (int)threadIdx.x + i * kThreads;
            const int j = id / (UN / 8), n = n_unit + (id % (UN / 8)) * 8;
            v[i] = *(const __attribute__((address_space(1))) u32x4*)(s.B + (long long)min(j, s.rank - 1) * p.d_out +
                                                                     min(n, p.d_out - 8));
        }
        __syncthreads();  // the previous unit's fragment reads are done
#pragma unroll
        for (int i = 0; i < STAGE; ++i) {
            const int id = (int)threadIdx.x + i * kThreads;
            const int j = id / (UN / 8), n = n_unit + (id % (UN / 8)) * 8;
            const bool live = j < s.rank && n < p.d_out;
            *reinterpret_cast<u32x4*>(lds_b + j * PITCH + (n - n_unit)) = live ? v[i] : u32x4{0u, 0u, 0u, 0u};
        }
    }
    // fine-tune segments: the unit of the first column block also stores the unscaled h rows
    if (u.kd == LQ_SEG_FINETUNE && p.h_out && p.h_offsets && n_block == 0) {
        float* dst = p.h_out + p.h_offsets[u.seg] + (long long)(u.pos - u.first) * s.rank;
        for (int id = (int)threadIdx.x; id < u.len * s.rank; id += kThreads) {
            const int i = id / s.rank, j = id - i * s.rank;
            float sum = 0.f;
            for (int part = 0; part < p.ksplit; ++part)
                sum += p.hpart[((long long)part * p.n_tokens + u.pos + i) * p.rstride + j];
            dst[id] = sum;
        }
    }
    __syncthreads();

    const int n_wave = n_unit + w * WN;
    if (n_wave >= p.d_out) return;
    u32x4 bfrag[PAIRS][2][KSTEPS];
#pragma unroll
    for (int q = 0; q < PAIRS; ++q)
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const u16* col = lds_b + w * WN + 32 * q + 8 * (c >> 2) + 4 * m + (c & 3);
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                unsigned int e[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) e[i] = col[(32 * ks + 8 * g + i) * PITCH];
                bfrag[q][m][ks] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
            }
        }

    const int n_tiles = (u.len + 15) / 16;
    const int n_lane = n_wave + 8 * g;  // + 32 q

    // software pipeline: the next tile's row index, y and h are in flight while this one is computed.
    // Loads are unconditional (dead rows and columns read a live address); only the stores are masked.
    const int safe_row = max(row_of(p, u.pos), 0);
    int n_ld[PAIRS];
#pragma unroll
    for (int q = 0; q < PAIRS; ++q) n_ld[q] = min(n_lane + 32 * q, p.d_out - 8);
    int row_n;
    u32x4 y_n[PAIRS];
    f32x4 h_n[KSTEPS][2];
    auto fetch = [&](int tile) {
        const int i = tile * 16 + c;
        row_n = i < u.len ? row_of(p, u.pos + i) : -1;
        const u16* yrow = p.y + (long long)(row_n >= 0 ? row_n : safe_row) * p.ldy;
#pragma unroll
        for (int q = 0; q < PAIRS; ++q) y_n[q] = *reinterpret_cast<const u32x4*>(yrow + n_ld[q]);
        const float* hp = p.hpart + (long long)(u.pos + min(i, u.len - 1)) * p.rstride + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            h_n[ks][0] = *reinterpret_cast<const f32x4*>(hp + 32 * ks);
            h_n[ks][1] = *reinterpret_cast<const f32x4*>(hp + 32 * ks + 4);
        }
        if constexpr (MULTI) {
            for (int part = 1; part < p.ksplit; ++part) {
                const float* hq = hp + (long long)part * p.n_tokens * p.rstride;
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) {
                    h_n[ks][0] += *reinterpret_cast<const f32x4*>(hq + 32 * ks);
                    h_n[ks][1] += *reinterpret_cast<const f32x4*>(hq + 32 * ks + 4);
                }
            }
        }
    };
    fetch(0);
    for (int tile = 0; tile < n_tiles; ++tile) {
        const int row = row_n;
        u32x4 yv[PAIRS];
        f32x4 hv[KSTEPS][2];
#pragma unroll
        for (int q = 0; q < PAIRS; ++q) yv[q] = y_n[q];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) { hv[ks][0] = h_n[ks][0]; hv[ks][1] = h_n[ks][1]; }
        fetch(min(tile + 1, n_tiles - 1));  // unconditional, so the loads in flight are counted statically

        u32x4 h_hi[KSTEPS], h_lo[KSTEPS];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int j = 32 * ks + 8 * g + i;
                const float raw = i < 4 ? hv[ks][0][i & 3] : hv[ks][1][i & 3];
                v[i] = (row >= 0 && j < s.rank) ? raw * s.scale : 0.f;
            }
            split_bf16(v, h_hi[ks], h_lo[ks]);
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
        if (row >= 0) {
#pragma unroll
            for (int q = 0; q < PAIRS; ++q) {
                if (n_lane + 32 * q < p.d_out) {
                    float yf[8];
                    unpack8(yv[q], yf);
                    u32x4 o;
                    o.x = pack_bf16x2(yf[0] + acc[q][0][0], yf[1] + acc[q][0][1]);
                    o.y = pack_bf16x2(yf[2] + acc[q][0][2], yf[3] + acc[q][0][3]);
                    o.z = pack_bf16x2(yf[4] + acc[q][1][0], yf[5] + acc[q][1][1]);
                    o.w = pack_bf16x2(yf[6] + acc[q][1][2], yf[7] + acc[q][1][3]);
                    *reinterpret_cast<u32x4*>(p.y + (long long)row * p.ldy + n_lane + 32 * q) = o;
                }
            }
        }
    }
}

// =================================================================================================
// expand, short segments: one wave per unit of <= 4 rows x 512 columns.  The wave sums the partial h
// of its rows into its own LDS slab (scaled), then for every rank row j streams B[j][n .. n + 8) with
// one 16-byte load per lane and accumulates h[t][j] * B[j][n + i] for the four rows.
// =================================================================================================
struct ShortLds {
    __attribute__((aligned(16))) float hs[kWaves][LQ_MAX_RANK][kTT];  // per wave: hs[rank][row], scaled
};

__device__ __forceinline__ void expand_short_unit(const FwdParams& p, const Unit& u, const SegInfo& s, int n_block,
                                                  ShortLds& sh)
{
    const int lane = lane_id(), w = uniform((int)threadIdx.x / kWave);
    float (*hs)[kTT] = sh.hs[w];
    const bool save = u.kd == LQ_SEG_FINETUNE && p.h_out && p.h_offsets && n_block == 0;
    const long long h_base = save ? p.h_offsets[u.seg] + (long long)(u.pos - u.first) * s.rank : 0;
    for (int i = lane; i < s.rank * kTT; i += kWave) {
        const int t = i / s.rank, j = i - t * s.rank;
        float sum = 0.f;
        if (t < u.len) {
            for (int part = 0; part < p.ksplit; ++part)
                sum += p.hpart[((long long)part * p.n_tokens + u.pos + t) * p.rstride + j];
            if (save) p.h_out[h_base + (long long)t * s.rank + j] = sum;
        }
        hs[j][t] = sum * s.scale;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    int row[kTT];
#pragma unroll
    for (int t = 0; t < kTT; ++t) row[t] = t < u.len ? row_of(p, u.pos + t) : -1;
    const int n = n_block * kShortN + lane * 8;
    if (n < p.d_out) {
        const int safe_row = max(row[0], 0);
        u32x4 yv[kTT];
#pragma unroll
        for (int t = 0; t < kTT; ++t)
            yv[t] = *reinterpret_cast<const u32x4*>(p.y + (long long)(row[t] >= 0 ? row[t] : safe_row) * p.ldy + n);
        float acc[kTT][8];
#pragma unroll
        for (int t = 0; t < kTT; ++t)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[t][i] = 0.f;
#pragma unroll 8
        for (int j = 0; j < s.rank; ++j) {
            const u32x4 v = *(const __attribute__((address_space(1))) u32x4*)(s.B + (long long)j * p.d_out + n);
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
                float yf[8];
                unpack8(yv[t], yf);
                u32x4 o;
                o.x = pack_bf16x2(yf[0] + acc[t][0], yf[1] + acc[t][1]);
                o.y = pack_bf16x2(yf[2] + acc[t][2], yf[3] + acc[t][3]);
                o.z = pack_bf16x2(yf[4] + acc[t][4], yf[5] + acc[t][5]);
                o.w = pack_bf16x2(yf[6] + acc[t][6], yf[7] + acc[t][7]);
                *reinterpret_cast<u32x4*>(p.y + (long long)row[t] * p.ldy + n) = o;
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
__global__ __launch_bounds__(kThreads) void shrink_kernel(FwdParams p)
{
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    const int n_seg = uniform(min(*p.n_segments, p.max_segments));
    const SegLane c0 = load_seg_lane(p, n_seg, lane_id());
    const int n_units = count_chunks(p, n_seg, c0, kTileM, kAll) * p.ksplit;
    // Workgroup b runs on XCD b % 8 (round-robin dispatch).  Each XCD takes one contiguous eighth of the
    // units, so the tiles of a segment share their adapter's A through one L2 instead of eight.
    const int n_xcd = (int)gridDim.x % kXcds == 0 ? kXcds : 1;
    const int per_xcd = (n_units + n_xcd - 1) / n_xcd;
    const int first = ((int)blockIdx.x % n_xcd) * per_xcd, last = min(n_units, first + per_xcd);
    for (int id = first + (int)blockIdx.x / n_xcd; id < last; id += (int)gridDim.x / n_xcd) {
        Unit u;
        if (!find_chunk(p, n_seg, c0, id / p.ksplit, kTileM, kAll, u)) continue;
        const SegInfo s = load_adapter(p, u);
        if (!s.ok) continue;
        shrink_unit<NT>(p, u, s, id % p.ksplit, lds_f);
    }
}

template <int KSTEPS, int PAIRS, bool MULTI>
__global__ __launch_bounds__(kThreads) void expand_kernel(FwdParams p)
{
    extern __shared__ __attribute__((aligned(16))) u16 lds_b[];
    __shared__ ShortLds sh;
    const int n_seg = uniform(min(*p.n_segments, p.max_segments));
    const SegLane c0 = load_seg_lane(p, n_seg, lane_id());

    // long units, one per workgroup iteration
    constexpr int UN = kWaves * 32 * PAIRS;
    const int long_blocks = (p.d_out + UN - 1) / UN;
    const int n_long = count_chunks(p, n_seg, c0, kChunkT, kLong) * long_blocks;
    for (int id = (int)blockIdx.x; id < n_long; id += (int)gridDim.x) {
        Unit u;
        if (!find_chunk(p, n_seg, c0, id / long_blocks, kChunkT, kLong, u)) continue;
        const SegInfo s = load_adapter(p, u);
        if (!s.ok) continue;
        expand_long_unit<KSTEPS, PAIRS, MULTI>(p, u, s, id % long_blocks, lds_b);
    }

    // short units, one per wave iteration, dealt round-robin over the workgroups first so that a few
    // hundred units spread over all compute units
    const int short_blocks = (p.d_out + kShortN - 1) / kShortN;
    const int n_short = count_chunks(p, n_seg, c0, kTT, kShort) * short_blocks;
    const int w = uniform((int)threadIdx.x / kWave);
    for (int id = w * (int)gridDim.x + (int)blockIdx.x; id < n_short; id += kWaves * (int)gridDim.x) {
        Unit u;
        if (!find_chunk(p, n_seg, c0, id / short_blocks, kTT, kShort, u)) continue;
        const SegInfo s = load_adapter(p, u);
        if (!s.ok) continue;
        expand_short_unit(p, u, s, id % short_blocks, sh);
    }
}

int rstride_for(int max_rank) { return (max_rank + 31) / 32 * 32; }
int ksplit_cap(int n_tokens) { return n_tokens <= 16384 ? kMaxKSplit : 1; }
int nt_for(int max_rank) { return max_rank <= 16 ? 1 : max_rank <= 32 ? 2 : max_rank <= 64 ? 4 : 8; }
size_t shrink_lds_bytes(int nt) { return (size_t)(kWaves / 2) * (kTileM / 16) * nt * 4 * kWave * sizeof(float); }
size_t expand_lds_bytes(int ksteps, int pairs) { return (size_t)32 * ksteps * (kWaves * 32 * pairs + 8) * sizeof(u16); }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// number of workgroups of `kernel` that are resident at once on the current device
template <typename K>
int resident_grid(K kernel, size_t dyn_lds)
{
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, dyn_lds) != hipSuccess || per_cu <= 0)
        per_cu = 1;
    return cus * per_cu;
}

template <int NT>
int shrink_grid()
{
    static int grid = 0;
    if (!grid) grid = resident_grid(shrink_kernel<NT>, shrink_lds_bytes(NT));
    return grid;
}

// Few rows: cut d_in into slices so that the shrink units still cover the machine.  A pure function of
// host arguments, so the two halves of the split variant agree on it.
int choose_ksplit(int n_tokens, int seg_bound, int d_in, int grid)
{
    const long long tiles_est = (n_tokens + kTileM - 1) / kTileM + seg_bound / 2;
    int ks = 1;
    while (ks < ksplit_cap(n_tokens) && tiles_est * ks * 2 <= grid && d_in >= ks * 2 * kWaves * kBlockK) ks *= 2;
    return ks;
}

template <int NT>
hipError_t launch_shrink(const FwdParams& p, hipStream_t st)
{
    hipLaunchKernelGGL(shrink_kernel<NT>, dim3(shrink_grid<NT>()), dim3(kThreads), shrink_lds_bytes(NT), st, p);
    return hipGetLastError();
}

template <int KSTEPS, int PAIRS, bool MULTI>
hipError_t launch_expand_as(const FwdParams& p, hipStream_t st)
{
    static int grid = 0;
    const size_t lds = expand_lds_bytes(KSTEPS, PAIRS);
    if (!grid) {
        if (lds > 48 * 1024)
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(expand_kernel<KSTEPS, PAIRS, MULTI>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        grid = resident_grid(expand_kernel<KSTEPS, PAIRS, MULTI>, lds);
    }
    hipLaunchKernelGGL((expand_kernel<KSTEPS, PAIRS, MULTI>), dim3(grid), dim3(kThreads), lds, st, p);
    return hipGetLastError();
}

template <int KSTEPS, int PAIRS>
hipError_t launch_expand(const FwdParams& p, hipStream_t st)
{
    return p.ksplit > 1 ? launch_expand_as<KSTEPS, PAIRS, true>(p, st) : launch_expand_as<KSTEPS, PAIRS, false>(p, st);
}

}  // namespace
}  // namespace lq

extern "C" size_t lora_forward_workspace_bytes(int32_t n_tokens, int32_t max_rank, int32_t d_in, int32_t d_out,
                                               int32_t variant)
{
    (void)d_in; (void)d_out; (void)variant;
    if (n_tokens < 0 || max_rank < 1) return lq::kWsHeaderBytes;
    return (size_t)lq::kWsHeaderBytes +
           (size_t)lq::ksplit_cap(n_tokens) * (size_t)n_tokens * (size_t)lq::rstride_for(max_rank) * sizeof(float);
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
    if (variant < LQ_VARIANT_SPLIT || variant > LQ_VARIANT_EXPAND_ONLY) return LQ_ERR_INVALID_ARG;
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
    p.rstride = rstride_for(max_rank);
    p.ksplit = 1;

    int seg_bound = max_segments;
    if (seg_bound > n_tokens) seg_bound = n_tokens;
    if ((long long)seg_bound > 3LL * n_adapters) seg_bound = 3 * n_adapters;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nt = nt_for(max_rank);
    const int grid_s = nt == 1 ? shrink_grid<1>() : nt == 2 ? shrink_grid<2>() : nt == 4 ? shrink_grid<4>() : shrink_grid<8>();
    p.ksplit = choose_ksplit(n_tokens, seg_bound, d_in, grid_s);
    hipError_t e = hipSuccess;
    if (variant != LQ_VARIANT_EXPAND_ONLY) {
        e = nt == 1 ? launch_shrink<1>(p, st) : nt == 2 ? launch_shrink<2>(p, st)
          : nt == 4 ? launch_shrink<4>(p, st) : launch_shrink<8>(p, st);
        if (e != hipSuccess) return LQ_ERR_HIP;
        if (variant == LQ_VARIANT_SHRINK_ONLY) return LQ_OK;
    }
    e = max_rank <= 32 ? launch_expand<1, 2>(p, st) : max_rank <= 64 ? launch_expand<2, 2>(p, st) : launch_expand<4, 1>(p, st);
    return e == hipSuccess ? LQ_OK : LQ_ERR_HIP;
}
