// Device code of the row-slab forward (the kernel and its launch are in lq_slab.hip): a workgroup takes a slab of at
// most 32 rows of one segment;
//   phase 1: h = x A_a^T over all of d_in (the 8 waves take alternate 64-wide k blocks and add their results in LDS)
//   phase 2: y += s h B_a (the 8 waves take alternate 64-column blocks)
// All global accesses are row-wise 16-byte accesses (an instruction covers 8 rows x 128 contiguous bytes); data
// reaches the MFMA operand layout through slabs of LDS that belong to one wave, so the streaming loops contain no
// workgroup barrier.  Loads are issued ahead into the registers the previous block has just left, unconditionally
// and from clamped addresses, in the order they are consumed, so that the number in flight is static.
#pragma once

#include "lq_internal.h"

namespace lq {
namespace {

constexpr int kSlabRows = 32;          // rows of a unit: two 16-row MFMA tiles
constexpr int kKB = 64;                // k elements per block (phase 1), columns per block (phase 2)
constexpr int kPitch = kKB + 8;        // elements per slab row (16-byte aligned, bank spread)
constexpr int kChunk = 32 * kPitch;    // elements of a 32-row slab
constexpr int kSlabBig = 0x7fffffff;
constexpr size_t kWaveBytes = 16384;   // LDS of one wave: its slabs, later its share of the reduction buffer

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// 16 bytes of an adapter matrix at element offset `off` (< 2^31): a wave-uniform base and a 32-bit byte offset per
// lane, the form that needs no 64-bit address arithmetic in vector registers
__device__ __forceinline__ u32x4 load_at(gconst_u16 base, unsigned int off)
{
    typedef const __attribute__((address_space(1))) char* gconst_char;
    return *reinterpret_cast<gconst_u32x4>(reinterpret_cast<gconst_char>(base) + (size_t)(off * 2u));
}

// projections a pass can hold in registers: its accumulators are NP x 2 x NT MFMA tiles
template <int NT> constexpr int pass_projections() { return NT == 1 ? kMaxProj : NT == 2 ? 3 : 1; }

// =================================================================================================
// phase 1: acc[q][mt][nt] = this wave's share of x[rows] . A_q[ranks]^T for the NP projections of the pass
// (D[row][rank]: lane (c, kg) receives rows 4 kg .. + 3 of tile mt, rank c of tile nt)
// =================================================================================================
template <int NT, int NP, int MT, class PP>
__device__ __forceinline__ void slab_shrink(const PP& p, const Unit&, const SegInfo (&s)[NP], const int* lds_row,
                                            u16* slab, f32x4 (&acc)[NP][2][NT])
{
    constexpr int NJ = 2 * MT;            // load instructions per block of x (8 rows each)
    constexpr int NA = 2 * NT;            // load instructions per block of one A (8 rank rows each)
    constexpr int NCH = (NT + 1) / 2;     // 32-rank chunks of A
    const int lane = lane_id(), w = uniform((int)threadIdx.x / kWave), c = lane & 15, kg = lane >> 4;
    const int r8 = lane >> 3, piece = lane & 7;
    u16* xs = slab;             // [32][kPitch]
    u16* as = slab + kChunk;    // [2][32][kPitch]
    const int rank = s[0].rank;

    const int nblk = (p.d_in + kKB - 1) / kKB;
    const int n_mine = w < nblk ? (nblk - w + kWaves - 1) / kWaves : 0;  // blocks w, w + 8, ...
    if (n_mine == 0) return;  // wave uniform
    // Slabs that run side by side would otherwise all sweep the same k range in step, which (with a power-of-two row
    // pitch) keeps hitting the same few channels; so the sweep starts at a block that depends on the XCD the
    // workgroup runs on (workgroups are dealt to the 8 XCDs in turn).  The slabs of one XCD keep the same order: they
    // share its L2, and slabs of one segment then find the adapter's A there instead of fetching it again.
    const int rot = (int)((((unsigned)blockIdx.x & 7u) * (unsigned)nblk) >> 3);
    auto k_of = [&](int j) {  // first k of this wave's j-th block (past the end: the last one again)
        int b = w + kWaves * min(j, n_mine - 1) + rot;
        if (b >= nblk) b -= nblk;
        return b * kKB;
    };

    const int safe_row = max(lds_row[0], 0);
    const u16* xrow[NJ];
#pragma unroll
    for (int i = 0; i < NJ; ++i) {
        const int r = lds_row[r8 + 8 * i];
        xrow[i] = p.x + (long long)(r >= 0 ? r : safe_row) * p.ldx + piece * 8;
    }
    unsigned int aoff[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) aoff[i] = (unsigned int)(min(r8 + 8 * i, rank - 1) * p.d_in);

    // a lane's 8 columns lie wholly inside or wholly beyond d_in; beyond, it re-reads column 0 (and A counts as zero)
    auto col_of = [&](int k0) { return k0 + piece * 8 < p.d_in ? k0 : -piece * 8; };
    constexpr int XS = NP >= 3 ? 1 : 2;  // register sets of x = blocks it is requested ahead (one where registers are short)
    u32x4 xv[XS][NJ];
    auto x_load = [&](int j, u32x4 (&v)[NJ]) {
        const int kc = col_of(k_of(j));
#pragma unroll
        for (int i = 0; i < NJ; ++i) v[i] = *reinterpret_cast<const u32x4*>(xrow[i] + kc);
    };
    // The A stream: a block's A is NC chunks (projection q, 32 ranks ch), four load instructions each; chunk n of
    // block j is number j NC + n of the stream, lives in register set (j NC + n) % 2 and goes through LDS buffer
    // (j NC + n) % 2.  A set is refilled with the chunk two further on as soon as it has been written to LDS.
    constexpr int NC = NP * NCH;
    constexpr int NL = NA < 4 ? NA : 4;  // load instructions per chunk
    u32x4 av[2][NL];
    auto a_load = [&](int j, auto chunk, u32x4 (&v)[NL]) {
        constexpr int N = decltype(chunk)::value;  // chunk N of block j (N may run past NC: the blocks further on)
        constexpr int q = (N % NC) / NCH, ch = (N % NC) % NCH;
        const unsigned int kc = (unsigned int)(col_of(k_of(j + N / NC)) + piece * 8);  // >= 0
#pragma unroll
        for (int i2 = 0; i2 < NL; ++i2) v[i2] = load_at(s[q].A, aoff[ch * 4 + i2] + kc);
    };
    // (loads return in order, so they are issued in the order they are consumed, and the scheduler is kept from
    // reordering them: a wait for the oldest then leaves all younger ones in flight)
    x_load(0, xv[0]);
    __builtin_amdgcn_sched_barrier(0);
    a_load(0, std::integral_constant<int, 0>{}, av[0]);
    __builtin_amdgcn_sched_barrier(0);
    a_load(0, std::integral_constant<int, 1>{}, av[1]);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (XS == 2) x_load(1, xv[1]);
    __builtin_amdgcn_sched_barrier(0);

    // (live: false for the block that pads an odd count to the pair the loop below runs; it adds zeros)
    auto block = [&](int j, auto slot, bool live_block) {
        constexpr int J = decltype(slot)::value;
        // x of block j: registers -> slab -> fragments; the registers take block j + XS
#pragma unroll
        for (int i = 0; i < NJ; ++i) *reinterpret_cast<u32x4*>(xs + (r8 + 8 * i) * kPitch + piece * 8) = xv[J % XS][i];
        x_load(j + XS, xv[J % XS]);
        __builtin_amdgcn_sched_barrier(0);
        wave_sync();
        u32x4 xf[MT][2];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int h = 0; h < 2; ++h) xf[mt][h] = *reinterpret_cast<const u32x4*>(xs + (mt * 16 + c) * kPitch + 32 * h + kg * 8);
        const bool in_cur = live_block && k_of(j) + piece * 8 < p.d_in;
        auto chunk = [&](auto index) {
            constexpr int N = decltype(index)::value;
            constexpr int q = N / NCH, ch = N % NCH, S = (J * NC + N) & 1;
            u16* buf = as + S * kChunk;
#pragma unroll
            for (int i2 = 0; i2 < NL; ++i2) {
                constexpr u32x4 zero = {0u, 0u, 0u, 0u};
                const bool live = in_cur && r8 + 8 * (ch * 4 + i2) < rank;
                *reinterpret_cast<u32x4*>(buf + (r8 + 8 * i2) * kPitch + piece * 8) = live ? av[S][i2] : zero;
            }
            a_load(j, std::integral_constant<int, N + 2>{}, av[S]);
            __builtin_amdgcn_sched_barrier(0);
            wave_sync();
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                constexpr int dummy = 0;
                const int nt = ch * 2 + t < NT ? ch * 2 + t : dummy;  // (keeps the dead branch's index inside the array)
                if (ch * 2 + t < NT) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const u32x4 af = *reinterpret_cast<const u32x4*>(buf + (t * 16 + c) * kPitch + 32 * h + kg * 8);
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
                            acc[q][mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(xf[mt][h]), as_bf16x8(af),
                                                                                     acc[q][mt][nt], 0, 0, 0);
                    }
                }
            }
        };
        // (a buffer is rewritten two chunks later, behind the wave_sync of the chunk in between; with a single
        // chunk per block, behind the one at the end of the block)
        chunk(std::integral_constant<int, 0>{});
        if constexpr (NC > 1) chunk(std::integral_constant<int, 1>{});
        if constexpr (NC > 2) chunk(std::integral_constant<int, 2>{});
        if constexpr (NC > 3) chunk(std::integral_constant<int, 3>{});
        static_assert(NC <= 4, "the chunks of a block are listed by name");
        wave_sync();  // the x slab is rewritten by the next block
    };
    // (pairs of blocks with a single exit: the accumulators stay where they are across the loop)
    for (int j = 0; j < n_mine; j += 2) {
        block(j, std::integral_constant<int, 0>{}, true);
        block(j + 1, std::integral_constant<int, 1>{}, j + 1 < n_mine);
    }
}

// =================================================================================================
// phase 2 for one projection: y[rows][columns of the part] += (scaled h, as bf16 high + low fragments) . B
// D[column][row] with the columns of two MFMA tiles interleaved, so that a lane ends up with 4 consecutive
// columns of a row; every 16-row tile of products makes a round trip through the wave's 4 KB slab to reach the
// row-wise layout y is accessed in.
// =================================================================================================
template <int NT, int MT, class PP>
__device__ __forceinline__ void slab_expand(const PP&, const Unit& u, const SegInfo& s, const Proj& pj,
                                            const int* lds_row, const u32x4* hf, u16* bs, float* ds, int blk_begin,
                                            int blk_end)
{
    constexpr int NJ = 2 * MT;
    constexpr int NB = 2 * NT;
    constexpr int KSTEPS = (NT + 1) / 2;
    const int lane = lane_id(), w = uniform((int)threadIdx.x / kWave), c = lane & 15, g = lane >> 4;
    const int r8 = lane >> 3, piece = lane & 7;
    const int nblk = blk_end - blk_begin;
    const int n_mine = w < nblk ? (nblk - w + kWaves - 1) / kWaves : 0;
    if (n_mine == 0) return;  // wave uniform
    const int rot = (int)((((unsigned)blockIdx.x & 7u) * (unsigned)nblk) >> 3);  // as in phase 1: one order per XCD
    auto n_of = [&](int j) {  // first column of this wave's j-th block (past the end: the last one again)
        int b = w + kWaves * min(j, n_mine - 1) + rot;
        if (b >= nblk) b -= nblk;
        return (blk_begin + b) * kKB;
    };
    const int safe_row = max(lds_row[0], 0);
    int row[NJ];
    u16* yrow[NJ];
#pragma unroll
    for (int i = 0; i < NJ; ++i) {
        row[i] = lds_row[r8 + 8 * i];
        yrow[i] = pj.y + (long long)(row[i] >= 0 ? row[i] : safe_row) * pj.ldy;
    }
    unsigned int boff[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) boff[i] = (unsigned int)(min(r8 + 8 * i, s.rank - 1) * pj.d_out);

    // The B stream: a block's B is KSTEPS chunks of 32 rank rows, four load instructions each; chunk ks of block j is
    // number j KSTEPS + ks of the stream and lives in register set (j KSTEPS + ks) % 2; a set is refilled with the
    // chunk two further on as soon as it has been written to LDS.
    constexpr int NL = NB < 4 ? NB : 4;  // load instructions per chunk
    u32x4 yv[2][NJ], bv[2][NL];
    auto y_load = [&](int j, u32x4 (&v)[NJ]) {
        const int n_ld = min(n_of(j) + 8 * piece, pj.d_out - 8);
#pragma unroll
        for (int i = 0; i < NJ; ++i) v[i] = *reinterpret_cast<const u32x4*>(yrow[i] + n_ld);
    };
    auto b_load = [&](int j, auto chunk, u32x4 (&v)[NL]) {
        constexpr int N = decltype(chunk)::value;
        const unsigned int n_ld = (unsigned int)min(n_of(j + N / KSTEPS) + 8 * piece, pj.d_out - 8);
#pragma unroll
        for (int i2 = 0; i2 < NL; ++i2) v[i2] = load_at(s.B, boff[(N % KSTEPS) * 4 + i2] + n_ld);
    };
    // (issued in the order they are consumed, see phase 1; with KSTEPS > 1 both chunks belong to block 0)
    b_load(0, std::integral_constant<int, 0>{}, bv[0]);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (KSTEPS == 1) {
        y_load(0, yv[0]);
        __builtin_amdgcn_sched_barrier(0);
        b_load(0, std::integral_constant<int, 1>{}, bv[1]);
    } else {
        b_load(0, std::integral_constant<int, 1>{}, bv[1]);
        __builtin_amdgcn_sched_barrier(0);
        y_load(0, yv[0]);
    }
    __builtin_amdgcn_sched_barrier(0);
    y_load(1, yv[1]);
    __builtin_amdgcn_sched_barrier(0);

    // (live: false for the block that pads an odd count to the pair the loop below runs; it stores nothing)
    auto block = [&](int j, auto slot, bool live_block) {
        constexpr int J = decltype(slot)::value;
        const int n_c = n_of(j) + 8 * piece;
        // B of block j, 32 ranks at a time: registers -> slab -> transposed fragments
        u32x4 bfrag[2][2][KSTEPS];
        auto chunk = [&](auto index) {
            constexpr int ks = decltype(index)::value, S = (J * KSTEPS + ks) & 1;
#pragma unroll
            for (int i2 = 0; i2 < 4; ++i2) {
                constexpr u32x4 zero = {0u, 0u, 0u, 0u};
                u32x4 v = zero;  // rank rows beyond the adapter's (and beyond the tiles of this launch) are zero
                if (i2 < NL && r8 + 8 * (ks * 4 + i2) < s.rank) v = bv[S][i2 < NL ? i2 : 0];
                *reinterpret_cast<u32x4*>(bs + (r8 + 8 * i2) * kPitch + piece * 8) = v;
            }
            b_load(j, std::integral_constant<int, ks + 2>{}, bv[S]);
            __builtin_amdgcn_sched_barrier(0);
            wave_sync();
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int m = 0; m < 2; ++m)
                    // lane c: column 32 q + 8 (c / 4) + 4 m + c % 4 of the block, rank rows 32 ks + 8 g .. + 7
                    bfrag[q][m][ks] = lds_read_transposed_16x32(bs + 32 * q + 4 * m, kPitch, 8);
            wave_sync();  // the slab is rewritten by the next chunk
        };
        chunk(std::integral_constant<int, 0>{});
        if constexpr (KSTEPS > 1) chunk(std::integral_constant<int, 1>{});
        if constexpr (KSTEPS > 2) chunk(std::integral_constant<int, 2>{});
        if constexpr (KSTEPS > 3) chunk(std::integral_constant<int, 3>{});
        static_assert(KSTEPS <= 4, "the chunks of a block are listed by name");
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            u32x4 h_hi[KSTEPS], h_lo[KSTEPS];
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                h_hi[ks] = hf[((t * KSTEPS + ks) * 2 + 0) * kWave + lane];
                h_lo[ks] = hf[((t * KSTEPS + ks) * 2 + 1) * kWave + lane];
            }
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    f32x4 d = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KSTEPS; ++ks) {
                        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(bfrag[q][m][ks]), as_bf16x8(h_lo[ks]), d, 0, 0, 0);
                        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(bfrag[q][m][ks]), as_bf16x8(h_hi[ks]), d, 0, 0, 0);
                    }
                    // row c of the tile, columns 32 q + 8 g + 4 m .. + 3 = 16-byte chunk 8 q + 2 g + m (swizzled with the row)
                    *reinterpret_cast<f32x4*>(ds + c * 64 + (((8 * q + 2 * g + m) ^ c) & 15) * 4) = d;
                }
            wave_sync();
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int i = 2 * t + jj, rt = 8 * jj + r8;  // load instruction i of the block = row rt of tile t
                const f32x4 d0 = *reinterpret_cast<const f32x4*>(ds + rt * 64 + (((2 * piece) ^ rt) & 15) * 4);
                const f32x4 d1 = *reinterpret_cast<const f32x4*>(ds + rt * 64 + (((2 * piece + 1) ^ rt) & 15) * 4);
                if (live_block && row[i] >= 0 && t * 16 + rt < u.len && n_c < pj.d_out) {
                    float yf[8];
                    unpack8(yv[J][i], yf);
                    u32x4 o;
                    o.x = pack_bf16x2(yf[0] + d0[0], yf[1] + d0[1]);
                    o.y = pack_bf16x2(yf[2] + d0[2], yf[3] + d0[3]);
                    o.z = pack_bf16x2(yf[4] + d1[0], yf[5] + d1[1]);
                    o.w = pack_bf16x2(yf[6] + d1[2], yf[7] + d1[3]);
                    *reinterpret_cast<u32x4*>(pj.y + (long long)row[i] * pj.ldy + n_c) = o;
                }
            }
            wave_sync();  // the slab is rewritten by the next tile
        }
        __builtin_amdgcn_sched_barrier(0);
        y_load(j + 2, yv[J]);
        __builtin_amdgcn_sched_barrier(0);
    };
    for (int j = 0; j < n_mine; j += 2) {
        block(j, std::integral_constant<int, 0>{}, true);
        block(j + 1, std::integral_constant<int, 1>{}, j + 1 < n_mine);
    }
}


// =================================================================================================
// phase 1 of one pass and the sum over the 8 waves in a fixed order: every wave parks its accumulators in its own
// share of the LDS ([register][lane]); after one barrier the 512 threads share the (register, lane) values, add the
// eight partial sums as a balanced tree and hand every live element to emit(projection q of the pass (as an
// integral constant), row i of the unit, rank j, sum).  work: kWaves x kWaveBytes of LDS.  Ends without a barrier.
// =================================================================================================
template <int NT, int NP, class PP, class Emit>
__device__ __forceinline__ void slab_shrink_sum(const PP& p, const Unit& u0, const SegInfo (&s)[NP], const int* lds_row,
                                                unsigned char* work, Emit&& emit)
{
    constexpr int REGS = NP * 2 * NT * 4;  // accumulator registers of a wave
    static_assert((size_t)REGS * kWave * sizeof(float) <= kWaveBytes, "a wave's accumulators fit its share of the LDS");
    static_assert((size_t)3 * kChunk * sizeof(u16) <= kWaveBytes, "a wave's slabs fit its share of the LDS");
    const int lane = lane_id(), w = uniform((int)threadIdx.x / kWave);
    const int rank = s[0].rank;
    f32x4 acc[NP][2][NT];
#pragma unroll
    for (int q = 0; q < NP; ++q)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[q][mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    u16* slab = reinterpret_cast<u16*>(work + (size_t)w * kWaveBytes);
    if (u0.len <= 16) slab_shrink<NT, NP, 1>(p, u0, s, lds_row, slab, acc);  // workgroup uniform
    else slab_shrink<NT, NP, 2>(p, u0, s, lds_row, slab, acc);
    {
        float* mine = reinterpret_cast<float*>(slab) + lane;
#pragma unroll
        for (int q = 0; q < NP; ++q)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) mine[(((q * 2 + mt) * NT + nt) * 4 + v) * kWave] = acc[q][mt][nt][v];
    }
    __syncthreads();
    // thread (wave w, lane) takes register 8 it + w of lane `lane`: NP * NT iterations, projection it / NT
    auto one = [&](auto index) {
        constexpr int it = decltype(index)::value;
        constexpr int PER_WAVE = (int)(kWaveBytes / sizeof(float));
        constexpr int q = it / NT;
        const int r = 8 * (it % NT) + w;  // register within the projection: (mt * NT + nt) * 4 + v
        const int v = r & 3, nt = (r >> 2) % NT, mt = (r >> 2) / NT;
        const float* at = reinterpret_cast<const float*>(work) + (q * 2 * NT * 4 + r) * kWave + lane;
        float t[kWaves];
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) t[ww] = at[ww * PER_WAVE];
        const float sum = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
        const int i = mt * 16 + (lane >> 4) * 4 + v, j = nt * 16 + (lane & 15);
        if (i < u0.len && j < rank) emit(std::integral_constant<int, q>{}, i, j, sum);
    };
    static_assert(NP * NT <= 8, "the iterations are listed by name");
    one(std::integral_constant<int, 0>{});
    if constexpr (NP * NT > 1) one(std::integral_constant<int, 1>{});
    if constexpr (NP * NT > 2) one(std::integral_constant<int, 2>{});
    if constexpr (NP * NT > 3) one(std::integral_constant<int, 3>{});
    if constexpr (NP * NT > 4) one(std::integral_constant<int, 4>{});
    if constexpr (NP * NT > 5) one(std::integral_constant<int, 5>{});
    if constexpr (NP * NT > 6) one(std::integral_constant<int, 6>{});
    if constexpr (NP * NT > 7) one(std::integral_constant<int, 7>{});
}

// the unit's row indices (rows[0 .. 32): -1 beyond the unit and for an invalid table entry) and, behind them, the
// rows' scales: the adapter's, or the tokens' own (dynamic scaling, Section 3.3).  The caller adds the barrier.
template <class PP>
__device__ __forceinline__ void slab_unit_rows(const PP& p, const Unit& u, const SegInfo& s0, int* rows)
{
    if ((int)threadIdx.x < kSlabRows) {
        const int i = (int)threadIdx.x;
        const int row = i < u.len ? row_of(p, u.pos + i) : -1;
        rows[i] = row;
        reinterpret_cast<float*>(rows + kSlabRows)[i] = p.token_scales ? p.token_scales[max(row, 0)] : s0.scale;
    }
}

// the adapters of the pass's projections; false (workgroup uniform, error bit set) if one of them is unusable
template <int NP, class PP>
__device__ __forceinline__ bool slab_adapters(const PP& p, const Unit& u0, const SegInfo& s0, int pi0, SegInfo (&s)[NP])
{
    bool ok = true;
#pragma unroll
    for (int q = 0; q < NP; ++q) {
        if (pi0 + q == 0) {
            s[q] = s0;
        } else {
            Unit uq = u0;
            uq.pi = pi0 + q;
            s[q] = load_adapter(p, uq);
        }
        ok = ok && s[q].ok;
    }
    return ok;
}

// Rows per unit: the segments are cut into even chunks of at most `per` rows; `per` is the smallest value (16 to 32)
// for which the chunks fit one round of the grid (sum of ceil(len / per) <= live rows / per + segments).  A batch
// that does not fit one round at 32 rows takes several, handed out by tickets.
template <class PP>
__device__ __forceinline__ int slab_rows_per(const PP& p, const Segs<PP>& sg)
{
    int per = kSlabRows;
    if (sg.n_seg <= kCachedBatches * kWave) {
        int live = 0, n_live = 0;
#pragma unroll
        for (int b = 0; b < kCachedBatches; ++b) {
            const int len = sg.c[b].en - sg.c[b].st;
            const bool on = len > 0 && ((p.kinds >> sg.c[b].kd) & 1);
            live += wave_sum(on ? len : 0);
            n_live += wave_sum(on ? 1 : 0);
        }
        const int grid = (int)gridDim.x, slots = grid - n_live;
        if (slots > 0) per = min(kSlabRows, max(16, small_div(live + slots - 1, slots)));
        // (that bound charges every segment a whole extra chunk.  Just above 16 rows it matters: a slab of 17 rows
        // runs two row tiles, the second nearly empty; so 16 is tried by the exact count)
        if (per > 16 && per <= 20) {
            int n = 0;
#pragma unroll
            for (int b = 0; b < kCachedBatches; ++b) {
                const int len = sg.c[b].en - sg.c[b].st;
                const bool on = len > 0 && ((p.kinds >> sg.c[b].kd) & 1);
                n += wave_sum(on ? (len + 15) >> 4 : 0);
            }
            if (n <= grid) per = 16;
        }
    }
    return per;
}

// While a unit runs, the tables and chunk counts that every wave holds in registers (one segment and one adapter per
// lane) wait in LDS: the unit needs the registers, the search for the next unit needs the tables.  All waves hold
// the same values; wave 0 writes them, a workgroup barrier later every wave reads them back.
constexpr int kStashInts = 24;
constexpr size_t kStashBytes = (size_t)kStashInts * kWave * sizeof(int);
template <class PP>
__device__ __forceinline__ void stash_tables(const Segs<PP>& sg, const ClassScan& cc, int* stash_base)
{
    if ((int)threadIdx.x >= kWave) return;
    int* stash = stash_base + lane_id();
#pragma unroll
    for (int b = 0; b < kCachedBatches; ++b) {
        int* at = stash + b * 12 * kWave;
        at[0 * kWave] = sg.c[b].st; at[1 * kWave] = sg.c[b].en; at[2 * kWave] = sg.c[b].ad; at[3 * kWave] = sg.c[b].kd;
        at[4 * kWave] = (int)sg.a[b].a_lo; at[5 * kWave] = (int)sg.a[b].a_hi;
        at[6 * kWave] = (int)sg.a[b].b_lo; at[7 * kWave] = (int)sg.a[b].b_hi;
        at[8 * kWave] = sg.a[b].rank; at[9 * kWave] = __float_as_int(sg.a[b].scale);
        at[10 * kWave] = cc.nch[b]; at[11 * kWave] = cc.incl[b];
    }
}
template <class PP>
__device__ __forceinline__ void unstash_tables(Segs<PP>& sg, ClassScan& cc, const int* stash_base)
{
    const int* stash = stash_base + lane_id();
#pragma unroll
    for (int b = 0; b < kCachedBatches; ++b) {
        const int* at = stash + b * 12 * kWave;
        sg.c[b].st = at[0 * kWave]; sg.c[b].en = at[1 * kWave]; sg.c[b].ad = at[2 * kWave]; sg.c[b].kd = at[3 * kWave];
        sg.a[b].a_lo = (unsigned int)at[4 * kWave]; sg.a[b].a_hi = (unsigned int)at[5 * kWave];
        sg.a[b].b_lo = (unsigned int)at[6 * kWave]; sg.a[b].b_hi = (unsigned int)at[7 * kWave];
        sg.a[b].rank = at[8 * kWave]; sg.a[b].scale = __int_as_float(at[9 * kWave]);
        cc.nch[b] = at[10 * kWave]; cc.incl[b] = at[11 * kWave];
    }
}

}  // namespace
}  // namespace lq
