// Row-slab variant of the segmented multi-adapter LoRA forward (Section 3.3): one launch in which a
// workgroup takes a slab of at most 32 rows of one segment through BOTH products, so that h never leaves the
// compute unit: no partial-h buffer, no device-wide wait, and both phases are spread over the machine the same
// way.  The price is that every slab re-reads its adapter's matrices; they come from the L2 cache (slabs of
// one segment run side by side), which the measured access pattern bears: 256 workgroups that each stream 22
// rows of x and y and re-read 512 KB of A and B run at 4.3 TB/s of algorithmic bytes, against 4.9 TB/s without
// the re-reads.
#include "lq_slab.h"

namespace lq {
namespace {

constexpr int kMaxParts = 8;           // column parts a short batch's units are cut into
constexpr size_t kHfragBytes = 16384;  // [projection of the pass][row tile][k step][high | low][lane] x 16 B
// LDS of the kernel: the h fragments, the waves' shares, the unit's row indices and scales, the stashed tables
constexpr size_t kWorkOffset = kHfragBytes;
constexpr size_t kRowsOffset = kWorkOffset + kWaves * kWaveBytes;
constexpr size_t kStashOffset = kRowsOffset + 2 * kSlabRows * sizeof(int);
constexpr size_t kSlabLdsBytes = kStashOffset + kStashBytes;

// =================================================================================================
// one pass of a unit: NP projections (pi0 ..) through phase 1, the sum over the waves, and phase 2
// =================================================================================================
template <int NT, int NP, class PP>
__device__ __forceinline__ void slab_pass(const PP& p, const Unit& u0, const SegInfo& s0, int pi0, int part, int parts,
                                          unsigned char* lds)
{
    constexpr int KSTEPS = (NT + 1) / 2;
    static_assert((size_t)NP * 2 * KSTEPS * 2 * kWave * 16 <= kHfragBytes, "the pass's h fragments fit");
    u32x4* hfrag = reinterpret_cast<u32x4*>(lds);
    unsigned char* work = lds + kWorkOffset;
    const int* lds_row = reinterpret_cast<const int*>(lds + kRowsOffset);
    const float* lds_scale = reinterpret_cast<const float*>(lds_row + kSlabRows);
    const int w = uniform((int)threadIdx.x / kWave);

    SegInfo s[NP];
    if (!slab_adapters(p, u0, s0, pi0, s)) return;  // workgroup uniform; the error bit is set
    const int rank = s[0].rank;

    // the fragments start as zeros: rows and ranks beyond the live ones stay that way
    {
        constexpr u32x4 zero = {0u, 0u, 0u, 0u};
        static_assert(kHfragBytes == (size_t)2 * kThreads * 16, "two 16-byte stores per thread");
        hfrag[threadIdx.x] = zero;
        hfrag[threadIdx.x + kThreads] = zero;
    }
    // phase 1; every finished h element goes to h_out (fine-tune segments) and, scaled and split into a bf16 high and
    // low part, into the fragments phase 2 reads
    u16* hf16 = reinterpret_cast<u16*>(hfrag);
    const bool save = u0.kd == LQ_SEG_FINETUNE && p.h_offsets && part == 0;
    slab_shrink_sum<NT, NP>(p, u0, s, lds_row, work, [&](auto qc, int i, int j, float sum) {
        constexpr int q = decltype(qc)::value;
        if (save) {
            float* h_out = proj_of(p, pi0 + q).h_out;
            if (h_out) h_out[p.h_offsets[u0.seg] + (long long)(u0.pos - u0.first + i) * rank + j] = sum;
        }
        const float scaled = sum * lds_scale[i];
        const unsigned int hi = pack_bf16x2(scaled, 0.f) & 0xffffu;
        const unsigned int lo = pack_bf16x2(scaled - bf16_lo(hi), 0.f) & 0xffffu;
        // fragment (projection q, row tile i / 16, k step j / 32): lane (j % 32 / 8) * 16 + i % 16 holds ranks 8 (j / 8) .. + 7
        const int slot = ((q * 2 + (i >> 4)) * KSTEPS + (j >> 5)) * 2;
        const int ln = ((j >> 3) & 3) * 16 + (i & 15);
        hf16[((slot + 0) * kWave + ln) * 8 + (j & 7)] = (u16)hi;
        hf16[((slot + 1) * kWave + ln) * 8 + (j & 7)] = (u16)lo;
    });
    __syncthreads();

    u16* bs = reinterpret_cast<u16*>(work + (size_t)w * kWaveBytes);
    float* ds = reinterpret_cast<float*>(bs + kChunk);
    static_assert(kChunk * sizeof(u16) % 16 == 0, "the D slab is 16-byte aligned");
#pragma unroll
    for (int q = 0; q < NP; ++q) {
        const Proj pj = proj_of(p, pi0 + q);
        const int nblk = (pj.d_out + kKB - 1) / kKB;
        const int begin = small_div(part * nblk, parts), end = small_div((part + 1) * nblk, parts);
        const u32x4* hf = hfrag + q * 2 * KSTEPS * 2 * kWave;
        if (u0.len <= 16) slab_expand<NT, 1>(p, u0, s[q], pj, lds_row, hf, bs, ds, begin, end);  // workgroup uniform
        else slab_expand<NT, 2>(p, u0, s[q], pj, lds_row, hf, bs, ds, begin, end);
    }
    __syncthreads();  // before the next pass or unit reuses the LDS
}

template <int NT, bool GROUP, class PP>
__device__ __forceinline__ void slab_unit(const PP& p, const Unit& u, const SegInfo& s0, int part, int parts, unsigned char* lds)
{
    slab_unit_rows(p, u, s0, reinterpret_cast<int*>(lds + kRowsOffset));
    __syncthreads();
    constexpr int NPP = GROUP ? pass_projections<NT>() : 1;
    const int n_proj = n_proj_of(p);
    for (int pi0 = 0; pi0 < n_proj; pi0 += NPP) {
        const int np = min(NPP, n_proj - pi0);  // workgroup uniform
        if (NPP >= 4 && np == 4) slab_pass<NT, (NPP >= 4 ? 4 : 1)>(p, u, s0, pi0, part, parts, lds);
        else if (NPP >= 3 && np == 3) slab_pass<NT, (NPP >= 3 ? 3 : 1)>(p, u, s0, pi0, part, parts, lds);
        else if (NPP >= 2 && np == 2) slab_pass<NT, (NPP >= 2 ? 2 : 1)>(p, u, s0, pi0, part, parts, lds);
        else slab_pass<NT, 1>(p, u, s0, pi0, part, parts, lds);
    }
}

// NT: 16-rank tiles of the launch (ranks up to 16 NT)
template <int NT, bool GROUP>
__global__ __launch_bounds__(kThreads) void slab_kernel(KernelArg<GROUP> p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    __shared__ int s_slot[2];
    auto sg = load_segs(p);
    const int grid = (int)gridDim.x;
    const int per = slab_rows_per(p, sg);
    const LenClass all{1, kSlabBig, p.kinds, true};
    ClassScan cc = scan_class(p, sg, per, all);
    // Workgroups are dealt to the 8 XCDs in turn (workgroup i runs on XCD i % 8), and every XCD has its own L2.  The
    // chunks are numbered segment by segment, so XCD x takes the x-th eighth of them: the slabs of one segment then
    // sit on one XCD (or two) and find their adapter's matrices in its L2, instead of every XCD fetching every adapter.
    // A batch with few chunks is also cut by columns: every part of a chunk repeats phase 1 and takes its share of
    // the column blocks in phase 2; the parts of one chunk get ids r, r + 8, ..., the same XCD again.
    const int n8 = (cc.total + 7) >> 3;  // chunks per XCD
    const int parts = cc.total > 0 && 2 * cc.total <= grid ? min(kMaxParts, small_div(grid, cc.total)) : 1;
    const int n_units = 8 * n8 * parts;
    int* stash = reinterpret_cast<int*>(lds_raw + kStashOffset);
    for_each_unit(p.tickets + 0, n_units, s_slot, [&](int gid, int) {
        int slot = gid, part = 0;
        if (parts > 1) {
            const int blk = small_div(gid, 8 * parts), r = gid - blk * 8 * parts;
            part = r >> 3;
            slot = blk * 8 + (r & 7);
        }
        const int chunk = (slot & 7) * n8 + (slot >> 3);
        if (chunk >= cc.total) return;  // (padding)
        Unit u;
        SegInfo s;
        u.pi = 0;
        if (!find_unit(p, sg, cc, chunk, per, all, u, s)) return;
        stash_tables(sg, cc, stash);
        slab_unit<NT, GROUP>(p, u, s, part, parts, lds_raw);  // (has a workgroup barrier after its first step)
        unstash_tables(sg, cc, stash);
    });
}

template <int NT>
hipError_t launch_slab(const FwdParams& p, hipStream_t st)
{
    static DeviceGrid cache;
    const int grid = cache.get([] {
        return std::min(resident_grid(slab_kernel<NT, false>, kSlabLdsBytes), resident_grid(slab_kernel<NT, true>, kSlabLdsBytes));
    });
    if (p.n_proj == 1)
        return launch_kernel(kKernelSlab, slab_kernel<NT, false>, dim3(grid), dim3(kThreads), kSlabLdsBytes, st,
                             static_cast<const FwdCore&>(p));
    return launch_kernel(kKernelSlab, slab_kernel<NT, true>, dim3(grid), dim3(kThreads), kSlabLdsBytes, st, p);
}

}  // namespace

hipError_t run_slab(const FwdParams& p, hipStream_t st)
{
    const int nt = nt_for(p.max_rank);
    return nt == 1 ? launch_slab<1>(p, st) : nt == 2 ? launch_slab<2>(p, st) : nt == 4 ? launch_slab<4>(p, st) : launch_slab<8>(p, st);
}

}  // namespace lq
