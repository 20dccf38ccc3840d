// Device-side reading of the segment tables, shared by the forward and backward kernels.
//
// The token rows of segment g are perm[seg_starts[g] .. seg_starts[g+1]).  Work is handed out in
// chunks of at most `per` consecutive positions of one segment; chunk ids count through the segments
// of a length class in order.  Every wave resolves chunk ids on its own with one wave scan per 64
// segments (the first 128 are cached in registers; the tables are small and cache resident), so no
// plan buffer or extra launch is needed and the grid can be a fixed number of resident workgroups.
//
// P is a kernel parameter block with the members seg_starts, seg_adapter, seg_kind, n_segments,
// max_segments, n_adapters, max_rank, ranks, scales, perm, n_tokens, err (and, for the adapter lookups,
// proj0.A_ptrs / B_ptrs and proj_of).
#pragma once

#include "lq_common.h"

namespace lq {

struct SegLane { int st, en, ad, kd; };  // table entries of segment (batch * 64 + lane); empty beyond n_seg

// The tables may have been written by the caller: a segment's positions must lie inside [0, n_tokens] and must
// not run backwards.  One that does not is treated as empty and reported (bit 0 of the error word), so that no
// later index derived from it can leave perm, the activations or the partial-h buffer.
template <class P>
__device__ __forceinline__ void guard_seg_range(const P& p, SegLane& c)
{
    if (c.st < 0 || c.en < c.st || c.en > p.n_tokens) {
        atomicOr(p.err, kErrBadSegment);
        c.st = c.en = 0;
    }
}

template <class P>
__device__ __forceinline__ SegLane load_seg_lane(const P& p, int n_seg, int s)
{
    // the tables hold max_segments entries, so the loads can go out before n_seg has arrived
    const int sc = min(s, p.max_segments - 1);
    SegLane c;
    c.st = p.seg_starts[sc];
    c.en = p.seg_starts[sc + 1];
    c.ad = p.seg_adapter[sc];
    c.kd = p.seg_kind[sc];
    if (s >= n_seg) c.st = c.en = c.ad = c.kd = 0;
    guard_seg_range(p, c);
    return c;
}

// the first kCachedBatches * 64 segments, one per lane and batch, held in registers by every wave
constexpr int kCachedBatches = 2;
struct SegCache { SegLane c[kCachedBatches]; };

// (the table entries are requested before the segment count is waited for: one round trip, not two)
template <class P>
__device__ __forceinline__ SegCache load_seg_cache(const P& p, int& n_seg)
{
    SegCache sc;
    const int n_raw = *p.n_segments;
#pragma unroll
    for (int b = 0; b < kCachedBatches; ++b) {
        const int s = min(b * kWave + lane_id(), p.max_segments - 1);  // the tables hold max_segments entries
        sc.c[b].st = p.seg_starts[s];
        sc.c[b].en = p.seg_starts[s + 1];
        sc.c[b].ad = p.seg_adapter[s];
        sc.c[b].kd = p.seg_kind[s];
    }
    n_seg = __builtin_amdgcn_readfirstlane(min(n_raw, p.max_segments));
#pragma unroll
    for (int b = 0; b < kCachedBatches; ++b) {
        if (b * kWave + lane_id() >= n_seg) sc.c[b].st = sc.c[b].en = sc.c[b].ad = sc.c[b].kd = 0;
        guard_seg_range(p, sc.c[b]);
    }
    return sc;
}

template <class P>
__device__ __forceinline__ SegLane seg_batch(const P& p, int n_seg, const SegCache& sc, int s0)
{
    if (s0 == 0) return sc.c[0];
    if (s0 == kWave) return sc.c[1];
    return load_seg_lane(p, n_seg, s0 + lane_id());
}

struct Unit { int seg, pos, len, first, seg_len, ad, kd, pi; };  // chunk [pos, pos + len) of segment seg = [first, first + seg_len); pi: projection of a grouped call (set by the caller of the lookup)

// A class of chunks: those of the segments with lo <= rows < hi whose kind's bit is set in `kinds`.  A
// segment is cut into ceil(rows / per) chunks; with `even` set they all get ceil(rows / chunks) rows
// (so no chunk is less than half full), otherwise `per` rows each with a shorter last one.
struct LenClass { int lo, hi, kinds; bool even = false; };

__device__ __forceinline__ int chunks_in(int len, int kind, int per, LenClass cls)
{
    return (len >= cls.lo && len < cls.hi && len > 0 && ((cls.kinds >> kind) & 1)) ? (len + per - 1) / per : 0;
}
// position (relative to the segment's first row) and rows of the local-th chunk of a segment in a class
__device__ __forceinline__ void chunk_rows(int seg_len, int local, int per, LenClass cls, int& rel, int& rows)
{
    int each = per;
    if (cls.even) {
        const int n = (seg_len + per - 1) / per;
        each = small_div(seg_len + n - 1, n);
    }
    rel = local * each;
    rows = min(each, seg_len - rel);
}

__device__ __forceinline__ int wave_sum(int v) { return lane_value(wave_inclusive_scan(v), kWave - 1); }

// number of chunks of `per` rows over the segments of a class; wave uniform
template <class P>
__device__ __forceinline__ int count_chunks(const P& p, int n_seg, const SegCache& sc, int per, LenClass cls)
{
    int total = 0;
    for (int s0 = 0; s0 < n_seg; s0 += kWave) {
        const SegLane c = seg_batch(p, n_seg, sc, s0);
        total += wave_sum(chunks_in(c.en - c.st, c.kd, per, cls));
    }
    return total;
}

// the id-th chunk (ids count through the segments of the class in order); wave uniform result
template <class P>
__device__ __forceinline__ bool find_chunk(const P& p, int n_seg, const SegCache& sc, int id, int per, LenClass cls,
                                           Unit& u)
{
    int base = 0;
    for (int s0 = 0; s0 < n_seg; s0 += kWave) {
        const SegLane c = seg_batch(p, n_seg, sc, s0);
        const int nch = chunks_in(c.en - c.st, c.kd, per, cls);
        const int incl = wave_inclusive_scan(nch);
        const int total = uniform(__shfl(incl, kWave - 1, kWave));
        if (id < base + total) {
            const unsigned long long m = __ballot(base + incl > id);
            const int l = __ffsll((long long)m) - 1;
            const int local = id - base - uniform(__shfl(incl - nch, l, kWave));
            u.seg = s0 + l;
            u.first = uniform(__shfl(c.st, l, kWave));
            u.pos = u.first + local * per;
            u.seg_len = uniform(__shfl(c.en, l, kWave)) - u.first;
            u.len = min(per, u.first + u.seg_len - u.pos);
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
typedef const __attribute__((address_space(1))) u32x4* gconst_u32x4;

struct SegInfo {
    gconst_u16 A; gconst_u16 B;
    int rank; float scale;
    bool ok;
};

template <class P>
__device__ __forceinline__ SegInfo load_adapter(const P& p, const Unit& u)
{
    SegInfo s;
    s.A = s.B = nullptr;
    s.rank = 0;
    s.scale = 0.f;
    s.ok = u.ad >= 0 && u.ad < p.n_adapters;
    if (s.ok) {
        s.rank = p.ranks[u.ad];
        s.scale = p.scales[u.ad];
        const auto pj = proj_of(p, u.pi);
        s.A = (gconst_u16)(pj.A_ptrs[u.ad]);
        s.B = (gconst_u16)(pj.B_ptrs[u.ad]);
        s.ok = s.rank >= 1 && s.rank <= p.max_rank && s.A && s.B;
    }
    if (!s.ok && threadIdx.x == 0) atomicOr(p.err, kErrBadSegment);
    return s;
}

// ---- unit lookup with the first 128 segments and the first 128 adapters held in registers -----------
// At kernel start every lane loads the table entries of "its" two segments and the rank, scale and
// matrix pointers of "its" two adapters, all in one round trip.  A lookup is then prefix sums with DPP
// moves, a ballot and a few lane reads, and the matrix data can be requested right after it: a cold
// start costs two dependent round trips (tables, then data) instead of three.  Segments and adapters
// beyond the first 128 take the slower on-demand path above.
struct AdLane { unsigned int a_lo, a_hi, b_lo, b_hi; int rank; float scale; };

template <class P>
struct Segs {
    int n_seg;
    SegLane c[kCachedBatches];
    AdLane a[kCachedBatches];
};

template <class P>
__device__ __forceinline__ Segs<P> load_segs(const P& p)
{
    Segs<P> sg;
    const int n_raw = *p.n_segments;
    SegLane raw[kCachedBatches];
#pragma unroll
    for (int b = 0; b < kCachedBatches; ++b) {
        const int sc = min(b * kWave + lane_id(), p.max_segments - 1);  // the tables hold max_segments entries
        raw[b].st = p.seg_starts[sc];
        raw[b].en = p.seg_starts[sc + 1];
        raw[b].ad = p.seg_adapter[sc];
        raw[b].kd = p.seg_kind[sc];
    }
#pragma unroll
    for (int b = 0; b < kCachedBatches; ++b) {
        const int ad = min(b * kWave + lane_id(), p.n_adapters - 1);
        const unsigned long long pa = reinterpret_cast<unsigned long long>(p.proj0.A_ptrs[ad]);
        const unsigned long long pb = reinterpret_cast<unsigned long long>(p.proj0.B_ptrs[ad]);
        sg.a[b].a_lo = (unsigned int)pa; sg.a[b].a_hi = (unsigned int)(pa >> 32);
        sg.a[b].b_lo = (unsigned int)pb; sg.a[b].b_hi = (unsigned int)(pb >> 32);
        sg.a[b].rank = p.ranks[ad];
        sg.a[b].scale = p.scales[ad];
    }
    sg.n_seg = uniform(min(n_raw, p.max_segments));
#pragma unroll
    for (int b = 0; b < kCachedBatches; ++b) {
        sg.c[b] = raw[b];
        if (b * kWave + lane_id() >= sg.n_seg) sg.c[b].st = sg.c[b].en = sg.c[b].ad = sg.c[b].kd = 0;
        guard_seg_range(p, sg.c[b]);
    }
    return sg;
}

// the adapter of a unit: from the registers if it is one of the first 128 (of the call's first projection), else loaded
template <class P>
__device__ __forceinline__ SegInfo cached_adapter(const P& p, const Segs<P>& sg, const Unit& u)
{
    if (u.pi != 0 || u.ad < 0 || u.ad >= kCachedBatches * kWave) return load_adapter(p, u);
    const bool hi = u.ad >= kWave;  // wave uniform
    const int l = u.ad & (kWave - 1);
    const AdLane& a = hi ? sg.a[1] : sg.a[0];
    const unsigned long long pa =
        ((unsigned long long)(unsigned int)lane_value((int)a.a_hi, l) << 32) | (unsigned int)lane_value((int)a.a_lo, l);
    const unsigned long long pb =
        ((unsigned long long)(unsigned int)lane_value((int)a.b_hi, l) << 32) | (unsigned int)lane_value((int)a.b_lo, l);
    SegInfo s;
    s.A = (gconst_u16)reinterpret_cast<const u16*>(pa);
    s.B = (gconst_u16)reinterpret_cast<const u16*>(pb);
    s.rank = lane_value(a.rank, l);
    s.scale = __int_as_float(lane_value(__float_as_int(a.scale), l));
    s.ok = u.ad < p.n_adapters && s.rank >= 1 && s.rank <= p.max_rank && pa != 0 && pb != 0;
    if (!s.ok && threadIdx.x == 0) atomicOr(p.err, kErrBadSegment);
    return s;
}

// chunk counts of one length class: prefix sums over the cached segments, totals over all
struct ClassScan { int nch[kCachedBatches], incl[kCachedBatches]; int tot0, tot_cached, total; };

template <class P>
__device__ __forceinline__ ClassScan scan_class(const P& p, const Segs<P>& sg, int per, LenClass cls)
{
    ClassScan cs;
    cs.nch[0] = chunks_in(sg.c[0].en - sg.c[0].st, sg.c[0].kd, per, cls);
    cs.incl[0] = wave_inclusive_scan(cs.nch[0]);
    cs.tot0 = lane_value(cs.incl[0], kWave - 1);
    static_assert(kCachedBatches == 2, "the second batch is handled by name");
    cs.nch[1] = cs.incl[1] = 0;
    if (sg.n_seg > kWave) {  // wave uniform: most batches have at most 64 segments
        cs.nch[1] = chunks_in(sg.c[1].en - sg.c[1].st, sg.c[1].kd, per, cls);
        cs.incl[1] = wave_inclusive_scan(cs.nch[1]);
    }
    cs.tot_cached = cs.tot0 + lane_value(cs.incl[1], kWave - 1);
    cs.total = cs.tot_cached;
    for (int s0 = kCachedBatches * kWave; s0 < sg.n_seg; s0 += kWave) {
        const SegLane c = load_seg_lane(p, sg.n_seg, s0 + lane_id());
        cs.total += wave_sum(chunks_in(c.en - c.st, c.kd, per, cls));
    }
    return cs;
}

// the id-th chunk of the class and its adapter; false (and the error bit set) if the segment is unusable
template <class P>
__device__ __forceinline__ bool find_unit(const P& p, const Segs<P>& sg, const ClassScan& cs, int id, int per,
                                          LenClass cls, Unit& u, SegInfo& s)
{
    if (id < cs.tot_cached) {
        const bool hi = id >= cs.tot0;  // wave uniform
        const int base = hi ? cs.tot0 : 0;
        const int incl = hi ? cs.incl[1] : cs.incl[0], nch = hi ? cs.nch[1] : cs.nch[0];
        const SegLane& c = hi ? sg.c[1] : sg.c[0];
        const unsigned long long m = __ballot(base + incl > id);
        const int l = uniform(__ffsll((long long)m) - 1);
        const int local = id - base - lane_value(incl - nch, l);
        u.seg = (hi ? kWave : 0) + l;
        u.first = lane_value(c.st, l);
        u.seg_len = lane_value(c.en, l) - u.first;
        int rel;
        chunk_rows(u.seg_len, local, per, cls, rel, u.len);
        u.pos = u.first + rel;
        u.ad = lane_value(c.ad, l);
        u.kd = lane_value(c.kd, l);
        s = cached_adapter(p, sg, u);
        return s.ok;
    }
    // beyond the cached segments: walk the tables
    int base = cs.tot_cached;
    for (int s0 = kCachedBatches * kWave; s0 < sg.n_seg; s0 += kWave) {
        const SegLane c = load_seg_lane(p, sg.n_seg, s0 + lane_id());
        const int nch = chunks_in(c.en - c.st, c.kd, per, cls);
        const int incl = wave_inclusive_scan(nch);
        const int total = lane_value(incl, kWave - 1);
        if (id < base + total) {
            const unsigned long long m = __ballot(base + incl > id);
            const int l = uniform(__ffsll((long long)m) - 1);
            const int local = id - base - lane_value(incl - nch, l);
            u.seg = s0 + l;
            u.first = lane_value(c.st, l);
            u.seg_len = lane_value(c.en, l) - u.first;
            int rel;
            chunk_rows(u.seg_len, local, per, cls, rel, u.len);
            u.pos = u.first + rel;
            u.ad = lane_value(c.ad, l);
            u.kd = lane_value(c.kd, l);
            s = load_adapter(p, u);
            return s.ok;
        }
        base += total;
    }
    return false;
}

// row of the activations for a position of the segment order; -1 if the table holds an invalid row
template <class P>
__device__ __forceinline__ int row_of(const P& p, int pos)
{
    // branch free: with perm == NULL a dummy entry is loaded and ignored
    const int32_t* tab = p.perm ? p.perm : p.seg_starts;
    const int v = tab[p.perm ? pos : 0];
    const int row = p.perm ? v : pos;
    return (row >= 0 && row < p.n_tokens) ? row : -1;
}

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& v) { return __builtin_bit_cast(bf16x8, v); }

}  // namespace lq
