// Segment-metadata builder: per-token (adapter, kind) -> perm / seg_starts / seg_adapter / seg_kind /
// h_offsets / n_segments.  One workgroup of 16 waves performs a stable counting sort on the key
// kind * n_adapters + adapter (the batch order fine-tune | prefill+evaluation | decode of
// Algorithm 1, refined by adapter) and run-length encodes the non-empty keys.  Integer only; the
// result is unique, so it is compared bit for bit with the CPU oracle.
#include "lq_internal.h"

namespace lq {
namespace {

constexpr int kBuildThreads = 1024;
constexpr int kBuildWaves = kBuildThreads / kWave;
constexpr int kKeyRounds = 8;   // 64-token rounds whose keys a wave holds in registers
constexpr int kBuildLdsBudget = 60000;  // bytes of dynamic LDS used for the histograms when they fit

template <int WAVES = kBuildWaves>
__device__ __forceinline__ int block_exclusive_scan(int v, int* s_tot, int& total)
{
    const int lane = lane_id(), w = (int)threadIdx.x / kWave;
    const int incl = wave_inclusive_scan(v);
    __syncthreads();  // s_tot may still be read from a previous scan
    if (lane == kWave - 1) s_tot[w] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
        const int t = s_tot[i];
        if (i < w) before += t;
        all += t;
    }
    total = all;
    return before + incl - v;
}

// two exclusive scans (an int and a 64-bit count) that share their barriers
template <int WAVES = kBuildWaves>
__device__ __forceinline__ void block_exclusive_scan_pair(int v, long long h, int* s_tot, long long* s_tot64, int& ex_v,
                                                          long long& ex_h, int& total_v, long long& total_h)
{
    const int lane = lane_id(), w = (int)threadIdx.x / kWave;
    const int incl_v = wave_inclusive_scan(v);
    const long long incl_h = wave_inclusive_scan64(h);
    __syncthreads();
    if (lane == kWave - 1) {
        s_tot[w] = incl_v;
        s_tot64[w] = incl_h;
    }
    __syncthreads();
    int before_v = 0, all_v = 0;
    long long before_h = 0, all_h = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
        const int t = s_tot[i];
        const long long t64 = s_tot64[i];
        if (i < w) { before_v += t; before_h += t64; }
        all_v += t;
        all_h += t64;
    }
    total_v = all_v;
    total_h = all_h;
    ex_v = before_v + incl_v - v;
    ex_h = before_h + incl_h - h;
}

__device__ __forceinline__ int token_key(const int32_t* __restrict__ token_adapter,
                                         const uint8_t* __restrict__ token_kind, int t, int n_adapters)
{
    const int a = token_adapter[t];
    const int k = token_kind[t];
    return (a >= 0 && a < n_adapters && k <= LQ_SEG_DECODE) ? k * n_adapters + a : -1;
}

// Lanes of a 64-token round that hold the same key.  A batch whose tokens arrive grouped has one or two
// keys per round, found with one ballot each: up to four such passes set `peers` (the lanes with this
// lane's key) for the lanes they cover and return the lanes still to do.
__device__ __forceinline__ unsigned long long leader_passes(int key, unsigned long long& peers)
{
    const bool valid = key >= 0;
    unsigned long long todo = __ballot(valid);
    peers = 0;
    for (int pass = 0; pass < 4 && todo; ++pass) {
        const int k = lane_value(key, __ffsll((long long)todo) - 1);
        const unsigned long long same = __ballot(valid && key == k);
        if (valid && key == k) peers = same;
        todo &= ~same;
    }
    return todo;
}
// The same for every lane, packed as leader | rank among the peers << 8 | their number << 16 (0 for a lane
// without a key); rounds with more than four keys finish by voting on the key's bits one at a time.
__device__ __forceinline__ int key_group(int key, int key_bits)
{
    const int lane = lane_id();
    unsigned long long peers;
    const unsigned long long todo = leader_passes(key, peers);
    if (todo) {
        const bool mine = (todo >> lane) & 1;
        unsigned long long left = todo;
        for (int b = 0; b < key_bits; ++b) {
            const bool bit = mine && ((key >> b) & 1);
            const unsigned long long vote = __ballot(bit);
            left &= bit ? vote : ~vote;
        }
        if (mine) peers = left;
    }
    if (key < 0) return 0;
    return (__ffsll((long long)peers) - 1) | (__popcll(peers & ((1ull << lane) - 1ull)) << 8) | (__popcll(peers) << 16);
}

// WAVES: 16, or 4 for a batch of up to 256 tokens (a small workgroup starts sooner and its barriers are cheaper)
template <bool LDS_HIST, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void build_segments_kernel(
    const int32_t* __restrict__ token_adapter, const uint8_t* __restrict__ token_kind, int n_tokens,
    const int32_t* __restrict__ ranks, int n_adapters,
    int32_t* __restrict__ perm, int32_t* __restrict__ seg_starts, int32_t* __restrict__ seg_adapter,
    uint8_t* __restrict__ seg_kind, int64_t* __restrict__ h_offsets, int32_t* __restrict__ n_segments,
    int32_t* ws_hist)
{
    extern __shared__ int32_t lds_hist[];
    __shared__ int s_tot[WAVES];
    __shared__ long long s_tot64[WAVES];

    const int tid = (int)threadIdx.x, lane = lane_id(), w = tid / kWave;
    const int n_keys = 3 * n_adapters;
    const int n_entries = n_keys * WAVES;
    // hist[key * 16 + wave]: tokens with that key in that wave's token range; scanned in place into
    // the position in perm where that wave's first such token goes.
    // (a compile-time choice, so that the common case gets LDS atomics instead of flat ones)
    auto hist_at = [&](int i) -> int32_t* {
        if constexpr (LDS_HIST) return lds_hist + i;
        else return ws_hist + i;
    };

    // each wave owns a contiguous token range (a multiple of 64 long), walked 64 tokens at a time
    int per_wave = (n_tokens + WAVES - 1) / WAVES;
    per_wave = (per_wave + kWave - 1) / kWave * kWave;
    const int t_begin = min(n_tokens, w * per_wave);
    const int t_end = min(n_tokens, t_begin + per_wave);

    // What the later phases need from memory is requested first, so that these round trips overlap the
    // clearing of the histograms: the keys of the wave's first kKeyRounds x 64 tokens (all of them in a
    // batch of up to 8192 tokens, and then they stay in registers for the scatter) and the rank of the
    // first key this thread turns into a segment.
    int keys[kKeyRounds];
    auto load_keys = [&](int base0) {  // all loads go out before the first one is used
#pragma unroll
        for (int r = 0; r < kKeyRounds; ++r) {
            const int t = base0 + r * kWave + lane;
            keys[r] = t < t_end ? token_key(token_adapter, token_kind, t, n_adapters) : -1;
        }
    };
    const bool keys_fit = per_wave <= kKeyRounds * kWave;  // workgroup uniform
    load_keys(t_begin);
    const int keys_per_thread = (n_keys + (WAVES * kWave) - 1) / (WAVES * kWave);
    const int k_begin = min(n_keys, tid * keys_per_thread);
    const int k_end = min(n_keys, k_begin + keys_per_thread);
    const int rank_first = k_begin < n_adapters ? ranks[k_begin] : 0;
    auto rank_of_key = [&](int k) { return k == k_begin ? rank_first : ranks[k]; };  // k < n_adapters

    for (int i = tid; i < n_entries; i += (WAVES * kWave)) *hist_at(i) = 0;
    __syncthreads();

    int key_bits = 0;
    while ((1 << key_bits) < n_keys) ++key_bits;
    // 64 additions to one LDS word are slow, so in a batch with several rounds per wave the first lane of
    // every group of equal keys adds for its group (and the grouping is kept for the scatter while the
    // keys stay in registers).  A small batch (one round per wave) has few tokens per key: it adds lane by
    // lane and leaves the grouping to the scatter.
    const bool group_early = per_wave > kWave;  // workgroup uniform
    int groups[kKeyRounds];
    for (int base0 = t_begin; base0 < t_end; base0 += kKeyRounds * kWave) {
        if (base0 != t_begin) load_keys(base0);
#pragma unroll
        for (int r = 0; r < kKeyRounds; ++r) {
            if (group_early) {
                groups[r] = key_group(keys[r], key_bits);
                if (keys[r] >= 0 && (groups[r] & 0xff) == lane) atomicAdd(hist_at(keys[r] * WAVES + w), groups[r] >> 16);
            } else if (keys[r] >= 0) {
                atomicAdd(hist_at(keys[r] * WAVES + w), 1);
            }
        }
    }
    __syncthreads();

    // exclusive scan over (key major, wave minor)
    const int per_thread = (n_entries + (WAVES * kWave) - 1) / (WAVES * kWave);
    const int e_begin = min(n_entries, tid * per_thread);
    const int e_end = min(n_entries, e_begin + per_thread);
    int local = 0;
    for (int i = e_begin; i < e_end; ++i) local += *hist_at(i);
    int n_live = 0;
    int run = block_exclusive_scan<WAVES>(local, s_tot, n_live);
    for (int i = e_begin; i < e_end; ++i) {
        const int c = *hist_at(i);
        *hist_at(i) = run;
        run += c;
    }
    __syncthreads();

    // segments = non-empty keys, in key order
    int my_segs = 0;
    long long my_h = 0;
    for (int k = k_begin; k < k_end; ++k) {
        const int start = *hist_at(k * WAVES);
        const int next = (k + 1 < n_keys) ? *hist_at((k + 1) * WAVES) : n_live;
        const int cnt = next - start;
        if (cnt > 0) {
            ++my_segs;
            if (k < n_adapters) my_h += (long long)cnt * rank_of_key(k);  // kind 0 = fine-tune keeps h
        }
    }
    int total_segs = 0, seg = 0;
    long long total_h = 0, h_run = 0;
    block_exclusive_scan_pair<WAVES>(my_segs, my_h, s_tot, s_tot64, seg, h_run, total_segs, total_h);
    for (int k = k_begin; k < k_end; ++k) {
        const int start = *hist_at(k * WAVES);
        const int next = (k + 1 < n_keys) ? *hist_at((k + 1) * WAVES) : n_live;
        const int cnt = next - start;
        if (cnt > 0) {
            const int kind = k / n_adapters, a = k - kind * n_adapters;
            seg_starts[seg] = start;
            seg_adapter[seg] = a;
            seg_kind[seg] = (uint8_t)kind;
            h_offsets[seg] = h_run;
            if (kind == LQ_SEG_FINETUNE) h_run += (long long)cnt * rank_of_key(k);
            ++seg;
        }
    }
    if (tid == 0) {
        seg_starts[total_segs] = n_live;
        h_offsets[total_segs] = total_h;
        *n_segments = total_segs;
    }
    __syncthreads();  // all reads of the scanned offsets are done before the scatter advances them

    // Stable scatter: the first lane of every group of equal keys draws the slots of the whole group, the
    // others add their rank in the group.
    for (int base0 = t_begin; base0 < t_end; base0 += kKeyRounds * kWave) {
        if (!keys_fit) load_keys(base0);
#pragma unroll
        for (int r = 0; r < kKeyRounds; ++r) {
            const int t = base0 + r * kWave + lane;
            const int key = keys[r];
            if (__ballot(key >= 0) == 0) continue;  // wave uniform: nothing in this round
            const int grp = group_early && keys_fit ? groups[r] : key_group(key, key_bits);
            const int leader = key >= 0 ? (grp & 0xff) : lane;
            int slot = 0;
            if (key >= 0 && lane == leader) slot = atomicAdd(hist_at(key * WAVES + w), grp >> 16);
            slot = __shfl(slot, leader, kWave);
            if (key >= 0) perm[slot + ((grp >> 8) & 0xff)] = t;
        }
    }
}

// =================================================================================================
// The same with several workgroups, for batches of thousands of tokens (one workgroup is bound by the
// instruction rate of its compute unit: about 1.6 us per 1024 tokens).  Every workgroup counts and later
// scatters its own slice of the tokens; in between the per-key counts of all workgroups meet in the
// workspace ([key][workgroup], device-scope stores and loads) behind one device-wide barrier, and every
// workgroup works out for itself where its tokens of every key go.  Workgroup 0 writes the segment
// tables.  Needs at most 1024 keys' histograms in LDS (one key per thread), else the kernel above is used.
// =================================================================================================
constexpr int kMultiMinTokens = 2048;  // below this one workgroup is as fast
constexpr int kMultiMaxGroups = 16;

__global__ __launch_bounds__(kBuildThreads) void build_segments_multi_kernel(
    const int32_t* __restrict__ token_adapter, const uint8_t* __restrict__ token_kind, int n_tokens,
    const int32_t* __restrict__ ranks, int n_adapters,
    int32_t* __restrict__ perm, int32_t* __restrict__ seg_starts, int32_t* __restrict__ seg_adapter,
    uint8_t* __restrict__ seg_kind, int64_t* __restrict__ h_offsets, int32_t* __restrict__ n_segments,
    int32_t* header, int32_t* counts)
{
    extern __shared__ int32_t lds_hist[];  // [key][16 waves]
    __shared__ int s_tot[kBuildWaves];
    __shared__ long long s_tot64[kBuildWaves];

    const int tid = (int)threadIdx.x, lane = lane_id(), w = tid / kWave;
    const int g = (int)blockIdx.x, n_groups = (int)gridDim.x;
    const int n_keys = 3 * n_adapters;  // <= 1024: thread k owns key k

    // every wave of the grid owns a contiguous token range (a multiple of 64 long)
    int per_wave = (n_tokens + n_groups * kBuildWaves - 1) / (n_groups * kBuildWaves);
    per_wave = (per_wave + kWave - 1) / kWave * kWave;
    const int t_begin = (int)min((long long)n_tokens, (long long)(g * kBuildWaves + w) * per_wave);
    const int t_end = min(n_tokens, t_begin + per_wave);

    int keys[kKeyRounds];
    auto load_keys = [&](int base0) {
#pragma unroll
        for (int r = 0; r < kKeyRounds; ++r) {
            const int t = base0 + r * kWave + lane;
            keys[r] = t < t_end ? token_key(token_adapter, token_kind, t, n_adapters) : -1;
        }
    };
    const bool keys_fit = per_wave <= kKeyRounds * kWave;  // grid uniform
    load_keys(t_begin);
    const int my_rank = tid < n_adapters ? ranks[tid] : 0;
    const int gen0 = __hip_atomic_load(header + kBarGen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // before arriving

    for (int i = tid; i < n_keys * kBuildWaves; i += kBuildThreads) lds_hist[i] = 0;
    __syncthreads();

    int key_bits = 0;
    while ((1 << key_bits) < n_keys) ++key_bits;
    int groups[kKeyRounds];
    for (int base0 = t_begin; base0 < t_end; base0 += kKeyRounds * kWave) {
        if (base0 != t_begin) load_keys(base0);
#pragma unroll
        for (int r = 0; r < kKeyRounds; ++r) {
            groups[r] = key_group(keys[r], key_bits);
            if (keys[r] >= 0 && (groups[r] & 0xff) == lane) atomicAdd(lds_hist + keys[r] * kBuildWaves + w, groups[r] >> 16);
        }
    }
    __syncthreads();

    // this workgroup's count of every key goes to the workspace; then all workgroups meet
    if (tid < n_keys) {
        int mine = 0;
#pragma unroll
        for (int i = 0; i < kBuildWaves; ++i) mine += lds_hist[tid * kBuildWaves + i];
        __hip_atomic_store(counts + tid * n_groups + g, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!grid_barrier(header, header, gen0, [] {})) {
        // the counts never met (bit 1 of the error word is set): an empty batch is the only safe answer
        if (g == 0 && tid == 0) {
            seg_starts[0] = 0;
            h_offsets[0] = 0;
            *n_segments = 0;
        }
        return;
    }

    // key k: tokens in all workgroups, and in the workgroups before this one
    int total = 0, before = 0;
    if (tid < n_keys) {
        for (int i = 0; i < n_groups; ++i) {
            const int c = __hip_atomic_load(counts + tid * n_groups + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            total += c;
            if (i < g) before += c;
        }
    }
    int n_live = 0;
    const int key_start = block_exclusive_scan(total, s_tot, n_live);  // position in perm of the key's first token
    if (tid < n_keys) {  // where each of this workgroup's waves puts its first token of the key
        int run = key_start + before;
#pragma unroll
        for (int i = 0; i < kBuildWaves; ++i) {
            const int c = lds_hist[tid * kBuildWaves + i];
            lds_hist[tid * kBuildWaves + i] = run;
            run += c;
        }
    }

    // segments = non-empty keys, in key order (every workgroup runs the scans, workgroup 0 writes)
    const bool seg_here = tid < n_keys && total > 0;
    const long long my_h = seg_here && tid < n_adapters ? (long long)total * my_rank : 0;  // kind 0 = fine-tune keeps h
    int total_segs = 0, seg = 0;
    long long total_h = 0, h_run = 0;
    block_exclusive_scan_pair(seg_here ? 1 : 0, my_h, s_tot, s_tot64, seg, h_run, total_segs, total_h);
    if (g == 0) {
        if (seg_here) {
            const int kind = tid / n_adapters, a = tid - kind * n_adapters;
            seg_starts[seg] = key_start;
            seg_adapter[seg] = a;
            seg_kind[seg] = (uint8_t)kind;
            h_offsets[seg] = h_run;
        }
        if (tid == 0) {
            seg_starts[total_segs] = n_live;
            h_offsets[total_segs] = total_h;
            *n_segments = total_segs;
        }
    }
    __syncthreads();  // the offsets are in LDS before the scatter advances them

    for (int base0 = t_begin; base0 < t_end; base0 += kKeyRounds * kWave) {
        if (!keys_fit) load_keys(base0);
#pragma unroll
        for (int r = 0; r < kKeyRounds; ++r) {
            const int t = base0 + r * kWave + lane;
            const int key = keys[r];
            if (__ballot(key >= 0) == 0) continue;  // wave uniform: nothing in this round
            const int grp = keys_fit ? groups[r] : key_group(key, key_bits);
            const int leader = key >= 0 ? (grp & 0xff) : lane;
            int slot = 0;
            if (key >= 0 && lane == leader) slot = atomicAdd(lds_hist + key * kBuildWaves + w, grp >> 16);
            slot = __shfl(slot, leader, kWave);
            if (key >= 0) perm[slot + ((grp >> 8) & 0xff)] = t;
        }
    }
}

}  // namespace
}  // namespace lq

extern "C" size_t lora_build_workspace_bytes(int32_t n_tokens, int32_t n_adapters)
{
    (void)n_tokens;
    if (n_adapters < 0) n_adapters = 0;
    return (size_t)lq::kWsHeaderBytes + (size_t)3 * (size_t)n_adapters * lq::kBuildWaves * sizeof(int32_t);
}

extern "C" lq_status lora_build_segments(const int32_t* token_adapter, const uint8_t* token_kind, int32_t n_tokens,
                                         const int32_t* ranks, int32_t n_adapters,
                                         int32_t* perm, int32_t* seg_starts, int32_t* seg_adapter, uint8_t* seg_kind,
                                         int64_t* h_offsets, int32_t* n_segments, int32_t max_segments,
                                         void* workspace, size_t workspace_bytes, void* stream)
{
    if (n_tokens < 0 || n_adapters <= 0 || max_segments < 0) return LQ_ERR_INVALID_ARG;
    if (!ranks || !seg_starts || !seg_adapter || !seg_kind || !h_offsets || !n_segments) return LQ_ERR_INVALID_ARG;
    if (n_tokens > 0 && (!token_adapter || !token_kind || !perm)) return LQ_ERR_INVALID_ARG;
    if (n_adapters > LQ_MAX_ADAPTERS) return LQ_ERR_UNSUPPORTED;
    const int64_t n_keys = 3 * (int64_t)n_adapters;
    const int64_t need_segments = n_tokens < n_keys ? n_tokens : n_keys;
    if (max_segments < need_segments) return LQ_ERR_INVALID_ARG;
    const size_t hist_bytes = (size_t)n_keys * lq::kBuildWaves * sizeof(int32_t);
    const int use_lds = hist_bytes <= (size_t)lq::kBuildLdsBudget;
    int32_t* ws_hist = nullptr;
    if (!use_lds) {
        if (!workspace || workspace_bytes < lora_build_workspace_bytes(n_tokens, n_adapters)) return LQ_ERR_WORKSPACE;
        ws_hist = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + lq::kWsHeaderBytes);
    }
    const hipStream_t st = static_cast<hipStream_t>(stream);
    // thousands of tokens: several workgroups, if the workspace is there for their counts and barrier
    if (n_tokens >= lq::kMultiMinTokens && n_keys <= lq::kBuildThreads && use_lds && workspace &&
        workspace_bytes >= lora_build_workspace_bytes(n_tokens, n_adapters)) {
        int n_groups = (n_tokens + 1023) / 1024;
        if (n_groups > lq::kMultiMaxGroups) n_groups = lq::kMultiMaxGroups;
        int32_t* header = static_cast<int32_t*>(workspace);
        int32_t* counts = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + lq::kWsHeaderBytes);
        const hipError_t e = lq::launch_kernel(lq::kKernelBuild, lq::build_segments_multi_kernel, dim3(n_groups),
                                               dim3(lq::kBuildThreads), hist_bytes, st, token_adapter, token_kind, n_tokens, ranks,
                                               n_adapters, perm, seg_starts, seg_adapter, seg_kind, h_offsets, n_segments, header,
                                               counts);
        return e == hipSuccess ? LQ_OK : LQ_ERR_HIP;
    }
    hipError_t e;
    if (use_lds && n_tokens <= 4 * lq::kWave) {  // a small batch: four waves
        e = lq::launch_kernel(lq::kKernelBuild, lq::build_segments_kernel<true, 4>, dim3(1), dim3(4 * lq::kWave), hist_bytes / 4, st,
                              token_adapter, token_kind, n_tokens, ranks, n_adapters, perm, seg_starts, seg_adapter, seg_kind,
                              h_offsets, n_segments, ws_hist);
    } else if (use_lds) {
        e = lq::launch_kernel(lq::kKernelBuild, lq::build_segments_kernel<true, lq::kBuildWaves>, dim3(1), dim3(lq::kBuildThreads),
                              hist_bytes, st, token_adapter, token_kind, n_tokens, ranks, n_adapters, perm, seg_starts, seg_adapter,
                              seg_kind, h_offsets, n_segments, ws_hist);
    } else {
        e = lq::launch_kernel(lq::kKernelBuild, lq::build_segments_kernel<false, lq::kBuildWaves>, dim3(1), dim3(lq::kBuildThreads), 0,
                              st, token_adapter, token_kind, n_tokens, ranks, n_adapters, perm, seg_starts, seg_adapter, seg_kind,
                              h_offsets, n_segments, ws_hist);
    }
    return e == hipSuccess ? LQ_OK : LQ_ERR_HIP;
}
