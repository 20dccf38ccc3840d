// Declarations shared by the forward and backward translation units (not part of the C ABI).
#pragma once

#include <hip/hip_ext.h>

#include <atomic>
#include <type_traits>

#include "lq_segments.h"

namespace lq {

// Parameter block of the shrink / expand / fused kernels.  The backward pass reuses the same kernels
// with the roles swapped (g = dy B^T is a shrink over d_out, dx += s g A is an expand over d_in).
// One linear layer of a call.  A grouped call has several that read the same x (the Q, K, V projections of
// Algorithm 1, the MLP's gate and up); the batch, its tables, the ranks and the scales are common to them.
constexpr int kMaxProj = LQ_MAX_GROUP;
struct Proj {
    u16* y; long long ldy; int d_out;
    const void* const* A_ptrs; const void* const* B_ptrs;
    float* h_out;
};

// FwdCore is the parameter block of a call with one linear layer, FwdParams (below) that of a grouped call; the
// device functions are templates over the two (n_proj_of and proj_of tell them apart).  The kernels are short of
// scalar registers: the larger block as the argument of every kernel makes a single call re-read its arguments
// from memory over and over (measured: + 1.2 us per call); and a local copy of a block ends up in scratch memory.
struct FwdCore {
    const u16* x; long long ldx;
    int d_in;
    int n_proj; Proj proj0;  // the first (or only) linear layer
    const int32_t* ranks; const float* scales; int n_adapters; int max_rank;
    const float* token_scales;  // per token row; when given it replaces scales[adapter] (null: per-adapter scales)
    const int32_t* perm; int n_tokens;
    const int32_t* seg_starts; const int32_t* seg_adapter; const uint8_t* seg_kind;
    const int32_t* n_segments; int max_segments;
    const long long* h_offsets;
    float* hpart;    // [projection][ksplit][n_tokens][rstride] h of each slice of d_in by position in segment order (unscaled)
    long long hproj; // elements of hpart per projection
    int ksplit;      // a power of two
    int ks_log2;
    int rstride;     // 32, 64 or 128
    int* header;     // the workspace header (4096 bytes): ticket counters and the barrier's words
    int* err;        // error word (normally word 0 of the header)
    int ksplit_hint; // host only: > 0 forces this split (the expand half of a pair repeats the shrink half's)
    int kinds;       // bit k set: segments of kind k take part (forward: all; backward: fine-tune only)
    int coherent;    // fused variant: the h slices are written and read with device-scope accesses
    unsigned int hpart_bytes;  // size of hpart (for the buffer descriptor of the device-scope 16-byte loads)
    int* tickets;    // workspace header words 4..: unit tickets ([0,1] shrink phase, [2,3] expand phase); the barrier's words: kBar*
};

struct FwdParams : FwdCore {
    Proj more[kMaxProj - 1];  // the other linear layers of a grouped call
};

__device__ __forceinline__ int n_proj_of(const FwdCore&) { return 1; }
__device__ __forceinline__ int n_proj_of(const FwdParams& p) { return p.n_proj; }
__device__ __forceinline__ Proj proj_of(const FwdCore& p, int) { return p.proj0; }

// linear layer pi of a call (pi wave uniform).  Every member is picked by value: a run-time index into the kernel's
// parameter block (or a choice between references into it) would make the compiler keep a copy of the whole block
// in scratch memory (measured: + 20 us per launch).
__device__ __forceinline__ Proj proj_of(const FwdParams& p, int pi)
{
    static_assert(kMaxProj == 4, "the entries are picked by name");
#define LQ_PICK(member) (pi == 0 ? p.proj0.member : pi == 1 ? p.more[0].member : pi == 2 ? p.more[1].member : p.more[2].member)
    Proj q;
    { u16* const v = LQ_PICK(y); q.y = v; }
    { const long long v = LQ_PICK(ldy); q.ldy = v; }
    { const int v = LQ_PICK(d_out); q.d_out = v; }
    { const void* const* const v = LQ_PICK(A_ptrs); q.A_ptrs = v; }
    { const void* const* const v = LQ_PICK(B_ptrs); q.B_ptrs = v; }
    { float* const v = LQ_PICK(h_out); q.h_out = v; }
#undef LQ_PICK
    return q;
}

constexpr int kThreads = 512;              // threads of a workgroup of the forward kernels
constexpr int kWaves = kThreads / kWave;

// ---- unit hand-out --------------------------------------------------------------------------------
// A workgroup's first two units are fixed: its own index and that plus the grid size.  Units differ in
// size by more than 10x, so the later ones are drawn from a counter instead of striding; the draw is
// issued when a unit starts and read when it ends.  (Not for the first unit: all workgroups start
// together, 256 draws on one address take microseconds, and the loads behind a draw cannot be used
// before it returns.)  Relaxed device-scope atomics: no data depends on the counters.  The last
// workgroup to leave puts both counters back to zero, so they are zero between launches.  One barrier
// per unit, which also separates the units' uses of the LDS.
//   ctr[0] draws so far, ctr[1] workgroups that left; slot: two ints of LDS
//   it0 = 1: the workgroup's first unit has been run already; start with the second
template <class Body>
__device__ __forceinline__ void for_each_unit(int* ctr, int n_units, int* slot, Body&& body, int it0 = 0)
{
    const int grid = (int)gridDim.x;
    const bool more = n_units > grid, draws = n_units > 2 * grid;
    int id = (int)blockIdx.x + it0 * grid;
    for (int it = it0; id < n_units; ++it) {
        int next = id + grid;
        if (it > 0 && threadIdx.x == 0)
            next = draws ? 2 * grid + __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : n_units;
        body(id, it);
        if (!more) break;
        if (threadIdx.x == 0) slot[it & 1] = next;
        __syncthreads();
        id = uniform(slot[it & 1]);
    }
    if (draws && threadIdx.x == 0) {
        const int left = __hip_atomic_fetch_add(ctr + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (left == grid - 1) {
            __hip_atomic_store(ctr + 0, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(ctr + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// GROUP = false: the instantiation for a call with one linear layer.  The compiler is told so, and everything
// that sorts units by projection folds away (a decode batch's start is bound by its instruction count).
// The argument of a kernel: the whole block for a grouped call, its core for a single call.
template <bool GROUP> using KernelArg = std::conditional_t<GROUP, FwdParams, FwdCore>;


// number of workgroups of `kernel` that are resident at once on the current device
template <typename K>
inline int resident_grid(K kernel, size_t dyn_lds)
{
    int dev = 0, cus = 0, per_cu = 0;
    if (dyn_lds > 48 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)dyn_lds);
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, dyn_lds) != hipSuccess || per_cu <= 0)
        per_cu = 1;
    return cus * per_cu;
}

inline int nt_for(int max_rank) { return max_rank <= 16 ? 1 : max_rank <= 32 ? 2 : max_rank <= 64 ? 4 : 8; }  // 16-rank tiles

// The row-slab variant (LQ_VARIANT_SLAB): one launch, no partial-h buffer, no device-wide wait.
hipError_t run_slab(const FwdParams& p, hipStream_t stream);

constexpr int kAllKinds = 7;
constexpr int kFinetuneOnly = 1 << LQ_SEG_FINETUNE;

// A launch grid that depends on the device (resident workgroups), worked out once per device: `compute` runs on
// the first call on a device (two threads that race there store the same value).
constexpr int kMaxDevices = 64;
struct DeviceGrid {
    std::atomic<int> grid[kMaxDevices];
    template <class F>
    int get(F&& compute)
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return compute();
        int g = grid[dev].load(std::memory_order_relaxed);
        if (g <= 0) {
            g = compute();
            grid[dev].store(g, std::memory_order_relaxed);
        }
        return g;
    }
};

bool aligned16(const void* p);
int rstride_for(int max_rank);
int auto_variant(int max_rank, long long out_columns);  // LQ_VARIANT_AUTO's choice: LQ_VARIANT_SLAB or LQ_VARIANT_FUSED
size_t h_slices_bytes(int n_tokens, int max_rank);   // bytes of the partial-h region of a workspace

// Fills p.ksplit and enqueues: variant LQ_VARIANT_SPLIT / _FUSED / _SHRINK_ONLY / _EXPAND_ONLY.
// p.ksplit_hint > 0 forces that split (the expand half of a pair must use the shrink half's value).
hipError_t run_shrink_expand(FwdParams& p, int variant, hipStream_t stream);

// ---- device-wide barrier of a launch whose workgroups are all resident (grid = occupancy x compute units) ----
// Data that crosses it must be written and read with device-scope accesses (the XCDs' L2 caches are not
// coherent with each other); the barrier itself uses no cache write-back or invalidation.  header: the
// workspace header; err: the error word; gen0: the generation word read before this workgroup arrives.  The
// wait is bounded; a timeout sets bit 1 of the error word and the caller's next phase is skipped.
constexpr int kErrBarrierTimeout = 2;
constexpr int kBarrierSpinLimit = 1 << 20;

// Words of the workspace header used by the barrier, every counter on a 128-byte line of its own: 256
// arrivals on one word take ~5 us (additions to one address are served one after the other), so a
// workgroup arrives at one of 16 counters, and the last one at each of those arrives at the top counter.
// All counters are back at zero when the barrier opens.
constexpr int kBarGen = 32, kBarTop = 64, kBarSub = 96, kBarLine = 32, kBarFan = 16;  // int offsets from the header

// The generation word counts the barriers that opened (modulo 2^30).  A workgroup whose wait runs out sets bit 1
// of the error word and poisons the generation word (kBarPoison), which sends every workgroup that is still
// waiting, or that arrives later, or that starts later, down the same path: the caller's next phase is skipped by
// all of them (up to the race between the poison and a barrier that opens at the same moment).  The poison
// stays until the caller zeroes the workspace header.
constexpr int kBarPoison = 1 << 30;
__device__ __forceinline__ bool barrier_poisoned(int gen0) { return (gen0 & kBarPoison) != 0; }

// `overlap` runs in every thread between the workgroup's arrival and its wait for the others.  Returns true
// (in every thread of the workgroup) if the barrier opened, false if the wait ran out here or elsewhere.
template <class Overlap>
__device__ __forceinline__ bool grid_barrier(int* header, int* err, int gen0, Overlap&& overlap)
{
    // every thread's device-scope (written-through) stores are acknowledged before its workgroup arrives
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const int opened = (gen0 + 1) & (kBarPoison - 1);
    if (threadIdx.x == 0 && !barrier_poisoned(gen0)) {
        int* gen = header + kBarGen;
        const int grid = (int)gridDim.x, k = (int)blockIdx.x % kBarFan;
        const int n_k = (grid - k + kBarFan - 1) / kBarFan, n_sub = min(grid, kBarFan);
        int* sub = header + kBarSub + k * kBarLine;
        if (__hip_atomic_fetch_add(sub, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_k - 1) {
            __hip_atomic_store(sub, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int* top = header + kBarTop;
            if (__hip_atomic_fetch_add(top, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_sub - 1) {
                __hip_atomic_store(top, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(gen, opened, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    overlap();
    int failed = 0;
    if (threadIdx.x == 0) {
        int* gen = header + kBarGen;
        int spins = 0, now = gen0;
        while (!barrier_poisoned(gen0)) {
            now = __hip_atomic_load(gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (now != gen0) break;
            __builtin_amdgcn_s_sleep(8);
            if (++spins > kBarrierSpinLimit) break;
        }
        if (now != opened) {
            failed = 1;
            atomicOr(err, kErrBarrierTimeout);
            if (!barrier_poisoned(now))
                __hip_atomic_store(gen, gen0 | kBarPoison, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    failed = __syncthreads_or(failed);
    asm volatile("" ::: "memory");  // loads of the next phase stay behind the barrier
    return failed == 0;
}

// ---- optional timing of the library's own launches (lora_profile_enable / lora_profile_read) ----------------
// When enabled, a launch goes through hipExtLaunchKernelGGL with a pair of events that receive the
// dispatch's own start and end time stamps (what a kernel trace reports), and is filed under its id.
enum KernelId { kKernelBuild = 0, kKernelShrink, kKernelExpand, kKernelFused, kKernelWgrad, kKernelWreduce, kKernelSlab, kKernelIds };
bool profile_on();
void profile_events(int kernel_id, hipEvent_t* start, hipEvent_t* stop);  // a fresh pair (null, null when full)

template <class K, class... Args>
hipError_t launch_kernel(int kernel_id, K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args)
{
    if (profile_on()) {
        hipEvent_t e0 = nullptr, e1 = nullptr;
        profile_events(kernel_id, &e0, &e1);
        hipExtLaunchKernelGGL(kernel, grid, block, (unsigned int)lds, st, e0, e1, 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
    }
    return hipGetLastError();
}

}  // namespace lq
