// Shared device-side helpers for the lqlora kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lqlora.h"

namespace lq {

constexpr int kWave = 64;
constexpr int kWsHeaderBytes = 256;   // workspace offset 0: int32 device error flags, rest reserved
constexpr int kErrBadSegment = 1;     // adapter id or rank outside the supported range

typedef unsigned short u16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// ---- bf16 <-> fp32 ---------------------------------------------------------------------------
// A 32-bit word holds two bf16 values: element 2i in the low half, 2i+1 in the high half.
__device__ __forceinline__ float bf16_lo(unsigned int w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned int w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN.
__device__ __forceinline__ unsigned int f32_to_bf16_bits(float f)
{
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

__device__ __forceinline__ void unpack8(const u32x4& w, float* f)
{
    f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x);
    f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
    f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z);
    f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
}

// ---- wave primitives ---------------------------------------------------------------------------
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int o = __shfl_up(v, d, kWave);
        if (lane_id() >= d) v += o;
    }
    return v;
}
__device__ __forceinline__ long long wave_inclusive_scan64(long long v)
{
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        long long o = __shfl_up(v, d, kWave);
        if (lane_id() >= d) v += o;
    }
    return v;
}
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// ---- chunk lookup ------------------------------------------------------------------------------
// The token rows of segment g are perm[seg_starts[g] .. seg_starts[g+1]).  Work is handed out in
// chunks of at most `tokens_per_chunk` consecutive positions of one segment; chunk ids count
// through the segments in order.  Every wave resolves its chunk id on its own with one wave scan
// per 64 segments (the tables are small and cache resident), so no plan buffer or extra launch
// is needed and the grid can be sized from host-known upper bounds.
struct Chunk {
    int seg;   // -1: chunk id beyond the last chunk
    int pos;   // first position in perm
    int len;   // rows in this chunk
    int first; // position of the segment's first row
};

__device__ __forceinline__ Chunk find_chunk(const int32_t* __restrict__ seg_starts, int n_seg, int chunk_id,
                                            int tokens_per_chunk)
{
    Chunk c;
    c.seg = -1; c.pos = 0; c.len = 0; c.first = 0;
    const int lane = lane_id();
    int base = 0;
    for (int s0 = 0; s0 < n_seg; s0 += kWave) {
        const int s = s0 + lane;
        int st = 0, en = 0;
        if (s < n_seg) { st = seg_starts[s]; en = seg_starts[s + 1]; }
        const int len = en > st ? en - st : 0;
        const int nch = (len + tokens_per_chunk - 1) / tokens_per_chunk;
        const int incl = wave_inclusive_scan(nch);
        const int total = __shfl(incl, kWave - 1, kWave);
        if (chunk_id < base + total) {
            const unsigned long long m = __ballot(base + incl > chunk_id);
            const int l = __ffsll((long long)m) - 1;
            const int excl = __shfl(incl - nch, l, kWave);
            const int sst = __shfl(st, l, kWave);
            const int sen = __shfl(en, l, kWave);
            const int local = chunk_id - base - excl;
            c.seg = s0 + l;
            c.first = sst;
            c.pos = sst + local * tokens_per_chunk;
            c.len = min(tokens_per_chunk, sen - c.pos);
            return c;
        }
        base += total;
    }
    return c;
}

}  // namespace lq
