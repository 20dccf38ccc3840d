// Shared device-side helpers for the lqlora kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lqlora.h"

namespace lq {

constexpr int kWave = 64;
constexpr int kWsHeaderBytes = 4096;  // workspace offset 0: int32 device error flags; ticket and barrier words follow
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
// two fp32 -> packed bf16 with the hardware conversion (round to nearest even)
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi)
{
    const f32x2 v{lo, hi};
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ void unpack8(const u32x4& w, float* f)
{
    f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x);
    f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
    f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z);
    f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
}

// ---- transposing LDS read (gfx950 ds_read_b64_tr_b16) ------------------------------------------
// A 16 x 32 block of 16-bit elements that lies row-major in LDS ([k row][column], `pitch` elements per row)
// as the 16x16x32 MFMA wants it: lane (c = lane % 16, kg = lane / 16) gets column c, rows 8 kg .. 8 kg + 7.
// Within every group of 16 lanes the instruction gathers the 8-byte pieces the lanes point at and hands lane
// i the i%4-th element of the pieces of lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12; so lane q of a group points
// at row q / 4 of the group's four rows, columns 4 (q % 4) .. + 3, and two reads cover the 8 rows.
// block: element (k row 0, column 0) of the block; 8-byte aligned, pitch a multiple of 4.
typedef __attribute__((ext_vector_type(4))) short s16x4;
// The four 4-column pieces need not be adjacent: piece i starts at column piece_stride * i (lane c then gets
// column piece_stride * (c / 4) + c % 4).
__device__ __forceinline__ u32x4 lds_read_transposed_16x32(const u16* block, int pitch, int piece_stride = 4)
{
    typedef __attribute__((address_space(3))) s16x4* lds_ptr;
    const int lane = lane_id(), q = lane & 15, kg = lane >> 4;
    const u16* p = block + (8 * kg + (q >> 2)) * pitch + piece_stride * (q & 3);
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p);
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * pitch));
    typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
    const u32x2 lo = __builtin_bit_cast(u32x2, a), hi = __builtin_bit_cast(u32x2, b);
    return u32x4{lo.x, lo.y, hi.x, hi.y};
}

// ---- wave primitives ---------------------------------------------------------------------------
// v + (v of another lane, picked by a DPP control; 0 where that lane lies outside the row or the row is
// masked off)
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_add(int v)
{
    return v + __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}
// Inclusive prefix sum over the 64 lanes with DPP moves (no LDS traffic): four shifted adds inside every
// row of 16 lanes, then lane 15 of rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    v = dpp_add<0x111, 0xf>(v);  // row_shr:1
    v = dpp_add<0x112, 0xf>(v);  // row_shr:2
    v = dpp_add<0x114, 0xf>(v);  // row_shr:4
    v = dpp_add<0x118, 0xf>(v);  // row_shr:8
    v = dpp_add<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
    return v;
}
// the same for 64-bit values in [0, 2^54): the low 24 bits and the rest are scanned as two ints (neither
// sum can overflow) and put together again
__device__ __forceinline__ long long wave_inclusive_scan64(long long v)
{
    const int lo = wave_inclusive_scan((int)(v & 0xffffff));
    const int hi = wave_inclusive_scan((int)(v >> 24));
    return (long long)lo + ((long long)hi << 24);
}
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int lane_value(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }  // lane: wave uniform

// n / d for 0 <= n and 1 <= d, both wave uniform and small: a reciprocal estimate and one correction
// instead of the ~40-instruction exact sequence
__device__ __forceinline__ int small_div(int n, int d)
{
    if (n >= (1 << 22)) return n / d;
    int q = (int)((float)n * __builtin_amdgcn_rcpf((float)d));
    const int r = n - q * d;
    if (r >= d) ++q;
    if (r < 0) --q;
    return q;
}

}  // namespace lq
