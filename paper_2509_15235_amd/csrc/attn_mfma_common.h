// Pieces shared by the matrix-core attention kernels: vector types, cross-half reductions
// and the workspace layout of split partial results.
#pragma once

#include "vs_device.h"

namespace vs {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

typedef __attribute__((address_space(3))) void lds_void;

// s_waitcnt immediate that waits until at most n vector-memory loads are outstanding and
// for nothing else (expcnt = 7, lgkmcnt = 15 are their maxima). Loads return in order.
constexpr int wait_vm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

constexpr float kLazy = 8.f; // log2 slack of the running softmax reference

// max(a, b, c); chains of these become v_max3_f32. (Not inline assembly: the compiler pads
// the wait states an MFMA result needs before a vector instruction may read it only for
// instructions it can see, and an asm statement reading a fresh MFMA result returned stale
// registers now and then - run-to-run differences in the softmax reference.)
__device__ __forceinline__ float max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

// max / sum over the two 32-lane halves, result in every lane (v_permlane32_swap)
__device__ __forceinline__ float half_max(float x) {
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Partial results of one (sequence, KV head, split, 32-row block): D/32 accumulator blocks,
// each stored as 2 x [64 lanes x 8 values] (register r = 4*q4 + e of lane l at
// ((db*2 + q4/2)*64 + l)*8 + (q4%2)*4 + e: a lane's eight values are one 16-byte piece, a wave's
// store or load of a piece is 1 KB of consecutive memory), followed elsewhere by 32 x (max, sum)
// in fp32. A partial output
// row is divided by its own sum before it is rounded: a convex combination of V rows, as large
// as the largest visible |V| and no larger. It is stored as bf16, which has V's own exponent
// range (fp16 would turn any |v| > 65504 into infinity) and costs half the bytes of fp32: what a
// split costs is mostly the write-back of these bytes at the end of the kernel. The 2^-9
// rounding of each partial enters the merged row once (the merge weights sum to one), next to
// the 2^-9 rounding of the final bf16 result.
__device__ __forceinline__ u32x2 pack_partial(float a, float b, float c, float d, float inv) {
    const f32x2 lo = {a * inv, b * inv}, hi = {c * inv, d * inv};
    u32x2 w;
    w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
    w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
    return w;
}
__device__ __forceinline__ f32x4 unpack_partial(u32x2 w) {
    const f32x4 r = {__uint_as_float(w[0] << 16), __uint_as_float(w[0] & 0xffff0000u), __uint_as_float(w[1] << 16),
                     __uint_as_float(w[1] & 0xffff0000u)};
    return r;
}
// One 32-channel accumulator block of a row block, divided by the rows' sums: two 16-byte pieces per
// lane. `blk` = start of the (unit, split, row block) partial block, db = channel block.
template <int D>
__device__ __forceinline__ void store_partial(uint16_t* blk, int db, int lane, const f32x16& a, float inv) {
#pragma unroll
    for (int hp = 0; hp < 2; ++hp) {
        const u32x2 lo = pack_partial(a[8 * hp], a[8 * hp + 1], a[8 * hp + 2], a[8 * hp + 3], inv);
        const u32x2 hi = pack_partial(a[8 * hp + 4], a[8 * hp + 5], a[8 * hp + 6], a[8 * hp + 7], inv);
        const u32x4 w = {lo[0], lo[1], hi[0], hi[1]};
        *(u32x4*)(blk + ((db * 2 + hp) * 64 + lane) * 8) = w;
    }
}
__device__ __forceinline__ int64_t part_block(const AttnParams& p, int64_t unit, int split, int rbk) {
    return (unit * p.num_splits + split) * (int64_t)(p.rows_pad / kRowBlock) + rbk;
}
// (max, sum) pairs are grouped per row block with the splits adjacent: index of the
// first of the 32 rows of (unit, rbk, split), in pairs.
__device__ __forceinline__ int64_t ml_block(const AttnParams& p, int64_t unit, int split, int rbk) {
    return ((unit * (p.rows_pad / kRowBlock) + rbk) * p.num_splits + split) * (int64_t)kRowBlock;
}

} // namespace vs
