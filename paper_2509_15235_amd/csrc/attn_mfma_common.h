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

// ---- Balanced schedule: the key ranges of a whole ragged batch, cut into shares of equal cost.
// The keys of all sequences, counted in 64-key steps, are laid end to end (sequence 0 first); share c
// of W covers steps [bound(c), bound(c + 1)) of that line, and the part of a sequence that falls
// into a share is a piece of work: a share that crosses from one sequence into the next is worked
// off piece by piece. A piece costs its steps plus kBalPieceCost (queries, first tiles, the
// pipeline's fill and drain: what happens before a piece's first and after its last step takes about
// as long as six steps). Lane i of a wave holds sequence i (at most 64 sequences). Main and combine
// kernel both derive the shares from the prefix lengths with the routines below, so they agree on
// where every piece's partial result lies: slot (share + sequence) of its KV head.
constexpr int kBalPieceCost = 6;
constexpr int kBalSnap = 3; // no piece this short (in steps) is left behind at a sequence's end

// this lane's sequence: its first step on the line and its number of steps (0: not usable)
__device__ __forceinline__ void bal_scan(const AttnParams& p, int lane, int& start, int& steps, int& total, bool& usable) {
    const int32_t S = lane < p.B ? p.prefix_len[lane] : -1;
    usable = lane < p.B && prefix_ok(p, S);
    steps = usable ? (S + p.tree_keys + kIterKeys - 1) / kIterKeys : 0;
    int inc = steps;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    start = inc - steps;
    total = __builtin_amdgcn_readlane(inc, 63);
}

// the steps [a, b) of a sequence (first step s0, t steps) that fall into [lo, hi) of the line; false: none
__device__ __forceinline__ bool bal_piece(int lo, int hi, int s0, int t, int& a, int& b) {
    a = max(lo, s0) - s0;
    b = min(hi, s0 + t) - s0;
    return b > a;
}

// cost of the most expensive share under the boundaries held one per lane (lane c: first step of share c)
__device__ __forceinline__ int bal_worst(const AttnParams& p, int lane, int start, int steps, int total, int bounds) {
    const int up = __shfl_down(bounds, 1);
    const int hi = lane + 1 < p.bal_chunks ? up : total;
    int cost = 0;
    for (int i = 0; i < p.B; ++i) {
        int a, b;
        if (bal_piece(bounds, hi, __builtin_amdgcn_readlane(start, i), __builtin_amdgcn_readlane(steps, i), a, b))
            cost += kBalPieceCost + (b - a);
    }
    if (lane >= p.bal_chunks) cost = 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cost = max(cost, __shfl_xor(cost, o));
    return cost;
}

// lane c (c < W): first step of share c; the other lanes: the end of the line.
// Two cuts are priced (most expensive share, a piece costing its steps plus kBalPieceCost) and the
// cheaper one is taken:
//  * even: the line with kBalPieceCost units inserted in front of every sequence is divided into W
//    equal parts; a boundary that falls into such a start-up stretch, or within kBalSnap steps of
//    either end of a sequence, moves onto the sequence's boundary (no stubs);
//  * regular, when W is a multiple of the number of sequences: every sequence gets W / B shares of
//    ceil(longest sequence / (W / B)) steps - what equal splits per sequence would be. Batches of
//    (nearly) equal lengths keep their equal splits this way.
// All lanes work side by side (a lane per share, a uniform loop over the sequences): a serial fill,
// share after share, costs a lone wave more than ten microseconds.
__device__ __forceinline__ int bal_bounds(const AttnParams& p, int lane, int start, int steps, int total) {
    const int W = p.bal_chunks;
    const int nseq = __popcll(__ballot(steps > 0));
    // start-up stretches in front of this lane's sequence: the usable sequences before it
    const int before = __popcll(__ballot(steps > 0) & ((1ull << lane) - 1ull));
    const int lstart = start + kBalPieceCost * before; // this lane's sequence on the stretched line
    const int ltotal = total + kBalPieceCost * nseq;
    const int raw = (int)((int64_t)min(lane, W) * ltotal / W);
    const int snap = min(kBalSnap, ltotal / W / 4);
    int even = lane < W ? -1 : total;
    for (int i = 0; i < p.B; ++i) {
        const int l0 = __builtin_amdgcn_readlane(lstart, i), s0 = __builtin_amdgcn_readlane(start, i);
        const int t = __builtin_amdgcn_readlane(steps, i);
        const int lend = l0 + kBalPieceCost + t;
        if (t > 0 && l0 <= raw && raw < lend) {
            if (raw - l0 <= kBalPieceCost + snap) even = s0;
            else if (lend - raw <= snap) even = s0 + t;
            else even = s0 + (raw - l0 - kBalPieceCost);
        }
    }
    if (even < 0) even = total; // raw == ltotal only for lanes >= W; an empty batch has no stretch to fall into
    int bounds = even;
    if (W % p.B == 0) {
        const int r = W / p.B;
        int smax = steps;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) smax = max(smax, __shfl_xor(smax, o));
        const int k = (smax + r - 1) / r;
        const int b = min(lane / r, p.B - 1), j = lane % r;
        const int sb = __shfl(start, b), tb = __shfl(steps, b);
        const int regular = lane < W ? sb + min(j * k, tb) : total;
        if (bal_worst(p, lane, start, steps, total, regular) <= bal_worst(p, lane, start, steps, total, even)) bounds = regular;
    }
    return bounds;
}

} // namespace vs
