// Device-side helpers shared by the attention and acceptance kernels.
#pragma once

#include "vs_internal.h"

namespace vs {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
    return __uint_as_float((uint32_t)b << 16);
}

// fp32 → bf16 storage, round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)float_to_bf16_bits(lo) | ((uint32_t)float_to_bf16_bits(hi) << 16);
}

// Loads one tree's parent row into LDS and checks it (parent[0] == -1, 0 <= parent[i] < i).
// Every thread of the workgroup must call it; blockDim.x >= T. Returns the vs_status.
__device__ __forceinline__ int32_t load_tree(const int32_t* __restrict__ parent_row, int T,
                                             int32_t* sp, int32_t* sflag) {
    const int tid = threadIdx.x;
    if (tid == 0) *sflag = 0;
    __syncthreads();
    if (tid < T) {
        const int32_t pv = parent_row[tid];
        sp[tid] = pv;
        if (tid == 0) {
            if (pv != -1) atomicOr(sflag, 1);
        } else if (pv < 0 || pv >= tid) {
            atomicOr(sflag, 2);
        }
    }
    __syncthreads();
    const int32_t f = *sflag;
    return (f & 1) ? VS_STATUS_BAD_ROOT : ((f & 2) ? VS_STATUS_BAD_PARENT : VS_STATUS_OK);
}

// Ancestor-or-self bit mask of `node` for a tree already validated by load_tree.
__device__ __forceinline__ uint64_t ancestor_mask(const int32_t* sp, int node) {
    uint64_t m = 1ull << node;
    int j = node;
    while (j > 0) {
        j = sp[j];
        m |= 1ull << j;
    }
    return m;
}

// Is this sequence's prefix length usable? (inside the host's bound and inside the cache)
__device__ __forceinline__ bool prefix_ok(const AttnParams& p, int32_t S) {
    if (S < 0 || S > p.max_prefix_len) return false;
    if (p.tree_keys == 0 && S < 1) return false; // nothing to attend to
    const int64_t need = (int64_t)S + p.tree_keys;
    const int64_t have = p.paged ? (int64_t)p.max_blocks * p.block_size : p.capacity;
    return need <= have;
}

// Element offset of logical token `tok` of KV head `kvh` in sequence `b`'s cache.
// Paged mode clamps a block id outside the pool to block 0 so that no access can leave
// the pool (the status array reports the bad entry separately).
__device__ __forceinline__ int64_t token_offset(const AttnParams& p, int b, int kvh, int tok) {
    if (p.paged) {
        int32_t blk = p.block_table[(int64_t)b * p.max_blocks + (tok >> p.block_shift)];
        if ((uint32_t)blk >= (uint32_t)p.num_blocks) blk = 0;
        return (int64_t)blk * p.stride_block + (int64_t)kvh * p.stride_head +
               (int64_t)(tok & (p.block_size - 1)) * p.stride_tok;
    }
    return (int64_t)b * p.stride_seq + (int64_t)kvh * p.stride_head + (int64_t)tok * p.stride_tok;
}

// The workgroup that owns a sequence's status entry calls this (all of its threads):
// writes tree / prefix problems, otherwise scans the block-table entries in use.
__device__ __forceinline__ void report_status(const AttnParams& p, int b, int32_t tree_code,
                                              bool s_ok, int32_t S, int32_t* sflag) {
    if (!p.status) return;
    int32_t code = tree_code;
    if (code == VS_STATUS_OK && !s_ok) code = VS_STATUS_BAD_PREFIX;
    if (code == VS_STATUS_OK && p.paged) {
        // *sflag is 0 here (load_tree leaves it 0 for a valid tree)
        const int nblk = (S + p.tree_keys + p.block_size - 1) >> p.block_shift;
        for (int i = threadIdx.x; i < nblk; i += blockDim.x) {
            const int32_t blk = p.block_table[(int64_t)b * p.max_blocks + i];
            if ((uint32_t)blk >= (uint32_t)p.num_blocks) atomicOr(sflag, 4);
        }
        __syncthreads();
        if (*sflag & 4) code = VS_STATUS_BAD_BLOCK;
    }
    if (threadIdx.x == 0) p.status[b] = code;
}

} // namespace vs
