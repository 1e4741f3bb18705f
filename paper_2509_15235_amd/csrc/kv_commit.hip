// Commit of the accepted path into the pre-allocated KV cache (paper Section 3.1: draft
// tokens after the first rejected one are discarded; Appendix A: the cache is allocated
// once, so keeping the accepted tokens means moving their rows inside it).
//
// Node path[k]'s row sits at logical slot S + path[k] and has to end up at slot S + k.
// One thread owns one 16-byte piece of a (layer, KV head, K-or-V) row position and moves it
// for k = 1 .. accepted_len in ascending order. Since path[k] >= k, no source is
// overwritten before it is read, whatever the other threads do: pieces never overlap
// between threads. Eight moves are in flight per thread (all loads, then all stores),
// which keeps the ascending order where it matters: a batch's destinations lie below the
// next batch's sources.
//
// A workgroup serves one sequence: it checks the path, the prefix length and (paged) the
// block-table entries of every slot it may touch before anything moves; a sequence that
// fails a check is reported through `status`, keeps its cache and its prefix length.
#include "vs_internal.h"

namespace vs {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int kCommitThreads = 256;
constexpr int kCommitBatch = 8;

__global__ __launch_bounds__(kCommitThreads) void kv_commit_kernel(const CommitParams p) {
    __shared__ int32_t spath[VS_MAX_TREE];
    __shared__ int32_t sflag;
    const int b = blockIdx.y;
    const int tid = threadIdx.x;
    const int32_t S = p.prefix_len[b];
    const int32_t alen = p.accepted_len[b];
    if (tid == 0) sflag = 0;
    __syncthreads();
    // ---- checks (every workgroup of the sequence repeats them; they are a few dozen loads)
    const bool alen_ok = alen >= 0 && alen < p.T;
    if (tid < p.T) {
        const int32_t v = p.path[(int64_t)b * p.T + tid];
        spath[tid] = v;
        if (alen_ok && tid <= alen) {
            const int32_t prev = tid == 0 ? -1 : p.path[(int64_t)b * p.T + tid - 1];
            const bool ok = tid == 0 ? (v == 0) : (v > prev && v < p.T);
            if (!ok) atomicOr(&sflag, 1);
        }
    }
    const int64_t have = p.paged ? (int64_t)p.max_blocks * p.block_size : p.capacity;
    const bool s_ok = S >= 0 && (int64_t)S + p.T <= have;
    if (s_ok && p.paged) {
        const int first = S >> p.block_shift, last = (S + p.T - 1) >> p.block_shift;
        for (int i = first + tid; i <= last; i += kCommitThreads) {
            const int32_t blk = p.block_table[(int64_t)b * p.max_blocks + i];
            if ((uint32_t)blk >= (uint32_t)p.num_blocks) atomicOr(&sflag, 2);
        }
    }
    __syncthreads();
    const int32_t f = sflag;
    int32_t code = VS_STATUS_OK;
    if (!alen_ok || (f & 1)) code = VS_STATUS_BAD_PATH;
    else if (!s_ok) code = VS_STATUS_BAD_PREFIX;
    else if (f & 2) code = VS_STATUS_BAD_BLOCK;
    if (blockIdx.x == 0 && tid == 0) {
        if (p.status) p.status[b] = code;
        p.new_prefix_len[b] = code == VS_STATUS_OK ? S + alen + 1 : S;
    }
    if (code != VS_STATUS_OK || alen == 0) return;

    // ---- this thread's piece: (layer, K or V, KV head, 16-byte chunk of the row)
    int64_t item = (int64_t)blockIdx.x * kCommitThreads + tid;
    if (item >= p.items_per_seq) return;
    const int chunk = (int)(item % p.chunks_per_row);
    item /= p.chunks_per_row;
    const int kvh = (int)(item % p.Hkv);
    item /= p.Hkv;
    const int which = (int)(item & 1);
    const int64_t layer = item >> 1;
    char* base = (char*)(which ? p.v : p.k) + layer * p.stride_layer_bytes + (int64_t)kvh * p.stride_head_bytes +
                 (int64_t)chunk * 16;
    if (!p.paged) base += (int64_t)b * p.stride_seq_bytes;
    auto row = [&](int32_t tok) -> char* {
        if (p.paged) {
            const int32_t blk = p.block_table[(int64_t)b * p.max_blocks + (tok >> p.block_shift)]; // checked above
            return base + (int64_t)blk * p.stride_block_bytes + (int64_t)(tok & (p.block_size - 1)) * p.stride_tok_bytes;
        }
        return base + (int64_t)tok * p.stride_tok_bytes;
    };
    for (int k0 = 1; k0 <= alen; k0 += kCommitBatch) {
        u32x4 r[kCommitBatch];
#pragma unroll
        for (int u = 0; u < kCommitBatch; ++u)
            if (k0 + u <= alen) r[u] = *(const u32x4*)row(S + spath[k0 + u]);
#pragma unroll
        for (int u = 0; u < kCommitBatch; ++u)
            if (k0 + u <= alen && spath[k0 + u] != k0 + u) *(u32x4*)row(S + k0 + u) = r[u];
    }
}

} // namespace

hipError_t launch_kv_commit(const CommitParams& p, hipStream_t s) {
    const dim3 grid((unsigned)((p.items_per_seq + kCommitThreads - 1) / kCommitThreads), (unsigned)p.B);
    hipLaunchKernelGGL(kv_commit_kernel, grid, dim3(kCommitThreads), 0, s, p);
    return hipGetLastError();
}

} // namespace vs
