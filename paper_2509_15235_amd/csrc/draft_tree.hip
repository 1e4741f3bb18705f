// Draft-tree construction (paper Section 3.1 adopts EAGLE-2's context-aware dynamic draft
// tree; Appendix A: 30 draft tokens, depth 3, 8 nodes kept per expansion). A node's score
// is the sum of the draft model's log-probabilities along its path. An expansion step gives
// every frontier node its K most likely tokens as children and keeps the K best-scored
// children as the next frontier; at the end the N best-scored candidates of all levels are
// the tree. The draft model's forward pass is not part of this: its logits are inputs.
//
// Three kernels: (1) a bandwidth-bound scan that reduces every 4096-float chunk of a logits
// row to (maximum, sum of exp, the chunk's K largest entries); (2) one workgroup per sequence
// that merges the chunks into each row's top K and log-sum-exp, scores the F*K candidates and
// picks the next frontier; (3) one workgroup per sequence for the final selection, which
// ranks candidates by counting and emits parent[] / tokens[] in candidate order.
//
// Selection without bookkeeping: entries are extracted in the strict total order
// (value descending, index ascending), so "the next one" is simply the best entry that comes
// strictly after the previous winner in that order - nothing has to be marked as taken.
#include "vs_device.h"

namespace vs {

namespace {

constexpr int kVec = 4;          // 16-byte loads per thread and chunk (chunk = 4096 floats)
constexpr int kSelThreads = 256;

struct Ent {
    float v;
    int32_t i;
};

// a comes strictly before b in (value descending, index ascending)
__device__ __forceinline__ bool before(float av, int32_t ai, float bv, int32_t bi) {
    return av > bv || (av == bv && ai < bi);
}

__device__ __forceinline__ Ent wave_first(Ent e) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(e.v, o);
        const int32_t oi = __shfl_xor(e.i, o);
        if (before(ov, oi, e.v, e.i)) {
            e.v = ov;
            e.i = oi;
        }
    }
    return e;
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

constexpr int32_t kNone = INT32_MAX; // index of "no entry": loses every comparison at value -inf

// grid = (chunks, B*F), block = 256.
__global__ __launch_bounds__(kArgmaxBlock) void draft_topk_partial_kernel(const DraftExpandParams p) {
    __shared__ float sv[kArgmaxBlock / kWave];
    __shared__ int32_t si[kArgmaxBlock / kWave];
    __shared__ float ss[kArgmaxBlock / kWave];
    const int chunk = blockIdx.x;
    const int64_t row = blockIdx.y;
    const float* __restrict__ lg = p.logits + row * p.ld;
    const int begin = chunk * p.chunk_elems;
    const int end = min(p.V, begin + p.chunk_elems);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // every thread holds 16 entries: from 16-byte loads when rows are aligned, else scalar
    float a[4 * kVec];
    int32_t base_idx[kVec]; // index of a[4*j]; entries 4*j .. 4*j+3 are consecutive
    int32_t lim[kVec];      // how many of the four are real entries of this chunk
    const int nvec = (end - begin) >> 2;
    if (p.vec_ok) {
        const f32x4* __restrict__ lv = (const f32x4*)(lg + begin);
#pragma unroll
        for (int j = 0; j < kVec; ++j) {
            const int k = threadIdx.x + j * kArgmaxBlock;
            const f32x4 x = (k < nvec) ? __builtin_nontemporal_load(lv + k) : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            base_idx[j] = begin + 4 * k;
            lim[j] = (k < nvec) ? 4 : 0; // the chunk's last 1-3 floats (V % 4) are the scalar tail below
#pragma unroll
            for (int e = 0; e < 4; ++e) a[4 * j + e] = x[e];
        }
    } else {
#pragma unroll
        for (int j = 0; j < kVec; ++j) {
            const int k = threadIdx.x + j * kArgmaxBlock;
            base_idx[j] = begin + 4 * k;
            lim[j] = max(0, min(4, end - (begin + 4 * k)));
#pragma unroll
            for (int e = 0; e < 4; ++e) a[4 * j + e] = (begin + 4 * k + e < end) ? lg[begin + 4 * k + e] : -INFINITY;
        }
    }
    // scalar tail of the vector path: at most 3 entries, owned by the threads 0..2
    float tail_v = -INFINITY;
    int32_t tail_i = kNone;
    if (p.vec_ok) {
        const int t = begin + 4 * nvec + threadIdx.x;
        if (t < end) {
            tail_v = lg[t];
            tail_i = t;
        }
    }
    auto valid = [&](int j, int e) { return e < lim[j]; };

    // ---- maximum and sum of exp
    float m = tail_v;
#pragma unroll
    for (int q = 0; q < 4 * kVec; ++q) m = fmaxf(m, a[q]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (lane == 0) sv[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    float s = 0.f;
    if (m > -INFINITY) {
#pragma unroll
        for (int q = 0; q < 4 * kVec; ++q) s += __builtin_amdgcn_exp2f((a[q] - m) * 1.4426950408889634f);
        if (tail_i != kNone) s += __builtin_amdgcn_exp2f((tail_v - m) * 1.4426950408889634f);
    }
    s = wave_sum(s);
    if (lane == 0) ss[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        p.part_m[row * p.chunks + chunk] = m;
        p.part_s[row * p.chunks + chunk] = (ss[0] + ss[1]) + (ss[2] + ss[3]);
    }

    // ---- the chunk's K first entries in (value descending, index ascending)
    float last_v = INFINITY;
    int32_t last_i = -1;
    Ent mine = {-INFINITY, kNone}; // this thread's first entry after (last_v, last_i)
    bool rescan = true;
    float* out_v = p.part_tv + (row * p.chunks + chunk) * p.K;
    int32_t* out_i = p.part_ti + (row * p.chunks + chunk) * p.K;
    for (int r = 0; r < p.K; ++r) {
        if (rescan) {
            mine = {-INFINITY, kNone};
#pragma unroll
            for (int j = 0; j < kVec; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float v = a[4 * j + e];
                    const int32_t i = base_idx[j] + e;
                    if (valid(j, e) && before(last_v, last_i, v, i) && before(v, i, mine.v, mine.i)) mine = {v, i};
                }
            if (tail_i != kNone && before(last_v, last_i, tail_v, tail_i) && before(tail_v, tail_i, mine.v, mine.i))
                mine = {tail_v, tail_i};
        }
        Ent w = wave_first(mine);
        __syncthreads(); // sv / si are free again
        if (lane == 0) {
            sv[wave] = w.v;
            si[wave] = w.i;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kArgmaxBlock / kWave; ++q)
            if (before(sv[q], si[q], w.v, w.i)) w = {sv[q], si[q]};
        if (threadIdx.x == 0) {
            out_v[r] = w.v;
            out_i[r] = w.i; // kNone when the chunk has fewer than r+1 entries
        }
        last_v = w.v;
        last_i = w.i;
        rescan = (mine.i == w.i); // only the winner's owner has to look for its next entry
        if (w.i == kNone) rescan = false;
    }
}

// grid = B, block = 256.
__global__ __launch_bounds__(kSelThreads) void draft_expand_select_kernel(const DraftExpandParams p) {
    __shared__ float s_lse[VS_MAX_TREE];
    __shared__ float s_score[kMaxDraftCand];
    __shared__ int32_t s_token[kMaxDraftCand];
    __shared__ uint8_t s_keep[kMaxDraftCand];
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int F = p.F, K = p.K, C = F * K;
    const int keep = min(K, C);

    // ---- per row (one wave at a time per row): log-sum-exp and the K first entries of the merged lists
    for (int f = wave; f < F; f += kSelThreads / kWave) {
        const int64_t row = (int64_t)b * F + f;
        const float* pm = p.part_m + row * p.chunks;
        const float* ps = p.part_s + row * p.chunks;
        float m = -INFINITY;
        for (int c = lane; c < p.chunks; c += kWave) m = fmaxf(m, pm[c]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
        float z = 0.f;
        for (int c = lane; c < p.chunks; c += kWave) {
            const float mc = pm[c];
            if (mc > -INFINITY) z += ps[c] * __builtin_amdgcn_exp2f((mc - m) * 1.4426950408889634f);
        }
        z = wave_sum(z);
        const float lse = m + __logf(z);
        if (lane == 0) s_lse[f] = lse;
        const float* tv = p.part_tv + row * p.chunks * K;
        const int32_t* ti = p.part_ti + row * p.chunks * K;
        const int n = p.chunks * K;
        float last_v = INFINITY;
        int32_t last_i = -1;
        const float cum = p.cum_in ? p.cum_in[row] : 0.f;
        for (int r = 0; r < K; ++r) {
            Ent mine = {-INFINITY, kNone};
            for (int q = lane; q < n; q += kWave) {
                const float v = tv[q];
                const int32_t i = ti[q];
                if (i != kNone && before(last_v, last_i, v, i) && before(v, i, mine.v, mine.i)) mine = {v, i};
            }
            const Ent w = wave_first(mine);
            if (lane == 0) {
                s_token[f * K + r] = w.i;
                s_score[f * K + r] = cum + (w.v - lse);
            }
            last_v = w.v;
            last_i = w.i;
        }
    }
    __syncthreads();

    // ---- next frontier: the `keep` first candidates in (score descending, index ascending), by counting
    for (int c = tid; c < C; c += kSelThreads) {
        const float sc = s_score[c];
        int rank = 0;
        for (int o = 0; o < C; ++o) rank += before(s_score[o], o, sc, c) ? 1 : 0;
        s_keep[c] = rank < keep ? 1 : 0;
    }
    __syncthreads();
    for (int c = tid; c < C; c += kSelThreads) {
        const int64_t g = (int64_t)b * p.cand_capacity + p.cand_base + c;
        p.cand_token[g] = s_token[c];
        p.cand_score[g] = s_score[c];
        p.cand_parent[g] = p.frontier_cand ? p.frontier_cand[(int64_t)b * F + c / K] : -1;
        if (s_keep[c]) {
            int pos = 0;
            for (int o = 0; o < c; ++o) pos += s_keep[o];
            if (pos >= keep) continue; // only NaN scores can rank more than `keep` candidates first
            p.next_frontier_cand[(int64_t)b * keep + pos] = p.cand_base + c;
            p.next_cum[(int64_t)b * keep + pos] = s_score[c];
        }
    }
}

// grid = B, block = 256.
__global__ __launch_bounds__(kSelThreads) void draft_tree_build_kernel(const DraftBuildParams p) {
    __shared__ float s_score[kMaxDraftTotal];
    __shared__ int32_t s_parent[kMaxDraftTotal];
    __shared__ uint8_t s_pick[kMaxDraftTotal];
    __shared__ int32_t s_bad;
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int M = p.M, N = p.N;
    const int take = min(N, M);
    const int32_t* tok = p.cand_token + (int64_t)b * p.cand_capacity;
    const float* score = p.cand_score + (int64_t)b * p.cand_capacity;
    const int32_t* par = p.cand_parent + (int64_t)b * p.cand_capacity;
    if (tid == 0) s_bad = 0;
    __syncthreads();
    for (int c = tid; c < M; c += kSelThreads) {
        s_score[c] = score[c];
        const int32_t pc = par[c];
        s_parent[c] = pc;
        if (pc < -1 || pc >= c) atomicOr(&s_bad, 1);
    }
    __syncthreads();
    for (int c = tid; c < M; c += kSelThreads) {
        const float sc = s_score[c];
        int rank = 0;
        for (int o = 0; o < M; ++o) rank += before(s_score[o], o, sc, c) ? 1 : 0;
        s_pick[c] = rank < take ? 1 : 0;
    }
    __syncthreads();
    if (!s_bad) {
        for (int c = tid; c < M; c += kSelThreads)
            if (s_pick[c] && s_parent[c] >= 0 && !s_pick[s_parent[c]]) atomicOr(&s_bad, 1);
    }
    __syncthreads();
    const bool bad = s_bad != 0;
    int32_t* o_parent = p.parent + (int64_t)b * (N + 1);
    int32_t* o_tokens = p.tokens + (int64_t)b * (N + 1);
    int32_t* o_cand = p.node_cand + (int64_t)b * (N + 1);
    for (int t = tid; t <= N; t += kSelThreads) { // the root, and -1 wherever no node is written below
        if (!bad && t >= 1 && t <= take) continue;
        o_parent[t] = -1;
        o_tokens[t] = (t == 0 && p.root_token) ? p.root_token[b] : -1;
        o_cand[t] = -1;
    }
    if (tid == 0) {
        p.num_nodes[b] = bad ? 0 : take + 1;
        if (p.status) p.status[b] = bad ? VS_STATUS_BAD_CANDIDATE : VS_STATUS_OK;
    }
    if (bad) return;
    for (int c = tid; c < M; c += kSelThreads) {
        if (!s_pick[c]) continue;
        int node = 1;
        for (int o = 0; o < c; ++o) node += s_pick[o];
        if (node > take) continue; // only NaN scores can rank more than `take` candidates first
        const int32_t pc = s_parent[c];
        int pnode = 0;
        if (pc >= 0) {
            pnode = 1;
            for (int o = 0; o < pc; ++o) pnode += s_pick[o];
        }
        o_parent[node] = pnode;
        o_tokens[node] = tok[c];
        o_cand[node] = c;
    }
}

} // namespace

hipError_t launch_draft_expand(const DraftExpandParams& p, hipStream_t s) {
    hipLaunchKernelGGL(draft_topk_partial_kernel, dim3(p.chunks, p.B * p.F), dim3(kArgmaxBlock), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(draft_expand_select_kernel, dim3(p.B), dim3(kSelThreads), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_draft_tree_build(const DraftBuildParams& p, hipStream_t s) {
    hipLaunchKernelGGL(draft_tree_build_kernel, dim3(p.B), dim3(kSelThreads), 0, s, p);
    return hipGetLastError();
}

} // namespace vs
