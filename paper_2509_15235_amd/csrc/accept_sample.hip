// Stochastic acceptance over a draft tree (paper Section 3.1: accept a draft token with
// probability min(1, p / p_hat), otherwise continue with norm(max(0, p - p_hat)) and, when
// no candidate is left, draw the next token from it). The tree's candidates come from a
// deterministic top-k expansion, so the proposal for a candidate is a point mass: child c
// with token x is accepted iff u_accept[c] < r(x), r being the target softmax at the
// current node with the tokens rejected so far removed and the rest renormalised.
//
// Two kernels: (1) a bandwidth-bound scan that reduces each logits row to per-chunk
// (maximum, sum of exp) pairs; (2) one workgroup per sequence that walks the tree on those
// pairs alone - removing a token subtracts its weight from its chunk - and draws the bonus
// token by inverting the residual's cumulative sum in index order: chunk sums first, then
// one scan inside the chunk that holds the target. The second kernel touches the logits
// only for the candidates' own entries, for that one chunk, and for a chunk whose sum a
// removal cancelled (re-summed without the removed tokens).
#include "vs_device.h"

namespace vs {

namespace {

constexpr int kVec = 4;                  // 16-byte loads per thread and chunk (chunk = 4096 floats)
constexpr int kWalkThreads = 256;
constexpr int kPerThread = 16;           // chunk elements per thread of the walk kernel
static_assert(kWalkThreads * kPerThread == 4096, "the walk kernel scans one 4096-float chunk at a time");

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// grid = (chunks, B*T), block = 256: (max of the raw logits, sum of 2^((l - max) * k)) per chunk,
// k = log2(e) / temperature.
__global__ __launch_bounds__(kArgmaxBlock) void softmax_stats_partial_kernel(const SampleParams p) {
    __shared__ float sm[kArgmaxBlock / kWave];
    __shared__ float ss[kArgmaxBlock / kWave];
    const int chunk = blockIdx.x;
    const int64_t row = blockIdx.y;
    const float* __restrict__ lg = p.logits + row * p.ld;
    const int begin = chunk * p.chunk_elems;
    const int end = min(p.V, begin + p.chunk_elems);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    f32x4 a[kVec];
    const int nvec = p.vec_ok ? (end - begin) >> 2 : 0;
    const f32x4* __restrict__ lv = (const f32x4*)(lg + begin);
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < kVec; ++j) {
        const int k = threadIdx.x + j * kArgmaxBlock;
        a[j] = (k < nvec) ? __builtin_nontemporal_load(lv + k) : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
        for (int e = 0; e < 4; ++e) m = fmaxf(m, a[j][e]);
    }
    for (int t = begin + 4 * nvec + threadIdx.x; t < end; t += kArgmaxBlock) m = fmaxf(m, lg[t]);
    m = wave_max(m);
    if (lane == 0) sm[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    float s = 0.f;
    if (m > -INFINITY) {
#pragma unroll
        for (int j = 0; j < kVec; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) s += __builtin_amdgcn_exp2f((a[j][e] - m) * p.k_log2); // exp2(-inf) = 0
        for (int t = begin + 4 * nvec + threadIdx.x; t < end; t += kArgmaxBlock)
            s += __builtin_amdgcn_exp2f((lg[t] - m) * p.k_log2);
    }
    s = wave_sum(s);
    if (lane == 0) ss[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        p.part_m[row * p.chunks + chunk] = m;
        p.part_s[row * p.chunks + chunk] = (ss[0] + ss[1]) + (ss[2] + ss[3]);
    }
}

// grid = B, block = 256. Every thread runs the (short, sequential) walk on the same LDS
// data, so its branches are uniform and the whole workgroup can turn to a chunk-wide pass
// when one is needed.
__global__ __launch_bounds__(kWalkThreads) void accept_sample_walk_kernel(const SampleParams p) {
    __shared__ int32_t sp[VS_MAX_TREE];
    __shared__ int32_t sflag;
    __shared__ float sM[VS_MAX_TREE];      // row maxima
    __shared__ float sex[VS_MAX_TREE];     // weight of node c's token in its parent's row
    __shared__ int32_t sremoved[VS_MAX_TREE];
    __shared__ float sred[kWalkThreads / kWave];
    __shared__ float sch[kMaxSampleChunks]; // residual weight per chunk of the current row
    __shared__ int32_t spick, slast;
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = p.T;
    const int32_t tree_code = load_tree(p.parent + (int64_t)b * T, T, sp, &sflag);
    const int32_t* draft = p.draft + (int64_t)b * T;

    // ---- row maxima: four threads per row merge its chunks
    {
        const int i = tid >> 2, sub = tid & 3;
        float m = -INFINITY;
        const int64_t row = (int64_t)b * T + i;
        if (i < T)
            for (int c = sub; c < p.chunks; c += 4) m = fmaxf(m, p.part_m[row * p.chunks + c]);
        m = fmaxf(m, __shfl_xor(m, 1));
        m = fmaxf(m, __shfl_xor(m, 2));
        if (i < T && sub == 0) sM[i] = m;
    }
    __syncthreads();
    if (tree_code != VS_STATUS_OK) {
        if (tid < T) p.path[(int64_t)b * T + tid] = -1;
        if (tid == 0) {
            if (p.status) p.status[b] = tree_code;
            p.accepted_len[b] = 0;
            p.bonus[b] = -1;
        }
        return;
    }
    // ---- every candidate's weight in its parent's row, one thread per node
    if (tid >= 1 && tid < T) {
        const int par = sp[tid];
        const int32_t x = draft[tid];
        float ex = 0.f;
        if (x >= 0 && x < p.V && sM[par] > -INFINITY)
            ex = __builtin_amdgcn_exp2f((p.logits[((int64_t)b * T + par) * p.ld + x] - sM[par]) * p.k_log2);
        sex[tid] = ex;
    }
    __syncthreads();

    // Sum of sch[0..chunks), the same value in every thread. Two barriers.
    auto chunk_total = [&]() -> float {
        float s = 0.f;
        for (int c = tid; c < p.chunks; c += kWalkThreads) s += sch[c];
        s = wave_sum(s);
        __syncthreads(); // sred is free again
        if (lane == 0) sred[wave] = s;
        __syncthreads();
        return (sred[0] + sred[1]) + (sred[2] + sred[3]);
    };
    // This thread's 16 consecutive weights of chunk c of row `node`, removed tokens zeroed.
    auto load_weights = [&](int node, int c, int nrem, float (&w)[kPerThread]) {
        const float* lg = p.logits + ((int64_t)b * T + node) * p.ld;
        const float M = sM[node];
        const int j0 = c * p.chunk_elems + tid * kPerThread;
        if (p.vec_ok && j0 + kPerThread <= p.V) {
            const f32x4* lv = (const f32x4*)(lg + j0);
#pragma unroll
            for (int q = 0; q < kPerThread / 4; ++q) {
                const f32x4 a = lv[q];
#pragma unroll
                for (int e = 0; e < 4; ++e) w[4 * q + e] = __builtin_amdgcn_exp2f((a[e] - M) * p.k_log2);
            }
        } else {
#pragma unroll
            for (int e = 0; e < kPerThread; ++e)
                w[e] = (j0 + e < p.V) ? __builtin_amdgcn_exp2f((lg[j0 + e] - M) * p.k_log2) : 0.f;
        }
        for (int r = 0; r < nrem; ++r) {
            const int off = sremoved[r] - j0;
            if ((unsigned)off < (unsigned)kPerThread) {
#pragma unroll
                for (int e = 0; e < kPerThread; ++e)
                    if (e == off) w[e] = 0.f;
            }
        }
    };

    // ---- the walk
    int cur = 0, alen = 0, nrem = 0;
    float Z = 0.f;
    for (;;) {
        // residual weights of cur's row per chunk, relative to the row maximum
        const int64_t row = (int64_t)b * T + cur;
        const float M = sM[cur];
        __syncthreads(); // the previous node's sch / sremoved are no longer read
        for (int c = tid; c < p.chunks; c += kWalkThreads) {
            const float mc = p.part_m[row * p.chunks + c];
            sch[c] = (mc > -INFINITY) ? p.part_s[row * p.chunks + c] * __builtin_amdgcn_exp2f((mc - M) * p.k_log2) : 0.f;
        }
        __syncthreads();
        Z = chunk_total();
        nrem = 0;
        int next = -1;
        for (int c = cur + 1; c < T && next < 0; ++c) {
            if (sp[c] != cur) continue;
            const int32_t x = draft[c];
            bool gone = x < 0 || x >= p.V;
            for (int r = 0; r < nrem; ++r) gone = gone || sremoved[r] == x;
            const float ex = gone ? 0.f : sex[c];
            const float prob = (Z > 0.f) ? ex / Z : 0.f;
            if (p.u_accept[(int64_t)b * T + c] < prob) {
                next = c;
            } else if (!gone) {
                const int xc = x / p.chunk_elems;
                const float old = sch[xc];
                __syncthreads(); // every thread has read the list and the chunk sum
                if (tid == 0) sremoved[nrem] = x;
                ++nrem;
                __syncthreads();
                float fresh = old - ex;
                if (!(fresh >= 0.25f * old)) {
                    // the subtraction cancelled most of the chunk: sum it again without the removed tokens
                    float w[kPerThread];
                    load_weights(cur, xc, nrem, w);
                    float s = 0.f;
#pragma unroll
                    for (int e = 0; e < kPerThread; ++e) s += w[e];
                    s = wave_sum(s);
                    __syncthreads();
                    if (lane == 0) sred[wave] = s;
                    __syncthreads();
                    fresh = (sred[0] + sred[1]) + (sred[2] + sred[3]);
                }
                __syncthreads();
                if (tid == 0) sch[xc] = fresh;
                __syncthreads();
                Z = chunk_total();
            }
        }
        if (next < 0) break;
        cur = next;
        ++alen;
    }

    // ---- bonus token: inverse of the residual's cumulative sum, index order
    const float target = p.u_bonus[b] * Z;
    int kb = -1;
    float before = 0.f;
    {
        // every thread scans the chunk sums the same way
        float acc = 0.f;
        int last_pos = -1;
        for (int k = 0; k < p.chunks; ++k) {
            const float cs = sch[k];
            if (cs > 0.f) last_pos = k;
            if (kb < 0 && acc + cs > target) {
                kb = k;
                before = acc;
            }
            acc += cs;
        }
        if (kb < 0) { // u * total rounded up to the whole mass: last token with weight
            kb = last_pos;
            before = -INFINITY;
        }
    }
    if (tid == 0) {
        spick = INT32_MAX;
        slast = -1;
    }
    __syncthreads();
    if (kb >= 0) {
        float w[kPerThread];
        load_weights(cur, kb, nrem, w);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < kPerThread; ++e) s += w[e];
        // inclusive scan of the threads' sums: inside the wave, then across the four waves
        float inc = s;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const float up = __shfl_up(inc, o);
            if (lane >= o) inc += up;
        }
        if (lane == 63) sred[wave] = inc;
        __syncthreads();
        for (int wv = 0; wv < wave; ++wv) inc += sred[wv];
        const float local = target - before; // +inf when the whole mass is below the target
        const int j0 = kb * p.chunk_elems + tid * kPerThread;
        int last = -1;
#pragma unroll
        for (int e = 0; e < kPerThread; ++e)
            if (w[e] > 0.f) last = j0 + e;
        if (last >= 0) atomicMax(&slast, last);
        if (inc > local && last >= 0) {
            // first element of this thread whose running sum passes the target; the scan's and
            // the running sum's roundings may disagree by an ulp, then the last weighted one
            float acc = inc - s;
            int cand = -1;
#pragma unroll
            for (int e = 0; e < kPerThread; ++e) {
                acc += w[e];
                if (cand < 0 && acc > local && w[e] > 0.f) cand = j0 + e;
            }
            if (cand < 0) cand = last;
            atomicMin(&spick, cand);
        }
    }
    __syncthreads();
    // ---- results
    if (tid < T) {
        // path[k] = the ancestor of cur at depth k (cur's depth is alen)
        int32_t node = -1;
        if (tid <= alen) {
            node = cur;
            for (int k = alen; k > tid; --k) node = sp[node];
        }
        p.path[(int64_t)b * T + tid] = node;
    }
    if (tid == 0) {
        int32_t pick = spick;
        if (pick == INT32_MAX) pick = slast; // -1: no token carries weight (inputs must be finite)
        if (p.status) p.status[b] = VS_STATUS_OK;
        p.accepted_len[b] = alen;
        p.bonus[b] = pick;
    }
}

} // namespace

hipError_t launch_accept_sample(const SampleParams& p, hipStream_t s) {
    hipLaunchKernelGGL(softmax_stats_partial_kernel, dim3(p.chunks, p.B * p.T), dim3(kArgmaxBlock), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(accept_sample_walk_kernel, dim3(p.B), dim3(kWalkThreads), 0, s, p);
    return hipGetLastError();
}

} // namespace vs
