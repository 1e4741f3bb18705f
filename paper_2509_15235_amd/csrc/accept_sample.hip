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
constexpr int kKeepStats = 4096;          // (max, sum) pairs the walk kernel can keep in LDS (32 KB)
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
    // one-dimensional grid: workgroup id = row * chunks + chunk (the host keeps the product below 2^31)
    const int64_t row = blockIdx.x / (uint32_t)p.chunks;
    const int chunk = (int)(blockIdx.x - (uint32_t)row * (uint32_t)p.chunks);
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
// when one is needed. Everything the walk compares is fetched up front (row maxima and
// masses, the uniforms, every candidate's weight in its parent's row), so a step of the walk
// costs no memory round trip: removing a rejected token just lowers the row's mass. Only when
// that subtraction would cancel (the rejected token held > 95 % of the mass), and once at the
// end for the bonus draw, the row's per-chunk masses are needed - from the copy of all rows'
// chunk statistics in LDS when those fit, else from memory.
__global__ __launch_bounds__(kWalkThreads) void accept_sample_walk_kernel(const SampleParams p) {
    __shared__ int32_t sp[VS_MAX_TREE];
    __shared__ int32_t sflag;
    __shared__ float sM[VS_MAX_TREE];      // row maxima
    __shared__ float sZ[VS_MAX_TREE];      // row masses relative to the maxima
    __shared__ float sex[VS_MAX_TREE];     // weight of node c's token in its parent's row
    __shared__ float su[VS_MAX_TREE];      // u_accept
    __shared__ int32_t sdraft[VS_MAX_TREE];
    __shared__ int32_t sremoved[VS_MAX_TREE];
    __shared__ float sremoved_ex[VS_MAX_TREE];
    __shared__ float sred[kWalkThreads / kWave];
    __shared__ float sch[kMaxSampleChunks]; // residual weight per chunk of the current row
    __shared__ float skeep_m[kKeepStats], skeep_s[kKeepStats]; // every row's chunk statistics, when they fit
    __shared__ int32_t spick, slast;
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = p.T;
    // Everything that does not depend on the tree is requested before the tree is waited for: the
    // bonus uniform (used at the very end), this thread's draft token and acceptance uniform, and
    // the first sixteen chunk statistics of this thread's row (four threads per row; one memory
    // round trip covers vocabularies up to 64 chunks). Malformed trees are reported below; none
    // of these addresses depends on the tree's contents.
    const float u_bonus = p.u_bonus[b];
    constexpr int kPre = 16;
    const int ri = tid >> 2, sub = tid & 3;
    const int64_t rrow = (int64_t)b * T + ri;
    float pm[kPre], ps[kPre];
    auto fetch_stats = [&](int c0) {
#pragma unroll
        for (int q = 0; q < kPre; ++q) {
            const int c = c0 + 4 * q;
            const bool ok = ri < T && c < p.chunks;
            pm[q] = ok ? p.part_m[rrow * p.chunks + c] : -INFINITY;
            ps[q] = ok ? p.part_s[rrow * p.chunks + c] : 0.f;
        }
    };
    fetch_stats(sub);
    const int32_t x_own = (tid < T) ? p.draft[(int64_t)b * T + tid] : -1;
    const float u_own = (tid < T) ? p.u_accept[(int64_t)b * T + tid] : 0.f;
    const int32_t tree_code = load_tree(p.parent + (int64_t)b * T, T, sp, &sflag);
    // node tid's logit in the parent's row (parent index clamped: a malformed tree is reported
    // below and must not steer a load out of bounds)
    const bool has_logit = tid >= 1 && tid < T && x_own >= 0 && x_own < p.V;
    float l_own = 0.f;
    if (has_logit) {
        const int par = min(max(sp[tid], 0), T - 1);
        l_own = p.logits[((int64_t)b * T + par) * p.ld + x_own];
    }

    // ---- row maxima and masses, merged online. When all rows' chunk statistics fit (T * chunks
    // <= kKeepStats) they also stay in LDS, so that the per-chunk masses a rejection or the bonus
    // draw needs later cost no second trip to memory.
    const bool keep = T * p.chunks <= kKeepStats;
    {
        float m = -INFINITY, z = 0.f;
        for (int c0 = sub; c0 < p.chunks; c0 += 4 * kPre) {
            if (c0 != sub) fetch_stats(c0);
            if (keep) {
#pragma unroll
                for (int q = 0; q < kPre; ++q) {
                    const int c = c0 + 4 * q;
                    if (ri < T && c < p.chunks) {
                        skeep_m[ri * p.chunks + c] = pm[q];
                        skeep_s[ri * p.chunks + c] = ps[q];
                    }
                }
            }
            float bm = m;
#pragma unroll
            for (int q = 0; q < kPre; ++q) bm = fmaxf(bm, pm[q]);
            if (bm > -INFINITY) {
                z *= __builtin_amdgcn_exp2f((m - bm) * p.k_log2); // m = -inf: z is 0 and stays 0
#pragma unroll
                for (int q = 0; q < kPre; ++q)
                    if (pm[q] > -INFINITY) z += ps[q] * __builtin_amdgcn_exp2f((pm[q] - bm) * p.k_log2);
                m = bm;
            }
        }
        float mm = fmaxf(m, __shfl_xor(m, 1));
        mm = fmaxf(mm, __shfl_xor(mm, 2));
        if (m > -INFINITY) z *= __builtin_amdgcn_exp2f((m - mm) * p.k_log2);
        z += __shfl_xor(z, 1);
        z += __shfl_xor(z, 2);
        if (ri < T && sub == 0) {
            sM[ri] = mm;
            sZ[ri] = z;
        }
    }
    if (tid < T) {
        su[tid] = u_own;
        sdraft[tid] = x_own;
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
    // ---- every candidate's weight in its parent's row, one thread per node (the logit itself was
    // requested at the top, together with the chunk statistics)
    if (tid >= 1 && tid < T) {
        const float Mp = sM[sp[tid]];
        sex[tid] = (has_logit && Mp > -INFINITY) ? __builtin_amdgcn_exp2f((l_own - Mp) * p.k_log2) : 0.f;
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
    // This thread's 16 consecutive weights of chunk c of row `node`, the first nrem removed tokens zeroed.
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
    // Takes removed token r out of its chunk's mass (tokens 0..r are gone at that point).
    auto remove_from_chunks = [&](int node, int r) {
        const int xc = sremoved[r] / p.chunk_elems;
        const float old = sch[xc];
        float fresh = old - sremoved_ex[r];
        if (!(fresh >= 0.25f * old)) {
            // the subtraction cancelled most of the chunk: sum it again without the removed tokens
            float w[kPerThread];
            load_weights(node, xc, r + 1, w);
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < kPerThread; ++e) s += w[e];
            s = wave_sum(s);
            __syncthreads();
            if (lane == 0) sred[wave] = s;
            __syncthreads();
            fresh = (sred[0] + sred[1]) + (sred[2] + sred[3]);
        }
        __syncthreads(); // every thread has read the old value
        if (tid == 0) sch[xc] = fresh;
        __syncthreads();
    };
    // Per-chunk masses of row `node` with the first nrem removed tokens taken out; returns their sum.
    auto materialize = [&](int node, int nrem) -> float {
        const int64_t row = (int64_t)b * T + node;
        const float M = sM[node];
        __syncthreads();
        for (int c = tid; c < p.chunks; c += kWalkThreads) {
            const float mc = keep ? skeep_m[node * p.chunks + c] : p.part_m[row * p.chunks + c];
            const float sc = keep ? skeep_s[node * p.chunks + c] : p.part_s[row * p.chunks + c];
            sch[c] = (mc > -INFINITY) ? sc * __builtin_amdgcn_exp2f((mc - M) * p.k_log2) : 0.f;
        }
        __syncthreads();
        for (int r = 0; r < nrem; ++r) remove_from_chunks(node, r);
        return chunk_total();
    };

    // ---- the walk. Every wave runs it on registers: lane c holds node c's parent, draft token,
    // weight and uniform (T <= 64), the children of the current node are a ballot, and a child's
    // values are read with v_readlane - no LDS access and no dependent address per candidate
    // (a scan over LDS copies cost ~100 clocks per tree node and step). The removed tokens of
    // the current node sit one per lane for the duplicate check; LDS keeps the copy that the
    // chunk-wide passes read.
    const int32_t par_c = (lane < T) ? sp[lane] : -2;
    const int32_t x_c = (lane < T) ? sdraft[lane] : -1;
    const float ex_c = (lane >= 1 && lane < T) ? sex[lane] : 0.f;
    const float u_c = (lane < T) ? su[lane] : 2.f;
    int cur = 0, alen = 0, nrem = 0;
    float Z = 0.f;
    bool have_chunks = false;
    for (;;) {
        Z = sZ[cur];
        nrem = 0;
        have_chunks = false;
        int32_t rem_x = 0; // lane r < nrem: the r-th removed token
        int next = -1;
        uint64_t kids = __ballot(par_c == cur); // children in increasing node order
        while (kids != 0 && next < 0) {
            const int c = __builtin_ctzll(kids);
            kids &= kids - 1;
            const int32_t x = __builtin_amdgcn_readlane(x_c, c);
            bool gone = x < 0 || x >= p.V;
            gone = gone || __ballot(lane < nrem && rem_x == x) != 0;
            const float ex = gone ? 0.f : __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, ex_c), c));
            const float u = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, u_c), c));
            const float prob = (Z > 0.f) ? ex / Z : 0.f;
            if (u < prob) {
                next = c;
            } else if (!gone) {
                __syncthreads(); // every thread has read the list
                if (tid == 0) {
                    sremoved[nrem] = x;
                    sremoved_ex[nrem] = ex;
                }
                if (lane == nrem) rem_x = x;
                ++nrem;
                __syncthreads();
                if (have_chunks) {
                    remove_from_chunks(cur, nrem - 1);
                    Z = chunk_total();
                } else if (Z - ex >= 0.05f * Z) {
                    Z -= ex;
                } else {
                    Z = materialize(cur, nrem);
                    have_chunks = true;
                }
            }
        }
        if (next < 0) break;
        cur = next;
        ++alen;
    }
    if (!have_chunks) Z = materialize(cur, nrem);

    // ---- bonus token: inverse of the residual's cumulative sum, index order
    const float target = u_bonus * Z;
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
        // one LDS atomic per wave, not per thread (256 atomics on one address take microseconds)
        int wlast = last;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) wlast = max(wlast, __shfl_xor(wlast, o));
        if (lane == 0 && wlast >= 0) atomicMax(&slast, wlast);
        int cand = INT32_MAX;
        if (inc > local && last >= 0) {
            // first element of this thread whose running sum passes the target; the scan's and
            // the running sum's roundings may disagree by an ulp, then the last weighted one
            float acc = inc - s;
            cand = -1;
#pragma unroll
            for (int e = 0; e < kPerThread; ++e) {
                acc += w[e];
                if (cand < 0 && acc > local && w[e] > 0.f) cand = j0 + e;
            }
            if (cand < 0) cand = last;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) cand = min(cand, __shfl_xor(cand, o));
        if (lane == 0 && cand != INT32_MAX) atomicMin(&spick, cand);
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
    hipLaunchKernelGGL(softmax_stats_partial_kernel, dim3((unsigned)((int64_t)p.chunks * p.B * p.T)), dim3(kArgmaxBlock), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(accept_sample_walk_kernel, dim3(p.B), dim3(kWalkThreads), 0, s, p);
    return hipGetLastError();
}

} // namespace vs
