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
constexpr int kExpandThreads = 1024;

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
constexpr int kCandCap = 128;        // entries of a wave's candidate list in LDS

// Larger float -> larger key (no NaN); every real key is > 0, which stands for "no entry".
__device__ __forceinline__ uint32_t order_key(float v) {
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// The first K of a wave's entries in (value descending, index ascending); every lane passes NE
// entries (index kNone = none). emit(rank, value, index) is called once per rank 0..K-1 by
// some lane; ranks past the number of entries get (-inf, kNone).
// How: the K-th largest of the lanes' own maxima (found bit by bit with ballots) is a lower
// bound of the K-th largest entry, so the entries at or above it are a small superset of the
// answer; they are compacted into the wave's LDS list and ranked by counting. A plateau of
// equal values or a nearly empty wave can overflow the list: then the entries are extracted
// one by one instead. No workgroup barrier inside; cv / ci are private to the wave.
template <int NE, typename Emit>
__device__ __forceinline__ void wave_topk(const float (&v)[NE], const int32_t (&i)[NE], int K, float* cv,
                                          int32_t* ci, Emit emit) {
    const int lane = threadIdx.x & 63;
    uint32_t best = 0;
#pragma unroll
    for (int e = 0; e < NE; ++e)
        if (i[e] != kNone) best = max(best, order_key(v[e]));
    uint32_t res = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t trial = res | (1u << bit);
        if (__popcll(__ballot(best >= trial)) >= K) res = trial;
    }
    const float tau = res ? key_value(res) : -INFINITY; // res == 0: fewer than K lanes hold entries
    int n = 0;
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        const bool pred = i[e] != kNone && v[e] >= tau;
        const uint64_t mask = __ballot(pred);
        const int pos = n + __popcll(mask & ((1ull << lane) - 1ull));
        if (pred && pos < kCandCap) {
            cv[pos] = v[e];
            ci[pos] = i[e];
        }
        n += __popcll(mask);
    }
    if (n <= kCandCap) {
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup"); // the list is read by other lanes of this wave
        for (int t = lane; t < n; t += kWave) {
            const float tv = cv[t];
            const int32_t ti = ci[t];
            int rank = 0;
            for (int o = 0; o < n; ++o) rank += before(cv[o], ci[o], tv, ti) ? 1 : 0;
            if (rank < K) emit(rank, tv, ti);
        }
        for (int r = n + lane; r < K; r += kWave) emit(r, -INFINITY, kNone);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup"); // reads done before the list is reused
    } else {
        float last_v = INFINITY;
        int32_t last_i = -1;
        for (int r = 0; r < K; ++r) {
            Ent mine = {-INFINITY, kNone};
#pragma unroll
            for (int e = 0; e < NE; ++e)
                if (i[e] != kNone && before(last_v, last_i, v[e], i[e]) && before(v[e], i[e], mine.v, mine.i))
                    mine = {v[e], i[e]};
            const Ent w = wave_first(mine);
            if (lane == 0) emit(r, w.v, w.i);
            last_v = w.v;
            last_i = w.i;
        }
    }
}

// grid = (chunks, B*F), block = 256.
__global__ __launch_bounds__(kArgmaxBlock) void draft_topk_partial_kernel(const DraftExpandParams p) {
    __shared__ float sv[kArgmaxBlock / kWave];
    __shared__ float ss[kArgmaxBlock / kWave];
    __shared__ float s_cv[(kArgmaxBlock / kWave) * kCandCap];
    __shared__ int32_t s_ci[(kArgmaxBlock / kWave) * kCandCap];
    __shared__ float s_wv[(kArgmaxBlock / kWave) * kMaxDraftK];
    __shared__ int32_t s_wi[(kArgmaxBlock / kWave) * kMaxDraftK];
    // one-dimensional grid: workgroup id = row * chunks + chunk (the host keeps the product below 2^31)
    const int64_t row = blockIdx.x / (uint32_t)p.chunks;
    const int chunk = (int)(blockIdx.x - (uint32_t)row * (uint32_t)p.chunks);
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

    // ---- the chunk's K first entries in (value descending, index ascending): per wave, then merged
    {
        float ev[4 * kVec + 1];
        int32_t ei[4 * kVec + 1];
#pragma unroll
        for (int j = 0; j < kVec; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ev[4 * j + e] = a[4 * j + e];
                ei[4 * j + e] = valid(j, e) ? base_idx[j] + e : kNone;
            }
        ev[4 * kVec] = tail_v;
        ei[4 * kVec] = tail_i;
        const int K = p.K;
        wave_topk(ev, ei, K, s_cv + wave * kCandCap, s_ci + wave * kCandCap, [&](int r, float v, int32_t i) {
            s_wv[wave * kMaxDraftK + r] = v;
            s_wi[wave * kMaxDraftK + r] = i;
        });
        __syncthreads();
        if (wave == 0) {
            constexpr int kWaves = kArgmaxBlock / kWave;
            float mv[1];
            int32_t mi[1];
            const int w = lane / K, r = lane - w * K; // lane < kWaves * K <= 64 holds wave w's r-th entry
            const bool has = lane < kWaves * K;
            mv[0] = has ? s_wv[w * kMaxDraftK + r] : -INFINITY;
            mi[0] = has ? s_wi[w * kMaxDraftK + r] : kNone;
            float* out_v = p.part_tv + (row * p.chunks + chunk) * K;
            int32_t* out_i = p.part_ti + (row * p.chunks + chunk) * K;
            wave_topk(mv, mi, K, s_cv, s_ci, [&](int rr, float v, int32_t i) {
                out_v[rr] = v;
                out_i[rr] = i; // kNone when the chunk has fewer than rr+1 entries
            });
        }
    }
}

// grid = B, block = 1024: one wave per frontier row (rows beyond sixteen take turns).
__global__ __launch_bounds__(kExpandThreads) void draft_expand_select_kernel(const DraftExpandParams p) {
    __shared__ float s_score[kMaxDraftCand];
    __shared__ int32_t s_token[kMaxDraftCand];
    __shared__ uint8_t s_keep[kMaxDraftCand];
    __shared__ float s_cv[(kExpandThreads / kWave) * kCandCap];
    __shared__ int32_t s_ci[(kExpandThreads / kWave) * kCandCap];
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int F = p.F, K = p.K, C = F * K;
    const int keep = min(K, C);
    // candidate tid's parent (the frontier row it extends): requested now, written out at the end
    // (C <= kMaxDraftCand = the block size, so a thread owns at most one candidate)
    const int32_t par_own = (tid < C && p.frontier_cand) ? p.frontier_cand[(int64_t)b * F + tid / K] : -1;

    // ---- per row: log-sum-exp and the K first entries of the merged chunk lists
    for (int f = wave; f < F; f += kExpandThreads / kWave) {
        const int64_t row = (int64_t)b * F + f;
        const float* pm = p.part_m + row * p.chunks;
        const float* ps = p.part_s + row * p.chunks;
        const float* tv = p.part_tv + row * p.chunks * K;
        const int32_t* ti = p.part_ti + row * p.chunks * K;
        const int n = p.chunks * K;
        // everything the row needs is requested before anything is used: chunk statistics (the first
        // 64 chunks; a longer row loops below), the chunk lists when they fit in registers, the score
        constexpr int kRegEnt = 8;
        const bool in_regs = n <= kWave * kRegEnt;
        float m0 = (lane < p.chunks) ? pm[lane] : -INFINITY;
        float s0 = (lane < p.chunks) ? ps[lane] : 0.f;
        float rv[kRegEnt];
        int32_t ri[kRegEnt];
#pragma unroll
        for (int q = 0; q < kRegEnt; ++q) {
            const int e = lane + q * kWave;
            rv[q] = (in_regs && e < n) ? tv[e] : -INFINITY;
            ri[q] = (in_regs && e < n) ? ti[e] : kNone;
        }
        const float cum = p.cum_in ? p.cum_in[row] : 0.f;
        float m = m0;
        for (int c = lane + kWave; c < p.chunks; c += kWave) m = fmaxf(m, pm[c]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
        float z = (m0 > -INFINITY) ? s0 * __builtin_amdgcn_exp2f((m0 - m) * 1.4426950408889634f) : 0.f;
        for (int c = lane + kWave; c < p.chunks; c += kWave) {
            const float mc = pm[c];
            if (mc > -INFINITY) z += ps[c] * __builtin_amdgcn_exp2f((mc - m) * 1.4426950408889634f);
        }
        z = wave_sum(z);
        const float lse = m + __logf(z);
        auto emit = [&](int r, float v, int32_t i) {
            s_token[f * K + r] = i;
            s_score[f * K + r] = cum + (v - lse);
        };
        if (in_regs) {
            wave_topk(rv, ri, K, s_cv + wave * kCandCap, s_ci + wave * kCandCap, emit);
        } else { // very long rows: the lists are re-read from the workspace (L2) for every extracted entry
            float last_v = INFINITY;
            int32_t last_i = -1;
            for (int r = 0; r < K; ++r) {
                Ent mine = {-INFINITY, kNone};
                for (int q = lane; q < n; q += kWave) {
                    const float v = tv[q];
                    const int32_t i = ti[q];
                    if (i != kNone && before(last_v, last_i, v, i) && before(v, i, mine.v, mine.i)) mine = {v, i};
                }
                const Ent w = wave_first(mine);
                if (lane == 0) emit(r, w.v, w.i);
                last_v = w.v;
                last_i = w.i;
            }
        }
    }
    __syncthreads();

    // ---- next frontier: the `keep` first candidates in (score descending, index ascending), by counting
    if (C <= kWave) {
        // one wave, registers only: lane c holds candidate c, the others' scores come by v_readlane,
        // the position among the kept ones is a population count of a ballot
        if (wave != 0) return;
        const float sc = (lane < C) ? s_score[lane] : -INFINITY;
        int rank = 0;
        for (int o = 0; o < C; ++o) {
            const float so = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, sc), o));
            rank += before(so, o, sc, lane) ? 1 : 0;
        }
        const bool kept = lane < C && rank < keep;
        const uint64_t kept_mask = __ballot(kept);
        if (lane < C) {
            const int64_t g = (int64_t)b * p.cand_capacity + p.cand_base + lane;
            p.cand_token[g] = s_token[lane];
            p.cand_score[g] = sc;
            p.cand_parent[g] = par_own;
            const int pos = __builtin_popcountll(kept_mask & ((1ull << lane) - 1ull));
            if (kept && pos < keep) { // pos >= keep: only NaN scores can rank more than `keep` candidates first
                p.next_frontier_cand[(int64_t)b * keep + pos] = p.cand_base + lane;
                p.next_cum[(int64_t)b * keep + pos] = sc;
            }
        }
        return;
    }
    for (int c = tid; c < C; c += kExpandThreads) {
        const float sc = s_score[c];
        int rank = 0;
        for (int o = 0; o < C; ++o) rank += before(s_score[o], o, sc, c) ? 1 : 0;
        s_keep[c] = rank < keep ? 1 : 0;
    }
    __syncthreads();
    for (int c = tid; c < C; c += kExpandThreads) {
        const int64_t g = (int64_t)b * p.cand_capacity + p.cand_base + c;
        p.cand_token[g] = s_token[c];
        p.cand_score[g] = s_score[c];
        p.cand_parent[g] = par_own;
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
    constexpr int kWords = kMaxDraftTotal / 64;
    __shared__ __attribute__((aligned(16))) float s_score[kMaxDraftTotal + 4];
    __shared__ int32_t s_parent[kMaxDraftTotal];
    __shared__ uint64_t s_mask[kWords];   // picked candidates, one bit each
    __shared__ int32_t s_before[kWords];  // picked candidates below word w
    __shared__ int32_t s_bad;
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int M = p.M, N = p.N;
    const int take = min(N, M);
    const int32_t* tok = p.cand_token + (int64_t)b * p.cand_capacity;
    const float* score = p.cand_score + (int64_t)b * p.cand_capacity;
    const int32_t* par = p.cand_parent + (int64_t)b * p.cand_capacity;
    const int rounds = (M + kSelThreads - 1) / kSelThreads; // every thread runs all rounds: the ballots need whole waves
    if (tid == 0) s_bad = 0;
    __syncthreads();
    if (tid < ((M + 3) & ~3) - M) s_score[M + tid] = -INFINITY; // padding of the last group of four
    for (int c = tid; c < M; c += kSelThreads) {
        s_score[c] = score[c];
        const int32_t pc = par[c];
        s_parent[c] = pc;
        if (pc < -1 || pc >= c) atomicOr(&s_bad, 1);
    }
    __syncthreads();
    // rank by counting (four scores per LDS read; a padding entry is -inf at an index >= M > c,
    // which comes before nothing), picked = rank < take, one bit per candidate
    const int M4 = (M + 3) & ~3;
    for (int r = 0; r < rounds; ++r) {
        const int c = r * kSelThreads + tid;
        bool pick = false;
        if (c < M) {
            const float sc = s_score[c];
            int rank = 0;
            for (int o = 0; o < M4; o += 4) {
                const f32x4 so = *(const f32x4*)&s_score[o];
#pragma unroll
                for (int e = 0; e < 4; ++e) rank += before(so[e], o + e, sc, c) ? 1 : 0;
            }
            pick = rank < take;
        }
        const uint64_t m = __ballot(pick);
        if (lane == 0) s_mask[c >> 6] = m;
    }
    __syncthreads();
    const int words = (M + 63) >> 6;
    if (tid == 0) {
        int acc = 0;
        for (int w = 0; w < words; ++w) {
            s_before[w] = acc;
            acc += __builtin_popcountll(s_mask[w]);
        }
    }
    auto picked = [&](int c) { return (s_mask[c >> 6] >> (c & 63)) & 1ull; };
    if (!s_bad) {
        for (int c = tid; c < M; c += kSelThreads)
            if (picked(c) && s_parent[c] >= 0 && !picked(s_parent[c])) atomicOr(&s_bad, 1);
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
    // node id = 1 + number of picked candidates with a smaller index
    auto node_of = [&](int c) { return 1 + s_before[c >> 6] + __builtin_popcountll(s_mask[c >> 6] & ((1ull << (c & 63)) - 1ull)); };
    for (int c = tid; c < M; c += kSelThreads) {
        if (!picked(c)) continue;
        const int node = node_of(c);
        if (node > take) continue; // only NaN scores can rank more than `take` candidates first
        const int32_t pc = s_parent[c];
        o_parent[node] = pc >= 0 ? node_of(pc) : 0;
        o_tokens[node] = tok[c];
        o_cand[node] = c;
    }
}

} // namespace

hipError_t launch_draft_expand(const DraftExpandParams& p, hipStream_t s) {
    hipLaunchKernelGGL(draft_topk_partial_kernel, dim3((unsigned)((int64_t)p.chunks * p.B * p.F)), dim3(kArgmaxBlock), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(draft_expand_select_kernel, dim3(p.B), dim3(kExpandThreads), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_draft_tree_build(const DraftBuildParams& p, hipStream_t s) {
    hipLaunchKernelGGL(draft_tree_build_kernel, dim3(p.B), dim3(kSelThreads), 0, s, p);
    return hipGetLastError();
}

} // namespace vs
