// Greedy acceptance over a draft tree (paper Section 3.1 at temperature 0): a draft token
// survives iff it equals the target's argmax at its parent; the deepest surviving node
// ends the accepted path and its own argmax is the bonus token.
//
// Two kernels: (1) a bandwidth-bound scan that reduces each logits row to per-chunk
// (max, first index) pairs, (2) one workgroup per sequence that finishes the row argmax
// and walks the tree.
#include <atomic>

#include "vs_device.h"

// Scratch of vs_tree_accept_noalloc: the per-(row, chunk) results that vs_tree_accept keeps in the
// caller's workspace. One copy per GPU, held until the process ends. In host code the array's
// name is only a handle for hipGetSymbolAddress: the device address is asked for once per device
// and everything that touches the memory uses that address.
constexpr size_t kNoallocScratchBytes = VS_ACCEPT_NOALLOC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];

namespace vs {

namespace {

constexpr int kVecPerThread = 4; // 16-byte loads per thread and chunk

struct Best {
    float v;
    int32_t i;
};

// Candidate (v, i) replaces the incumbent iff it is larger, or equal with a lower index.
// NaN candidates never win ('>' and '==' are false for NaN).
__device__ __forceinline__ void take(Best& b, float v, int32_t i) {
    if (v > b.v || (v == b.v && i < b.i)) {
        b.v = v;
        b.i = i;
    }
}

__device__ __forceinline__ Best wave_best(Best b) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(b.v, o);
        const int32_t oi = __shfl_xor(b.i, o);
        take(b, ov, oi);
    }
    return b;
}

// grid = B*T*chunks, block = 256. Writes one (value, index) pair per (row, chunk).
__global__ __launch_bounds__(kArgmaxBlock) void argmax_partial_kernel(const AcceptParams p) {
    __shared__ float sv[kArgmaxBlock / kWave];
    __shared__ int32_t si[kArgmaxBlock / kWave];
    // one-dimensional grid: workgroup id = row * chunks + chunk (the host keeps the product below 2^31)
    const int64_t row = blockIdx.x / (uint32_t)p.chunks;
    const int chunk = (int)(blockIdx.x - (uint32_t)row * (uint32_t)p.chunks);
    const float* __restrict__ lg = p.logits + row * p.ld;
    const int begin = chunk * p.chunk_elems;
    const int end = min(p.V, begin + p.chunk_elems);
    Best best = {-INFINITY, INT32_MAX};
    if (p.vec_ok) {
        // chunk_elems = 4 * kArgmaxBlock * kVecPerThread: every thread's loads are issued
        // before the first compare. The maximum is found on values alone (one v_max per
        // element); the index is recovered afterwards as the lowest position that equals the
        // wave's maximum. NaN never equals anything and never survives fmaxf, -0 == +0.
        const int nvec = (end - begin) >> 2;
        const f32x4* __restrict__ lv = (const f32x4*)(lg + begin);
        f32x4 a[kVecPerThread];
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j) {
            const int k = threadIdx.x + j * kArgmaxBlock;
            a[j] = (k < nvec) ? __builtin_nontemporal_load(lv + k) : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        }
        float m = -INFINITY;
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) m = fmaxf(m, a[j][e]);
        for (int t = begin + 4 * nvec + threadIdx.x; t < end; t += kArgmaxBlock) m = fmaxf(m, lg[t]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
        int32_t idx = INT32_MAX;
        for (int t = begin + 4 * nvec + threadIdx.x; t < end; t += kArgmaxBlock)
            if (lg[t] == m) idx = min(idx, t);
#pragma unroll
        for (int j = kVecPerThread - 1; j >= 0; --j) {
            const int k = threadIdx.x + j * kArgmaxBlock;
#pragma unroll
            for (int e = 3; e >= 0; --e)
                if (k < nvec && a[j][e] == m) idx = begin + 4 * k + e;
        }
        best.v = m;       // the wave's maximum; lanes without it keep INT32_MAX and lose the tie
        best.i = idx;
    } else {
        for (int t = begin + threadIdx.x; t < end; t += kArgmaxBlock) take(best, lg[t], t);
    }
    best = wave_best(best);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        sv[wave] = best.v;
        si[wave] = best.i;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kArgmaxBlock / kWave; ++w) take(best, sv[w], si[w]);
        p.part_val[row * p.chunks + chunk] = best.v;
        p.part_idx[row * p.chunks + chunk] = best.i;
    }
}

// grid = B, block = 256. Finishes the argmax of the sequence's T rows, then wave 0 walks
// the tree (one lane per node).
__global__ __launch_bounds__(256) void accept_walk_kernel(const AcceptParams p) {
    __shared__ int32_t sp[VS_MAX_TREE];
    __shared__ int32_t sflag;
    __shared__ int32_t samax[VS_MAX_TREE];
    __shared__ int32_t spath[VS_MAX_TREE];
    __shared__ int32_t sdraft[VS_MAX_TREE];
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = p.T;
    // four threads per row share the row's chunk results (T <= 64 rows, 256 threads). Nothing here
    // depends on the tree, so everything is requested before the tree is waited for (one memory
    // round trip instead of two): the row's first logit (NaN rule), the draft tokens, and sixteen
    // chunk results per thread (all of them for vocabularies up to 64 chunks).
    constexpr int kPre = 16;
    const int i = tid >> 2, sub = tid & 3;
    const int64_t row = (int64_t)b * T + i;
    const float* pv = p.part_val + row * p.chunks;
    const int32_t* pi = p.part_idx + row * p.chunks;
    float v[kPre];
    int32_t x[kPre];
    auto fetch = [&](int c0) {
#pragma unroll
        for (int q = 0; q < kPre; ++q) {
            const int c = c0 + 4 * q;
            const bool ok = i < T && c < p.chunks;
            v[q] = ok ? pv[c] : -INFINITY;
            x[q] = ok ? pi[c] : INT32_MAX;
        }
    };
    fetch(sub);
    const float first = (i < T && sub == 0) ? p.logits[row * p.ld] : 0.f;
    const int32_t draft_own = (tid < T) ? p.draft[(int64_t)b * T + tid] : -1;
    const int32_t tree_code = load_tree(p.parent + (int64_t)b * T, T, sp, &sflag);
    if (tid < T) sdraft[tid] = draft_own;
    {
        Best best = {-INFINITY, INT32_MAX};
        for (int c0 = sub; c0 < p.chunks; c0 += 4 * kPre) {
            if (c0 != sub) fetch(c0);
#pragma unroll
            for (int q = 0; q < kPre; ++q) take(best, v[q], x[q]);
        }
#pragma unroll
        for (int o = 1; o <= 2; o <<= 1) {
            const float ov = __shfl_xor(best.v, o);
            const int32_t oi = __shfl_xor(best.i, o);
            take(best, ov, oi);
        }
        if (i < T && sub == 0) {
            // what a left-to-right '>' scan returns: a NaN in column 0 is never displaced,
            // and a row with nothing above -inf keeps index 0
            int32_t idx = best.i;
            if (first != first || idx == INT32_MAX) idx = 0;
            samax[i] = idx;
            if (p.row_argmax) p.row_argmax[row] = idx;
        }
    }
    if (tid < T) spath[tid] = -1;
    __syncthreads();

    int32_t best_node = 0, alen = 0;
    if (wave == 0 && tree_code == VS_STATUS_OK) {
        int32_t key = -1;
        if (lane < T) {
            bool ok = true;
            int32_t dep = 0;
            int j = lane;
            while (j > 0) {
                const int pj = sp[j];
                ok = ok && (sdraft[j] == samax[pj]);
                j = pj;
                ++dep;
            }
            if (ok) key = dep * 64 + (63 - lane); // deepest first, then lowest index
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) key = max(key, __shfl_xor(key, o));
        best_node = 63 - (key & 63); // the root is always accepted, so key >= 63
        alen = key >> 6;
        if (lane == 0) {
            int j = best_node;
            for (int k = alen; k >= 0 && j >= 0; --k) {
                spath[k] = j;
                j = sp[j];
            }
        }
    }
    __syncthreads();
    if (tid < T) p.path[(int64_t)b * T + tid] = spath[tid];
    if (tid == 0) {
        if (p.status) p.status[b] = tree_code;
        const bool good = tree_code == VS_STATUS_OK;
        p.accepted_len[b] = good ? alen : 0;
        p.bonus[b] = good ? samax[best_node] : -1;
    }
}

constexpr int kMaxDevices = 64;
std::atomic<void*> scratch_of[kMaxDevices]; // device address of `scratch` on each device, null = not asked yet

// Device address of the current device's copy of `scratch`; asks the runtime on the first call
// per device. Returns null (and leaves no sticky error) when that fails.
void* scratch_address() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    void* ptr = scratch_of[dev].load(std::memory_order_acquire);
    if (ptr) return ptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
        (void)hipGetLastError();
        return nullptr;
    }
    scratch_of[dev].store(ptr, std::memory_order_release);
    return ptr;
}

} // namespace

hipError_t launch_accept(const AcceptParams& p, hipStream_t s) {
    hipLaunchKernelGGL(argmax_partial_kernel, dim3((unsigned)((int64_t)p.chunks * p.B * p.T)), dim3(kArgmaxBlock), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(accept_walk_kernel, dim3(p.B), dim3(256), 0, s, p);
    return hipGetLastError();
}

} // namespace vs

extern "C" int32_t vs_tree_accept_noalloc(const float* logits, int64_t ld_logits, int32_t V, const int32_t* draft_tokens,
                                          const int32_t* parent, int32_t B, int32_t T, int32_t* accepted_len,
                                          int32_t* path, int32_t* bonus_token, int32_t* row_argmax, int32_t* status,
                                          void* stream) {
    using namespace vs;
    if (!logits || !draft_tokens || !parent || !accepted_len || !path || !bonus_token) return VS_ERR_NULL;
    if (B < 1 || T < 1 || T > VS_MAX_TREE || V < 1 || ld_logits < V) return VS_ERR_SHAPE;
    const size_t need = vs_accept_workspace_bytes(B, T, V);
    if (need == 0 || need > kNoallocScratchBytes) return VS_ERR_WORKSPACE; // beyond the static scratch: use vs_tree_accept
    if (const int32_t dc = check_device()) return dc;
    unsigned char* ws = (unsigned char*)scratch_address();
    if (!ws) return VS_ERR_HIP;
    // same layout as vs_tree_accept's workspace: values, then (256-byte aligned) indices. Nothing
    // has to start at zero: the scan writes every pair the walk reads.
    const int32_t chunks = (V + kAcceptChunk - 1) / kAcceptChunk;
    const size_t n = (size_t)B * T * chunks;
    AcceptParams p{};
    p.logits = logits;
    p.ld = ld_logits;
    p.V = V;
    p.draft = draft_tokens;
    p.parent = parent;
    p.B = B;
    p.T = T;
    p.accepted_len = accepted_len;
    p.path = path;
    p.bonus = bonus_token;
    p.row_argmax = row_argmax;
    p.status = status;
    p.chunks = chunks;
    p.chunk_elems = kAcceptChunk;
    p.vec_ok = (((uintptr_t)logits & 15u) == 0 && ld_logits % 4 == 0) ? 1 : 0;
    p.part_val = (float*)ws;
    p.part_idx = (int32_t*)(ws + (n * sizeof(float) + 255) / 256 * 256);
    return launch_accept(p, (hipStream_t)stream) == hipSuccess ? VS_OK : VS_ERR_HIP;
}
