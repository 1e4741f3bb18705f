// Tree-masked attention without matrix cores: one wavefront per (sequence, node, query
// head). Serves fp32 storage and acts as the on-device cross-check of the MFMA kernel.
// Math: paper Eq. 1 with a softmax scale, restricted to the keys a node may see
// (all prefix tokens + the tree slots of its ancestor-or-self set, Section 3.1).
#include "vs_device.h"

namespace vs {

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_bits_to_float(*p); }
    static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = float_to_bf16_bits(v); }
};

__device__ __forceinline__ float wave_max(float v) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// grid = (T, Hq, B), block = 64. Lane j scores key j0 + j of each 64-key chunk; for the
// value product lane c owns channels c, c + 64, ...
template <typename TIn, int D>
__global__ __launch_bounds__(kWave) void attn_generic_kernel(const AttnParams p) {
    constexpr int CPL = D / kWave; // channels per lane
    __shared__ int32_t sp[VS_MAX_TREE];
    __shared__ int32_t sflag;
    __shared__ float sq[D];
    __shared__ float spj[kWave];
    __shared__ int64_t soff[kWave];

    const int node = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x;
    const int kvh = h / p.group;

    int32_t tree_code = VS_STATUS_OK;
    if (p.tree_keys == 0) {
        if (lane == 0) sflag = 0;
        __syncthreads();
    } else {
        tree_code = load_tree(p.parent + (int64_t)b * p.T, p.T, sp, &sflag);
    }
    const int32_t S = p.prefix_len[b];
    const bool s_ok = prefix_ok(p, S);
    if (node == 0 && h == 0) report_status(p, b, tree_code, s_ok, S, &sflag);
    if (tree_code != VS_STATUS_OK || !s_ok) return;

    const uint64_t mask = p.tree_keys == 0 ? 0ull : (p.tree_mask ? p.tree_mask[(int64_t)b * p.T + node] : ancestor_mask(sp, node));
    const TIn* q = (const TIn*)p.q + (((int64_t)b * p.T + node) * p.Hq + h) * D;
    for (int c = lane; c < D; c += kWave) sq[c] = Elem<TIn>::load(q + c);
    __syncthreads();

    const TIn* kbase = (const TIn*)p.k;
    const TIn* vbase = (const TIn*)p.v;
    const int n = S + p.tree_keys;
    float m = -INFINITY, l = 0.f;
    float acc[CPL];
#pragma unroll
    for (int i = 0; i < CPL; ++i) acc[i] = 0.f;

    for (int j0 = 0; j0 < n; j0 += kWave) {
        const int j = j0 + lane;
        bool vis = false;
        int64_t off = 0;
        float s = -INFINITY;
        if (j < n) {
            vis = (j < S) || ((mask >> (j - S)) & 1ull);
            if (vis) {
                off = token_offset(p, b, kvh, j);
                const TIn* kr = kbase + off;
                float dot = 0.f;
#pragma unroll 8
                for (int c = 0; c < D; ++c) dot = fmaf(sq[c], Elem<TIn>::load(kr + c), dot);
                s = dot * p.scale;
            }
        }
        const float cm = wave_max(s);
        const float m_new = fmaxf(m, cm);
        float pj = 0.f, alpha = 1.f;
        if (m_new > -INFINITY) {
            pj = vis ? expf(s - m_new) : 0.f;
            alpha = expf(m - m_new); // m = -inf → 0
        }
        l = l * alpha + wave_sum(pj);
        m = m_new;
#pragma unroll
        for (int i = 0; i < CPL; ++i) acc[i] *= alpha;
        __syncthreads();
        spj[lane] = pj;
        soff[lane] = off;
        __syncthreads();
        const int cnt = min(kWave, n - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float w = spj[jj];
            if (w != 0.f) { // invisible keys are skipped, never multiplied
                const TIn* vr = vbase + soff[jj];
#pragma unroll
                for (int i = 0; i < CPL; ++i) acc[i] = fmaf(w, Elem<TIn>::load(vr + lane + i * kWave), acc[i]);
            }
        }
    }
    TIn* o = (TIn*)p.out + (((int64_t)b * p.T + node) * p.Hq + h) * D;
    const float inv = 1.f / l;
#pragma unroll
    for (int i = 0; i < CPL; ++i) Elem<TIn>::store(o + lane + i * kWave, acc[i] * inv);
}

hipError_t launch_attention_generic(const AttnParams& p, int dtype, hipStream_t s) {
    dim3 grid(p.T, p.Hq, p.B), block(kWave);
    if (dtype == VS_BF16) {
        if (p.d == 64) hipLaunchKernelGGL((attn_generic_kernel<uint16_t, 64>), grid, block, 0, s, p);
        else hipLaunchKernelGGL((attn_generic_kernel<uint16_t, 128>), grid, block, 0, s, p);
    } else {
        if (p.d == 64) hipLaunchKernelGGL((attn_generic_kernel<float, 64>), grid, block, 0, s, p);
        else hipLaunchKernelGGL((attn_generic_kernel<float, 128>), grid, block, 0, s, p);
    }
    return hipGetLastError();
}

} // namespace vs
