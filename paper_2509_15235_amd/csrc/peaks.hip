// Measurement helpers (not part of the method): three trivial kernels that show what this
// machine's memory system and matrix cores deliver, so that the roofline fractions reported
// for the attention and scan kernels can be read against measured peaks as well as against
// the data-sheet ones. Declared in include/vispec_peaks.h, timed by bench.py.
#include "vs_device.h"

#include "vispec_peaks.h"

namespace vs {

namespace {

constexpr int kPeakThreads = 256;

// Streaming read: every thread folds 16-byte pieces of `src` into one word; one word per
// workgroup leaves (so the loads cannot be dropped). `n16` pieces, grid-stride, four loads in
// flight per thread.
__global__ __launch_bounds__(kPeakThreads) void peak_read_kernel(const u32x4* __restrict__ src, int64_t n16,
                                                                uint32_t* __restrict__ sink) {
    const int64_t stride = (int64_t)gridDim.x * kPeakThreads;
    int64_t i = (int64_t)blockIdx.x * kPeakThreads + threadIdx.x;
    uint32_t acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride),
                    c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a[0] ^ a[1] ^ a[2] ^ a[3] ^ b[0] ^ b[1] ^ b[2] ^ b[3] ^ c[0] ^ c[1] ^ c[2] ^ c[3] ^ d[0] ^ d[1] ^ d[2] ^ d[3];
    }
    for (; i < n16; i += stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i);
        acc ^= a[0] ^ a[1] ^ a[2] ^ a[3];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
    if ((threadIdx.x & 63) == 0) atomicXor(sink + blockIdx.x, acc);
}

// Plain copy, 16 bytes per thread and step.
__global__ __launch_bounds__(kPeakThreads) void peak_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                                int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * kPeakThreads;
    for (int64_t i = (int64_t)blockIdx.x * kPeakThreads + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Matrix-core loop: every wave runs `iters` rounds of sixteen v_mfma_f32_32x32x16_bf16 on four
// independent accumulators (the dependency pattern of the attention kernels' P.V product) with
// operands taken from `operands` (8 bf16 per lane and operand, two operands per lane; what they
// hold - constants or noise - decides how much power the loop draws and hence its clock).
__global__ __launch_bounds__(512, 2) void peak_mfma_kernel(const u32x4* __restrict__ operands, int32_t iters,
                                                          float* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    const bf16x8 a = __builtin_bit_cast(bf16x8, operands[(threadIdx.x >> 6) * 128 + lane]);
    const bf16x8 b = __builtin_bit_cast(bf16x8, operands[(threadIdx.x >> 6) * 128 + 64 + lane]);
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) t += acc[j][r];
    sink[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = t;
}

} // namespace

} // namespace vs

extern "C" {

int32_t vs_peak_hbm_read(const void* src, size_t bytes, void* sink, int32_t workgroups, void* stream) {
    if (!src || !sink) return VS_ERR_NULL;
    if (bytes < 16 || workgroups < 1 || workgroups > VS_PEAK_MAX_WORKGROUPS || ((uintptr_t)src & 15u)) return VS_ERR_SHAPE;
    if (const int32_t dc = vs::check_device()) return dc;
    hipLaunchKernelGGL(vs::peak_read_kernel, dim3(workgroups), dim3(vs::kPeakThreads), 0, (hipStream_t)stream,
                       (const vs::u32x4*)src, (int64_t)(bytes / 16), (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? VS_OK : VS_ERR_HIP;
}

int32_t vs_peak_hbm_copy(void* dst, const void* src, size_t bytes, int32_t workgroups, void* stream) {
    if (!src || !dst) return VS_ERR_NULL;
    if (bytes < 16 || workgroups < 1 || workgroups > VS_PEAK_MAX_WORKGROUPS || (((uintptr_t)src | (uintptr_t)dst) & 15u))
        return VS_ERR_SHAPE;
    if (const int32_t dc = vs::check_device()) return dc;
    hipLaunchKernelGGL(vs::peak_copy_kernel, dim3(workgroups), dim3(vs::kPeakThreads), 0, (hipStream_t)stream,
                       (vs::u32x4*)dst, (const vs::u32x4*)src, (int64_t)(bytes / 16));
    return hipGetLastError() == hipSuccess ? VS_OK : VS_ERR_HIP;
}

int32_t vs_peak_mfma_bf16(const void* operands, int32_t iters, void* sink, int32_t workgroups, void* stream) {
    if (!operands || !sink) return VS_ERR_NULL;
    if (iters < 1 || workgroups < 1 || workgroups > VS_PEAK_MAX_WORKGROUPS || ((uintptr_t)operands & 15u)) return VS_ERR_SHAPE;
    if (const int32_t dc = vs::check_device()) return dc;
    hipLaunchKernelGGL(vs::peak_mfma_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)stream,
                       (const vs::u32x4*)operands, iters, (float*)sink);
    return hipGetLastError() == hipSuccess ? VS_OK : VS_ERR_HIP;
}

double vs_peak_mfma_flops(int32_t iters, int32_t workgroups) {
    // 8 waves per workgroup x iters x 16 instructions x (2 x 32 x 32 x 16) flops
    return 8.0 * (double)workgroups * (double)iters * 16.0 * 32768.0;
}

} // extern "C"
