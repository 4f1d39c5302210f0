// Calibration kernels for the benchmark (not part of the method): what this GPU sustains on a plain
// streaming copy and on a loop of nothing but bf16 MFMAs, measured in the same run as the path itself so
// that roofline fractions can be quoted against achievable as well as published peaks.
#include "../../include/lsm_bench.h"
#include "lsm_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// dst[i] = src[i], 16 bytes per thread and step, grid-stride
__global__ __launch_bounds__(256) void k_calib_copy(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16) {
    const size_t stride = size_t(gridDim.x) * blockDim.x;
    for (size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Every wave issues `iters` rounds of four independent 32x32x16 bf16 MFMAs on operands that never leave
// its registers; the accumulators are summed into `out` at the end so that nothing is optimised away.
__global__ __launch_bounds__(256) void k_calib_mfma(float* __restrict__ out, int iters) {
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) {
        a[e] = __bf16(0.001f * float((lane + e) & 7));
        b[e] = __bf16(0.002f * float((lane * 3 + e) & 7));
    }
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
    for (int x = 0; x < 16; ++x) s += (c0[x] + c1[x]) + (c2[x] + c3[x]);
    out[size_t(blockIdx.x) * blockDim.x + threadIdx.x] = s;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
}  // namespace

extern "C" {

int lsm_calib_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src) return LSM_ERR_NULL;
    if (misaligned(dst) || misaligned(src)) return LSM_ERR_ALIGN;
    if (bytes == 0 || (bytes & 15u)) return LSM_ERR_SHAPE;
    hipLaunchKernelGGL(k_calib_copy, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<u32x4*>(dst),
                       static_cast<const u32x4*>(src), bytes / 16);
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_LAUNCH;
}

double lsm_calib_mfma_flops(int workgroups, int iters) {
    return double(workgroups) * 4.0 /* waves */ * double(iters) * 4.0 /* MFMAs */ * 2.0 * 32 * 32 * 16;
}

int lsm_calib_mfma(float* out, int workgroups, int iters, void* stream) {
    if (!out) return LSM_ERR_NULL;
    if (misaligned(out)) return LSM_ERR_ALIGN;
    if (workgroups < 1 || workgroups > 65535 || iters < 1) return LSM_ERR_SHAPE;
    hipLaunchKernelGGL(k_calib_mfma, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), out, iters);
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_LAUNCH;
}

}  // extern "C"
