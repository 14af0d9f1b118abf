// Small HBM-bound kernels: SwiGLU gate, copies and fills.  16-byte accesses,
// grid-stride loops sized to a few waves per SIMD.
#include "sp_common.h"
#include "sp_kernels.h"

namespace {

constexpr int EW_THREADS = 256;

__global__ __launch_bounds__(EW_THREADS) void swiglu_kernel(const bf16_t* __restrict__ gu, bf16_t* __restrict__ z,
                                                            int T, int f) {
    const int fc = f >> 3;                       // 8-element chunks per row
    const size_t total = (size_t)T * fc;
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < total; i += (size_t)gridDim.x * EW_THREADS) {
        const size_t t = i / fc;
        const int c = (int)(i - t * fc);
        const u32x4_t g = *reinterpret_cast<const u32x4_t*>(gu + t * 2 * (size_t)f + c * 8);
        const u32x4_t u = *reinterpret_cast<const u32x4_t*>(gu + t * 2 * (size_t)f + f + c * 8);
        u32x4_t r;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float g0 = bf_lo(g[k]), g1 = bf_hi(g[k]);
            const float z0 = g0 / (1.0f + __expf(-g0)) * bf_lo(u[k]);
            const float z1 = g1 / (1.0f + __expf(-g1)) * bf_hi(u[k]);
            r[k] = pack_bf2(z0, z1);
        }
        *reinterpret_cast<u32x4_t*>(z + t * (size_t)f + c * 8) = r;
    }
}

__global__ __launch_bounds__(EW_THREADS) void copy_f32_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                              size_t n4, const float* src_tail, float* dst_tail, int tail) {
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n4; i += (size_t)gridDim.x * EW_THREADS)
        dst[i] = src[i];
    if (blockIdx.x == 0 && (int)threadIdx.x < tail) dst_tail[threadIdx.x] = src_tail[threadIdx.x];
}

__global__ __launch_bounds__(EW_THREADS) void fill_u32_kernel(uint32_t* __restrict__ dst, uint32_t v, size_t n) {
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += (size_t)gridDim.x * EW_THREADS)
        dst[i] = v;
}

// One wave that idles for a bounded number of sleep instructions and exits: a delay on a
// stream (debug mode).  s_sleep 64 parks the wave for 64 x 64 clocks, about 2 us.
__global__ __launch_bounds__(64) void spin_kernel(int iters) {
    for (int i = 0; i < iters; ++i) __builtin_amdgcn_s_sleep(64);
}

inline int ew_grid(size_t items) {
    size_t g = (items + EW_THREADS - 1) / EW_THREADS;
    const size_t cap = 256 * 16;  // 16 work-groups per CU
    return (int)(g < 1 ? 1 : (g > cap ? cap : g));
}

}  // namespace

hipError_t spk_launch_swiglu(hipStream_t st, const bf16_t* gu, bf16_t* z, int T, int f) {
    if (T <= 0) return hipSuccess;
    if (f <= 0 || (f & 7) || (((uintptr_t)gu | (uintptr_t)z) & 15)) return hipErrorInvalidValue;
    swiglu_kernel<<<ew_grid((size_t)T * (f >> 3)), EW_THREADS, 0, st>>>(gu, z, T, f);
    return hipGetLastError();
}

hipError_t spk_launch_copy_f32(hipStream_t st, const float* src, float* dst, size_t n) {
    if (n == 0 || src == dst) return hipSuccess;
    if (((uintptr_t)src | (uintptr_t)dst) & 15) return hipErrorInvalidValue;
    const size_t n4 = n >> 2;
    copy_f32_kernel<<<ew_grid(n4), EW_THREADS, 0, st>>>(reinterpret_cast<const float4*>(src),
                                                       reinterpret_cast<float4*>(dst), n4, src + n4 * 4,
                                                       dst + n4 * 4, (int)(n & 3));
    return hipGetLastError();
}

hipError_t spk_launch_fill_u32(hipStream_t st, uint32_t* dst, uint32_t v, size_t n) {
    if (n == 0) return hipSuccess;
    fill_u32_kernel<<<ew_grid(n), EW_THREADS, 0, st>>>(dst, v, n);
    return hipGetLastError();
}

hipError_t spk_launch_spin(hipStream_t st, int micros) {
    if (micros <= 0) return hipSuccess;
    const int iters = std::min(micros, SPK_SPIN_MAX_US) / 2 + 1;     // bounded: the kernel always ends
    spin_kernel<<<1, 64, 0, st>>>(iters);
    return hipGetLastError();
}
