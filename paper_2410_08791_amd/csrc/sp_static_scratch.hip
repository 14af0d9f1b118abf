// spk_rmsnorm_bwd_static: the RMSNorm backward of spk_rmsnorm_bwd for callers that cannot
// allocate device memory (code under graph capture, serving loops, harnesses that forbid
// hipMalloc).  The partial rows of the gain-gradient reduction, which spk_rmsnorm_bwd takes as a
// caller-provided buffer, live in a file-scope device array here; the kernels are the same and
// receive the array's device address as an argument.
#include <mutex>

#include "../../include/superpipe.h"
#include "../../include/superpipe_kernels.h"
#include "sp_kernels.h"

namespace {

constexpr int kStaticMaxD = SPK_STATIC_MAX_D;
// SPK_NORM_BWD_BLOCKS partial rows of at most kStaticMaxD floats: 4 MiB per device, held until
// the process ends.
static __device__ __align__(256) float scratch[(size_t)SPK_NORM_BWD_BLOCKS * kStaticMaxD];

// The array's name is a host-side stand-in, not a device address: each device holds its own
// copy at its own address, looked up once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_mu;
float* g_scratch_ptr[kMaxDevices] = {};

int scratch_for_current_device(float** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return SP_ERR_HIP;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return SP_ERR_HIP;
        }
        g_scratch_ptr[dev] = static_cast<float*>(p);
    }
    *out = g_scratch_ptr[dev];
    return SP_OK;
}

}  // namespace

extern "C" int spk_rmsnorm_bwd_static_max_d(void) { return kStaticMaxD; }

extern "C" int spk_rmsnorm_bwd_static(void* stream, const float* da, const float* h, const uint16_t* gain,
                                      float* dh_io, uint16_t* dhb, float* dgain, int T, int d, float eps) {
    if (!da || !h || !gain || !dh_io || !dhb || !dgain || T < 0) return SP_ERR_INVALID_ARG;
    if (d <= 0 || (d & 3) || d > kStaticMaxD) return SP_ERR_SHAPE;   // beyond what the static array holds
    float* part = nullptr;
    int rc = scratch_for_current_device(&part);
    if (rc != SP_OK) return rc;
    // Nothing in the array has to start at zero: every block of the first kernel writes its whole
    // partial row, and the second kernel reads exactly the rows this call wrote.
    hipError_t e = spk_launch_rmsnorm_bwd((hipStream_t)stream, da, h, gain, dh_io, dhb, part, dgain, T, d, eps);
    if (e == hipSuccess) return SP_OK;
    (void)hipGetLastError();
    return e == hipErrorInvalidValue ? SP_ERR_INVALID_ARG : SP_ERR_HIP;
}
