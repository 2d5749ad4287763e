// The analysis call for callers that cannot allocate (code under graph capture, tight serving loops,
// harnesses that forbid hipMalloc): crossquant_kernel_analysis needs two work vectors for the scale
// factors; here they live in a static device array instead of coming from the caller.
//
// `scratch` is a host-side stand-in for the array: its device address differs per device and is looked
// up once per device with hipGetSymbolAddress (with that device current); only that address is ever
// handed to a kernel.  Every call on a device shares the device's one array and the array keeps the last
// call's contents: the scale-finalize kernel overwrites the T + I entries the analysis kernel then
// reads, nothing has to start at zero, and calls that overlap on one device race on it.
#include <mutex>

#include "../../include/crossquant.h"
#include "cq_kernels.h"

namespace cq {

// a_i at [0, T), b_j at [CQ_ANALYSIS_STATIC_MAX, CQ_ANALYSIS_STATIC_MAX + I): 2 x 2^19 floats = 4 MiB per device
static __device__ __align__(256) float scratch[2 * CQ_ANALYSIS_STATIC_MAX];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_mu;
float* g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each device, once known

hipError_t scratch_address(float** ptr) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<float*>(p);
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

hipError_t launch_kernel_analysis_static(const uint16_t* X, int T, int I, int64_t ldx, const float* t, const float* c,
                                         float alpha, int qmax, uint16_t* xrk, unsigned long long* counters,
                                         hipStream_t stream) {
    if (T > CQ_ANALYSIS_STATIC_MAX || I > CQ_ANALYSIS_STATIC_MAX) return hipErrorInvalidValue;
    float* ws = nullptr;
    const hipError_t e = scratch_address(&ws);
    if (e != hipSuccess) return e;
    return launch_kernel_analysis(X, T, I, ldx, t, c, ws, ws + CQ_ANALYSIS_STATIC_MAX, alpha, qmax, xrk, counters, stream);
}

}  // namespace cq
