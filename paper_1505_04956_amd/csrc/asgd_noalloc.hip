// Eq. 8 for callers that cannot allocate device memory: the partial sums of the reduction live in a static device
// array instead of a context's hipMalloc'ed scratch.  Same kernels as asgd_quant_error().
#include <mutex>

#include "asgd_internal.h"

using namespace asgd;

namespace {

constexpr int NOALLOC_MAX_PARTIALS = 2048;      // partial sums one call may use (16 KB per GPU, held until the process ends)

// Scratch of the reduction.  In host code this name is only a handle for the symbol, not a device address: the address
// on a given GPU comes from hipGetSymbolAddress(), once per device, and that pointer is what the kernels are given.
static __device__ __align__(256) double scratch[NOALLOC_MAX_PARTIALS];

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
double *g_scratch_ptr[MAX_DEVICES] = {nullptr};

// device address of `scratch` on the current device (looked up at the first call on that device)
hipError_t scratch_on_current_device(double **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<double *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" int asgd_quant_error_noalloc(const float *x_dev, int64_t N, int k, int d, const float *w_dev, double *out_dev,
                                        void *hip_stream)
{
    if (!x_dev || !w_dev || !out_dev || N < 1 || k < 1 || d < 1) return ASGD_EINVAL;
    // sizes beyond what the fixed scratch and the kernels' index arithmetic are laid out for
    if (N > ((int64_t)1 << 40) || d > 65536 || (double)k * d > (double)(1 << 24)) return ASGD_EINVAL;
    if (quant_partials_count() > NOALLOC_MAX_PARTIALS) return ASGD_EINVAL;
    if (((uintptr_t)x_dev & 7u) != 0 || ((uintptr_t)out_dev & 7u) != 0) return ASGD_EINVAL;
    double *partials = nullptr;
    if (scratch_on_current_device(&partials) != hipSuccess) return ASGD_EHIP;
    // every launch overwrites all the partial sums it reads afterwards: nothing has to start at zero
    hipError_t e = launch_quant_error(x_dev, N, d, k, w_dev, partials, out_dev, (hipStream_t)hip_stream);
    return e == hipSuccess ? ASGD_OK : ASGD_EHIP;
}
