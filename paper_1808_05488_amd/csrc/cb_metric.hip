// Quality metric of the threshold selection procedure (Sec. III-F): where no annotated frames
// exist, the change-based model's output is compared with the original model's.  Here: the sum of
// squared differences of two tensors, accumulated in float64 in a fixed order -- every workgroup
// owns a fixed slice, reduces it in a fixed tree, and one thread adds the workgroups' partial
// sums in index order -- so the result does not depend on scheduling.
#include <atomic>

#include "cb_kernels.h"

namespace cb {

namespace {

__device__ __forceinline__ double widen64(float v) { return (double)v; }
__device__ __forceinline__ double widen64(uint16_t v) { return (double)__uint_as_float((uint32_t)v << 16); }

template <typename T>
__global__ __launch_bounds__(256) void ssd_partial_kernel(const T* __restrict__ a, const T* __restrict__ b, size_t n,
                                                          double* __restrict__ partial)
{
    __shared__ double red[256];
    const size_t per = (n + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n ? lo + per : n;
    double s = 0.0;
    for (size_t i = lo + threadIdx.x; i < hi; i += 256) {
        const double d = widen64(a[i]) - widen64(b[i]);
        s += d * d;
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// acc[0] (+)= the partial sums, added in index order by one thread
__global__ void ssd_final_kernel(const double* __restrict__ partial, int np, double* __restrict__ acc, int accumulate)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double s = 0.0;
    for (int i = 0; i < np; ++i) s += partial[i];
    acc[0] = accumulate ? acc[0] + s : s;
}

// Scratch of the entry point that allocates nothing: SSD_PARTIALS partial sums and the total.  Every GPU
// the library runs on holds its own copy for the life of the process.  In host code the array's name
// is only a handle for hipGetSymbolAddress; kernels and copies get the address looked up below.
constexpr int kMaxDevices = 64;
__device__ __align__(256) double scratch[SSD_PARTIALS + 32];
std::atomic<double*> g_scratch_ptr[kMaxDevices];

}  // namespace

hipError_t ssd_static_scratch(double** partial, double** acc)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    double* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        // once per device, with that device current (two threads may both look it up: same answer)
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *partial = p;
    *acc = p + SSD_PARTIALS;
    return hipSuccess;
}

hipError_t launch_ssd(const void* a, const void* b, size_t n, int bf16, double* partial, double* acc, int accumulate,
                      hipStream_t st)
{
    const int np = SSD_PARTIALS;
    if (bf16)
        hipLaunchKernelGGL(ssd_partial_kernel<uint16_t>, dim3(np), dim3(256), 0, st, (const uint16_t*)a,
                           (const uint16_t*)b, n, partial);
    else
        hipLaunchKernelGGL(ssd_partial_kernel<float>, dim3(np), dim3(256), 0, st, (const float*)a, (const float*)b, n,
                           partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(ssd_final_kernel, dim3(1), dim3(64), 0, st, partial, np, acc, accumulate);
    return hipGetLastError();
}

}  // namespace cb
