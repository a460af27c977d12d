// Test helper (not part of the library): leaves every compute unit's LDS full of a given 32-bit pattern, so
// that a test can show that a kernel does not depend on what an earlier kernel left there.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
constexpr uint32_t kLdsBytes = 160u * 1024u;
__global__ __launch_bounds__(1024) void fill_kernel(uint32_t pattern, uint32_t* sink) {
    extern __shared__ uint32_t lds[];
    for (uint32_t i = threadIdx.x; i < kLdsBytes / 4u; i += blockDim.x) lds[i] = pattern;
    __syncthreads();
    // (read something back so that the stores are not dropped)
    if (threadIdx.x == 0 && lds[(blockIdx.x * 97u) % (kLdsBytes / 4u)] != pattern) sink[0] = 1u;
}
}  // namespace

extern "C" int lds_fill(uint32_t pattern, uint32_t* sink_dev, void* stream) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(fill_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
        return -1;
    // one workgroup fills a whole CU's LDS; several rounds so that every CU gets one
    hipLaunchKernelGGL(fill_kernel, dim3(2048), dim3(1024), kLdsBytes, static_cast<hipStream_t>(stream), pattern, sink_dev);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
