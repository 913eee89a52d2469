// The copy kernel of libmaddness_calib.so (see stream_copy.h): bandwidth calibration only.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stream_copy.h"

namespace {

typedef unsigned copy_v4 __attribute__((ext_vector_type(4)));

// Plain streaming copy, 4 x 16 bytes per thread and iteration, non-temporal.
__global__ __launch_bounds__(256) void copy_kernel(const copy_v4 *__restrict__ src,
                                                   copy_v4 *__restrict__ dst, size_t n16)
{
    size_t base = (size_t)blockIdx.x * 1024;
    const size_t stride = (size_t)gridDim.x * 1024;
    for (; base < n16; base += stride) {
        copy_v4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const size_t i = base + u * 256 + threadIdx.x;
            if (i < n16) v[u] = __builtin_nontemporal_load(&src[i]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const size_t i = base + u * 256 + threadIdx.x;
            if (i < n16) __builtin_nontemporal_store(v[u], &dst[i]);
        }
    }
}

}  // namespace

extern "C" int calib_stream_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst) return -1;
    if (bytes % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0 || reinterpret_cast<uintptr_t>(dst) % 16 != 0)
        return -3;
    const size_t n16 = bytes / 16;
    if (n16 == 0) return 0;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        cus = 256;
    size_t blocks = (n16 + 1023) / 1024;
    if (blocks > (size_t)cus * 4) blocks = (size_t)cus * 4;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const copy_v4 *>(src), static_cast<copy_v4 *>(dst), n16);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
