// A plain device-to-device copy with the access shape of the weight stream: every lane moves 16 bytes with
// a nontemporal load, a wavefront instruction covers 1 KiB of consecutive bytes.  It exists so that hardware
// counters (bytes fetched / written per dispatch) can be scaled by what they read for a transfer of exactly
// known size made of the same kind of memory requests.
#include "iflow_common.h"

namespace iflow {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void calibration_copy_kernel(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst, int64_t n16)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = __builtin_nontemporal_load(src + i);
}

// The same loads without the stores: what the memory system delivers to a kernel that only reads (the attainable
// ceiling of a weight stream).  Every lane folds its 16 bytes into one word and stores it only if it is a value that
// the data cannot produce in practice, so that the loads cannot be optimised away.
__global__ __launch_bounds__(256) void calibration_read_kernel(const u32x4_t *__restrict__ src, uint32_t *__restrict__ sink, int64_t n16)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) {
        const u32x4_t v = __builtin_nontemporal_load(src + i);
        const uint32_t f = v.x ^ (v.y * 3u) ^ (v.z * 5u) ^ (v.w * 7u);
        if (f == 0x9E3779B9u && (v.x & 0xFFFFu) == 0x1234u) sink[0] = f;
    }
}

hipError_t launch_calibration_read(const void *src, size_t bytes, void *sink, hipStream_t s)
{
    const int64_t n16 = (int64_t)(bytes / 16);
    const int64_t grid = (n16 + 255) / 256;
    if (grid > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(calibration_read_kernel, dim3((unsigned)grid), dim3(256), 0, s,
                       static_cast<const u32x4_t *>(src), static_cast<uint32_t *>(sink), n16);
    return hipGetLastError();
}

hipError_t launch_calibration_copy(const void *src, void *dst, size_t bytes, hipStream_t s)
{
    const int64_t n16 = (int64_t)(bytes / 16);
    const int64_t grid = (n16 + 255) / 256;
    if (grid > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3((unsigned)grid), dim3(256), 0, s,
                       static_cast<const u32x4_t *>(src), static_cast<u32x4_t *>(dst), n16);
    return hipGetLastError();
}

}  // namespace iflow
