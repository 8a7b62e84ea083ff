// Plain device-to-device copy kernel of known size, used only to calibrate
// rocprofv3's FETCH_SIZE / WRITE_SIZE counters (bench.py --probe-copy): the
// counters' reading for this kernel, divided by the bytes it is known to move,
// is the scale factor applied to the same counters of the library's kernels.
// Not part of libfsdp_flat.
#include <hip/hip_runtime.h>

#include <cstdint>

typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void fsdp_probe_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst,
                                                              int64_t nvec)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < nvec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// dst, src: device, 16-byte aligned; nbytes: multiple of 16.  Returns the hipError_t of the launch.
extern "C" int fsdp_probe_copy(void* dst, const void* src, int64_t nbytes, void* hip_stream)
{
    if (!dst || !src || nbytes <= 0 || (nbytes & 15) || (reinterpret_cast<uintptr_t>(dst) & 15) ||
        (reinterpret_cast<uintptr_t>(src) & 15))
        return static_cast<int>(hipErrorInvalidValue);
    const int64_t nvec = nbytes / 16;
    const int64_t blocks = (nvec + 255) / 256;
    if (blocks > 0x7FFFFFFFLL) return static_cast<int>(hipErrorInvalidValue);
    hipLaunchKernelGGL(fsdp_probe_copy_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const f32x4*>(src), static_cast<f32x4*>(dst),
                       nvec);
    return static_cast<int>(hipGetLastError());
}
