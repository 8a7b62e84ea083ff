// Plain streaming kernels of known size, measurement support for bench.py (not
// part of libfsdp_flat): a device-to-device copy, a read-only pass and a
// write-only pass over a buffer.  bench.py times them in the same run as the
// library's kernels (the achievable HBM ceilings of the box next to the
// published 8 TB/s), and `bench.py --probe-copy` runs the copy alone so that
// rocprofv3's FETCH_SIZE / WRITE_SIZE counters can be scaled by their reading
// for a kernel whose traffic is known.
#include <hip/hip_runtime.h>

#include <cstdint>

typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void fsdp_probe_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst,
                                                              int64_t nvec)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < nvec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Every 16-byte vector is loaded; the loads are kept alive by a store that no
// lane ever executes for the data bench.py passes (all bits zero).
__global__ __launch_bounds__(256) void fsdp_probe_read_kernel(const f32x4* __restrict__ src, int64_t nvec,
                                                              float* __restrict__ sink)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < nvec) {
        const f32x4 v = __builtin_nontemporal_load(src + i);
        if (__float_as_uint(v.x) == 0x7FC0FFEEu && __float_as_uint(v.y) == 0x7FC0FFEEu) *sink = v.z + v.w;
    }
}

__global__ __launch_bounds__(256) void fsdp_probe_write_kernel(f32x4* __restrict__ dst, int64_t nvec, float value)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < nvec) __builtin_nontemporal_store(f32x4{value, value, value, value}, dst + i);
}

namespace {
bool bad_buffer(const void* p, int64_t nbytes)
{
    return !p || nbytes <= 0 || (nbytes & 15) || (reinterpret_cast<uintptr_t>(p) & 15) || (nbytes / 16 + 255) / 256 > 0x7FFFFFFFLL;
}
}  // namespace

// dst, src: device, 16-byte aligned; nbytes: multiple of 16.  Each returns the hipError_t of its launch.
extern "C" int fsdp_probe_copy(void* dst, const void* src, int64_t nbytes, void* hip_stream)
{
    if (bad_buffer(dst, nbytes) || bad_buffer(src, nbytes)) return static_cast<int>(hipErrorInvalidValue);
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(fsdp_probe_copy_kernel, dim3(static_cast<uint32_t>((nvec + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const f32x4*>(src), static_cast<f32x4*>(dst),
                       nvec);
    return static_cast<int>(hipGetLastError());
}

// sink: device, one float (never written for zero-filled sources)
extern "C" int fsdp_probe_read(const void* src, int64_t nbytes, float* sink, void* hip_stream)
{
    if (bad_buffer(src, nbytes) || !sink) return static_cast<int>(hipErrorInvalidValue);
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(fsdp_probe_read_kernel, dim3(static_cast<uint32_t>((nvec + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const f32x4*>(src), nvec, sink);
    return static_cast<int>(hipGetLastError());
}

extern "C" int fsdp_probe_write(void* dst, int64_t nbytes, float value, void* hip_stream)
{
    if (bad_buffer(dst, nbytes)) return static_cast<int>(hipErrorInvalidValue);
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(fsdp_probe_write_kernel, dim3(static_cast<uint32_t>((nvec + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<f32x4*>(dst), nvec, value);
    return static_cast<int>(hipGetLastError());
}
