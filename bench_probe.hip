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
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < nvec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Every 16-byte vector is loaded; the loads are kept alive by a store that no
// lane ever executes for the data bench.py passes (all bits zero).
__global__ __launch_bounds__(256) void fsdp_probe_read_kernel(const f32x4* __restrict__ src, int64_t nvec,
                                                              float* __restrict__ sink)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < nvec) {
        const f32x4 v = __builtin_nontemporal_load(src + i);
        if (__float_as_uint(v.x) == 0x7FC0FFEEu && __float_as_uint(v.y) == 0x7FC0FFEEu) *sink = v.z + v.w;
    }
}

__global__ __launch_bounds__(256) void fsdp_probe_write_kernel(f32x4* __restrict__ dst, int64_t nvec, float value)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < nvec) __builtin_nontemporal_store(f32x4{value, value, value, value}, dst + i);
}

// The unshard's traffic from one flat array: every lane loads 16 bytes (four floats) and stores 8 bytes (their
// upper halves, a truncating stand-in for the cast), both contiguous across the wave.
typedef uint32_t u32x2p __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4p __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void fsdp_probe_cast_kernel(const u32x4p* __restrict__ src, u32x2p* __restrict__ dst,
                                                              int64_t nvec)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < nvec) {
        const u32x4p x = __builtin_nontemporal_load(src + i);
        __builtin_nontemporal_store(u32x2p{(x.x >> 16) | (x.y & 0xFFFF0000u), (x.z >> 16) | (x.w & 0xFFFF0000u)}, dst + i);
    }
}

// The rank walk's memory traffic with almost no arithmetic around it: every
// lane reads 16 bytes (8 bf16) at the same offset of each of n streams, in
// order, sums them in fp32, and (store != 0) writes its 8 sums as fp32, or
// (store == 0) nothing.  bench.py --probe-mix times the forms: what the same
// reads cost with and without the small write stream next to them, and what the
// shape of the stores does to it.
struct ProbeStreams {
    const uint32_t* p[64];
};
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void fsdp_probe_streams_kernel(ProbeStreams t, int n, int64_t nvec, int store,
                                                                 float* __restrict__ out)
{
    const int64_t c = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (c >= nvec) return;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = -0.0f;
    for (int w = 0; w < n; ++w) {
        const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t.p[w]) + c);
        acc[0] += __uint_as_float(x.x << 16); acc[1] += __uint_as_float(x.x & 0xFFFF0000u);
        acc[2] += __uint_as_float(x.y << 16); acc[3] += __uint_as_float(x.y & 0xFFFF0000u);
        acc[4] += __uint_as_float(x.z << 16); acc[5] += __uint_as_float(x.z & 0xFFFF0000u);
        acc[6] += __uint_as_float(x.w << 16); acc[7] += __uint_as_float(x.w & 0xFFFF0000u);
    }
    // Without the store the sums are kept alive by a comparison that zero-filled streams never satisfy.
    // store == 1: each of the two store instructions is contiguous across the wave (the lane's two vectors
    // land 256 vectors apart inside the workgroup's 8 KiB of output; only the traffic matters here);
    // store == 2: the lane's 32 bytes side by side, so that each store instruction covers every other 16
    // bytes of its span: the pattern that nontemporal stores handle badly.
    if (store != 0 || acc[0] == 12345.678f) {
        f32x4* o = reinterpret_cast<f32x4*>(out) + static_cast<int64_t>(blockIdx.x) * 512;
        const bool side_by_side = store == 2 || (static_cast<int64_t>(blockIdx.x) + 1) * 256 > nvec;   // or a partial block
        const int first = side_by_side ? 2 * threadIdx.x : threadIdx.x;
        const int second = side_by_side ? 2 * threadIdx.x + 1 : 256 + threadIdx.x;
        __builtin_nontemporal_store(f32x4{acc[0], acc[1], acc[2], acc[3]}, o + first);
        __builtin_nontemporal_store(f32x4{acc[4], acc[5], acc[6], acc[7]}, o + second);
    }
}

// The fused update's memory traffic with almost no arithmetic: the rank walk
// above (n streams of 16-bit values, 16 bytes per lane and stream), then three
// fp32 arrays of the same element count read and written in place (plain
// accesses), eight elements per lane.  What the memory system gives this mix of
// many read streams and three read-modify-write streams, whatever the kernel.
__global__ __launch_bounds__(256) void fsdp_probe_update_kernel(ProbeStreams t, int n, int64_t nvec, float* __restrict__ p,
                                                                float* __restrict__ m, float* __restrict__ v)
{
    const int64_t c = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (c >= nvec) return;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = -0.0f;
    for (int w = 0; w < n; ++w) {
        const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t.p[w]) + c);
        acc[0] += __uint_as_float(x.x << 16); acc[1] += __uint_as_float(x.x & 0xFFFF0000u);
        acc[2] += __uint_as_float(x.y << 16); acc[3] += __uint_as_float(x.y & 0xFFFF0000u);
        acc[4] += __uint_as_float(x.z << 16); acc[5] += __uint_as_float(x.z & 0xFFFF0000u);
        acc[6] += __uint_as_float(x.w << 16); acc[7] += __uint_as_float(x.w & 0xFFFF0000u);
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        f32x4* pp = reinterpret_cast<f32x4*>(p + c * 8 + 4 * q);
        f32x4* pm = reinterpret_cast<f32x4*>(m + c * 8 + 4 * q);
        f32x4* pv = reinterpret_cast<f32x4*>(v + c * 8 + 4 * q);
        const f32x4 g = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        const f32x4 mk = *pm * 0.9f + g;
        const f32x4 vk = *pv * 0.999f + g * g;
        *pp = *pp - mk * 0.0001f;
        *pm = mk;
        *pv = vk;
    }
}

namespace {
bool bad_buffer(const void* p, int64_t nbytes)
{
    return !p || nbytes <= 0 || (nbytes & 15) || (reinterpret_cast<uintptr_t>(p) & 15) || (nbytes / 16 + 63) / 64 > 0x7FFFFFFFLL;
}
bool bad_lanes(int lanes) { return lanes != 64 && lanes != 128 && lanes != 256; }
}  // namespace

// dst, src: device, 16-byte aligned; nbytes: multiple of 16; lanes: workgroup size, 64, 128 or 256 (single-wave
// workgroups measure 2 % faster than 256-lane ones on MI355X).  Each returns the hipError_t of its launch.
extern "C" int fsdp_probe_copy(void* dst, const void* src, int64_t nbytes, int lanes, void* hip_stream)
{
    if (bad_buffer(dst, nbytes) || bad_buffer(src, nbytes) || bad_lanes(lanes)) return static_cast<int>(hipErrorInvalidValue);
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(fsdp_probe_copy_kernel, dim3(static_cast<uint32_t>((nvec + lanes - 1) / lanes)), dim3(lanes), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const f32x4*>(src), static_cast<f32x4*>(dst),
                       nvec);
    return static_cast<int>(hipGetLastError());
}

// sink: device, one float (never written for zero-filled sources)
extern "C" int fsdp_probe_read(const void* src, int64_t nbytes, float* sink, int lanes, void* hip_stream)
{
    if (bad_buffer(src, nbytes) || !sink || bad_lanes(lanes)) return static_cast<int>(hipErrorInvalidValue);
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(fsdp_probe_read_kernel, dim3(static_cast<uint32_t>((nvec + lanes - 1) / lanes)), dim3(lanes), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const f32x4*>(src), nvec, sink);
    return static_cast<int>(hipGetLastError());
}

extern "C" int fsdp_probe_write(void* dst, int64_t nbytes, float value, int lanes, void* hip_stream)
{
    if (bad_buffer(dst, nbytes) || bad_lanes(lanes)) return static_cast<int>(hipErrorInvalidValue);
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(fsdp_probe_write_kernel, dim3(static_cast<uint32_t>((nvec + lanes - 1) / lanes)), dim3(lanes), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<f32x4*>(dst), nvec, value);
    return static_cast<int>(hipGetLastError());
}

// streams: host array of n (1..64) device buffers of nbytes each (16-byte aligned, nbytes a multiple of 16);
// out: device, 2 * nbytes bytes (written only when store != 0).
extern "C" int fsdp_probe_streams(const void* const* streams, int n, int64_t nbytes, int store, float* out,
                                  void* hip_stream)
{
    if (!streams || n < 1 || n > 64 || bad_buffer(out, nbytes)) return static_cast<int>(hipErrorInvalidValue);
    ProbeStreams t = {};
    for (int w = 0; w < n; ++w) {
        if (bad_buffer(streams[w], nbytes)) return static_cast<int>(hipErrorInvalidValue);
        t.p[w] = static_cast<const uint32_t*>(streams[w]);
    }
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(fsdp_probe_streams_kernel, dim3(static_cast<uint32_t>((nvec + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), t, n, nvec, store, out);
    return static_cast<int>(hipGetLastError());
}

// As fsdp_probe_streams, plus p, m, v: device, 2 * nbytes bytes each (fp32, one per 16-bit stream value), updated in place.
extern "C" int fsdp_probe_update(const void* const* streams, int n, int64_t nbytes, float* p, float* m, float* v,
                                 void* hip_stream)
{
    if (!streams || n < 1 || n > 64 || bad_buffer(p, nbytes) || bad_buffer(m, nbytes) || bad_buffer(v, nbytes))
        return static_cast<int>(hipErrorInvalidValue);
    ProbeStreams t = {};
    for (int w = 0; w < n; ++w) {
        if (bad_buffer(streams[w], nbytes)) return static_cast<int>(hipErrorInvalidValue);
        t.p[w] = static_cast<const uint32_t*>(streams[w]);
    }
    const int64_t nvec = nbytes / 16;
    hipLaunchKernelGGL(fsdp_probe_update_kernel, dim3(static_cast<uint32_t>((nvec + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), t, n, nvec, p, m, v);
    return static_cast<int>(hipGetLastError());
}

// The runtime's own device-to-device copy of the same buffers, for comparison with the copy kernel above.
extern "C" int fsdp_probe_memcpy(void* dst, const void* src, int64_t nbytes, void* hip_stream)
{
    if (bad_buffer(dst, nbytes) || bad_buffer(src, nbytes)) return static_cast<int>(hipErrorInvalidValue);
    return static_cast<int>(hipMemcpyAsync(dst, src, static_cast<size_t>(nbytes), hipMemcpyDeviceToDevice,
                                           static_cast<hipStream_t>(hip_stream)));
}

// src: device, 2 * nbytes_out bytes of floats; dst: device, nbytes_out bytes (a multiple of 8); both 16-byte aligned.
extern "C" int fsdp_probe_cast(void* dst, const void* src, int64_t nbytes_out, int lanes, void* hip_stream)
{
    if (!dst || !src || nbytes_out <= 0 || (nbytes_out & 7) || (reinterpret_cast<uintptr_t>(dst) & 15) ||
        (reinterpret_cast<uintptr_t>(src) & 15) || bad_lanes(lanes) || (nbytes_out / 8 + 63) / 64 > 0x7FFFFFFFLL)
        return static_cast<int>(hipErrorInvalidValue);
    const int64_t nvec = nbytes_out / 8;
    hipLaunchKernelGGL(fsdp_probe_cast_kernel, dim3(static_cast<uint32_t>((nvec + lanes - 1) / lanes)), dim3(lanes), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const u32x4p*>(src), static_cast<u32x2p*>(dst), nvec);
    return static_cast<int>(hipGetLastError());
}
