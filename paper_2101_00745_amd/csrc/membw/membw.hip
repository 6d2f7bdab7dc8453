// Plain streaming kernels the benchmark uses to measure what the memory system delivers on the same buffers
// the SCC passes run on: a device-to-device copy and a read-only pass.  Not part of the SCC library or its ABI.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// each thread moves kPerThread 16-byte pieces, 256 threads apart: every wavefront instruction covers 1 KB
// of consecutive addresses
constexpr int kPerThread = 2;

__global__ __launch_bounds__(256) void membw_copy(const f32x4* __restrict__ src, f32x4* __restrict__ dst, long long n16)
{
    const long long base = (long long)blockIdx.x * (256 * kPerThread) + threadIdx.x;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const long long idx = base + (long long)i * 256;
        if (idx < n16) dst[idx] = src[idx];
    }
}

__global__ __launch_bounds__(256) void membw_read(const f32x4* __restrict__ src, float* __restrict__ sink, long long n16)
{
    const long long base = (long long)blockIdx.x * (256 * kPerThread) + threadIdx.x;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const long long idx = base + (long long)i * 256;
        if (idx < n16) s += src[idx];
    }
    if (s[0] + s[1] + s[2] + s[3] == 123.456f) sink[0] = s[0];   // never true for the benchmark's data: keeps the loads
}

}  // namespace

extern "C" {

// dst[0 .. bytes) = src[0 .. bytes): device pointers, 16-byte aligned, bytes a multiple of 16.  Returns the HIP status.
int membw_copy_bytes(const void* src, void* dst, long long bytes, void* stream)
{
    const long long n16 = bytes / 16;
    const long long blocks = (n16 + 256 * kPerThread - 1) / (256 * kPerThread);
    membw_copy<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>((const f32x4*)src, (f32x4*)dst, n16);
    return (int)hipGetLastError();
}

// reads src[0 .. bytes) once; `sink` is a device float that is never written for ordinary data
int membw_read_bytes(const void* src, void* sink, long long bytes, void* stream)
{
    const long long n16 = bytes / 16;
    const long long blocks = (n16 + 256 * kPerThread - 1) / (256 * kPerThread);
    membw_read<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>((const f32x4*)src, (float*)sink, n16);
    return (int)hipGetLastError();
}

}  // extern "C"
