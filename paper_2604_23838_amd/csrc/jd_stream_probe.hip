// Benchmark helpers.  Plain streaming kernels of known traffic (a read-only sweep and a copy): they
// give the benchmark a measured ceiling for HBM reads next to the published peak, and give the
// profiler's byte counters a kernel of known size to be scaled against.  And a stream confined to a
// subset of the compute units, on which the CU-budgeted decode call is tested and timed.
#include "../../include/jigsaw_decode_bench.h"
#include <hip/hip_runtime.h>
#include <vector>

namespace {

constexpr int kThreads = 256;
constexpr int kBlocksPerCu = 2;  // measured best for the read sweep: all CUs move through one 8 MiB window

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// Streaming (non-temporal) loads, like the attention kernels' page loads: every byte is read once.
__global__ __launch_bounds__(kThreads) void stream_read_kernel(const u32x4* __restrict__ src, size_t n16, unsigned* sink)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * kThreads;
    size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    unsigned acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride),
                    c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i);
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u) *sink = acc;  // practically never taken; keeps the loads alive
}

__global__ __launch_bounds__(kThreads) void stream_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * kThreads;
    for (size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

int grid_blocks()
{
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    return cus * kBlocksPerCu;
}

}  // namespace

extern "C" {

jd_status jd_debug_stream_read(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!src || !sink || (reinterpret_cast<uintptr_t>(src) & 15u) || bytes < 16) return JD_ERR_INVALID_ARG;
    hipLaunchKernelGGL(stream_read_kernel, dim3(grid_blocks()), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), bytes / 16, static_cast<unsigned*>(sink));
    return hipGetLastError() == hipSuccess ? JD_OK : JD_ERR_HIP;
}

jd_status jd_debug_stream_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!src || !dst || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) || bytes < 16)
        return JD_ERR_INVALID_ARG;
    hipLaunchKernelGGL(stream_copy_kernel, dim3(grid_blocks()), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint4*>(dst), static_cast<const uint4*>(src), bytes / 16);
    return hipGetLastError() == hipSuccess ? JD_OK : JD_ERR_HIP;
}

jd_status jd_bench_stream_create_cu_masked(int32_t num_cus, void** stream_out)
{
    if (!stream_out) return JD_ERR_INVALID_ARG;
    *stream_out = nullptr;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return JD_ERR_HIP;
    // Every die must keep units for the workgroups the dispatcher sends it, whichever way the driver maps
    // mask bits to dies.  With k = num_cus / 8 a multiple of 8, the bits {per_die * x + c : x < 8, c < k}
    // give every die exactly k units both when the bits are die-major (die = bit / per_die) and when they
    // are dealt round-robin over the dies (die = bit % 8).
    constexpr int kDies = 8;
    const int per_die = cus / kDies;
    if (cus % kDies != 0 || per_die % kDies != 0 || num_cus < 64 || num_cus > cus || num_cus % 64 != 0)
        return JD_ERR_INVALID_ARG;
    const int k = num_cus / kDies;
    std::vector<uint32_t> mask((cus + 31) / 32, 0u);
    for (int x = 0; x < kDies; ++x)
        for (int c = 0; c < k; ++c) {
            const int bit = per_die * x + c;
            mask[bit / 32] |= 1u << (bit % 32);
        }
    hipStream_t s = nullptr;
    if (hipExtStreamCreateWithCUMask(&s, static_cast<uint32_t>(mask.size()), mask.data()) != hipSuccess) {
        (void)hipGetLastError();
        return JD_ERR_HIP;
    }
    *stream_out = s;
    return JD_OK;
}

jd_status jd_bench_stream_destroy(void* stream)
{
    if (!stream) return JD_ERR_INVALID_ARG;
    return hipStreamDestroy(static_cast<hipStream_t>(stream)) == hipSuccess ? JD_OK : JD_ERR_HIP;
}

}  // extern "C"
