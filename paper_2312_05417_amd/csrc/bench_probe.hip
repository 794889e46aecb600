// Measuring sticks of bench.py: NOT part of the re-ranking library (libespn.so) and not declared in its header.
// Built as libespn_benchprobe.so and loaded by the benchmark only.
//
//   espn_bench_stream_read   a plain contiguous read with nothing that depends on what is read: the rate a
//                            dependency-free streaming kernel reaches on this machine, to put beside the gather +
//                            MaxSim kernel (whose reads hang on two dependent look-ups per document, Sec. 4)
//   espn_bench_copy          a plain copy of known size: the calibration of the profiler's byte counters
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <algorithm>

namespace espn_bench {
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

// The buffer is cut into pieces of `piece` 16-byte chunks (256 KiB) that the workgroups take in turn, piece x by
// workgroup x % gridDim.x, 8 non-temporal loads in flight per lane: the workgroups running at one time read
// neighbouring pieces, which spreads them evenly over the memory channels (7.0-7.2 TB/s on MI355X; ordinary loads 6.2-6.4;
// every workgroup walking one long stretch of its own, megabytes apart from its neighbours': 6.0-6.3).  What is read
// only feeds an xor that is almost never stored.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4v *__restrict__ src, size_t n, size_t piece,
                                                          unsigned long long *__restrict__ sink)
{
    uint4v acc = {0u, 0u, 0u, 0u};
    for (size_t begin = (size_t)blockIdx.x * piece; begin < n; begin += (size_t)gridDim.x * piece) {
        const size_t end = begin + piece < n ? begin + piece : n;
        size_t i = begin + threadIdx.x;
        for (; i + 7 * 256 < end; i += 8 * 256) {
            uint4v v[8];
#pragma unroll
            for (int y = 0; y < 8; ++y) v[y] = __builtin_nontemporal_load(src + i + 256 * y);
#pragma unroll
            for (int y = 0; y < 8; ++y) acc ^= v[y];
        }
        for (; i < end; i += 256) acc ^= __builtin_nontemporal_load(src + i);
    }
    if ((acc.x & acc.y & acc.z & acc.w) == 0xffffffffu) *sink = ((unsigned long long)acc.x << 32) | acc.y;
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4v *__restrict__ src, uint4v *__restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

int n_compute_units()
{
    int dev = 0, n_cu = 256;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) n_cu = 256;
    return n_cu;
}
}  // namespace espn_bench
using namespace espn_bench;

#define PROBE_API extern "C" __attribute__((visibility("default")))

// src: DEVICE, 16-byte aligned; bytes: a multiple of 16; sink: DEVICE, 8 bytes, written only if the xor of
// everything read is all ones.  Returns 0, 1 for a bad argument, 2 if the launch failed.
PROBE_API int espn_bench_stream_read(const void *src, size_t bytes, uint64_t *sink, void *stream)
{
    if (bytes == 0) return 0;
    if (!src || !sink || (reinterpret_cast<uintptr_t>(src) & 15u) != 0 || bytes % 16 != 0) return 1;
    const size_t n = bytes / 16;
    // eight workgroups per compute unit at most, pieces of 256 KiB
    const size_t piece = (size_t)(256 << 10) / 16;
    const size_t blocks = std::max<size_t>(1, std::min<size_t>((size_t)n_compute_units() * 8, (n + piece - 1) / piece));
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4v *>(src), n, piece, reinterpret_cast<unsigned long long *>(sink));
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// Reads `bytes` at src and writes them at dst (both DEVICE, 16-byte aligned, bytes a multiple of 16).
PROBE_API int espn_bench_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (bytes == 0) return 0;
    if (!src || !dst || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) != 0 || bytes % 16 != 0)
        return 1;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)n_compute_units() * 8), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4v *>(src), static_cast<uint4v *>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
