// Measurement aids: a plain device-to-device copy of known size -- hardware traffic counters
// (bytes fetched / written per dispatch) are calibrated against what they report for it -- and a
// plain read stream, the rate of which is what a kernel that must read every byte once can reach.
#include "sv_kernels.h"

namespace sv {
namespace {

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Reads 64 KiB per workgroup pass: eight 16-byte non-temporal loads per lane in flight, as the scoring
// kernel has them; the loaded words are folded and one word per workgroup is stored, so that the loads
// cannot be dropped.
constexpr int kReadThreads = 256, kReadUnroll = 8;
constexpr size_t kReadTile16 = (size_t)kReadThreads * kReadUnroll;   // 16-byte words per workgroup pass

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kReadThreads) void read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
    uint32_t fold = 0;
    for (size_t base = (size_t)blockIdx.x * kReadTile16; base < n16; base += (size_t)gridDim.x * kReadTile16) {
        u32x4 v[kReadUnroll];
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) {
            const size_t i = base + (size_t)u * kReadThreads + threadIdx.x;
            v[u] = u32x4(0u);
            if (i < n16) v[u] = __builtin_nontemporal_load(src + i);
        }
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) fold ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    // one plain store per lane-0 of a wavefront (several workgroups share a word: the sink's content is
    // unspecified, it only keeps the loads alive)
    fold ^= __shfl_xor(fold, 32, 64);
    fold ^= __shfl_xor(fold, 16, 64);
    fold ^= __shfl_xor(fold, 8, 64);
    fold ^= __shfl_xor(fold, 4, 64);
    fold ^= __shfl_xor(fold, 2, 64);
    fold ^= __shfl_xor(fold, 1, 64);
    if ((threadIdx.x & 63) == 0) sink[(blockIdx.x * (kReadThreads / 64) + threadIdx.x / 64) & (kReadSinkWords - 1)] = fold;
}

}  // namespace

hipError_t launch_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t stream) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t want = (n16 + kReadTile16 - 1) / kReadTile16;
    const unsigned grid = (unsigned)(want < (1u << 20) ? want : (1u << 20));
    hipLaunchKernelGGL(read_kernel, dim3(grid), dim3(kReadThreads), 0, stream, static_cast<const u32x4*>(src), n16, sink);
    return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t want = (n16 + 255) / 256;
    const unsigned grid = (unsigned)(want < 65536 ? want : 65536);
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, stream, static_cast<uint4*>(dst),
                       static_cast<const uint4*>(src), n16);
    return hipGetLastError();
}

}  // namespace sv
