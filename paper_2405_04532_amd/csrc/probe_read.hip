// Measurement probe, not part of the W4A8 boundary: a plain streaming read of a device buffer.
//
// The memory-bound GEMM launches of the decode workloads last 5 - 20 us; at that length the time a kernel needs to
// start, to see its first data and to drain is a large share of the whole.  This probe tells how long the simplest
// possible kernel -- every workgroup reads one contiguous slab with 16-byte loads, sixteen in flight per lane, and
// combines the words so that the loads cannot be dropped -- takes for the same number of bytes in the same launch
// regime (replayed from a graph, sources rotated through more memory than the caches hold).  The benchmark reports it
// next to the GEMM so that the fraction of the published peak can be read against what a plain read reaches.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace {

constexpr int kThreads = 512, kUnroll = 8;

__global__ __launch_bounds__(kThreads) void read_kernel(const uint4* __restrict__ src, size_t n16, uint32_t* sink)
{
    // equal slabs of whole 128-byte lines; the last ones may be short or empty
    const size_t per = ((n16 + gridDim.x - 1) / gridDim.x + 7) / 8 * 8;
    const size_t first = (size_t)blockIdx.x * per;
    if (first >= n16) return;
    const uint4* p = src + first;
    const size_t mine = n16 - first < per ? n16 - first : per;
    uint4 acc = make_uint4(0, 0, 0, 0);
    // Two rounds of kUnroll loads per lane are always in flight: the next round is requested before the one before
    // it is used.  Addresses past the slab are clamped to its last word (and their data dropped), so the requests
    // of the last rounds need no branch.
    auto fetch = [&](uint4 (&v)[kUnroll], size_t i) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const size_t at = i + (size_t)u * kThreads;
            v[u] = p[at < mine ? at : mine - 1];
        }
    };
    auto fold = [&](const uint4 (&v)[kUnroll], size_t i) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            if (i + (size_t)u * kThreads < mine) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
    };
    constexpr size_t kRound = (size_t)kUnroll * kThreads;
    const size_t rounds = (mine + kRound - 1) / kRound;
    uint4 a[kUnroll], b[kUnroll];
    size_t i = threadIdx.x;
    fetch(a, i);
    for (size_t r = 0; r < rounds; r += 2, i += 2 * kRound) {
        fetch(b, i + kRound);
        fold(a, i);
        fetch(a, i + 2 * kRound);
        fold(b, i + kRound);
    }
    const uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x2405u + threadIdx.x * 0x9e3779b9u) sink[blockIdx.x] = r;   // data dependent: keeps the loads alive
}

}  // namespace

// src: device, bytes a multiple of 16, read once.  sink: device, >= 4 * workgroups bytes (written only by accident of
// the data).  workgroups in [1, 65536].  Returns 0, or 1 on a bad argument, or 2 if the launch failed.
extern "C" int qoq_probe_read(const void* src, size_t bytes, void* sink, int workgroups, void* stream)
{
    if (!src || !sink || bytes == 0 || bytes % 16 || workgroups < 1 || workgroups > 65536) return 1;
    if (reinterpret_cast<uintptr_t>(src) % 16) return 1;
    hipLaunchKernelGGL(read_kernel, dim3((unsigned)workgroups), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), bytes / 16, static_cast<uint32_t*>(sink));
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
