// Data-free offline transforms of QoQ for gfx950 (Section 4.3 of arXiv 2405.04532): channel salience and
// channel gather for the activation-aware reordering, scaled-Hadamard rotation of block-input tensors.
// These run when a model is prepared, not in the serving loop (at run time the reordering is the gather fused
// into the activation quantizer, qoq_act.hip, and the rotation is folded into the preceding layer's weights),
// so they are written for exactness first: the rotation sums in FP64, where sums of FP16 numbers are exact for
// these sizes, and rounds once to FP16.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "qoq_fp16.h"
#include "qoq_internal.h"

namespace qoq {
namespace {

constexpr int kRowsPerSlab = 64;

// salience[k] = max_m |x[m, k]| (Section 4.3: the magnitude of the input activations decides a channel's
// salience).  One thread per 8 channels and slab of rows; non-negative floats order like their bit patterns,
// so the slabs meet with an integer atomic maximum on a zero-filled array.
__global__ __launch_bounds__(256) void channel_absmax_kernel(const __half* __restrict__ x, int64_t M, int64_t K, int* __restrict__ out_bits)
{
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= K / 8) return;
    const int64_t r0 = (int64_t)blockIdx.y * kRowsPerSlab, r1 = min(M, r0 + kRowsPerSlab);
    float mx[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int64_t r = r0; r < r1; ++r) {
        const uint4 v = reinterpret_cast<const uint4*>(x + r * K)[c];
        const __half* h = reinterpret_cast<const __half*>(&v);
#pragma unroll
        for (int j = 0; j < 8; ++j) mx[j] = fmaxf(mx[j], fabsf(__half2float(h[j])));
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) atomicMax(out_bits + c * 8 + j, __float_as_int(mx[j]));
}

// dst[r, j] = src[r, perm[j]]; one thread per 8 output channels.  Indices are clamped to the row.
__global__ __launch_bounds__(256) void gather_channels_kernel(const __half* __restrict__ src, const int32_t* __restrict__ perm,
                                                              int64_t rows, int64_t K, __half* __restrict__ dst)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t chunks = K / 8;
    if (idx >= rows * chunks) return;
    const int64_t r = idx / chunks, c = idx % chunks;
    const unsigned short* row = reinterpret_cast<const unsigned short*>(src + r * K);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int p = min(max(perm[c * 8 + j], 0), (int)K - 1);
        w[j >> 1] |= (uint32_t)row[p] << (16 * (j & 1));
    }
    reinterpret_cast<uint4*>(dst + r * K)[c] = make_uint4(w[0], w[1], w[2], w[3]);
}

// dst[r, b*n .. b*n+n) = src[r, b*n .. b*n+n) H_n * scale, H_n the Sylvester Hadamard matrix (entry (i, j) =
// (-1)^popcount(i & j)), by the in-place butterfly: log2(n) stages of n/2 additions and subtractions.
// One workgroup per (row, block).  FP64 throughout: every partial sum of at most 8192 FP16 numbers is a multiple
// of 2^-24 below 2^29 and therefore exact, so the result is the exact product times `scale`, rounded once.
constexpr int kMaxHadamard = 8192;
__global__ __launch_bounds__(256) void hadamard_kernel(const __half* __restrict__ src, int64_t K, int n, double scale,
                                                       __half* __restrict__ dst)
{
    __shared__ double buf[kMaxHadamard];
    const int64_t base = (int64_t)blockIdx.y * K + (int64_t)blockIdx.x * n;
    for (int i = threadIdx.x; i < n; i += 256) buf[i] = (double)__half2float(src[base + i]);
    __syncthreads();
    for (int h = 1; h < n; h <<= 1) {
        for (int t = threadIdx.x; t < n / 2; t += 256) {
            const int i = (t / h) * 2 * h + (t % h);
            const double a = buf[i], b = buf[i + h];
            buf[i] = a + b;
            buf[i + h] = a - b;
        }
        __syncthreads();
    }
    for (int i = threadIdx.x; i < n; i += 256) dst[base + i] = __ushort_as_half(double_to_half_rne(buf[i] * scale));
}

}  // namespace

hipError_t launch_channel_absmax(const void* x, int64_t M, int64_t K, float* absmax, hipStream_t s)
{
    hipError_t e = launch_zero(absmax, (size_t)K * sizeof(float), s);
    if (e != hipSuccess || M == 0) return e;
    const dim3 grid((unsigned)((K / 8 + 255) / 256), (unsigned)((M + kRowsPerSlab - 1) / kRowsPerSlab));
    channel_absmax_kernel<<<grid, 256, 0, s>>>(static_cast<const __half*>(x), M, K, reinterpret_cast<int*>(absmax));
    return hipGetLastError();
}

hipError_t launch_gather_channels(const void* src, const int32_t* perm, int64_t rows, int64_t K, void* dst, hipStream_t s)
{
    const int64_t n = rows * (K / 8);
    if (n == 0) return hipSuccess;
    gather_channels_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(static_cast<const __half*>(src), perm, rows, K,
                                                                        static_cast<__half*>(dst));
    return hipGetLastError();
}

int hadamard_max_block() { return kMaxHadamard; }

hipError_t launch_hadamard(const void* src, int64_t rows, int64_t K, int64_t block, void* dst, hipStream_t s)
{
    if (rows == 0) return hipSuccess;
    const double scale = 1.0 / std::sqrt((double)block);     // correctly rounded on the host
    const dim3 grid((unsigned)(K / block), (unsigned)rows);
    hadamard_kernel<<<grid, 256, 0, s>>>(static_cast<const __half*>(src), K, (int)block, scale, static_cast<__half*>(dst));
    return hipGetLastError();
}

// Host side: most salient channel first, ties by channel index.
void channel_order_host(const float* salience, int64_t K, int32_t* perm)
{
    std::vector<int32_t> idx((size_t)K);
    std::iota(idx.begin(), idx.end(), 0);
    std::stable_sort(idx.begin(), idx.end(), [&](int32_t a, int32_t b) { return salience[a] > salience[b]; });
    std::copy(idx.begin(), idx.end(), perm);
}

}  // namespace qoq
