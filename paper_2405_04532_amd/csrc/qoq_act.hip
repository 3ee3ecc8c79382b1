// Per-token symmetric INT8 activation quantization (Section 6.1 of arXiv 2405.04532; Eq. 1 in
// its symmetric form), with the per-token sums the per-channel GEMM epilogue needs
// (Section 5.2.2: sum of the quantized row for the exact zero-point fold of Eq. 6, and the
// sum of the unquantized row, t_X of Eq. 7).  Memory bound: 2 bytes read, 1 byte written per
// element.  One workgroup per token row.  Rows of up to 32768 elements are read once and held in
// registers between the absmax reduction and the rounding pass (all loads of a row are in flight
// together, which is what matters at decode sizes where the call is pure latency); longer rows
// are read twice (the second read hits cache).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "qoq_internal.h"

namespace qoq {
namespace {

constexpr int kThreads = 256;

__device__ inline float block_reduce_max(float v, float* smem)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = smem[0];
    for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, smem[w]);
    __syncthreads();
    return r;
}

__global__ __launch_bounds__(kThreads) void act_quant_kernel(const __half* __restrict__ x, int64_t K,
                                                             int8_t* __restrict__ qx, __half* __restrict__ sx,
                                                             int32_t* __restrict__ rowsum, float* __restrict__ tx)
{
    __shared__ float s_f[kThreads / 64];
    __shared__ int s_i[kThreads / 64];
    const int64_t m = blockIdx.x;
    const uint4* row = reinterpret_cast<const uint4*>(x + m * K);  // 8 halves per 16 bytes
    const int64_t chunks = K / 8;

    float amax = 0.f;
    for (int64_t c = threadIdx.x; c < chunks; c += kThreads) {
        const uint4 v = row[c];
        const __half2* h = reinterpret_cast<const __half2*>(&v);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 f = __half22float2(h[j]);
            amax = fmaxf(amax, fmaxf(fabsf(f.x), fabsf(f.y)));
        }
    }
    amax = block_reduce_max(amax, s_f);

    // sx = fp16(absmax / 127): the FP32 quotient of an FP16 value by 127 never lies close
    // enough to an FP16 rounding midpoint for the intermediate rounding to matter.
    __half sxh = __float2half_rn(amax / 127.0f);
    if (__half2float(sxh) == 0.f) sxh = __float2half_rn(1.0f);
    const float s = __half2float(sxh);

    int isum = 0;
    float fsum = 0.f;
    uint2* qrow = reinterpret_cast<uint2*>(qx + m * K);
    for (int64_t c = threadIdx.x; c < chunks; c += kThreads) {
        const uint4 v = row[c];
        const __half2* h = reinterpret_cast<const __half2*>(&v);
        uint32_t packed[2] = {0u, 0u};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 f = __half22float2(h[j]);
            // true IEEE division, then round half away from zero
            int a = (int)roundf(f.x / s), b = (int)roundf(f.y / s);
            a = max(-127, min(127, a));
            b = max(-127, min(127, b));
            isum += a + b;
            fsum += f.x + f.y;
            packed[j >> 1] |= ((uint32_t)(a & 0xFF) << (16 * (j & 1))) | ((uint32_t)(b & 0xFF) << (16 * (j & 1) + 8));
        }
        qrow[c] = make_uint2(packed[0], packed[1]);
    }
    for (int o = 32; o > 0; o >>= 1) {
        isum += __shfl_xor(isum, o, 64);
        fsum += __shfl_xor(fsum, o, 64);
    }
    if ((threadIdx.x & 63) == 0) { s_i[threadIdx.x >> 6] = isum; s_f[threadIdx.x >> 6] = fsum; }
    __syncthreads();
    if (threadIdx.x == 0) {
        int it = 0; float ft = 0.f;
        for (int w = 0; w < kThreads / 64; ++w) { it += s_i[w]; ft += s_f[w]; }
        sx[m] = sxh;
        if (rowsum) rowsum[m] = it;
        if (tx) tx[m] = ft;
    }
}

// Single-read variant: 512 threads, up to kCache 16-byte chunks (8 halves each) per thread in registers.
constexpr int kWide = 512;
constexpr int kCache = 8;

__global__ __launch_bounds__(kWide) void act_quant_cached_kernel(const __half* __restrict__ x, int64_t K,
                                                                 int8_t* __restrict__ qx, __half* __restrict__ sx,
                                                                 int32_t* __restrict__ rowsum, float* __restrict__ tx)
{
    __shared__ float s_f[kWide / 64];
    __shared__ int s_i[kWide / 64];
    const int64_t m = blockIdx.x;
    const uint4* row = reinterpret_cast<const uint4*>(x + m * K);
    const int chunks = (int)(K / 8);

    uint4 v[kCache];
#pragma unroll
    for (int i = 0; i < kCache; ++i) {
        const int c = (int)threadIdx.x + i * kWide;
        v[i] = c < chunks ? row[c] : make_uint4(0u, 0u, 0u, 0u);
    }
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < kCache; ++i) {
        const __half2* h = reinterpret_cast<const __half2*>(&v[i]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 f = __half22float2(h[j]);
            amax = fmaxf(amax, fmaxf(fabsf(f.x), fabsf(f.y)));
        }
    }
    for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
    if ((threadIdx.x & 63) == 0) s_f[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = s_f[0];
#pragma unroll
    for (int w = 1; w < kWide / 64; ++w) amax = fmaxf(amax, s_f[w]);
    __syncthreads();

    __half sxh = __float2half_rn(amax / 127.0f);   // see act_quant_kernel for why FP32 suffices here
    if (__half2float(sxh) == 0.f) sxh = __float2half_rn(1.0f);
    const float s = __half2float(sxh);

    int isum = 0;
    float fsum = 0.f;
    uint2* qrow = reinterpret_cast<uint2*>(qx + m * K);
#pragma unroll
    for (int i = 0; i < kCache; ++i) {
        const int c = (int)threadIdx.x + i * kWide;
        if (c < chunks) {
            const __half2* h = reinterpret_cast<const __half2*>(&v[i]);
            uint32_t packed[2] = {0u, 0u};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float2 f = __half22float2(h[j]);
                int a = (int)roundf(f.x / s), b = (int)roundf(f.y / s);   // IEEE division, round half away from zero
                a = max(-127, min(127, a));
                b = max(-127, min(127, b));
                isum += a + b;
                fsum += f.x + f.y;
                packed[j >> 1] |= ((uint32_t)(a & 0xFF) << (16 * (j & 1))) | ((uint32_t)(b & 0xFF) << (16 * (j & 1) + 8));
            }
            qrow[c] = make_uint2(packed[0], packed[1]);
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        isum += __shfl_xor(isum, o, 64);
        fsum += __shfl_xor(fsum, o, 64);
    }
    if ((threadIdx.x & 63) == 0) { s_i[threadIdx.x >> 6] = isum; s_f[threadIdx.x >> 6] = fsum; }
    __syncthreads();
    if (threadIdx.x == 0) {
        int it = 0; float ft = 0.f;
        for (int w = 0; w < kWide / 64; ++w) { it += s_i[w]; ft += s_f[w]; }
        sx[m] = sxh;
        if (rowsum) rowsum[m] = it;
        if (tx) tx[m] = ft;
    }
}

}  // namespace

hipError_t launch_act_quant(const void* x_fp16, int64_t M, int64_t K, int8_t* qx, void* sx, int32_t* rowsum,
                            float* tx, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    if (K <= (int64_t)kWide * kCache * 8) {
        act_quant_cached_kernel<<<dim3((unsigned)M), kWide, 0, s>>>(static_cast<const __half*>(x_fp16), K, qx,
                                                                   static_cast<__half*>(sx), rowsum, tx);
        return hipGetLastError();
    }
    act_quant_kernel<<<dim3((unsigned)M), kThreads, 0, s>>>(static_cast<const __half*>(x_fp16), K, qx,
                                                           static_cast<__half*>(sx), rowsum, tx);
    return hipGetLastError();
}

}  // namespace qoq
