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
#include "qoq_fp16.h"
#include "qoq_half_decide.h"

namespace qoq {
namespace {

constexpr int kThreads = 256;

// ---- reductions over a wave without LDS traffic: four cross-lane (DPP) steps leave every row of 16 lanes with its
// own result, the four row results are read into scalar registers and combined there.
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
constexpr int kQuadSwap1 = 0xB1, kQuadSwap2 = 0x4E, kRowHalfMirror = 0x141, kRowMirror = 0x140;   // lanes ^1, ^2, 7-l, 15-l
__device__ __forceinline__ float wave_max_nonneg(float v)   // v >= 0: the bit patterns order like the values
{
    int b = __float_as_int(v);
    b = max(b, dpp_i32<kQuadSwap1>(b));
    b = max(b, dpp_i32<kQuadSwap2>(b));
    b = max(b, dpp_i32<kRowHalfMirror>(b));
    b = max(b, dpp_i32<kRowMirror>(b));
    const int r = max(max(__builtin_amdgcn_readlane(b, 0), __builtin_amdgcn_readlane(b, 16)),
                      max(__builtin_amdgcn_readlane(b, 32), __builtin_amdgcn_readlane(b, 48)));
    return __int_as_float(r);
}
__device__ __forceinline__ int wave_sum_i32(int v)
{
    v += dpp_i32<kQuadSwap1>(v);
    v += dpp_i32<kQuadSwap2>(v);
    v += dpp_i32<kRowHalfMirror>(v);
    v += dpp_i32<kRowMirror>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}
__device__ __forceinline__ float wave_sum_f32(float v)
{
    v += __int_as_float(dpp_i32<kQuadSwap1>(__float_as_int(v)));
    v += __int_as_float(dpp_i32<kQuadSwap2>(__float_as_int(v)));
    v += __int_as_float(dpp_i32<kRowHalfMirror>(__float_as_int(v)));
    v += __int_as_float(dpp_i32<kRowMirror>(__float_as_int(v)));
    return (__int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0)) + __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32)) + __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48)));
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
    auto moved = [](double d, auto ctrl) {
        const long long b = __double_as_longlong(d);
        const int lo = dpp_i32<decltype(ctrl)::value>((int)(b & 0xFFFFFFFFll)), hi = dpp_i32<decltype(ctrl)::value>((int)(b >> 32));
        return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
    };
    v += moved(v, std::integral_constant<int, kQuadSwap1>());
    v += moved(v, std::integral_constant<int, kQuadSwap2>());
    v += moved(v, std::integral_constant<int, kRowHalfMirror>());
    v += moved(v, std::integral_constant<int, kRowMirror>());
    auto lane = [](double d, int l) {
        const long long b = __double_as_longlong(d);
        const int lo = __builtin_amdgcn_readlane((int)(b & 0xFFFFFFFFll), l), hi = __builtin_amdgcn_readlane((int)(b >> 32), l);
        return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
    };
    return (lane(v, 0) + lane(v, 16)) + (lane(v, 32) + lane(v, 48));
}

// round_half_away(x / s), clamped to [-127, 127], for FP16 values x and s > 0 (held in FP32), without a division.
// x and s have 11-bit significands, so the exact quotient is either exactly on a rounding midpoint k + 1/2 or at
// least 2^-12 away from every midpoint (|x / s| < 256); x * fl(1 / s) is within 3e-5 of the quotient, and pushing
// it 1e-4 away from zero sends exact midpoints up and nothing else across: the result is the one the correctly
// rounded division followed by round-half-away gives, bit for bit (checked against exact rational arithmetic on
// the FP16 neighbours of all midpoints of several thousand scales, and on the GPU against the CPU reference).
__device__ __forceinline__ int quantize_code(float x, float inv_s)
{
    const float t = x * inv_s;
    const int a = (int)(t + copysignf(0.5f + 1e-4f, t));   // conversion truncates toward zero
    return max(-127, min(127, a));
}

__device__ inline float block_reduce_max(float v, float* smem)
{
    v = wave_max_nonneg(v);
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
    const float inv_s = 1.0f / s;

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
            const int a = quantize_code(f.x, inv_s), b = quantize_code(f.y, inv_s);   // round half away from zero
            isum += a + b;
            fsum += f.x + f.y;
            packed[j >> 1] |= ((uint32_t)(a & 0xFF) << (16 * (j & 1))) | ((uint32_t)(b & 0xFF) << (16 * (j & 1) + 8));
        }
        qrow[c] = make_uint2(packed[0], packed[1]);
    }
    isum = wave_sum_i32(isum);
    fsum = wave_sum_f32(fsum);
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

// Single-read variant: up to 512 threads, up to kCache 16-byte chunks (8 halves each) per thread in registers.
// The kernels index by blockDim.x: with many rows to do and short rows the launcher takes 256 threads per row, so
// that twice as many rows (and bytes) are in flight per compute unit -- at large M the latency of the row load,
// not issue or bandwidth, sets the pace (vector pipe active 0.2 of the time with four rows per compute unit).
constexpr int kWide = 512;
constexpr int kCache = 8;
constexpr int64_t kMaxCachedK = (int64_t)kWide * kCache * 8;

// Quantize a token row that the workgroup holds in registers (chunk c = threadIdx.x + i * blockDim.x in v[i],
// zeros past the end): absmax, scale, INT8 codes, sums.  Used by the plain quantizer and by the producers the
// quantization is fused into.
template <int CACHE>
__device__ inline void quantize_cached_row(const uint4 (&v)[CACHE], int chunks, int64_t m, int64_t K,
                                           int8_t* __restrict__ qx, __half* __restrict__ sx,
                                           int32_t* __restrict__ rowsum, float* __restrict__ tx, float* s_f, int* s_i)
{
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < CACHE; ++i) {
        const __half2* h = reinterpret_cast<const __half2*>(&v[i]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 f = __half22float2(h[j]);
            amax = fmaxf(amax, fmaxf(fabsf(f.x), fabsf(f.y)));
        }
    }
    amax = wave_max_nonneg(amax);
    if ((threadIdx.x & 63) == 0) s_f[threadIdx.x >> 6] = amax;
    __syncthreads();
    const int waves = (int)blockDim.x >> 6;
    amax = s_f[0];
#pragma unroll
    for (int w = 1; w < kWide / 64; ++w)
        if (w < waves) amax = fmaxf(amax, s_f[w]);
    __syncthreads();

    __half sxh = __float2half_rn(amax / 127.0f);   // see act_quant_kernel for why FP32 suffices here
    if (__half2float(sxh) == 0.f) sxh = __float2half_rn(1.0f);
    const float s = __half2float(sxh);
    const float inv_s = 1.0f / s;

    int isum = 0;
    float fsum = 0.f;
    uint2* qrow = reinterpret_cast<uint2*>(qx + m * K);
#pragma unroll
    for (int i = 0; i < CACHE; ++i) {
        const int c = (int)threadIdx.x + i * (int)blockDim.x;
        if (c < chunks) {
            const __half2* h = reinterpret_cast<const __half2*>(&v[i]);
            uint32_t packed[2] = {0u, 0u};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float2 f = __half22float2(h[j]);
                const int a = quantize_code(f.x, inv_s), b = quantize_code(f.y, inv_s);   // round half away from zero
                isum += a + b;
                fsum += f.x + f.y;
                packed[j >> 1] |= ((uint32_t)(a & 0xFF) << (16 * (j & 1))) | ((uint32_t)(b & 0xFF) << (16 * (j & 1) + 8));
            }
            qrow[c] = make_uint2(packed[0], packed[1]);
        }
    }
    if (!rowsum && !tx) {                          // group mode needs neither sum: no second reduction
        if (threadIdx.x == 0) sx[m] = sxh;
        return;
    }
    isum = wave_sum_i32(isum);
    fsum = wave_sum_f32(fsum);
    if ((threadIdx.x & 63) == 0) { s_i[threadIdx.x >> 6] = isum; s_f[threadIdx.x >> 6] = fsum; }
    __syncthreads();
    if (threadIdx.x == 0) {
        int it = 0; float ft = 0.f;
        for (int w = 0; w < waves; ++w) { it += s_i[w]; ft += s_f[w]; }
        sx[m] = sxh;
        if (rowsum) rowsum[m] = it;
        if (tx) tx[m] = ft;
    }
}

template <int CACHE>
__global__ __launch_bounds__(kWide) void act_quant_cached_kernel(const __half* __restrict__ x, int64_t K,
                                                                 int8_t* __restrict__ qx, __half* __restrict__ sx,
                                                                 int32_t* __restrict__ rowsum, float* __restrict__ tx)
{
    __shared__ float s_f[kWide / 64];
    __shared__ int s_i[kWide / 64];
    const int64_t m = blockIdx.x;
    const uint4* row = reinterpret_cast<const uint4*>(x + m * K);
    const int chunks = (int)(K / 8);
    uint4 v[CACHE];
#pragma unroll
    for (int i = 0; i < CACHE; ++i) {
        const int c = (int)threadIdx.x + i * (int)blockDim.x;
        v[i] = c < chunks ? row[c] : make_uint4(0u, 0u, 0u, 0u);
    }
    quantize_cached_row(v, chunks, m, K, qx, sx, rowsum, tx, s_f, s_i);
}

// The same with the input channels taken in a new order (activation-aware channel reordering, Section 4.3):
// qx[m, j] = quantize(x[m, perm[j]]).  The gather is fused into the quantizer's single read of the row; the
// per-token scale does not depend on the order.  Indices are clamped to the row.
__global__ __launch_bounds__(kWide) void act_quant_reordered_kernel(const __half* __restrict__ x, const int32_t* __restrict__ perm,
                                                                    int64_t K, int8_t* __restrict__ qx, __half* __restrict__ sx,
                                                                    int32_t* __restrict__ rowsum, float* __restrict__ tx)
{
    __shared__ float s_f[kWide / 64];
    __shared__ int s_i[kWide / 64];
    const int64_t m = blockIdx.x;
    const unsigned short* row = reinterpret_cast<const unsigned short*>(x + m * K);
    const int chunks = (int)(K / 8);
    uint4 v[kCache];
#pragma unroll
    for (int i = 0; i < kCache; ++i) {
        const int c = (int)threadIdx.x + i * (int)blockDim.x;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (c < chunks) {
            const int4 p0 = reinterpret_cast<const int4*>(perm)[2 * c], p1 = reinterpret_cast<const int4*>(perm)[2 * c + 1];
            const int idx[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
            for (int j = 0; j < 8; ++j)
                w[j >> 1] |= (uint32_t)row[min(max(idx[j], 0), (int)K - 1)] << (16 * (j & 1));
        }
        v[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    quantize_cached_row(v, chunks, m, K, qx, sx, rowsum, tx, s_f, s_i);
}

// ---- producers with the quantization fused in (Section 5.1: the activations are quantized inside the
// normalisation in front of the QKV / first FFN projection and inside the activation function in front of the
// second FFN projection).  The producer is evaluated in FP64 and rounded once to FP16 (the exact bit routine
// below), which defines the tensor an unfused pipeline would hand to the quantizer; the codes are then decided
// from that FP16 value exactly as in the stand-alone kernel.
__device__ inline void unpack8(const uint4& v, double (&f)[8])
{
    const __half* h = reinterpret_cast<const __half*>(&v);
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] = (double)__half2float(h[j]);
}

__device__ inline uint4 pack8(const double (&f)[8])
{
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        w[j] = (uint32_t)double_to_half_rne(f[2 * j]) | ((uint32_t)double_to_half_rne(f[2 * j + 1]) << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// The machine operations behind the FP32 decision routines of qoq_half_decide.h.  keep(): an empty asm on the value,
// which keeps the compiler from merging an FP32 product with a conversion next to it (of an FP16 factor, or of the
// product to FP16) into one mixed-precision multiply-add with a zero addend: that turns a product of -0 into +0.
struct DevF32 {
    static __device__ __forceinline__ uint32_t bits(float x) { return __float_as_uint(x); }
    static __device__ __forceinline__ float from_bits(uint32_t u) { return __uint_as_float(u); }
    static __device__ __forceinline__ uint32_t half_bits(float x) { return (uint32_t)__half_as_ushort(__float2half_rn(x)); }
    static __device__ __forceinline__ float keep(float x)
    {
        asm volatile("" : "+v"(x));
        return x;
    }
};
__device__ __forceinline__ float opaque(float x) { return DevF32::keep(x); }

// Element idx (chunk idx / 8, half idx % 8) of the cached chunks := bits.  Written as compile-time indexed selects: a
// register array indexed at run time would be moved to scratch memory.
template <int CACHE>
__device__ __forceinline__ void patch_half(uint4 (&v)[CACHE], int idx, uint32_t bits)
{
#pragma unroll
    for (int i = 0; i < CACHE; ++i) {
        uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (idx == i * 8 + j) w[j >> 1] = (w[j >> 1] & ~(0xFFFFu << (16 * (j & 1)))) | (bits << (16 * (j & 1)));
        v[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// gate / (1 + exp(-gate)) in FP64 for the elements FP32 could not decide.  exp by its definition: -gate = n ln2 + r
// with |r| <= ln2 / 2 (ln2 split so that n * ln2_hi is exact for |n| < 2^20), the Taylor series of exp(r) to the
// term r^13 / 13! (the next one is below 2^-55) and a scaling by 2^n that saturates to 0 or infinity.  Within 2^-49
// of the true value, which rounds to the same FP16 number unless the value lies that close to a midpoint.  One
// FP64 instruction occupies the SIMD for 8 cycles whatever the number of active lanes, so the length of this
// routine (about 40 of them, against several hundred in a general-purpose exp and division) is what the rare path costs.
__device__ __forceinline__ double silu_f64(double g)
{
    const double z = fmin(fmax(-g, -1000.0), 1000.0);  // beyond +-745 exp is 0 or infinite anyway; keeps n small for +-inf and NaN
    const double nf = rint(z * 1.4426950408889634074);
    const double r = fma(-nf, 1.9082149292705877e-10, fma(-nf, 6.93147180369123816490e-01, z));
    double e = 1.0 / 6227020800.0;
    e = fma(e, r, 1.0 / 479001600.0);
    e = fma(e, r, 1.0 / 39916800.0);
    e = fma(e, r, 1.0 / 3628800.0);
    e = fma(e, r, 1.0 / 362880.0);
    e = fma(e, r, 1.0 / 40320.0);
    e = fma(e, r, 1.0 / 5040.0);
    e = fma(e, r, 1.0 / 720.0);
    e = fma(e, r, 1.0 / 120.0);
    e = fma(e, r, 1.0 / 24.0);
    e = fma(e, r, 1.0 / 6.0);
    e = fma(e, r, 0.5);
    e = fma(e, r, 1.0);
    e = fma(e, r, 1.0);
    e = ldexp(e, (int)nf);                             // 2^n over- and underflows as exp does
    return g / (1.0 + e);
}

// y = x * (1 / sqrt(mean(x^2) + eps)) * gamma
template <int CACHE>
__global__ __launch_bounds__(kWide) void rmsnorm_quant_kernel(const __half* __restrict__ x, const __half* __restrict__ gamma,
                                                              double eps, int64_t K, __half* __restrict__ y,
                                                              int8_t* __restrict__ qx, __half* __restrict__ sx,
                                                              int32_t* __restrict__ rowsum, float* __restrict__ tx)
{
    __shared__ float s_f[kWide / 64];
    __shared__ int s_i[kWide / 64];
    __shared__ double s_d[kWide / 64];
    const int64_t m = blockIdx.x;
    const uint4* row = reinterpret_cast<const uint4*>(x + m * K);
    const uint4* grow = reinterpret_cast<const uint4*>(gamma);
    const int chunks = (int)(K / 8);
    uint4 v[CACHE], gv[CACHE];                         // the weights are fetched with the row, not after the reduction
    double ss = 0.0;
#pragma unroll
    for (int i = 0; i < CACHE; ++i) {
        const int c = (int)threadIdx.x + i * (int)blockDim.x;
        v[i] = c < chunks ? row[c] : make_uint4(0u, 0u, 0u, 0u);
        gv[i] = c < chunks ? grow[c] : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int i = 0; i < CACHE; ++i) {
        double f[8];
        unpack8(v[i], f);
#pragma unroll
        for (int j = 0; j < 8; ++j) ss += f[j] * f[j];
    }
    ss = wave_sum_f64(ss);
    if ((threadIdx.x & 63) == 0) s_d[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = 0.0;
#pragma unroll
    for (int w = 0; w < kWide / 64; ++w)
        if (w < ((int)blockDim.x >> 6)) ss += s_d[w];
    const double inv = 1.0 / sqrt(ss / (double)K + eps);
    const float inv32 = (float)inv, inv_lo = (float)(inv - (double)inv32);   // inv = inv32 + inv_lo to 2^-48
    uint64_t risky = 0;                                // elements to redo in FP64, bit = chunk * 8 + half
#pragma unroll
    for (int i = 0; i < CACHE; ++i) {
        const int c = (int)threadIdx.x + i * (int)blockDim.x;
        if (c < chunks) {
            const __half* hx = reinterpret_cast<const __half*>(&v[i]);
            const __half* hg = reinterpret_cast<const __half*>(&gv[i]);
            uint32_t w[4], diff[4];
            // FP32 first: fl32(r), x * fl32(r) and the product with gamma each round once, so the result is within
            // 3 * 2^-24 (relative) of the FP64 product; the bounds are taken at 4 * 2^-23, their own rounding included
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float x0 = opaque(__half2float(hx[2 * j])), x1 = opaque(__half2float(hx[2 * j + 1]));
                const float g0 = opaque(__half2float(hg[2 * j])), g1 = opaque(__half2float(hg[2 * j + 1]));
                diff[j] = half2_bits_from_bounds<DevF32>(x0 * inv32 * g0, x1 * inv32 * g1,
                                                 1.0f - 4 * 0x1p-23f, 1.0f + 4 * 0x1p-23f, w[j]);
            }
            if (diff[0] | diff[1] | diff[2] | diff[3]) {   // every second wave and chunk has such an element
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if ((diff[j >> 1] >> (16 * (j & 1))) & 0xFFFFu) {
                        // next to a rounding midpoint: the same product with its rounding errors carried along
                        float hi, lo;
                        scaled_product_pair<DevF32>(__half2float(hx[j]), inv32, inv_lo, __half2float(hg[j]), hi, lo);
                        uint32_t b = 0;
                        if (!half_bits_from_pair<DevF32>(hi, lo, b)) risky |= 1ull << (i * 8 + j);
                        w[j >> 1] = (w[j >> 1] & ~(0xFFFFu << (16 * (j & 1)))) | (b << (16 * (j & 1)));
                    }
                }
            }
            v[i] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
    // what is left (overflow range, values within 2^-36 of a midpoint): FP64, one at a time
    while (risky) {
        const int idx = __ffsll((unsigned long long)risky) - 1;
        risky &= risky - 1;
        const int64_t k = ((int64_t)threadIdx.x + (int64_t)(idx >> 3) * (int64_t)blockDim.x) * 8 + (idx & 7);
        const double fx = (double)__half2float(x[m * K + k]), fg = (double)__half2float(gamma[k]);
        patch_half(v, idx, (uint32_t)double_to_half_rne(fx * inv * fg));
    }
    if (y) {
#pragma unroll
        for (int i = 0; i < CACHE; ++i) {
            const int c = (int)threadIdx.x + i * (int)blockDim.x;
            if (c < chunks) reinterpret_cast<uint4*>(y + m * K)[c] = v[i];
        }
    }
    quantize_cached_row(v, chunks, m, K, qx, sx, rowsum, tx, s_f, s_i);
}

// gate_up [M, 2K]: y = gate / (1 + exp(-gate)) * up with gate = first K columns, up = last K
template <int CACHE>
__global__ __launch_bounds__(kWide) void silu_mul_quant_kernel(const __half* __restrict__ gate_up, int64_t K,
                                                               __half* __restrict__ y, int8_t* __restrict__ qx,
                                                               __half* __restrict__ sx, int32_t* __restrict__ rowsum,
                                                               float* __restrict__ tx)
{
    __shared__ float s_f[kWide / 64];
    __shared__ int s_i[kWide / 64];
    const int64_t m = blockIdx.x;
    const uint4* grow = reinterpret_cast<const uint4*>(gate_up + m * 2 * K);
    const uint4* urow = reinterpret_cast<const uint4*>(gate_up + m * 2 * K + K);
    const int chunks = (int)(K / 8);
    uint4 v[CACHE];
    uint64_t risky = 0;                                // elements to redo in FP64, bit = chunk * 8 + half
#pragma unroll
    for (int i = 0; i < CACHE; ++i) {
        const int c = (int)threadIdx.x + i * (int)blockDim.x;
        v[i] = make_uint4(0u, 0u, 0u, 0u);
        if (c < chunks) {
            const uint4 gv = grow[c], uv = urow[c];
            const __half* hg = reinterpret_cast<const __half*>(&gv);
            const __half* hu = reinterpret_cast<const __half*>(&uv);
            uint32_t w[4], diff[4];
            // FP32 first: expf and the hardware reciprocal (1 unit in the last place each), the addition and the two
            // products (half a unit each) leave the result within 3.5 * 2^-23 (relative) of the FP64 value; the bounds
            // are taken at 8 * 2^-23, their own rounding included
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float g0 = opaque(__half2float(hg[2 * j])), g1 = opaque(__half2float(hg[2 * j + 1]));
                const float s0 = g0 * __builtin_amdgcn_rcpf(1.0f + expf(-g0)), s1 = g1 * __builtin_amdgcn_rcpf(1.0f + expf(-g1));
                diff[j] = half2_bits_from_bounds<DevF32>(s0 * opaque(__half2float(hu[2 * j])), s1 * opaque(__half2float(hu[2 * j + 1])),
                                                 1.0f - 8 * 0x1p-23f, 1.0f + 8 * 0x1p-23f, w[j]);
            }
            if (diff[0] | diff[1] | diff[2] | diff[3]) {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if ((diff[j >> 1] >> (16 * (j & 1))) & 0xFFFFu) risky |= 1ull << (i * 8 + j);
            }
            v[i] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
    // the few elements (about 1 in 500) whose FP32 value is too close to a rounding midpoint: FP64, one at a time
    while (risky) {
        const int idx = __ffsll((unsigned long long)risky) - 1;
        risky &= risky - 1;
        const int64_t k = ((int64_t)threadIdx.x + (int64_t)(idx >> 3) * (int64_t)blockDim.x) * 8 + (idx & 7);
        const double dg = (double)__half2float(gate_up[m * 2 * K + k]), du = (double)__half2float(gate_up[m * 2 * K + K + k]);
        patch_half(v, idx, (uint32_t)double_to_half_rne(silu_f64(dg) * du));
    }
    if (y) {
#pragma unroll
        for (int i = 0; i < CACHE; ++i) {
            const int c = (int)threadIdx.x + i * (int)blockDim.x;
            if (c < chunks) reinterpret_cast<uint4*>(y + m * K)[c] = v[i];
        }
    }
    quantize_cached_row(v, chunks, m, K, qx, sx, rowsum, tx, s_f, s_i);
}

}  // namespace

// Threads per token row: 512, or 256 where there are rows enough to fill the chip several times over and a row is
// at most two chunks per thread then (with few rows the time of one row counts, and more threads shorten it).
static int64_t row_threads(int64_t M, int64_t K)
{
    return (M >= 2048 && K <= (int64_t)256 * 2 * 8) ? 256 : kWide;
}

hipError_t launch_act_quant(const void* x_fp16, int64_t M, int64_t K, int8_t* qx, void* sx, int32_t* rowsum,
                            float* tx, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    if (K <= kMaxCachedK) {
        // as many cached 16-byte chunks per thread as the row needs: short rows spend nothing on empty ones
        const int64_t wide = row_threads(M, K);
        auto* kern = K <= wide * 8 ? act_quant_cached_kernel<1>
                   : K <= wide * 2 * 8 ? act_quant_cached_kernel<2>
                   : K <= wide * 4 * 8 ? act_quant_cached_kernel<4> : act_quant_cached_kernel<kCache>;
        kern<<<dim3((unsigned)M), (unsigned)wide, 0, s>>>(static_cast<const __half*>(x_fp16), K, qx, static_cast<__half*>(sx), rowsum, tx);
        return hipGetLastError();
    }
    act_quant_kernel<<<dim3((unsigned)M), kThreads, 0, s>>>(static_cast<const __half*>(x_fp16), K, qx,
                                                           static_cast<__half*>(sx), rowsum, tx);
    return hipGetLastError();
}

hipError_t launch_act_quant_reordered(const void* x_fp16, const int32_t* perm, int64_t M, int64_t K, int8_t* qx, void* sx,
                                      int32_t* rowsum, float* tx, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    if (K > kMaxCachedK) return hipErrorInvalidValue;
    act_quant_reordered_kernel<<<dim3((unsigned)M), kWide, 0, s>>>(static_cast<const __half*>(x_fp16), perm, K, qx,
                                                                  static_cast<__half*>(sx), rowsum, tx);
    return hipGetLastError();
}

int64_t fused_quant_max_k() { return kMaxCachedK; }

hipError_t launch_rmsnorm_quant(const void* x_fp16, const void* gamma_fp16, double eps, int64_t M, int64_t K, void* y_fp16,
                                int8_t* qx, void* sx, int32_t* rowsum, float* tx, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    // shorter rows need fewer cached chunks per thread: far fewer registers, more waves per CU
    const int64_t wide = row_threads(M, K);
    auto* kern = K <= wide * 2 * 8 ? rmsnorm_quant_kernel<2>
               : K <= wide * 4 * 8 ? rmsnorm_quant_kernel<4> : rmsnorm_quant_kernel<kCache>;
    kern<<<dim3((unsigned)M), (unsigned)wide, 0, s>>>(static_cast<const __half*>(x_fp16), static_cast<const __half*>(gamma_fp16), eps, K,
                                            static_cast<__half*>(y_fp16), qx, static_cast<__half*>(sx), rowsum, tx);
    return hipGetLastError();
}

hipError_t launch_silu_mul_quant(const void* gate_up_fp16, int64_t M, int64_t K, void* y_fp16, int8_t* qx, void* sx,
                                 int32_t* rowsum, float* tx, hipStream_t s)
{
    if (M == 0) return hipSuccess;
    const int64_t wide = row_threads(M, K);
    auto* kern = K <= wide * 2 * 8 ? silu_mul_quant_kernel<2>
               : K <= wide * 4 * 8 ? silu_mul_quant_kernel<4> : silu_mul_quant_kernel<kCache>;
    kern<<<dim3((unsigned)M), (unsigned)wide, 0, s>>>(static_cast<const __half*>(gate_up_fp16), K, static_cast<__half*>(y_fp16), qx,
                                            static_cast<__half*>(sx), rowsum, tx);
    return hipGetLastError();
}

}  // namespace qoq
