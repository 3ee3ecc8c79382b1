// Offline weight path: progressive group quantization (Section 4.1 of arXiv 2405.04532,
// Eq. 3-4 with the protective range), the per-channel variant (Section 5.2.2), and the
// store in matrix-core consumption order (Section 5.2.1).  Runs once per layer.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "qoq_internal.h"

namespace qoq {
namespace {

constexpr int kThreads = 256;

// Exact round-to-nearest-even conversion of a non-negative finite double to FP16 bits.
__device__ inline uint16_t double_to_half_bits(double d)
{
    if (!(d > 0.0)) return 0;
    int e;
    (void)frexp(d, &e);
    int ex = e - 1;  // d = 1.xxx * 2^ex
    if (ex < -14) {
        const double r = rint(ldexp(d, 24));  // subnormal step 2^-24; 1024 carries into the first normal
        return (uint16_t)(int)r;
    }
    double r = rint(ldexp(d, 10 - ex));  // in [1024, 2048]
    if (r >= 2048.0) { r = 1024.0; ex += 1; }
    if (ex > 15) return 0x7C00;
    return (uint16_t)(((ex + 15) << 10) | ((int)r - 1024));
}

__device__ inline float half_bits_to_float(uint16_t h) { return __half2float(__ushort_as_half(h)); }

// FP16 scale = fp16(range / steps); a zero scale (empty range) becomes 1.0.
__device__ inline uint16_t make_scale(double range, double steps)
{
    uint16_t h = double_to_half_bits(range / steps);
    return h == 0 ? (uint16_t)0x3C00 : h;
}

__device__ inline int round_half_away(double v) { return (int)round(v); }

__device__ inline float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline float wave_min(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline int wave_max_i(int v)
{
    for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline int wave_min_i(int v)
{
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
    return v;
}

// Row-wide min and max of an FP16 row, result broadcast to every thread of the block.
__device__ inline void row_min_max(const __half* row, int64_t K, float& lo, float& hi)
{
    __shared__ float s_lo[kThreads / 64], s_hi[kThreads / 64];
    float mn = 0.f, mx = 0.f;  // the range always contains 0
    for (int64_t k = (int64_t)threadIdx.x * 2; k < K; k += kThreads * 2) {
        const __half2 v = *reinterpret_cast<const __half2*>(row + k);
        const float a = __low2float(v), b = __high2float(v);
        mn = fminf(mn, fminf(a, b));
        mx = fmaxf(mx, fmaxf(a, b));
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) { s_lo[threadIdx.x >> 6] = mn; s_hi[threadIdx.x >> 6] = mx; }
    __syncthreads();
    lo = s_lo[0]; hi = s_hi[0];
    for (int w = 1; w < kThreads / 64; ++w) { lo = fminf(lo, s_lo[w]); hi = fmaxf(hi, s_hi[w]); }
}

// Place this lane's two adjacent codes (k_local = 2*lane, 2*lane+1) into their packed dword,
// combine the four lanes that share a dword, and let the first of them store it.
__device__ inline void store_group_codes(uint8_t* codes, int64_t nf, int i, int64_t g, int64_t G, int lane,
                                         int code_a, int code_b)
{
    int sh_a, sh_b;
    const size_t off = code_dword_offset(nf, i, g, G, 2 * lane, sh_a);
    (void)code_dword_offset(nf, i, g, G, 2 * lane + 1, sh_b);
    uint32_t v = ((uint32_t)code_a << sh_a) | ((uint32_t)code_b << sh_b);
    v |= __shfl_xor(v, 1, 64);
    v |= __shfl_xor(v, 2, 64);
    if ((lane & 3) == 0) *reinterpret_cast<uint32_t*>(codes + off) = v;
}

// One block per logical output channel; each wave quantizes one group of 128 at a time.
__global__ __launch_bounds__(kThreads) void pack_group_kernel(const __half* __restrict__ w, BlobLayout L,
                                                              uint8_t* __restrict__ blob)
{
    const int64_t n = blockIdx.x;
    const __half* row = w + n * L.K;
    float lo, hi;
    row_min_max(row, L.K, lo, hi);
    const double absmax = fmax((double)hi, -(double)lo);
    const uint16_t s0_bits = make_scale(absmax, 119.0);  // level 1, protective range (Eq. 3)
    const double s0 = (double)half_bits_to_float(s0_bits);
    if (threadIdx.x == 0) reinterpret_cast<uint16_t*>(blob + L.scale_off)[n] = s0_bits;

    int64_t nf; int i;
    phys_row(n, nf, i);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint8_t* codes = blob + L.codes_off;
    uint16_t* meta = reinterpret_cast<uint16_t*>(blob + L.meta_off);
    for (int64_t g = wave; g < L.G; g += kThreads / 64) {
        const __half2 v = *reinterpret_cast<const __half2*>(row + g * kGroup + 2 * lane);
        int qa = round_half_away((double)__low2float(v) / s0);
        int qb = round_half_away((double)__high2float(v) / s0);
        qa = max(-119, min(119, qa));
        qb = max(-119, min(119, qb));
        // level 2 (Eq. 4): asymmetric UINT4 on the INT8 intermediates, range widened to hold 0
        const int gmin = wave_min_i(min(min(qa, qb), 0));
        const int gmax = wave_max_i(max(max(qa, qb), 0));
        const int s1 = max(1, (gmax - gmin + 14) / 15);
        const int z = min(15, (2 * (-gmin) + s1) / (2 * s1));
        const int na = 2 * qa + (2 * z + 1) * s1, nb = 2 * qb + (2 * z + 1) * s1;
        const int ca = na <= 0 ? 0 : min(15, na / (2 * s1));
        const int cb = nb <= 0 ? 0 : min(15, nb / (2 * s1));
        store_group_codes(codes, nf, i, g, L.G, lane, ca, cb);
        if (lane == 0)
            meta[meta_offset(nf, i, g, L.N / 16) / 2] = (uint16_t)(s1 | (((128 - z * s1) & 0xFF) << 8));
    }
}

__global__ __launch_bounds__(kThreads) void pack_channel_kernel(const __half* __restrict__ w, BlobLayout L,
                                                                uint8_t* __restrict__ blob)
{
    const int64_t n = blockIdx.x;
    const __half* row = w + n * L.K;
    float lo, hi;
    row_min_max(row, L.K, lo, hi);
    const uint16_t sw_bits = make_scale((double)hi - (double)lo, 15.0);
    const double sw = (double)half_bits_to_float(sw_bits);
    const int z = max(0, min(15, round_half_away(-(double)lo / sw)));
    if (threadIdx.x == 0) {
        reinterpret_cast<uint16_t*>(blob + L.scale_off)[n] = sw_bits;
        (blob + L.zero_off)[n] = (uint8_t)z;
    }
    int64_t nf; int i;
    phys_row(n, nf, i);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint8_t* codes = blob + L.codes_off;
    for (int64_t g = wave; g < L.G; g += kThreads / 64) {
        const __half2 v = *reinterpret_cast<const __half2*>(row + g * kGroup + 2 * lane);
        const int ca = max(0, min(15, round_half_away((double)__low2float(v) / sw + (double)z)));
        const int cb = max(0, min(15, round_half_away((double)__high2float(v) / sw + (double)z)));
        store_group_codes(codes, nf, i, g, L.G, lane, ca, cb);
    }
}

__global__ void write_header_kernel(BlobLayout L, uint8_t* blob)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        BlobHeader h;
        h.magic = kMagic; h.version = kVersion; h.N = L.N; h.K = L.K; h.mode = L.mode; h.group = kGroup;
        h.codes_off = L.codes_off; h.meta_off = L.meta_off; h.scale_off = L.scale_off;
        h.zero_off = L.zero_off; h.total = L.total;
        *reinterpret_cast<BlobHeader*>(blob) = h;
    }
}

// One thread per packed dword: gathers its 8 codes from the logical [N, K] byte tensor.
__global__ __launch_bounds__(kThreads) void pack_quantized_kernel(const uint8_t* __restrict__ q,
                                                                  const uint8_t* __restrict__ s1,
                                                                  const uint8_t* __restrict__ z,
                                                                  const uint16_t* __restrict__ s_fp16,
                                                                  BlobLayout L, uint8_t* __restrict__ blob)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;  // (n, g, j): j = dword group of 8 k
    const int64_t per_row = L.G * 16;
    if (idx >= L.N * per_row) return;
    const int64_t n = idx / per_row;
    const int64_t g = (idx % per_row) / 16;
    const int j = (int)(idx % 16);
    int64_t nf; int i;
    phys_row(n, nf, i);
    const uint8_t* src = q + n * L.K + g * kGroup + 8 * j;
    uint32_t v = 0;
    size_t off = 0;
    for (int t = 0; t < 8; ++t) {
        int sh;
        off = code_dword_offset(nf, i, g, L.G, 8 * j + t, sh);
        v |= (uint32_t)(src[t] & 15) << sh;
    }
    *reinterpret_cast<uint32_t*>(blob + L.codes_off + off) = v;
    if (j == 0) {
        if (L.mode == 0) {
            const int sc = s1[n * L.G + g], zz = z[n * L.G + g];
            reinterpret_cast<uint16_t*>(blob + L.meta_off)[meta_offset(nf, i, g, L.N / 16) / 2] =
                (uint16_t)(sc | (((128 - zz * sc) & 0xFF) << 8));
        }
        if (g == 0) {
            reinterpret_cast<uint16_t*>(blob + L.scale_off)[n] = s_fp16[n];
            if (L.mode == 1) (blob + L.zero_off)[n] = z[n];
        }
    }
}

// One thread per logical (n, k).
__global__ __launch_bounds__(kThreads) void unpack_kernel(const uint8_t* __restrict__ blob, BlobLayout L,
                                                          uint8_t* __restrict__ q, uint8_t* __restrict__ s1,
                                                          uint8_t* __restrict__ z, uint16_t* __restrict__ s_fp16)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= L.N * L.K) return;
    const int64_t n = idx / L.K, k = idx % L.K, g = k / kGroup;
    const int k_local = (int)(k % kGroup);
    int64_t nf; int i;
    phys_row(n, nf, i);
    int sh;
    const size_t off = code_dword_offset(nf, i, g, L.G, k_local, sh);
    const uint32_t v = *reinterpret_cast<const uint32_t*>(blob + L.codes_off + off);
    q[idx] = (uint8_t)((v >> sh) & 15);
    if (k_local == 0) {
        if (L.mode == 0) {
            const uint16_t m = reinterpret_cast<const uint16_t*>(blob + L.meta_off)[meta_offset(nf, i, g, L.N / 16) / 2];
            const int sc = m & 0xFF;
            int b = m >> 8;
            if (b > 128) b -= 256;  // bias = 128 - z*s1 lies in [-112, 128]
            s1[n * L.G + g] = (uint8_t)sc;
            z[n * L.G + g] = (uint8_t)((128 - b) / sc);
        }
        if (k == 0) {
            s_fp16[n] = reinterpret_cast<const uint16_t*>(blob + L.scale_off)[n];
            if (L.mode == 1) z[n] = (blob + L.zero_off)[n];
        }
    }
}

}  // namespace

hipError_t launch_pack_weights(const void* w_fp16, const BlobLayout& L, uint8_t* blob, hipStream_t s)
{
    write_header_kernel<<<1, 64, 0, s>>>(L, blob);
    if (L.mode == 0)
        pack_group_kernel<<<dim3((unsigned)L.N), kThreads, 0, s>>>(static_cast<const __half*>(w_fp16), L, blob);
    else
        pack_channel_kernel<<<dim3((unsigned)L.N), kThreads, 0, s>>>(static_cast<const __half*>(w_fp16), L, blob);
    return hipGetLastError();
}

hipError_t launch_pack_quantized(const uint8_t* q, const uint8_t* s1, const uint8_t* z, const void* s_fp16,
                                 const BlobLayout& L, uint8_t* blob, hipStream_t s)
{
    write_header_kernel<<<1, 64, 0, s>>>(L, blob);
    const int64_t total = L.N * L.G * 16;
    pack_quantized_kernel<<<dim3((unsigned)((total + kThreads - 1) / kThreads)), kThreads, 0, s>>>(
        q, s1, z, static_cast<const uint16_t*>(s_fp16), L, blob);
    return hipGetLastError();
}

hipError_t launch_unpack(const uint8_t* blob, const BlobLayout& L, uint8_t* q, uint8_t* s1, uint8_t* z,
                         void* s_fp16, hipStream_t s)
{
    const int64_t total = L.N * L.K;
    unpack_kernel<<<dim3((unsigned)((total + kThreads - 1) / kThreads)), kThreads, 0, s>>>(
        blob, L, q, s1, z, static_cast<uint16_t*>(s_fp16));
    return hipGetLastError();
}

}  // namespace qoq
