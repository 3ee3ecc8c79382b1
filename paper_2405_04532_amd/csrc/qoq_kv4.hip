// KV4 cache and decode attention for gfx950 (Sections 5.1 "KV Cache Management" and 5.3 of arXiv 2405.04532,
// re-designed for CDNA4).
//
// Cache.  Keys and values are quantized when they are written: per token and KV head, Eq. 1 with 4 bits on the
// range of that head's 128 values widened to contain 0, FP16 scale s and integer zero z (stored as FP16).  A
// page holds 64 consecutive tokens of one (sequence, KV head): 4 KiB of key codes, their 64 (s, z) pairs, 4 KiB
// of value codes, their 64 pairs -- the parameters sit directly behind the codes they belong to, in the same
// page.  The pages of a (sequence, head) are contiguous.
//   codes of a token: 16 dwords; dword w holds elements 8w .. 8w+7, element 8w+2j in bits 4j.. of the low half,
//   element 8w+2j+1 in bits 4j.. of the high half: (x >> 4j) & 0x000F000F is a pair of consecutive elements,
//   and OR 0x64006400 makes it the FP16 pair (1024 + a, 1024 + b) -- the integer-to-FP16 conversion without a
//   conversion instruction that Section 5.3 takes from earlier work.  One packed add of -(1024 + z) then gives
//   the exact integers (code - z) as FP16: two vector operations per pair (plus the shifts).
//
// Decode kernel.  One workgroup of four waves per (sequence, KV head); all R = H / Hkv query heads that share
// the KV head are handled together, so the cache is read once.  Every wave streams chunks of the sequence;
// inside a wave a token is spread over 128 / E lanes (E = 32, 16 or 8 elements per lane, fewer when more query
// heads need registers), so a wave load covers 64 * E / 128 whole tokens = 1 KiB of contiguous cache.
//   score = (log2 e / sqrt(D)) * s_K * sum_d q_d (code_d - z_K)      v_dot2_f32_f16: FP16 products, FP32 sums
//   online softmax in base 2 per lane group (no communication between tokens inside the loop)
//   acc_d += (p * s_V) * (code_d - z_V)                               FP32 accumulators, one mixed FMA per element
// The paper moves the products of its kernel from FP32 to FP16 to lift the compute roof of its GPU; here the
// multiplications take FP16 operands and the sums stay FP32, which the dot and mixed-FMA instructions give for
// free.  The partial (max, sum, acc) of all lane groups and waves meet in LDS at the end.
// The scale/zero words of a chunk are loaded together with its codes, one chunk ahead of the arithmetic (the
// prefetch of the dequantization parameters of Section 5.3).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "qoq_fp16.h"
#include "qoq_internal.h"

namespace qoq {
namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;                       // head dimension
constexpr int kPageTokens = 64;
constexpr int kCodeBytes = kPageTokens * kD / 2;          // 4096
constexpr int kParamBytes = kPageTokens * 4;              // 256
constexpr int kHalfPage = kCodeBytes + kParamBytes;       // keys (or values) of a page
constexpr int kPageBytes = 2 * kHalfPage;                 // 8704

__device__ __forceinline__ float wave_min(float v) { for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64)); return v; }
__device__ __forceinline__ float wave_max(float v) { for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64)); return v; }

// ------------------------------------------------------------------------------------------
// Append: one wave per (sequence, token, KV head, key|value) vector of 128 FP16 values; lane l holds elements
// 2l, 2l+1.  Every decision is taken as the reference definition takes it: s = FP16((hi - lo) / 15) by one exact
// rounding of the FP64 quotient, z and the codes by floor(t + 1/2) of FP64 quotients (a quotient of two FP16
// values that is not exactly a half-integer is many orders of magnitude further from it than FP64's error).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void kv4_append_kernel(const __half* __restrict__ k, const __half* __restrict__ v,
                                                         const int32_t* __restrict__ positions, int64_t B, int64_t T,
                                                         int64_t Hkv, int64_t S_max, uint8_t* __restrict__ cache)
{
    const int lane = threadIdx.x & 63;
    const int64_t vec = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);     // ((b * T + t) * Hkv + h) * 2 + which
    if (vec >= B * T * Hkv * 2) return;
    const int which = (int)(vec & 1);
    const int64_t bth = vec >> 1;
    const int64_t h = bth % Hkv, bt = bth / Hkv, t = bt % T, b = bt / T;
    const int64_t pos = (int64_t)positions[b] + t;
    if (pos < 0 || pos >= S_max) return;                                   // outside the cache: not written
    const __half* src = (which ? v : k) + bth * kD;
    const uint32_t raw = reinterpret_cast<const uint32_t*>(src)[lane];
    const float x0 = __half2float(__ushort_as_half((unsigned short)(raw & 0xFFFFu)));
    const float x1 = __half2float(__ushort_as_half((unsigned short)(raw >> 16)));
    const float lo = fminf(wave_min(fminf(x0, x1)), 0.f), hi = fmaxf(wave_max(fmaxf(x0, x1)), 0.f);
    uint16_t s_bits = double_to_half_rne(((double)hi - (double)lo) / 15.0);
    if ((s_bits & 0x7FFFu) == 0) s_bits = 0x3C00u;                         // all-zero vector: s = 1
    const double s = (double)__half2float(__ushort_as_half(s_bits));
    const double zf = fmin(fmax(floor(-(double)lo / s + 0.5), 0.0), 15.0);
    const uint32_t c0 = (uint32_t)fmin(fmax(floor((double)x0 / s + zf + 0.5), 0.0), 15.0);
    const uint32_t c1 = (uint32_t)fmin(fmax(floor((double)x1 / s + zf + 0.5), 0.0), 15.0);
    // dword w = lanes 4w .. 4w+3; lane 4w+j contributes pair j
    const int j = lane & 3;
    uint32_t word = (c0 << (4 * j)) | (c1 << (16 + 4 * j));
    word |= __shfl_xor(word, 1, 64);
    word |= __shfl_xor(word, 2, 64);
    const int64_t n_pages = (S_max + kPageTokens - 1) / kPageTokens;
    uint8_t* page = cache + ((b * Hkv + h) * n_pages + pos / kPageTokens) * kPageBytes + which * kHalfPage;
    const int tin = (int)(pos % kPageTokens);
    if (j == 0) reinterpret_cast<uint32_t*>(page + tin * (kD / 2))[lane >> 2] = word;
    if (lane == 0) {
        const uint16_t z_bits = __half_as_ushort(__float2half_rn((float)zf));    // integer 0..15: exact
        reinterpret_cast<uint32_t*>(page + kCodeBytes)[tin] = (uint32_t)s_bits | ((uint32_t)z_bits << 16);
    }
}

// Inverse of the layout (tests): one thread per (sequence, head, token, key|value, dword).
__global__ __launch_bounds__(256) void kv4_unpack_kernel(const uint8_t* __restrict__ cache, int64_t B, int64_t Hkv, int64_t S_max,
                                                         uint8_t* __restrict__ k_codes, __half* __restrict__ k_s,
                                                         __half* __restrict__ k_z, uint8_t* __restrict__ v_codes,
                                                         __half* __restrict__ v_s, __half* __restrict__ v_z)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;           // (((b * Hkv + h) * S + t) * 2 + which) * 16 + w
    if (idx >= B * Hkv * S_max * 32) return;
    const int w = (int)(idx & 15), which = (int)((idx >> 4) & 1);
    const int64_t bht = idx >> 5, t = bht % S_max, bh = bht / S_max;
    const int64_t n_pages = (S_max + kPageTokens - 1) / kPageTokens;
    const uint8_t* page = cache + (bh * n_pages + t / kPageTokens) * kPageBytes + which * kHalfPage;
    const int tin = (int)(t % kPageTokens);
    const uint32_t word = reinterpret_cast<const uint32_t*>(page + tin * (kD / 2))[w];
    uint8_t* dst = (which ? v_codes : k_codes) + bht * kD + 8 * w;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        dst[2 * j] = (uint8_t)((word >> (4 * j)) & 0xFu);
        dst[2 * j + 1] = (uint8_t)((word >> (16 + 4 * j)) & 0xFu);
    }
    if (w == 0) {
        const uint32_t prm = reinterpret_cast<const uint32_t*>(page + kCodeBytes)[tin];
        (which ? v_s : k_s)[bht] = __ushort_as_half((unsigned short)(prm & 0xFFFFu));
        (which ? v_z : k_z)[bht] = __ushort_as_half((unsigned short)(prm >> 16));
    }
}

// ------------------------------------------------------------------------------------------
// Decode attention.
// ------------------------------------------------------------------------------------------
template <int E> struct CodeWords;                       // E / 8 dwords of codes per lane and token
template <> struct CodeWords<32> { typedef uint4 type; };
template <> struct CodeWords<16> { typedef uint2 type; };
template <> struct CodeWords<8> { typedef uint32_t type; };

__device__ __forceinline__ uint32_t word_of(const uint4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
__device__ __forceinline__ uint32_t word_of(const uint2& v, int i) { return i == 0 ? v.x : v.y; }
__device__ __forceinline__ uint32_t word_of(const uint32_t& v, int) { return v; }

// pair j (elements 2j, 2j+1 of the dword) as exact FP16 integers (code - z); c = (-(1024 + z)) in both halves
__device__ __forceinline__ h2 code_pair(uint32_t word, int j, h2 c)
{
    const uint32_t bits = ((word >> (4 * j)) & 0x000F000Fu) | 0x64006400u;
    return __builtin_bit_cast(h2, bits) + c;
}

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = 4;
constexpr int kNT = 4;                                   // tokens per lane and chunk

template <int R, int E>
__global__ __launch_bounds__(kDecodeThreads) void kv4_decode_kernel(const __half* __restrict__ q, const uint8_t* __restrict__ cache,
                                                                    const int32_t* __restrict__ seq_lens, int64_t Hkv,
                                                                    int64_t S_max, __half* __restrict__ out)
{
    constexpr int LPT = kD / E;                          // lanes per token
    constexpr int TPW = 64 / LPT;                        // tokens per wave load
    constexpr int CH = kNT * TPW;                        // tokens per chunk (divides the page)
    constexpr int W = E / 8;                             // code dwords per lane and token
    constexpr int NP = kDecodeWaves * TPW;               // partial results per query head
    typedef typename CodeWords<E>::type Words;
    __shared__ float s_acc[NP][R][kD];
    __shared__ float s_m[NP][R], s_l[NP][R];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tl = lane / LPT, p = lane % LPT;
    const int64_t bh = blockIdx.x;                       // b * Hkv + hk
    const int64_t b = bh / Hkv, hk = bh % Hkv;
    const int64_t n_pages = (S_max + kPageTokens - 1) / kPageTokens;
    const int L = (int)min((int64_t)max(seq_lens[b], 0), S_max);
    const uint8_t* stream = cache + bh * n_pages * kPageBytes;
    __half* out_bh = out + (b * Hkv * R + hk * R) * kD;
    if (L == 0) {                                        // empty cache: zero rows
        for (int x = threadIdx.x; x < R * kD; x += kDecodeThreads) out_bh[x] = __float2half_rn(0.f);
        return;
    }

    // this lane's slice of every query head sharing the KV head
    h2 qv[R][E / 2];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(q + (b * Hkv * R + hk * R + r) * kD + p * E);
#pragma unroll
        for (int e = 0; e < E / 2; ++e) qv[r][e] = __builtin_bit_cast(h2, src[e]);
    }

    struct Chunk { Words kc[kNT], vc[kNT]; uint32_t kp[kNT], vp[kNT]; };
    auto load_chunk = [&](Chunk& c, int chunk) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kNT; ++i) {
            const int t = chunk * CH + i * TPW + tl;     // < n_pages * 64: inside the allocation even past L
            const uint8_t* page = stream + (int64_t)(t / kPageTokens) * kPageBytes;
            const int tin = t % kPageTokens;
            c.kc[i] = *reinterpret_cast<const Words*>(page + tin * (kD / 2) + p * (E / 2));
            c.kp[i] = reinterpret_cast<const uint32_t*>(page + kCodeBytes)[tin];
            c.vc[i] = *reinterpret_cast<const Words*>(page + kHalfPage + tin * (kD / 2) + p * (E / 2));
            c.vp[i] = reinterpret_cast<const uint32_t*>(page + kHalfPage + kCodeBytes)[tin];
        }
    };

    float m[R], l[R], acc[R][E];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        m[r] = -1e30f; l[r] = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[r][e] = 0.f;
    }
    const float kScale = 1.4426950408889634f * 0.08838834764831845f;      // log2(e) / sqrt(128)
    const int n_chunks = (L + CH - 1) / CH;

    Chunk cur;
    if (wave < n_chunks) load_chunk(cur, wave);
    for (int chunk = wave; chunk < n_chunks; chunk += kDecodeWaves) {
        Chunk nxt;
        if (chunk + kDecodeWaves < n_chunks) load_chunk(nxt, chunk + kDecodeWaves);

        float sc[R][kNT], vscale[kNT];
        h2 vz[kNT];
        bool valid[kNT];
#pragma unroll
        for (int i = 0; i < kNT; ++i) {
            valid[i] = chunk * CH + i * TPW + tl < L;
            // parameters of tokens past the end are whatever the cache holds: never let them into the arithmetic
            const uint32_t kp = valid[i] ? cur.kp[i] : 0u, vp = valid[i] ? cur.vp[i] : 0u;
            const float ks = __half2float(__ushort_as_half((unsigned short)(kp & 0xFFFFu)));
            const _Float16 kz = __builtin_bit_cast(_Float16, (unsigned short)(kp >> 16));
            const h2 kc2 = {(_Float16)(-1024.0f) - kz, (_Float16)(-1024.0f) - kz};
            vscale[i] = __half2float(__ushort_as_half((unsigned short)(vp & 0xFFFFu)));
            const _Float16 z = __builtin_bit_cast(_Float16, (unsigned short)(vp >> 16));
            vz[i] = (h2){(_Float16)(-1024.0f) - z, (_Float16)(-1024.0f) - z};
            float dot[R];
#pragma unroll
            for (int r = 0; r < R; ++r) dot[r] = 0.f;
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const uint32_t word = word_of(cur.kc[i], w);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const h2 kh = code_pair(word, j, kc2);
#pragma unroll
                    for (int r = 0; r < R; ++r) dot[r] = __builtin_amdgcn_fdot2(kh, qv[r][w * 4 + j], dot[r], false);
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
#pragma unroll
                for (int o = 1; o < LPT; o <<= 1) dot[r] += __shfl_xor(dot[r], o, 64);
                sc[r][i] = dot[r] * (ks * kScale);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float m_new = m[r];
#pragma unroll
            for (int i = 0; i < kNT; ++i) m_new = valid[i] ? fmaxf(m_new, sc[r][i]) : m_new;
            const float alpha = exp2f(m[r] - m_new);
            m[r] = m_new;
            l[r] *= alpha;
#pragma unroll
            for (int e = 0; e < E; ++e) acc[r][e] *= alpha;
#pragma unroll
            for (int i = 0; i < kNT; ++i) {
                const float pr = valid[i] ? exp2f(sc[r][i] - m_new) : 0.f;
                l[r] += pr;
                sc[r][i] = pr * vscale[i];               // weight of (code - z) of the value
            }
        }
#pragma unroll
        for (int i = 0; i < kNT; ++i) {
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const uint32_t word = word_of(cur.vc[i], w);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const h2 vh = code_pair(word, j, vz[i]);
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        acc[r][w * 8 + 2 * j] = fmaf(sc[r][i], (float)vh.x, acc[r][w * 8 + 2 * j]);
                        acc[r][w * 8 + 2 * j + 1] = fmaf(sc[r][i], (float)vh.y, acc[r][w * 8 + 2 * j + 1]);
                    }
                }
            }
        }
        cur = nxt;
    }

    // ---- partial results of all lane groups and waves meet in LDS -------------------------------
    const int slot = wave * TPW + tl;
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int e = 0; e < E; ++e) s_acc[slot][r][p * E + e] = acc[r][e];
        if (p == 0) { s_m[slot][r] = m[r]; s_l[slot][r] = l[r]; }
    }
    __syncthreads();
    for (int x = threadIdx.x; x < R * kD; x += kDecodeThreads) {
        const int r = x / kD, d = x % kD;
        float mm = -1e30f;
        for (int i = 0; i < NP; ++i) mm = fmaxf(mm, s_m[i][r]);
        float num = 0.f, den = 0.f;
        for (int i = 0; i < NP; ++i) {
            const float f = exp2f(s_m[i][r] - mm);
            num = fmaf(s_acc[i][r][d], f, num);
            den = fmaf(s_l[i][r], f, den);
        }
        out_bh[r * kD + d] = __float2half_rn(num / den);
    }
}

}  // namespace

size_t kv4_cache_bytes(int64_t B, int64_t Hkv, int64_t S_max)
{
    const int64_t n_pages = (S_max + kPageTokens - 1) / kPageTokens;
    return (size_t)(B * Hkv * n_pages) * kPageBytes;
}

hipError_t launch_kv4_append(const void* k, const void* v, const int32_t* positions, int64_t B, int64_t T, int64_t Hkv,
                             int64_t S_max, uint8_t* cache, hipStream_t s)
{
    const int64_t vecs = B * T * Hkv * 2;
    if (vecs == 0) return hipSuccess;
    kv4_append_kernel<<<(unsigned)((vecs + 3) / 4), 256, 0, s>>>(static_cast<const __half*>(k), static_cast<const __half*>(v), positions,
                                                                  B, T, Hkv, S_max, cache);
    return hipGetLastError();
}

hipError_t launch_kv4_unpack(const uint8_t* cache, int64_t B, int64_t Hkv, int64_t S_max, uint8_t* k_codes, void* k_s, void* k_z,
                             uint8_t* v_codes, void* v_s, void* v_z, hipStream_t s)
{
    const int64_t n = B * Hkv * S_max * 32;
    if (n == 0) return hipSuccess;
    kv4_unpack_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(cache, B, Hkv, S_max, k_codes, static_cast<__half*>(k_s),
                                                                   static_cast<__half*>(k_z), v_codes, static_cast<__half*>(v_s),
                                                                   static_cast<__half*>(v_z));
    return hipGetLastError();
}

hipError_t launch_kv4_decode(const void* q, const uint8_t* cache, const int32_t* seq_lens, int64_t B, int64_t H, int64_t Hkv,
                             int64_t S_max, void* out, hipStream_t s)
{
    if (B == 0) return hipSuccess;
    const dim3 grid((unsigned)(B * Hkv));
    const __half* qh = static_cast<const __half*>(q);
    __half* oh = static_cast<__half*>(out);
    switch (H / Hkv) {
        case 1: kv4_decode_kernel<1, 32><<<grid, kDecodeThreads, 0, s>>>(qh, cache, seq_lens, Hkv, S_max, oh); break;
        case 2: kv4_decode_kernel<2, 16><<<grid, kDecodeThreads, 0, s>>>(qh, cache, seq_lens, Hkv, S_max, oh); break;
        case 4: kv4_decode_kernel<4, 8><<<grid, kDecodeThreads, 0, s>>>(qh, cache, seq_lens, Hkv, S_max, oh); break;
        case 8: kv4_decode_kernel<8, 8><<<grid, kDecodeThreads, 0, s>>>(qh, cache, seq_lens, Hkv, S_max, oh); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace qoq
