// KV4 cache and decode attention for gfx950 (Sections 5.1 "KV Cache Management" and 5.3 of arXiv 2405.04532,
// re-designed for CDNA4).
//
// Cache.  Keys and values are quantized when they are written: per token and KV head, Eq. 1 with 4 bits on the
// range of that head's 128 values widened to contain 0, FP16 scale s and integer zero z (stored as FP16).  A
// page holds 64 consecutive tokens of one (sequence, KV head): 4 KiB of key codes, their 64 (s, z) pairs, 4 KiB
// of value codes, their 64 pairs -- the parameters sit directly behind the codes they belong to, in the same
// page.  The pages of a (sequence, head) are contiguous.
//   key codes of a token: 16 dwords; dword w holds elements 8w .. 8w+7, element 8w+2j in bits 4j.. of the low
//   half, element 8w+2j+1 in bits 4j.. of the high half: (x >> 4j) & 0x000F000F is a pair of consecutive
//   elements, and OR 0x64006400 makes it the FP16 pair (1024 + a, 1024 + b) -- the integer-to-FP16 conversion
//   without a conversion instruction that Section 5.3 takes from earlier work.  One packed add of -(1024 + z)
//   then gives the exact integers (code - z) as FP16.  The odd nibbles need no shift: (x & 0x00F000F0) |
//   0x64006400 is (1024 + 16a, 1024 + 16b), and one packed multiply-add, * 1/16 - (64 + z), is exact too.
//   Two vector operations per pair of elements, plus one shift per dword.
//   value codes: tokens are stored in pairs (2t, 2t+1), 128 bytes per pair: dword i holds elements 4i .. 4i+3
//   of token 2t in its low half (element 4i+j in bits 4j..) and of token 2t+1 in its high half, so the same
//   unpacking yields pairs (token 2t, token 2t+1) of ONE element: the weighted sum over tokens then runs on
//   v_dot2_f32_f16 against the pair of softmax weights, two tokens per instruction.  A token still owns whole
//   16-bit words, so appending one token is 32 plain 2-byte stores.
//
// Decode kernel.  One workgroup of four waves per (sequence, KV head); all R = H / Hkv query heads that share
// the KV head are handled together, so the cache is read once.  Every wave streams chunks of the sequence;
// inside a wave a token is spread over 128 / E lanes (E = 32, 16 or 8 elements per lane, fewer when more query
// heads need registers), so a wave load covers 64 * E / 128 whole tokens = 1 KiB of contiguous cache.
//   score = (log2 e / sqrt(D)) * s_K * sum_d q_d (code_d - z_K)      v_dot2_f32_f16: FP16 products, FP32 sums
//   online softmax in base 2 per lane group (no communication between tokens inside the loop)
//   acc_d += dot2((code_d - z_V) of tokens 2t, 2t+1; FP16(p * s_V) of the same two tokens)   FP32 accumulators
// The paper moves the products of its kernel from FP32 to FP16 to lift the compute roof of its GPU; here the
// multiplications take FP16 operands and the sums stay FP32, which the dot instructions give for free.  The partial (max, sum, acc) of all lane groups and waves meet in LDS at the end.
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
    const int64_t n_pages = (S_max + kPageTokens - 1) / kPageTokens;
    uint8_t* page = cache + ((b * Hkv + h) * n_pages + pos / kPageTokens) * kPageBytes + which * kHalfPage;
    const int tin = (int)(pos % kPageTokens);
    if (which == 0) {
        // keys: dword w = lanes 4w .. 4w+3; lane 4w+j contributes pair j
        const int j = lane & 3;
        uint32_t word = (c0 << (4 * j)) | (c1 << (16 + 4 * j));
        word |= __shfl_xor(word, 1, 64);
        word |= __shfl_xor(word, 2, 64);
        if (j == 0) reinterpret_cast<uint32_t*>(page + tin * (kD / 2))[lane >> 2] = word;
    } else {
        // values: 16-bit word i = lanes 2i, 2i+1 (elements 4i .. 4i+3), in the half of dword i that belongs to this
        // token of its pair
        const int j = (lane & 1) * 2;
        uint32_t word = (c0 << (4 * j)) | (c1 << (4 * j + 4));
        word |= __shfl_xor(word, 1, 64);
        if ((lane & 1) == 0)
            reinterpret_cast<uint16_t*>(page + (tin >> 1) * kD)[(lane >> 1) * 2 + (tin & 1)] = (uint16_t)word;
    }
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
    uint8_t* dst = (which ? v_codes : k_codes) + bht * kD + 8 * w;
    if (which == 0) {
        const uint32_t word = reinterpret_cast<const uint32_t*>(page + tin * (kD / 2))[w];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            dst[2 * j] = (uint8_t)((word >> (4 * j)) & 0xFu);
            dst[2 * j + 1] = (uint8_t)((word >> (16 + 4 * j)) & 0xFu);
        }
    } else {
        const uint16_t* pair = reinterpret_cast<const uint16_t*>(page + (tin >> 1) * kD);
#pragma unroll
        for (int i = 0; i < 2; ++i) {                     // elements 8w + 4i .. + 3 sit in 16-bit word 2w + i of this token
            const uint32_t half = pair[(2 * w + i) * 2 + (tin & 1)];
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[4 * i + j] = (uint8_t)((half >> (4 * j)) & 0xFu);
        }
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
// the four FP16 pairs of a code dword, minus the zero point: out[j] = (nibble j of the low half, of the high half)
// c = -(1024 + z), c16 = -(64 + z), per half
// (x & mask) | bits in one instruction.  All three sources are vector registers: with the two constants in scalar
// registers the instruction would exceed its one-scalar-operand limit and the compiler splits it in two.
__device__ __forceinline__ h2 and_or(uint32_t x, uint32_t mask, uint32_t bits)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(mask), "v"(bits));
    return __builtin_bit_cast(h2, r);
}
__device__ __forceinline__ void unpack4(uint32_t word, h2 c, h2 c16, h2 (&out)[4])
{
    const h2 sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    const uint32_t hi = word >> 8;
    out[0] = and_or(word, 0x000F000Fu, 0x64006400u) + c;
    out[1] = and_or(word, 0x00F000F0u, 0x64006400u) * sixteenth + c16;
    out[2] = and_or(hi, 0x000F000Fu, 0x64006400u) + c;
    out[3] = and_or(hi, 0x00F000F0u, 0x64006400u) * sixteenth + c16;
}

__device__ __forceinline__ h2 pack_rne(float a, float b) { return (h2){(_Float16)a, (_Float16)b}; }

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = 4;
constexpr int kNT = 4;                                   // tokens (two pairs) per lane and chunk

// E elements per lane: a token (pair) is spread over 128 / E lanes.
template <int R, int E>
__global__ __launch_bounds__(kDecodeThreads) void kv4_decode_kernel(const __half* __restrict__ q, const uint8_t* __restrict__ cache,
                                                                    const int32_t* __restrict__ seq_lens, int64_t Hkv,
                                                                    int64_t S_max, __half* __restrict__ out)
{
    constexpr int LPT = kD / E;                          // lanes per token
    constexpr int TPW = 64 / LPT;                        // lane groups = tokens per wave load of keys
    constexpr int CH = kNT * TPW;                        // tokens per chunk (divides the page)
    constexpr int WK = E / 8;                            // key dwords per lane and token
    constexpr int WV = E / 4;                            // value dwords per lane and token pair
    constexpr int NP = kDecodeWaves * TPW;               // partial results per query head
    static_assert(E == 32 || E == 16 || E == 8, "elements per lane");
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

    // A lane group handles two token pairs per chunk: pairs tl and tl + TPW of the chunk's 2 * TPW pairs.
    struct Chunk { uint32_t kc[kNT][WK], vc[2][WV], kp[kNT], vp[kNT]; };
    auto load_chunk = [&](Chunk& c, int chunk) __attribute__((always_inline)) {
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
            const int t0 = chunk * CH + 2 * (tl + pr * TPW);   // < n_pages * 64: inside the allocation even past L
            const uint8_t* page = stream + (int64_t)(t0 / kPageTokens) * kPageBytes;
            const int tin = t0 % kPageTokens;            // even
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint32_t* kw = reinterpret_cast<const uint32_t*>(page + (tin + u) * (kD / 2) + p * (E / 2));
#pragma unroll
                for (int w = 0; w < WK; ++w) c.kc[2 * pr + u][w] = kw[w];
                c.kp[2 * pr + u] = reinterpret_cast<const uint32_t*>(page + kCodeBytes)[tin + u];
                c.vp[2 * pr + u] = reinterpret_cast<const uint32_t*>(page + kHalfPage + kCodeBytes)[tin + u];
            }
            const uint32_t* vw = reinterpret_cast<const uint32_t*>(page + kHalfPage + (tin >> 1) * kD + p * E);
#pragma unroll
            for (int w = 0; w < WV; ++w) c.vc[pr][w] = vw[w];
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

    // One chunk of arithmetic.  `chunk` may lie past the end of the sequence (then every token is masked).
    auto process = [&](const Chunk& cur, int chunk) __attribute__((always_inline)) {
        float sc[R][kNT], vscale[kNT];
        _Float16 vzero[kNT];
        bool valid[kNT];
#pragma unroll
        for (int i = 0; i < kNT; ++i) {
            valid[i] = chunk * CH + 2 * (tl + (i >> 1) * TPW) + (i & 1) < L;
            // parameters of tokens past the end are whatever the cache holds: never let them into the arithmetic
            const uint32_t kp = valid[i] ? cur.kp[i] : 0u, vp = valid[i] ? cur.vp[i] : 0u;
            const float ks = __half2float(__ushort_as_half((unsigned short)(kp & 0xFFFFu)));
            const _Float16 kz = __builtin_bit_cast(_Float16, (unsigned short)(kp >> 16));
            const h2 c = {(_Float16)(-1024.0f) - kz, (_Float16)(-1024.0f) - kz};
            const h2 c16 = {(_Float16)(-64.0f) - kz, (_Float16)(-64.0f) - kz};
            vscale[i] = __half2float(__ushort_as_half((unsigned short)(vp & 0xFFFFu)));
            vzero[i] = __builtin_bit_cast(_Float16, (unsigned short)(vp >> 16));
            float dot[R];
#pragma unroll
            for (int r = 0; r < R; ++r) dot[r] = 0.f;
#pragma unroll
            for (int w = 0; w < WK; ++w) {
                h2 kh[4];
                unpack4(cur.kc[i][w], c, c16, kh);       // kh[j] = elements 8w + 2j, 8w + 2j + 1
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int r = 0; r < R; ++r) dot[r] = __builtin_amdgcn_fdot2(kh[j], qv[r][w * 4 + j], dot[r], false);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
#pragma unroll
                for (int o = 1; o < LPT; o <<= 1) dot[r] += __shfl_xor(dot[r], o, 64);
                sc[r][i] = dot[r] * (ks * kScale);
            }
        }
        h2 wgt[R][2];                                    // FP16 weights (p * s_V) of the two tokens of each pair
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
            float wf[kNT];
#pragma unroll
            for (int i = 0; i < kNT; ++i) {
                const float pr = valid[i] ? exp2f(sc[r][i] - m_new) : 0.f;
                l[r] += pr;
                wf[i] = pr * vscale[i];
            }
            wgt[r][0] = pack_rne(wf[0], wf[1]);
            wgt[r][1] = pack_rne(wf[2], wf[3]);
        }
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
            const h2 c = {(_Float16)(-1024.0f) - vzero[2 * pr], (_Float16)(-1024.0f) - vzero[2 * pr + 1]};
            const h2 c16 = {(_Float16)(-64.0f) - vzero[2 * pr], (_Float16)(-64.0f) - vzero[2 * pr + 1]};
#pragma unroll
            for (int w = 0; w < WV; ++w) {
                h2 vh[4];
                unpack4(cur.vc[pr][w], c, c16, vh);      // vh[j] = element 4w + j of the pair's two tokens
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        acc[r][w * 4 + j] = __builtin_amdgcn_fdot2(vh[j], wgt[r][pr], acc[r][w * 4 + j], false);
            }
        }
    };

    // Wave w takes chunks w, w + 4, ...; all waves run the same number of iterations (a wave without a chunk in
    // the last one re-reads the final chunk, masked).  Two buffers alternate, and every path through the loop
    // issues a fixed number of loads, so the compiler's wait counts are exact: while a chunk is computed the next
    // one stays in flight.  (With loads under a condition it waits for everything outstanding.)
    const int n_iter = (n_chunks + kDecodeWaves - 1) / kDecodeWaves;
    auto chunk_of = [&](int it) __attribute__((always_inline)) { return it * kDecodeWaves + wave; };
    auto fetch = [&](Chunk& c, int it) __attribute__((always_inline)) { load_chunk(c, min(chunk_of(it), n_chunks - 1)); };
    Chunk A, Bf;
    fetch(A, 0);
    int it = 0;
    for (; it + 2 < n_iter; it += 2) {
        fetch(Bf, it + 1);
        process(A, chunk_of(it));
        fetch(A, it + 2);
        process(Bf, chunk_of(it + 1));
    }
    if (it + 2 == n_iter) {
        fetch(Bf, it + 1);
        process(A, chunk_of(it));
        process(Bf, chunk_of(it + 1));
    } else {
        process(A, chunk_of(it));
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
