// KV4 cache and decode attention for gfx950 (Sections 5.1 "KV Cache Management" and 5.3 of arXiv 2405.04532,
// re-designed for CDNA4).
//
// Cache.  Keys and values are quantized when they are written: per token and KV head, Eq. 1 with 4 bits on the
// range of that head's 128 values widened to contain 0, FP16 scale s and integer zero z (stored as the FP16
// number -(1024 + z), the form the decode kernel consumes).  A
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
//   value codes: stored tile by tile (16 tokens x 128 elements = 1 KiB) in the order the matrix instruction that
//   forms P.V wants its operand: lane l = 16 kb + r of a wave owns the 16 bytes at 16 l; its dword 2u + h holds, for
//   the four elements d = 4 (r + 16 u) + j (nibble j), token 4 kb + 2h in the low half and token 4 kb + 2h + 1 in the
//   high half.  The same unpacking then yields FP16 pairs (token, next token) of one element, and two such pairs are
//   the four k-values of an MFMA operand row.  A token still owns whole 16-bit words (32 of them), so appending a
//   token is 32 plain 2-byte stores.
//
// Decode kernel.  One workgroup of four waves per (sequence, KV head); every wave streams chunks of the sequence,
// 16-token tiles at a time, and both products run on v_mfma_f32_16x16x16_f16 (FP16 operands, FP32 sums):
//   S[token][head]  = sum_d (code - z_K)[token][d] * q[head][d]     A = unpacked keys, B = the queries of the up
//                                                                    to 16 heads that share the KV head (GQA
//                                                                    costs nothing extra), 8 MFMAs per tile
//   score = S * s_K[token] * log2(e) / sqrt(D); online softmax in base 2
//   O[d][head]     += sum_token (code - z_V)[token][d] * (p * s_V)[token][head]    8 MFMAs per tile
// The output layout of the first product (a lane holds 4 tokens of one head) is exactly the operand layout of the
// second, so the softmax runs in place and nothing moves between lanes except the running maximum.  The paper's
// kernel computes on scalar cores and fights their compute roof (Section 5.3: FP16 instead of FP32 arithmetic,
// two-operation dequantization); here the two-operation dequantization is kept and the multiply-adds go to the
// matrix cores, which leaves the vector pipe with the unpacking and the softmax only.
// The scale/zero words of a chunk are loaded together with its codes, one chunk ahead of the arithmetic (the
// prefetch of the dequantization parameters of Section 5.3).  Partial (max, sum, acc) of the four waves meet in LDS.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

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

// byte offset, inside the value codes of a page, of the 16-bit word of token `tin` (0..63) and elements 4 q4 .. 4 q4 + 3
__device__ __forceinline__ int v_word_offset(int tin, int q4)
{
    const int tile = tin >> 4, kb = (tin >> 2) & 3, h = (tin >> 1) & 1, half = tin & 1;
    const int r = q4 & 15, u = q4 >> 4;
    return tile * 1024 + (kb * 16 + r) * 16 + (2 * u + h) * 4 + half * 2;
}

// ------------------------------------------------------------------------------------------
// Append: one wave per (sequence, KV head, aligned quad of token positions); 16 lanes per token, lane w of a token
// holds its elements 8w .. 8w+7 (one 16-byte load), keys first, then values.  A quad of tokens is 4 x 64
// contiguous bytes of key codes and ONE contiguous 256-byte block of value codes (the value layout groups the
// four tokens of an operand k-block), which a complete quad assembles in LDS and writes with 16-byte stores; a
// quad that this call covers only in part (a decode step appends a single token) writes its own 2-byte words.
// Every decision is taken as the reference definition takes it: s = FP16((hi - lo) / 15) by one exact rounding
// of the FP64 quotient, z and the codes by floor(t + 1/2) decided exactly from FP32 quotients (below).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void kv4_append_kernel(const __half* __restrict__ k, const __half* __restrict__ v,
                                                         const int32_t* __restrict__ positions, int64_t B, int64_t T,
                                                         int64_t Hkv, int64_t S_max, int64_t quads, uint8_t* __restrict__ cache)
{
    __shared__ uint4 s_block[4][16];                                       // per wave: the value codes of its quad
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 4, w = lane & 15;                                // token of the quad, 16-byte chunk of its row
    const int64_t item = (int64_t)blockIdx.x * 4 + wave;                   // (b * Hkv + h) * quads + j
    if (item >= B * Hkv * quads) return;
    const int64_t j = item % quads, bh = item / quads, h = bh % Hkv, b = bh / Hkv;
    const int64_t p0 = positions[b];
    const int64_t pos = ((p0 >> 2) + j) * 4 + g;                           // floor(p0 / 4) also for negative p0
    const int64_t t = pos - p0;
    const bool valid = t >= 0 && t < T && pos >= 0 && pos < S_max;         // outside the call or the cache: not written
    const bool whole = __builtin_amdgcn_ballot_w64(valid) == ~0ull;
    if (__builtin_amdgcn_ballot_w64(valid) == 0) return;
    const int64_t n_pages = (S_max + kPageTokens - 1) / kPageTokens;
    const int64_t pos_c = valid ? pos : 0;
    uint8_t* page = cache + (bh * n_pages + pos_c / kPageTokens) * kPageBytes;
    const int tin = (int)(pos_c % kPageTokens);
    const int64_t row = ((b * T + (valid ? t : 0)) * Hkv + h) * kD;

#pragma unroll
    for (int which = 0; which < 2; ++which) {
        const uint4 raw = reinterpret_cast<const uint4*>((which ? v : k) + row)[w];
        const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            x[e] = __half2float(__ushort_as_half((unsigned short)(rw[e >> 1] >> (16 * (e & 1)))));
        float lo = 0.f, hi = 0.f;                                          // the range is widened to contain 0
#pragma unroll
        for (int e = 0; e < 8; ++e) { lo = fminf(lo, x[e]); hi = fmaxf(hi, x[e]); }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            lo = fminf(lo, __shfl_xor(lo, o, 64));
            hi = fmaxf(hi, __shfl_xor(hi, o, 64));
        }
        uint16_t s_bits = double_to_half_rne(((double)hi - (double)lo) / 15.0);
        if ((s_bits & 0x7FFFu) == 0) s_bits = 0x3C00u;                     // all-zero vector: s = 1
        // floor(x / s + 1/2) from the correctly rounded FP32 quotient q of two FP16 numbers: its integer part and
        // the comparison of its fractional part with 1/2 are both exact, and q lies on the same side of every
        // half-integer as x / s does (an exact tie is representable and divides exactly; otherwise x / s is at
        // least 2^-22 from a half-integer below 1 and 2^-12 above, at least four times FP32's rounding error
        // there).  The integer zero point is added afterwards, in integers.
        const float sc = __half2float(__ushort_as_half(s_bits));
        auto round_half_up = [](float q) { const float f = floorf(q); return (int)f + (q - f >= 0.5f ? 1 : 0); };
        const int zi = min(max(round_half_up(-lo / sc), 0), 15);
        uint32_t c[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) c[e] = (uint32_t)min(max(round_half_up(x[e] / sc) + zi, 0), 15);
        if (which == 0) {
            // keys: dword w = elements 8w .. 8w+7, element 8w+2j in nibble j of the low half, 8w+2j+1 of the high half
            uint32_t word = 0;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) word |= (c[2 * jj] << (4 * jj)) | (c[2 * jj + 1] << (16 + 4 * jj));
            if (valid) reinterpret_cast<uint32_t*>(page + tin * (kD / 2))[w] = word;
        } else {
            // values: 16-bit words of element quads 2w (elements 8w .. 8w+3) and 2w+1
            const uint32_t h0 = c[0] | (c[1] << 4) | (c[2] << 8) | (c[3] << 12);
            const uint32_t h1 = c[4] | (c[5] << 4) | (c[6] << 8) | (c[7] << 12);
            if (whole) {
                // inside the quad's 256-byte block: chunk r = q4 % 16, dword 2 (q4 / 16) + (g >> 1), half g & 1
                uint16_t* blk = reinterpret_cast<uint16_t*>(&s_block[wave][0]);
                const int q4a = 2 * w, q4b = 2 * w + 1;
                blk[(q4a & 15) * 8 + (2 * (q4a >> 4) + (g >> 1)) * 2 + (g & 1)] = (uint16_t)h0;
                blk[(q4b & 15) * 8 + (2 * (q4b >> 4) + (g >> 1)) * 2 + (g & 1)] = (uint16_t)h1;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // the wave's own LDS writes, then its reads
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                if (lane < 16) {
                    const int tin0 = tin & ~3;                             // lanes 0..15 are token 0 of the quad: tin % 4 == 0
                    uint8_t* dst = page + kHalfPage + (tin0 >> 4) * 1024 + (((tin0 >> 2) & 3) * 16 + lane) * 16;
                    *reinterpret_cast<uint4*>(dst) = s_block[wave][lane];
                }
            } else if (valid) {
                *reinterpret_cast<uint16_t*>(page + kHalfPage + v_word_offset(tin, 2 * w)) = (uint16_t)h0;
                *reinterpret_cast<uint16_t*>(page + kHalfPage + v_word_offset(tin, 2 * w + 1)) = (uint16_t)h1;
            }
        }
        if (valid && w == 0) {
            // the zero point is stored as the FP16 number -(1024 + z) (an exact integer), the constant the decode
            // kernel adds to its unpacked codes
            const uint16_t z_bits = __half_as_ushort(__float2half_rn(-1024.0f - (float)zi));
            reinterpret_cast<uint32_t*>(page + which * kHalfPage + kCodeBytes)[tin] = (uint32_t)s_bits | ((uint32_t)z_bits << 16);
        }
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
#pragma unroll
        for (int i = 0; i < 2; ++i) {                     // elements 8w + 4i .. + 3 sit in one 16-bit word
            const uint32_t half = *reinterpret_cast<const uint16_t*>(page + v_word_offset(tin, 2 * w + i));
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[4 * i + j] = (uint8_t)((half >> (4 * j)) & 0xFu);
        }
    }
    if (w == 0) {
        const uint32_t prm = reinterpret_cast<const uint32_t*>(page + kCodeBytes)[tin];
        (which ? v_s : k_s)[bht] = __ushort_as_half((unsigned short)(prm & 0xFFFFu));
        (which ? v_z : k_z)[bht] = __float2half_rn(-1024.0f - __half2float(__ushort_as_half((unsigned short)(prm >> 16))));
    }
}

// ------------------------------------------------------------------------------------------
// Decode attention.
// ------------------------------------------------------------------------------------------
// the four FP16 pairs of a code dword, minus the zero point: out[j] = (nibble j of the low half, of the high half)
// c = -(1024 + z), c16 = -(64 + z) = c + 960, per half
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

typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ h4 join(h2 a, h2 b) { return __builtin_shufflevector(a, b, 0, 1, 2, 3); }
__device__ __forceinline__ _Float16 half_bits(uint32_t v) { return __builtin_bit_cast(_Float16, (unsigned short)v); }

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = 4;
constexpr int kMaxRatio = 16;                            // query heads per KV head: the columns of one MFMA

constexpr int kPartial = kD + 2;                         // floats per (split, head): 128 sums, the maximum, the weight sum

// NTL tiles of 16 tokens per chunk.  SPLIT: the sequence is cut into gridDim.y contiguous ranges of chunks, one
// workgroup each, whose (unnormalised sums, maximum, weight sum) go to the workspace for kv4_combine_kernel; used
// when there are too few (sequence, KV head) pairs to fill the chip (grouped-query models).
template <int NTL, bool SPLIT>
__global__ __launch_bounds__(kDecodeThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void kv4_decode_kernel(const __half* __restrict__ q, const uint8_t* __restrict__ cache,
                                                                    const int32_t* __restrict__ seq_lens, int64_t Hkv, int R,
                                                                    int64_t S_max, __half* __restrict__ out, float* __restrict__ ws)
{
    constexpr int CH = 16 * NTL;                         // tokens per chunk (divides the page)
    __shared__ float s_acc[kDecodeWaves][kMaxRatio][kD];
    __shared__ float s_m[kDecodeWaves][kMaxRatio], s_l[kDecodeWaves][kMaxRatio];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r16 = lane & 15, kb = lane >> 4;           // operand row (token / element slot / head) and k-block
    const int64_t bh = blockIdx.x;                       // b * Hkv + hk
    const int64_t b = bh / Hkv, hk = bh % Hkv;
    const int64_t n_pages = (S_max + kPageTokens - 1) / kPageTokens;
    const int L_seq = (int)min((int64_t)max(seq_lens[b], 0), S_max);
    const uint8_t* stream = cache + bh * n_pages * kPageBytes;
    __half* out_bh = out + (b * Hkv + hk) * R * kD;
    float* ws_bh = SPLIT ? ws + ((size_t)bh * gridDim.y + blockIdx.y) * R * kPartial : nullptr;
    // this workgroup's range of chunks [c0, c1) and the length it masks against
    const int chunks_seq = (L_seq + CH - 1) / CH;
    const int per_split = SPLIT ? (chunks_seq + (int)gridDim.y - 1) / (int)gridDim.y : chunks_seq;
    const int c0 = SPLIT ? min(chunks_seq, (int)blockIdx.y * per_split) : 0;
    const int c1 = SPLIT ? min(chunks_seq, c0 + per_split) : chunks_seq;
    const int L = min(L_seq, c1 * CH);
    if (c0 >= c1) {                                      // nothing to attend to: zero rows / an empty partial result
        for (int x = threadIdx.x; x < R * (SPLIT ? kPartial : kD); x += kDecodeThreads) {
            if (SPLIT) ws_bh[x] = x % kPartial == kD ? -1e30f : 0.f;
            else out_bh[x] = __float2half_rn(0.f);
        }
        return;
    }

    // B operand of S = K q^T: column r16 = query head, k-block kb = elements 32 kb .. 32 kb + 31 (heads >= R: zero)
    h2 qv[16];
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(q + ((b * Hkv + hk) * R + min(r16, R - 1)) * kD + kb * 32);
#pragma unroll
        for (int e = 0; e < 16; ++e) qv[e] = __builtin_bit_cast(h2, r16 < R ? src[e] : 0u);
    }

    struct Chunk {
        uint4 kc[NTL];      // keys: token r16 of the tile, elements 32 kb ..
        uint4 vc[NTL];      // values: this lane's 16 bytes of the tile
        uint32_t kz[NTL];   // (s, z) of token r16 (zero point for unpacking)
        uint4 ks[NTL];      // (s, z) of tokens 4 kb .. 4 kb + 3 (scales of the scores this lane receives)
        uint4 vp[NTL];      // (s, z) of tokens 4 kb .. 4 kb + 3 of the values
    };
    // Every address is a wave-uniform tile base plus a lane offset that never changes: the five loads of a tile
    // cost no vector address arithmetic.
    const uint32_t off_kc = (uint32_t)(r16 * (kD / 2) + kb * 16), off_kz = (uint32_t)(kCodeBytes + r16 * 4);
    const uint32_t off_ks = (uint32_t)(kCodeBytes + kb * 16), off_vc = (uint32_t)(kHalfPage + lane * 16);
    const uint32_t off_vp = (uint32_t)(kHalfPage + kCodeBytes + kb * 16);
    auto load_chunk = [&](Chunk& c, int chunk) __attribute__((always_inline)) {
#pragma unroll
        for (int tt = 0; tt < NTL; ++tt) {
            const int t0 = __builtin_amdgcn_readfirstlane(chunk * CH + tt * 16);   // < n_pages * 64: inside the allocation
            const uint8_t* page = stream + (int64_t)(t0 / kPageTokens) * kPageBytes;
            const int tin = t0 % kPageTokens;            // first token of the tile inside its page (a multiple of 16)
            const uint8_t* codes = page + tin * (kD / 2);          // key codes of the tile; its value codes lie 4352 further
            const uint8_t* prm = page + tin * 4;                   // (s, z) words of the tile
            c.kc[tt] = *reinterpret_cast<const uint4*>(codes + off_kc);
            c.kz[tt] = *reinterpret_cast<const uint32_t*>(prm + off_kz);
            c.ks[tt] = *reinterpret_cast<const uint4*>(prm + off_ks);
            c.vc[tt] = *reinterpret_cast<const uint4*>(codes + off_vc);
            c.vp[tt] = *reinterpret_cast<const uint4*>(prm + off_vp);
        }
    };

    float m = -1e30f, l = 0.f;                           // of head r16, over the tokens this lane has seen
    f4 acc[8];                                           // acc[4u + j][x]: element d = 16 kb + 4x + 64u + j of head r16
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = (f4){0.f, 0.f, 0.f, 0.f};
    const float kScale = 1.4426950408889634f * 0.08838834764831845f;      // log2(e) / sqrt(128)
    const int n_chunks = c1;                             // chunk indices past the range are clamped to its last chunk

    const h2 k960 = {(_Float16)960.0f, (_Float16)960.0f};
    // One chunk of arithmetic.  MASKED: the chunk reaches past the end of the sequence (possibly entirely); the
    // parameters of tokens past the end are whatever the cache holds and must not enter the arithmetic.
    auto process_as = [&](const Chunk& cur, int chunk, auto masked_tag) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        f4 sc[NTL];
        float m_new = m;
#pragma unroll
        for (int tt = 0; tt < NTL; ++tt) {
            const int t0 = chunk * CH + tt * 16;
            uint32_t kz = cur.kz[tt];
            if (MASKED) kz = t0 + r16 < L ? kz : 0xE4000000u;               // -(1024 + 0)
            const h2 c = __builtin_bit_cast(h2, __builtin_amdgcn_perm(kz, kz, 0x07060706u));   // high half in both halves
            const h2 c16 = c + k960;
            const uint32_t kw[4] = {cur.kc[tt].x, cur.kc[tt].y, cur.kc[tt].z, cur.kc[tt].w};
            f4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                h2 kh[4];
                unpack4(kw[w], c, c16, kh);              // kh[j] = elements 8w + 2j, 8w + 2j + 1 of this lane's 32
                d = __builtin_amdgcn_mfma_f32_16x16x16f16(join(kh[0], kh[1]), join(qv[4 * w], qv[4 * w + 1]), d, 0, 0, 0);
                d = __builtin_amdgcn_mfma_f32_16x16x16f16(join(kh[2], kh[3]), join(qv[4 * w + 2], qv[4 * w + 3]), d, 0, 0, 0);
            }
            const uint32_t sw[4] = {cur.ks[tt].x, cur.ks[tt].y, cur.ks[tt].z, cur.ks[tt].w};
#pragma unroll
            for (int x = 0; x < 4; ++x) {                // d[x] = token 4 kb + x of the tile, head r16
                const float ks = (float)half_bits(sw[x]);
                sc[tt][x] = d[x] * (ks * kScale);
                if (MASKED) sc[tt][x] = t0 + 4 * kb + x < L ? sc[tt][x] : -1e30f;
                m_new = fmaxf(m_new, sc[tt][x]);
            }
        }
        m_new = fmaxf(m_new, __shfl_xor(m_new, 16, 64));  // the four k-blocks of a head agree on the maximum
        m_new = fmaxf(m_new, __shfl_xor(m_new, 32, 64));
        if (__builtin_amdgcn_ballot_w64(m_new != m) != 0) {                  // rare once a few chunks have been seen
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            m = m_new;
            l *= alpha;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] *= alpha;
        }
#pragma unroll
        for (int tt = 0; tt < NTL; ++tt) {
            const int t0 = chunk * CH + tt * 16;
            uint32_t pw[4] = {cur.vp[tt].x, cur.vp[tt].y, cur.vp[tt].z, cur.vp[tt].w};
            float wf[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                if (MASKED) pw[x] = t0 + 4 * kb + x < L ? pw[x] : 0xE4000000u;   // scale 0, zero point 0
                // a masked score is -1e30: its weight underflows to 0 unless nothing valid has been seen yet
                // (then m is -1e30 too), which the zero scale takes care of
                const float pr = __builtin_amdgcn_exp2f(sc[tt][x] - m);
                l += MASKED ? (t0 + 4 * kb + x < L ? pr : 0.f) : pr;
                wf[x] = pr * (float)half_bits(pw[x]);
            }
            const h4 bw = {(_Float16)wf[0], (_Float16)wf[1], (_Float16)wf[2], (_Float16)wf[3]};   // B: tokens 4 kb .., head r16
            const uint32_t vw[4] = {cur.vc[tt].x, cur.vc[tt].y, cur.vc[tt].z, cur.vc[tt].w};
            h2 vh[2][2][4];                              // [u][h][j]: (token 4 kb + 2h, + 1) of element 4 (r16 + 16 u) + j
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const h2 c = __builtin_bit_cast(h2, __builtin_amdgcn_perm(pw[2 * h + 1], pw[2 * h], 0x07060302u));
                const h2 c16 = c + k960;
#pragma unroll
                for (int u = 0; u < 2; ++u) unpack4(vw[2 * u + h], c, c16, vh[u][h]);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[4 * u + j] = __builtin_amdgcn_mfma_f32_16x16x16f16(join(vh[u][0][j], vh[u][1][j]), bw, acc[4 * u + j], 0, 0, 0);
        }
    };
    auto process = [&](const Chunk& cur, int chunk) __attribute__((always_inline)) {
        if (chunk * CH + CH <= L) process_as(cur, chunk, std::false_type{});
        else process_as(cur, chunk, std::true_type{});
    };

    // Wave w takes chunks w, w + 4, ...; all waves run the same number of iterations (a wave without a chunk in
    // the last one re-reads the final chunk, masked).  Two buffers alternate, and every path through the loop
    // issues a fixed number of loads, so the compiler's wait counts are exact: while a chunk is computed the next
    // one stays in flight.  (With loads under a condition it waits for everything outstanding.)
    const int n_iter = (c1 - c0 + kDecodeWaves - 1) / kDecodeWaves;
    auto chunk_of = [&](int it) __attribute__((always_inline)) { return c0 + it * kDecodeWaves + wave; };
    auto fetch = [&](Chunk& c, int it) __attribute__((always_inline)) { load_chunk(c, min(chunk_of(it), n_chunks - 1)); };
    Chunk A, Bf;
    fetch(A, 0);
    int it = 0;
    // Only a wave's last chunk can reach past the end of the sequence: every earlier one lies before the final chunk.
    for (; it + 2 < n_iter; it += 2) {
        fetch(Bf, it + 1);
        process_as(A, chunk_of(it), std::false_type{});
        fetch(A, it + 2);
        process_as(Bf, chunk_of(it + 1), std::false_type{});
    }
    if (it + 2 == n_iter) {
        fetch(Bf, it + 1);
        process_as(A, chunk_of(it), std::false_type{});
        process(Bf, chunk_of(it + 1));
    } else {
        process(A, chunk_of(it));
    }

    // ---- the four waves' partial results meet in LDS --------------------------------------------
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (r16 < R) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int x = 0; x < 4; ++x) s_acc[wave][r16][16 * kb + 4 * x + 64 * u + j] = acc[4 * u + j][x];
        if (kb == 0) { s_m[wave][r16] = m; s_l[wave][r16] = l; }
    }
    __syncthreads();
    for (int x = threadIdx.x; x < R * kD; x += kDecodeThreads) {
        const int r = x / kD, d = x % kD;
        float mm = -1e30f;
#pragma unroll
        for (int i = 0; i < kDecodeWaves; ++i) mm = fmaxf(mm, s_m[i][r]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int i = 0; i < kDecodeWaves; ++i) {
            const float f = __builtin_amdgcn_exp2f(s_m[i][r] - mm);
            num = fmaf(s_acc[i][r][d], f, num);
            den = fmaf(s_l[i][r], f, den);
        }
        if (SPLIT) {
            ws_bh[r * kPartial + d] = num;
            if (d == 0) { ws_bh[r * kPartial + kD] = mm; ws_bh[r * kPartial + kD + 1] = den; }
        } else {
            out_bh[r * kD + d] = __float2half_rn(num / den);
        }
    }
}

// Second pass of the split variant: one workgroup of 128 threads per (sequence, query head).
__global__ __launch_bounds__(kD) void kv4_combine_kernel(const float* __restrict__ ws, int NS, int R, __half* __restrict__ out)
{
    const int64_t bh = blockIdx.x / R;                   // (sequence, KV head)
    const int r = (int)(blockIdx.x % R), d = threadIdx.x;
    const float* part = ws + (size_t)bh * NS * R * kPartial + (size_t)r * kPartial;
    float mm = -1e30f;
    for (int s = 0; s < NS; ++s) mm = fmaxf(mm, part[(size_t)s * R * kPartial + kD]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < NS; ++s) {
        const float f = __builtin_amdgcn_exp2f(part[(size_t)s * R * kPartial + kD] - mm);
        num = fmaf(part[(size_t)s * R * kPartial + d], f, num);
        den = fmaf(part[(size_t)s * R * kPartial + kD + 1], f, den);
    }
    out[(size_t)blockIdx.x * kD + d] = __float2half_rn(den > 0.f ? num / den : 0.f);
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
    if (B * T * Hkv == 0) return hipSuccess;
    const int64_t quads = (T + 3) / 4 + 1;        // aligned quads of positions a run of T tokens can touch
    const int64_t items = B * Hkv * quads;
    kv4_append_kernel<<<(unsigned)((items + 3) / 4), 256, 0, s>>>(static_cast<const __half*>(k), static_cast<const __half*>(v), positions,
                                                                   B, T, Hkv, S_max, quads, cache);
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

// Number of sequence ranges the split variant would use for this problem (1 = single pass).  Cutting the sequence pays only
// while the (sequence, KV head) pairs alone leave compute units idle: measured at 8 KV heads, 1 x 8192 tokens goes from 51 to
// 15 us with 8 ranges and 8 x 2048 from 16 to 11 us with 4, while at 64 sequences (512 pairs) every cut is slower than none
// (18.6 us whole, 22.2 in 2 ranges, 25.5 in 4): each range repeats the set-up and adds a second launch that merges them.
constexpr int64_t kDecodeFill = 256;
int kv4_decode_splits(int64_t B, int64_t Hkv, int64_t S_max)
{
    const int64_t pairs = B * Hkv;
    if (pairs <= 0) return 1;
    int64_t ns = kDecodeFill / pairs;                    // about one workgroup per compute unit
    ns = std::min<int64_t>(ns, 8);
    ns = std::min<int64_t>(ns, S_max / 512);             // ranges of at least 512 tokens
    return (int)std::max<int64_t>(ns, 1);
}

size_t kv4_decode_workspace_bytes(int64_t B, int64_t H, int64_t Hkv, int64_t S_max)
{
    const int ns = kv4_decode_splits(B, Hkv, S_max);
    return ns <= 1 ? 0 : (size_t)(B * H) * ns * kPartial * sizeof(float);
}

hipError_t launch_kv4_decode(const void* q, const uint8_t* cache, const int32_t* seq_lens, int64_t B, int64_t H, int64_t Hkv,
                             int64_t S_max, void* out, void* workspace, size_t workspace_bytes, hipStream_t s)
{
    if (B == 0) return hipSuccess;
    const __half* qh = static_cast<const __half*>(q);
    __half* oh = static_cast<__half*>(out);
    const int R = (int)(H / Hkv);
    if (R < 1 || R > kMaxRatio) return hipErrorInvalidValue;
    const int ns = kv4_decode_splits(B, Hkv, S_max);
    if (workspace && ns > 1 && workspace_bytes >= kv4_decode_workspace_bytes(B, H, Hkv, S_max)) {
        float* ws = static_cast<float*>(workspace);
        const dim3 grid((unsigned)(B * Hkv), (unsigned)ns);
        kv4_decode_kernel<2, true><<<grid, kDecodeThreads, 0, s>>>(qh, cache, seq_lens, Hkv, R, S_max, oh, ws);
        kv4_combine_kernel<<<(unsigned)(B * H), kD, 0, s>>>(ws, ns, R, oh);
        return hipGetLastError();
    }
    kv4_decode_kernel<2, false><<<dim3((unsigned)(B * Hkv)), kDecodeThreads, 0, s>>>(qh, cache, seq_lens, Hkv, R, S_max, oh, nullptr);
    return hipGetLastError();
}

}  // namespace qoq
