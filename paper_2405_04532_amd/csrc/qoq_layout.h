// Packed-weight blob layout for gfx950 (internal to the library).
//
// Idea kept from Section 5.2.1 of arXiv 2405.04532: weights (and their level-2 scales and
// zeros) are stored in the order the matrix-core instruction consumes them, so each lane
// fetches its operands with one 128-bit load and no per-fragment address arithmetic.  The
// map itself is new: it is laid out for the operand fragments of v_mfma_i32_16x16x64_i8.
//
// Blob = [header 256 B][codes][meta][scales][zeros], every section 256-byte aligned.
//
// codes: "units" of 1 KiB = 16 physical rows x 128 k (one quantization group per row).
//   unit(nf, g) at ((nf * K/128) + g) * 1024, nf = physical 16-row fragment, g = group.
//   Inside a unit lane l = kb*16 + i (i = physical row in the fragment, kb = 0..3) owns the
//   16 bytes at l*16 = dwords d0..d3.  d0,d1 feed the MFMA of k-step 0 (k_local 0..63),
//   d2,d3 k-step 1 (k_local 64..127).  In a k-step the lane covers k_local%64 = kb*16 + t,
//   t = 0..15, and code t sits in dword (t >> 3) at bit 8*(t & 3) + 4*((t & 7) >> 2):
//   the low nibbles of a dword are operand bytes t = 0..3, the high nibbles t = 4..7, so
//   `x & 0x0F0F0F0F` and `(x >> 4) & 0x0F0F0F0F` are whole operand registers (the
//   three-operation unpack of Section 5.2.2).
//   Physical row (nf, i) holds logical output channel
//       n = (nf / 4) * 64 + 16 * (i / 4) + 4 * (nf % 4) + (i % 4)
//   so that after the MFMA (lane group q = lane/16 holds rows 4q..4q+3 of each fragment) one
//   lane owns 16 consecutive logical n of a 64-channel block: 32-byte FP16 row segments.
//
// meta (group mode): 16 x uint16 per (group, fragment), group-major: entry ((g * N/16 + nf) * 16 + i),
//   so the metadata of neighbouring fragments for one group is contiguous;
//   entry = s1 | (bias << 8) with
//   bias = (128 - z * s1) & 0xFF, the byte constant of the subtraction-after-multiplication
//   dequantizer (Section 5.2.3): code * s1 + bias == w_hat + 128 in every byte, no carries.
// scales: FP16 [N] in logical order (s0, or sw in per-channel mode).
// zeros (per-channel mode): uint8 [N] in logical order.
#pragma once
#include <stddef.h>
#include <stdint.h>

#ifdef __HIPCC__
#define QOQ_HD __host__ __device__ inline
#else
#define QOQ_HD inline
#endif

namespace qoq {

constexpr int kGroup = 128;
constexpr uint32_t kMagic = 0x57514F51u;  // "QOQW"
constexpr uint32_t kVersion = 1;
constexpr size_t kHeaderBytes = 256;

struct BlobHeader {
    uint32_t magic, version;
    int64_t N, K;
    int32_t mode, group;
    uint64_t codes_off, meta_off, scale_off, zero_off, total;
};

struct BlobLayout {
    int64_t N, K, G;
    int mode;
    size_t codes_off, meta_off, scale_off, zero_off, total;
};

QOQ_HD size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

QOQ_HD bool shape_ok(int64_t N, int64_t K, int mode)
{
    return N > 0 && K > 0 && (K % kGroup) == 0 && (N % 64) == 0 && (mode == 0 || mode == 1) &&
           N <= (1 << 24) && K <= (1 << 24);
}

QOQ_HD BlobLayout make_layout(int64_t N, int64_t K, int mode)
{
    BlobLayout L;
    L.N = N; L.K = K; L.G = K / kGroup; L.mode = mode;
    L.codes_off = kHeaderBytes;
    L.meta_off = align256(L.codes_off + (size_t)N * (size_t)K / 2);
    size_t meta_bytes = mode == 0 ? (size_t)N * (size_t)L.G * 2 : 0;
    L.scale_off = align256(L.meta_off + meta_bytes);
    L.zero_off = align256(L.scale_off + (size_t)N * 2);
    size_t zero_bytes = mode == 1 ? (size_t)N : 0;
    L.total = align256(L.zero_off + zero_bytes);
    return L;
}

// Does a header read back from a blob describe exactly the layout `L` (same shape, mode and section offsets)?
QOQ_HD bool header_matches(const BlobHeader& h, const BlobLayout& L)
{
    return h.magic == kMagic && h.version == kVersion && h.N == L.N && h.K == L.K && h.mode == L.mode &&
           h.group == kGroup && h.codes_off == L.codes_off && h.meta_off == L.meta_off && h.scale_off == L.scale_off &&
           h.zero_off == L.zero_off && h.total == L.total;
}

// logical output channel -> (physical fragment, row in fragment)
QOQ_HD void phys_row(int64_t n, int64_t& nf, int& i)
{
    const int r = (int)(n & 63);
    nf = (n >> 6) * 4 + ((r & 15) >> 2);
    i = 4 * (r >> 4) + (r & 3);
}

QOQ_HD int64_t logical_row(int64_t nf, int i)
{
    return (nf >> 2) * 64 + 16 * (i >> 2) + 4 * (nf & 3) + (i & 3);
}

// Byte offset (inside the codes section) of the dword holding code (nf, i, g, k_local) and
// the bit position of its nibble.
QOQ_HD size_t code_dword_offset(int64_t nf, int i, int64_t g, int64_t G, int k_local, int& shift)
{
    const int s = k_local >> 6, kb = (k_local >> 4) & 3, t = k_local & 15;
    shift = 8 * (t & 3) + 4 * ((t & 7) >> 2);
    return ((size_t)(nf * G + g) * 64 + (size_t)(kb * 16 + i)) * 16 + (size_t)(2 * s + (t >> 3)) * 4;
}

QOQ_HD size_t meta_offset(int64_t nf, int i, int64_t g, int64_t nf_total)
{
    return ((size_t)(g * nf_total + nf) * 16 + (size_t)i) * 2;
}

}  // namespace qoq
