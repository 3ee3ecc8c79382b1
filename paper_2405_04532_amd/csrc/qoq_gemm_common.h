// Pieces shared by the translation units of the W4A8 GEMM kernels (internal to the library): kernel arguments,
// the register dequantizer (Sections 5.2.2-5.2.3 of arXiv 2405.04532), the epilogue of four channels of one token
// (Section 5.2.2, Eq. 5-7) and the fence-free loads and stores of the cross-workgroup hand-over.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qoq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kNFrag = 4;  // 16-row fragments per wave = 64 output channels

struct GemmDev {
    const int8_t* qx;
    const uint4* codes;
    const uint16_t* meta;
    const __half* scales;
    const uint8_t* zeros;
    const __half* sx;
    const int32_t* rowsum;
    __half* out16;
    int32_t* out32;
    int* counters;  // split-k: one per output tile, zero on entry and on exit
    int4* parts;    // split-k: [tile][split][value][thread]
    int M, N, K, G, gps, S;  // gps = groups per k-split, S = number of k-splits (tiled kernel)
    int upw;                 // stream kernel: work units per workgroup
    int token_sum;           // per-channel FP16 epilogue in the token-sum form: `rowsum` then holds the FP32 sums t_X
};

enum { OUT_FP16 = 0, OUT_I32 = 1 };

__device__ inline uint32_t pk_mad_u16(uint32_t a, uint32_t s, uint32_t b)
{
    us2 r = __builtin_bit_cast(us2, a) * __builtin_bit_cast(us2, s) + __builtin_bit_cast(us2, b);
    return __builtin_bit_cast(uint32_t, r);
}

// Two packed dwords (16 codes) -> one 16-byte INT8 MFMA operand.
template <bool GROUP>
__device__ inline v4i dequant(uint32_t x0, uint32_t x1, uint32_t S, uint32_t B)
{
    const uint32_t m = 0x0F0F0F0Fu;
    uint32_t o0 = x0 & m, o1 = (x0 >> 4) & m, o2 = x1 & m, o3 = (x1 >> 4) & m;
    if (GROUP) {
        const uint32_t sign = 0x80808080u;
        o0 = pk_mad_u16(o0, S, B) ^ sign;
        o1 = pk_mad_u16(o1, S, B) ^ sign;
        o2 = pk_mad_u16(o2, S, B) ^ sign;
        o3 = pk_mad_u16(o3, S, B) ^ sign;
    }
    v4i r;
    r.x = (int)o0; r.y = (int)o1; r.z = (int)o2; r.w = (int)o3;
    return r;
}

__device__ inline v4i as_v4i(uint4 t) { return (v4i){(int)t.x, (int)t.y, (int)t.z, (int)t.w}; }

// Direct global -> LDS copy, 16 (or 4) bytes per lane; lane l lands at lds_addr + 16*l (4*l).
// `base` is wave-uniform, `voff` the lane's byte offset.  Opaque to the compiler on purpose.
// M0 (the copy's LDS base) is a reserved register that nothing else in these kernels uses, so
// it is not listed as a clobber.
__device__ __forceinline__ const void* to_sgpr(const void* ptr)   // value is wave-uniform; pin it to scalar registers
{
    const uint64_t v = reinterpret_cast<uint64_t>(ptr);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ void dma16(const void* base, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(to_sgpr(base)) : "memory");
}
__device__ __forceinline__ void dma4(const void* base, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(to_sgpr(base)) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
// Bank swizzle of activation rows kept in LDS as whole 128-byte lines (eight 16-byte chunks per token row): chunk c
// of row r is stored at chunk position c ^ row_swizzle(r).  The LDS of gfx950 has 64 banks of 4 bytes and serves
// a 16-byte fragment read 16 lanes at a time; those lanes take the same chunk of 16 consecutive rows, i.e. 8 even
// rows (first half of the banks) and 8 odd ones (second half), and (r >> 1) & 7 gives each of the eight a different
// position.  (Measured: swizzles that only use r & 7 leave two-way conflicts on every such read.)
__device__ __forceinline__ int row_swizzle(int r) { return (r >> 1) & 7; }   // r = row % 16

// Compiler-visible write-through store / cache-bypassing load (two relaxed device-scope 8-byte atomics each): the
// compiler tracks their registers and waits itself.  For code with no copy queue to preserve, and wherever
// control flow lies between a load and its use (the compiler may copy a register it believes already loaded).
__device__ __forceinline__ void store_through(int4* ptr, int a, int b, int c, int d)
{
    unsigned long long* q = reinterpret_cast<unsigned long long*>(ptr);
    __hip_atomic_store(q, (unsigned long long)(uint32_t)a | ((unsigned long long)(uint32_t)b << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(q + 1, (unsigned long long)(uint32_t)c | ((unsigned long long)(uint32_t)d << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ v4i load_through(const int4* ptr)
{
    unsigned long long* q = const_cast<unsigned long long*>(reinterpret_cast<const unsigned long long*>(ptr));
    const unsigned long long lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return (v4i){(int)(uint32_t)lo, (int)(uint32_t)(lo >> 32), (int)(uint32_t)hi, (int)(uint32_t)(hi >> 32)};
}
template <bool GROUP, int OUT>
__device__ __forceinline__ void finish4(const GemmDev& p, int m, int n0, v4i v, const float (&sn)[4],
                                        const int (&zn)[4], float sxm, int rs)
{
    int t[4] = {v.x, v.y, v.z, v.w};
    // Per-channel zero point: exact integer fold acc - z * rowsum (Eq. 6), or, in the token-sum form (Eq. 7),
    // acc * sx * s - t_X * (z * s) in FP32 with `rs` carrying the bits of t_X.
    const bool token_sum = !GROUP && OUT == OUT_FP16 && p.token_sum;
    if constexpr (!GROUP) {
        if (!token_sum) {
#pragma unroll
            for (int j = 0; j < 4; ++j) t[j] -= zn[j] * rs;
        }
    }
    if constexpr (OUT == OUT_I32) {
        *reinterpret_cast<int4*>(p.out32 + (size_t)m * p.N + n0) = make_int4(t[0], t[1], t[2], t[3]);
    } else {
        const float txm = __int_as_float(rs);
        uint32_t h[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            float ra = (float)t[2 * j] * (sxm * sn[2 * j]), rb = (float)t[2 * j + 1] * (sxm * sn[2 * j + 1]);
            if (token_sum) {
                ra -= txm * ((float)zn[2 * j] * sn[2 * j]);
                rb -= txm * ((float)zn[2 * j + 1] * sn[2 * j + 1]);
            }
            const __half a = __float2half_rn(ra);
            const __half b = __float2half_rn(rb);
            h[j] = (uint32_t)__half_as_ushort(a) | ((uint32_t)__half_as_ushort(b) << 16);
        }
        *reinterpret_cast<uint2*>(p.out16 + (size_t)m * p.N + n0) = make_uint2(h[0], h[1]);
    }
}


// qoq_gemm_astat.hip: the activation-stationary kernels for token tiles of 16, 32 and 64 (tile_m codes 69, 70, 71).
// `nwg` workgroups per token tile and k-slice share the layer's 16-channel fragments; p.S k-slices of p.gps groups.
hipError_t launch_astat(const GemmDev& p, int tile_m, int nwg, bool group, bool fp16, hipStream_t s);
// Largest number of quantization groups one workgroup of that kernel can keep resident for `tile` tokens.
int astat_max_groups(int tile);

}  // namespace qoq
