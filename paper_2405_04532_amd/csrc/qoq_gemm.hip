// W4A8 GEMM for gfx950 (Section 5.2 of arXiv 2405.04532, re-designed for CDNA4).
//
// out^T tile = W_tile (MFMA operand A, rows = output channels) x X_tile^T (operand B, columns
// = tokens), v_mfma_i32_16x16x64_i8, exact INT32 accumulation.
//   * weights: each lane streams its pre-ordered 128-bit words straight from global memory
//     into registers (one word = one lane's codes for a whole quantization group of one
//     row: two MFMA k-steps), prefetched one group ahead.  No LDS, no address arithmetic
//     beyond a running pointer (Section 5.2.1).
//   * UINT4 -> INT8 in registers (Sections 5.2.2-5.2.3): 3 logic ops unpack 8 codes into two
//     operand registers; per group one packed 16-bit multiply-add per register computes
//     code*s1 + (128 - z*s1) in all four bytes at once (no carries because the protective
//     range keeps every byte in [1, 255]), and one XOR turns the +128 bias into two's
//     complement.  The per-channel variant feeds the codes unchanged and folds the zero
//     point into the epilogue through the token's row sum (Eq. 6).
//   * activations: INT8 tile staged through LDS in operand-fragment order (conflict-free
//     128-bit reads), double buffered, one barrier per group of 128 k.
//   * small M: grid-level split-k with exact INT32 atomics into the workspace, then a
//     scaling pass (Section 5.2.4 mentions split-k for small m).
//   * epilogue (Section 5.2.2): FP32 acc * (sx[m] * s[n]), one rounding to FP16.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "qoq_internal.h"

namespace qoq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kWaves = 4;
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
    int M, N, K, G, gps;  // gps = groups per k-split
};

enum { OUT_FP16 = 0, OUT_I32 = 1, OUT_ATOMIC = 2 };

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

template <int MF, bool GROUP, int OUT>
__global__ __launch_bounds__(kThreads) void gemm_kernel(GemmDev p)
{
    constexpr int kPasses = (MF * 128 + kThreads - 1) / kThreads;  // 16-byte chunks of the A tile per thread
    __shared__ uint4 a_lds[2][MF * 2 * 64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sb = blockIdx.x * kWaves + wave;  // 64-channel block of this wave
    const bool active = sb < p.N / 64;
    const int m0 = blockIdx.y * (16 * MF);
    const int g_begin = blockIdx.z * p.gps;
    const int g_end = min(p.G, g_begin + p.gps);

    v4i acc[kNFrag][MF];
#pragma unroll
    for (int f = 0; f < kNFrag; ++f)
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) acc[f][mf] = (v4i){0, 0, 0, 0};

    // this thread's slots of the activation tile
    int a_row[kPasses], a_chunk[kPasses];
    bool a_valid[kPasses];
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps) {
        const int idx = ps * kThreads + threadIdx.x;
        a_row[ps] = idx >> 3;
        a_chunk[ps] = idx & 7;
        a_valid[ps] = a_row[ps] < 16 * MF && m0 + a_row[ps] < p.M;
    }
    auto load_a = [&](int g, uint4* regs) {
#pragma unroll
        for (int ps = 0; ps < kPasses; ++ps) {
            regs[ps] = make_uint4(0, 0, 0, 0);
            if (a_valid[ps])
                regs[ps] = *reinterpret_cast<const uint4*>(p.qx + (size_t)(m0 + a_row[ps]) * p.K + (size_t)g * kGroup +
                                                           a_chunk[ps] * 16);
        }
    };
    auto store_a = [&](int stage, const uint4* regs) {
#pragma unroll
        for (int ps = 0; ps < kPasses; ++ps) {
            const int r = a_row[ps], c = a_chunk[ps];
            if (r < 16 * MF) a_lds[stage][((r >> 4) * 2 + (c >> 2)) * 64 + (c & 3) * 16 + (r & 15)] = regs[ps];
        }
    };

    // this lane's stream of weight words: fragment f of block sb, group g
    const size_t unit_stride = 64;  // uint4 per unit
    auto load_w = [&](int g, uint4* wq, uint32_t* mt) {
#pragma unroll
        for (int f = 0; f < kNFrag; ++f) {
            const size_t unit = (size_t)(sb * kNFrag + f) * p.G + g;
            wq[f] = p.codes[unit * unit_stride + lane];
            if (GROUP) mt[f] = p.meta[unit * 16 + (lane & 15)];
        }
    };

    uint4 a_regs[kPasses], wq[kNFrag], wq_next[kNFrag];
    uint32_t mt[kNFrag], mt_next[kNFrag];
    if (g_begin < g_end) {
        load_a(g_begin, a_regs);
        if (active) load_w(g_begin, wq, mt);
        store_a(0, a_regs);
    }
    __syncthreads();

    int stage = 0;
    for (int g = g_begin; g < g_end; ++g) {
        const bool more = g + 1 < g_end;
        if (more) {
            load_a(g + 1, a_regs);
            if (active) load_w(g + 1, wq_next, mt_next);
        }
        if (active) {
            uint32_t S[kNFrag], B[kNFrag];
            if (GROUP) {
#pragma unroll
                for (int f = 0; f < kNFrag; ++f) {
                    S[f] = (mt[f] & 0xFFu) * 0x00010001u;
                    B[f] = (mt[f] >> 8) * 0x01010101u;
                }
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                v4i a_op[MF];
#pragma unroll
                for (int mf = 0; mf < MF; ++mf) {
                    const uint4 t = a_lds[stage][(mf * 2 + s) * 64 + lane];
                    a_op[mf] = (v4i){(int)t.x, (int)t.y, (int)t.z, (int)t.w};
                }
#pragma unroll
                for (int f = 0; f < kNFrag; ++f) {
                    const uint32_t x0 = s == 0 ? wq[f].x : wq[f].z;
                    const uint32_t x1 = s == 0 ? wq[f].y : wq[f].w;
                    const v4i w_op = dequant<GROUP>(x0, x1, GROUP ? S[f] : 0u, GROUP ? B[f] : 0u);
#pragma unroll
                    for (int mf = 0; mf < MF; ++mf)
                        acc[f][mf] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w_op, a_op[mf], acc[f][mf], 0, 0, 0);
                }
            }
        }
        if (more) {
            store_a(stage ^ 1, a_regs);
#pragma unroll
            for (int f = 0; f < kNFrag; ++f) { wq[f] = wq_next[f]; mt[f] = mt_next[f]; }
        }
        __syncthreads();
        stage ^= 1;
    }

    if (!active) return;
    // lane (q, ml) owns, for every m-fragment, token m0 + mf*16 + ml and the 16 consecutive
    // output channels n_base .. n_base+15 (value j = 4*f + r is acc[f][mf][r])
    const int q = lane >> 4, ml = lane & 15;
    const int n_base = sb * 64 + 16 * q;

    if (OUT == OUT_ATOMIC) {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) {
            const int m = m0 + mf * 16 + ml;
            if (m >= p.M) continue;
            int32_t* dst = p.out32 + (size_t)m * p.N + n_base;
#pragma unroll
            for (int f = 0; f < kNFrag; ++f)
#pragma unroll
                for (int r = 0; r < 4; ++r) atomicAdd(dst + 4 * f + r, acc[f][mf][r]);
        }
        return;
    }

    int zero[16];
    if (!GROUP) {
        const uint4 zz = *reinterpret_cast<const uint4*>(p.zeros + n_base);
        const uint32_t zw[4] = {zz.x, zz.y, zz.z, zz.w};
#pragma unroll
        for (int j = 0; j < 16; ++j) zero[j] = (int)((zw[j >> 2] >> (8 * (j & 3))) & 0xFFu);
    }
    float sn[16];
    if (OUT == OUT_FP16) {
        const uint4 s_lo = *reinterpret_cast<const uint4*>(p.scales + n_base);
        const uint4 s_hi = *reinterpret_cast<const uint4*>(p.scales + n_base + 8);
        const uint32_t sw[8] = {s_lo.x, s_lo.y, s_lo.z, s_lo.w, s_hi.x, s_hi.y, s_hi.z, s_hi.w};
#pragma unroll
        for (int j = 0; j < 16; ++j)
            sn[j] = __half2float(__ushort_as_half((unsigned short)((sw[j >> 1] >> (16 * (j & 1))) & 0xFFFFu)));
    }
#pragma unroll
    for (int mf = 0; mf < MF; ++mf) {
        const int m = m0 + mf * 16 + ml;
        if (m >= p.M) continue;
        int v[16];
#pragma unroll
        for (int f = 0; f < kNFrag; ++f)
#pragma unroll
            for (int r = 0; r < 4; ++r) v[4 * f + r] = acc[f][mf][r];
        if (!GROUP) {
            const int rs = p.rowsum[m];
#pragma unroll
            for (int j = 0; j < 16; ++j) v[j] -= zero[j] * rs;
        }
        if (OUT == OUT_I32) {
            int4* dst = reinterpret_cast<int4*>(p.out32 + (size_t)m * p.N + n_base);
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[j] = make_int4(v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]);
        } else {
            const float sxm = __half2float(p.sx[m]);
            uint32_t h[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const __half a = __float2half_rn((float)v[2 * j] * (sxm * sn[2 * j]));
                const __half b = __float2half_rn((float)v[2 * j + 1] * (sxm * sn[2 * j + 1]));
                h[j] = (uint32_t)__half_as_ushort(a) | ((uint32_t)__half_as_ushort(b) << 16);
            }
            uint4* dst = reinterpret_cast<uint4*>(p.out16 + (size_t)m * p.N + n_base);
            dst[0] = make_uint4(h[0], h[1], h[2], h[3]);
            dst[1] = make_uint4(h[4], h[5], h[6], h[7]);
        }
    }
}

__global__ __launch_bounds__(kThreads) void zero_i32_kernel(int4* dst, size_t n4)
{
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kThreads)
        dst[i] = make_int4(0, 0, 0, 0);
}

// Split-k second pass: 8 consecutive channels of one token per thread.
template <bool GROUP, bool TO_FP16>
__global__ __launch_bounds__(kThreads) void finalize_kernel(const int32_t* __restrict__ ws, GemmDev p)
{
    const size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t per_row = (size_t)p.N / 8;
    if (idx >= (size_t)p.M * per_row) return;
    const int m = (int)(idx / per_row);
    const int n0 = (int)(idx % per_row) * 8;
    const int4 a = *reinterpret_cast<const int4*>(ws + (size_t)m * p.N + n0);
    const int4 b = *reinterpret_cast<const int4*>(ws + (size_t)m * p.N + n0 + 4);
    int v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    if (!GROUP) {
        const int rs = p.rowsum[m];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] -= (int)p.zeros[n0 + j] * rs;
    }
    if (TO_FP16) {
        const float sxm = __half2float(p.sx[m]);
        uint32_t h[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const __half x = __float2half_rn((float)v[2 * j] * (sxm * __half2float(p.scales[n0 + 2 * j])));
            const __half y = __float2half_rn((float)v[2 * j + 1] * (sxm * __half2float(p.scales[n0 + 2 * j + 1])));
            h[j] = (uint32_t)__half_as_ushort(x) | ((uint32_t)__half_as_ushort(y) << 16);
        }
        *reinterpret_cast<uint4*>(p.out16 + (size_t)m * p.N + n0) = make_uint4(h[0], h[1], h[2], h[3]);
    } else {
        int4* dst = reinterpret_cast<int4*>(p.out32 + (size_t)m * p.N + n0);
        dst[0] = make_int4(v[0], v[1], v[2], v[3]);
        dst[1] = make_int4(v[4], v[5], v[6], v[7]);
    }
}

template <int MF, bool GROUP>
void launch_variant(const GemmDev& p, int out_mode, dim3 grid, hipStream_t s)
{
    if (out_mode == OUT_FP16) gemm_kernel<MF, GROUP, OUT_FP16><<<grid, kThreads, 0, s>>>(p);
    else if (out_mode == OUT_I32) gemm_kernel<MF, GROUP, OUT_I32><<<grid, kThreads, 0, s>>>(p);
    else gemm_kernel<MF, GROUP, OUT_ATOMIC><<<grid, kThreads, 0, s>>>(p);
}

template <bool GROUP>
void launch_tile(const GemmDev& p, int tile_m, int out_mode, dim3 grid, hipStream_t s)
{
    switch (tile_m) {
        case 16: launch_variant<1, GROUP>(p, out_mode, grid, s); break;
        case 32: launch_variant<2, GROUP>(p, out_mode, grid, s); break;
        case 64: launch_variant<4, GROUP>(p, out_mode, grid, s); break;
        default: launch_variant<8, GROUP>(p, out_mode, grid, s); break;
    }
}

}  // namespace

void pick_gemm_config(int64_t M, int64_t N, int64_t K, int forced_tile_m, int forced_split_k, int& tile_m,
                      int& split_k)
{
    const int64_t G = K / kGroup;
    tile_m = forced_tile_m ? forced_tile_m : (M <= 16 ? 16 : M <= 32 ? 32 : M <= 64 ? 64 : 128);
    const int64_t blocks = ((N + 255) / 256) * ((M + tile_m - 1) / tile_m);
    int64_t split = forced_split_k;
    if (split <= 0) {
        split = 1;
        if (blocks < 256) {
            split = (512 + blocks - 1) / blocks;
            const int64_t max_split = G / 2 > 0 ? G / 2 : 1;  // keep at least two groups per slice
            if (split > max_split) split = max_split;
        }
    }
    if (split > G) split = G;
    if (split < 1) split = 1;
    const int64_t gps = (G + split - 1) / split;
    split_k = (int)((G + gps - 1) / gps);
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s)
{
    if (a.M == 0) return hipSuccess;
    const BlobLayout L = make_layout(a.N, a.K, a.mode);
    GemmDev p;
    p.qx = a.qx;
    p.codes = reinterpret_cast<const uint4*>(a.blob + L.codes_off);
    p.meta = reinterpret_cast<const uint16_t*>(a.blob + L.meta_off);
    p.scales = reinterpret_cast<const __half*>(a.blob + L.scale_off);
    p.zeros = a.blob + L.zero_off;
    p.sx = static_cast<const __half*>(a.sx);
    p.rowsum = a.rowsum;
    p.out16 = static_cast<__half*>(a.out_fp16);
    p.out32 = a.out_i32;
    p.M = (int)a.M; p.N = (int)a.N; p.K = (int)a.K; p.G = (int)L.G;
    p.gps = (int)((L.G + a.split_k - 1) / a.split_k);
    const dim3 grid((unsigned)((a.N + 255) / 256), (unsigned)((a.M + a.tile_m - 1) / a.tile_m), (unsigned)a.split_k);
    const bool group = a.mode == 0;
    if (a.split_k == 1) {
        const int out_mode = a.out_fp16 ? OUT_FP16 : OUT_I32;
        if (group) launch_tile<true>(p, a.tile_m, out_mode, grid, s);
        else launch_tile<false>(p, a.tile_m, out_mode, grid, s);
        return hipGetLastError();
    }
    // split-k: exact INT32 partial sums meet in the workspace, then one scaling pass
    const size_t n4 = (size_t)a.M * (size_t)a.N / 4;
    zero_i32_kernel<<<dim3((unsigned)((n4 + kThreads - 1) / kThreads > 2048 ? 2048 : (n4 + kThreads - 1) / kThreads)),
                      kThreads, 0, s>>>(reinterpret_cast<int4*>(a.workspace), n4);
    GemmDev pa = p;
    pa.out32 = a.workspace;
    if (group) launch_tile<true>(pa, a.tile_m, OUT_ATOMIC, grid, s);
    else launch_tile<false>(pa, a.tile_m, OUT_ATOMIC, grid, s);
    const size_t items = (size_t)a.M * (size_t)a.N / 8;
    const dim3 fgrid((unsigned)((items + kThreads - 1) / kThreads));
    if (group) {
        if (a.out_fp16) finalize_kernel<true, true><<<fgrid, kThreads, 0, s>>>(a.workspace, p);
        else finalize_kernel<true, false><<<fgrid, kThreads, 0, s>>>(a.workspace, p);
    } else {
        if (a.out_fp16) finalize_kernel<false, true><<<fgrid, kThreads, 0, s>>>(a.workspace, p);
        else finalize_kernel<false, false><<<fgrid, kThreads, 0, s>>>(a.workspace, p);
    }
    return hipGetLastError();
}

}  // namespace qoq
