// W4A8 GEMM for gfx950 (Section 5.2 of arXiv 2405.04532, re-designed for CDNA4).
//
// out^T tile = W_tile (MFMA operand A, rows = output channels) x X_tile^T (operand B, columns = tokens),
// INT8 x INT8 -> INT32 on the matrix cores, exact accumulation.
//   * Weights stay packed (two codes per byte) in HBM and in LDS, in the order the MFMA lanes consume them
//     (Section 5.2.1): one 128-bit word per lane and quantization group, no address arithmetic per fragment.
//   * UINT4 -> INT8 in registers (Sections 5.2.2-5.2.3): 3 logic ops unpack 8 codes into two operand
//     registers; per group one packed 16-bit multiply-add per register computes code*s1 + (128 - z*s1) in
//     all four bytes at once (no carries because the protective range keeps every byte in [1, 255]), and
//     one XOR turns the +128 bias into two's complement.  The per-channel variant feeds the codes unchanged
//     and folds the zero point into the epilogue through the token's row sum (Eq. 6).
//   * Three kernels.
//     "stream" (64-token tiles, memory bound, v_mfma_i32_16x16x64_i8): a multi-stage pipeline of direct
//     global->LDS copies (the asynchronous-copy software pipeline of Section 5.2.4 in its gfx950 form) over
//     a balanced, stream-k style partition of the work.
//       - Work unit = one quantization group of one 64-channel block (4 KiB of packed weights).  The
//         N/64 * K/128 units are dealt out in equal contiguous runs to about one workgroup per CU, whatever
//         the layer shape; a run may start and end in the middle of a block.
//       - HBM latency under load is about 1.5-2.5 us here, so some 50-100 KiB per CU must be in flight.
//         Each of eight consumer waves (fragment f, group parity e) copies the units it will itself consume
//         into a private LDS ring, four units deep: no barrier guards the weights.  Activations come from L2 and
//         need far less lead, but a wave's outstanding copies retire in order, so a wave issuing both would
//         stall its deep weight prefetch on every activation wait: four producer waves copy the activation
//         slabs, level-2 metadata and channel scales a couple of iterations ahead; one barrier per iteration
//         (two groups) publishes them.  Copies are issued from inline assembly and waited for with explicit
//         s_waitcnt vmcnt(n): the compiler's own bookkeeping would wait for ALL outstanding copies before
//         every LDS read.
//       - A block finished inside one run is scaled and stored at once.  Blocks shared by several runs meet
//         in the workspace: partial INT32 tiles are written through to memory, a per-block counter elects
//         the last workgroup to arrive, which adds all partials (integer sums are exact and order
//         independent) and runs the epilogue.
//     "rstream" (16- and 32-token tiles): the same partition with nothing staged in LDS; every wave loads the
//     operand words of its own units straight into registers (see the comment in front of it).
//     "mma" (larger M, compute bound, v_mfma_i32_32x32x32_i8): large output tiles, one wave per SIMD, a
//     hand software-pipelined main loop; see the comment in front of it.
//   * Epilogue (Section 5.2.2): FP32 acc * (sx[m] * s[n]), one rounding to FP16.
#include <hip/hip_fp16.h>
#include <algorithm>
#include <hip/hip_runtime.h>

#include "qoq_internal.h"
#include "qoq_gemm_common.h"
#include "qoq_walk.h"

namespace qoq {
namespace {

// Hand-over of partial tiles between workgroups (which may sit on different XCDs, each with its own L2)
// without device-wide fences: a release/acquire fence pair writes back and invalidates a whole L2 and was
// measured to cost tens of microseconds per GEMM here.  Partial tiles are instead written with sc1
// (write-through) stores and read with sc1 loads, which go to memory past the non-coherent caches; a
// workgroup waits for its own stores to complete (s_waitcnt) before it bumps the tile's counter with a
// relaxed device-scope atomic, and the last arriver reads the partials only after that atomic has returned.

// ------------------------------------------------------------------------------------------
// "stream" kernel: 16*MF <= 64 tokens; twelve waves; grid = (workgroups, m-tiles).
// Consumer wave c = 2*f + e handles fragment f of the current 64-channel block and, in each
// iteration, the group of parity e of a pair of consecutive groups.
// ------------------------------------------------------------------------------------------

// Write-through store / cache-bypassing load of 16 bytes (device-coherent without fences).
// A store of more than 8 bytes reads its data registers over several cycles after issue; the instruction that
// follows must not write them (a documented wait-state requirement the compiler honours for its own stores but
// cannot for inline assembly, which it does not know to be a store: partial sums whose registers were reused at
// once came out corrupted in a few lanes).  Hence the idle cycles inside the store statements.  The streaming
// kernel goes further and keeps its stores out of the loop altogether (below): they go out after the last copy,
// together with the wait for their completion, from registers the same statement keeps alive.
__device__ __forceinline__ void store_sc1(int4* ptr, v4i v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 3" :: "v"(ptr), "v"(v) : "memory");
}
template <int CNT>
__device__ __forceinline__ void store_sc1_and_wait(int4* ptr, int stride, const v4i (&v)[CNT])
{
    static_assert(CNT == 1 || CNT == 2 || CNT == 4 || CNT == 8, "fragments per lane (of one or two tiles)");
    if constexpr (CNT == 8) {
        asm volatile("global_store_dwordx4 %0, %8, off sc1\n\tglobal_store_dwordx4 %1, %9, off sc1\n\t"
                     "global_store_dwordx4 %2, %10, off sc1\n\tglobal_store_dwordx4 %3, %11, off sc1\n\t"
                     "global_store_dwordx4 %4, %12, off sc1\n\tglobal_store_dwordx4 %5, %13, off sc1\n\t"
                     "global_store_dwordx4 %6, %14, off sc1\n\tglobal_store_dwordx4 %7, %15, off sc1\n\ts_waitcnt vmcnt(0)"
                     :: "v"(ptr), "v"(ptr + stride), "v"(ptr + 2 * stride), "v"(ptr + 3 * stride), "v"(ptr + 4 * stride),
                     "v"(ptr + 5 * stride), "v"(ptr + 6 * stride), "v"(ptr + 7 * stride), "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]),
                     "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]) : "memory");
        return;
    }
    if constexpr (CNT == 1)
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" :: "v"(ptr), "v"(v[0]) : "memory");
    else if constexpr (CNT == 2)
        asm volatile("global_store_dwordx4 %0, %2, off sc1\n\tglobal_store_dwordx4 %1, %3, off sc1\n\ts_waitcnt vmcnt(0)"
                     :: "v"(ptr), "v"(ptr + stride), "v"(v[0]), "v"(v[1]) : "memory");
    else
        asm volatile("global_store_dwordx4 %0, %4, off sc1\n\tglobal_store_dwordx4 %1, %5, off sc1\n\t"
                     "global_store_dwordx4 %2, %6, off sc1\n\tglobal_store_dwordx4 %3, %7, off sc1\n\ts_waitcnt vmcnt(0)"
                     :: "v"(ptr), "v"(ptr + stride), "v"(ptr + 2 * stride), "v"(ptr + 3 * stride), "v"(v[0]), "v"(v[1]), "v"(v[2]),
                     "v"(v[3]) : "memory");
}
__device__ __forceinline__ void load_sc1_nowait(v4i& v, const int4* ptr)
{
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(ptr) : "memory");
}
__device__ __forceinline__ void wait_loads(v4i& a, v4i& b, v4i& c, v4i& d)
{
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) :: "memory");
}

constexpr int kStreamThreads = 768;  // eight consumer waves + four producer waves

// Blocks shared with other workgroups: this workgroup has written its partial tiles (at most two) to the
// workspace and waited for them.  It bumps each block's counter; whoever arrives last at a block adds every
// contributor's partial tile and runs the epilogue.  Called by all THREADS threads of the workgroup.
template <int MF, bool GROUP, int OUT, int THREADS>
__device__ __forceinline__ void finish_shared_blocks(const GemmDev& p, int npart, int part_block0, int part_block1, int m0, int* s_flag)
{
    const int G = p.G, blocks = p.N / 64;
    // ---- blocks shared with other workgroups ---------------------------------------------------
    // Every step here is a round trip to memory (about a microsecond), so whatever can be in flight together is:
    // both counters, then every partial-tile load and every epilogue constant of both blocks.
    __syncthreads();
    if (threadIdx.x < npart) {
        const int b = threadIdx.x == 0 ? part_block0 : part_block1;
        const int w_first = (b * G) / p.upw, w_last = (b * G + G - 1) / p.upw;
        int* ctr = p.counters + blockIdx.y * blocks + b;
        const int old = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = old == w_last - w_first;
        s_flag[threadIdx.x] = last;
        if (last) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    // last to arrive at a block: add every contributor's partial tile, element by element, and finish it
    constexpr int kEl = MF * kThreads;                                     // int4 elements of a partial tile
    constexpr int kRounds = (kEl + THREADS - 1) / THREADS;   // elements per thread
    constexpr int kBatch = MF == 4 ? 5 : 6;                                // contributors loaded at once
    v4i t[2 * kRounds * kBatch];
    uint2 c_s[2 * kRounds];
    uint32_t c_z[2 * kRounds];
    float c_sx[2 * kRounds];
    int c_rs[2 * kRounds];
#pragma unroll
    for (int x = 0; x < 2 * kRounds * kBatch; ++x) t[x] = (v4i){0, 0, 0, 0};
    bool mine[2];
    int blk[2], wf[2], wl[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        mine[k] = k < npart && s_flag[k];                                  // everything here is workgroup-uniform
        blk[k] = __builtin_amdgcn_readfirstlane(k == 0 ? part_block0 : part_block1);
        wf[k] = __builtin_amdgcn_readfirstlane((blk[k] * G) / p.upw);
        wl[k] = __builtin_amdgcn_readfirstlane((blk[k] * G + G - 1) / p.upw);
    }
    // a contributor's partial tile of block blk[k] is its first one iff its run starts inside that block
    auto first_partial = [&](int ww, int k) __attribute__((always_inline)) {
        const int us = ww * p.upw;
        return us >= blk[k] * G && us < (blk[k] + 1) * G;
    };
    auto element = [&](int r, int& el, int& m, int& n_rel) __attribute__((always_inline)) {
        el = min((int)threadIdx.x + r * THREADS, kEl - 1);          // clamped: loads stay in bounds
        const int mf = el / kThreads, ft = (el % kThreads) >> 6, ln = el & 63;
        m = m0 + mf * 16 + (ln & 15);
        n_rel = 16 * (ln >> 4) + 4 * ft;
    };
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        if (!mine[k]) continue;
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            int el, m, n_rel;
            element(r, el, m, n_rel);
            const int n0 = blk[k] * 64 + n_rel, mc = min(m, p.M - 1);
            c_s[k * kRounds + r] = OUT == OUT_FP16 ? *reinterpret_cast<const uint2*>(p.scales + n0) : make_uint2(0, 0);
            c_z[k * kRounds + r] = GROUP ? 0u : *reinterpret_cast<const uint32_t*>(p.zeros + n0);
            c_sx[k * kRounds + r] = OUT == OUT_FP16 ? __half2float(p.sx[mc]) : 0.f;
            c_rs[k * kRounds + r] = GROUP ? 0 : p.rowsum[mc];
        }
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        if (!mine[k]) continue;
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            int el, m, n_rel;
            element(r, el, m, n_rel);
            if ((int)threadIdx.x + r * THREADS >= kEl) continue;     // whole waves: no element in this round
#pragma unroll
            for (int x = 0; x < kBatch; ++x) {
                const int ww = wf[k] + x;
                if (ww > wl[k]) break;                                      // these loads go to memory: none is issued twice
                const int which = first_partial(ww, k) ? 0 : 1;
                t[(k * kRounds + r) * kBatch + x] =
                    load_through(p.parts + ((size_t)(blockIdx.y * gridDim.x + ww) * 2 + which) * kEl + el);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        if (!mine[k]) continue;
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            int el, m, n_rel;
            element(r, el, m, n_rel);
            v4i sum = (v4i){0, 0, 0, 0};
#pragma unroll
            for (int x = 0; x < kBatch; ++x)
                if (wf[k] + x <= wl[k]) sum += t[(k * kRounds + r) * kBatch + x];
            for (int w = wf[k] + kBatch; w <= wl[k]; w += 4) {              // more contributors than one batch holds
                v4i u[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int ww = w + x;
                    u[x] = (v4i){0, 0, 0, 0};
                    if (ww > wl[k]) continue;
                    const int which = first_partial(ww, k) ? 0 : 1;
                    u[x] = load_through(p.parts + ((size_t)(blockIdx.y * gridDim.x + ww) * 2 + which) * kEl + el);
                }
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    if (w + x <= wl[k]) sum += u[x];
            }
            if ((int)threadIdx.x + r * THREADS >= kEl || m >= p.M) continue;
            const uint2 sw = c_s[k * kRounds + r];
            const float sn[4] = {__half2float(__ushort_as_half((unsigned short)(sw.x & 0xFFFFu))),
                                 __half2float(__ushort_as_half((unsigned short)(sw.x >> 16))),
                                 __half2float(__ushort_as_half((unsigned short)(sw.y & 0xFFFFu))),
                                 __half2float(__ushort_as_half((unsigned short)(sw.y >> 16)))};
            const uint32_t zw = c_z[k * kRounds + r];
            const int zn[4] = {(int)(zw & 0xFFu), (int)((zw >> 8) & 0xFFu), (int)((zw >> 16) & 0xFFu), (int)(zw >> 24)};
            finish4<GROUP, OUT>(p, m, blk[k] * 64 + n_rel, sum, sn, zn, c_sx[k * kRounds + r], c_rs[k * kRounds + r]);
        }
    }
}

template <int MF, bool GROUP, int OUT>
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void stream_kernel(GemmDev p)
{
    // Weights: every consumer wave owns a deep private ring of 1 KiB units.  Activations, metadata and
    // scales: shallow rings, one slot per iteration (= two consecutive groups of a block), filled by
    // four producer waves (producer (pk, ph) copies half ph of the activation blocks of the pk-th group of
    // the pair; the ph = 0 ones also the group's metadata, producer (0, 1) the block's scales).  Producers and
    // consumers run separate, tight loops that meet at the same barriers: with one loop for both roles every
    // wave branched around the other role's code, and the producers' ten copies plus that branching set
    // the pace of the whole workgroup (measured with s_memtime probes).
    // Ring depths: three slots are the minimum of the scheme (one read, one landing, one in flight).  Depths of
    // 3 to 10 weight units per wave were measured to stream equally fast (the loop is not limited by bytes in
    // flight), and a deep ring only lengthens the burst of copies that must land before the first iteration.
    constexpr int kWRing = 4;
    constexpr int kARing = 4;
    constexpr int kABlocks = 2 * MF;                                  // 1 KiB blocks (m-fragment, k-step) per group
    constexpr int kAHalf = kABlocks / 2;                              // activation blocks per producer wave
    static_assert(kWRing - 2 < 64 && (kARing - 2) * (kAHalf + 1) < 64, "vmcnt range");
    __shared__ uint4 wring[8][kWRing][64];            // private ring of weight units per consumer wave
    __shared__ uint4 aring[kARing][2][kABlocks * 64]; // activation slabs of the iteration's two groups
    __shared__ uint4 mring[kARing][2][16];            // level-2 metadata: 4 fragments x 16 rows x uint16
    __shared__ uint4 sring[kARing][16];               // block's FP16 scales (128 B) and zeros (64 B)
    __shared__ int4 red[kNFrag * MF * 64];
    __shared__ float sx_lds[16 * MF];
    __shared__ int rs_lds[16 * MF];
    __shared__ int s_flag[2];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool producer = wave >= 8;
    const int pk = wave & 1;                               // producer: which group of the pair
    const int ph = (wave >> 1) & 1;                        // producer: which half of the group's activation blocks
    const int f = (wave & 7) >> 1, e = wave & 1;           // consumer: fragment, group parity
    const int wg = blockIdx.x;
    const int m0 = blockIdx.y * (16 * MF);
    const int G = p.G;
    const int blocks = p.N / 64;
    const int total = blocks * G;
    const int u0 = min(total, wg * p.upw), u1 = min(total, u0 + p.upw);
    if (u0 >= u1) return;                                  // whole workgroup: nothing to do
    const int q = lane >> 4, ml = lane & 15;
    const int nf_total = p.N / 16;

    // The run's iteration structure in closed form (qoq_walk.h), all wave-uniform.
    RunShape run = make_run(u0, u1, G, 2);
    run.b0 = __builtin_amdgcn_readfirstlane(run.b0); run.g0 = __builtin_amdgcn_readfirstlane(run.g0);
    run.full = __builtin_amdgcn_readfirstlane(run.full); run.last_len = __builtin_amdgcn_readfirstlane(run.last_len);
    const int T = __builtin_amdgcn_readfirstlane(run.T);

    v4i acc[MF];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf) acc[mf] = (v4i){0, 0, 0, 0};

    // ---- copy roles -----------------------------------------------------------------------
    // producer: lane 4r+c copies 16-byte chunk c ^ h(r) of row r of a 16-row activation block: a quad
    // reads one 64-byte row segment; h spreads the rows over the LDS banks for the fragment reads
    uint32_t a_voff[kAHalf];                               // blocks ph * kAHalf .. of the group
    {
        const int r = lane >> 2, c = lane & 3;
        const int h = ((r >> 1) ^ (r >> 2)) & 3;
#pragma unroll
        for (int j = 0; j < kAHalf; ++j) {
            const int b = ph * kAHalf + j;
            const int row = min(m0 + (b >> 1) * 16 + r, p.M - 1);  // rows past M repeat the last one; never stored
            a_voff[j] = (uint32_t)row * (uint32_t)p.K + (uint32_t)((b & 1) * 64 + (c ^ h) * 16);
        }
    }
    const uint32_t m_voff = (uint32_t)(lane & 31) * 4u;                      // 128 B of metadata; upper lanes re-read
    // scales: lanes 0..31 fetch the block's 64 FP16 scales, lanes 32..47 its 64 zero bytes
    const uint32_t zero_delta = (uint32_t)(reinterpret_cast<const char*>(p.zeros) - reinterpret_cast<const char*>(p.scales));
    const uint32_t s_voff = (lane < 32 || GROUP) ? (uint32_t)(lane & 31) * 4u : zero_delta + (uint32_t)((lane - 32) & 15) * 4u;
    const uint32_t s_blk_stride = (lane < 32 || GROUP) ? 128u : 64u;         // bytes per block in either array
    const uint32_t wring_addr = (uint32_t)(uintptr_t)&wring[0][0][0] + (uint32_t)(wave & 7) * (kWRing * 1024);
    const uint32_t aring_addr = (uint32_t)(uintptr_t)&aring[0][0][0] + (uint32_t)(pk * kABlocks + ph * kAHalf) * 1024u;
    const uint32_t mring_addr = (uint32_t)(uintptr_t)&mring[0][0][0] + (uint32_t)pk * 256;
    const uint32_t sring_addr = (uint32_t)(uintptr_t)&sring[0][0];
    constexpr uint32_t kASlot = 2 * kABlocks * 1024;
    const char* abase = reinterpret_cast<const char*>(p.qx);
    const char* sbase = reinterpret_cast<const char*>(p.scales);
    const uint32_t w_voff = (uint32_t)lane * 16u;
    const char* codes_base = reinterpret_cast<const char*>(p.codes);
    const char* meta_base = reinterpret_cast<const char*>(p.meta);
    const uint32_t m_g_stride = (uint32_t)nf_total * 32u;

    // Tables: lane j of a wave holds what the wave needs to know about iteration tbase + j (iterations past the
    // end of the run repeat the last one: every iteration issues the same number of copies, the wait counts rely
    // on it, and a repeated copy reads valid memory).  The loop reads them with v_readlane instead of stepping a
    // state machine in scalar registers: with twelve waves per workgroup the scalar instructions, not the
    // copies, set the pace of an iteration.
    //   info  = first group | (units - 1) << 24 | ends a segment << 25 | that segment is a whole block << 26
    //   block = 64-channel block
    //   off0  = consumer: byte offset of the wave's weight unit; producer: column offset of its group
    //   off1  = producer: byte offset of the group's metadata row
    struct Tables { uint32_t info, block, off0, off1; };
    auto build_tables = [&](int base) __attribute__((always_inline)) {
        Tables t;
        const IterInfo o = run_iteration(run, min(base + lane, T - 1));
        t.info = (uint32_t)o.g | ((uint32_t)(o.n - 1) << 24) | ((uint32_t)(o.seg_end ? 1 : 0) << 25) |
                 ((uint32_t)(o.complete ? 1 : 0) << 26);
        t.block = (uint32_t)o.block;
        if (producer) {
            const int gsel = min(o.g + (pk < o.n ? pk : 0), G - 1);
            t.off0 = (uint32_t)gsel * (uint32_t)kGroup;
            t.off1 = (uint32_t)gsel * m_g_stride + (uint32_t)o.block * (uint32_t)(kNFrag * 32);
        } else {
            const int gsel = min(o.g + (e < o.n ? e : 0), G - 1);
            t.off0 = (uint32_t)((o.block * kNFrag + f) * G + gsel) << 10;
            t.off1 = 0;
        }
        return t;
    };
    int tbase = 0;
    Tables tb = build_tables(0);
    auto lookup = [](uint32_t table, int j) __attribute__((always_inline)) { return (uint32_t)__builtin_amdgcn_readlane((int)table, j); };

    // Copies for the iteration with table index j.
    int islot = 0;
    auto issue_producer = [&](int j) __attribute__((always_inline)) {
        const uint32_t aoff = lookup(tb.off0, j);
#pragma unroll
        for (int b = 0; b < kAHalf; ++b)
            dma16(abase, a_voff[b] + aoff, aring_addr + islot * kASlot + b * 1024);
        if (GROUP && ph == 0) dma4(meta_base, m_voff + lookup(tb.off1, j), mring_addr + islot * 512);
        if (pk == 0 && ph == 1) dma4(sbase, s_voff + lookup(tb.block, j) * s_blk_stride, sring_addr + islot * 256);
        islot = islot + 1 == kARing ? 0 : islot + 1;
    };
    auto issue_consumer = [&](int j) __attribute__((always_inline)) {
        dma16(codes_base, w_voff + lookup(tb.off0, j), wring_addr + islot * 1024);
        islot = islot + 1 == kWRing ? 0 : islot + 1;
    };

    const int hsw = ((ml >> 1) ^ (ml >> 2)) & 3;
    const int a_src = 4 * ml + (q ^ hsw);   // slot of (row ml, chunk q) inside a 1 KiB activation block
    int wslot = 0, aslot = 0;               // ring slots of the iteration being consumed
    auto compute = [&]() {
        const uint4 wq = wring[wave & 7][wslot][lane];
        uint32_t S = 0, B = 0;
        if (GROUP) {
            const uint32_t mt = reinterpret_cast<const uint16_t*>(&mring[aslot][e][0])[f * 16 + ml];
            S = __builtin_amdgcn_perm(mt, mt, 0x0c000c00u);  // s1 in both 16-bit lanes
            B = __builtin_amdgcn_perm(mt, mt, 0x01010101u);  // bias in all four bytes
        }
        const uint4* slab = aring[aslot][e];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i a_op[MF];
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) a_op[mf] = as_v4i(slab[(mf * 2 + ks) * 64 + a_src]);
            const v4i w_op = dequant<GROUP>(ks ? wq.z : wq.x, ks ? wq.w : wq.y, S, B);
#pragma unroll
            for (int mf = 0; mf < MF; ++mf)
                acc[mf] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w_op, a_op[mf], acc[mf], 0, 0, 0);
        }
    };

    // ---- main loop --------------------------------------------------------------------------
    // Each iteration consumes one slot of every ring while later ones are being copied.  A wave first
    // waits until at most the copies of the (ring - 2) younger iterations it issued are outstanding,
    // so its own copies for this iteration have landed; the barrier then publishes every wave's
    // copies and proves that the slots refilled next are no longer being read.
    const int tid = f * 64 + lane;                          // owner lanes: index inside a partial tile
    const bool owner = !producer && e == 0;
    int4* my_parts = p.parts + (size_t)(blockIdx.y * gridDim.x + wg) * 2 * (MF * kThreads);
    int npart = 0, part_block0 = 0, part_block1 = 0;   // (scalars: an indexed array would be moved to LDS)
    // Partial tiles of the run (at most two: a first segment that starts inside a block, a last one that ends
    // inside a block) stay in registers and are written out after the loop, so that no store sits among the copies.
    v4i part0[MF], part1[MF];
    bool has_part0 = false, has_part1 = false;
#pragma unroll
    for (int mf = 0; mf < MF; ++mf) part0[mf] = part1[mf] = (v4i){0, 0, 0, 0};
    int seg_index = 0;

    // bookkeeping every wave keeps identically: segments of the run that end inside a shared block
    auto close_segment = [&](bool complete, int block_now) __attribute__((always_inline)) {
        if (!complete) { if (npart == 0) part_block0 = block_now; else part_block1 = block_now; ++npart; }
        ++seg_index;
    };

    if (producer) {
        // ---- producer loop: copies only; same barriers as the consumer loop below --------------------
        const int my_dma = kAHalf + ((GROUP && ph == 0) ? 1 : 0) + ((pk == 0 && ph == 1) ? 1 : 0);
#pragma unroll
        for (int k = 0; k < kARing - 1; ++k) issue_producer(k);
        // per-token epilogue constants go through LDS so that the consumer waves never issue a
        // register load whose compiler-placed wait would drain their copy queue
        if (pk == 1 && ph == 1 && lane < 16 * MF) {
            const int m = min(m0 + lane, p.M - 1);
            sx_lds[lane] = OUT == OUT_FP16 ? __half2float(p.sx[m]) : 0.f;
            rs_lds[lane] = GROUP ? 0 : p.rowsum[m];
        }
        for (int it = 0; it < T; ++it) {
            int j = it - tbase;
            if (j + kARing - 1 >= 64) { tb = build_tables(it); tbase = it; j = 0; }
            const uint32_t info = lookup(tb.info, j);
            if (my_dma == kAHalf) wait_vmcnt<(kARing - 2) * kAHalf>();
            else wait_vmcnt<(kARing - 2) * (kAHalf + 1)>();
            __syncthreads();
            issue_producer(j + kARing - 1);
            if (!(info & (1u << 25))) continue;
            __syncthreads();                               // the consumers' hand-over barrier
            close_segment((info >> 26) & 1, (int)lookup(tb.block, j));
        }
    } else {
        // ---- consumer loop ------------------------------------------------------------------------------
#pragma unroll
        for (int k = 0; k < kWRing - 1; ++k) issue_consumer(k);
        for (int it = 0; it < T; ++it) {
            int j = it - tbase;
            if (j + kWRing - 1 >= 64) { tb = build_tables(it); tbase = it; j = 0; }
            const uint32_t info = lookup(tb.info, j);
            wait_vmcnt<kWRing - 2>();
            __syncthreads();
            issue_consumer(j + kWRing - 1);
            if (e == 0 || (info & (1u << 24))) compute();
            const int aslot_now = aslot;
            wslot = wslot + 1 == kWRing ? 0 : wslot + 1;
            aslot = aslot + 1 == kARing ? 0 : aslot + 1;
            if (!(info & (1u << 25))) continue;
            const int block_now = (int)lookup(tb.block, j);

            // ---- end of this run's share of block_now: parity-1 waves hand over, owners finish -----
            if (e == 1) {
    #pragma unroll
                for (int mf = 0; mf < MF; ++mf) {
                    red[(f * MF + mf) * 64 + lane] = make_int4(acc[mf].x, acc[mf].y, acc[mf].z, acc[mf].w);
                    acc[mf] = (v4i){0, 0, 0, 0};
                }
            }
            __syncthreads();
            const bool complete = (info >> 26) & 1;
            if (owner) {
                float sn[4] = {0.f, 0.f, 0.f, 0.f};
                int zn[4] = {0, 0, 0, 0};
                if (complete) {
                    const char* sc = reinterpret_cast<const char*>(&sring[aslot_now][0]);
                    const uint2 sw = *reinterpret_cast<const uint2*>(sc + (16 * q + 4 * f) * 2);
                    sn[0] = __half2float(__ushort_as_half((unsigned short)(sw.x & 0xFFFFu)));
                    sn[1] = __half2float(__ushort_as_half((unsigned short)(sw.x >> 16)));
                    sn[2] = __half2float(__ushort_as_half((unsigned short)(sw.y & 0xFFFFu)));
                    sn[3] = __half2float(__ushort_as_half((unsigned short)(sw.y >> 16)));
                    if (!GROUP) {
                        const uint32_t zw = *reinterpret_cast<const uint32_t*>(sc + 128 + 16 * q + 4 * f);
    #pragma unroll
                        for (int j = 0; j < 4; ++j) zn[j] = (int)((zw >> (8 * j)) & 0xFFu);
                    }
                }
    #pragma unroll
                for (int mf = 0; mf < MF; ++mf) {
                    const int4 o = red[(f * MF + mf) * 64 + lane];
                    v4i v = acc[mf];
                    v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
                    acc[mf] = (v4i){0, 0, 0, 0};
                    if (complete) {
                        const int m = m0 + mf * 16 + ml;
                        if (m < p.M)
                            finish4<GROUP, OUT>(p, m, block_now * 64 + 16 * q + 4 * f, v, sn, zn, sx_lds[mf * 16 + ml],
                                                rs_lds[mf * 16 + ml]);
                    } else if (seg_index == 0) {
                        part0[mf] = v;
                    } else {
                        part1[mf] = v;
                    }
                }
            }
            if (!complete) { if (seg_index == 0) has_part0 = true; else has_part1 = true; }
            close_segment(complete, block_now);
        }
        if (owner) {
            if (has_part0 && has_part1) {                  // one wait for both
                v4i both[2 * MF];
#pragma unroll
                for (int mf = 0; mf < MF; ++mf) { both[mf] = part0[mf]; both[MF + mf] = part1[mf]; }
                store_sc1_and_wait<2 * MF>(my_parts + tid, kThreads, both);
            } else if (has_part0) {
                store_sc1_and_wait<MF>(my_parts + tid, kThreads, part0);
            } else if (has_part1) {
                store_sc1_and_wait<MF>(my_parts + MF * kThreads + tid, kThreads, part1);
            }
        }
    }
    wait_vmcnt<0>();   // tail copies still target the rings; partial tiles have reached memory
    if (npart == 0) return;

    finish_shared_blocks<MF, GROUP, OUT, kStreamThreads>(p, npart, part_block0, part_block1, m0, s_flag);
}

// ------------------------------------------------------------------------------------------
// "rstream" kernel: the same work partition as the kernel above, but no staging through LDS at all.
// Wave w of eight takes the w-th unit of each iteration (eight consecutive groups of one block) and, for that
// group, ALL four 16-channel fragments of the block: the 4 x 1 KiB of packed weights and the 16*MF x 128 bytes
// of activations go straight from memory into its registers (each lane loads exactly the 16-byte words its
// MFMA operands consist of), one iteration ahead.  Nothing is shared between waves, so the loop has no
// barriers, and an activation word is fetched once per four units instead of being read from LDS by every
// wave that consumes it -- LDS bandwidth, not HBM, bounded the staged kernel.  The eight partial sums of a
// block meet once per segment of the run, through LDS.
// ------------------------------------------------------------------------------------------
constexpr int kRsThreads = 512;
constexpr int kRsWaves = 8;

template <int MF, bool GROUP, int OUT>
__global__ __launch_bounds__(kRsThreads) void rstream_kernel(GemmDev p)
{
    constexpr int kEl = MF * kThreads;                              // int4 elements of a 64-channel tile: (mf * 4 + f) * 64 + lane
    constexpr int kRounds = (kEl + kRsThreads - 1) / kRsThreads;    // elements per thread after the reduction
    __shared__ int4 red[kRsWaves][kEl];
    __shared__ int s_flag[2];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wg = blockIdx.x;
    const int m0 = blockIdx.y * (16 * MF);
    const int G = p.G;
    const int blocks = p.N / 64;
    const int total = blocks * G;
    const int u0 = min(total, wg * p.upw), u1 = min(total, u0 + p.upw);
    if (u0 >= u1) return;                                  // whole workgroup: nothing to do
    const int q = lane >> 4, ml = lane & 15;
    const int nf_total = p.N / 16;

    RunShape run = make_run(u0, u1, G, kRsWaves);
    const int T = __builtin_amdgcn_readfirstlane(run.T);
    auto iteration = [&](int it) __attribute__((always_inline)) {
        IterInfo o = run_iteration(run, it);               // wave-uniform
        o.block = __builtin_amdgcn_readfirstlane(o.block);
        o.g = __builtin_amdgcn_readfirstlane(o.g);
        o.n = __builtin_amdgcn_readfirstlane(o.n);
        o.seg_end = __builtin_amdgcn_readfirstlane((int)o.seg_end) != 0;
        o.complete = __builtin_amdgcn_readfirstlane((int)o.complete) != 0;
        return o;
    };

    // lane (ml, q) holds, of every operand, row ml and the 16-byte k-chunk q
    uint32_t a_off[MF];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf)                        // rows past M repeat the last one; never stored
        a_off[mf] = (uint32_t)min(m0 + mf * 16 + ml, p.M - 1) * (uint32_t)p.K + (uint32_t)(q * 16);
    const char* abase = reinterpret_cast<const char*>(p.qx);

    struct Item { uint4 w[kNFrag]; uint32_t mt[kNFrag]; v4i a[MF][2]; };
    auto load_item = [&](Item& item, const IterInfo& o) __attribute__((always_inline)) {
        if (wave >= o.n) return;                           // no unit for this wave in that iteration
        const int g = o.g + wave;
        const int blk = o.block;
#pragma unroll
        for (int f = 0; f < kNFrag; ++f) {
            const int nf = blk * kNFrag + f;
            item.w[f] = p.codes[(size_t)((nf * G + g) << 6) + lane];
            if (GROUP) item.mt[f] = p.meta[((size_t)g * nf_total + nf) * 16 + ml];
        }
#pragma unroll
        for (int mf = 0; mf < MF; ++mf)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                item.a[mf][ks] = *reinterpret_cast<const v4i*>(abase + (a_off[mf] + (uint32_t)(g * kGroup + ks * 64)));
    };

    v4i acc[kNFrag][MF];
#pragma unroll
    for (int f = 0; f < kNFrag; ++f)
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) acc[f][mf] = (v4i){0, 0, 0, 0};
    auto compute = [&](const Item& item) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int f = 0; f < kNFrag; ++f) {
                uint32_t S = 0, B = 0;
                if (GROUP) {
                    S = __builtin_amdgcn_perm(item.mt[f], item.mt[f], 0x0c000c00u);  // s1 in both 16-bit lanes
                    B = __builtin_amdgcn_perm(item.mt[f], item.mt[f], 0x01010101u);  // bias in all four bytes
                }
                const v4i w_op = dequant<GROUP>(ks ? item.w[f].z : item.w[f].x, ks ? item.w[f].w : item.w[f].y, S, B);
#pragma unroll
                for (int mf = 0; mf < MF; ++mf)
                    acc[f][mf] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w_op, item.a[mf][ks], acc[f][mf], 0, 0, 0);
            }
    };

    // Partial tiles of the run (at most two: a first segment that starts inside a block, a last one that ends
    // inside a block) stay in registers, spread over the threads, until the loop is over.
    v4i part0[kRounds], part1[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) part0[r] = part1[r] = (v4i){0, 0, 0, 0};
    bool has_part0 = false, has_part1 = false;
    int npart = 0, part_block0 = 0, part_block1 = 0, seg_index = 0;   // (scalars: an indexed array would be moved to LDS)
    int4* my_parts = p.parts + (size_t)(blockIdx.y * gridDim.x + wg) * 2 * kEl;

    // One item ahead: the loads of the next iteration go out, then the current one is computed.  (Deeper
    // register prefetch with a fixed number of loads per iteration was measured and is no faster: the loop is not
    // bound by the bytes a wave has in flight.)
    IterInfo cur_i = iteration(0);
    Item cur;
    load_item(cur, cur_i);
    for (int it = 0; it < T; ++it) {
        IterInfo nxt_i = cur_i;
        Item nxt;                                          // (left unset when there is no next iteration: never used then)
        if (it + 1 < T) {
            nxt_i = iteration(it + 1);
            load_item(nxt, nxt_i);
        }
        if (wave < cur_i.n) compute(cur);
        if (cur_i.seg_end) {
            // ---- end of this run's share of a block: the eight waves' sums meet in LDS ----------------
            const bool complete = cur_i.complete;
            const int block_now = cur_i.block;
            uint2 c_s[kRounds];
            uint32_t c_z[kRounds];
            float c_sx[kRounds];
            int c_rs[kRounds];
            if (complete) {                                // epilogue constants: in flight across the barrier
#pragma unroll
                for (int r = 0; r < kRounds; ++r) {
                    const int el = min((int)threadIdx.x + r * kRsThreads, kEl - 1);
                    const int mf = el >> 8, f = (el >> 6) & 3, ln = el & 63;
                    const int m = min(m0 + mf * 16 + (ln & 15), p.M - 1);
                    const int n0 = block_now * 64 + 16 * (ln >> 4) + 4 * f;
                    c_s[r] = OUT == OUT_FP16 ? *reinterpret_cast<const uint2*>(p.scales + n0) : make_uint2(0, 0);
                    c_z[r] = GROUP ? 0u : *reinterpret_cast<const uint32_t*>(p.zeros + n0);
                    c_sx[r] = OUT == OUT_FP16 ? __half2float(p.sx[m]) : 0.f;
                    c_rs[r] = GROUP ? 0 : p.rowsum[m];
                }
            }
#pragma unroll
            for (int f = 0; f < kNFrag; ++f)
#pragma unroll
                for (int mf = 0; mf < MF; ++mf) {
                    red[wave][(mf * kNFrag + f) * 64 + lane] = make_int4(acc[f][mf].x, acc[f][mf].y, acc[f][mf].z, acc[f][mf].w);
                    acc[f][mf] = (v4i){0, 0, 0, 0};
                }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int el = (int)threadIdx.x + r * kRsThreads;
                if (el >= kEl) continue;
                v4i sum = (v4i){0, 0, 0, 0};
#pragma unroll
                for (int w = 0; w < kRsWaves; ++w) {
                    const int4 o = red[w][el];
                    sum += (v4i){o.x, o.y, o.z, o.w};
                }
                if (complete) {
                    const int mf = el >> 8, f = (el >> 6) & 3, ln = el & 63;
                    const int m = m0 + mf * 16 + (ln & 15);
                    if (m < p.M) {
                        const float sn[4] = {__half2float(__ushort_as_half((unsigned short)(c_s[r].x & 0xFFFFu))),
                                             __half2float(__ushort_as_half((unsigned short)(c_s[r].x >> 16))),
                                             __half2float(__ushort_as_half((unsigned short)(c_s[r].y & 0xFFFFu))),
                                             __half2float(__ushort_as_half((unsigned short)(c_s[r].y >> 16)))};
                        const int zn[4] = {(int)(c_z[r] & 0xFFu), (int)((c_z[r] >> 8) & 0xFFu), (int)((c_z[r] >> 16) & 0xFFu),
                                           (int)(c_z[r] >> 24)};
                        finish4<GROUP, OUT>(p, m, block_now * 64 + 16 * (ln >> 4) + 4 * f, sum, sn, zn, c_sx[r], c_rs[r]);
                    }
                } else if (seg_index == 0) {
                    part0[r] = sum;
                } else {
                    part1[r] = sum;
                }
            }
            if (!complete) {
                if (seg_index == 0) has_part0 = true; else has_part1 = true;
                if (npart == 0) part_block0 = block_now; else part_block1 = block_now;
                ++npart;
            }
            ++seg_index;
            __syncthreads();                               // `red` is free again
        }
        cur = nxt;
        cur_i = nxt_i;
    }

    // partial tiles -> workspace (write-through), then the hand-over
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int el = (int)threadIdx.x + r * kRsThreads;
        if (el >= kEl) continue;
        if (has_part0) store_through(my_parts + el, part0[r].x, part0[r].y, part0[r].z, part0[r].w);
        if (has_part1) store_through(my_parts + kEl + el, part1[r].x, part1[r].y, part1[r].z, part1[r].w);
    }
    wait_vmcnt<0>();
    if (npart == 0) return;
    finish_shared_blocks<MF, GROUP, OUT, kRsThreads>(p, npart, part_block0, part_block1, m0, s_flag);
}

// ------------------------------------------------------------------------------------------
// Lockstep-streaming kernel (64-token tiles, wide layers or a few hundred tokens).  Same copy scheme as the LDS-staged
// kernel, but a workgroup works on NB = 2 or 4 adjacent 64-channel blocks at once, so that the two activation slabs
// an iteration stages serve all of them: per byte of weights 1/NB of the activation bytes go through the vector
// cache, and 1/NB of the barriers are met.  Every consumer wave takes two of the 4 * NB fragments.
//   NB = 2 ("pairs"): wave (fp, e) takes fragments 2fp, 2fp + 1 and, in every iteration, the group of parity e: a
//       slab is read from LDS once per two fragments (80 KiB of LDS reads per 16 KiB of weights instead of the 144 a
//       wave-per-fragment cut needs, which made a first version no faster than the single-block kernel); at the end
//       of a pair the parity-1 waves hand their sums to the parity-0 waves through LDS, which run the epilogue.
//   NB = 4 ("quads"): wave w takes fragments 2w, 2w + 1 and both groups; no wave needs another's sums; 160 KiB of LDS
//       reads per 32 KiB of weights stay below what the copies cost.
// Workgroups own whole pairs / quads (p.upw of them, all K): no partial tiles, no workspace.  N % (64 * NB) == 0.
// The host picks this kernel where that many whole pairs / quads, times the token tiles, still fill the chip.
// ------------------------------------------------------------------------------------------
template <int NB, int MF, bool GROUP, int OUT>
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void lockstep_kernel(GemmDev p)
{
    static_assert(NB == 2 || NB == 4, "pairs or quads");
    static_assert(MF == 1 || MF == 2 || MF == 4, "token tiles of 16, 32 or 64");
    constexpr bool kParity = NB == 2;                  // consumer waves split the two groups of an iteration between them
    constexpr int kRing = 3;
    constexpr int kABlocks = 2 * MF;                   // 1 KiB blocks (m-fragment, k-step) per group
    constexpr int kAHalf = kABlocks / 2;
    constexpr int kWUnits = kParity ? 2 : 4;           // weight units a consumer wave copies per iteration
    constexpr int kMetaBytes = NB * 128;               // per group: 4 * NB fragments x 16 rows x uint16
    constexpr int kScaleBytes = NB * 128, kZeroBytes = NB * 64;
    constexpr int kMetaCopies = kMetaBytes / 256, kScaleCopies = kScaleBytes / 256;   // a copy moves 256 B; zero bytes: one copy
    constexpr int kSSlot = kScaleBytes + 256;          // scales, then the zero bytes (a 256-byte copy even where 128 are used)
    __shared__ uint4 wring[8][kRing][kWUnits][64];     // per consumer wave: [fragment] (pairs) or [group][fragment] (quads)
    __shared__ uint4 aring[kRing][2][kABlocks * 64];   // activation slabs of the iteration's two groups
    __shared__ uint4 mring[kRing][2][kMetaBytes / 16];
    __shared__ uint4 sring[kRing][kSSlot / 16];
    __shared__ int4 red[kParity ? 4 : 1][kParity ? 2 * MF * 64 : 1];   // pairs: sums of the parity-1 waves at the end of a pair
    __shared__ float sx_lds[16 * MF];
    __shared__ int rs_lds[16 * MF];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool producer = wave >= 8;
    const int pk = wave & 1, ph = (wave >> 1) & 1;     // producer: group of the iteration, half of its activation blocks
    const int w8 = wave & 7;
    const int e = kParity ? (w8 & 1) : 0;              // pairs: the consumer's group parity
    const int frag0 = kParity ? 2 * (w8 >> 1) : 2 * w8;   // the consumer's first fragment
    const int m0 = blockIdx.y * (16 * MF);
    const int G = p.G;
    const int sets = p.N / (64 * NB);                  // pairs or quads of blocks
    const int sb0 = min(sets, (int)blockIdx.x * p.upw), sb1 = min(sets, sb0 + p.upw);
    if (sb0 >= sb1) return;
    const int q = lane >> 4, ml = lane & 15;
    const int T = (sb1 - sb0) * ((G + 1) / 2);

    v4i acc[2][MF];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) acc[i][mf] = (v4i){0, 0, 0, 0};

    // ---- copies ---------------------------------------------------------------------------
    uint32_t a_voff[kAHalf];
    {
        const int r = lane >> 2, c = lane & 3;
        const int h = ((r >> 1) ^ (r >> 2)) & 3;
#pragma unroll
        for (int j = 0; j < kAHalf; ++j) {
            const int b = ph * kAHalf + j;
            const int row = min(m0 + (b >> 1) * 16 + r, p.M - 1);   // rows past M repeat the last one; never stored
            a_voff[j] = (uint32_t)row * (uint32_t)p.K + (uint32_t)((b & 1) * 64 + (c ^ h) * 16);
        }
    }
    const uint32_t lane4 = (uint32_t)lane * 4u, lane16 = (uint32_t)lane * 16u;
    const uint32_t wring_addr = (uint32_t)(uintptr_t)&wring[0][0][0][0] + (uint32_t)w8 * (kRing * kWUnits * 1024);
    const uint32_t aring_addr = (uint32_t)(uintptr_t)&aring[0][0][0] + (uint32_t)(pk * kABlocks + ph * kAHalf) * 1024u;
    const uint32_t mring_addr = (uint32_t)(uintptr_t)&mring[0][0][0] + (uint32_t)pk * kMetaBytes;
    const uint32_t sring_addr = (uint32_t)(uintptr_t)&sring[0][0];
    constexpr uint32_t kASlot = 2 * kABlocks * 1024, kWSlot = kWUnits * 1024, kMSlot = 2 * kMetaBytes;
    const char* abase = reinterpret_cast<const char*>(p.qx);
    const char* sbase = reinterpret_cast<const char*>(p.scales);
    const char* zbase = reinterpret_cast<const char*>(p.zeros);
    const char* codes_base = reinterpret_cast<const char*>(p.codes);
    const char* meta_base = reinterpret_cast<const char*>(p.meta);
    const uint32_t m_g_stride = (uint32_t)(p.N / 16) * 32u;
    // the 128 zero bytes of a pair fill half a copy: the upper lanes repeat them
    const uint32_t z_voff = kZeroBytes == 256 ? lane4 : (uint32_t)(lane & 31) * 4u;

    // The copy front runs kRing - 1 iterations ahead of the iteration being consumed; past the end of the run it
    // stays on the last iteration (every iteration issues the same number of copies, and a repeated copy reads
    // valid memory into a slot nobody reads any more).
    int csb = sb0, cg = 0, cleft = T;                  // set, first group, iterations left at the copy front
    auto issue = [&](int slot) __attribute__((always_inline)) {
        const int two = cg + 1 < G ? 1 : 0;            // the iteration has a second group
        if (producer) {
            const uint32_t gsel = (uint32_t)(cg + (pk & two));
#pragma unroll
            for (int b = 0; b < kAHalf; ++b)
                dma16(abase, a_voff[b] + gsel * (uint32_t)kGroup, aring_addr + slot * kASlot + b * 1024);
            if (GROUP && ph == 0) {
#pragma unroll
                for (int c = 0; c < kMetaCopies; ++c)
                    dma4(meta_base, lane4 + gsel * m_g_stride + (uint32_t)csb * kMetaBytes + c * 256u, mring_addr + slot * kMSlot + c * 256);
            }
            if (pk == 0 && ph == 1) {
#pragma unroll
                for (int c = 0; c < kScaleCopies; ++c)
                    dma4(sbase, lane4 + (uint32_t)csb * kScaleBytes + c * 256u, sring_addr + slot * kSSlot + c * 256);
            }
            if (!GROUP && pk == 1 && ph == 1) dma4(zbase, z_voff + (uint32_t)csb * kZeroBytes, sring_addr + slot * kSSlot + kScaleBytes);
        } else {
            const uint32_t nf = (uint32_t)G << 10;      // the next fragment's units lie G KiB further
            if constexpr (kParity) {
                const uint32_t unit = ((uint32_t)(csb * (4 * NB) + frag0) * (uint32_t)G + (uint32_t)(cg + (e & two))) << 10;
                dma16(codes_base, lane16 + unit, wring_addr + slot * kWSlot);
                dma16(codes_base, lane16 + unit + nf, wring_addr + slot * kWSlot + 1024);
            } else {
                const uint32_t unit = ((uint32_t)(csb * (4 * NB) + frag0) * (uint32_t)G + (uint32_t)cg) << 10;
                const uint32_t ng = (uint32_t)two << 10;   // the next group's unit follows (the same one again on an odd tail)
                dma16(codes_base, lane16 + unit, wring_addr + slot * kWSlot);
                dma16(codes_base, lane16 + unit + nf, wring_addr + slot * kWSlot + 1024);
                dma16(codes_base, lane16 + unit + ng, wring_addr + slot * kWSlot + 2048);
                dma16(codes_base, lane16 + unit + ng + nf, wring_addr + slot * kWSlot + 3072);
            }
        }
        if (cleft > 1) {
            --cleft;
            cg += 2;
            if (cg >= G) { cg = 0; ++csb; }
        }
    };

    const int hsw = ((ml >> 1) ^ (ml >> 2)) & 3;
    const int a_src = 4 * ml + (q ^ hsw);
    auto compute = [&](int slot, int grp) __attribute__((always_inline)) {   // the wave's two fragments x group grp of the iteration
        const int u = kParity ? 0 : 2 * grp;
        const uint4 wq0 = wring[w8][slot][u][lane], wq1 = wring[w8][slot][u + 1][lane];
        uint32_t S0 = 0, B0 = 0, S1 = 0, B1 = 0;
        if (GROUP) {
            const uint16_t* mrow = reinterpret_cast<const uint16_t*>(&mring[slot][grp][0]);
            const uint32_t mt0 = mrow[frag0 * 16 + ml], mt1 = mrow[(frag0 + 1) * 16 + ml];
            S0 = __builtin_amdgcn_perm(mt0, mt0, 0x0c000c00u); B0 = __builtin_amdgcn_perm(mt0, mt0, 0x01010101u);
            S1 = __builtin_amdgcn_perm(mt1, mt1, 0x0c000c00u); B1 = __builtin_amdgcn_perm(mt1, mt1, 0x01010101u);
        }
        const uint4* slab = aring[slot][grp];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i a_op[MF];
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) a_op[mf] = as_v4i(slab[(mf * 2 + ks) * 64 + a_src]);
            const v4i w0 = dequant<GROUP>(ks ? wq0.z : wq0.x, ks ? wq0.w : wq0.y, S0, B0);
            const v4i w1 = dequant<GROUP>(ks ? wq1.z : wq1.x, ks ? wq1.w : wq1.y, S1, B1);
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) {
                acc[0][mf] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w0, a_op[mf], acc[0][mf], 0, 0, 0);
                acc[1][mf] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w1, a_op[mf], acc[1][mf], 0, 0, 0);
            }
        }
    };
    // epilogue of the wave's two fragments of set sb; `other` = sums to add first (pairs: the parity-1 wave's)
    auto finish = [&](int sb, int slot, const int4* other) __attribute__((always_inline)) {
        const char* sc = reinterpret_cast<const char*>(&sring[slot][0]);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int f = frag0 + i;                   // fragment of the set: block f / 4, fragment f % 4 of it
            const int nl = (f >> 2) * 64 + 16 * q + 4 * (f & 3);
            const uint2 sw = *reinterpret_cast<const uint2*>(sc + nl * 2);
            float sn[4];
            int zn[4] = {0, 0, 0, 0};
            if (!GROUP) {
                const uint32_t zw = *reinterpret_cast<const uint32_t*>(sc + kScaleBytes + nl);
#pragma unroll
                for (int j = 0; j < 4; ++j) zn[j] = (int)((zw >> (8 * j)) & 0xFFu);
            }
            sn[0] = __half2float(__ushort_as_half((unsigned short)(sw.x & 0xFFFFu)));
            sn[1] = __half2float(__ushort_as_half((unsigned short)(sw.x >> 16)));
            sn[2] = __half2float(__ushort_as_half((unsigned short)(sw.y & 0xFFFFu)));
            sn[3] = __half2float(__ushort_as_half((unsigned short)(sw.y >> 16)));
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) {
                v4i v = acc[i][mf];
                if (other) {
                    const int4 o = other[(i * MF + mf) * 64 + lane];
                    v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
                }
                acc[i][mf] = (v4i){0, 0, 0, 0};
                const int m = m0 + mf * 16 + ml;
                if (m < p.M) finish4<GROUP, OUT>(p, m, sb * (64 * NB) + nl, v, sn, zn, sx_lds[mf * 16 + ml], rs_lds[mf * 16 + ml]);
            }
        }
    };

    // ---- main loop: one wait + one barrier per iteration, as in the staged kernel -------------------------
#pragma unroll
    for (int k = 0; k < kRing - 1; ++k) issue(k);
    if (wave == 11 && lane < 16 * MF) {
        const int m = min(m0 + lane, p.M - 1);
        sx_lds[lane] = OUT == OUT_FP16 ? __half2float(p.sx[m]) : 0.f;
        rs_lds[lane] = GROUP ? 0 : p.rowsum[m];
    }
    // copies per iteration and wave: consumers kWUnits; producers their activation blocks plus metadata, scales or zero bytes
    const int my_dma = !producer ? kWUnits
                     : kAHalf + ((GROUP && ph == 0) ? kMetaCopies : 0) + ((pk == 0 && ph == 1) ? kScaleCopies : 0) +
                           ((!GROUP && pk == 1 && ph == 1) ? 1 : 0);
    int sb = sb0, g = 0, slot = 0;
    for (int it = 0; it < T; ++it) {
        // (1 ... 6 copies per wave and iteration, depending on role, mode and tile)
        if (my_dma == 1) wait_vmcnt<(kRing - 2) * 1>();
        else if (my_dma == 2) wait_vmcnt<(kRing - 2) * 2>();
        else if (my_dma == 3) wait_vmcnt<(kRing - 2) * 3>();
        else if (my_dma == 4) wait_vmcnt<(kRing - 2) * 4>();
        else if (my_dma == 5) wait_vmcnt<(kRing - 2) * 5>();
        else wait_vmcnt<(kRing - 2) * 6>();
        __syncthreads();
        issue(slot == 0 ? kRing - 1 : slot - 1);
        const bool two = g + 1 < G, last = g + 2 >= G;   // uniform over the workgroup
        if constexpr (kParity) {
            if (!producer && (e == 0 || two)) compute(slot, e);
            if (last) {
                if (!producer && e == 1) {
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int mf = 0; mf < MF; ++mf) {
                            red[w8 >> 1][(i * MF + mf) * 64 + lane] = make_int4(acc[i][mf].x, acc[i][mf].y, acc[i][mf].z, acc[i][mf].w);
                            acc[i][mf] = (v4i){0, 0, 0, 0};
                        }
                }
                __syncthreads();
                if (!producer && e == 0) finish(sb, slot, &red[w8 >> 1][0]);
            }
        } else {
            if (!producer) {
                compute(slot, 0);
                if (two) compute(slot, 1);
                if (last) finish(sb, slot, nullptr);
            }
        }
        g += 2;
        if (g >= G) { g = 0; ++sb; }
        slot = slot + 1 == kRing ? 0 : slot + 1;
    }
    wait_vmcnt<0>();   // tail copies still target the rings
}

// ------------------------------------------------------------------------------------------
// "mma" kernel (compute bound, M > 64).  Four waves per workgroup, exactly one per SIMD; a wave owns
// 128 tokens x (32 * CF) channels in 4 x CF accumulator tiles of v_mfma_i32_32x32x32_i8 (CF = 4: 256
// accumulator registers per lane).  Four workgroup shapes share the code:
//     CF = 4, waves 2 x 2 : 256 tokens x 256 channels  (large problems: fewest bytes per MFMA)
//     CF = 2, waves 1 x 4 : 128 tokens x 256 channels  (few tokens)
//     CF = 2, waves 2 x 2 : 256 tokens x 128 channels  (few channels)
//     CF = 3, waves 2 x 2 : 256 tokens x 192 channels  (tile counts that fill the CUs where 256 x 256 leaves a
//                           quarter idle, e.g. N = 12288).  A wave's three 32-row fragments are then every second
//                           one of the tile's six, so that both waves see the same half of every 64-channel block.
// With one wave per SIMD nothing but that wave's own instruction stream keeps the matrix pipe busy, so the
// main loop is software pipelined by hand into "chunks" of one MFMA (32 cycles) plus what fits in its
// shadow: a quarter of the dequantization of a LATER weight operand (one operand = 4 dwords, reused by the
// four token fragments of the wave: 3.5 vector instructions per MFMA), at most two LDS reads and at most
// one copy.  A scheduling barrier after every chunk keeps the compiler from regrouping them.
//
// Copies are global->LDS DMA.  Activations, packed weights (the 16-byte lane word covers both halves of a group) and
// metadata live in rings of three group slabs; an activation copy moves eight tokens x 128 k, i.e. whole cache
// lines.  The main loop works in half-group steps (k = 64); every half-stage's operands are read into registers
// during the half-stage before.  There is one barrier per group, in the middle of its second half-stage: a wave
// first waits for its own copies of group g+1, all waves meet (that publishes g+1 and proves group g's slabs are
// no longer read), and the slabs of group g are refilled with group g+3 -- four half-stages of lead.  The rest of
// the half-stage overlaps the first LDS reads and the first dequantization of g+1, so the matrix pipe does not
// drain at the barrier.  grid = (m-tiles * n-tiles, k-slices).
// ------------------------------------------------------------------------------------------
typedef int v16i __attribute__((ext_vector_type(16)));
constexpr int kMmaThreads = 256;
// Ring depth (template parameter DEPTH): slabs of one quantization group each -- activations (tokens of the tile x
// 128 k), weights (channels of the tile x 128 k, 1 KiB per 16 channels), metadata.  3 = one workgroup per compute
// unit that hides the memory latency by its own lead of two groups; 2 = rings small enough for two workgroups per
// compute unit (two waves per SIMD: while one waits for its copies or at its barrier, the other one's matrix
// instructions keep the pipe busy).
constexpr int kMSlotBytes = 1024;                   // metadata: 256 B per copying wave

template <bool GROUP, int OUT, int CF, int WM, int DEPTH>
__global__ __launch_bounds__(kMmaThreads, DEPTH == 2 ? 2 : 1) void mma_kernel(GemmDev p)
{
    static_assert(DEPTH == 2 || DEPTH == 3, "ring depth");
    constexpr int kASlots = DEPTH, kWSlots = DEPTH;
    constexpr int WN = 4 / WM;                      // waves along the channels
    constexpr int TMt = 128 * WM, TNt = 32 * CF * WN;   // tile: tokens x channels
    constexpr int kABlocks = TMt / 16;              // 1 KiB blocks (16 tokens x 64 k) per activation slab
    constexpr int kUnits = TNt / 16;                // 1 KiB weight units per slab
    constexpr int kASlotBytes = 2 * kABlocks * 1024, kWSlotBytes = kUnits * 1024;   // a group of a tile: 128 B per token
    constexpr int kACopies = kABlocks / 4, kWCopies = kUnits / 4;     // per wave
    constexpr int NB = 2 * CF;                      // blocks (k32-step jj, channel fragment cf) per half-stage
    constexpr int NC = 4 * NB;                      // chunks per half-stage
    constexpr int BAR = CF == 4 ? 16 : CF == 3 ? 12 : 4;   // chunk in front of which the half-stage's barrier sits
    constexpr int kFragStep = (CF & 1) ? WN : 1;    // distance, in 32-row fragments, between a wave's fragments
    static_assert(!(CF & 1) || WN == 2, "an odd CF interleaves the fragments of two waves");
    __shared__ __attribute__((aligned(16))) char aring[kASlots * kASlotBytes];
    __shared__ __attribute__((aligned(16))) char wring[kWSlots * kWSlotBytes];
    __shared__ __attribute__((aligned(16))) char mring[kWSlots * kMSlotBytes];
    __shared__ __attribute__((aligned(16))) char ering[2304];   // sx[256] fp16 | s[256] fp16 | rowsum[256] | zeros[256]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int G = p.G;
    // split-k: blockIdx.y selects a run of p.gps groups; the slices of a tile meet in the workspace (below)
    const int slice = blockIdx.y;
    const int g_first = slice * p.gps, Gs = min(G - g_first, p.gps);
    // Workgroup -> tile.  Consecutive workgroup ids land on consecutive XCDs (8, each with its own L2), so
    // workgroup i is the (i / 8)-th of XCD i % 8.  Each XCD gets a contiguous run of a tile order that walks
    // panels of four token tiles column by column: the 32 tiles an XCD works on at a time form a 4 x 8 block
    // sharing 4 activation slabs and 8 weight slabs through that XCD's L2.
    const int n_tiles = (p.N + TNt - 1) / TNt, m_tiles = (p.M + TMt - 1) / TMt;
    int tm, tn;
    {
        const int T = n_tiles * m_tiles, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int q = T >> 3, r = T & 7;
        const int L = xcd * q + min(xcd, r) + slot;      // slot < q + (xcd < r) because blockIdx.x < T
        constexpr int kPanel = 4;
        const int per_panel = kPanel * n_tiles;
        const int panel = L / per_panel;
        const int rows = min(kPanel, m_tiles - panel * kPanel);
        const int rem = L - panel * per_panel;
        tn = rem / rows;
        tm = panel * kPanel + (rem - tn * rows);
    }
    const int m_base = tm * TMt, n_base = tn * TNt;
    const int nf_base = tn * kUnits;                     // first 16-row fragment (unit row) of the tile
    const int nf_total = p.N / 16;

    // ---- copy role: wave w copies a quarter of the tile's tokens, weight units kWCopies*w.. and their metadata.
    // One activation copy = eight tokens x one whole quantization group: every eight lanes fetch one whole 128-byte
    // line (the vector cache works in whole lines: 16 tokens x 64 bytes per copy, half a line each, was measured to
    // cost it twice the requests for the same bytes).  Lane 8r+c fetches 16-byte chunk c ^ row_swizzle(r) of token
    // row r, which keeps the fragment reads free of bank conflicts.  The
    // copies of a group are issued in two halves, after the barriers of two consecutive half-stages.
    constexpr int kAll = 2 * kACopies + kWCopies + (GROUP ? 1 : 0);   // copies per wave and group
    static_assert((DEPTH - 1) * kAll < 64, "vmcnt range");
    static_assert(kAll <= NC - BAR, "one copy per chunk after the barrier");
    static_assert(kACopies % 2 == 0, "copy t of either half starts at row 8 * (t & 1) modulo 16");
    uint32_t a_voff[2][kACopies];                      // [half of the group's copies][copy]
    {
        const int r = lane >> 3, c = lane & 7;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int t = 0; t < kACopies; ++t) {
                const int row = min(m_base + ((wave * 2 + hf) * kACopies + t) * 8 + r, p.M - 1);   // rows past M repeat the last one
                a_voff[hf][t] = (uint32_t)row * (uint32_t)p.K + (uint32_t)((c ^ row_swizzle(((t & 1) << 3) | r)) * 16);   // (a wave's copies start at a multiple of 16 rows)
            }
    }
    const uint32_t w_voff = (uint32_t)lane * 16u;
    // metadata: 32 B per unit; lane l copies dword l % 8 of the wave's unit l / 8 (units past N repeat the last one,
    // lanes past the wave's units repeat its last dword)
    const int m_lane = min(lane, kWCopies * 8 - 1);
    const uint32_t m_voff = (uint32_t)min(nf_base + wave * kWCopies + (m_lane >> 3), nf_total - 1) * 32u + (uint32_t)(m_lane & 7) * 4u;
    const uint32_t a_dst = (uint32_t)(uintptr_t)&aring[0] + (uint32_t)(wave * 2 * kACopies) * 1024u;
    const uint32_t w_dst = (uint32_t)(uintptr_t)&wring[0] + (uint32_t)(wave * kWCopies) * 1024u;
    const uint32_t m_dst = (uint32_t)(uintptr_t)&mring[0] + (uint32_t)wave * 256u;
    const char* abase = reinterpret_cast<const char*>(p.qx);
    const char* wrow[kWCopies];
#pragma unroll
    for (int u = 0; u < kWCopies; ++u)   // units past N repeat the last one; their results are never stored
        wrow[u] = reinterpret_cast<const char*>(p.codes) + (size_t)min(nf_base + wave * kWCopies + u, nf_total - 1) * G * 1024;
    const char* mrow = reinterpret_cast<const char*>(p.meta);
    const size_t m_g_stride = (size_t)nf_total * 32;
    int ca = g_first, cw = g_first;   // next group of activations / weights to copy; past the end of the slice the last one is copied again into a free slab
    const int cw_last = g_first + Gs - 1;
    auto copy_a = [&](int t, int hf, int slot) {
        dma16(abase + (size_t)ca * kGroup, a_voff[hf][t], a_dst + (uint32_t)(slot * kASlotBytes + (hf * kACopies + t) * 1024));
    };
    auto copy_w = [&](int u, int slot) { dma16(wrow[u] + (size_t)cw * 1024, w_voff, w_dst + (uint32_t)(slot * kWSlotBytes + u * 1024)); };
    auto copy_m = [&](int slot) { if (GROUP) dma4(mrow + (size_t)cw * m_g_stride, m_voff, m_dst + (uint32_t)(slot * kMSlotBytes)); };
    auto adv_a = [&]() { ca = min(ca + 1, cw_last); };
    auto adv_w = [&]() { cw = min(cw + 1, cw_last); };
    // k-th copy a wave issues after a group's barrier: the next group but two, into the slabs the barrier has freed
    auto refill = [&](int k, int islot) {
        if (k < 2 * kACopies) copy_a(k % kACopies, k / kACopies, islot);
        else if (k < 2 * kACopies + kWCopies) copy_w(k - 2 * kACopies, islot);
        else if (k == 2 * kACopies + kWCopies) copy_m(islot);
    };

    // Epilogue constants of the tile (token scales, channel scales; per-channel mode: token sums, zero points)
    // are copied into LDS first of all, so they are the oldest entries of each wave's copy queue and cost no
    // separate wait.  256 entries of each are fetched whatever the tile shape; indices past M / N repeat the
    // last valid dword and are never used.
    {
        const uint32_t e_dst = (uint32_t)(uintptr_t)&ering[0];
        const int d = wave * 64 + lane;
        if (OUT == OUT_FP16) {
            if (wave < 2)      // waves 0, 1: 2 x 64 dwords = 256 token scales
                dma4(reinterpret_cast<const char*>(p.sx) + (size_t)m_base * 2, (uint32_t)min(d, (p.M - m_base - 1) >> 1) * 4u,
                     e_dst + (uint32_t)wave * 256u);
            else               // waves 2, 3: 256 channel scales
                dma4(reinterpret_cast<const char*>(p.scales) + (size_t)n_base * 2,
                     (uint32_t)min(d - 128, ((p.N - n_base) >> 1) - 1) * 4u, e_dst + 512u + (uint32_t)(wave - 2) * 256u);
        }
        if (!GROUP) {
            dma4(reinterpret_cast<const char*>(p.rowsum) + (size_t)m_base * 4, (uint32_t)min(d, p.M - m_base - 1) * 4u,
                 e_dst + 1024u + (uint32_t)wave * 256u);
            if (wave == 0)
                dma4(reinterpret_cast<const char*>(p.zeros) + (size_t)n_base, (uint32_t)min(lane, ((p.N - n_base) >> 2) - 1) * 4u,
                     e_dst + 2048u);
        }
    }

    // prologue: the first DEPTH groups, each in the order of the steady state
#pragma unroll
    for (int gg = 0; gg < DEPTH; ++gg) {
#pragma unroll
        for (int k = 0; k < kAll; ++k) refill(k, gg);
        adv_a();
        adv_w();
    }

    // ---- compute role ---------------------------------------------------------------------------
    const int wm = wave / WN, wn = wave % WN;            // 128-token part, (32 * CF)-channel part of the tile
    const int frag0 = (CF & 1) ? wn : wn * CF;           // first 32-row fragment of the wave inside the tile
    const int r32 = lane & 31, kb2 = lane >> 5;
    v16i acc[CF][4];                                     // [channel fragment][token fragment]
#pragma unroll
    for (int a = 0; a < CF; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

    // LDS byte offsets of this lane's operands inside a slab.
    //   activations, token fragment tf (+ tf * 4096), half hf of the group, k32-step jj of that half: token
    //   wm*128 + tf*32 + r32 -> row of 128 bytes, 16-byte chunk (4hf + 2jj + kb2) ^ row_swizzle(token % 16)
    uint32_t a_rd[2][2], w_rd[2];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
            a_rd[hf][jj] = (uint32_t)((wm * 128 + r32) * 128 + (((4 * hf + 2 * jj + kb2) ^ row_swizzle(r32 & 15)) * 16));
        //   weights, channel fragment cf (+ cf * 2048; 32 rows = units 2cf, 2cf+1), both halves in one lane word:
        //   unit 2 * (frag0 + cf * kFragStep) + r32/16, lane word ((2jj + kb2) % 4) * 16 + r32 % 16
        w_rd[jj] = (uint32_t)((2 * frag0 + (r32 >> 4)) * 1024 + ((((2 * jj + kb2) & 3) * 16) + (r32 & 15)) * 16);
    }
    //   metadata of that unit u: in the 256 B of copying wave u / kWCopies, 32 B per unit
    uint32_t m_rd[CF];
#pragma unroll
    for (int cf = 0; cf < CF; ++cf) {
        const int u = 2 * (frag0 + cf * kFragStep) + (r32 >> 4);
        m_rd[cf] = (uint32_t)((u / kWCopies) * 256 + ((u % kWCopies) * 16 + (r32 & 15)) * 2);
    }

    auto lds_a = [&](uint32_t slab, int hf, int jj, int tf) {
        return as_v4i(*reinterpret_cast<const uint4*>(aring + slab + a_rd[hf][jj] + tf * 4096));
    };
    auto lds_w = [&](uint32_t slab, int blk) {           // lane word (both halves) of block blk = (jj, cf)
        return *reinterpret_cast<const uint4*>(wring + slab + w_rd[blk / CF] + (blk % CF) * (2048 * kFragStep));
    };
    auto lds_m = [&](uint32_t slab, int cf) {
        return (uint32_t)*reinterpret_cast<const uint16_t*>(mring + slab + m_rd[cf]);
    };
    const uint32_t nib_mask = 0x0F0F0F0Fu, sign = 0x80808080u;
    auto src_dword = [&](uint4 r, int half, int d) { return half == 0 ? (d < 2 ? r.x : r.y) : (d < 2 ? r.z : r.w); };
    auto deq1 = [&](uint4 r, int half, int d, uint32_t S, uint32_t B) {   // dword d of the operand of k-half `half`
        const uint32_t x = src_dword(r, half, d);
        uint32_t v = (d & 1) ? (x >> 4) & nib_mask : x & nib_mask;
        if (GROUP) v = pk_mad_u16(v, S, B) ^ sign;
        return (int)v;
    };
    // The same dequantization cut into four phases of 3-4 instructions, one phase per chunk, with the
    // multiply-add of one dword and the sign flip of the previous one interleaved so that no result is
    // consumed by the very next instruction.  t[] carries the dwords in progress, o[] receives the operand.
    auto deq_phase = [&](int ph, uint4 r, int half, uint32_t S, uint32_t B, uint32_t (&t)[4], v4i& o) {
        if (ph == 0) {
            t[0] = src_dword(r, half, 0) & nib_mask;
            t[1] = (src_dword(r, half, 1) >> 4) & nib_mask;
            if (GROUP) t[0] = pk_mad_u16(t[0], S, B);
        } else if (ph == 1) {
            if (GROUP) t[1] = pk_mad_u16(t[1], S, B);
            o.x = (int)(GROUP ? t[0] ^ sign : t[0]);
            t[2] = src_dword(r, half, 2) & nib_mask;
            t[3] = (src_dword(r, half, 3) >> 4) & nib_mask;
        } else if (ph == 2) {
            if (GROUP) t[2] = pk_mad_u16(t[2], S, B);
            o.y = (int)(GROUP ? t[1] ^ sign : t[1]);
            if (GROUP) t[3] = pk_mad_u16(t[3], S, B);
        } else {
            o.z = (int)(GROUP ? t[2] ^ sign : t[2]);
            o.w = (int)(GROUP ? t[3] ^ sign : t[3]);
        }
    };

    // first barrier: group 0 has landed everywhere
    wait_vmcnt<(DEPTH - 1) * kAll>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    uint32_t S[CF], B[CF], mt[CF];
#pragma unroll
    for (int cf = 0; cf < CF; ++cf) {
        S[cf] = B[cf] = mt[cf] = 0;
        if (GROUP) {
            mt[cf] = lds_m(0, cf);
            S[cf] = __builtin_amdgcn_perm(mt[cf], mt[cf], 0x0c000c00u);
            B[cf] = __builtin_amdgcn_perm(mt[cf], mt[cf], 0x01010101u);
        }
    }
    // Register-level pipeline.  rq[blk]: lane words (both k-halves) of the NB blocks of a group.  CF = 4: blocks
    // 4..7 are read during blocks 0..3 of the first half-stage, blocks 0..3 of the next group after the barrier
    // of the second.  CF = 2: all four of the next group are read during the second half-stage, each as soon as
    // its register is free.  a0: activations of k32-step 0 of a half-stage, a1[s]: k32-step 1 (two sets); both
    // are read after the barrier of the half-stage before.
    uint4 rq[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) rq[i] = (CF == 2 || i < NB / 2) ? lds_w(0, i) : make_uint4(0, 0, 0, 0);
    v4i a0[4], a1[2][4];
#pragma unroll
    for (int tf = 0; tf < 4; ++tf) { a0[tf] = lds_a(0, 0, 0, tf); a1[0][tf] = lds_a(0, 0, 1, tf); a1[1][tf] = (v4i){0, 0, 0, 0}; }
    v4i w_cur = {deq1(rq[0], 0, 0, S[0], B[0]), deq1(rq[0], 0, 1, S[0], B[0]), deq1(rq[0], 0, 2, S[0], B[0]), deq1(rq[0], 0, 3, S[0], B[0])};
    v4i w_nxt = {0, 0, 0, 0};
    uint32_t dq[4] = {0, 0, 0, 0};
    deq_phase(0, rq[1], 0, S[1 % CF], B[1 % CF], dq, w_nxt);   // block 1 is one phase ahead, as in the steady state

    int gs = 0;                                          // g % DEPTH
    for (int g = 0; g < Gs; ++g) {
        const int gp1 = gs == DEPTH - 1 ? 0 : gs + 1;
#pragma unroll
        for (int s = 0; s < 2; ++s) {                    // half-stage h = 2g + s
            const uint32_t a_nxt = (uint32_t)((s == 0 ? gs : gp1) * kASlotBytes);   // slab of the next half-stage: half 1 - s of this / the next group
            const uint32_t w_this = (uint32_t)(gs * kWSlotBytes), w_next = (uint32_t)(gp1 * kWSlotBytes);
            const uint32_t m_nxt = (uint32_t)(gp1 * kMSlotBytes);
#pragma unroll
            for (int c = 0; c < NC; ++c) {               // chunk = (block b = (jj, cf), token fragment tf)
                const int b = c >> 2, tf = c & 3, jj = b / CF, cf = b % CF;
                if (c == BAR && s == 1) {
                    // One barrier per group, in its second half-stage.  Before it a wave waits for its own copies of
                    // group g+1 (those of g+2 may be in flight) and for its outstanding LDS reads; all waves meeting
                    // publishes group g+1 and proves that nobody reads group g's slabs any more (its second k-half
                    // went to registers during the first half-stage): they are refilled with group g+DEPTH.
                    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"((DEPTH - 2) * kAll) : "memory");
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                }
                if (tf == 0 && c != 0) w_cur = w_nxt;    // (for c == 0 the hand-over happened at the end of the previous half-stage)
                acc[cf][tf] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w_cur, jj == 0 ? a0[tf] : a1[s][tf], acc[cf][tf], 0, 0, 0);
                {   // one phase of a later operand: chunks (b,0..2) finish block b+1, chunk (b,3) starts block b+2;
                    // blocks NB, NB+1 are blocks 0, 1 of the next half-stage
                    const int ph = (tf + 1) & 3;
                    const int tb = ph == 0 ? b + 2 : b + 1;
                    const int half = tb >= NB ? 1 - s : s;
                    deq_phase(ph, rq[tb % NB], half, S[tb % CF], B[tb % CF], dq, w_nxt);
                }
                if (CF == 4) {
                    if (tf == 0) {                       // lane words four blocks ahead
                        if (s == 0 && b < 4) rq[b + 4] = lds_w(w_this, b + 4);
                        if (s == 1 && b >= 4) rq[b - 4] = lds_w(w_next, b - 4);
                    }
                    if (b >= 4 && (tf & 1)) {            // activations of the next half-stage, two fragments per block
                        const int q = (b & 1) * 2 + (tf >> 1);
                        if (b < 6) a0[q] = lds_a(a_nxt, 1 - s, 0, q);
                        else a1[1 - s][q] = lds_a(a_nxt, 1 - s, 1, q);
                    }
                    if (GROUP && s == 1) {               // level-2 constants of the next group, each after the last use of the old one
                        if (b == 4) mt[tf] = lds_m(m_nxt, tf);
                        const int pc = c == 20 ? 0 : c == 22 ? 1 : c == 24 ? 2 : c == 28 ? 3 : -1;
                        if (pc >= 0) {
                            S[pc] = __builtin_amdgcn_perm(mt[pc], mt[pc], 0x0c000c00u);
                            B[pc] = __builtin_amdgcn_perm(mt[pc], mt[pc], 0x01010101u);
                        }
                    }
                } else if (CF == 3) {
                    // 24 chunks, barrier in front of chunk 12.  Lane words: 3..5 of this group during blocks 0..2 of
                    // the first half-stage, 0..2 of the next group during blocks 3..5 of the second (each register is
                    // free by then: block b's second half is dequantized one block ahead).  Activations of the next
                    // half-stage in the eight chunks after the barrier (a0 is last used in block 2).  Level-2 constants
                    // of the next group: S[cf] is last used in chunk 4 * (cf + 2) + 1 and next in chunk 4 * cf + 19.
                    if (tf == 0) {
                        if (s == 0 && b < 3) rq[b + 3] = lds_w(w_this, b + 3);
                        if (s == 1 && b >= 3) rq[b - 3] = lds_w(w_next, b - 3);
                    }
                    if (c >= 12 && c <= 15) a0[c - 12] = lds_a(a_nxt, 1 - s, 0, c - 12);
                    if (c >= 16 && c <= 19) a1[1 - s][c - 16] = lds_a(a_nxt, 1 - s, 1, c - 16);
                    if (GROUP && s == 1) {
                        if (b == 3 && tf < 3) mt[tf] = lds_m(m_nxt, tf);
                        const int pc = c == 16 ? 0 : c == 18 ? 1 : c == 20 ? 2 : -1;
                        if (pc >= 0) {
                            S[pc] = __builtin_amdgcn_perm(mt[pc], mt[pc], 0x0c000c00u);
                            B[pc] = __builtin_amdgcn_perm(mt[pc], mt[pc], 0x01010101u);
                        }
                    }
                } else {
                    if (s == 1) {                        // lane words of the next group, each once its register is free
                        const int e = c == 4 ? 0 : c == 5 ? 1 : c == 8 ? 2 : c == 12 ? 3 : -1;
                        if (e >= 0) rq[e] = lds_w(w_next, e);
                    }
                    if (c >= 5 && c <= 8) a0[c - 5] = lds_a(a_nxt, 1 - s, 0, c - 5);          // a0[q] is last used in chunk 4 + q
                    if (c >= 9 && c <= 12) a1[1 - s][c - 9] = lds_a(a_nxt, 1 - s, 1, c - 9);
                    if (GROUP && s == 1) {
                        if (c == 4) mt[0] = lds_m(m_nxt, 0);
                        if (c == 6) mt[1] = lds_m(m_nxt, 1);
                        const int pc = c == 8 ? 0 : c == 12 ? 1 : -1;                  // old S[0] / S[1] are last used in chunks 5 / 9
                        if (pc >= 0) {
                            S[pc] = __builtin_amdgcn_perm(mt[pc], mt[pc], 0x0c000c00u);
                            B[pc] = __builtin_amdgcn_perm(mt[pc], mt[pc], 0x01010101u);
                        }
                    }
                }
                if (s == 1 && c >= BAR) refill(c - BAR, gs);   // refill the slabs the barrier has just freed
                __builtin_amdgcn_sched_barrier(0);
            }
            w_cur = w_nxt;
            if (s == 1) { adv_a(); adv_w(); }
        }
        gs = gp1;
    }

    wait_vmcnt<0>();   // the repeated tail copies still target the ring

    // ---- split-k: every slice writes its partial tile through to memory and bumps the tile's counter; the last
    // one to arrive adds the others' (integer sums: exact, order independent) and alone runs the epilogue.
    // Same fence-free hand-over as in the streaming kernel; the counter is left at zero for the next launch.
    if (p.S > 1) {
        __shared__ int s_last;
        constexpr int NJ = CF * 16;                      // int4 per thread in a partial tile
        const int tile_id = tm * n_tiles + tn;
        int4* mine = p.parts + ((size_t)(tile_id * p.S + slice) * NJ) * kMmaThreads + threadIdx.x;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int cf = j >> 4, tf = (j >> 2) & 3, qd = j & 3;
            store_sc1(mine + (size_t)j * kMmaThreads, (v4i){acc[cf][tf][4 * qd], acc[cf][tf][4 * qd + 1], acc[cf][tf][4 * qd + 2],
                                                            acc[cf][tf][4 * qd + 3]});
        }
        wait_vmcnt<0>();
        __syncthreads();
        if (threadIdx.x == 0) {
            int* ctr = p.counters + tile_id;
            const int old = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = old == p.S - 1;
            if (s_last) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (!s_last) return;
        for (int s2 = 0; s2 < p.S; ++s2) {
            if (s2 == slice) continue;
            const int4* theirs = p.parts + ((size_t)(tile_id * p.S + s2) * NJ) * kMmaThreads + threadIdx.x;
#pragma unroll
            for (int j0 = 0; j0 < NJ; j0 += 16) {          // sixteen loads in flight: the sum is pure load latency
                v4i t[16];
#pragma unroll
                for (int x = 0; x < 16; ++x) load_sc1_nowait(t[x], theirs + (size_t)(j0 + x) * kMmaThreads);
#pragma unroll
                for (int x = 0; x < 16; x += 4) wait_loads(t[x], t[x + 1], t[x + 2], t[x + 3]);
#pragma unroll
                for (int x = 0; x < 16; ++x) {
                    const int j = j0 + x, cf = j >> 4, tf = (j >> 2) & 3, qd = j & 3;
                    acc[cf][tf][4 * qd] += t[x].x;
                    acc[cf][tf][4 * qd + 1] += t[x].y;
                    acc[cf][tf][4 * qd + 2] += t[x].z;
                    acc[cf][tf][4 * qd + 3] += t[x].w;
                }
            }
        }
    }

    const __half* e_sx = reinterpret_cast<const __half*>(ering);
    const __half* e_sn = e_sx + 256;
    const int* e_rs = reinterpret_cast<const int*>(ering + 1024);
    const uint8_t* e_zn = reinterpret_cast<const uint8_t*>(ering + 2048);

    // ---- epilogue.  Lane (token r32, half hb = kb2) of fragment (cf, tf) holds physical rows 8*(v/4) + 4*hb + v%4,
    // i.e. logical channels 64*(cf/2) + 32*(v4%2) + 16*hb + 8*(cf%2) + 4*(v4/2) + v%4 of the wave's 32*CF: for fixed
    // (cf/2, v4%2) the four pieces (cf%2, v4/2) are 16 consecutive channels = one 32-byte row segment per token.
    const int hb = kb2;
    if constexpr (CF & 1) {
        // Interleaved fragments: the wave's fragment cf is half `wn` of the tile's 64-channel block cf, so for fixed
        // (cf, v4 % 2) the two pieces v4 / 2 are 8 consecutive channels = one 16-byte row segment per token.
#pragma unroll
        for (int cf = 0; cf < CF; ++cf) {
#pragma unroll
            for (int vl = 0; vl < 2; ++vl) {
                const int nl = 64 * cf + 32 * vl + 16 * hb + 8 * wn;   // first of the 8 channels, inside the tile
                const int n8 = n_base + nl;
                if (n8 >= p.N) continue;                 // N % 16 == 0: an 8-channel segment is all in or all out
                float sn[8];
                int zn[8];
#pragma unroll
                for (int x = 0; x < 8; ++x) { sn[x] = OUT == OUT_FP16 ? __half2float(e_sn[nl + x]) : 0.f; zn[x] = GROUP ? 0 : (int)e_zn[nl + x]; }
#pragma unroll
                for (int tf = 0; tf < 4; ++tf) {
                    const int ml = wm * 128 + tf * 32 + r32;
                    const int m = m_base + ml;
                    if (m >= p.M) continue;
                    const float sxm = OUT == OUT_FP16 ? __half2float(e_sx[ml]) : 0.f;
                    const int rs = GROUP ? 0 : e_rs[ml];
                    const bool token_sum = !GROUP && OUT == OUT_FP16 && p.token_sum;   // Eq. 7 form, rs = bits of t_X
                    const float txm = __int_as_float(rs);
                    int t[8];
#pragma unroll
                    for (int piece = 0; piece < 2; ++piece) {
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            t[4 * piece + x] = acc[cf][tf][4 * (2 * piece + vl) + x];
                            if (!GROUP && !token_sum) t[4 * piece + x] -= zn[4 * piece + x] * rs;
                        }
                    }
                    if constexpr (OUT == OUT_I32) {
                        int4* dst = reinterpret_cast<int4*>(p.out32 + (size_t)m * p.N + n8);
                        dst[0] = make_int4(t[0], t[1], t[2], t[3]);
                        dst[1] = make_int4(t[4], t[5], t[6], t[7]);
                    } else {
                        uint32_t h[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            float ra = (float)t[2 * j] * (sxm * sn[2 * j]), rb = (float)t[2 * j + 1] * (sxm * sn[2 * j + 1]);
                            if (token_sum) {
                                ra -= txm * ((float)zn[2 * j] * sn[2 * j]);
                                rb -= txm * ((float)zn[2 * j + 1] * sn[2 * j + 1]);
                            }
                            const __half lo = __float2half_rn(ra);
                            const __half hi = __float2half_rn(rb);
                            h[j] = (uint32_t)__half_as_ushort(lo) | ((uint32_t)__half_as_ushort(hi) << 16);
                        }
                        *reinterpret_cast<uint4*>(p.out16 + (size_t)m * p.N + n8) = make_uint4(h[0], h[1], h[2], h[3]);
                    }
                }
            }
        }
        return;
    }
#pragma unroll
    for (int ch = 0; ch < CF / 2; ++ch) {
#pragma unroll
        for (int vl = 0; vl < 2; ++vl) {
            const int nl = wn * 32 * CF + 64 * ch + 32 * vl + 16 * hb;   // first of the 16 channels, inside the tile
            const int n16 = n_base + nl;
            if (n16 >= p.N) continue;                    // N % 64 == 0: a 16-channel segment is all in or all out
            float sn[16];
            int zn[16];
#pragma unroll
            for (int x = 0; x < 16; ++x) { sn[x] = OUT == OUT_FP16 ? __half2float(e_sn[nl + x]) : 0.f; zn[x] = GROUP ? 0 : (int)e_zn[nl + x]; }
#pragma unroll
            for (int tf = 0; tf < 4; ++tf) {
                const int ml = wm * 128 + tf * 32 + r32;
                const int m = m_base + ml;
                if (m >= p.M) continue;
                const float sxm = OUT == OUT_FP16 ? __half2float(e_sx[ml]) : 0.f;
                const int rs = GROUP ? 0 : e_rs[ml];
                const bool token_sum = !GROUP && OUT == OUT_FP16 && p.token_sum;   // Eq. 7 form, rs = bits of t_X
                const float txm = __int_as_float(rs);
                int t[16];
#pragma unroll
                for (int piece = 0; piece < 4; ++piece) {
                    const int cf = 2 * ch + (piece >> 1), v4 = 2 * (piece & 1) + vl;
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        t[4 * piece + x] = acc[cf][tf][4 * v4 + x];
                        if (!GROUP && !token_sum) t[4 * piece + x] -= zn[4 * piece + x] * rs;
                    }
                }
                if constexpr (OUT == OUT_I32) {
                    int4* dst = reinterpret_cast<int4*>(p.out32 + (size_t)m * p.N + n16);
#pragma unroll
                    for (int q = 0; q < 4; ++q) dst[q] = make_int4(t[4 * q], t[4 * q + 1], t[4 * q + 2], t[4 * q + 3]);
                } else {
                    uint32_t h[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        float ra = (float)t[2 * j] * (sxm * sn[2 * j]), rb = (float)t[2 * j + 1] * (sxm * sn[2 * j + 1]);
                        if (token_sum) {
                            ra -= txm * ((float)zn[2 * j] * sn[2 * j]);
                            rb -= txm * ((float)zn[2 * j + 1] * sn[2 * j + 1]);
                        }
                        const __half lo = __float2half_rn(ra);
                        const __half hi = __float2half_rn(rb);
                        h[j] = (uint32_t)__half_as_ushort(lo) | ((uint32_t)__half_as_ushort(hi) << 16);
                    }
                    uint4* dst = reinterpret_cast<uint4*>(p.out16 + (size_t)m * p.N + n16);
                    dst[0] = make_uint4(h[0], h[1], h[2], h[3]);
                    dst[1] = make_uint4(h[4], h[5], h[6], h[7]);
                }
            }
        }
    }
}

template <int MF, bool GROUP>
void launch_stream(const GemmDev& p, bool fp16, dim3 grid, hipStream_t s)
{
    // 64-token tiles: the LDS-staged kernel; smaller tiles: the register-streaming kernel (measured faster there:
    // its activation traffic shrinks with the tile while the staged kernel's per-iteration barriers do not)
    if constexpr (MF == 4) {
        if (fp16) stream_kernel<MF, GROUP, OUT_FP16><<<grid, kStreamThreads, 0, s>>>(p);
        else stream_kernel<MF, GROUP, OUT_I32><<<grid, kStreamThreads, 0, s>>>(p);
    } else {
        if (fp16) rstream_kernel<MF, GROUP, OUT_FP16><<<grid, kRsThreads, 0, s>>>(p);
        else rstream_kernel<MF, GROUP, OUT_I32><<<grid, kRsThreads, 0, s>>>(p);
    }
}

template <bool GROUP, int CF, int WM, int DEPTH = 3>
void launch_mma(const GemmDev& p, bool fp16, hipStream_t s)
{
    constexpr int TMt = 128 * WM, TNt = 32 * CF * (4 / WM);
    const dim3 grid((unsigned)(((p.N + TNt - 1) / TNt) * ((p.M + TMt - 1) / TMt)), (unsigned)p.S);
    if (fp16) mma_kernel<GROUP, OUT_FP16, CF, WM, DEPTH><<<grid, kMmaThreads, 0, s>>>(p);
    else mma_kernel<GROUP, OUT_I32, CF, WM, DEPTH><<<grid, kMmaThreads, 0, s>>>(p);
}

// tile_m selects the kernel and its shape: 16 / 32 / 64 = streaming kernel with that many tokens per tile;
// 128 = compute-bound kernel, 256 tokens x 256 channels; 129 = 128 tokens x 256 channels; 130 = 256 x 128;
// 131 = 256 x 192.
template <bool GROUP>
void launch_any(const GemmDev& p, int tile_m, int nwg, bool fp16, hipStream_t s)
{
    if (tile_m >= 69 && tile_m <= 71) {
        (void)launch_astat(p, tile_m, nwg, GROUP, fp16, s);
    } else if (tile_m == 66) {
        const dim3 grid((unsigned)nwg, (unsigned)((p.M + 63) / 64));
        if (fp16) lockstep_kernel<4, 4, GROUP, OUT_FP16><<<grid, kStreamThreads, 0, s>>>(p);
        else lockstep_kernel<4, 4, GROUP, OUT_I32><<<grid, kStreamThreads, 0, s>>>(p);
    } else if (tile_m == 65) {
        const dim3 grid((unsigned)nwg, (unsigned)((p.M + 63) / 64));
        if (fp16) lockstep_kernel<2, 4, GROUP, OUT_FP16><<<grid, kStreamThreads, 0, s>>>(p);
        else lockstep_kernel<2, 4, GROUP, OUT_I32><<<grid, kStreamThreads, 0, s>>>(p);
    } else if (tile_m == 67) {
        const dim3 grid((unsigned)nwg, (unsigned)((p.M + 31) / 32));
        if (fp16) lockstep_kernel<2, 2, GROUP, OUT_FP16><<<grid, kStreamThreads, 0, s>>>(p);
        else lockstep_kernel<2, 2, GROUP, OUT_I32><<<grid, kStreamThreads, 0, s>>>(p);
    } else if (tile_m == 68) {
        const dim3 grid((unsigned)nwg, (unsigned)((p.M + 15) / 16));
        if (fp16) lockstep_kernel<2, 1, GROUP, OUT_FP16><<<grid, kStreamThreads, 0, s>>>(p);
        else lockstep_kernel<2, 1, GROUP, OUT_I32><<<grid, kStreamThreads, 0, s>>>(p);
    } else if (tile_m <= 64) {
        const dim3 grid((unsigned)nwg, (unsigned)((p.M + tile_m - 1) / tile_m));
        if (tile_m == 16) launch_stream<1, GROUP>(p, fp16, grid, s);
        else if (tile_m == 32) launch_stream<2, GROUP>(p, fp16, grid, s);
        else launch_stream<4, GROUP>(p, fp16, grid, s);
    } else if (tile_m == 129) {
        launch_mma<GROUP, 2, 1>(p, fp16, s);
    } else if (tile_m == 130) {
        launch_mma<GROUP, 2, 2>(p, fp16, s);
    } else if (tile_m == 131) {
        launch_mma<GROUP, 3, 2>(p, fp16, s);
    } else if (tile_m == 132) {
        launch_mma<GROUP, 2, 1, 2>(p, fp16, s);

    } else {
        launch_mma<GROUP, 4, 2>(p, fp16, s);
    }
}

}  // namespace

// ---- launch configuration --------------------------------------------------------------------------
// tile_m: 16 / 32 / 64 = streaming kernel with that many tokens per tile; 128 / 129 / 130 / 131 = compute-bound
// kernel with 256 x 256, 128 x 256, 256 x 128, 256 x 192 (tokens x channels) tiles.  split_k: streaming kernel = number of
// workgroups the unit stream is dealt to (per token tile); compute-bound kernel = k-slices per tile.
static void mma_tile_shape(int tile_m, int64_t& tm, int64_t& tn)
{
    tm = (tile_m == 129 || tile_m == 132) ? 128 : 256;
    tn = tile_m == 130 ? 128 : tile_m == 131 ? 192 : 256;
}
static int64_t mma_tiles(int64_t M, int64_t N, int tile_m)
{
    int64_t tm, tn;
    mma_tile_shape(tile_m, tm, tn);
    return ((M + tm - 1) / tm) * ((N + tn - 1) / tn);
}
// k-slices of the compute-bound kernel: only when its tiles leave most CUs idle and every slice still has a
// long run of groups (a partial tile costs 128-256 KiB of traffic each way plus a device-wide hand-over).
static int mma_split(int64_t M, int64_t N, int64_t G, int tile_m, int forced_split)
{
    const int64_t tiles = mma_tiles(M, N, tile_m);
    int64_t S = 1;
    if (forced_split > 0) S = forced_split;
    else if (tiles < 160) S = std::min<int64_t>(256 / tiles, G / 24);
    if (S > G) S = G;
    if (S < 1) S = 1;
    const int64_t gps = (G + S - 1) / S;
    return (int)((G + gps - 1) / gps);
}
// Cost model fitted to measurements on MI355X (all four shapes on the Llama-2-7B and Llama-3-70B layers at
// M = 512 ... 4096, within 5%), in microseconds: workgroups run in rounds of one per CU; a workgroup needs about
// 8 us of prologue and epilogue plus, per group, a time that grows with the share of the CUs that are busy (the
// clock drops as more matrix cores run): light-load time x (1 + 0.45 load^2); a split adds the hand-over.
static double mma_cost(int64_t M, int64_t N, int64_t G, int tile_m, int& S)
{
    S = mma_split(M, N, G, tile_m, 0);
    const int64_t wgs = mma_tiles(M, N, tile_m) * S;
    if (tile_m == 132) {
        // two workgroups per compute unit (128 x 256 tiles, shallower rings): worth it only when the compute units
        // really get two each; a pair then takes about 1.85 times one workgroup's time per group at full load
        if (S > 1 || wgs < 384) return 1e30;
        // whole rounds of 512 workgroups at full load; what is left over runs two per compute unit if it is more
        // than 256 workgroups, else alone (at the pace of the 128 x 256 tile; measured on Llama-3-70B QKV at 2048
        // tokens, 640 tiles: 154 us, against 165 us for the 256 x 192 tile the coarser estimate preferred)
        const int64_t full = wgs / 512, rem = wgs - full * 512;
        double t = (double)full * (8.0 + 1.14 * 1.45 * (double)G);
        if (rem > 256) {
            const double l = (double)rem / 512.0;
            t += 8.0 + 1.14 * (1.0 + 0.45 * l * l) * (double)G;
        } else if (rem > 0) {
            const double l = (double)rem / 256.0;
            t += 8.0 + 0.62 * (1.0 + 0.45 * l * l) * (double)G;
        }
        return t;
    }
    const int64_t rounds = (wgs + 255) / 256;
    const double load = (double)wgs / (double)(rounds * 256);
    const double light = tile_m == 128 ? 1.18 : tile_m == 131 ? 0.92 : tile_m == 130 ? 0.64 : 0.62;
    const double per_group = light * (1.0 + 0.45 * load * load);
    return (double)rounds * (8.0 + per_group * (double)((G + S - 1) / S)) +
           (S > 1 ? (tile_m == 128 ? 30.0 : tile_m == 131 ? 22.0 : 9.0) : 0.0);
}

// Streaming kernels: partition and cost of running `tile`-token tiles, in microseconds (fitted to measurements of the
// Llama-2-7B layers at 16 ... 128 tokens: about 4.3 us of launch, set-up and first loads, then 1.0 / 1.25 / 0.49 us
// per iteration of eight / eight / two (block, group) units for 16 / 32 / 64-token tiles, 0.8 us (0.3 us) per further
// block of a workgroup, and 3 us (7.8 us for the LDS-staged kernel) for the hand-over when blocks are shared).  All token tiles of a launch
// together get one workgroup per CU: with few blocks (N small) it is faster to cut the tokens into more, smaller
// tiles that run side by side, each re-reading the weights through L2, than to leave most CUs idle.  Per token tile
// the units are dealt either in equal contiguous shares (blocks shared, hand-over) or as whole blocks (k per
// workgroup, no partial tiles), whichever is estimated cheaper.
// One iteration of the pair-streaming kernel (two blocks x two groups), microseconds (measured 0.79 - 0.94).
constexpr double kPairIteration = 0.88;
constexpr double kPairIteration32 = 0.70, kPairIteration16 = 0.60;   // pairs with 32- and 16-token tiles
constexpr double kQuadIteration = 1.40;   // four blocks x two groups (measured 1.4 - 1.7)
struct StreamPlan { int64_t nwg; double cost; };
static StreamPlan stream_plan(int64_t M, int64_t N, int64_t G, int tile, int64_t forced_nwg)
{
    const int64_t blocks = N / 64, units = blocks * G, m_tiles = (M + tile - 1) / tile;
    const int64_t per_it = tile == 64 ? 2 : 8;
    const double t_it = tile == 64 ? 0.49 : tile == 32 ? 1.25 : 1.0, handover = tile == 64 ? 7.8 : 3.0, fixed = 4.3;
    const double weight_mb = (double)N * (double)G * (double)kGroup / 2.0e6;
    const int64_t max_wg = (units + 1) / 2;              // at least one full iteration of the staged kernel each
    // cost of dealing the units of every token tile to n workgroups
    auto cost_of = [&](int64_t n, int64_t& n_eff) {
        const int64_t upw = (units + n - 1) / n;
        n_eff = (units + upw - 1) / upw;
        const int64_t rounds = (m_tiles * n_eff + 255) / 256;
        // every token tile reads all the weights (~4.5 TB/s from memory); tiles that run side by side on the same
        // XCD (workgroup ids a multiple of 8 apart) find in its L2 what the 32 MB of L2 can hold of them
        const double miss = std::min(1.0, weight_mb / 32.0);
        const double reads = (n_eff % 8 == 0 && rounds == 1) ? 1.0 + miss * (double)(m_tiles - 1) : (double)m_tiles;
        // every further block of a workgroup's run ends in an exchange of partial sums and an epilogue
        double loop = (double)rounds * ((double)((upw + per_it - 1) / per_it) * t_it +
                                        (double)((upw + G - 1) / G - 1) * (tile == 64 ? 0.3 : 0.8));
        // a long run of the 16-token kernel streams 25 GB/s per workgroup (0.16 us per 4 KiB unit; measured on
        // K = 28672: 128 workgroups of 224 units 40.6 us, 256 of 112 units 27.7 us)
        if (tile == 16 && upw >= 64) loop = std::max(loop, (double)rounds * (double)upw * 0.16);
        // the hand-over follows the loop; a later round pays it again and waits 1.5 us for its first copies
        return fixed + std::max(loop, weight_mb * reads / 4.5) + (double)rounds * (upw % G ? handover : 0.0) +
               (double)(rounds - 1) * 1.5;
    };
    StreamPlan best{1, 0.0};
    if (forced_nwg > 0) {
        best.cost = cost_of(std::max<int64_t>(1, std::min(forced_nwg, max_wg)), best.nwg);
        return best;
    }
    bool first = true;
    for (const int64_t budget : {(int64_t)256, std::max<int64_t>(1, 256 / m_tiles)}) {
        const int64_t k = (blocks + budget - 1) / budget;
        for (const int64_t n : {std::min(budget, max_wg), (blocks + k - 1) / k}) {   // equal shares; whole blocks
            StreamPlan c;
            c.cost = cost_of(std::max<int64_t>(1, std::min(n, max_wg)), c.nwg);
            if (first || c.cost < best.cost) { best = c; first = false; }
        }
    }
    return best;
}

// Pair-streaming kernel: whole pairs of blocks per workgroup, kp of them; one iteration = two blocks x two groups; all
// 64-token tiles of the launch together fill the chip once.
static StreamPlan pair_plan(int64_t M, int64_t N, int64_t G, int64_t forced_nwg, int nb = 2, int tile = 64)
{
    const int64_t pairs = N / (64 * nb), m_tiles = (M + tile - 1) / tile;   // nb = 4: quads
    const int64_t kp = forced_nwg > 0 ? (pairs + std::min(forced_nwg, pairs) - 1) / std::min(forced_nwg, pairs)
                                      : std::min(pairs, (pairs * m_tiles + 255) / 256);
    const int64_t nwg = (pairs + kp - 1) / kp;
    const int64_t rounds = (m_tiles * nwg + 255) / 256;
    const double weight_mb = (double)N * (double)G * (double)kGroup / 2.0e6;
    const double miss = std::min(1.0, weight_mb / 32.0);
    const double reads = (nwg % 8 == 0 && rounds == 1) ? 1.0 + miss * (double)(m_tiles - 1) : (double)m_tiles;
    const double t_it = nb == 4 ? kQuadIteration : tile == 64 ? kPairIteration : tile == 32 ? kPairIteration32 : kPairIteration16;
    const double loop = (double)rounds * ((double)(kp * ((G + 1) / 2)) * t_it +
                                          (double)(kp - 1) * 0.3) + (double)(rounds - 1) * 1.5;
    return {nwg, 4.3 + std::max(loop, weight_mb * reads / 4.5)};
}

// Activation-stationary kernels (tile_m 69 / 70 / 71 = 16 / 32 / 64 tokens): k-slices so that a slice's groups fit a
// workgroup's registers, and the workgroups per (token tile, k-slice) that share the layer's 16-channel fragments.
static int astat_tile(int tile_m) { return tile_m == 71 ? 64 : tile_m == 70 ? 32 : 16; }
static void astat_slices(int64_t G, int tile_m, int64_t& S, int64_t& gps)
{
    const int64_t cap = astat_max_groups(astat_tile(tile_m));
    S = (G + cap - 1) / cap;
    gps = (G + S - 1) / S;
    S = (G + gps - 1) / gps;
}
static int64_t astat_nwg(int64_t M, int64_t N, int64_t G, int tile_m, int64_t forced_nwg)
{
    const int64_t tile = astat_tile(tile_m), m_tiles = (M + tile - 1) / tile, frags = N / 16;
    int64_t S, gps;
    astat_slices(G, tile_m, S, gps);
    int64_t nwg = forced_nwg > 0 ? forced_nwg : std::max<int64_t>(1, 256 / (m_tiles * S));
    nwg = std::min(nwg, frags);
    if (S > 1) nwg = std::max(nwg, (frags + 127) / 128);   // at most 128 fragments per workgroup when slices meet in the workspace
    return nwg;
}

void pick_gemm_config(int64_t M, int64_t N, int64_t K, int mode, const GemmTuning& forced, int& tile_m, int& split_k)
{
    const int64_t G = K / kGroup;
    const bool pairs_ok = N % 128 == 0;                // the pair-streaming kernel takes whole block pairs
    (void)mode;
    const int natural = M <= 16 ? 16 : M <= 32 ? 32 : 64;   // smallest streaming tile that holds min(M, 64) tokens
    int stream_tile = natural;
    StreamPlan plan = stream_plan(M, N, G, natural, 0);
    for (int t = natural / 2; t >= 16; t /= 2) {             // smaller tiles, more of them
        const StreamPlan c = stream_plan(M, N, G, t, 0);
        if (c.cost < 0.99 * plan.cost) { plan = c; stream_tile = t; }
    }
    tile_m = forced.tile_m ? forced.tile_m : (M <= 64 ? stream_tile : 128);
    // The activation-stationary kernels are the fastest wherever a workgroup's registers hold the activations of
    // all of K, or of half of it (two k-slices meeting in the workspace), and there is at least a fragment per
    // compute unit.  Measured on the Llama-2-7B layers: up to 32 tokens 5 - 30% ahead of the register-streaming and
    // lockstep kernels for K = 4096 and 5 - 13% for K = 11008 (two slices).  At 33 - 64 tokens loading the [64, K]
    // slab into every compute unit costs about 3 us more than at 16 tokens (the compute unit's vector cache takes in
    // about 100 bytes per ns; reading the slab pre-tiled straight into registers was measured no faster), which only
    // the widest layers win back (gate/up: 17.1 us against 18.3 us; QKV: 13.0 against 12.3); layers of 192 - 704
    // fragments are best served as two 32-token tiles, one workgroup per compute unit (Llama-2-7B O 7.6 us against
    // 7.9, Llama-3-8B QKV 8.4 against 9.0, Llama-3-70B QKV 18.1 against 19.3).
    if (!forced.tile_m && M <= 64) {
        const int64_t frags = N / 16;
        int cand = M <= 16 ? 69 : M <= 32 ? 70 : 71;
        bool take = M <= 32 ? frags >= 192 : frags >= 1024;
        if (M > 32 && frags >= 192 && frags <= 704) { cand = 70; take = true; }
        int64_t S, gps;
        astat_slices(G, cand, S, gps);
        const bool fits = M <= 32 ? S <= 2 : (S == 1 && G <= (cand == 71 ? 32 : 64));
        if (take && fits) tile_m = cand;
    }
    if (tile_m >= 69 && tile_m <= 71) {
        split_k = (int)astat_nwg(M, N, G, tile_m, forced.split_k);
        return;
    }
    if (tile_m == 65 && !pairs_ok) tile_m = 64;
    if (tile_m == 67 && !pairs_ok) tile_m = 32;
    if (tile_m == 68 && !pairs_ok) tile_m = 16;
    if (tile_m == 67 || tile_m == 68) {                    // pairs with 32- / 16-token tiles
        split_k = (int)pair_plan(M, N, G, forced.split_k, 2, tile_m == 67 ? 32 : 16).nwg;
        return;
    }
    const bool quads_ok = N % 256 == 0;
    if (tile_m == 66 && !quads_ok) tile_m = pairs_ok ? 65 : 64;
    // block pairs or quads in lockstep, when cheaper than the single-block plan
    int lock = 0;                                            // 0 = none, 65 = pairs, 66 = quads, 67 / 68 = pairs with 32 / 16-token tiles
    double lock_cost = 0.97 * plan.cost;
    if (stream_tile == 64 && pairs_ok && pair_plan(M, N, G, 0).cost < lock_cost) { lock = 65; lock_cost = pair_plan(M, N, G, 0).cost; }
    if (stream_tile == 64 && quads_ok && pair_plan(M, N, G, 0, 4).cost < 0.97 * lock_cost) { lock = 66; lock_cost = pair_plan(M, N, G, 0, 4).cost; }
    if (stream_tile == natural && natural < 64 && pairs_ok) {
        // 32- and 16-token tiles: the register-streaming kernels reach 3.5 / 4.0 TB/s on layers that keep the whole
        // chip busy (measured), which the plan's estimate does not include
        const double weight_mb = (double)N * (double)G * (double)kGroup / 2.0e6;
        const double ref = std::max(plan.cost, 4.3 + weight_mb / (natural == 32 ? 3.5 : 4.0));
        const double c = pair_plan(M, N, G, 0, 2, natural).cost;
        if (c < 0.97 * ref) { lock = natural == 32 ? 67 : 68; lock_cost = c; }
    }
    const bool pair_wins = lock != 0;
    if (!forced.tile_m && M <= 64 && pair_wins) tile_m = lock;
    if (tile_m == 65 || tile_m == 66) {
        split_k = (int)pair_plan(M, N, G, forced.split_k, tile_m == 65 ? 2 : 4).nwg;
        return;
    }
    if (tile_m == 67 || tile_m == 68) {
        split_k = (int)pair_plan(M, N, G, forced.split_k, 2, tile_m == 67 ? 32 : 16).nwg;
        return;
    }
    if (!forced.tile_m && M > 64) {
        // Cheapest of the four tile shapes of the compute-bound kernel or, for a few hundred tokens, the streaming
        // kernels (they re-read the weights once per token tile but spread K over the whole chip).
        int S;
        double best = mma_cost(M, N, G, 128, S);
        for (int cand = 129; cand <= 132; ++cand) {
            const double c = mma_cost(M, N, G, cand, S);
            if (c < 0.98 * best) { best = c; tile_m = cand; }
        }
        const double stream_cost = pair_wins ? lock_cost : plan.cost;
        double chosen = best;
        if (stream_cost < (pair_wins ? 0.95 : 0.9) * best) { tile_m = pair_wins ? lock : stream_tile; chosen = stream_cost; }
        // Or 64-token activation-stationary tiles side by side, all token tiles together on the 256 compute units
        // (K <= 4096: one workgroup holds all of K; measured 6.5 us + 1.15 ... 1.5 us per fragment of a workgroup's
        // run on the Llama-2-7B and Llama-3-8B layers at 96 ... 512 tokens: QKV at M = 128 15.5 us against 18.4 us,
        // gate+up 22.5 against 27.8, Llama-3-8B QKV at M = 384 18.7 against 23.0).
        if (G <= 32 && M <= 512) {
            const int64_t m_tiles = (M + 63) / 64, n = std::max<int64_t>(1, 256 / m_tiles);
            const double c = 6.5 + 1.4 * (double)((N / 16 + n - 1) / n);
            if (c < 0.97 * chosen) {
                tile_m = 71;
                split_k = (int)astat_nwg(M, N, G, tile_m, 0);
                return;
            }
        }
        if (tile_m == 65 || tile_m == 66) {
            split_k = (int)pair_plan(M, N, G, 0, tile_m == 65 ? 2 : 4).nwg;
            return;
        }
    }
    if (tile_m <= 64) {
        const int64_t units = (N / 64) * G;
        const int64_t nwg = (tile_m == stream_tile && forced.split_k <= 0) ? plan.nwg : stream_plan(M, N, G, tile_m, forced.split_k).nwg;
        const int64_t upw = (units + nwg - 1) / nwg;
        split_k = (int)((units + upw - 1) / upw);
        return;
    }
    split_k = mma_split(M, N, G, tile_m, forced.split_k);
}

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int tile_m, int split_k)
{
    if (tile_m >= 69 && tile_m <= 71) {               // k-slices of the activation-stationary kernels meet per fragment
        int64_t S, gps;
        astat_slices(K / kGroup, tile_m, S, gps);
        if (S <= 1) return 0;
        const int64_t tile = astat_tile(tile_m), m_tiles = (M + tile - 1) / tile, frags = N / 16;
        return align256((size_t)(m_tiles * frags) * sizeof(int)) + (size_t)(m_tiles * frags * S) * (size_t)(tile * 64);
    }
    if (tile_m >= 65 && tile_m <= 68) return 0;        // whole block pairs / quads per workgroup: nothing is exchanged
    if (tile_m <= 64) {
        const int64_t m_tiles = (M + tile_m - 1) / tile_m;
        const int64_t units = (N / 64) * (K / kGroup);
        const int64_t upw = (units + split_k - 1) / split_k;
        if (upw * 1 >= units && split_k <= 1) return 0;
        const size_t counters = align256((size_t)(m_tiles * (N / 64)) * sizeof(int));
        return counters + (size_t)m_tiles * (size_t)split_k * 2 * (size_t)(tile_m * 64) * sizeof(int32_t);
    }
    if (split_k <= 1) return 0;
    int64_t tm, tn;
    mma_tile_shape(tile_m, tm, tn);
    const size_t tiles = (size_t)mma_tiles(M, N, tile_m);
    return align256(tiles * sizeof(int)) + tiles * (size_t)split_k * (size_t)(tm * tn) * sizeof(int32_t);
}

size_t gemm_counter_bytes(int64_t M, int64_t N, int64_t K, int tile_m, int split_k)
{
    if (gemm_workspace_bytes(M, N, K, tile_m, split_k) == 0) return 0;
    if (tile_m >= 69 && tile_m <= 71) {
        const int64_t tile = astat_tile(tile_m);
        return align256((size_t)(((M + tile - 1) / tile) * (N / 16)) * sizeof(int));
    }
    if (tile_m <= 64) return align256((size_t)(((M + tile_m - 1) / tile_m) * (N / 64)) * sizeof(int));
    return align256((size_t)mma_tiles(M, N, tile_m) * sizeof(int));
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
    p.rowsum = a.tx ? reinterpret_cast<const int32_t*>(a.tx) : a.rowsum;
    p.token_sum = a.tx ? 1 : 0;
    p.out16 = static_cast<__half*>(a.out_fp16);
    p.out32 = a.out_i32;
    p.M = (int)a.M; p.N = (int)a.N; p.K = (int)a.K; p.G = (int)L.G;
    p.counters = reinterpret_cast<int*>(a.workspace);
    int nwg = 0;
    size_t counters;
    if (a.tile_m >= 69 && a.tile_m <= 71) {
        int64_t S, gps;
        astat_slices(L.G, a.tile_m, S, gps);
        p.upw = 0;
        nwg = a.split_k;
        p.S = (int)S; p.gps = (int)gps;
        counters = gemm_counter_bytes(a.M, a.N, a.K, a.tile_m, a.split_k);
    } else if (a.tile_m >= 65 && a.tile_m <= 68) {
        const int64_t width = a.tile_m == 66 ? 256 : 128;
        if (a.N % width != 0) return hipErrorInvalidValue;
        const int64_t pairs = a.N / width;
        p.upw = (int)((pairs + a.split_k - 1) / a.split_k);   // whole block pairs per workgroup
        nwg = a.split_k;
        p.S = 1; p.gps = (int)L.G;
        counters = 0;
    } else if (a.tile_m <= 64) {
        const int64_t units = (a.N / 64) * L.G;
        p.upw = (int)((units + a.split_k - 1) / a.split_k);
        nwg = a.split_k;
        p.S = 1; p.gps = (int)L.G;
        counters = align256((size_t)(((a.M + a.tile_m - 1) / a.tile_m) * (a.N / 64)) * sizeof(int));
    } else {
        p.upw = 0;
        p.S = a.split_k;
        p.gps = (int)((L.G + a.split_k - 1) / a.split_k);
        counters = align256((size_t)mma_tiles(a.M, a.N, a.tile_m) * sizeof(int));
    }
    p.parts = reinterpret_cast<int4*>(reinterpret_cast<uint8_t*>(a.workspace) + (a.parts_offset ? a.parts_offset : counters));
    if (a.mode == 0) launch_any<true>(p, a.tile_m, nwg, a.out_fp16 != nullptr, s);
    else launch_any<false>(p, a.tile_m, nwg, a.out_fp16 != nullptr, s);
    return hipGetLastError();
}

namespace {
__global__ __launch_bounds__(256) void zero_kernel(int4* dst, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256)
        dst[i] = make_int4(0, 0, 0, 0);
}
}  // namespace


hipError_t launch_zero(void* dst, size_t bytes, hipStream_t s)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t blocks = (n16 + 255) / 256;
    zero_kernel<<<dim3((unsigned)(blocks > 4096 ? 4096 : blocks)), 256, 0, s>>>(static_cast<int4*>(dst), n16);
    return hipGetLastError();
}

}  // namespace qoq
