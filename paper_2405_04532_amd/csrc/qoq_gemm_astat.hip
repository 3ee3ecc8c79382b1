// Activation-stationary W4A8 GEMM kernels for token tiles of 16, 32 and 64 (decode sizes), gfx950.
//
// The LDS-staged streaming kernels fetch, for every 64-channel block of weights, the whole [tokens, K] slab of INT8
// activations again.  At 64 tokens that is twice the bytes of the weights themselves, all of it through the
// compute unit's vector cache, which returns data in request order and keeps a bounded number of bytes in flight:
// activation lines that hit in L2 queue behind weight lines that come from memory, and the weights get a third of
// what the cache can keep in flight.  Here the activations are loaded ONCE per workgroup and stay in registers for
// the whole kernel, in the layout of the matrix instruction's token operand, so that the main loop requests nothing
// but packed weights (Section 5.2.4 of arXiv 2405.04532 states the goal: at small m the GEMM is bound by weight
// traffic -- the loop should then move weights only).
//
//   * Workgroup = eight waves, two per SIMD, 256 registers per lane each.  Wave w keeps the activations of the
//     quantization groups g_lo + w * J' + j (j = 0 .. J'-1, J' <= J) of the workgroup's k-slice: J * MF * 2 operands
//     of 16 bytes per lane (MF = tokens / 16), at most 128 registers -- together the 256 KiB a [64, 4096] INT8 slab
//     takes; J <= 4 at 64 tokens, <= 8 at 32 and 16 tokens (sixteen groups per wave at 16 tokens, i.e. all of
//     K = 11008 in one workgroup, lost to two k-slices of eight: every compute unit then loads half the slab).
//     (Four waves with twice the registers each were tried first: the compiler then parks part of the activations
//     in accumulation registers and copies them back in front of every matrix instruction.)  Slots past the end
//     of the slice hold zeros, so the loop needs no bounds logic: whatever weights are loaded for such a slot are
//     multiplied by zero.
//   * Work item = one 16-channel fragment of the packed layout (1 KiB per quantization group, contiguous over the
//     groups).  The layer's fragments are dealt in contiguous, equal runs to the workgroups, so a workgroup reads
//     one contiguous stretch of the packed weights, each wave its own J' consecutive KiB of every fragment, each lane exactly the 16 bytes its
//     matrix-instruction operand consists of (Section 5.2.1: stored in consumption order) -- straight into
//     registers, a ring of D units ahead, no LDS staging, no barrier inside a fragment.
//   * Per unit: the register dequantizer of Sections 5.2.2-5.2.3 (3-operation unpack, packed multiply-add, sign
//     flip) and 2 * MF v_mfma_i32_16x16x64_i8.
//   * End of a fragment: the eight waves' sums over their groups meet in LDS (double buffered: one barrier per
//     fragment); thread t then owns four consecutive channels of one token and runs the epilogue (Eq. 5-7).
//   * More tokens than a tile: token tiles on blockIdx.y, run side by side; the tiles of one fragment run share its
//     weights through L2 (the host keeps token tiles x fragment runs x k-slices at one workgroup per compute unit).
//   * K longer than 8 * J groups: k-slices on blockIdx.z.  Every slice writes its fragment sums through to the
//     workspace; after the loop it bumps the fragments' arrival counters, and whoever arrives last at a fragment
//     adds the slices (integer sums: exact and order independent) and runs the epilogue.  Same fence-free
//     hand-over as in the other kernels: write-through stores, a wait, a relaxed device-scope counter,
//     cache-bypassing loads.
#include <hip/hip_runtime.h>

#include "qoq_gemm_common.h"
#include "qoq_layout.h"

namespace qoq {
namespace {

constexpr int kAsThreads = 512;
constexpr int kAsWaves = 8;
constexpr int kAsMaxFrags = 128;     // fragments per workgroup when k-slices meet in the workspace (host-checked)

template <int MF, int J, int R, bool GROUP, int OUT>
__global__ __launch_bounds__(kAsThreads) void astat_kernel(GemmDev p)
{
    // R = fragments whose units are in flight ahead of the one being multiplied: a ring of R * J units per wave
    static_assert(J * MF <= 16, "128 registers of activations per lane");
    constexpr int D = R * J;
    constexpr int kEl = MF * 64;                       // int4 elements of a fragment tile: mf * 64 + lane
    // LDS: first every wave's private staging area of the activation preload, afterwards, in the same bytes, the
    // double-buffered exchange of the waves' fragment sums.
    constexpr int kWaveStage = 16 * 1024;
    __shared__ __attribute__((aligned(16))) char lds_raw[kAsWaves * kWaveStage];
    static_assert(2 * kAsWaves * kEl * 16 <= kAsWaves * kWaveStage, "the exchange buffers fit in the staging areas");
    int4 (*red)[kAsWaves][kEl] = reinterpret_cast<int4 (*)[kAsWaves][kEl]>(lds_raw);
    __shared__ int s_last[kAsMaxFrags];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q = lane >> 4, ml = lane & 15;
    const int mt_idx = blockIdx.y;
    const int m0 = mt_idx * (16 * MF);
    const int G = p.G, nf_total = p.N / 16;
    // fragments of this workgroup: contiguous runs whose lengths differ by at most one
    const int nwg = gridDim.x, base = nf_total / nwg, rem = nf_total - base * nwg;
    const int wg = blockIdx.x;
    const int f0 = wg * base + min(wg, rem), f1 = f0 + base + (wg < rem ? 1 : 0);
    if (f0 >= f1) return;                              // whole workgroup: nothing to do
    const int slice = blockIdx.z;
    const int g_lo = slice * p.gps, g_hi = min(G, g_lo + p.gps);   // this workgroup's groups
    // Wave w owns the groups g_lo + w * jeff + j, j < jeff: a contiguous stretch, so that at any moment the eight
    // waves of a workgroup (and, the workgroups running in step, all of them) read eight different 128-byte
    // columns of the activation rows spread over the whole row -- with interleaved ownership every wave would be in
    // the same kilobyte of the row at the same time, which a few L2 channels then have to serve to the whole chip.
    const int jeff = (p.gps + kAsWaves - 1) / kAsWaves;             // <= J (host-checked)
    auto slot_valid = [&](int j) __attribute__((always_inline)) { return j < jeff && g_lo + wave * jeff + j < g_hi; };
    auto group_of = [&](int j) __attribute__((always_inline)) { return min(g_lo + wave * jeff + min(j, jeff - 1), g_hi - 1); };

    // ---- weights: ring of D units per wave, filled ahead ----------------------------------------
    uint4 w[D];
    uint32_t mt[D];
    auto load_unit = [&](int slot, int j, int nf) __attribute__((always_inline)) {
        const int g = group_of(j);
        w[slot] = p.codes[((size_t)nf * G + g) * 64 + lane];
        mt[slot] = GROUP ? (uint32_t)p.meta[((size_t)g * nf_total + nf) * 16 + ml] : 0u;
    };
    const int nfr = f1 - f0;

    // ---- activations: loaded once, resident for the whole kernel ---------------------------------
    // lane (ml, q) holds, of every (group, m-fragment, k-step) operand, token row ml and the 16-byte k-chunk q.
    // Loading those words directly costs the vector cache one request per 64-byte half line (16 rows x 64 B per
    // instruction) and was measured three times slower than reading whole lines, so they go through LDS: every
    // wave copies the columns of ITS OWN groups (JP * 128 contiguous bytes of each token row, whole 128-byte lines,
    // 1 KiB per instruction) into a private 16 KiB staging area by global->LDS DMA and reads its operands back --
    // one or two passes, no barrier: the waves do not wait for one another.  Inside a row the 16-byte chunks are
    // stored XORed with the row number (64-bank LDS: the 16 lanes served together read the same chunk of 16
    // consecutive rows), which keeps the operand reads free of bank conflicts.
    v4i a[J][MF][2];
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) a[j][mf][0] = a[j][mf][1] = (v4i){0, 0, 0, 0};   // slots past the slice stay zero
    {
        constexpr int JP = J >= 8 ? 8 : 4;                                   // groups per pass
        constexpr int RP = (128 / JP) < MF * 16 ? (128 / JP) : MF * 16;      // token rows per pass
        constexpr int kRowPasses = MF * 16 / RP, kJPasses = (J + JP - 1) / JP, kDma = RP * JP / 8;
        static_assert(kDma * 1024 <= kWaveStage && RP % 16 == 0, "a pass fits the wave's staging area");
        const char* abase = reinterpret_cast<const char*>(p.qx);
        const uint32_t region = (uint32_t)(uintptr_t)&lds_raw[0] + (uint32_t)wave * kWaveStage;
        const char* region_ptr = lds_raw + wave * kWaveStage;
        auto issue_pass = [&](int rp, int jp) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < kDma; ++i) {
                const int flat = i * 64 + lane;                              // 16-byte position inside the pass
                const int row_local = flat / (JP * 8), pos = flat % (JP * 8);
                const uint32_t row = (uint32_t)min(m0 + rp * RP + row_local, p.M - 1);   // rows past M repeat the last one
                const uint32_t col = min((uint32_t)(g_lo + wave * jeff + jp * JP) * (uint32_t)kGroup +
                                             (uint32_t)((pos ^ (row_local & 15)) * 16),
                                         (uint32_t)p.K - 16u);                // groups past K re-read the end of the row
                dma16(abase, row * (uint32_t)p.K + col, region + (uint32_t)(i * 1024));
            }
        };
        auto read_pass = [&](int rp, int jp) __attribute__((always_inline)) {
#pragma unroll
            for (int mm = 0; mm < RP / 16; ++mm)
#pragma unroll
                for (int jj = 0; jj < JP; ++jj) {
                    const int mf = rp * (RP / 16) + mm, j = jp * JP + jj;
                    if (j < J) {
                        if (slot_valid(j)) {                                 // wave-uniform
                            const int row_local = mm * 16 + ml;
#pragma unroll
                            for (int ks = 0; ks < 2; ++ks)
                                a[j][mf][ks] = *reinterpret_cast<const v4i*>(region_ptr + row_local * (JP * 128) +
                                                                             (((jj * 8 + ks * 4 + q) ^ (row_local & 15)) * 16));
                        }
                    }
                }
        };
        // Order of the requests: the first pass of activations, then the first R fragments of weights (a trip to
        // memory: data returns in request order, so they must not stand in front of the first pass; behind it
        // their latency passes while the pass is unpacked), then the other passes.  The waits count what this wave
        // requested after the pass it waits for: kNW weight loads (build.py checks that the compiler emits
        // exactly that many).
        constexpr int kNW = R * J * (GROUP ? 2 : 1);
        static_assert(kNW < 64, "vmcnt range");
        issue_pass(0, 0);
        asm volatile("; astat weight prologue begin" ::: "memory");
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int j = 0; j < J; ++j) load_unit(r * J + j, j, f0 + min(r, nfr - 1));
        asm volatile("; astat weight prologue end" ::: "memory");
        wait_vmcnt<kNW>();
        read_pass(0, 0);
#pragma unroll
        for (int pp = 1; pp < kRowPasses * kJPasses; ++pp) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");               // the reads of the pass before are done
            issue_pass(pp / kJPasses, pp % kJPasses);
            wait_vmcnt<0>();
            read_pass(pp / kJPasses, pp % kJPasses);
        }
    }
    __syncthreads();    // the staging areas become the exchange buffers of the fragment sums

    // ---- epilogue role: thread t owns element t of every fragment tile (one token, four consecutive channels) ----
    const int el = threadIdx.x;
    const int e_ln = el & 63;
    const int e_m = m0 + (el >> 6) * 16 + (e_ln & 15);
    const bool e_on = el < kEl;
    float c_sx = 0.f;
    int c_rs = 0;
    if (e_on) {
        const int mc = min(e_m, p.M - 1);
        c_sx = OUT == OUT_FP16 ? __half2float(p.sx[mc]) : 0.f;
        c_rs = GROUP ? 0 : p.rowsum[mc];
    }
    auto channel_of = [&](int nf) __attribute__((always_inline)) { return (nf >> 2) * 64 + 16 * (e_ln >> 4) + 4 * (nf & 3); };
    auto epilogue = [&](int nf, v4i sum, uint2 sw, uint32_t zw) __attribute__((always_inline)) {
        const float sn[4] = {__half2float(__ushort_as_half((unsigned short)(sw.x & 0xFFFFu))),
                             __half2float(__ushort_as_half((unsigned short)(sw.x >> 16))),
                             __half2float(__ushort_as_half((unsigned short)(sw.y & 0xFFFFu))),
                             __half2float(__ushort_as_half((unsigned short)(sw.y >> 16)))};
        const int zn[4] = {(int)(zw & 0xFFu), (int)((zw >> 8) & 0xFFu), (int)((zw >> 16) & 0xFFu), (int)(zw >> 24)};
        finish4<GROUP, OUT>(p, e_m, channel_of(nf), sum, sn, zn, c_sx, c_rs);
    };
    const size_t part_stride = (size_t)p.S * kEl;      // int4 elements per fragment in the workspace
    int4* parts_mt = p.parts + (size_t)mt_idx * nf_total * part_stride;

    // ---- main loop over the fragments, R per trip so that every ring slot is a compile-time constant -----------
    int buf = 0;
    for (int fi0 = 0; fi0 < nfr; fi0 += R) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int fi = fi0 + r;
            if (fi >= nfr) break;                          // workgroup-uniform
            const int nf = f0 + fi;
            const int nf_ahead = f0 + min(fi + R, nfr - 1);   // past the last fragment: reload it (valid memory, never used)
            uint2 c_s = make_uint2(0, 0);
            uint32_t c_z = 0;
            if (e_on && p.S == 1) {                        // epilogue constants: in flight during the fragment
                if (OUT == OUT_FP16) c_s = *reinterpret_cast<const uint2*>(p.scales + channel_of(nf));
                if (!GROUP) c_z = *reinterpret_cast<const uint32_t*>(p.zeros + channel_of(nf));
            }
            v4i acc[MF];
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) acc[mf] = (v4i){0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const int slot = r * J + j;
                const uint4 wq = w[slot];
                uint32_t S = 0, B = 0;
                if (GROUP) {
                    S = __builtin_amdgcn_perm(mt[slot], mt[slot], 0x0c000c00u);   // s1 in both 16-bit lanes
                    B = __builtin_amdgcn_perm(mt[slot], mt[slot], 0x01010101u);   // bias in all four bytes
                }
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const v4i w_op = dequant<GROUP>(ks ? wq.z : wq.x, ks ? wq.w : wq.y, S, B);
#pragma unroll
                    for (int mf = 0; mf < MF; ++mf)
                        acc[mf] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w_op, a[j][mf][ks], acc[mf], 0, 0, 0);
                }
                // the slot's words are consumed: refill it with the same unit of the fragment R places ahead
                load_unit(slot, j, nf_ahead);
                // keep the units in program order: otherwise the compiler gathers the first touch of every slot at
                // the top of the fragment and with it the waits for loads issued only a few hundred cycles earlier
                __builtin_amdgcn_sched_barrier(0);
            }
            // the waves' sums meet in LDS; the buffers alternate, so one barrier per fragment is enough (a wave
            // writes buffer b again only after the barrier of the fragment in between, which every wave reaches
            // after its reads of b)
#pragma unroll
            for (int mf = 0; mf < MF; ++mf)
                red[buf][wave][mf * 64 + lane] = make_int4(acc[mf].x, acc[mf].y, acc[mf].z, acc[mf].w);
            __syncthreads();
            if (e_on) {
                v4i sum = (v4i){0, 0, 0, 0};
#pragma unroll
                for (int ww = 0; ww < kAsWaves; ++ww) {
                    const int4 o = red[buf][ww][el];
                    sum += (v4i){o.x, o.y, o.z, o.w};
                }
                if (p.S == 1) {
                    if (e_m < p.M) epilogue(nf, sum, c_s, c_z);
                } else {
                    store_through(parts_mt + (size_t)nf * part_stride + (size_t)slice * kEl + el, sum.x, sum.y, sum.z, sum.w);
                }
            }
            buf ^= 1;
        }
    }
    if (p.S == 1) return;

    // ---- k-slices meet: wait for the partial sums to reach memory, bump every fragment's counter, finish the
    // fragments at which this workgroup arrived last ----------------------------------------------------------
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int i = threadIdx.x; i < nfr; i += kAsThreads) {
        int* ctr = p.counters + mt_idx * nf_total + f0 + i;
        const int old = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = old == p.S - 1;
        if (last) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last[i] = last;
    }
    __syncthreads();
    if (!e_on) return;
    for (int i = 0; i < nfr; ++i) {
        if (!s_last[i]) continue;                      // workgroup-uniform
        const int nf = f0 + i;
        uint2 c_s = make_uint2(0, 0);
        uint32_t c_z = 0;
        if (OUT == OUT_FP16) c_s = *reinterpret_cast<const uint2*>(p.scales + channel_of(nf));
        if (!GROUP) c_z = *reinterpret_cast<const uint32_t*>(p.zeros + channel_of(nf));
        const int4* src = parts_mt + (size_t)nf * part_stride + el;
        v4i sum = (v4i){0, 0, 0, 0};
        int s = 0;
        for (; s + 4 <= p.S; s += 4) {                 // four loads in flight: the sum is pure load latency
            const v4i t0 = load_through(src + (size_t)s * kEl), t1 = load_through(src + (size_t)(s + 1) * kEl);
            const v4i t2 = load_through(src + (size_t)(s + 2) * kEl), t3 = load_through(src + (size_t)(s + 3) * kEl);
            sum += t0 + t1 + t2 + t3;
        }
        for (; s < p.S; ++s) sum += load_through(src + (size_t)s * kEl);
        if (e_m < p.M) epilogue(nf, sum, c_s, c_z);
    }
}

template <int MF, int J, int R, bool GROUP>
void launch_j(const GemmDev& p, dim3 grid, bool fp16, hipStream_t s)
{
    if (fp16) astat_kernel<MF, J, R, GROUP, OUT_FP16><<<grid, kAsThreads, 0, s>>>(p);
    else astat_kernel<MF, J, R, GROUP, OUT_I32><<<grid, kAsThreads, 0, s>>>(p);
}

template <bool GROUP>
hipError_t launch_mode(const GemmDev& p, int tile, dim3 grid, bool fp16, hipStream_t s)
{
    const int need = (p.gps + kAsWaves - 1) / kAsWaves;   // groups per wave
    if (tile == 64) {
        if (need <= 2) launch_j<4, 2, 2, GROUP>(p, grid, fp16, s);
        else if (need <= 3) launch_j<4, 3, 2, GROUP>(p, grid, fp16, s);
        else if (need <= 4) launch_j<4, 4, 2, GROUP>(p, grid, fp16, s);
        else return hipErrorInvalidValue;
    } else if (tile == 32) {
        if (need <= 4) launch_j<2, 4, 2, GROUP>(p, grid, fp16, s);
        else if (need <= 8) launch_j<2, 8, 1, GROUP>(p, grid, fp16, s);
        else return hipErrorInvalidValue;
    } else {
        if (need <= 4) launch_j<1, 4, 2, GROUP>(p, grid, fp16, s);
        else if (need <= 8) launch_j<1, 8, 1, GROUP>(p, grid, fp16, s);
        else return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

int astat_max_groups(int tile) { return kAsWaves * (tile == 64 ? 4 : 8); }

hipError_t launch_astat(const GemmDev& p, int tile_m, int nwg, bool group, bool fp16, hipStream_t s)
{
    const int tile = tile_m == 71 ? 64 : tile_m == 70 ? 32 : 16;
    const int nf_total = p.N / 16;
    if (nwg < 1 || p.S < 1 || p.gps < 1 || p.gps > astat_max_groups(tile)) return hipErrorInvalidValue;
    if (p.S > 1 && (nf_total + nwg - 1) / nwg > kAsMaxFrags) return hipErrorInvalidValue;
    const dim3 grid((unsigned)nwg, (unsigned)((p.M + tile - 1) / tile), (unsigned)p.S);
    return group ? launch_mode<true>(p, tile, grid, fp16, s) : launch_mode<false>(p, tile, grid, fp16, s);
}

}  // namespace qoq
