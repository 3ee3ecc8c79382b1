// Measurement probe, not part of the W4A8 boundary: what the INT8 matrix cores sustain on this machine.
//
// One wave per SIMD on every compute unit issues v_mfma_i32_32x32x32_i8 back to back into 16 accumulator tiles, the
// shape of the compute-bound GEMM's main loop, with no memory or LDS traffic at all.  The modes differ in the operand
// data and in the vector work issued beside the matrix instructions: the matrix cores are power limited, so the clock
// they sustain, and with it the attainable rate, depends on how many operand bits toggle between consecutive
// instructions and on what else the compute unit is doing.  The benchmark reports these rates next to the GEMM's so
// that its fraction of the published peak can be read against what the hardware sustains with this kind of work.
//   mode 0  small constant operands (nothing toggles)
//   mode 1  random INT8 operands, eight register sets rotated between instructions
//   mode 2  mode 1 plus, per matrix instruction, the vector work of the in-register UINT4 -> INT8 dequantizer
//           (unpack, packed multiply-add, sign flip: Sections 5.2.2-5.2.3 of arXiv 2405.04532)
//   mode 3  mode 2 with operand statistics of the GEMM: one operand random bytes (dequantized weights), the other small
//           integers (quantized activations: most codes within +-8)
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

template <int MODE>
__global__ __launch_bounds__(256) void mfma_kernel(int iters, int* sink)
{
    v4i a[8], b[8];
    uint32_t h = (threadIdx.x + blockIdx.x * 256u) * 2654435761u + 12345u;
    auto next = [&]() { h ^= h << 13; h ^= h >> 17; h ^= h << 5; return h; };
    auto small4 = [&]() {      // four signed bytes, each the difference of two 3-bit numbers: within +-7, mostly near 0
        uint32_t r = next(), w = 0;
        for (int k = 0; k < 4; ++k) {
            const int v = (int)((r >> (8 * k)) & 7) - (int)((r >> (8 * k + 3)) & 7);
            w |= ((uint32_t)v & 0xFFu) << (8 * k);
        }
        return (int)w;
    };
    for (int i = 0; i < 8; ++i) {
        if (MODE == 0) {
            a[i] = (v4i){(int)threadIdx.x, 1, 2, 3};
            b[i] = (v4i){4, 5, 6, (int)threadIdx.x};
        } else {
            a[i] = (v4i){(int)next(), (int)next(), (int)next(), (int)next()};
            b[i] = MODE == 3 ? (v4i){small4(), small4(), small4(), small4()} : (v4i){(int)next(), (int)next(), (int)next(), (int)next()};
        }
    }
    v16i c[16];
    for (int i = 0; i < 16; ++i)
        for (int j = 0; j < 16; ++j) c[i][j] = 0;
    uint32_t x[4] = {next(), next(), next(), next()}, y[4] = {0, 0, 0, 0};
    uint32_t S = 0x00030003u, B = 0x01010101u;
    const uint32_t M = 0x0f0f0f0fu, X = 0x80808080u;
    asm volatile("" : "+v"(S), "+v"(B));
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int ia = MODE == 0 ? 0 : (i & 7), ib = MODE == 0 ? 0 : ((i * 3) & 7);
            asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+a"(c[i]) : "v"(a[ia]), "v"(b[ib]));
            if (MODE >= 2)   // unpack + multiply-add + sign flip of one operand dword
                asm volatile("v_lshrrev_b32 %0, 4, %1\n\tv_and_b32 %0, %2, %0\n\tv_pk_mad_u16 %0, %3, %0, %4\n\ts_nop 0\n\tv_xor_b32 %0, %5, %0"
                             : "=&v"(y[i & 3]) : "v"(x[i & 3]), "v"(M), "v"(S), "v"(B), "v"(X));
        }
    }
    int s = 0;
    for (int i = 0; i < 16; ++i)
        for (int j = 0; j < 16; ++j) s += c[i][j];
    if (s == 0x7fffffff) sink[0] = s + (int)(y[0] + y[1] + y[2] + y[3]);   // data dependent: keeps the work alive
}

}  // namespace

// Runs `iters` rounds of 16 matrix instructions per wave on `workgroups` workgroups of four waves (one workgroup per
// compute unit is the intended use): 2 * 32^3 * 16 * iters * 4 * workgroups integer operations.  sink: device, >= 4 bytes.
// Returns 0, 1 on a bad argument, 2 if the launch failed.
extern "C" int qoq_probe_mfma(int mode, int iters, int workgroups, void* sink, void* stream)
{
    if (mode < 0 || mode > 3 || iters < 1 || workgroups < 1 || workgroups > 65536 || !sink) return 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int* out = static_cast<int*>(sink);
    switch (mode) {
        case 0: hipLaunchKernelGGL(mfma_kernel<0>, dim3((unsigned)workgroups), dim3(256), 0, s, iters, out); break;
        case 1: hipLaunchKernelGGL(mfma_kernel<1>, dim3((unsigned)workgroups), dim3(256), 0, s, iters, out); break;
        case 2: hipLaunchKernelGGL(mfma_kernel<2>, dim3((unsigned)workgroups), dim3(256), 0, s, iters, out); break;
        default: hipLaunchKernelGGL(mfma_kernel<3>, dim3((unsigned)workgroups), dim3(256), 0, s, iters, out); break;
    }
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
