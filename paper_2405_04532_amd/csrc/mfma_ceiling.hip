// Stand-alone probe of the INT8 matrix-core ceiling on gfx950 (measurement aid for the roofline of the
// compute-bound W4A8 GEMM kernel, not part of the library).
//
// One wave per SIMD on every CU issues v_mfma_i32_32x32x32_i8 back to back into 16 accumulator tiles held in
// accumulation registers, exactly the shape of the GEMM main loop, and the achieved rate is reported against
// the published dense INT8 peak.  The rows differ only in the operand DATA: the matrix cores are power
// limited, so the sustained clock, and with it the attainable rate, depends on how many operand bits toggle
// between consecutive instructions.  The last rows add the per-MFMA vector work of the in-register
// UINT4 -> INT8 dequantization (Section 5.2.2-5.2.3 of arXiv 2405.04532) to show what fits in an MFMA's shadow.
//
// Build: hipcc --offload-arch=gfx950 -O3 mfma_ceiling.hip -o mfma_ceiling      Run: ./mfma_ceiling
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

enum Mode { ZERO, CONSTANT, RANDOM_FIXED, RANDOM_ROTATED, ROTATED_DEQUANT };

template <int MODE>
__global__ __launch_bounds__(256) void probe(int iters, int* out)
{
    v4i a[8], b[8];
    uint32_t h = (threadIdx.x + blockIdx.x * 256u) * 2654435761u + 12345u;
    auto next = [&]() { h ^= h << 13; h ^= h >> 17; h ^= h << 5; return (int)h; };
    for (int i = 0; i < 8; ++i) {
        if (MODE == ZERO) { a[i] = (v4i){0, 0, 0, 0}; b[i] = (v4i){0, 0, 0, 0}; }
        else if (MODE == CONSTANT) { a[i] = (v4i){(int)threadIdx.x, 1, 2, 3}; b[i] = (v4i){4, 5, 6, (int)threadIdx.x}; }
        else { a[i] = (v4i){next(), next(), next(), next()}; b[i] = (v4i){next(), next(), next(), next()}; }
    }
    v16i c[16];
    for (int i = 0; i < 16; ++i) for (int j = 0; j < 16; ++j) c[i][j] = 0;
    uint32_t x[4] = {(uint32_t)next(), (uint32_t)next(), (uint32_t)next(), (uint32_t)next()}, y[4] = {0, 0, 0, 0};
    uint32_t S = 0x00030003u, B = 0x01010101u;
    const uint32_t M = 0x0f0f0f0fu, X = 0x80808080u;
    asm volatile("" : "+v"(S), "+v"(B));
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int ia = (MODE == RANDOM_ROTATED || MODE == ROTATED_DEQUANT) ? (i & 7) : 0;
            const int ib = (MODE == RANDOM_ROTATED || MODE == ROTATED_DEQUANT) ? ((i * 3) & 7) : 0;
            asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+a"(c[i]) : "v"(a[ia]), "v"(b[ib]));
            if (MODE == ROTATED_DEQUANT)   // unpack + multiply-add + sign flip of one operand dword (3.5 instructions per MFMA)
                asm volatile("v_lshrrev_b32 %0, 4, %1\n\tv_and_b32 %0, %2, %0\n\tv_pk_mad_u16 %0, %3, %0, %4\n\ts_nop 0\n\tv_xor_b32 %0, %5, %0"
                             : "=&v"(y[i & 3]) : "v"(x[i & 3]), "v"(M), "v"(S), "v"(B), "v"(X));
        }
    }
    int s = 0;
    for (int i = 0; i < 16; ++i) for (int j = 0; j < 16; ++j) s += c[i][j];
    if (s == 0x7fffffff) out[0] = s + (int)(y[0] + y[1] + y[2] + y[3]);
}

int main()
{
    int* out = nullptr;
    if (hipMalloc(&out, 64) != hipSuccess) { printf("no GPU\n"); return 1; }
    hipEvent_t e0, e1;
    (void)hipEventCreate(&e0);
    (void)hipEventCreate(&e1);
    hipDeviceProp_t prop;
    (void)hipGetDeviceProperties(&prop, 0);
    const int cus = prop.multiProcessorCount;
    const double peak = 5033.0;   // published dense INT8 TOP/s of MI355X
    printf("device %s, %d CUs; one wave per SIMD, 16 accumulator tiles, v_mfma_i32_32x32x32_i8\n", prop.gcnArchName, cus);
    auto run = [&](const char* name, auto launch, int iters) {
        launch(iters / 10);
        (void)hipDeviceSynchronize();
        (void)hipEventRecord(e0);
        launch(iters);
        (void)hipEventRecord(e1);
        (void)hipEventSynchronize(e1);
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        const double mfma = (double)iters * 16;
        const double tops = 2.0 * 32 * 32 * 32 * mfma * cus * 4 / ms / 1e9;
        printf("%-58s %8.3f ms %8.1f TOP/s %6.3f of peak %6.2f ns per MFMA\n", name, ms, tops, tops / peak, ms * 1e6 / mfma);
    };
    const int iters = 40000;   // about 10 ms per row: long enough for the clock to settle
#define ROW(MODE, NAME) run(NAME, [&](int it) { probe<MODE><<<cus, 256>>>(it, out); }, iters)
    ROW(ZERO, "operands all zero");
    ROW(CONSTANT, "small constant operands");
    ROW(RANDOM_FIXED, "random INT8 operands, same registers every MFMA");
    ROW(RANDOM_ROTATED, "random INT8 operands, eight register sets rotated");
    ROW(ROTATED_DEQUANT, "  same + dequantization vector work per MFMA");
    (void)hipFree(out);
    return 0;
}
