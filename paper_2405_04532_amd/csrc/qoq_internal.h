// Internal launch interfaces between the C-ABI layer and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qoq_layout.h"

namespace qoq {

// qoq_pack.hip
hipError_t launch_pack_weights(const void* w_fp16, const BlobLayout& L, uint8_t* blob, hipStream_t s);
hipError_t launch_pack_quantized(const uint8_t* q, const uint8_t* s1, const uint8_t* z, const void* s_fp16,
                                 const BlobLayout& L, uint8_t* blob, hipStream_t s);
hipError_t launch_unpack(const uint8_t* blob, const BlobLayout& L, uint8_t* q, uint8_t* s1, uint8_t* z,
                         void* s_fp16, hipStream_t s);

// qoq_act.hip
hipError_t launch_act_quant(const void* x_fp16, int64_t M, int64_t K, int8_t* qx, void* sx, int32_t* rowsum,
                            float* tx, hipStream_t s);

// producers with the quantization fused in (rows of at most fused_quant_max_k() elements)
int64_t fused_quant_max_k();
hipError_t launch_rmsnorm_quant(const void* x_fp16, const void* gamma_fp16, double eps, int64_t M, int64_t K, void* y_fp16,
                                int8_t* qx, void* sx, int32_t* rowsum, float* tx, hipStream_t s);
hipError_t launch_silu_mul_quant(const void* gate_up_fp16, int64_t M, int64_t K, void* y_fp16, int8_t* qx, void* sx,
                                 int32_t* rowsum, float* tx, hipStream_t s);

// qoq_gemm.hip
struct GemmArgs {
    const int8_t* qx;
    const void* sx;          // FP16 [M] (null for the INT32 entry)
    const int32_t* rowsum;   // INT32 [M], per-channel mode
    const float* tx;         // FP32 [M] sums of the unquantized tokens: per-channel FP16 epilogue in the token-sum form
    const uint8_t* blob;
    int64_t M, N, K;
    int mode;
    void* out_fp16;          // [M, N] FP16, or null
    int32_t* out_i32;        // [M, N] INT32, or null
    void* workspace;         // split-k counters and partial tiles when split_k > 1
    int tile_m;              // 16, 32, 64 (streaming kernels) or 128 ... 131 (compute-bound kernel, four tile shapes)
    int split_k;             // compute-bound kernel: k-slices per tile; streaming kernel: workgroups sharing the unit stream
    size_t parts_offset = 0; // byte offset of the partial tiles inside the workspace; 0 = directly behind the counters
};
// Bytes of arrival counters at the start of the workspace of a (tile_m, split_k) launch (0 if it exchanges nothing).
size_t gemm_counter_bytes(int64_t M, int64_t N, int64_t K, int tile_m, int split_k);
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);

// Workspace a (tile_m, split_k) launch needs: per-tile counters, then the partial tiles.
size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int tile_m, int split_k);
hipError_t launch_zero(void* dst, size_t bytes, hipStream_t s);

// Data-free offline transforms (channel reordering, Hadamard rotation).
hipError_t launch_act_quant_reordered(const void* x_fp16, const int32_t* perm, int64_t M, int64_t K, int8_t* qx, void* sx,
                                      int32_t* rowsum, float* tx, hipStream_t s);
hipError_t launch_channel_absmax(const void* x, int64_t M, int64_t K, float* absmax, hipStream_t s);
hipError_t launch_gather_channels(const void* src, const int32_t* perm, int64_t rows, int64_t K, void* dst, hipStream_t s);
hipError_t launch_hadamard(const void* src, int64_t rows, int64_t K, int64_t block, void* dst, hipStream_t s);
int hadamard_max_block();
void channel_order_host(const float* salience, int64_t K, int32_t* perm);

// KV4 cache (head dimension 128) and decode attention.
size_t kv4_cache_bytes(int64_t B, int64_t Hkv, int64_t S_max);
hipError_t launch_kv4_append(const void* k, const void* v, const int32_t* positions, int64_t B, int64_t T, int64_t Hkv,
                             int64_t S_max, uint8_t* cache, hipStream_t s);
hipError_t launch_kv4_unpack(const uint8_t* cache, int64_t B, int64_t Hkv, int64_t S_max, uint8_t* k_codes, void* k_s, void* k_z,
                             uint8_t* v_codes, void* v_s, void* v_z, hipStream_t s);
hipError_t launch_kv4_decode(const void* q, const uint8_t* cache, const int32_t* seq_lens, int64_t B, int64_t H, int64_t Hkv,
                             int64_t S_max, void* out, void* workspace, size_t workspace_bytes, hipStream_t s);
size_t kv4_decode_workspace_bytes(int64_t B, int64_t H, int64_t Hkv, int64_t S_max);

// Launch configuration the library picks for a problem (also sizes the workspace).
struct GemmTuning { int tile_m, split_k; };  // 0 = let the heuristic decide
void pick_gemm_config(int64_t M, int64_t N, int64_t K, int mode, const GemmTuning& forced, int& tile_m, int& split_k);

}  // namespace qoq
