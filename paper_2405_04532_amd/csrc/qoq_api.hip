// C-ABI layer: argument validation, error codes and dispatch.  No kernel code here.
#include <hip/hip_runtime.h>
#include <string.h>

#include <atomic>
#include <cmath>

#include "../../include/qoq_w4a8.h"
#include "qoq_internal.h"

namespace {

std::atomic<int> g_forced_tile_m{0};
std::atomic<int> g_forced_split_k{0};

qoq::GemmTuning forced() { return {g_forced_tile_m.load(), g_forced_split_k.load()}; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

// 1 = gfx950, 0 = something else, cached per device (the query is slow).
int arch_ok()
{
    static std::atomic<int> cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int c = cache[dev].load();
    if (c == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
        c = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 2;
        cache[dev].store(c);
    }
    return c == 1;
}

// ---- scratch of the entry point that allocates nothing ---------------------------------------------------
// One array per GPU (every device that loads the library holds its own copy at its own address until the
// process ends): a fixed region of arrival counters, then the partial tiles.  The counter region is the same for
// every shape, so partial tiles of one call never land where a later call expects counters; the kernels leave
// every counter they used at zero, and the array starts out zero-filled, so nothing is cleared per call.
constexpr size_t kScratchCounterBytes = (size_t)256 << 10;
constexpr size_t kScratchPartBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchCounterBytes + kScratchPartBytes];

// The array's name is a host-side stand-in, not a device address: its address on the CURRENT device is looked up
// once per device and kept; host code uses only that pointer.
int scratch_of_current_device(void** out)
{
    static std::atomic<void*> ptrs[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return QOQ_ERR_HIP;
    void* ptr = ptrs[dev].load();
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return QOQ_ERR_HIP;
        ptrs[dev].store(ptr);
    }
    *out = ptr;
    return QOQ_OK;
}

int check_shape(int64_t N, int64_t K, int mode) { return qoq::shape_ok(N, K, mode) ? QOQ_OK : QOQ_ERR_SHAPE; }

// x_fp16 != NULL: quantize the activations first (into qx, sx, rowsum) by a launch of the activation kernel.
int gemm_common(const int8_t* qx, const void* sx, const int32_t* rowsum, const void* packed, int64_t M, int64_t N,
                int64_t K, int mode, void* out16, int32_t* out32, void* ws, size_t ws_bytes, void* stream,
                const void* x_fp16 = nullptr, const float* tx = nullptr, bool static_scratch = false)
{
    if (check_shape(N, K, mode) != QOQ_OK || M < 0 || M > (1 << 24)) return QOQ_ERR_SHAPE;
    if (M * N >= ((int64_t)1 << 40)) return QOQ_ERR_SHAPE;
    if (M == 0) return QOQ_OK;  // empty batch: nothing to do
    if (!qx || !packed || (!out16 && !out32) || (out16 && !sx)) return QOQ_ERR_NULL;
    if (mode == QOQ_PER_CHANNEL && !rowsum && !tx) return QOQ_ERR_NULL;
    // the per-token vectors are fetched in 4-byte words (global->LDS copies in the compute-bound kernel)
    if (!aligned4(tx) || !aligned4(sx) || !aligned4(rowsum)) return QOQ_ERR_ALIGN;
    if (!aligned16(qx) || !aligned16(packed) || !aligned16(out16) || !aligned16(out32) || !aligned16(ws))
        return QOQ_ERR_ALIGN;
    int tile_m, split_k;
    qoq::pick_gemm_config(M, N, K, mode, forced(), tile_m, split_k);
    if ((uint64_t)M * (uint64_t)K >= ((uint64_t)1 << 32)) return QOQ_ERR_SHAPE;  // 32-bit activation offsets
    if (tile_m <= 71 && (uint64_t)N * (uint64_t)K >= ((uint64_t)1 << 33)) return QOQ_ERR_SHAPE;  // 32-bit weight offsets (4 GiB packed)
    const size_t need = qoq::gemm_workspace_bytes(M, N, K, tile_m, split_k);
    size_t parts_offset = 0;
    if (static_scratch) {
        // the library's own per-device array instead of a caller's workspace: fixed counter region, then partial tiles
        const size_t counters = qoq::gemm_counter_bytes(M, N, K, tile_m, split_k);
        if (counters > kScratchCounterBytes || need - counters > kScratchPartBytes) return QOQ_ERR_WORKSPACE;
        if (!arch_ok()) return QOQ_ERR_ARCH;
        if (need) {
            const int rc = scratch_of_current_device(&ws);
            if (rc != QOQ_OK) return rc;
            parts_offset = kScratchCounterBytes;
        }
    } else if (need && (!ws || ws_bytes < need)) {
        return QOQ_ERR_WORKSPACE;
    }
    if (x_fp16 && !aligned16(x_fp16)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    if (x_fp16 &&
        qoq::launch_act_quant(x_fp16, M, K, const_cast<int8_t*>(qx), const_cast<void*>(sx), const_cast<int32_t*>(rowsum),
                              nullptr, static_cast<hipStream_t>(stream)) != hipSuccess)
        return QOQ_ERR_HIP;
    qoq::GemmArgs a;
    a.qx = qx; a.sx = sx; a.rowsum = rowsum; a.tx = tx; a.blob = static_cast<const uint8_t*>(packed);
    a.M = M; a.N = N; a.K = K; a.mode = mode;
    a.out_fp16 = out16; a.out_i32 = out32; a.workspace = ws;
    a.tile_m = tile_m; a.split_k = split_k; a.parts_offset = parts_offset;
    return qoq::launch_gemm(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

}  // namespace

extern "C" {

const char* qoq_status_string(int status)
{
    switch (status) {
        case QOQ_OK: return "QOQ_OK";
        case QOQ_ERR_NULL: return "QOQ_ERR_NULL: a required pointer is NULL";
        case QOQ_ERR_SHAPE: return "QOQ_ERR_SHAPE: unsupported M/N/K/mode (need K % 128 == 0, N % 64 == 0)";
        case QOQ_ERR_ALIGN: return "QOQ_ERR_ALIGN: pointer not 16-byte aligned";
        case QOQ_ERR_BLOB: return "QOQ_ERR_BLOB: blob header does not match N, K, mode";
        case QOQ_ERR_WORKSPACE: return "QOQ_ERR_WORKSPACE: workspace missing or too small";
        case QOQ_ERR_ARCH: return "QOQ_ERR_ARCH: device is not gfx950";
        case QOQ_ERR_HIP: return "QOQ_ERR_HIP: HIP runtime error";
        default: return "QOQ_ERR_UNKNOWN";
    }
}

size_t qoq_packed_bytes(int64_t N, int64_t K, int mode)
{
    if (!qoq::shape_ok(N, K, mode)) return 0;
    return qoq::make_layout(N, K, mode).total;
}

size_t qoq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int mode)
{
    if (!qoq::shape_ok(N, K, mode) || M <= 0) return 0;
    int tile_m, split_k;
    qoq::pick_gemm_config(M, N, K, mode, forced(), tile_m, split_k);
    return qoq::gemm_workspace_bytes(M, N, K, tile_m, split_k);
}

int qoq_w4a8_linear(const void* x_fp16, const void* packed, int64_t M, int64_t N, int64_t K, int mode, void* out_fp16,
                    int8_t* qx, void* sx_fp16, int32_t* rowsum, void* workspace, size_t workspace_bytes, void* stream)
{
    if (M > 0 && !x_fp16) return QOQ_ERR_NULL;
    if (M > 0 && !out_fp16) return QOQ_ERR_NULL;
    return gemm_common(qx, sx_fp16, rowsum, packed, M, N, K, mode, out_fp16, nullptr, workspace, workspace_bytes, stream,
                       x_fp16);
}

int qoq_w4a8_gemm_token_sum(const int8_t* qx, const void* sx_fp16, const float* tx, const void* packed, int64_t M,
                            int64_t N, int64_t K, void* out_fp16, void* workspace, size_t workspace_bytes, void* stream)
{
    if (M > 0 && (!tx || !out_fp16)) return QOQ_ERR_NULL;
    return gemm_common(qx, sx_fp16, nullptr, packed, M, N, K, QOQ_PER_CHANNEL, out_fp16, nullptr, workspace,
                       workspace_bytes, stream, nullptr, tx);
}

int qoq_gemm_workspace_prepare(void* workspace, size_t workspace_bytes, void* stream)
{
    if (workspace_bytes == 0) return QOQ_OK;
    if (!workspace) return QOQ_ERR_NULL;
    if (!aligned16(workspace) || (workspace_bytes & 15u)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_zero(workspace, workspace_bytes, static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK
                                                                                                        : QOQ_ERR_HIP;
}

int qoq_set_gemm_config(int tile_m, int split_k)
{
    if (!(tile_m == 0 || tile_m == 16 || tile_m == 32 || tile_m == 64 || (tile_m >= 65 && tile_m <= 71) || (tile_m >= 128 && tile_m <= 132)) || split_k < 0)
        return QOQ_ERR_SHAPE;
    g_forced_tile_m.store(tile_m);
    g_forced_split_k.store(split_k);
    return QOQ_OK;
}

int qoq_query_gemm_config(int64_t M, int64_t N, int64_t K, int mode, int* tile_m, int* split_k)
{
    if (!tile_m || !split_k) return QOQ_ERR_NULL;
    if (!qoq::shape_ok(N, K, mode) || M <= 0) return QOQ_ERR_SHAPE;
    qoq::pick_gemm_config(M, N, K, mode, forced(), *tile_m, *split_k);
    return QOQ_OK;
}

int qoq_pack_weights(const void* w_fp16_dev, int64_t N, int64_t K, int mode, void* packed_dev, void* stream)
{
    if (check_shape(N, K, mode) != QOQ_OK) return QOQ_ERR_SHAPE;
    if (!w_fp16_dev || !packed_dev) return QOQ_ERR_NULL;
    if (!aligned16(w_fp16_dev) || !aligned16(packed_dev)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    const qoq::BlobLayout L = qoq::make_layout(N, K, mode);
    return qoq::launch_pack_weights(w_fp16_dev, L, static_cast<uint8_t*>(packed_dev),
                                    static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_pack_quantized(const uint8_t* q_u4, const uint8_t* s1_u8, const uint8_t* z_u8, const void* s_fp16, int64_t N,
                       int64_t K, int mode, void* packed_dev, void* stream)
{
    if (check_shape(N, K, mode) != QOQ_OK) return QOQ_ERR_SHAPE;
    if (!q_u4 || !z_u8 || !s_fp16 || !packed_dev || (mode == QOQ_GROUP128 && !s1_u8)) return QOQ_ERR_NULL;
    if (!aligned16(packed_dev)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    const qoq::BlobLayout L = qoq::make_layout(N, K, mode);
    return qoq::launch_pack_quantized(q_u4, s1_u8, z_u8, s_fp16, L, static_cast<uint8_t*>(packed_dev),
                                      static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_unpack_weights(const void* packed_dev, int64_t N, int64_t K, int mode, uint8_t* q_u4, uint8_t* s1_u8,
                       uint8_t* z_u8, void* s_fp16, void* stream)
{
    if (check_shape(N, K, mode) != QOQ_OK) return QOQ_ERR_SHAPE;
    if (!packed_dev || !q_u4 || !z_u8 || !s_fp16 || (mode == QOQ_GROUP128 && !s1_u8)) return QOQ_ERR_NULL;
    if (!aligned16(packed_dev)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    const qoq::BlobLayout L = qoq::make_layout(N, K, mode);
    // debug path: read the blob's own description back and compare it with the arguments (synchronizes)
    qoq::BlobHeader h;
    if (hipMemcpyAsync(&h, packed_dev, sizeof(h), hipMemcpyDeviceToHost, static_cast<hipStream_t>(stream)) != hipSuccess ||
        hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess)
        return QOQ_ERR_HIP;
    if (!qoq::header_matches(h, L)) return QOQ_ERR_BLOB;
    return qoq::launch_unpack(static_cast<const uint8_t*>(packed_dev), L, q_u4, s1_u8, z_u8, s_fp16,
                              static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_quant_act_per_token(const void* x_fp16_dev, int64_t M, int64_t K, int8_t* qx, void* sx_fp16, int32_t* rowsum,
                            float* tx, void* stream)
{
    if (M < 0 || M > (1 << 24) || K <= 0 || (K % qoq::kGroup) != 0 || K > (1 << 24)) return QOQ_ERR_SHAPE;
    if (M == 0) return QOQ_OK;  // empty batch: nothing to do
    if (!x_fp16_dev || !qx || !sx_fp16) return QOQ_ERR_NULL;
    if (!aligned16(x_fp16_dev) || !aligned16(qx)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_act_quant(x_fp16_dev, M, K, qx, sx_fp16, rowsum, tx, static_cast<hipStream_t>(stream)) ==
                   hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_rmsnorm_quant(const void* x_fp16, const void* gamma_fp16, double eps, int64_t M, int64_t K, void* y_fp16,
                      int8_t* qx, void* sx_fp16, int32_t* rowsum, float* tx, void* stream)
{
    if (M < 0 || M > (1 << 24) || K <= 0 || (K % qoq::kGroup) != 0 || K > qoq::fused_quant_max_k() || !(eps >= 0.0))
        return QOQ_ERR_SHAPE;
    if (M == 0) return QOQ_OK;
    if (!x_fp16 || !gamma_fp16 || !qx || !sx_fp16) return QOQ_ERR_NULL;
    if (!aligned16(x_fp16) || !aligned16(gamma_fp16) || !aligned16(qx) || !aligned16(y_fp16)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_rmsnorm_quant(x_fp16, gamma_fp16, eps, M, K, y_fp16, qx, sx_fp16, rowsum, tx,
                                     static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_silu_mul_quant(const void* gate_up_fp16, int64_t M, int64_t K, void* y_fp16, int8_t* qx, void* sx_fp16,
                       int32_t* rowsum, float* tx, void* stream)
{
    if (M < 0 || M > (1 << 24) || K <= 0 || (K % qoq::kGroup) != 0 || K > qoq::fused_quant_max_k()) return QOQ_ERR_SHAPE;
    if (M == 0) return QOQ_OK;
    if (!gate_up_fp16 || !qx || !sx_fp16) return QOQ_ERR_NULL;
    if (!aligned16(gate_up_fp16) || !aligned16(qx) || !aligned16(y_fp16)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_silu_mul_quant(gate_up_fp16, M, K, y_fp16, qx, sx_fp16, rowsum, tx,
                                      static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_channel_absmax(const void* x_fp16, int64_t M, int64_t K, float* absmax, void* stream)
{
    if (M < 0 || M > (1 << 24) || K <= 0 || (K % 8) != 0 || K > (1 << 24)) return QOQ_ERR_SHAPE;
    if (!absmax || (!x_fp16 && M > 0)) return QOQ_ERR_NULL;
    if (!aligned16(x_fp16) || !aligned16(absmax)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_channel_absmax(x_fp16, M, K, absmax, static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_channel_order_host(const float* salience_host, int64_t K, int32_t* perm_host)
{
    if (K <= 0 || K > (1 << 24)) return QOQ_ERR_SHAPE;
    if (!salience_host || !perm_host) return QOQ_ERR_NULL;
    for (int64_t k = 0; k < K; ++k)
        if (!std::isfinite(salience_host[k])) return QOQ_ERR_SHAPE;   // a NaN would break the sort's ordering
    qoq::channel_order_host(salience_host, K, perm_host);
    return QOQ_OK;
}

int qoq_gather_channels(const void* src_fp16, const int32_t* perm, int64_t rows, int64_t K, void* dst_fp16, void* stream)
{
    if (rows < 0 || rows > (1 << 24) || K <= 0 || (K % 8) != 0 || K > (1 << 24)) return QOQ_ERR_SHAPE;
    if (rows == 0) return QOQ_OK;
    if (!src_fp16 || !perm || !dst_fp16) return QOQ_ERR_NULL;
    if (src_fp16 == dst_fp16) return QOQ_ERR_SHAPE;        // not in place
    if (!aligned16(src_fp16) || !aligned16(dst_fp16) || !aligned16(perm)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_gather_channels(src_fp16, perm, rows, K, dst_fp16, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_quant_act_per_token_reordered(const void* x_fp16, const int32_t* perm, int64_t M, int64_t K, int8_t* qx, void* sx_fp16,
                                      int32_t* rowsum, float* tx, void* stream)
{
    if (M < 0 || M > (1 << 24) || K <= 0 || (K % qoq::kGroup) != 0 || K > qoq::fused_quant_max_k()) return QOQ_ERR_SHAPE;
    if (M == 0) return QOQ_OK;
    if (!x_fp16 || !perm || !qx || !sx_fp16) return QOQ_ERR_NULL;
    if (!aligned16(x_fp16) || !aligned16(qx) || !aligned16(perm)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_act_quant_reordered(x_fp16, perm, M, K, qx, sx_fp16, rowsum, tx, static_cast<hipStream_t>(stream)) ==
                   hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_hadamard_rotate(const void* src_fp16, int64_t rows, int64_t K, int64_t block, void* dst_fp16, void* stream)
{
    if (rows < 0 || rows > 65535 || K <= 0 || K > (1 << 24) || block < 1 || block > qoq::hadamard_max_block() ||
        (block & (block - 1)) != 0 || (K % block) != 0)
        return QOQ_ERR_SHAPE;
    if (rows == 0) return QOQ_OK;
    if (!src_fp16 || !dst_fp16) return QOQ_ERR_NULL;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_hadamard(src_fp16, rows, K, block, dst_fp16, static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK
                                                                                                                    : QOQ_ERR_HIP;
}

static bool kv4_shape_ok(int64_t B, int64_t Hkv, int64_t S_max, int64_t D)
{
    return D == 128 && B >= 0 && Hkv > 0 && S_max > 0 && B <= (1 << 20) && Hkv <= 1024 && S_max <= (1 << 24) &&
           B * Hkv * ((S_max + 63) / 64) < (int64_t)1 << 40;
}

size_t qoq_kv4_cache_bytes(int64_t B, int64_t Hkv, int64_t S_max, int64_t D)
{
    if (!kv4_shape_ok(B, Hkv, S_max, D)) return 0;
    return qoq::kv4_cache_bytes(B, Hkv, S_max);
}

int qoq_kv4_append(const void* k_fp16, const void* v_fp16, const int32_t* positions, int64_t B, int64_t T, int64_t Hkv,
                   int64_t D, int64_t S_max, void* cache, void* stream)
{
    if (!kv4_shape_ok(B, Hkv, S_max, D) || T < 0 || T > S_max) return QOQ_ERR_SHAPE;
    if (B == 0 || T == 0) return QOQ_OK;
    if (!k_fp16 || !v_fp16 || !positions || !cache) return QOQ_ERR_NULL;
    if (!aligned16(k_fp16) || !aligned16(v_fp16) || !aligned16(cache)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_kv4_append(k_fp16, v_fp16, positions, B, T, Hkv, S_max, static_cast<uint8_t*>(cache),
                                  static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

static int kv4_decode_common(const void* q_fp16, const void* cache, const int32_t* seq_lens, int64_t B, int64_t H, int64_t Hkv,
                             int64_t D, int64_t S_max, void* out_fp16, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!kv4_shape_ok(B, Hkv, S_max, D) || H <= 0 || H % Hkv != 0) return QOQ_ERR_SHAPE;
    if (H / Hkv > 16) return QOQ_ERR_SHAPE;     // the query heads of a KV head are the columns of one matrix instruction
    if (B == 0) return QOQ_OK;
    if (!q_fp16 || !cache || !seq_lens || !out_fp16) return QOQ_ERR_NULL;
    if (!aligned16(q_fp16) || !aligned16(cache) || !aligned16(out_fp16) || !aligned16(workspace)) return QOQ_ERR_ALIGN;
    if (workspace && workspace_bytes < qoq::kv4_decode_workspace_bytes(B, H, Hkv, S_max)) return QOQ_ERR_WORKSPACE;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_kv4_decode(q_fp16, static_cast<const uint8_t*>(cache), seq_lens, B, H, Hkv, S_max, out_fp16, workspace,
                                  workspace_bytes, static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_kv4_attention_decode(const void* q_fp16, const void* cache, const int32_t* seq_lens, int64_t B, int64_t H,
                             int64_t Hkv, int64_t D, int64_t S_max, void* out_fp16, void* stream)
{
    return kv4_decode_common(q_fp16, cache, seq_lens, B, H, Hkv, D, S_max, out_fp16, nullptr, 0, stream);
}

size_t qoq_kv4_attention_workspace_bytes(int64_t B, int64_t H, int64_t Hkv, int64_t D, int64_t S_max)
{
    if (!kv4_shape_ok(B, Hkv, S_max, D) || H <= 0 || H % Hkv != 0 || H / Hkv > 16) return 0;
    return qoq::kv4_decode_workspace_bytes(B, H, Hkv, S_max);
}

int qoq_kv4_attention_decode_split(const void* q_fp16, const void* cache, const int32_t* seq_lens, int64_t B, int64_t H,
                                   int64_t Hkv, int64_t D, int64_t S_max, void* out_fp16, void* workspace,
                                   size_t workspace_bytes, void* stream)
{
    return kv4_decode_common(q_fp16, cache, seq_lens, B, H, Hkv, D, S_max, out_fp16, workspace, workspace_bytes, stream);
}

int qoq_kv4_unpack(const void* cache, int64_t B, int64_t Hkv, int64_t S_max, int64_t D, uint8_t* k_codes, void* k_scale_fp16,
                   void* k_zero_fp16, uint8_t* v_codes, void* v_scale_fp16, void* v_zero_fp16, void* stream)
{
    if (!kv4_shape_ok(B, Hkv, S_max, D)) return QOQ_ERR_SHAPE;
    if (B == 0) return QOQ_OK;
    if (!cache || !k_codes || !k_scale_fp16 || !k_zero_fp16 || !v_codes || !v_scale_fp16 || !v_zero_fp16) return QOQ_ERR_NULL;
    if (!aligned16(cache)) return QOQ_ERR_ALIGN;
    if (!arch_ok()) return QOQ_ERR_ARCH;
    return qoq::launch_kv4_unpack(static_cast<const uint8_t*>(cache), B, Hkv, S_max, k_codes, k_scale_fp16, k_zero_fp16, v_codes,
                                  v_scale_fp16, v_zero_fp16, static_cast<hipStream_t>(stream)) == hipSuccess ? QOQ_OK : QOQ_ERR_HIP;
}

int qoq_w4a8_gemm(const int8_t* qx, const void* sx_fp16, const int32_t* rowsum, const void* packed, int64_t M,
                  int64_t N, int64_t K, int mode, void* out_fp16, void* workspace, size_t workspace_bytes,
                  void* stream)
{
    if (!out_fp16 && M != 0) return QOQ_ERR_NULL;
    return gemm_common(qx, sx_fp16, rowsum, packed, M, N, K, mode, out_fp16, nullptr, workspace, workspace_bytes,
                       stream);
}

int qoq_w4a8_gemm_noalloc(const int8_t* qx, const void* sx_fp16, const int32_t* rowsum, const void* packed, int64_t M,
                          int64_t N, int64_t K, int mode, void* out_fp16, void* stream)
{
    if (!out_fp16 && M != 0) return QOQ_ERR_NULL;
    return gemm_common(qx, sx_fp16, rowsum, packed, M, N, K, mode, out_fp16, nullptr, nullptr, 0, stream, nullptr, nullptr,
                       true);
}

int qoq_w4a8_gemm_i32(const int8_t* qx, const int32_t* rowsum, const void* packed, int64_t M, int64_t N, int64_t K,
                      int mode, int32_t* acc, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!acc && M != 0) return QOQ_ERR_NULL;
    return gemm_common(qx, nullptr, rowsum, packed, M, N, K, mode, nullptr, acc, workspace, workspace_bytes, stream);
}

}  // extern "C"
