/* qoq_w4a8.h -- C ABI of the MI355X (gfx950) W4A8 GEMM with progressive group quantization.
 *
 * Method: QoQ / QServe, arXiv 2405.04532.  Section 4.1 (progressive group quantization,
 * Eq. 3-4, protective range), Section 5.2 (W4A8 GEMM: weights stored in consumption order,
 * UINT4->INT8 dequantization in registers, INT8 matrix cores, FP16 scaling in the epilogue;
 * Eq. 5-7 for the per-channel variant), Section 6.1 (per-token symmetric INT8 activations).
 *
 * Conventions for every call
 *   - "dev" pointers are DEVICE pointers owned by the caller; the library keeps no reference
 *     after the call's work has run.  Nothing is copied to or from the host.
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Work is only
 *     enqueued on it; no call synchronizes, except where stated.
 *   - Weights are [N, K] row-major, N = output channels, K = input channels (the paper's
 *     n x k code tensors).  Activations are [M, K] row-major, one row per token.
 *   - Shapes: K % 128 == 0 (group size g = 128 along k), N % 64 == 0, M >= 0.  (64, not 16: the blob interleaves
 *     the rows of four 16-row matrix-core fragments so that one lane ends up with 4 consecutive output channels
 *     of each, i.e. whole 8-byte FP16 row segments in the epilogue; a 64-channel block is the unit of that
 *     permutation and of the work partition.  Pad N to a multiple of 64 with zero rows.)
 *     Tensor pointers must be 16-byte aligned; the per-token vectors (sx, rowsum, tx) 4-byte aligned.
 *   - Return value: QOQ_OK or an error code; on error nothing was enqueued and no output
 *     was touched.  Errors are never reported any other way (no abort, no exception).
 *   - The library allocates no device memory.  Scratch comes from the caller's `workspace`.
 */
#ifndef QOQ_W4A8_H
#define QOQ_W4A8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QOQ_OK = 0,
    QOQ_ERR_NULL = 1,       /* a required pointer is NULL */
    QOQ_ERR_SHAPE = 2,      /* M, N, K or mode outside the supported set */
    QOQ_ERR_ALIGN = 3,      /* a pointer is not 16-byte aligned */
    QOQ_ERR_BLOB = 4,       /* the packed-weight blob's header does not describe an [N, K] layer of this mode
                               (only calls that read the header report it: qoq_unpack_weights) */
    QOQ_ERR_WORKSPACE = 5,  /* workspace missing or smaller than qoq_gemm_workspace_bytes */
    QOQ_ERR_ARCH = 6,       /* current device is not gfx950 */
    QOQ_ERR_HIP = 7         /* a HIP runtime call failed (launch error) */
} qoq_status;

typedef enum {
    QOQ_GROUP128 = 0,       /* Section 4.1: INT8 per channel, then UINT4 per group of 128 */
    QOQ_PER_CHANNEL = 1     /* Section 5.2.2: UINT4 + zero point + FP16 scale per channel */
} qoq_mode;

/* Human-readable name of a status code (static storage, never NULL). */
const char* qoq_status_string(int status);

/* Size in bytes of the packed-weight blob for an [N, K] layer; 0 if the shape is unsupported. */
size_t qoq_packed_bytes(int64_t N, int64_t K, int mode);

/* Bytes of workspace qoq_w4a8_gemm / qoq_w4a8_gemm_i32 need for this problem (may be 0;
 * always a multiple of 16).  Used for split-k: per-tile arrival counters and partial tiles. */
size_t qoq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int mode);

/* Zero-fill a workspace (dev pointer, 16-byte aligned, size a multiple of 16) on `stream`.
 * A workspace must be zero-filled ONCE after allocation, before its first GEMM call: the
 * GEMM relies on its arrival counters being zero on entry and leaves them zero on exit, so
 * later calls need no further preparation (and no memset appears on the hot path). */
int qoq_gemm_workspace_prepare(void* workspace, size_t workspace_bytes, void* stream);

/* Offline weight path (Section 4.1 Eq. 3-4, Section 5.2.1): quantize FP16 weights and store
 * them in the order the GEMM consumes them.
 *   w_fp16_dev  [N, K] FP16, row-major (read only)
 *   packed_dev  qoq_packed_bytes(N, K, mode) bytes (written; opaque, self-describing header)
 * QOQ_GROUP128: level 1 s0[n] = fp16(max_k|W|/119), q0 = round(W/s0) in [-119, 119];
 *               level 2 per 128 consecutive k: s1 = ceil(range/15) (range widened to hold 0),
 *               z = round(-min/s1), Q = clamp(round(q0/s1 + z), 0, 15).  Ties round away from 0.
 * QOQ_PER_CHANNEL: sw[n] = fp16(range/15), z = round(-min/sw), Q = clamp(round(W/sw + z), 0, 15).
 * Inputs must be finite. */
int qoq_pack_weights(const void* w_fp16_dev, int64_t N, int64_t K, int mode,
                     void* packed_dev, void* stream);

/* Same packing from already-quantized tensors (codes produced elsewhere), all dev pointers:
 *   q_u4   [N, K]      one code 0..15 per byte
 *   s1_u8  [N, K/128]  level-2 scales (1..16; QOQ_GROUP128 only, else NULL)
 *   z_u8   [N, K/128]  level-2 zeros 0..15   (QOQ_PER_CHANNEL: [N])
 *   s_fp16 [N]         s0 (QOQ_GROUP128) or sw (QOQ_PER_CHANNEL)
 * Every (Q - z) * s1 must lie in [-128, 127] (guaranteed by the protective range). */
int qoq_pack_quantized(const uint8_t* q_u4, const uint8_t* s1_u8, const uint8_t* z_u8,
                       const void* s_fp16, int64_t N, int64_t K, int mode,
                       void* packed_dev, void* stream);

/* Inverse of the packing, for tests and debugging: logical tensors out of a blob, same
 * shapes as qoq_pack_quantized (s1_u8 may be NULL in per-channel mode).
 * This is the one call that reads device memory from the host: it copies the blob's 256-byte header back
 * (synchronizing `stream`) and returns QOQ_ERR_BLOB, enqueuing nothing, unless the header carries the library's
 * magic and version and describes exactly this (N, K, mode) with the section offsets the library would lay out.
 * The GEMM calls trust their (N, K, mode) arguments and never read the header. */
int qoq_unpack_weights(const void* packed_dev, int64_t N, int64_t K, int mode,
                       uint8_t* q_u4, uint8_t* s1_u8, uint8_t* z_u8, void* s_fp16, void* stream);

/* Per-token symmetric INT8 activation quantization (Section 6.1; Eq. 1 symmetric form):
 *   x_fp16_dev [M, K] FP16 in;  qx [M, K] INT8 out, sx_fp16 [M] out with
 *   sx = fp16(max_k|x|/127) (1.0 for an all-zero row), qx = round(x/sx) in [-127, 127].
 *   rowsum [M] INT32 = sum_k qx (nullable; the per-channel GEMM needs it, Eq. 6).
 *   tx [M] FP32 = sum_k x, the t_X of Eq. 7 (nullable). */
int qoq_quant_act_per_token(const void* x_fp16_dev, int64_t M, int64_t K,
                            int8_t* qx, void* sx_fp16, int32_t* rowsum, float* tx, void* stream);

/* W4A8 GEMM (Section 5.2): out[m, n] = fp16( acc[m, n] * sx[m] * s[n] ) with
 *   QOQ_GROUP128:    acc = sum_k qx[m,k] * ((Q[n,k] - z[n,g]) * s1[n,g]),  s = s0
 *   QOQ_PER_CHANNEL: acc = sum_k qx[m,k] * Q[n,k] - z[n] * rowsum[m],      s = sw  (Eq. 6)
 * accumulated exactly in INT32; the scaling is done in FP32 and rounded once to FP16.
 *   qx [M, K] INT8, sx_fp16 [M], rowsum [M] INT32 (per-channel only, else may be NULL),
 *   packed = blob of qoq_pack_weights for the same N, K, mode, out_fp16 [M, N] row-major.
 *   workspace: >= qoq_gemm_workspace_bytes(M, N, K, mode) bytes, 16-byte aligned (may be NULL
 *   if that size is 0), zero-filled once with qoq_gemm_workspace_prepare.  One workspace may
 *   serve any sequence of calls of any shapes it is large enough for, as long as they are
 *   ordered on one stream; calls that overlap in time need separate workspaces. */
int qoq_w4a8_gemm(const int8_t* qx, const void* sx_fp16, const int32_t* rowsum,
                  const void* packed, int64_t M, int64_t N, int64_t K, int mode,
                  void* out_fp16, void* workspace, size_t workspace_bytes, void* stream);

/* qoq_w4a8_gemm for callers that cannot allocate device memory or carry a workspace around: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels, same result bit for
 * bit; the split-k scratch (arrival counters and partial tiles) lives in an array inside the library instead of a
 * caller's workspace: 16 MiB of partial tiles and 256 KiB of counters per GPU, held by every GPU the library runs on
 * until the process ends.  The call allocates and frees nothing (the first call on a device looks up the array's
 * address on that device, which allocates nothing either; make that first call before a capture begins).
 *   - A problem whose launch configuration needs more scratch than that returns QOQ_ERR_WORKSPACE and enqueues
 *     nothing (use qoq_w4a8_gemm with a workspace; qoq_gemm_workspace_bytes tells the size: up to 16 MiB + the
 *     counters fit).
 *   - Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two streams, two threads)
 *     race on it; order them on one stream.  The array keeps the last call's partial tiles; its counters are left
 *     at zero by every call, which is all the next call relies on.
 * Other arguments and errors as for qoq_w4a8_gemm. */
int qoq_w4a8_gemm_noalloc(const int8_t* qx, const void* sx_fp16, const int32_t* rowsum, const void* packed,
                          int64_t M, int64_t N, int64_t K, int mode, void* out_fp16, void* stream);

/* Debug twin of qoq_w4a8_gemm: same main loop, returns the raw INT32 accumulators acc[M, N]
 * (per-channel: already zero-corrected) instead of scaling them. */
int qoq_w4a8_gemm_i32(const int8_t* qx, const int32_t* rowsum, const void* packed,
                      int64_t M, int64_t N, int64_t K, int mode,
                      int32_t* acc, void* workspace, size_t workspace_bytes, void* stream);

/* Activation quantization fused into the memory-bound kernel that produces the activations (Section 5.1: into
 * the normalisation in front of the QKV and first FFN projections, into the activation function in front of the
 * second FFN projection; RMSNorm and SiLU(gate) * up for the Llama-family layers the paper evaluates).
 *   qoq_rmsnorm_quant:   y[m, k] = x[m, k] * r[m] * gamma[k],  r[m] = 1 / sqrt(mean_k x[m, :]^2 + eps)
 *   qoq_silu_mul_quant:  y[m, k] = g / (1 + exp(-g)) * u,  g = gate_up[m, k], u = gate_up[m, K + k]  (gate_up is [M, 2K])
 * y is defined as the FP64 evaluation rounded once to FP16, the tensor an unfused pipeline would pass on (the kernels
 * reach exactly those bits from FP32 arithmetic with proven error bounds and evaluate in FP64 only where FP32 cannot
 * decide the rounding); (qx, sx, rowsum, tx) are then exactly qoq_quant_act_per_token(y).  One read of the input, no
 * intermediate tensor.
 *   x_fp16 / gate_up_fp16   FP16, row-major (read only); gamma_fp16 [K] FP16; eps >= 0
 *   y_fp16     [M, K] FP16, optional (NULL: the FP16 activations are not written at all)
 *   qx, sx_fp16, rowsum (nullable), tx (nullable): as for qoq_quant_act_per_token
 * K % 128 == 0 and K <= 32768 (a token row is held in registers); otherwise QOQ_ERR_SHAPE. */
int qoq_rmsnorm_quant(const void* x_fp16, const void* gamma_fp16, double eps, int64_t M, int64_t K, void* y_fp16,
                      int8_t* qx, void* sx_fp16, int32_t* rowsum, float* tx, void* stream);
int qoq_silu_mul_quant(const void* gate_up_fp16, int64_t M, int64_t K, void* y_fp16,
                       int8_t* qx, void* sx_fp16, int32_t* rowsum, float* tx, void* stream);

/* Per-channel W4A8 GEMM with the zero point subtracted after the multiplication exactly as Section 5.2.2
 * fuses it into the epilogue (its Eq. 6 with the quantized activations of the second term replaced by the
 * unquantized ones, Eq. 7):
 *     out[m, n] = fp16( acc[m, n] * sx[m] * sw[n]  -  tx[m] * (z[n] * sw[n]) ),   acc = sum_k qx * Q  (raw codes),
 * evaluated in FP32.  tx [M] FP32 = sum_k X[m, k] over the UNQUANTIZED activations, as produced by
 * qoq_quant_act_per_token.  It approximates qoq_w4a8_gemm in per-channel mode (which folds the zero point in
 * exact integers through the row sums of qx); the two differ by z*sw times the token's summed quantization error.
 *   packed     a blob packed with mode QOQ_PER_CHANNEL
 * Other arguments, workspace and error rules as for qoq_w4a8_gemm. */
int qoq_w4a8_gemm_token_sum(const int8_t* qx, const void* sx_fp16, const float* tx, const void* packed,
                            int64_t M, int64_t N, int64_t K, void* out_fp16,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Activation quantization and GEMM in one call: exactly
 *   qoq_quant_act_per_token(x -> qx, sx, rowsum);  qoq_w4a8_gemm(qx, sx, rowsum, packed -> out)
 * enqueued back to back on `stream` (Section 5.1 places the activation quantization directly in front of
 * the GEMM).  A single-launch variant, in which a few workgroups quantize the rows while the others
 * prefetch weights and a counter releases them, was measured slower than the two launches on MI355X (the
 * device-wide hand-over costs more than a launch) and is not part of the library.
 *   x_fp16     [M, K] FP16 row-major (read only)
 *   qx         [M, K] INT8 (written), sx_fp16 [M] FP16 (written)
 *   rowsum     [M] INT32 (written); required in per-channel mode, may be NULL in group mode
 *   workspace  as for qoq_w4a8_gemm (qoq_gemm_workspace_bytes)
 * Same shape, alignment and error rules as qoq_w4a8_gemm. */
int qoq_w4a8_linear(const void* x_fp16, const void* packed, int64_t M, int64_t N, int64_t K, int mode,
                    void* out_fp16, int8_t* qx, void* sx_fp16, int32_t* rowsum,
                    void* workspace, size_t workspace_bytes, void* stream);

/* ---- Data-free offline transforms (Section 4.3: "Activation-Aware Channel Reordering", "Block Input Module
 * Rotation") ------------------------------------------------------------------------------------------
 * Reordering: the salience of input channel k is max_m |X[m, k]| over calibration tokens; channels are sorted by
 * decreasing salience (ties by channel index) so that a quantization group holds channels of similar salience.
 * Weights are permuted once (gather, then qoq_pack_weights); at run time the activations are permuted inside the
 * quantizer.  X W^T is unchanged.
 *   qoq_channel_absmax     x_fp16 [M, K] device -> absmax [K] FP32 device (overwritten).  K % 8 == 0.
 *   qoq_channel_order_host salience [K] FP32 HOST -> perm [K] INT32 HOST: new channel j = old channel perm[j].
 *                          Every salience must be finite (a NaN has no place in an order): else QOQ_ERR_SHAPE.
 *   qoq_gather_channels    dst[r, j] = src[r, perm[j]], FP16 [rows, K] device, perm [K] INT32 device, not in place.
 *   qoq_quant_act_per_token_reordered   qoq_quant_act_per_token of x[:, perm] in one pass (K <= 32768).
 * perm entries outside [0, K) are clamped (a kernel cannot report them).
 * Rotation: dst = src (I (x) H_block) / sqrt(block), H the Sylvester Hadamard matrix, block a power of two
 * <= 8192 dividing K; the exact product (FP64 sums of FP16 numbers) rounded once to FP16.  Applied to the
 * activations of a block input and to the weights [N, K] of its input modules alike, it leaves X W^T unchanged.
 *   qoq_hadamard_rotate    src_fp16, dst_fp16 [rows, K] FP16 device (may coincide), rows <= 65535.
 * Errors as above (QOQ_ERR_SHAPE, QOQ_ERR_NULL, QOQ_ERR_ALIGN, QOQ_ERR_ARCH, QOQ_ERR_HIP). */
int qoq_channel_absmax(const void* x_fp16, int64_t M, int64_t K, float* absmax, void* stream);
int qoq_channel_order_host(const float* salience_host, int64_t K, int32_t* perm_host);
int qoq_gather_channels(const void* src_fp16, const int32_t* perm, int64_t rows, int64_t K, void* dst_fp16, void* stream);
int qoq_quant_act_per_token_reordered(const void* x_fp16, const int32_t* perm, int64_t M, int64_t K, int8_t* qx,
                                      void* sx_fp16, int32_t* rowsum, float* tx, void* stream);
int qoq_hadamard_rotate(const void* src_fp16, int64_t rows, int64_t K, int64_t block, void* dst_fp16, void* stream);

/* ---- KV4 cache and decode attention (Sections 5.1 "KV Cache Management" and 5.3; Eq. 1-2; the attention
 * equation of Section 3.1) ----------------------------------------------------------------------------
 * The cache holds keys and values as 4-bit codes with one FP16 scale and one FP16 zero point per token and KV
 * head (per-head, dynamic, asymmetric: Eq. 1 with q_min = 0, q_max = 15 on the range of that head's D values,
 * widened to contain 0; s = fp16((max - min) / 15), 1 for an all-zero vector; z = floor(-min / s + 1/2);
 * code = clamp(floor(x / s + z + 1/2), 0, 15); dequantized value (code - z) * s, Eq. 2).  It is an opaque device
 * buffer of qoq_kv4_cache_bytes(B, Hkv, S_max, D) bytes, owned by the caller, organised in pages of 64 tokens
 * per (sequence, KV head) with the scales and zeros stored behind the codes inside each page.  D must be 128.
 *
 * qoq_kv4_append: quantizes T new tokens per sequence and writes them at token positions
 * positions[b] .. positions[b] + T - 1 of sequence b (tokens that would fall outside [0, S_max) are dropped).
 *   k_fp16, v_fp16   [B, T, Hkv, D] FP16, device, read only
 *   positions        [B] INT32, device
 * qoq_kv4_attention_decode: one new query token per sequence,
 *   out[b, h, :] = softmax_t( q[b, h, :] . K^[b, floor(h / r), t, :] / sqrt(D) ) V^[b, floor(h / r), t, :],
 *   t < seq_lens[b], r = H / Hkv an integer in 1 .. 16; K^, V^ the dequantized cache.  Products take FP16 operands
 *   (the softmax weight times the value scale is rounded to FP16 for that), sums and the softmax are FP32, one
 *   rounding to FP16 at the end.  seq_lens[b] is clamped to [0, S_max]; an empty
 *   sequence gives a zero row.
 *   q_fp16 [B, H, D] FP16; seq_lens [B] INT32 device; out_fp16 [B, H, D] FP16 (written)
 * qoq_kv4_unpack (tests): codes as one byte each [B, Hkv, S_max, D] and the FP16 scales / zeros [B, Hkv, S_max]
 * of keys and values; positions never written hold whatever the buffer held.
 * Errors: QOQ_ERR_SHAPE (D != 128, negative sizes, H not a multiple of Hkv or more than 16 times Hkv), QOQ_ERR_NULL, QOQ_ERR_ALIGN (16 bytes),
 * QOQ_ERR_ARCH, QOQ_ERR_HIP.  Nothing is allocated; all work is enqueued on `stream`. */
size_t qoq_kv4_cache_bytes(int64_t B, int64_t Hkv, int64_t S_max, int64_t D);
int qoq_kv4_append(const void* k_fp16, const void* v_fp16, const int32_t* positions, int64_t B, int64_t T,
                   int64_t Hkv, int64_t D, int64_t S_max, void* cache, void* stream);
int qoq_kv4_attention_decode(const void* q_fp16, const void* cache, const int32_t* seq_lens, int64_t B, int64_t H,
                             int64_t Hkv, int64_t D, int64_t S_max, void* out_fp16, void* stream);
/* The same attention with the sequence cut into ranges that separate workgroups process (a second, small launch
 * adds them up): for problems with few (sequence, KV head) pairs -- grouped-query models at small batch -- whose
 * single-pass launch leaves most of the chip idle.  The result obeys the same definition; the sums are formed in a
 * different order.
 *   workspace   device scratch of at least qoq_kv4_attention_workspace_bytes(...) bytes, 16-byte aligned, contents
 *               irrelevant on entry and exit; two calls that overlap in time need separate workspaces.
 * qoq_kv4_attention_workspace_bytes returns 0 when the library would not split this problem; the call then runs the
 * single pass (workspace may be NULL).  A workspace that is too small: QOQ_ERR_WORKSPACE. */
size_t qoq_kv4_attention_workspace_bytes(int64_t B, int64_t H, int64_t Hkv, int64_t D, int64_t S_max);
int qoq_kv4_attention_decode_split(const void* q_fp16, const void* cache, const int32_t* seq_lens, int64_t B, int64_t H,
                                   int64_t Hkv, int64_t D, int64_t S_max, void* out_fp16, void* workspace,
                                   size_t workspace_bytes, void* stream);
int qoq_kv4_unpack(const void* cache, int64_t B, int64_t Hkv, int64_t S_max, int64_t D, uint8_t* k_codes,
                   void* k_scale_fp16, void* k_zero_fp16, uint8_t* v_codes, void* v_scale_fp16, void* v_zero_fp16,
                   void* stream);

/* Test/tuning hook: force the GEMM launch configuration instead of the built-in heuristic.
 * tile_m: 0 = auto; 16, 32, 64 = streaming kernel with that many tokens per tile; 65 = 64 tokens,
 * two adjacent blocks per workgroup in lockstep (N % 128 == 0; else as 64); 66 = four blocks in lockstep
 * (N % 256 == 0; else as 65); 67, 68 = two blocks in lockstep with 32 / 16 tokens per tile (else as 32 / 16);
 * 69, 70, 71 = activation-stationary kernel with 16 / 32 / 64 tokens per tile (activations resident in registers,
 * only weights streamed; K beyond what a workgroup holds is cut into slices that meet in the workspace);
 * 128, 129, 130, 131 = compute-bound kernel with tiles of 256 x 256, 128 x 256, 256 x 128, 256 x 192
 * (tokens x channels); 132 = 128 x 256 tiles with two workgroups per compute unit.
 * split_k >= 0 (0 = auto): for the compute-bound kernel the number of k-slices per output tile, for the
 * streaming kernels the number of workgroups the stream of work units is dealt to (activation-stationary kernels:
 * workgroups per token tile and k-slice that share the layer's 16-channel fragments).
 * Not part of the hot-call contract: the setting is process-wide (two atomics, no lock), so a thread that changes
 * it while another thread sizes a workspace or launches a GEMM changes that thread's configuration too.  Set it
 * once, before any qoq_gemm_workspace_bytes query whose result is still in use: workspace sizes depend on it, and a
 * GEMM call checks its workspace against the size of the configuration in force at the call (QOQ_ERR_WORKSPACE if
 * that is larger).  Returns QOQ_ERR_SHAPE for values outside the set. */
int qoq_set_gemm_config(int tile_m, int split_k);
/* The configuration a GEMM call of this shape would run with (host only, no device work): tile_m as above;
 * split_k = k-slices per tile (compute-bound kernel) or workgroups per token tile (streaming kernels).
 * QOQ_ERR_SHAPE for shapes the GEMM refuses, QOQ_ERR_NULL for null outputs. */
int qoq_query_gemm_config(int64_t M, int64_t N, int64_t K, int mode, int* tile_m, int* split_k);

#ifdef __cplusplus
}
#endif
#endif /* QOQ_W4A8_H */
