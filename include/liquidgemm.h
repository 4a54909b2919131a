/*
 * liquidgemm.h -- C ABI of the MI355X (gfx950) LiquidQuant W4A8 GEMM library.
 *
 * Problem (paper Sec. 2, "GEMM on GPUs"):  Y = X W^T  with  X [M,K] INT8 activations
 * (per-token scale s_x[M]),  W [N,K] weights stored as UINT4 LiquidQuant codes with one
 * (s_u8, a) pair per group of `group` consecutive k of one output channel (Sec. 4,
 * Eq. 7 and Eq. 12) and one FP32 scale s_w[N] per output channel (level 1, Sec. 4),
 * Y [M,N] FP16.  Per element
 *
 *     Wd[n,k]  = (code[n,k] * s_u8[n,k/group] + a[n,k/group]) XOR 0x80      (Eq. 12)
 *     ACC[m,n] = sum_k X[m,k] * Wd[n,k]                  INT8 x INT8 -> INT32 (Sec. 2)
 *     Y[m,n]   = fp16( (float)ACC[m,n] * s_x[m] * s_w[n] )                    (Sec. 4, 5.3)
 *
 * Conventions
 *   - All functions return 0 on success and a negative LQ_ERR_* code otherwise; no
 *     exceptions cross the boundary.  w4a8_last_error() returns a thread-local message
 *     for the last failing call of the calling thread.
 *   - Every buffer is owned by the caller; the library keeps no pointer after a call
 *     returns and allocates no caller-visible memory.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device memory
 *     on the current device and must be 16-byte aligned.  Device entry points only
 *     enqueue work on `hip_stream` (a hipStream_t passed as void*; NULL = default
 *     stream) and return without synchronising.
 *   - Shapes: N % 64 == 0, K % 256 == 0, group in {64, 128}, 0 <= M, K <= 131072
 *     (so that |ACC| <= K * 127 * 127 stays below 2^31), N <= 2^26 (a row of the output is
 *     addressed with 32-bit byte offsets).  M = 0 is a successful no-op.
 *     M itself is only bounded by int: the kernels address X with 32-bit byte offsets, and
 *     w4a8_gemm / w4a8_gemm_i32 / w4a8_gemm_variant run a batch with M * K >= 2^32 as
 *     consecutive launches over chunks of rows on the same stream (same result).  The
 *     grouped and W8A8 entry points do not chunk: there an expert (resp. the call) with
 *     rows * K >= 2^32 is rejected with LQ_ERR_INVALID.
 *   - The packed weight blob (W_packed, gparams) is opaque, position independent and
 *     specific to this library version (w4a8_version()); it can be stored and reloaded
 *     byte for byte.  Its size is given by liquidquant_packed_size().
 *   - Precondition of the device entry points (not checked on the device): every
 *     (code, s_u8, a) triple satisfies code * s_u8 + a <= 255 (Eq. 11).  The packers
 *     below guarantee it; behaviour on hand-made blobs that violate it is undefined
 *     (the per-byte arithmetic of Eq. 12 would carry into the neighbouring byte).
 */
#ifndef LIQUIDGEMM_H
#define LIQUIDGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LQ_OK 0
#define LQ_ERR_INVALID (-1)   /* bad shape, null pointer, unknown variant            */
#define LQ_ERR_ALIGN (-2)     /* a device pointer is not 16-byte aligned             */
#define LQ_ERR_WORKSPACE (-3) /* workspace_bytes < w4a8_gemm_workspace_size(...)     */
#define LQ_ERR_HIP (-4)       /* a HIP runtime call or kernel launch failed          */

/* Library / packed-layout version (changes whenever the blob layout changes). */
int w4a8_version(void);

/* Message of the last error raised on the calling thread ("" if none). */
const char *w4a8_last_error(void);

/* ------------------------------------------------------------------------------------
 * Offline LiquidQuant packer (host, Sec. 4 and Sec. 6 "Offline Quantization")
 * ------------------------------------------------------------------------------------ */

/* Sizes of the two parts of the packed blob: codes_bytes = N*K/2 (two codes per byte),
 * gparams_bytes = 2*N*K/group (one (s_u8, a) byte pair per group).  Either output
 * pointer may be NULL. */
int liquidquant_packed_size(int N, int K, int group, size_t *codes_bytes, size_t *gparams_bytes);

/* Two-level quantisation of W (host, [N,K] row-major FP32 holding the FP16 weights):
 *   level 1, per output channel (Sec. 4, Eq. 1 with z = 0, protective range):
 *       s_w[n] = max_k |W[n,k]| / 119 (FP32; 1 if the row is zero),
 *       Q_i8 = clamp(rint(W / s_w), -119, 119)
 *   level 2, per group (Eq. 7): min = min(Q_i8), R = max - min,
 *       s_u8 = max(1, round(R / 15)), code = min(15, round((Q_i8 - min) / s_u8)),
 *       a = 128 + min (Eq. 10)
 * then permutation into the gfx950 MFMA operand order and nibble packing (the analogue
 * of the dual-MMA packed layout of Sec. 5.2).  Outputs (host): W_packed (codes_bytes),
 * gparams (gparams_bytes), w_scales [N]. */
int liquidquant_pack_weights(const float *W, int N, int K, int group, void *W_packed,
                             uint8_t *gparams, float *w_scales);

/* Same, with W given as IEEE binary16 bit patterns (host, [N,K] row-major). */
int liquidquant_pack_weights_f16(const uint16_t *W_f16, int N, int K, int group, void *W_packed,
                                 uint8_t *gparams, float *w_scales);

/* Level 2 and packing only, from level-1 integers Q_i8 (host, [N,K], every |q| <= 119;
 * values outside that range are rejected with LQ_ERR_INVALID). */
int liquidquant_pack_from_i8(const int8_t *Q_i8, int N, int K, int group, void *W_packed,
                             uint8_t *gparams);

/* Inverse of the permutation (host, for tests and tooling): codes [N,K] one code per
 * byte in natural order, s_u8 [N,K/group], a [N,K/group].  Output pointers may be NULL. */
int liquidquant_unpack_weights(const void *W_packed, const uint8_t *gparams, int N, int K,
                               int group, uint8_t *codes, uint8_t *s_u8, uint8_t *a);

/* ------------------------------------------------------------------------------------
 * W4A8 GEMM (device, Sec. 5: load, unpack, LQQ dequantisation, INT8 MFMA, epilogue)
 * ------------------------------------------------------------------------------------ */

/* Bytes of device workspace w4a8_gemm* can use for this shape (0 when no kernel that can run
 * the shape splits K across blocks): 32 KiB of arrival tickets followed by room for the INT32
 * partial tiles of the grid-level split-K (the 256-row tile kernels with K slices keep a whole
 * [M,N] INT32 matrix per slice there, at most four).
 *   - The first 32 KiB (or the whole buffer if smaller) must be zero before the first call
 *     that uses the buffer: zero it yourself or enqueue w4a8_workspace_init() once.  The
 *     kernels leave the tickets zero again, so one initialisation serves any number of calls,
 *     shapes and HIP graph replays.  The rest needs no initialisation.
 *   - One workspace serves one call at a time: calls that may overlap in time on one GPU
 *     (different streams) need different workspaces; calls on one stream can share one.
 *   - With a smaller (or NULL) workspace the dispatcher runs the same kernels without the
 *     split (or with as many slices as the workspace holds), which is slower for small N but
 *     gives the same result; a variant that names its split (w4a8_gemm_variant) fails with
 *     LQ_ERR_WORKSPACE instead. */
size_t w4a8_gemm_workspace_size(int M, int N, int K, int group);

/* Enqueue the zeroing of a workspace's ticket area on `hip_stream` (a small fill kernel; safe
 * under HIP graph capture).  NULL or empty workspaces are a successful no-op. */
int w4a8_workspace_init(void *workspace, size_t workspace_bytes, void *hip_stream);

/* Y[M,N] (device, FP16 bits, row-major) = epilogue(X . dequant(W)^T).
 *   X           device [M,K] INT8 row-major
 *   act_scales  device [M] FP32, per-token scales s_x (Sec. 6)
 *   W_packed, gparams  device copies of the packer's outputs
 *   w_scales    device [N] FP32, per-channel scales s_w
 *   workspace   device, see w4a8_gemm_workspace_size(); may be NULL */
int w4a8_gemm(int M, int N, int K, int group, const int8_t *X, const float *act_scales,
              const void *W_packed, const uint8_t *gparams, const float *w_scales, uint16_t *Y,
              void *workspace, size_t workspace_bytes, void *hip_stream);

/* w4a8_gemm for callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments
 * without the workspace, same kernels, same result bit for bit.  The split-K state lives in
 * a workspace built into the library, 32 KiB of tickets + 32 MiB of partial tiles of static
 * device memory per GPU, held until the process ends; the call allocates nothing (no
 * hipMalloc / hipFree, no allocating library routine) and only enqueues kernels on
 * `hip_stream`.
 *   - Shapes whose dispatcher kernel would use more split-K workspace than that are rejected
 *     with LQ_ERR_WORKSPACE (the message names both sizes); use w4a8_gemm with a workspace
 *     of the caller for them.
 *   - Every call on a GPU shares that GPU's built-in workspace: calls that may overlap in time
 *     on one GPU (different streams, or graphs replayed concurrently) race on it and give
 *     undefined results; calls ordered on one stream are safe.  The tickets are zero when the
 *     library is loaded and every call leaves them zero; partial tiles need no clearing. */
int w4a8_gemm_static(int M, int N, int K, int group, const int8_t *X, const float *act_scales,
                     const void *W_packed, const uint8_t *gparams, const float *w_scales, uint16_t *Y,
                     void *hip_stream);

/* Parity hook: the raw INT32 accumulators ACC[M,N] (device, row-major) of the same
 * kernels, without the scaling epilogue. */
int w4a8_gemm_i32(int M, int N, int K, int group, const int8_t *X, const void *W_packed,
                  const uint8_t *gparams, int32_t *ACC, void *workspace, size_t workspace_bytes,
                  void *hip_stream);

/* Tuning / test hook: run one named kernel variant instead of the dispatcher's choice.
 * `variant` in [0, w4a8_variant_count()); -1 = dispatcher.  Y and ACC may each be NULL
 * (at least one must be given; act_scales / w_scales may be NULL when Y is).  Returns
 * LQ_ERR_INVALID if the variant cannot run this shape (e.g. M too large for a
 * decode kernel). */
int w4a8_gemm_variant(int variant, int M, int N, int K, int group, const int8_t *X,
                      const float *act_scales, const void *W_packed, const uint8_t *gparams,
                      const float *w_scales, uint16_t *Y, int32_t *ACC, void *workspace,
                      size_t workspace_bytes, void *hip_stream);
int w4a8_variant_count(void);
const char *w4a8_variant_name(int variant);            /* NULL if out of range        */
int w4a8_variant_supports(int variant, int M, int N, int K, int group); /* 1 if it can run the shape */
int w4a8_select_variant(int M, int N, int K, int group); /* the dispatcher's choice, <0 on error */
/* What w4a8_gemm / w4a8_gemm_i32 launch for a shape.  A batch whose 256 x 256 tiles make whole
 * rounds of the chip plus a rest that a kernel of its own serves better (a few rows, or several
 * hundred on smaller tiles) runs as two launches over consecutive rows: returns the variant
 * of the first, writes its rows to *rows_first (= M when there is one launch only) and the
 * variant of the launch over the remaining rows to *variant_rest (-1 when there is none).
 * <0 on error. */
int w4a8_select_plan(int M, int N, int K, int group, int *rows_first, int *variant_rest);

/* Layout hook: dequantise the whole packed matrix on the device with the kernels' own
 * unpack + Eq. 12 code path into Wd [N,K] INT8 row-major (device). */
int w4a8_dequant_dump(const void *W_packed, const uint8_t *gparams, int N, int K, int group,
                      int8_t *Wd, void *hip_stream);

/* ------------------------------------------------------------------------------------
 * Grouped GEMM (device; mixture-of-experts layers, Sec. 7.3): E independent W4A8 GEMMs that
 * share N, K and group, over disjoint runs of tokens, in at most three kernel launches.
 * ------------------------------------------------------------------------------------ */

/*   row_offsets host [E+1], row_offsets[0] = 0, non-decreasing: expert e owns rows
 *               row_offsets[e] .. row_offsets[e+1]-1 of X, act_scales and Y (experts without
 *               rows are skipped); read before the call returns
 *   X           device [row_offsets[E], K] INT8;  act_scales device [row_offsets[E]] FP32
 *   W_packed    device, the E packed code blobs back to back (codes_bytes each, in expert
 *               order); gparams likewise (gparams_bytes each); w_scales device [E, N] FP32
 *   Y           device [row_offsets[E], N] FP16 bits, or NULL
 *   ACC         device [row_offsets[E], N] raw INT32 accumulators (parity hook), or NULL
 * 1 <= E <= 64; every expert's rows * K < 2^32 (else LQ_ERR_INVALID: split the expert).
 * Per expert the result is exactly that of w4a8_gemm / w4a8_gemm_i32 on its rows.  No
 * workspace: the grid over all experts replaces the split of K. */
int w4a8_grouped_gemm(int E, const int *row_offsets, int N, int K, int group, const int8_t *X,
                      const float *act_scales, const void *W_packed, const uint8_t *gparams,
                      const float *w_scales, uint16_t *Y, int32_t *ACC, void *hip_stream);

/* ------------------------------------------------------------------------------------
 * W8A8 reference (Sec. 3.2, Sec. 7.3: the baseline without dequantisation that W4A8 is
 * measured against): the same tiled kernel skeleton with INT8 weights fed to the MFMA as
 * loaded.  A measuring stick, not a product path: no split-K, meant for M >= 128.
 * ------------------------------------------------------------------------------------ */

/* Host.  W_i8 [N,K] INT8 row-major -> W8_packed, N*K bytes in the kernel's operand order
 * (opaque).  N % 64 == 0, K % 256 == 0, K <= 131072. */
int w8a8_pack_weights(const int8_t *W_i8, int N, int K, void *W8_packed);

/* Device, asynchronous on hip_stream.  ACC[m,n] = sum_k X[m,k] * W[n,k] (INT32, exact),
 * Y[m,n] = fp16(ACC * act_scales[m] * w_scales[n]) as in w4a8_gemm.  Y or ACC may be NULL
 * (not both); the scales may be NULL when Y is.  All pointers device, 16-byte aligned,
 * caller-owned; M * K < 2^32.  With W_i8 = the dequantised LiquidQuant weights
 * (w4a8_dequant_dump) the results equal those of w4a8_gemm / w4a8_gemm_i32 bit for bit. */
int w8a8_gemm(int M, int N, int K, const int8_t *X, const float *act_scales, const void *W8_packed,
              const float *w_scales, uint16_t *Y, int32_t *ACC, void *hip_stream);

/* ------------------------------------------------------------------------------------
 * Activation quantisation (device, Sec. 6 "Serving System": dynamic per-token INT8 after
 * dividing by the smooth scale) -- produces the X and act_scales that w4a8_gemm consumes.
 * ------------------------------------------------------------------------------------ */

/*   X_f16       device [M,K] IEEE binary16 bit patterns, row-major
 *   smooth      device [K] FP32 smooth scales (positive, finite), or NULL for none
 *   X_i8        device [M,K] INT8 out:  clamp(rint(x' / s_x[m]), -127, 127),
 *               x' = (float)X / smooth
 *   act_scales  device [M] FP32 out:    s_x[m] = max_k |x'| / 127   (1 if the token is zero)
 * All arithmetic is correctly rounded FP32, so the result is defined bit for bit.
 * K % 8 == 0; M = 0 is a successful no-op.  Tokens containing NaN or infinity (or whose
 * divide overflows) give unspecified codes for that token only. */
int w4a8_quantize_activations(int M, int K, const uint16_t *X_f16, const float *smooth,
                              int8_t *X_i8, float *act_scales, void *hip_stream);

/* ------------------------------------------------------------------------------------
 * Calibration (measurement support): what this GPU delivers on the two resources of the
 * cost model of Sec. 3.2 with nothing else in the way.  Both only enqueue a kernel on
 * `hip_stream`; the caller times them.
 * ------------------------------------------------------------------------------------ */

/* T_LD: read `bytes` (rounded down to 16) of device memory at `buf` once, with the same
 * 16-byte non-temporal loads the GEMM kernels use for W; nothing of size is written. */
int w4a8_calib_stream_read(const void *buf, size_t bytes, void *hip_stream);

/* T_MMA: `iters` x 64 back-to-back INT8 32x32x32 MFMAs per wave on register operands, two
 * waves per SIMD on every CU.  random_operands = 0: constant operands; 1: pseudo-random
 * bytes that change from one MFMA to the next (the multipliers of this chip draw more power
 * on such data and clock lower).  *ops (host, may be NULL) receives the operation count
 * (2 per multiply-accumulate) of the launch. */
int w4a8_calib_mfma_i8(int iters, int random_operands, double *ops, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LIQUIDGEMM_H */
