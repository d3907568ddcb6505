/*
 * dmr_qlinear: the linear layer of a step routed by Dynamic Mixed-Precision Routing, for MI355X.
 *
 * The router of the paper picks, per decision step, which copy of the model serves the step
 * (Sec. 3, Eq. 1): the bf16 high-precision copy or the low-precision copy whose Linear layers
 * (all except lm_head, App. E "Per-cell configuration") hold 4-bit weights and take 16-bit
 * activations (Sec. 5.1 "Experimental Models and Precision").  A step routed low calls
 * dmr_qlinear_forward for each such layer, a step routed high calls dmr_qlinear_bf16_forward;
 * their cost ratio is the T_high / T_low of the paper's cost model (Sec. 4.3, Eq. 9), and App. B
 * locates that cost in streaming the weights from memory once per generated token.
 *
 * Quantised format at this boundary (the paper leaves it open; this is the build's reading):
 *   qweight  uint32 [N][K/8]   code q[n][8i+j] (0..15) in bits [4j,4j+4) of word i of row n
 *   scales   bf16   [N][K/g]   finite, > 0
 *   zeros    bf16   [N][K/g]   an integer code 0..15 held in bf16
 *   w^[n][k] = (q[n][k] - zeros[n][k/g]) * scales[n][k/g],   g = 128
 *
 * General conventions
 *   - Every pointer named d_* is DEVICE memory owned by the caller; the library never allocates
 *     or frees device memory.  Arrays are row-major and contiguous.  bf16 travels as uint16_t.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls enqueue work on
 *     it and return without synchronising; buffers must stay valid until that work is done.
 *   - Errors come back as a dmr_status_t; nothing throws or aborts.  All argument checks happen
 *     before the first HIP call, so a rejected call has touched nothing.  A failed launch
 *     returns DMR_ERR_HIP.
 *   - Shapes: K % 128 == 0, N % 16 == 0, g == 128, M >= 0 (M == 0 is DMR_OK and launches
 *     nothing).  Device pointers must be 16-byte aligned.  No bias, no activation function.
 *   - Non-finite activations are outside the contract.
 *   - Two calls that share an output or workspace buffer must not overlap in time.
 */
#ifndef DMR_QLINEAR_H
#define DMR_QLINEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dmr_qlinear dmr_qlinear_t; /* opaque, lives in host memory */

typedef enum {
    DMR_OK = 0,
    DMR_ERR_NULL = 1,        /* a required pointer is NULL                              */
    DMR_ERR_SHAPE = 2,       /* a dimension is negative, zero or not a permitted multiple */
    DMR_ERR_ALIGN = 3,       /* a device pointer is not 16-byte aligned                  */
    DMR_ERR_WORKSPACE = 4,   /* storage or workspace buffer smaller than the size query  */
    DMR_ERR_UNSUPPORTED = 5, /* a valid request this build has no kernel for (g != 128)  */
    DMR_ERR_HIP = 6          /* the HIP runtime refused a launch                         */
} dmr_status_t;

typedef enum {
    DMR_OUT_BF16 = 0, /* y is bf16 [M][N], rounded to nearest even from the fp32 accumulator */
    DMR_OUT_FP32 = 1  /* y is fp32 [M][N], the accumulator itself                            */
} dmr_out_t;

/* Bytes of device memory a layer needs for its re-tiled weights, scales and zero points
 * (dmr_qlinear_create's d_storage).  0 if the shape is not supported. */
size_t dmr_qlinear_storage_bytes(int64_t K, int64_t N, int32_t g);

/* Bytes of scratch dmr_qlinear_forward (resp. dmr_qlinear_bf16_forward) needs for this shape
 * (d_ws); may be 0, and then d_ws may be NULL.  Non-zero for batches of rollouts (a few to a few
 * hundred rows): either the activations re-ordered once per call, or fp32 partial sums when K is
 * split over workgroups because M x N alone would leave most of the chip idle.  Non-zero also for the
 * 4-bit and 3-bit tiled path (prefill, and more than 128 rows on very wide layers): per call it keeps there the operands of the zero-point
 * term (bf16, 12 (M + N) K / 128 bytes), one fp32 factor per (row, group) and a few flags.  The
 * workspace may arrive uninitialised; its contents are undefined after the call. */
size_t dmr_qlinear_workspace_bytes(int64_t M, int64_t K, int64_t N);
size_t dmr_qlinear_bf16_workspace_bytes(int64_t M, int64_t K, int64_t N);

/*
 * Prepare one low-precision Linear layer (a layer of the W4A16 copy, Sec. 5.1 / App. E): re-tile
 * the canonical arrays into d_storage in the order the kernels stream them.  One-off per layer,
 * integer only.  The canonical arrays may be released once the stream work has completed;
 * d_storage must outlive the handle.  *out receives a host-side handle.
 */
dmr_status_t dmr_qlinear_create(dmr_qlinear_t **out, int64_t K, int64_t N, int32_t g,
                                const uint32_t *d_qweight, /* [N][K/8]  */
                                const uint16_t *d_scales,  /* bf16 [N][K/g] */
                                const uint16_t *d_zeros,   /* bf16 [N][K/g] */
                                void *d_storage, size_t storage_bytes, void *stream);

/*
 * The paper's literal W4A16 setting, "default per-channel grouping" (App. E "Per-cell configuration"):
 * symmetric INT4 with one bf16 scale per output row and the fixed zero point 8,
 *   w^[n][k] = (q[n][k] - 8) * scales[n].
 * d_scales is bf16 [N].  The handle behaves like a group-wise one (g reported as K).  Storage
 * (dmr_qlinear_per_channel_storage_bytes) is 0.5 byte per weight plus one 4-byte scale word per row: no per-group
 * stream, so a decode step moves 0.5 instead of 0.53125 byte per weight.  The kernels are the group-wise ones
 * reading the row's one word for every group.
 */
size_t dmr_qlinear_per_channel_storage_bytes(int64_t K, int64_t N);
dmr_status_t dmr_qlinear_create_per_channel(dmr_qlinear_t **out, int64_t K, int64_t N,
                                            const uint32_t *d_qweight, /* [N][K/8] */
                                            const uint16_t *d_scales,  /* bf16 [N] */
                                            void *d_storage, size_t storage_bytes, void *stream);

/* The layer's weights as bf16 [N][K]: RNE_bf16((q - z) * s), exactly one correct answer. */
dmr_status_t dmr_qlinear_dequantize(const dmr_qlinear_t *layer, uint16_t *d_w_bf16, void *stream);

/*
 * A step routed to the low-precision copy (Sec. 3, Eq. 1 with r_t = low):
 *   y[m][n] = sum_k x[m][k] * (q[n][k] - z[n][k/g]) * s[n][k/g]
 * with the dequantisation fused into the product and fp32 accumulation.  d_x is bf16 [M][K];
 * d_y is [M][N] of the type `out` names.  Small M takes the weight-streaming paths (decode, a
 * group of parallel rollouts), large M the tiled MFMA path (prefill of a long prompt, App. B).
 * No path rounds a weight: every kernel multiplies the activations with the exact integer codes and
 * applies scale and zero point in fp32 (agreement with the fp64 definition at the 1e-5 rms(y) level on
 * the fp32 output; rows with scales the tiled path cannot carry, zero, subnormal or spanning more than
 * 2^20 within a row, are served by a slower exact kernel inside the same call).
 */
dmr_status_t dmr_qlinear_forward(const dmr_qlinear_t *layer, const uint16_t *d_x, int64_t M,
                                 void *d_y, dmr_out_t out, void *d_ws, size_t ws_bytes,
                                 void *stream);

/*
 * dmr_qlinear_forward for callers that cannot allocate device memory and therefore cannot bring the
 * workspace: code running under HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results (bit for bit) and errors as dmr_qlinear_forward, minus d_ws / ws_bytes: the
 * scratch (fp32 partial sums of the kernels that split K, re-ordered activations, the tiled path's
 * zero-point operands) is a fixed array of
 * DMR_STATIC_SCRATCH_BYTES in device memory that belongs to the library itself; each GPU the library runs
 * on holds one copy until the process ends.  The call allocates and frees nothing.  A shape whose
 * dmr_qlinear_workspace_bytes (dmr_qlinear_w3_workspace_bytes for a 3-bit layer) exceeds that size is
 * refused with DMR_ERR_WORKSPACE before anything is launched; such calls go through dmr_qlinear_forward.
 * All calls on one GPU share the one array: two calls whose work overlaps in time on the same GPU (different
 * streams, or threads) race on it; calls on one stream are ordered and safe.  Nothing needs clearing
 * between calls.  The first call on a device looks up the array's address (one runtime query).
 */
#define DMR_STATIC_SCRATCH_BYTES ((size_t)8 << 20)
dmr_status_t dmr_qlinear_forward_static(const dmr_qlinear_t *layer, const uint16_t *d_x, int64_t M,
                                        void *d_y, dmr_out_t out, void *stream);

/*
 * The same layer in the bf16 high-precision copy (Sec. 5.1; a step with r_t = high):
 *   y[m][n] = sum_k x[m][k] * W[n][k],  W bf16 [N][K], fp32 accumulation.
 * This is the denominator of the T_high / T_low ratio (Eq. 9).  Needs no handle; d_ws as
 * dmr_qlinear_bf16_workspace_bytes says.
 */
dmr_status_t dmr_qlinear_bf16_forward(const uint16_t *d_w, const uint16_t *d_x, int64_t M,
                                      int64_t K, int64_t N, void *d_y, dmr_out_t out, void *d_ws,
                                      size_t ws_bytes, void *stream);

/*
 * Decoder glue between the Linear layers of one routed step.  The models of Sec. 5.1 are pre-norm
 * decoders with RMSNorm and a SwiGLU MLP; the paper does not restate these operations, they are
 * taken in their textbook form, computed in fp32 with one rounding to bf16 at the end (the next
 * Linear takes bf16 activations):
 *   rmsnorm  out[m][k] = bf16( x[m][k] * gamma[k] / sqrt(mean_k(x[m][k]^2) + eps) )      (0 for a zero row)
 *   swiglu   out[m][i] = bf16( silu(in[m][i]) * in[m][I + i] ),  silu(a) = a / (1 + exp(-a)),
 *            in = [M][2 I], the gate half of the fused gate+up projection first, then the up half.
 * K and I must be multiples of 8; all pointers device memory, 16-byte aligned.
 */
dmr_status_t dmr_glue_rmsnorm(const uint16_t *d_x, const uint16_t *d_gamma, float eps, int64_t M,
                              int64_t K, uint16_t *d_out, void *stream);
dmr_status_t dmr_glue_swiglu(const uint16_t *d_in, int64_t M, int64_t I, uint16_t *d_out, void *stream);

/*
 * A Linear of either copy (Eq. 1) with its surrounding glue fused in, so that a decode step is a
 * chain of Linear launches only (App. B: decode cost is one pass over the weights per token, so
 * every extra launch between them is pure overhead):
 *   prologue  DMR_PRO_RMSNORM: the layer runs on rmsnorm(d_in, d_gamma, eps), d_in = [M][K]
 *             DMR_PRO_SWIGLU:  the layer runs on swiglu(d_in), d_in = [M][2 K]
 *             DMR_PRO_NONE:    d_in = [M][K] as in the plain forward
 *   epilogue  d_residual (bf16 [M][N]) or NULL: y = acc + residual in fp32, rounded once to `out`.
 * M = 1 (both copies) fuses the prologue into the staging of the activation row and the residual
 * into the output store of the weight-streaming kernel; 2 <= M <= 16 fuses the residual only, where
 * the streaming kernel of that size class serves the shape (a prologue would be recomputed by every
 * workgroup, so it runs as a kernel of its own into d_ws); anything else runs the glue
 * kernels into d_ws and then the plain forward.  d_ws as the matching *_fused_workspace_bytes query says (never 0 with a
 * prologue or a residual).
 */
typedef enum {
    DMR_PRO_NONE = 0,
    DMR_PRO_RMSNORM = 1,
    DMR_PRO_SWIGLU = 2
} dmr_prologue_t;

size_t dmr_qlinear_fused_workspace_bytes(const dmr_qlinear_t *layer, int64_t M, dmr_prologue_t pro,
                                         int32_t has_residual);
size_t dmr_qlinear_bf16_fused_workspace_bytes(int64_t M, int64_t K, int64_t N, dmr_prologue_t pro,
                                              int32_t has_residual);
dmr_status_t dmr_qlinear_forward_fused(const dmr_qlinear_t *layer, dmr_prologue_t pro,
                                       const uint16_t *d_in, const uint16_t *d_gamma, float eps,
                                       const uint16_t *d_residual, int64_t M, void *d_y, dmr_out_t out,
                                       void *d_ws, size_t ws_bytes, void *stream);
dmr_status_t dmr_qlinear_bf16_forward_fused(const uint16_t *d_w, dmr_prologue_t pro,
                                            const uint16_t *d_in, const uint16_t *d_gamma, float eps,
                                            const uint16_t *d_residual, int64_t M, int64_t K, int64_t N,
                                            void *d_y, dmr_out_t out, void *d_ws, size_t ws_bytes,
                                            void *stream);

/*
 * Offline step that produces the low-precision copy (App. E names AWQ/GPTQ; this is plain
 * asymmetric round-to-nearest, which yields the same format): fp32 weights [N][K] to canonical
 * qweight / scales / zeros.  Per (row, group): lo = min(w, 0), hi = max(w, 0),
 * s = RNE_bf16(float((hi - lo) / 15)) (1 if that is 0), z = clamp(rint(-lo / s), 0, 15),
 * q = clamp(rint(w / s) + z, 0, 15), divisions and rint in fp64 with the stored bf16 s.
 */
dmr_status_t dmr_qlinear_quantize(int64_t K, int64_t N, int32_t g, const float *d_w,
                                  uint32_t *d_qweight, uint16_t *d_scales, uint16_t *d_zeros,
                                  void *stream);

/*
 * The 3-bit variant of the low-precision copy: the paper's W3A16 group-128 cell (Sec. 5.1, App. E),
 * which it could only run fake-quantised and whose cost it projected as T_W4 / 1.15 (App. A).  Format:
 * codes 0..7, 32 per three words along k (code j in bits [3j, 3j+3) of the 96-bit little-endian run),
 * qweight3 uint32 [N][3K/32]; scales and zeros as for 4 bits, zero points 0..7.  The handle these
 * calls return is used with dmr_qlinear_dequantize / _forward / _destroy like a 4-bit one.  Every size class
 * runs native kernels that unpack the 3-bit codes in registers or on their way into LDS and keep them exact;
 * d_ws holds fp32 partial sums where K is split and, on the tiled path, the zero-point operands, factors
 * and flags described at dmr_qlinear_workspace_bytes; dmr_qlinear_w3_workspace_bytes gives the size.
 */
size_t dmr_qlinear_w3_storage_bytes(int64_t K, int64_t N, int32_t g);
size_t dmr_qlinear_w3_workspace_bytes(int64_t M, int64_t K, int64_t N);
dmr_status_t dmr_qlinear_w3_create(dmr_qlinear_t **out, int64_t K, int64_t N, int32_t g,
                                   const uint32_t *d_qweight3, /* [N][3K/32] */
                                   const uint16_t *d_scales,   /* bf16 [N][K/g] */
                                   const uint16_t *d_zeros,    /* bf16 [N][K/g] */
                                   void *d_storage, size_t storage_bytes, void *stream);
/* Round-to-nearest quantiser of the 3-bit format: as dmr_qlinear_quantize with 7 in place of 15. */
dmr_status_t dmr_qlinear_quantize_w3(int64_t K, int64_t N, int32_t g, const float *d_w,
                                     uint32_t *d_qweight3, uint16_t *d_scales, uint16_t *d_zeros,
                                     void *stream);
/* 4 or 3: which format a handle holds (0 for NULL). */
int32_t dmr_qlinear_bits(const dmr_qlinear_t *layer);

/*
 * Measurement aid, not part of a routed step: read `bytes` (a multiple of 16) of d_buf once with
 * 128-bit loads from `blocks` workgroups of 256 threads and leave one word per thread in d_sink
 * (blocks * 256 words).  Timing it over a buffer much larger than the caches gives the HBM read
 * rate that App. B's "constrained by memory bandwidth" refers to on this chip.
 */
dmr_status_t dmr_probe_hbm_read(const void *d_buf, size_t bytes, uint32_t *d_sink, int32_t blocks,
                                void *stream);

/*
 * Measurement aid, not part of a routed step: launch a kernel that does nothing with `blocks` workgroups of
 * `threads` threads (a multiple of 64, at most 1024) and `lds_bytes` (at most 64 KB) of dynamic LDS.  Its
 * time in a replayed graph is the fixed cost that every per-layer launch of a decode step pays before its
 * first byte (App. B: decode is one pass over the weights per token; at these layer sizes that pass is a few
 * microseconds, so the fixed cost decides how close a layer gets to the memory rate).
 */
dmr_status_t dmr_probe_empty_launch(int32_t blocks, int32_t threads, size_t lds_bytes, void *stream);

/*
 * Diagnostic, not part of a routed step: the name of the kernel class that serves M rows of a (K, N) layer
 * held in `format` ("w4_gemv", "w4_stream", "w4_panel", "w4_wide", "w4_skinny2", "w4_mid",
 * "w4_gemm256_rescale", "w4_gemm256x128_rescale", "w4_gemm128_rescale", "w4_gemm128_exact", the "w3_*" and "bf16_*" counterparts; "none" for an unsupported shape).  Pure host arithmetic,
 * the same the forward calls use; a decode row too long for the M = 1 kernels' LDS budget is served by a
 * fallback of the same name class.  Lets a test or a profile state which kernel it covers.
 */
typedef enum {
    DMR_FMT_W4_G128 = 0,        /* dmr_qlinear_create */
    DMR_FMT_W4_PER_CHANNEL = 1, /* dmr_qlinear_create_per_channel */
    DMR_FMT_W3_G128 = 2,        /* dmr_qlinear_w3_create */
    DMR_FMT_BF16 = 3            /* dmr_qlinear_bf16_forward */
} dmr_format_t;
const char *dmr_qlinear_kernel_path(dmr_format_t format, int64_t M, int64_t K, int64_t N);

/* Release the host handle (NULL is allowed).  Device memory is the caller's and is untouched. */
void dmr_qlinear_destroy(dmr_qlinear_t *layer);

/* Shape of a handle (for bindings); any out pointer may be NULL. */
dmr_status_t dmr_qlinear_shape(const dmr_qlinear_t *layer, int64_t *K, int64_t *N, int32_t *g);

const char *dmr_status_string(dmr_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* DMR_QLINEAR_H */
