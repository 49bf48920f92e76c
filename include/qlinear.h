/* qlinear.h -- C ABI of the MI355X (gfx950) quantized linear layer.
 *
 * The layer is the W8A8 / W4A8 linear of the paper's unified low-bit inference
 * framework (Method, "Unified Low-Bit Inference Framework for INT8 and W4A8"):
 *
 *   xq, sx = per-token symmetric int8 quantization of x        (Eq. 1-2, n = 8;
 *            one scale per token: Preliminary, granularity paragraph)
 *   acc    = xq * wq^T  in exact integer arithmetic, int32 accumulators
 *   y      = fp16( acc * sx[m] * sw[n] + bias[n] )              (W8A8, per-output-channel sw)
 *   y      = fp16( sx[m] * sum_g acc_g * sw[n,g] + bias[n] )    (W4A8, one fp16 sw per group of
 *                                                                128 consecutive k per channel)
 *
 * Reading of Eq. 2 used throughout (symmetric setting of the paper's
 * Experimental Setup): scale = max|X| / (2^(n-1) - 1); codes = round-half-to-even,
 * clamped to +-127 (int8) or +-7 (int4); an all-zero token/channel/group stores
 * scale 1.  Activations use code = rne(x * (127/amax)) (one fp32 multiply per
 * element); weights, quantized offline, use code = rne(w / stored_scale).
 *
 * Conventions
 *   - every pointer is a DEVICE pointer unless its comment says "host"
 *   - the caller owns every buffer; the library never allocates, frees or
 *     synchronizes; all work is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and is asynchronous
 *   - every call returns a ql_status; arguments are validated on the host
 *     before anything is launched, so a failing call has no side effects;
 *     ql_last_error() gives a thread-local message for the last failure
 *   - x is fp16 [M,K] row-major with leading dimension ldx (elements);
 *     w is fp16 [N,K] row-major, row n = output channel n (so y = x w^T);
 *     y is fp16 [M,N] row-major with leading dimension ldy
 *   - alignment: x, y 16-byte aligned, ldx % 8 == 0, ldy % 8 == 0; every other
 *     device buffer 16-byte aligned (256-byte for workspaces and weight blobs)
 *   - limits: K % 64 == 0 (int8 weights) or K % 128 == 0 (int4, group = 128);
 *     K <= 131072 so that no int32 accumulator can overflow; padded sizes
 *     ceil32(M)*K and ceil32(N)*K below 2^31; ldx <= 2^27 (QL_ERR_SHAPE beyond)
 *   - M == 0 is a valid no-op
 *
 * "Kernel layout": weights and quantized activations are consumed by the GEMM
 * kernels as 32-row x 32-k tiles of 1024 bytes, each tile stored in the order a
 * 64-lane wavefront feeds the 32x32x32 int8 matrix instruction (lane = row % 32
 * + 32 * ((k % 32) / 16), 16 consecutive k per lane); tiles are ordered
 * row-block-major, then k-block.  Rows are padded to a multiple of 32.  int4
 * tiles hold two k-blocks per 1024 bytes with the nibbles pre-ordered for a
 * shift/mask unpack, followed in the same blob by two copies of the group scales
 * ([K/128][ceil32(N)] for the prefill kernels, [ceil32(N)/16][K/128][16] for the
 * decode kernels).  The layout is opaque to callers: build it with ql_quant_weight /
 * ql_quant_act_per_token / ql_act_repack and read it back with ql_export_canonical.
 */
#ifndef QLINEAR_H
#define QLINEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ql_status {
    QL_OK = 0,
    QL_ERR_NULL = 1,        /* a required pointer is NULL */
    QL_ERR_SHAPE = 2,       /* a size is negative, zero where it may not be, or violates a divisibility rule */
    QL_ERR_ALIGN = 3,       /* a pointer or leading dimension violates the alignment rules above */
    QL_ERR_UNSUPPORTED = 4, /* bits/group combination or size beyond the stated limits */
    QL_ERR_WORKSPACE = 5,   /* workspace smaller than ql_workspace_bytes reports */
    QL_ERR_HIP = 6          /* a HIP runtime call failed (message in ql_last_error) */
} ql_status;

/* Library version (major*10000 + minor*100 + patch). */
int ql_version(void);

/* Host pointer to a thread-local, NUL-terminated description of the last error on this thread. */
const char *ql_last_error(void);

/* Size queries (host outputs, any may be NULL).
 *   canonical: int8 [N,K] (bits 8) or packed nibbles [N,K/2] (bits 4)
 *   scales:    fp32 [N] (bits 8, group 0) or fp16 [N,K/group] (bits 4)
 *   kernel:    the opaque kernel-layout blob
 * bits/group: (8, 0) or (4, 128). */
int ql_weight_bytes(int N, int K, int bits, int group,
                    size_t *canonical, size_t *scales, size_t *kernel);

/* Bytes of the kernel-layout copy of xq for M tokens: ceil32(M) * K. */
int ql_act_kernel_bytes(int M, int K, size_t *bytes /* host */);

/* Workspace for ql_w8a8_linear / ql_w4a8_linear for these sizes: the quantized activations in kernel layout
 * and their scales (required), followed by scratch for split-K partial sums (offered when the output has too
 * few tiles to occupy the GPU: more than 32 tokens, long K; up to 64 MiB).  The *_gemm calls take scratch only:
 * their ws may be NULL or smaller, then K is not split.
 * A workspace serves one call at a time: calls that may run concurrently need workspaces of their own. */
int ql_workspace_bytes(int M, int N, int K, int bits, size_t *bytes /* host */);

/* Per-token dynamic int8 activation quantization (Eq. 1-2 with n = 8, one scale per token).
 *   x           fp16 [M,K], leading dimension ldx
 *   xq_rowmajor int8 [M,K] contiguous, may be NULL
 *   xq_kernel   int8 kernel layout (ql_act_kernel_bytes), may be NULL; at least one of the two
 *   sx          fp32 [M]: amax/127 (1 for an all-zero token)
 * Non-finite inputs give unspecified codes. */
int ql_quant_act_per_token(const void *x, int64_t ldx, int M, int K,
                           int8_t *xq_rowmajor, int8_t *xq_kernel, float *sx, void *stream);

/* RMSNorm fused in front of the per-token quantizer (the normalisation a decoder layer applies to the input of its
 * QKV and gate/up projections; textbook definition, the paper does not spell it out):
 *     h[m,k] = x[m,k] / sqrt(mean_k(x[m,:]^2) + eps) * gamma[k],   then Eq. 1-2 on h as in ql_quant_act_per_token.
 * Arithmetic: the sum of squares is accumulated in fp64 (within ~1e-13 relative of the exact sum) and then rounded to
 * fp32 -- the correctly rounded exact sum except when the exact sum lies that close to an fp32 rounding boundary
 * (bit-identical to the reference arithmetic almost surely, not by construction); every later step is one
 * correctly rounded fp32 operation (divide by K, add eps, square root, reciprocal, two multiplies per element).
 *   x      device, fp16 [M, ldx] (as ql_quant_act_per_token);  gamma  device, fp16 [K], 16-byte aligned
 *   eps    finite, >= 0 (a token with mean(x^2) + eps == 0 is the caller's error: its codes are unspecified)
 *   outputs as ql_quant_act_per_token.  Errors: as there; QL_ERR_SHAPE for a bad eps. */
int ql_quant_act_rmsnorm(const void *x, int64_t ldx, int M, int K, const void *gamma, float eps, int8_t *xq_rowmajor,
                         int8_t *xq_kernel, float *sx, void *stream);

/* SwiGLU fused in front of the per-token quantizer (the gated MLP of a decoder layer between its fused gate+up
 * projection and its down projection; textbook definition, the paper names no activation function):
 *     h[m,j] = silu(gate[m,j]) * up[m,j],  silu(g) = g / (1 + exp(-g)),   then Eq. 1-2 on h as in
 *     ql_quant_act_per_token (h stays fp32, it is never rounded to fp16).
 * Arithmetic: every step one correctly rounded fp32 operation, the exponential included: t = clamp(-g, +-80),
 * n = rint(t * log2 e), r = (t - n * 0.693359375) - n * (-2.12194440e-4), p = Horner polynomial of degree 7 in r with
 * the Taylor coefficients (multiply, then add), exp(t) = p * 2^n, h = (g * (1 / (1 + exp(t)))) * u.  The codes and
 * scales are therefore a function of the inputs alone.
 *   gate_up  device, fp16 [M, ld]: columns 0..F-1 the gate half, F..2F-1 the up half (the output of the fused
 *            projection), 16-byte aligned, ld >= 2F, ld % 8 == 0;  F % 64 == 0 (it is the K of the down projection)
 *   outputs as ql_quant_act_per_token with K = F.  Errors: as there. */
int ql_quant_act_swiglu(const void *gate_up, int64_t ld, int M, int F, int8_t *xq_rowmajor, int8_t *xq_kernel,
                        float *sx, void *stream);

/* Row-major int8 [M,K] -> kernel layout (lets a caller supply its own quantized activations). */
int ql_act_repack(const int8_t *xq_rowmajor, int M, int K, int8_t *xq_kernel, void *stream);

/* Offline weight quantization (Eq. 1-2; per-output-channel for int8, group-wise along K for int4)
 * and conversion to the kernel layout ("weight layout" of the paper's framework).
 *   w            fp16 [N,K] contiguous
 *   bits, group  (8, 0): int8 codes, fp32 scale per output channel
 *                (4, 128): int4 codes in [-7,7], two's-complement nibbles packed two per byte
 *                along K (even k in bits 3:0), fp16 scale per (channel, group of 128 k)
 *   wq_canonical may be NULL; scales may be NULL for bits 4 only (they are also kept in the blob)
 *   wq_kernel    kernel-layout blob, may be NULL */
int ql_quant_weight(const void *w, int N, int K, int bits, int group,
                    void *wq_canonical, void *scales, void *wq_kernel, void *stream);

/* Kernel-layout blob -> canonical codes (and, for bits 4, canonical fp16 group scales; `scales`
 * is ignored for bits 8 and may be NULL for bits 4).  Inverse of the repack in ql_quant_weight. */
int ql_export_canonical(const void *wq_kernel, int N, int K, int bits, int group,
                        void *wq_canonical, void *scales, void *stream);

/* W8A8 linear layer: activation quantization + int8 GEMM + dequantization epilogue.
 *   sw   fp32 [N] per-output-channel weight scales;  bias fp16 [N] or NULL
 *   ws   workspace of at least ql_workspace_bytes(M,N,K,8) bytes */
int ql_w8a8_linear(const void *x, int64_t ldx, int M, int K,
                   const void *wq_kernel, const float *sw, const void *bias, int N,
                   void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

/* ql_w8a8_linear for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arithmetic, kernels and results as ql_w8a8_linear; the workspace
 * (quantized activations, their scales, split-K partial sums) is a static device array of QL_STATIC_WS_BYTES that
 * belongs to the library -- every GPU the library runs on holds it until the process ends.  The call allocates
 * and frees nothing (the array's device address is looked up once per device, on the first call there).
 *   limit   ceil32(M)*K + 4*M (each rounded up to 256) <= QL_STATIC_WS_BYTES, else QL_ERR_WORKSPACE and nothing
 *           is launched (use ql_w8a8_linear with your own workspace)
 *   sharing every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (different
 *           streams or threads) race; the array keeps the last call's contents, nothing in it has to start at zero
 * Other arguments and errors as ql_w8a8_linear. */
#define QL_STATIC_WS_BYTES (64u << 20)
int ql_w8a8_linear_static(const void *x, int64_t ldx, int M, int K,
                          const void *wq_kernel, const float *sw, const void *bias, int N,
                          void *y, int64_t ldy, void *stream);

/* W4A8 linear layer (group scales live in the blob). */
int ql_w4a8_linear(const void *x, int64_t ldx, int M, int K,
                   const void *w4_kernel, int group, const void *bias, int N,
                   void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

/* GEMM + epilogue on already-quantized activations (xq in kernel layout, sx fp32 [M]). */
int ql_w8a8_gemm(const int8_t *xq_kernel, const float *sx, int M, int K,
                 const void *wq_kernel, const float *sw, const void *bias, int N,
                 void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream);
int ql_w4a8_gemm(const int8_t *xq_kernel, const float *sx, int M, int K,
                 const void *w4_kernel, int group, const void *bias, int N,
                 void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

/* Test hooks: the same main loops with the raw integer accumulators written out.
 *   acc      int32 [M,N] contiguous: sum over all k (W4A8: sum over groups of the group partials)
 *   partials (W4A8 only, may be NULL) int32 [nrows, K/group, N] for tokens row0 .. row0+nrows-1 */
int ql_w8a8_gemm_acc_i32(const int8_t *xq_kernel, int M, int K, const void *wq_kernel, int N,
                         int32_t *acc, void *ws, size_t ws_bytes, void *stream);
int ql_w4a8_gemm_acc_i32(const int8_t *xq_kernel, int M, int K, const void *w4_kernel, int group,
                         int N, int32_t *acc, int32_t *partials, int row0, int nrows,
                         void *ws, size_t ws_bytes, void *stream);

/* Kernel selection, for tests and tuning (a setting of the calling thread: it applies to the GEMM calls this
 * thread makes afterwards; other threads keep theirs, initially 0):
 *   0 = automatic (decode kernels for M <= 32; up to 1024 tokens whichever of the decode kernels, working on
 *       blocks of 64 or 32 tokens, and the prefill tile kernels has the lower estimated time; prefill tiles beyond)
 *   1 = automatic among the prefill tile kernels (2: the same, always as one launch -- see ql_plan.rest_channels),
 *   100 = automatic among the decode kernels (M <= 1024)
 *   other values pick one implementation: 4, 6, 11, 13, 15, 17, 19, 20, 23 prefill tile shapes (26, 35, 37, 39, 43: the
 *   shapes 6, 15, 17, 19, 23 on the 16x16x64 matrix instruction); 202..232 / 302..332
 *   split-K with that many splits on 128x128 / 256x256 tiles; 101..104, 106, 108 decode kernels with that many
 *   groups of 16 channels per workgroup; 111 sixteen wavefronts; 121 tokens never staged in LDS; 122 / 123 token
 *   blocks of 32 / 64; 130 quantizer never fused into the decode GEMM.  Unknown values -> QL_ERR_UNSUPPORTED. */
int ql_set_kernel_variant(int variant);

/* What the automatic choice launches for a GEMM of this shape, and the time estimate it goes by (host
 * arithmetic only: no GPU call, no allocation; usable for scheduling and for tests of the choice).
 *   scratch_bytes  the split-K scratch the GEMM would get: the ws_bytes of ql_*_gemm, or the part of the
 *                  workspace of ql_*_linear that lies behind ql_act_kernel_bytes + scales (0: none)
 *   plan           host struct, filled on QL_OK
 * Errors: the shape errors of the GEMMs; QL_ERR_NULL for plan == NULL; QL_ERR_SHAPE for M == 0. */
enum { QL_FAMILY_DECODE = 1, QL_FAMILY_TILE = 2 };
typedef struct ql_plan {
    int family;         /* QL_FAMILY_DECODE: weight-streaming kernels (every workgroup owns tile_channels channels and
                           the whole K for a block of tile_tokens tokens); QL_FAMILY_TILE: prefill tile kernels */
    int variant;        /* the ql_set_kernel_variant value closest to this choice (0: int4 tiles, which have one shape) */
    int tile_tokens;    /* tokens x channels one workgroup owns */
    int tile_channels;
    int splits;         /* workgroups sharing one tile's K range (1: unsplit; > 1 needs the scratch) */
    double est_us;      /* the estimate the choice was made by, microseconds (model fitted to measurements on MI355X) */
    int rest_channels;  /* > 0: the GEMM runs as two launches on disjoint channel ranges -- the first N - rest_channels
                           channels as described above (whole passes over the CUs), the last rest_channels channels with */
    int rest_variant;   /* this configuration; est_us covers both.  Results are bit-identical to one launch. */
} ql_plan;
int ql_plan_gemm(int M, int N, int K, int bits, int group, size_t scratch_bytes, ql_plan *plan);

/* ---- The two enhanced W4A8 configurations of the paper (usable with int8 weights as well) -------------------
 * SmoothQuant (Eq. 3): Y = (X S^-1)(S W), s_j = max|X_j|^alpha / max|W_j|^(1-alpha) per input channel j.
 * Hadamard (Eq. 4):    Y = (X H)(H^T W), H a normalized Hadamard matrix: here the natural-order (Sylvester)
 *   matrix, block diagonal with `hadamard_block` = a power of two in [16,4096] that divides K
 *   (ql_hadamard_block gives the largest), applied as the in-place butterfly in fp32 (stages 1,2,4,... in
 *   order, then one multiply by fp32(1/sqrt(block))).
 * Offline: calibrate -> scales -> ql_quant_weight_transformed.  Online: ql_quant_act_per_token_transformed,
 * then ql_w8a8_gemm / ql_w4a8_gemm on its output.  Transformed values are fp32 and are never rounded to
 * fp16; the quantizers are those of ql_quant_act_per_token / ql_quant_weight.  Limit: K <= 16384. */

/* Largest power of two dividing K, at most 4096 (host output). */
int ql_hadamard_block(int K, int *block /* host */);

/* Running max|X_j| over calibration batches: xmax[j] = max(xmax[j], max_m |x[m,j]|).  xmax is fp32 [K] and
 * must hold zeros (or earlier results) on entry. */
int ql_smooth_calibrate(const void *x, int64_t ldx, int M, int K, float *xmax, void *stream);

/* smooth[j] = xmax[j]^alpha / (max_n |w[n,j]|)^(1-alpha), 1 where either maximum is 0;
 * inv_smooth[j] = 1 / smooth[j].  w fp16 [N,K] contiguous, alpha in [0,1] (the paper uses 0.5). */
int ql_smooth_scales(const float *xmax, const void *w, int N, int K, float alpha, float *smooth,
                     float *inv_smooth, void *stream);

/* Per-token int8 quantization of x * diag(inv_smooth) (inv_smooth fp32 [K] or NULL) followed by the block
 * Hadamard transform (hadamard_block, 0 = none); outputs as ql_quant_act_per_token. */
int ql_quant_act_per_token_transformed(const void *x, int64_t ldx, int M, int K, const float *inv_smooth,
                                       int hadamard_block, int8_t *xq_rowmajor, int8_t *xq_kernel, float *sx,
                                       void *stream);

/* ql_quant_weight applied to w * diag(smooth) (smooth fp32 [K] or NULL), rows then Hadamard-transformed
 * (hadamard_block, 0 = none).  w32: fp32 [N,K] scratch that receives the transformed weights. */
int ql_quant_weight_transformed(const void *w, int N, int K, int bits, int group, const float *smooth,
                                int hadamard_block, float *w32, void *wq_canonical, void *scales,
                                void *wq_kernel, void *stream);

/* ---- The other quantizer forms of the paper's Preliminary section -------------------------------------------
 * range: QL_RANGE_SYMMETRIC  s = max|X| / (2^(n-1) - 1), codes in +-(2^(n-1) - 1)   (what every call above uses)
 *        QL_RANGE_EQ2        Eq. 2 as printed: s = 2 max|X| / (2^n - 1), codes in [-2^(n-1), 2^(n-1) - 1]
 * scope: QL_SCOPE_FINE       per token (activations), per output channel / per group (weights)
 *        QL_SCOPE_TENSOR     per-tensor granularity: one scale from the whole tensor's own maximum
 *        QL_SCOPE_STATIC     activations only: one calibrated scale supplied by the caller (Experimental
 *                            Setup: scales derived from calibration data); values beyond its range are clamped
 * Arithmetic: Eq. 1 as printed, code = round-half-even(X / s) with the stored fp32 scale (IEEE division; for
 * 4-bit weights s is first rounded to fp16), then the clamp; a zero scale is stored as 1.  Exception:
 * activations with (QL_RANGE_SYMMETRIC, QL_SCOPE_FINE) are ql_quant_act_per_token itself.  The outputs have
 * the layouts of ql_quant_act_per_token / ql_quant_weight -- sx holds one (possibly repeated) entry per token,
 * per-tensor weight scales are stored per channel / per group -- so the GEMM entry points take them unchanged.
 * With QL_RANGE_EQ2 both operands can hold -2^(n-1): K is limited to 131040 so that int32 sums cannot overflow.
 * scratch: 4 bytes of device memory, 4-byte aligned, required for QL_SCOPE_TENSOR only (else may be NULL). */
typedef enum ql_range { QL_RANGE_SYMMETRIC = 0, QL_RANGE_EQ2 = 1 } ql_range;
typedef enum ql_scope { QL_SCOPE_FINE = 0, QL_SCOPE_TENSOR = 1, QL_SCOPE_STATIC = 2 } ql_scope;

/* Calibration of a static activation scale: *scale = max(*scale, s(max|x|)) for the given range, so that
 * calling it on every calibration batch leaves the scale of the largest value seen.  scale: device fp32
 * that holds 0 (or an earlier result) on entry. */
int ql_act_scale_calibrate(const void *x, int64_t ldx, int M, int K, int range, float *scale, void *stream);

/* static_scale: device fp32 (QL_SCOPE_STATIC only). */
int ql_quant_act_opt(const void *x, int64_t ldx, int M, int K, int range, int scope, const float *static_scale,
                     int8_t *xq_rowmajor, int8_t *xq_kernel, float *sx, void *scratch, void *stream);

/* scope: QL_SCOPE_FINE or QL_SCOPE_TENSOR. */
int ql_quant_weight_opt(const void *w, int N, int K, int bits, int group, int range, int scope,
                        void *wq_canonical, void *scales, void *wq_kernel, void *scratch, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QLINEAR_H */
