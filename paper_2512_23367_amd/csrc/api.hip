// C ABI of libqlinear: argument validation and dispatch.  Declarations and the meaning of every
// argument are in include/qlinear.h; nothing here allocates, frees or synchronizes.
#include <stdarg.h>
#include <stdio.h>

#include "common.h"
#include <cmath>
#include <mutex>

namespace ql {

static thread_local char g_err[512] = "";
static thread_local int g_variant = 0;   // kernel selection of the calling thread (ql_set_kernel_variant)

int fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return status;
}

int check_hip(hipError_t e, const char *what)
{
    if (e == hipSuccess) return QL_OK;
    return fail(QL_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

namespace {

constexpr int MAX_K = 131072;          // 131072 * 127 * 127 < 2^31: no int32 accumulator can overflow
constexpr int DECODE_MAX_M = 32;           // the decode kernels are the automatic choice up to here,
constexpr int DECODE_BLOCKED_MAX_M = 1024; // and up to here (in blocks of 64 tokens) when their estimated time is lower

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_bits(int bits, int group)
{
    if (bits == 8 && group == 0) return QL_OK;
    if (bits == 4 && group == 128) return QL_OK;
    return fail(QL_ERR_UNSUPPORTED, "unsupported (bits, group) = (%d, %d): use (8, 0) or (4, 128)", bits, group);
}

int check_nk(int N, int K, int bits)
{
    if (N <= 0 || K <= 0) return fail(QL_ERR_SHAPE, "N and K must be positive (N=%d K=%d)", N, K);
    const int kmul = bits == 4 ? 128 : 64;
    if (K % kmul) return fail(QL_ERR_SHAPE, "K=%d must be a multiple of %d for %d-bit weights", K, kmul, bits);
    if (K > MAX_K) return fail(QL_ERR_UNSUPPORTED, "K=%d exceeds %d (int32 accumulator range)", K, MAX_K);
    if ((double)round_up(N, TILE_ROWS) * K >= 2147483648.0)
        return fail(QL_ERR_UNSUPPORTED, "ceil32(N)*K must be below 2^31 (N=%d K=%d)", N, K);
    return QL_OK;
}

int check_mk(int M, int K)
{
    if (M < 0) return fail(QL_ERR_SHAPE, "M must be non-negative (M=%d)", M);
    if (K <= 0 || K % 64) return fail(QL_ERR_SHAPE, "K=%d must be a positive multiple of 64", K);
    if (K > MAX_K) return fail(QL_ERR_UNSUPPORTED, "K=%d exceeds %d", K, MAX_K);
    if ((double)round_up(M, TILE_ROWS) * K >= 2147483648.0)
        return fail(QL_ERR_UNSUPPORTED, "ceil32(M)*K must be below 2^31 (M=%d K=%d)", M, K);
    return QL_OK;
}

struct WsLayout {
    size_t xq_off, sx_off, total;
};

WsLayout ws_layout(int M, int K)
{
    WsLayout l;
    l.xq_off = 0;
    l.sx_off = (act_kernel_bytes(M, K) + 255) & ~(size_t)255;
    l.total = l.sx_off + (((size_t)M * sizeof(float) + 255) & ~(size_t)255);
    return l;
}

// Split-K scratch worth offering for this shape: room for 8 partial copies of the (128-padded) output when the
// output has too few 128x128 tiles to occupy the GPU, nothing otherwise; at most 64 MiB.  The GEMMs use what
// they are given and fall back to unsplit kernels when it is less.
size_t splitk_scratch(int M, int N)
{
    const size_t mp = round_up(M, 128), np = round_up(N, 128);
    if (M <= DECODE_MAX_M || (mp / 128) * (np / 128) >= 192) return 0;
    const size_t want = 8 * mp * np * 4;
    return want < ((size_t)64 << 20) ? want : ((size_t)64 << 20);
}

int check_out(const void *y, int64_t ldy, int N)
{
    if (!y) return fail(QL_ERR_NULL, "y is NULL");
    if (!aligned(y, 16)) return fail(QL_ERR_ALIGN, "y must be 16-byte aligned");
    if (ldy < N || ldy % 8) return fail(QL_ERR_ALIGN, "ldy=%lld must be >= N and a multiple of 8", (long long)ldy);
    return QL_OK;
}

// automatic choice between the two kernel families
bool decode_family(const GemmArgs &a)
{
    return a.M <= DECODE_MAX_M || (a.M <= DECODE_BLOCKED_MAX_M && decode_estimate_us(a) < prefill_estimate_us(a));
}

int run_gemm(GemmArgs &a, hipStream_t st)
{
    if (a.M == 0) return QL_OK;
    int variant = g_variant;
    if (variant == 0 && decode_family(a)) variant = 100;
#ifdef QL_TRACE_DISPATCH
    fprintf(stderr, "dispatch M=%d N=%d K=%d bits=%d: decode %.1f us, tiles %.1f us -> %d\n", a.M, a.N, a.K, a.bits,
            decode_estimate_us(a), prefill_estimate_us(a), variant);
#endif
    if (variant >= 100 && variant < 200) {
        if (a.M > DECODE_BLOCKED_MAX_M)
            return fail(QL_ERR_UNSUPPORTED, "decode kernels take at most %d tokens (M=%d)", DECODE_BLOCKED_MAX_M, a.M);
        return launch_gemm_decode(a, variant, st);
    }
    return launch_gemm_prefill(a, variant == 1 ? 0 : variant, st);   // 1: automatic choice among the tile kernels
}

int gemm_common(const int8_t *xq, const float *sx, int M, int K, const void *wq, const float *sw, int bits,
                int group, const void *bias, int N, void *y, int64_t ldy, void *ws, size_t ws_bytes,
                hipStream_t st)
{
    QL_TRY(check_bits(bits, group));
    QL_TRY(check_mk(M, K));
    QL_TRY(check_nk(N, K, bits));
    if (!xq || !sx || !wq || (bits == 8 && !sw)) return fail(QL_ERR_NULL, "a required pointer is NULL");
    if (!aligned(xq, 256) || !aligned(wq, 256) || !aligned(sx, 16) || (sw && !aligned(sw, 16)) ||
        (bias && !aligned(bias, 16)))
        return fail(QL_ERR_ALIGN, "xq/wq need 256-byte, sx/sw/bias 16-byte alignment");
    QL_TRY(check_out(y, ldy, N));
    if (!ws || !aligned(ws, 16)) ws = nullptr, ws_bytes = 0;   // optional scratch (split-K partial sums)
    GemmArgs a = {};
    a.xq = xq;
    a.sx = sx;
    a.wq = wq;
    a.sw = sw;
    a.bias = static_cast<const __half *>(bias);
    a.y = static_cast<__half *>(y);
    a.ldy = ldy;
    a.M = M;
    a.N = N;
    a.K = K;
    a.bits = bits;
    a.group = group;
    a.ws = ws;
    a.ws_bytes = ws_bytes;
    return run_gemm(a, st);
}

int linear_common(const void *x, int64_t ldx, int M, int K, const void *wq, const float *sw, int bits, int group,
                  const void *bias, int N, void *y, int64_t ldy, void *ws, size_t ws_bytes, hipStream_t st)
{
    QL_TRY(check_bits(bits, group));
    QL_TRY(check_mk(M, K));
    QL_TRY(check_nk(N, K, bits));
    if (M == 0) return QL_OK;
    if (!x || !ws) return fail(QL_ERR_NULL, "x or ws is NULL");
    if (!aligned(x, 16) || ldx < K || ldx % 8)
        return fail(QL_ERR_ALIGN, "x must be 16-byte aligned, ldx >= K and a multiple of 8 (ldx=%lld)", (long long)ldx);
    if (!aligned(ws, 256)) return fail(QL_ERR_ALIGN, "ws must be 256-byte aligned");
    const WsLayout l = ws_layout(M, K);
    if (ws_bytes < l.total)
        return fail(QL_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", ws_bytes, l.total);
    int8_t *xq = static_cast<int8_t *>(ws) + l.xq_off;
    float *sx = reinterpret_cast<float *>(static_cast<char *>(ws) + l.sx_off);
    // validate the GEMM's arguments before the first launch so a failing call has no side effects
    if (!wq || (bits == 8 && !sw)) return fail(QL_ERR_NULL, "a required pointer is NULL");
    if (!aligned(wq, 256) || (sw && !aligned(sw, 16)) || (bias && !aligned(bias, 16)))
        return fail(QL_ERR_ALIGN, "wq needs 256-byte, sw/bias 16-byte alignment");
    QL_TRY(check_out(y, ldy, N));
    if (M <= DECODE_MAX_M && (g_variant == 0 || (g_variant >= 100 && g_variant < 200)) && decode_fuses_quant(M, K, g_variant)) {
        // few tokens: the decode GEMM quantizes them itself, one launch instead of two
        GemmArgs a = {};
        a.x = static_cast<const __half *>(x);
        a.ldx = ldx;
        a.wq = wq;
        a.sw = sw;
        a.bias = static_cast<const __half *>(bias);
        a.y = static_cast<__half *>(y);
        a.ldy = ldy;
        a.M = M;
        a.N = N;
        a.K = K;
        a.bits = bits;
        a.group = group;
        return launch_gemm_decode(a, g_variant == 0 ? 100 : g_variant, st);
    }
    QL_TRY(launch_act_quant(static_cast<const __half *>(x), ldx, M, K, nullptr, xq, sx, st));
    // what lies behind the quantized activations is scratch for the GEMM (split-K partial sums)
    return gemm_common(xq, sx, M, K, wq, sw, bits, group, bias, N, y, ldy, static_cast<char *>(ws) + l.total,
                       ws_bytes - l.total, st);
}

}  // namespace
}  // namespace ql

using namespace ql;

// ---- workspace of ql_w8a8_linear_static: device memory that belongs to the library, for callers that cannot allocate.
// Every GPU the library runs on holds its own copy of the array (at its own address) until the process ends.  In
// host code the array's name is only a handle for hipGetSymbolAddress: the device address is looked up once per
// device, with that device current, and only that address is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[QL_STATIC_WS_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};

int static_scratch(void **out)
{
    int dev = -1;
    QL_TRY(check_hip(hipGetDevice(&dev), "hipGetDevice"));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(QL_ERR_UNSUPPORTED, "device index %d beyond %d", dev, MAX_DEVICES - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        QL_TRY(check_hip(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(static workspace)"));
        if (!ptr) return fail(QL_ERR_HIP, "hipGetSymbolAddress returned a null address for the static workspace");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return QL_OK;
}
}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int ql_version(void) { return 100; }

const char *ql_last_error(void) { return g_err; }

int ql_set_kernel_variant(int variant)
{
    // 0 automatic; 1 automatic among the tile kernels; prefill tile configurations; decode configurations; split-K with 2..32 splits on 128x128 / 256x256 tiles
    static const int prefill[] = {4, 6, 11, 13, 15, 17, 19, 20, 23, 26, 35, 37, 39, 43};
    bool known = variant == 0 || variant == 1 || variant == 2 || (variant >= 100 && variant <= 104) || variant == 106 || variant == 108 || variant == 111 || (variant >= 121 && variant <= 123) || variant == 130 ||
                 (variant >= 202 && variant <= 232) || (variant >= 302 && variant <= 332);
    for (int v : prefill) known = known || variant == v;
    if (!known)
        return fail(QL_ERR_UNSUPPORTED, "unknown kernel variant %d", variant);
    g_variant = variant;
    return QL_OK;
}

int ql_plan_gemm(int M, int N, int K, int bits, int group, size_t scratch_bytes, ql_plan *plan)
{
    QL_TRY(check_bits(bits, group));
    QL_TRY(check_mk(M, K));
    QL_TRY(check_nk(N, K, bits));
    if (!plan) return fail(QL_ERR_NULL, "plan is NULL");
    if (M == 0) return fail(QL_ERR_SHAPE, "M must be at least 1");
    GemmArgs a = {};
    a.M = M, a.N = N, a.K = K, a.bits = bits, a.group = group;
    a.ws = scratch_bytes ? reinterpret_cast<void *>(256) : nullptr;   // only tested against NULL while planning
    a.ws_bytes = scratch_bytes;
    *plan = ql_plan{};
    if (decode_family(a)) {
        int block = 0, c = 0;
        decode_plan(a, &block, &c);
        plan->family = QL_FAMILY_DECODE;
        plan->variant = 100 + c;
        plan->tile_tokens = block;
        plan->tile_channels = 16 * c;
        plan->splits = 1;
        plan->est_us = decode_estimate_us(a);
    } else {
        plan->family = QL_FAMILY_TILE;
        prefill_plan(a, &plan->variant, &plan->tile_tokens, &plan->tile_channels, &plan->splits, &plan->rest_channels,
                     &plan->rest_variant);
        plan->est_us = prefill_estimate_us(a);
    }
    return QL_OK;
}

int ql_weight_bytes(int N, int K, int bits, int group, size_t *canonical, size_t *scales, size_t *kernel)
{
    QL_TRY(check_bits(bits, group));
    QL_TRY(check_nk(N, K, bits));
    if (bits == 8) {
        if (canonical) *canonical = (size_t)N * K;
        if (scales) *scales = (size_t)N * sizeof(float);
        if (kernel) *kernel = w8_kernel_bytes(N, K);
    } else {
        if (canonical) *canonical = (size_t)N * K / 2;
        if (scales) *scales = (size_t)N * (K / group) * sizeof(__half);
        if (kernel) *kernel = w4_kernel_bytes(N, K, group);
    }
    return QL_OK;
}

int ql_act_kernel_bytes(int M, int K, size_t *bytes)
{
    QL_TRY(check_mk(M, K));
    if (!bytes) return fail(QL_ERR_NULL, "bytes is NULL");
    *bytes = act_kernel_bytes(M, K);
    return QL_OK;
}

int ql_workspace_bytes(int M, int N, int K, int bits, size_t *bytes)
{
    if (bits != 8 && bits != 4) return fail(QL_ERR_UNSUPPORTED, "bits must be 8 or 4");
    QL_TRY(check_mk(M, K));
    QL_TRY(check_nk(N, K, bits));
    if (!bytes) return fail(QL_ERR_NULL, "bytes is NULL");
    *bytes = ws_layout(M, K).total + splitk_scratch(M, N);
    return QL_OK;
}

int ql_quant_act_per_token(const void *x, int64_t ldx, int M, int K, int8_t *xq_rowmajor, int8_t *xq_kernel,
                           float *sx, void *stream)
{
    QL_TRY(check_mk(M, K));
    if (M == 0) return QL_OK;
    if (!x || !sx || (!xq_rowmajor && !xq_kernel)) return fail(QL_ERR_NULL, "x, sx and one of the outputs are required");
    if (!aligned(x, 16) || ldx < K || ldx % 8)
        return fail(QL_ERR_ALIGN, "x must be 16-byte aligned, ldx >= K and a multiple of 8 (ldx=%lld)", (long long)ldx);
    if ((xq_rowmajor && !aligned(xq_rowmajor, 16)) || (xq_kernel && !aligned(xq_kernel, 256)) || !aligned(sx, 4))
        return fail(QL_ERR_ALIGN, "xq_rowmajor needs 16-byte, xq_kernel 256-byte alignment");
    return launch_act_quant(static_cast<const __half *>(x), ldx, M, K, xq_rowmajor, xq_kernel, sx,
                            static_cast<hipStream_t>(stream));
}

int ql_quant_act_rmsnorm(const void *x, int64_t ldx, int M, int K, const void *gamma, float eps, int8_t *xq_rowmajor,
                         int8_t *xq_kernel, float *sx, void *stream)
{
    QL_TRY(check_mk(M, K));
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return fail(QL_ERR_SHAPE, "eps must be finite and non-negative");
    if (M == 0) return QL_OK;
    if (!x || !gamma || !sx || (!xq_rowmajor && !xq_kernel))
        return fail(QL_ERR_NULL, "x, gamma, sx and one of the outputs are required");
    if (!aligned(x, 16) || ldx < K || ldx % 8)
        return fail(QL_ERR_ALIGN, "x must be 16-byte aligned, ldx >= K and a multiple of 8 (ldx=%lld)", (long long)ldx);
    if (!aligned(gamma, 16)) return fail(QL_ERR_ALIGN, "gamma must be 16-byte aligned");
    if ((xq_rowmajor && !aligned(xq_rowmajor, 16)) || (xq_kernel && !aligned(xq_kernel, 256)) || !aligned(sx, 4))
        return fail(QL_ERR_ALIGN, "xq_rowmajor needs 16-byte, xq_kernel 256-byte alignment");
    return launch_act_quant_rmsnorm(static_cast<const __half *>(x), ldx, M, K, static_cast<const __half *>(gamma), eps,
                                    xq_rowmajor, xq_kernel, sx, static_cast<hipStream_t>(stream));
}

int ql_quant_act_swiglu(const void *gate_up, int64_t ld, int M, int F, int8_t *xq_rowmajor, int8_t *xq_kernel, float *sx,
                        void *stream)
{
    QL_TRY(check_mk(M, F));
    if (M == 0) return QL_OK;
    if (!gate_up || !sx || (!xq_rowmajor && !xq_kernel))
        return fail(QL_ERR_NULL, "gate_up, sx and one of the outputs are required");
    if (!aligned(gate_up, 16) || ld < 2 * (int64_t)F || ld % 8)
        return fail(QL_ERR_ALIGN, "gate_up must be 16-byte aligned, ld >= 2F and a multiple of 8 (ld=%lld)", (long long)ld);
    if ((xq_rowmajor && !aligned(xq_rowmajor, 16)) || (xq_kernel && !aligned(xq_kernel, 256)) || !aligned(sx, 4))
        return fail(QL_ERR_ALIGN, "xq_rowmajor needs 16-byte, xq_kernel 256-byte alignment");
    return launch_act_quant_swiglu(static_cast<const __half *>(gate_up), ld, M, F, xq_rowmajor, xq_kernel, sx,
                                   static_cast<hipStream_t>(stream));
}

int ql_act_repack(const int8_t *xq_rowmajor, int M, int K, int8_t *xq_kernel, void *stream)
{
    QL_TRY(check_mk(M, K));
    if (M == 0) return QL_OK;
    if (!xq_rowmajor || !xq_kernel) return fail(QL_ERR_NULL, "a required pointer is NULL");
    if (!aligned(xq_rowmajor, 16) || !aligned(xq_kernel, 256))
        return fail(QL_ERR_ALIGN, "xq_rowmajor needs 16-byte, xq_kernel 256-byte alignment");
    return launch_act_repack(xq_rowmajor, M, K, xq_kernel, static_cast<hipStream_t>(stream));
}

int ql_quant_weight(const void *w, int N, int K, int bits, int group, void *wq_canonical, void *scales,
                    void *wq_kernel, void *stream)
{
    QL_TRY(check_bits(bits, group));
    QL_TRY(check_nk(N, K, bits));
    if (!w) return fail(QL_ERR_NULL, "w is NULL");
    if (bits == 8 && !scales) return fail(QL_ERR_NULL, "scales is required for int8 weights");
    if (!wq_canonical && !wq_kernel && !scales) return fail(QL_ERR_NULL, "no output requested");
    if (!aligned(w, 16) || (wq_canonical && !aligned(wq_canonical, 16)) || (scales && !aligned(scales, 16)) ||
        (wq_kernel && !aligned(wq_kernel, 256)))
        return fail(QL_ERR_ALIGN, "w/wq_canonical/scales need 16-byte, wq_kernel 256-byte alignment");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bits == 8)
        return launch_weight_quant8(static_cast<const __half *>(w), N, K, static_cast<int8_t *>(wq_canonical),
                                    static_cast<float *>(scales), static_cast<int8_t *>(wq_kernel), st);
    return launch_weight_quant4(static_cast<const __half *>(w), N, K, group, static_cast<uint8_t *>(wq_canonical),
                                static_cast<__half *>(scales), static_cast<uint8_t *>(wq_kernel), st);
}

// ---- the other quantizer forms of the Preliminary section (Eq. 2 as printed, per-tensor, static scale)
static int check_options(int range, int scope, int K, bool weights)
{
    if (range != QL_RANGE_SYMMETRIC && range != QL_RANGE_EQ2) return fail(QL_ERR_UNSUPPORTED, "unknown range %d", range);
    if (scope != QL_SCOPE_FINE && scope != QL_SCOPE_TENSOR && !(scope == QL_SCOPE_STATIC && !weights))
        return fail(QL_ERR_UNSUPPORTED, "scope %d is not available for %s", scope, weights ? "weights" : "activations");
    if (range == QL_RANGE_EQ2 && K > 131040)
        return fail(QL_ERR_UNSUPPORTED, "K=%d: with codes of -128 on both sides int32 sums are safe up to K = 131040", K);
    return QL_OK;
}

int ql_act_scale_calibrate(const void *x, int64_t ldx, int M, int K, int range, float *scale, void *stream)
{
    QL_TRY(check_mk(M, K));
    QL_TRY(check_options(range, QL_SCOPE_STATIC, K, false));
    if (M == 0) return QL_OK;
    if (!x || !scale) return fail(QL_ERR_NULL, "x and scale are required");
    if (!aligned(x, 16) || ldx < K || ldx % 8 || !aligned(scale, 4))
        return fail(QL_ERR_ALIGN, "x must be 16-byte aligned, ldx >= K and a multiple of 8 (ldx=%lld)", (long long)ldx);
    return launch_act_calibrate(static_cast<const __half *>(x), ldx, M, K, range, scale, static_cast<hipStream_t>(stream));
}

int ql_quant_act_opt(const void *x, int64_t ldx, int M, int K, int range, int scope, const float *static_scale,
                     int8_t *xq_rowmajor, int8_t *xq_kernel, float *sx, void *scratch, void *stream)
{
    QL_TRY(check_options(range, scope, K, false));
    if (range == QL_RANGE_SYMMETRIC && scope == QL_SCOPE_FINE)
        return ql_quant_act_per_token(x, ldx, M, K, xq_rowmajor, xq_kernel, sx, stream);
    QL_TRY(check_mk(M, K));
    if (M == 0) return QL_OK;
    if (!x || !sx || (!xq_rowmajor && !xq_kernel)) return fail(QL_ERR_NULL, "x, sx and one of the outputs are required");
    if (scope == QL_SCOPE_STATIC && !static_scale) return fail(QL_ERR_NULL, "static_scale is required for QL_SCOPE_STATIC");
    if (scope == QL_SCOPE_TENSOR && !scratch) return fail(QL_ERR_NULL, "scratch is required for QL_SCOPE_TENSOR");
    if (!aligned(x, 16) || ldx < K || ldx % 8)
        return fail(QL_ERR_ALIGN, "x must be 16-byte aligned, ldx >= K and a multiple of 8 (ldx=%lld)", (long long)ldx);
    if ((xq_rowmajor && !aligned(xq_rowmajor, 16)) || (xq_kernel && !aligned(xq_kernel, 256)) || !aligned(sx, 4) ||
        (static_scale && !aligned(static_scale, 4)) || (scratch && !aligned(scratch, 4)))
        return fail(QL_ERR_ALIGN, "xq_rowmajor needs 16-byte, xq_kernel 256-byte, sx/static_scale/scratch 4-byte alignment");
    return launch_act_quant_opt(static_cast<const __half *>(x), ldx, M, K, range, scope, static_scale,
                                static_cast<unsigned *>(scratch), xq_rowmajor, xq_kernel, sx,
                                static_cast<hipStream_t>(stream));
}

int ql_quant_weight_opt(const void *w, int N, int K, int bits, int group, int range, int scope, void *wq_canonical,
                        void *scales, void *wq_kernel, void *scratch, void *stream)
{
    QL_TRY(check_bits(bits, group));
    QL_TRY(check_nk(N, K, bits));
    QL_TRY(check_options(range, scope, K, true));
    if (!w) return fail(QL_ERR_NULL, "w is NULL");
    if (bits == 8 && !scales) return fail(QL_ERR_NULL, "scales is required for int8 weights");
    if (!wq_canonical && !wq_kernel && !scales) return fail(QL_ERR_NULL, "no output requested");
    if (scope == QL_SCOPE_TENSOR && !scratch) return fail(QL_ERR_NULL, "scratch is required for QL_SCOPE_TENSOR");
    if (!aligned(w, 16) || (wq_canonical && !aligned(wq_canonical, 16)) || (scales && !aligned(scales, 16)) ||
        (wq_kernel && !aligned(wq_kernel, 256)) || (scratch && !aligned(scratch, 4)))
        return fail(QL_ERR_ALIGN, "w/wq_canonical/scales need 16-byte, wq_kernel 256-byte, scratch 4-byte alignment");
    return launch_weight_quant_opt(static_cast<const __half *>(w), N, K, bits, group, range, scope == QL_SCOPE_TENSOR,
                                   static_cast<unsigned *>(scratch), wq_canonical, scales, wq_kernel,
                                   static_cast<hipStream_t>(stream));
}

// ---- SmoothQuant / Hadamard variants (Eq. 3-4)
static int check_transform(int K, int hadamard_block)
{
    if (K > 16384) return fail(QL_ERR_UNSUPPORTED, "transforms: K=%d above 16384", K);
    if (hadamard_block != 0) {
        const bool pow2 = (hadamard_block & (hadamard_block - 1)) == 0;
        if (!pow2 || hadamard_block < 16 || hadamard_block > 4096 || K % hadamard_block)
            return fail(QL_ERR_SHAPE, "hadamard_block=%d must be 0 or a power of two in [16,4096] that divides K=%d",
                        hadamard_block, K);
    }
    return QL_OK;
}

int ql_hadamard_block(int K, int *block)
{
    if (K <= 0 || K % 64) return fail(QL_ERR_SHAPE, "K=%d must be a positive multiple of 64", K);
    if (!block) return fail(QL_ERR_NULL, "block is NULL");
    *block = hadamard_block_of(K);
    return QL_OK;
}

int ql_smooth_calibrate(const void *x, int64_t ldx, int M, int K, float *xmax, void *stream)
{
    QL_TRY(check_mk(M, K));
    if (M == 0) return QL_OK;
    if (!x || !xmax) return fail(QL_ERR_NULL, "x or xmax is NULL");
    if (!aligned(x, 16) || ldx < K || ldx % 8 || !aligned(xmax, 16))
        return fail(QL_ERR_ALIGN, "x, xmax 16-byte aligned, ldx >= K and a multiple of 8");
    return launch_channel_absmax(static_cast<const __half *>(x), ldx, M, K, xmax, static_cast<hipStream_t>(stream));
}

int ql_smooth_scales(const float *xmax, const void *w, int N, int K, float alpha, float *smooth, float *inv_smooth,
                     void *stream)
{
    QL_TRY(check_nk(N, K, 8));
    if (!xmax || !w || !smooth || !inv_smooth) return fail(QL_ERR_NULL, "a required pointer is NULL");
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return fail(QL_ERR_SHAPE, "alpha must lie in [0,1]");
    if (!aligned(xmax, 16) || !aligned(w, 16) || !aligned(smooth, 16) || !aligned(inv_smooth, 16))
        return fail(QL_ERR_ALIGN, "xmax, w, smooth, inv_smooth need 16-byte alignment");
    return launch_smooth_scales(xmax, static_cast<const __half *>(w), N, K, alpha, smooth, inv_smooth,
                                static_cast<hipStream_t>(stream));
}

int ql_quant_act_per_token_transformed(const void *x, int64_t ldx, int M, int K, const float *inv_smooth,
                                       int hadamard_block, int8_t *xq_rowmajor, int8_t *xq_kernel, float *sx,
                                       void *stream)
{
    QL_TRY(check_mk(M, K));
    if (hadamard_block != 0) QL_TRY(check_transform(K, hadamard_block));
    if (M == 0) return QL_OK;
    if (!x || !sx || (!xq_rowmajor && !xq_kernel)) return fail(QL_ERR_NULL, "a required pointer is NULL");
    if (!aligned(x, 16) || ldx < K || ldx % 8)
        return fail(QL_ERR_ALIGN, "x must be 16-byte aligned, ldx >= K and a multiple of 8 (ldx=%lld)", (long long)ldx);
    if ((xq_rowmajor && !aligned(xq_rowmajor, 16)) || (xq_kernel && !aligned(xq_kernel, 256)) || !aligned(sx, 4) ||
        (inv_smooth && !aligned(inv_smooth, 16)))
        return fail(QL_ERR_ALIGN, "xq_rowmajor/inv_smooth need 16-byte, xq_kernel 256-byte alignment");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hadamard_block == 0) {   // per-channel multiply only: the ordinary quantizer's layouts and any K
        if (!inv_smooth) return launch_act_quant(static_cast<const __half *>(x), ldx, M, K, xq_rowmajor, xq_kernel, sx, st);
        return launch_act_quant_smooth(static_cast<const __half *>(x), ldx, M, K, inv_smooth, xq_rowmajor, xq_kernel, sx, st);
    }
    return launch_act_quant_transform(static_cast<const __half *>(x), ldx, M, K, inv_smooth, hadamard_block, xq_rowmajor,
                                      xq_kernel, sx, st);
}

int ql_quant_weight_transformed(const void *w, int N, int K, int bits, int group, const float *smooth,
                                int hadamard_block, float *w32, void *wq_canonical, void *scales, void *wq_kernel,
                                void *stream)
{
    QL_TRY(check_bits(bits, group));
    QL_TRY(check_nk(N, K, bits));
    QL_TRY(check_transform(K, hadamard_block));
    if (!w || !w32) return fail(QL_ERR_NULL, "w or w32 is NULL");
    if (bits == 8 && !scales) return fail(QL_ERR_NULL, "scales is required for int8 weights");
    if (!wq_canonical && !wq_kernel && !scales) return fail(QL_ERR_NULL, "no output requested");
    if (!aligned(w, 16) || !aligned(w32, 16) || (smooth && !aligned(smooth, 16)) ||
        (wq_canonical && !aligned(wq_canonical, 16)) || (scales && !aligned(scales, 16)) ||
        (wq_kernel && !aligned(wq_kernel, 256)))
        return fail(QL_ERR_ALIGN, "w/w32/smooth/wq_canonical/scales need 16-byte, wq_kernel 256-byte alignment");
    hipStream_t st = static_cast<hipStream_t>(stream);
    QL_TRY(launch_weight_transform(static_cast<const __half *>(w), N, K, smooth, hadamard_block, w32, st));
    if (bits == 8)
        return launch_weight_quant8_f32(w32, N, K, static_cast<int8_t *>(wq_canonical), static_cast<float *>(scales),
                                        static_cast<int8_t *>(wq_kernel), st);
    return launch_weight_quant4_f32(w32, N, K, group, static_cast<uint8_t *>(wq_canonical),
                                    static_cast<__half *>(scales), static_cast<uint8_t *>(wq_kernel), st);
}

int ql_export_canonical(const void *wq_kernel, int N, int K, int bits, int group, void *wq_canonical,
                        void *scales, void *stream)
{
    QL_TRY(check_bits(bits, group));
    QL_TRY(check_nk(N, K, bits));
    if (!wq_kernel || (!wq_canonical && !(bits == 4 && scales))) return fail(QL_ERR_NULL, "a required pointer is NULL");
    if (!aligned(wq_kernel, 256) || (wq_canonical && !aligned(wq_canonical, 16)) || (scales && !aligned(scales, 2)))
        return fail(QL_ERR_ALIGN, "wq_kernel needs 256-byte, wq_canonical 16-byte alignment");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bits == 8)
        return launch_export8(static_cast<const int8_t *>(wq_kernel), N, K, static_cast<int8_t *>(wq_canonical), st);
    return launch_export4(static_cast<const uint8_t *>(wq_kernel), N, K, group, static_cast<uint8_t *>(wq_canonical),
                          static_cast<__half *>(scales), st);
}

int ql_w8a8_linear(const void *x, int64_t ldx, int M, int K, const void *wq_kernel, const float *sw,
                   const void *bias, int N, void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream)
{
    return linear_common(x, ldx, M, K, wq_kernel, sw, 8, 0, bias, N, y, ldy, ws, ws_bytes,
                         static_cast<hipStream_t>(stream));
}

int ql_w4a8_linear(const void *x, int64_t ldx, int M, int K, const void *w4_kernel, int group, const void *bias,
                   int N, void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream)
{
    return linear_common(x, ldx, M, K, w4_kernel, nullptr, 4, group, bias, N, y, ldy, ws, ws_bytes,
                         static_cast<hipStream_t>(stream));
}

int ql_w8a8_linear_static(const void *x, int64_t ldx, int M, int K, const void *wq_kernel, const float *sw,
                          const void *bias, int N, void *y, int64_t ldy, void *stream)
{
    QL_TRY(check_mk(M, K));
    QL_TRY(check_nk(N, K, 8));
    if (M == 0) return QL_OK;
    // quantized activations + their scales must fit; split-K scratch is taken as far as the rest reaches
    const size_t need = ws_layout(M, K).total;
    if (need > (size_t)QL_STATIC_WS_BYTES)
        return fail(QL_ERR_WORKSPACE,
                    "ql_w8a8_linear_static: M=%d K=%d needs %zu bytes of workspace, the library's own holds %zu "
                    "(use ql_w8a8_linear with a caller-allocated workspace)", M, K, need, (size_t)QL_STATIC_WS_BYTES);
    void *ws = nullptr;
    QL_TRY(static_scratch(&ws));
    size_t bytes = need + splitk_scratch(M, N);
    if (bytes > (size_t)QL_STATIC_WS_BYTES) bytes = QL_STATIC_WS_BYTES;
    return linear_common(x, ldx, M, K, wq_kernel, sw, 8, 0, bias, N, y, ldy, ws, bytes, static_cast<hipStream_t>(stream));
}

int ql_w8a8_gemm(const int8_t *xq_kernel, const float *sx, int M, int K, const void *wq_kernel, const float *sw,
                 const void *bias, int N, void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream)
{
    return gemm_common(xq_kernel, sx, M, K, wq_kernel, sw, 8, 0, bias, N, y, ldy, ws, ws_bytes,
                       static_cast<hipStream_t>(stream));
}

int ql_w4a8_gemm(const int8_t *xq_kernel, const float *sx, int M, int K, const void *w4_kernel, int group,
                 const void *bias, int N, void *y, int64_t ldy, void *ws, size_t ws_bytes, void *stream)
{
    return gemm_common(xq_kernel, sx, M, K, w4_kernel, nullptr, 4, group, bias, N, y, ldy, ws, ws_bytes,
                       static_cast<hipStream_t>(stream));
}

static int acc_common(const int8_t *xq, int M, int K, const void *wq, int bits, int group, int N, int32_t *acc,
                      int32_t *partials, int row0, int nrows, void *ws, size_t ws_bytes, hipStream_t st)
{
    QL_TRY(check_bits(bits, group));
    QL_TRY(check_mk(M, K));
    QL_TRY(check_nk(N, K, bits));
    if (!xq || !wq || !acc) return fail(QL_ERR_NULL, "a required pointer is NULL");
    if (!aligned(xq, 256) || !aligned(wq, 256) || !aligned(acc, 16) || (partials && !aligned(partials, 4)))
        return fail(QL_ERR_ALIGN, "xq/wq need 256-byte, acc 16-byte alignment");
    if (partials && (row0 < 0 || nrows < 0 || row0 + nrows > M))
        return fail(QL_ERR_SHAPE, "partials row range [%d, %d) outside [0, %d)", row0, row0 + nrows, M);
    GemmArgs a = {};
    a.xq = xq;
    a.wq = wq;
    a.acc = acc;
    a.partials = partials;
    a.row0 = row0;
    a.nrows = partials ? nrows : 0;
    a.M = M;
    a.N = N;
    a.K = K;
    a.bits = bits;
    a.group = group;
    if (ws && aligned(ws, 16)) a.ws = ws, a.ws_bytes = ws_bytes;
    return run_gemm(a, st);
}

int ql_w8a8_gemm_acc_i32(const int8_t *xq_kernel, int M, int K, const void *wq_kernel, int N, int32_t *acc,
                         void *ws, size_t ws_bytes, void *stream)
{
    return acc_common(xq_kernel, M, K, wq_kernel, 8, 0, N, acc, nullptr, 0, 0, ws, ws_bytes,
                      static_cast<hipStream_t>(stream));
}

int ql_w4a8_gemm_acc_i32(const int8_t *xq_kernel, int M, int K, const void *w4_kernel, int group, int N,
                         int32_t *acc, int32_t *partials, int row0, int nrows, void *ws, size_t ws_bytes,
                         void *stream)
{
    return acc_common(xq_kernel, M, K, w4_kernel, 4, group, N, acc, partials, row0, nrows, ws, ws_bytes,
                      static_cast<hipStream_t>(stream));
}

}  // extern "C"
#pragma GCC visibility pop
