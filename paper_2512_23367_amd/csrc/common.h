// Internal helpers shared by the HIP sources of libqlinear (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stddef.h>
#include <stdint.h>

#include "qlinear.h"

namespace ql {

// ---- error reporting -------------------------------------------------------------------------
int fail(int status, const char *fmt, ...);   // records the message, returns status
int check_hip(hipError_t e, const char *what);

#define QL_TRY(expr)                          \
    do {                                      \
        int _s = (expr);                      \
        if (_s != QL_OK) return _s;           \
    } while (0)

// ---- kernel layout ---------------------------------------------------------------------------
// A tile is 32 rows x 32 k of int8 = 1024 bytes, stored in the order a wavefront feeds the
// 32x32x32 int8 matrix instruction: lane = row % 32 + 32 * ((k % 32) / 16), 16 bytes per lane.
// Tiles are ordered row-block-major, then k-block.
constexpr int TILE_ROWS = 32;
constexpr int TILE_K = 32;
constexpr int TILE_BYTES = 1024;

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ inline int round_up(int a, int b) { return ceil_div(a, b) * b; }

// Byte offset of int8 element (row, k) in the kernel layout of a [rows, K] matrix.
__host__ __device__ inline size_t tile_offset_i8(int row, int k, int K)
{
    const size_t tile = (size_t)(row / TILE_ROWS) * (K / TILE_K) + (k / TILE_K);
    const int lane = (row % TILE_ROWS) + 32 * ((k % TILE_K) / 16);
    return tile * TILE_BYTES + lane * 16 + (k % 16);
}

// int4 kernel layout: 1024-byte tile pairs covering 32 rows x 64 k.  A lane's 16 bytes hold its
// 16 k of the even k-block (words 0,1) and of the odd k-block (words 2,3).  Within a word the
// eight nibbles p0..p7 (p0 = bits 3:0) hold k-offsets [0,4,1,5,2,6,3,7] so that
//   (word << 4) & 0xF0F0F0F0 -> bytes k0..k3 (each code * 16),  word & 0xF0F0F0F0 -> bytes k4..k7.
__host__ __device__ inline size_t tile_offset_w4_word(int row, int k, int K)   // byte offset of the 32-bit word
{
    const size_t pair = (size_t)(row / TILE_ROWS) * (K / 64) + (k / 64);
    const int kb = (k % 64) / 32;
    const int lane = (row % TILE_ROWS) + 32 * ((k % 32) / 16);
    const int word = 2 * kb + ((k % 16) / 8);
    return pair * TILE_BYTES + lane * 16 + word * 4;
}
__host__ __device__ inline int w4_nibble_pos(int k)    // nibble index 0..7 inside the word
{
    const int j8 = k % 8;
    return 2 * (j8 % 4) + (j8 / 4);
}

inline size_t act_kernel_bytes(int M, int K) { return (size_t)round_up(M, TILE_ROWS) * K; }
inline size_t w8_kernel_bytes(int N, int K) { return (size_t)round_up(N, TILE_ROWS) * K; }
inline size_t w4_codes_bytes(int N, int K) { return (size_t)round_up(N, TILE_ROWS) * K / 2; }
inline size_t w4_scales_offset(int N, int K) { return (w4_codes_bytes(N, K) + 255) & ~(size_t)255; }
// The int4 blob holds the group scales twice: [K/group][ceil32(N)] (a prefill tile's 128 channels of one
// group are contiguous) and, for the decode kernels, [ceil32(N)/16][K/group][16] (everything one
// workgroup's 16 channels need is contiguous).
inline size_t w4_scales_bytes(int N, int K, int group)
{
    return (((size_t)(K / group) * round_up(N, TILE_ROWS) * sizeof(__half)) + 255) & ~(size_t)255;
}
inline size_t w4_scales_dec_offset(int N, int K, int group) { return w4_scales_offset(N, K) + w4_scales_bytes(N, K, group); }
inline size_t w4_kernel_bytes(int N, int K, int group)
{
    return w4_scales_offset(N, K) + 2 * w4_scales_bytes(N, K, group);
}

// ---- launchers implemented in the .hip files ----------------------------------------------------
int launch_act_quant(const __half *x, int64_t ldx, int M, int K, int8_t *xq_rm, int8_t *xq_kl,
                     float *sx, hipStream_t st);
int launch_act_quant_smooth(const __half *x, int64_t ldx, int M, int K, const float *inv_smooth, int8_t *xq_rm,
                            int8_t *xq_kl, float *sx, hipStream_t st);
int launch_act_quant_rmsnorm(const __half *x, int64_t ldx, int M, int K, const __half *gamma, float eps, int8_t *xq_rm,
                             int8_t *xq_kl, float *sx, hipStream_t st);
int launch_act_quant_swiglu(const __half *gate_up, int64_t ld, int M, int K, int8_t *xq_rm, int8_t *xq_kl, float *sx,
                            hipStream_t st);
int launch_act_repack(const int8_t *xq_rm, int M, int K, int8_t *xq_kl, hipStream_t st);
int launch_weight_quant8(const __half *w, int N, int K, int8_t *canon, float *scales, int8_t *kl,
                         hipStream_t st);
int launch_weight_quant4(const __half *w, int N, int K, int group, uint8_t *canon, __half *scales,
                         uint8_t *kl, hipStream_t st);
int launch_weight_quant8_f32(const float *w, int N, int K, int8_t *canon, float *scales, int8_t *kl,
                             hipStream_t st);
int launch_weight_quant4_f32(const float *w, int N, int K, int group, uint8_t *canon, __half *scales,
                             uint8_t *kl, hipStream_t st);
int launch_act_quant_opt(const __half *x, int64_t ldx, int M, int K, int range, int scope,
                         const float *static_scale, unsigned *amax_scratch, int8_t *xq_rm, int8_t *xq_kl, float *sx,
                         hipStream_t st);
int launch_act_calibrate(const __half *x, int64_t ldx, int M, int K, int range, float *scale, hipStream_t st);
int launch_weight_quant_opt(const __half *w, int N, int K, int bits, int group, int range, bool per_tensor,
                            unsigned *amax_scratch, void *canon, void *scales, void *kl, hipStream_t st);
int hadamard_block_of(int K);
int launch_act_quant_transform(const __half *x, int64_t ldx, int M, int K, const float *inv_smooth, int hblock,
                               int8_t *xq_rm, int8_t *xq_kl, float *sx, hipStream_t st);
int launch_weight_transform(const __half *w, int N, int K, const float *smooth, int hblock, float *out,
                            hipStream_t st);
int launch_channel_absmax(const __half *x, int64_t ldx, int M, int K, float *xmax, hipStream_t st);
int launch_smooth_scales(const float *xmax, const __half *w, int N, int K, float alpha, float *s, float *inv_s,
                         hipStream_t st);
int launch_export8(const int8_t *kl, int N, int K, int8_t *canon, hipStream_t st);
int launch_export4(const uint8_t *kl, int N, int K, int group, uint8_t *canon, __half *scales,
                   hipStream_t st);

struct GemmArgs {
    const __half *x;       // decode only: fp16 tokens [M, ldx] to quantize inside the GEMM (then xq, sx unused)
    int64_t ldx;
    const int8_t *xq;      // kernel layout, ceil32(M) rows
    const float *sx;       // [M] (unused by the accumulator dump)
    const void *wq;        // kernel-layout blob
    const float *sw;       // [N] per-channel scales (W8A8)
    const __half *bias;    // [N] or nullptr
    __half *y;             // [M, ldy]
    int64_t ldy;
    int32_t *acc;          // accumulator dump [M,N] (test hook) or nullptr
    int64_t ldacc;         // its row stride (0: N)
    int32_t *partials;     // W4A8 group partials [nrows, G, N] or nullptr
    int row0, nrows;
    int M, N, K;
    int bits, group;
    void *ws;
    size_t ws_bytes;
};
int launch_gemm_prefill(const GemmArgs &a, int variant, hipStream_t st);
int launch_gemm_decode(const GemmArgs &a, int variant, hipStream_t st);
// estimated time (us) of the automatic choice of the tile kernels / of the decode kernels (33 tokens and more)
double prefill_estimate_us(const GemmArgs &a);
double decode_estimate_us(const GemmArgs &a);
// what the automatic choice would launch (host only)
void prefill_plan(const GemmArgs &a, int *variant, int *tile_tokens, int *tile_channels, int *splits, int *rest_channels,
                  int *rest_variant);
void decode_plan(const GemmArgs &a, int *token_block, int *channel_groups);
bool decode_fuses_quant(int M, int K, int variant);

}  // namespace ql
