// The operand transforms of the paper's two enhanced W4A8 configurations, for gfx950:
//   SmoothQuant (Eq. 3):  Y = (X S^-1)(S W),  s_j = max|X_j|^alpha / max|W_j|^(1-alpha)
//   Hadamard   (Eq. 4):  Y = (X H)(H^T W),   H a normalized Hadamard matrix
// Online: the activation side (per-channel multiply by 1/s_j, or a fast Walsh-Hadamard transform of every
// token) is fused in front of the per-token int8 quantizer (Eq. 1-2), one workgroup per token, fp32 throughout.
// Offline: calibration statistics, the scale vector, and the transformed fp32 weights handed to the weight
// quantizer.
//
// H is the natural-order (Sylvester) matrix, block diagonal with blocks of B = the largest power of two that
// divides K (at most 4096) so that any K % 64 == 0 works.  It is applied as the in-place butterfly in fp32,
// stages h = 1, 2, ..., B/2 in that order, every output one addition or subtraction, then one multiply by
// fp32(1/sqrt(B)): a fixed sequence of single fp32 operations per element, whatever lane does them.
// A lane holds chunks of 16 consecutive elements: stages h <= 8 in registers, the next six across the lanes
// of a wavefront (four of them as vector-ALU lane permutes), the last two (B > 1024) across wavefronts through LDS.
#include "common.h"
#include "quant_math.h"
#include <cmath>

namespace ql {
namespace {

constexpr int TW = 256;                 // threads per workgroup (one token / one weight row); at most 4 chunks of 16 per thread: K <= 16384

__device__ inline void load_chunk(const __half *row, int c, float (&v)[16])
{
    const Half16 h = reinterpret_cast<const Half16 *>(row)[c];
    const unsigned w[8] = {h.lo.x, h.lo.y, h.lo.z, h.lo.w, h.hi.x, h.hi.y, h.hi.z, h.hi.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v[2 * i] = half_bits_to_float(w[i] & 0xffffu);
        v[2 * i + 1] = half_bits_to_float(w[i] >> 16);
    }
}

__device__ inline void scale_chunk(const float *__restrict__ s, int c, float (&v)[16])
{
#pragma unroll
    for (int i = 0; i < 16; i += 4) {
        const float4 f = *reinterpret_cast<const float4 *>(s + (size_t)c * 16 + i);
        v[i] *= f.x, v[i + 1] *= f.y, v[i + 2] *= f.z, v[i + 3] *= f.w;   // one fp32 multiply each
    }
}

// Value of the same register in lane (lane ^ bit).  Inside a row of 16 lanes the data-parallel-primitive
// modifiers do it on the vector ALU (quad permutes for 1 and 2; 4 = reverse each half-row of 8, then reverse
// each quad; 8 = rotate the row by 8); 16 and 32 go through the LDS crossbar.
template <int CTRL>
__device__ inline float dpp_move(float v)
{
    // all rows and banks enabled and every source lane exists: the 'old' operand is never read
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

template <int BIT>
__device__ inline float lane_xor(float v)
{
    if constexpr (BIT == 1) return dpp_move<0xB1>(v);                        // quad_perm [1,0,3,2]
    else if constexpr (BIT == 2) return dpp_move<0x4E>(v);                   // quad_perm [2,3,0,1]
    else if constexpr (BIT == 4) return dpp_move<0x1B>(dpp_move<0x141>(v));  // row_half_mirror (i ^ 7), then quad_perm [3,2,1,0] (i ^ 3)
    else if constexpr (BIT == 8) return dpp_move<0x128>(v);                  // row_ror:8
    else return __shfl_xor(v, BIT, 64);
}

// one butterfly stage between lanes BIT apart: the lower lane keeps a + b, the upper one a - b (a = the lower lane's value)
template <int BIT, int NIT>
__device__ inline void lane_stage(float (&v)[NIT][16])
{
    // a + b below, b' - a' above: one fused multiply-add by +-1 (exact product, so the single rounding is that of
    // the addition or subtraction itself)
    const float sgn = (threadIdx.x & BIT) != 0 ? -1.0f : 1.0f;
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
        for (int i = 0; i < 16; ++i) v[it][i] = __builtin_fmaf(sgn, v[it][i], lane_xor<BIT>(v[it][i]));
}

// Block-diagonal Hadamard transform of the row whose chunk (it * TW + tid) sits in v[it]; lanes per block
// = hblock / 16 (a power of two that divides TW and the number of chunks, so a block never straddles an `it`).
// LB: log2(hblock) when it is known at compile time (every stage's presence is then resolved at compile time,
// which saves the register copies that merge the skipped and the executed path of each stage), -1 otherwise.
template <int NIT, int LB = -1>
__device__ inline void fwht_row(float (&v)[NIT][16], int hblock, float norm, float *xchg /* [TW][16] */)
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
#pragma unroll
        for (int h = 1; h < 16; h <<= 1)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if ((i & h) == 0) {
                    const float a = v[it][i], b = v[it][i | h];
                    v[it][i] = a + b;
                    v[it][i | h] = a - b;
                }
    }
    const int lanes = LB >= 0 ? (1 << (LB >= 0 ? LB : 0)) / 16 : hblock / 16;
    if (lanes > 1) lane_stage<1>(v);
    if (lanes > 2) lane_stage<2>(v);
    if (lanes > 4) lane_stage<4>(v);
    if (lanes > 8) lane_stage<8>(v);
    if (lanes > 16) lane_stage<16>(v);
    if (lanes > 32) lane_stage<32>(v);
    for (int bit = 64; bit < lanes; bit <<= 1) {   // across wavefronts
        const float sgn = (tid & bit) != 0 ? -1.0f : 1.0f;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            float o[16];
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; ++i) xchg[i * TW + tid] = v[it][i];
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; ++i) o[i] = xchg[i * TW + (tid ^ bit)];
#pragma unroll
            for (int i = 0; i < 16; ++i) v[it][i] = __builtin_fmaf(sgn, v[it][i], o[i]);
        }
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
        for (int i = 0; i < 16; ++i) v[it][i] *= norm;
}

// One workgroup per token: load, transform, per-token abs-max, quantize, store (row-major and/or tile order).
// (Collecting 8 tokens per workgroup for whole-line writes of the tile order, as the plain quantizer does at
// large M, was measured and is slower here: a workgroup transforms its tokens one after the other, and that
// serial latency costs more than the 16-byte writes save -- 37 us against 27 us for 4096 x 4096.)
template <int NIT, int LB>
__global__ __launch_bounds__(TW) void act_quant_transform_kernel(const __half *__restrict__ x, int64_t ldx, int K,
                                                                 const float *__restrict__ inv_smooth, int hblock,
                                                                 float norm, int8_t *__restrict__ xq_rm,
                                                                 int8_t *__restrict__ xq_kl, float *__restrict__ sx)
{
    __shared__ float xchg[16 * TW];
    __shared__ float red[TW / 64];
    const int m = blockIdx.x, tid = threadIdx.x;
    const int nchunks = K / 16;
    const __half *row = x + (size_t)m * ldx;
    float v[NIT][16];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int c = it * TW + tid;
        if (c < nchunks) {
            load_chunk(row, c, v[it]);
            if (inv_smooth) scale_chunk(inv_smooth, c, v[it]);
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) v[it][i] = 0.0f;
        }
    }
    if (LB > 0) fwht_row<NIT, LB>(v, hblock, norm, xchg);

    float amax = 0.0f;
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
        for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(v[it][i]));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    if ((tid & 63) == 0) red[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float scale, inv;
    token_scales_f32(amax, scale, inv);
    if (tid == 0) sx[m] = scale;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int c = it * TW + tid;
        if (c < nchunks) {
            const uint4 q = quant_chunk_f32(v[it], inv);
            if (xq_rm) *reinterpret_cast<uint4 *>(xq_rm + (size_t)m * K + (size_t)c * 16) = q;
            if (xq_kl) *reinterpret_cast<uint4 *>(xq_kl + tile_offset_i8(m, c * 16, K)) = q;
        }
    }
}

// Offline: one workgroup per weight row (output channel): S W and/or H^T W as fp32
template <int NIT>
__global__ __launch_bounds__(TW) void weight_transform_kernel(const __half *__restrict__ w, int K,
                                                              const float *__restrict__ smooth, int hblock, float norm,
                                                              float *__restrict__ out)
{
    __shared__ float xchg[16 * TW];
    const int n = blockIdx.x, tid = threadIdx.x;
    const int nchunks = K / 16;
    float v[NIT][16];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int c = it * TW + tid;
        if (c < nchunks) {
            load_chunk(w + (size_t)n * K, c, v[it]);
            if (smooth) scale_chunk(smooth, c, v[it]);
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) v[it][i] = 0.0f;
        }
    }
    if (hblock > 1) fwht_row<NIT>(v, hblock, norm, xchg);
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int c = it * TW + tid;
        if (c < nchunks) {
#pragma unroll
            for (int i = 0; i < 16; i += 4)
                *reinterpret_cast<float4 *>(out + (size_t)n * K + (size_t)c * 16 + i) =
                    make_float4(v[it][i], v[it][i + 1], v[it][i + 2], v[it][i + 3]);
        }
    }
}

// Calibration: running max|X_j| per input channel (non-negative floats order like their bit patterns)
__global__ void channel_absmax_kernel(const __half *__restrict__ x, int64_t ldx, int M, int K, int rows_per_block,
                                      unsigned *__restrict__ xmax_bits)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    const int m0 = blockIdx.y * rows_per_block;
    const int m1 = min(M, m0 + rows_per_block);
    float mx = 0.0f;
    for (int m = m0; m < m1; ++m) mx = fmaxf(mx, fabsf(__half2float(x[(size_t)m * ldx + k])));
    atomicMax(xmax_bits + k, __float_as_uint(mx));
}

// s_j = xmax_j^alpha / wmax_j^(1-alpha), 1 where either maximum is 0; inv_j = 1 / s_j (IEEE fp32 division)
__global__ void smooth_scales_kernel(const float *__restrict__ xmax, const __half *__restrict__ w, int N, int K,
                                     float alpha, float *__restrict__ s, float *__restrict__ inv_s)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    float wmax = 0.0f;
    for (int n = 0; n < N; ++n) wmax = fmaxf(wmax, fabsf(__half2float(w[(size_t)n * K + k])));
    const float xm = xmax[k];
    float sj = 1.0f;
    if (xm > 0.0f && wmax > 0.0f) sj = (float)(pow((double)xm, (double)alpha) / pow((double)wmax, 1.0 - (double)alpha));
    s[k] = sj;
    inv_s[k] = 1.0f / sj;
}

float block_norm(int hblock) { return (float)(1.0 / std::sqrt((double)hblock)); }

}  // namespace

int hadamard_block_of(int K)
{
    const int b = K & -K;
    return b < 4096 ? b : 4096;
}

int launch_act_quant_transform(const __half *x, int64_t ldx, int M, int K, const float *inv_smooth, int hblock,
                               int8_t *xq_rm, int8_t *xq_kl, float *sx, hipStream_t st)
{
    if (M == 0) return QL_OK;
    const int nit = ceil_div(K / 16, TW);
    const float norm = block_norm(hblock > 1 ? hblock : 1);
    int lb = 0;
    while (hblock > 1 && (1 << lb) < hblock) ++lb;
#define QL_LAUNCH(NIT, LB)                                                                                        \
    hipLaunchKernelGGL((act_quant_transform_kernel<NIT, LB>), dim3(M), dim3(TW), 0, st, x, ldx, K, inv_smooth,    \
                       hblock, norm, xq_rm, xq_kl, sx)
#define QL_BY_BLOCK(NIT)                                                                                          \
    switch (lb) {                                                                                                 \
    case 0: QL_LAUNCH(NIT, 0); break;                                                                             \
    case 4: QL_LAUNCH(NIT, 4); break;                                                                             \
    case 5: QL_LAUNCH(NIT, 5); break;                                                                             \
    case 6: QL_LAUNCH(NIT, 6); break;                                                                             \
    case 7: QL_LAUNCH(NIT, 7); break;                                                                             \
    case 8: QL_LAUNCH(NIT, 8); break;                                                                             \
    case 9: QL_LAUNCH(NIT, 9); break;                                                                             \
    case 10: QL_LAUNCH(NIT, 10); break;                                                                           \
    case 11: QL_LAUNCH(NIT, 11); break;                                                                           \
    case 12: QL_LAUNCH(NIT, 12); break;                                                                           \
    default: return fail(QL_ERR_UNSUPPORTED, "hadamard_block=%d", hblock);                                        \
    }
    if (nit == 1) { QL_BY_BLOCK(1) }
    else if (nit == 2) { QL_BY_BLOCK(2) }
    else if (nit == 3) { QL_BY_BLOCK(3) }
    else { QL_BY_BLOCK(4) }
#undef QL_BY_BLOCK
#undef QL_LAUNCH
    return check_hip(hipGetLastError(), "act_quant_transform launch");
}

int launch_weight_transform(const __half *w, int N, int K, const float *smooth, int hblock, float *out, hipStream_t st)
{
    const int nit = ceil_div(K / 16, TW);
    const float norm = block_norm(hblock > 1 ? hblock : 1);
#define QL_LAUNCH(NIT) \
    hipLaunchKernelGGL((weight_transform_kernel<NIT>), dim3(N), dim3(TW), 0, st, w, K, smooth, hblock, norm, out)
    if (nit == 1) QL_LAUNCH(1);
    else if (nit == 2) QL_LAUNCH(2);
    else if (nit == 3) QL_LAUNCH(3);
    else QL_LAUNCH(4);
#undef QL_LAUNCH
    return check_hip(hipGetLastError(), "weight_transform launch");
}

int launch_channel_absmax(const __half *x, int64_t ldx, int M, int K, float *xmax, hipStream_t st)
{
    if (M == 0) return QL_OK;
    const int rows_per_block = 64;
    hipLaunchKernelGGL(channel_absmax_kernel, dim3(ceil_div(K, 256), ceil_div(M, rows_per_block)), dim3(256), 0, st, x,
                       ldx, M, K, rows_per_block, reinterpret_cast<unsigned *>(xmax));
    return check_hip(hipGetLastError(), "channel_absmax launch");
}

int launch_smooth_scales(const float *xmax, const __half *w, int N, int K, float alpha, float *s, float *inv_s,
                         hipStream_t st)
{
    hipLaunchKernelGGL(smooth_scales_kernel, dim3(ceil_div(K, 256)), dim3(256), 0, st, xmax, w, N, K, alpha, s, inv_s);
    return check_hip(hipGetLastError(), "smooth_scales launch");
}

}  // namespace ql
