// Offline weight quantization (paper Eq. 1-2; per-output-channel scales for int8, group-wise
// scales along K for int4 -- Preliminary, granularity paragraph) and the conversion to and from the
// GEMM's tile order (the "weight layout" step of the paper's inference framework), for gfx950.
//
//   int8: s[n] = amax_n / 127 (fp32; 1 if zero);       code = clamp(rne(w / s[n]), +-127)
//   int4: s[n,g] = fp16(amax_{n,g} / 7) (1 if zero);   code = clamp(rne(w / float(s[n,g])), +-7)
//         canonical packing: two's-complement nibbles, even k in bits 3:0, odd k in bits 7:4
// Options (Preliminary section): `range` 1 = Eq. 2 as printed, s = 2 amax / (2^n - 1) and codes in
// [-2^(n-1), 2^(n-1) - 1]; `tensor_amax` (bit pattern of the whole matrix's max |w|) replaces the channel's /
// group's own maximum: per-tensor granularity, stored as equal per-channel / per-group scales.
// Not on the timed path: one workgroup per output channel, the row is read twice.
#include "common.h"

namespace ql {
namespace {

constexpr int CHUNK = 16;

struct alignas(16) Half16 {
    uint4 lo, hi;
};

// 16 consecutive weights as fp32: from fp16 (exact widening) or from the fp32 output of a transform kernel
__device__ inline void load16(const __half *row, int c, float (&v)[16])
{
    const Half16 h = reinterpret_cast<const Half16 *>(row)[c];
    const unsigned w[8] = {h.lo.x, h.lo.y, h.lo.z, h.lo.w, h.hi.x, h.hi.y, h.hi.z, h.hi.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v[2 * i] = __half2float(__ushort_as_half((unsigned short)(w[i] & 0xffffu)));
        v[2 * i + 1] = __half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
    }
}

__device__ inline void load16(const float *row, int c, float (&v)[16])
{
#pragma unroll
    for (int i = 0; i < 16; i += 4) {
        const float4 f = *reinterpret_cast<const float4 *>(row + (size_t)c * CHUNK + i);
        v[i] = f.x, v[i + 1] = f.y, v[i + 2] = f.z, v[i + 3] = f.w;
    }
}

__device__ inline float amax16(const float (&v)[16])
{
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(v[i]));
    return m;
}

__device__ inline int code_div(float x, float scale, float lo, float hi)
{
    const float t = x / scale;   // IEEE fp32 division by the stored scale
    float r = rintf(t);
    r = fminf(fmaxf(r, lo), hi);
    return (int)r;
}

// Eq. 2's scale from an abs-max; qmax = 2^(n-1) - 1
__device__ inline float scale_of(float amax, int range, float qmax)
{
    return range == QL_RANGE_EQ2 ? (2.0f * amax) / (2.0f * qmax + 1.0f) : amax / qmax;   // one IEEE fp32 division
}

template <typename T>
__global__ void weight_quant8_kernel(const T *__restrict__ w, int N, int K, int range,
                                     const unsigned *__restrict__ tensor_amax,
                                     int8_t *__restrict__ canon, float *__restrict__ scales,
                                     int8_t *__restrict__ kl)
{
    __shared__ float red[4];
    const int n = blockIdx.x;
    const int nchunks = K / CHUNK;
    if (n >= N) {   // padding rows of the kernel layout
        if (kl)
            for (int c = threadIdx.x; c < nchunks; c += blockDim.x)
                *reinterpret_cast<uint4 *>(kl + tile_offset_i8(n, c * CHUNK, K)) = make_uint4(0, 0, 0, 0);
        return;
    }
    const T *row = w + (size_t)n * K;
    float mx = 0.0f;
    if (tensor_amax) {
        mx = __uint_as_float(*tensor_amax);
    } else {
        for (int c = threadIdx.x; c < nchunks; c += blockDim.x) {
            float h[16];
            load16(row, c, h);
            mx = fmaxf(mx, amax16(h));
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    }

    float s = scale_of(mx, range, 127.0f);
    if (s == 0.0f) s = 1.0f;
    const float lo = range == QL_RANGE_EQ2 ? -128.0f : -127.0f;
    if (threadIdx.x == 0 && scales) scales[n] = s;

    for (int c = threadIdx.x; c < nchunks; c += blockDim.x) {
        float h[16];
        load16(row, c, h);
        unsigned q[4] = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 16; ++i) q[i / 4] |= (unsigned)(code_div(h[i], s, lo, 127.0f) & 0xff) << (8 * (i % 4));
        const uint4 o = make_uint4(q[0], q[1], q[2], q[3]);
        if (canon) *reinterpret_cast<uint4 *>(canon + (size_t)n * K + (size_t)c * CHUNK) = o;
        if (kl) *reinterpret_cast<uint4 *>(kl + tile_offset_i8(n, c * CHUNK, K)) = o;
    }
}

// group == 128: eight consecutive lanes hold one group.
template <typename T>
__global__ void weight_quant4_kernel(const T *__restrict__ w, int N, int Npad, int K, int range,
                                     const unsigned *__restrict__ tensor_amax,
                                     uint8_t *__restrict__ canon, __half *__restrict__ scales,
                                     uint8_t *__restrict__ kl_codes, __half *__restrict__ kl_scales,
                                     __half *__restrict__ kl_scales_dec)
{
    const int n = blockIdx.x;
    const int nchunks = K / CHUNK;
    const int G = K / 128;
    for (int c = threadIdx.x; c < nchunks; c += blockDim.x) {
        float h[16];
        if (n < N) {
            load16(w + (size_t)n * K, c, h);
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) h[i] = 0.0f;
        }
        float mx = amax16(h);
        mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 4, 64));
        if (tensor_amax) mx = (n < N) ? __uint_as_float(*tensor_amax) : 0.0f;
        const float s32 = scale_of(mx, range, 7.0f);   // IEEE fp32 division
        __half s16 = __float2half_rn(s32);
        if (__half2float(s16) == 0.0f) s16 = __float2half_rn(1.0f);
        const float s = __half2float(s16);
        const int g = c / 8;
        if ((c % 8) == 0) {
            if (n < N && scales) scales[(size_t)n * G + g] = s16;
            if (kl_scales) kl_scales[(size_t)g * Npad + n] = s16;
            if (kl_scales_dec) kl_scales_dec[((size_t)(n / 16) * G + g) * 16 + n % 16] = s16;
        }
        int q[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) q[i] = code_div(h[i], s, range == QL_RANGE_EQ2 ? -8.0f : -7.0f, 7.0f) & 0xf;
        if (n < N && canon) {
            unsigned lo = 0, hi = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lo |= (unsigned)(q[2 * i] | (q[2 * i + 1] << 4)) << (8 * i);
                hi |= (unsigned)(q[8 + 2 * i] | (q[8 + 2 * i + 1] << 4)) << (8 * i);
            }
            *reinterpret_cast<uint2 *>(canon + (size_t)n * (K / 2) + (size_t)c * 8) = make_uint2(lo, hi);
        }
        if (kl_codes) {
            unsigned w0 = 0, w1 = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                w0 |= (unsigned)q[i] << (4 * w4_nibble_pos(i));
                w1 |= (unsigned)q[8 + i] << (4 * w4_nibble_pos(i));
            }
            *reinterpret_cast<uint2 *>(kl_codes + tile_offset_w4_word(n, c * CHUNK, K)) = make_uint2(w0, w1);
        }
    }
}

// max |w| over the whole matrix as a bit pattern (non-negative floats order like unsigned integers);
// *out must hold 0 (or an earlier maximum) on entry
template <typename T>
__global__ void tensor_absmax_kernel(const T *__restrict__ w, size_t nchunks, unsigned *__restrict__ out)
{
    float mx = 0.0f;
    for (size_t c = blockIdx.x * (size_t)blockDim.x + threadIdx.x; c < nchunks; c += (size_t)gridDim.x * blockDim.x) {
        float h[16];
        load16(w + c * CHUNK, 0, h);
        mx = fmaxf(mx, amax16(h));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if ((threadIdx.x & 63) == 0 && mx > 0.0f) atomicMax(out, __float_as_uint(mx));
}

__global__ void fill_u32_kernel(unsigned *p, unsigned v) { *p = v; }

__global__ void export8_kernel(const int8_t *__restrict__ kl, int K, int8_t *__restrict__ canon)
{
    const int n = blockIdx.x;
    for (int c = threadIdx.x; c < K / CHUNK; c += blockDim.x)
        *reinterpret_cast<uint4 *>(canon + (size_t)n * K + (size_t)c * CHUNK) =
            *reinterpret_cast<const uint4 *>(kl + tile_offset_i8(n, c * CHUNK, K));
}

__global__ void export4_kernel(const uint8_t *__restrict__ kl_codes, const __half *__restrict__ kl_scales,
                               int Npad, int K, uint8_t *__restrict__ canon, __half *__restrict__ scales)
{
    const int n = blockIdx.x;
    const int G = K / 128;
    for (int c = threadIdx.x; c < K / CHUNK; c += blockDim.x) {
        const uint2 v = *reinterpret_cast<const uint2 *>(kl_codes + tile_offset_w4_word(n, c * CHUNK, K));
        int q[16];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            q[i] = (v.x >> (4 * w4_nibble_pos(i))) & 0xf;
            q[8 + i] = (v.y >> (4 * w4_nibble_pos(i))) & 0xf;
        }
        unsigned lo = 0, hi = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            lo |= (unsigned)(q[2 * i] | (q[2 * i + 1] << 4)) << (8 * i);
            hi |= (unsigned)(q[8 + 2 * i] | (q[8 + 2 * i + 1] << 4)) << (8 * i);
        }
        if (canon) *reinterpret_cast<uint2 *>(canon + (size_t)n * (K / 2) + (size_t)c * 8) = make_uint2(lo, hi);
        if (scales && (c % 8) == 0) scales[(size_t)n * G + c / 8] = kl_scales[(size_t)(c / 8) * Npad + n];
    }
}

}  // namespace

template <typename T>
static int launch_wq8(const T *w, int N, int K, int8_t *canon, float *scales, int8_t *kl, hipStream_t st,
                      int range = QL_RANGE_SYMMETRIC, const unsigned *tensor_amax = nullptr)
{
    const int rows = kl ? round_up(N, TILE_ROWS) : N;
    hipLaunchKernelGGL(weight_quant8_kernel<T>, dim3(rows), dim3(256), 0, st, w, N, K, range, tensor_amax, canon,
                       scales, kl);
    return check_hip(hipGetLastError(), "weight_quant8 launch");
}

template <typename T>
static int launch_wq4(const T *w, int N, int K, int group, uint8_t *canon, __half *scales, uint8_t *kl, hipStream_t st,
                      int range = QL_RANGE_SYMMETRIC, const unsigned *tensor_amax = nullptr)
{
    const int Npad = round_up(N, TILE_ROWS);
    const int rows = kl ? Npad : N;
    __half *kls = kl ? reinterpret_cast<__half *>(kl + w4_scales_offset(N, K)) : nullptr;
    __half *klsd = kl ? reinterpret_cast<__half *>(kl + w4_scales_dec_offset(N, K, group)) : nullptr;
    hipLaunchKernelGGL(weight_quant4_kernel<T>, dim3(rows), dim3(256), 0, st, w, N, Npad, K, range, tensor_amax,
                       canon, scales, kl, kls, klsd);
    return check_hip(hipGetLastError(), "weight_quant4 launch");
}

int launch_weight_quant8(const __half *w, int N, int K, int8_t *canon, float *scales, int8_t *kl,
                         hipStream_t st)
{
    return launch_wq8(w, N, K, canon, scales, kl, st);
}

int launch_weight_quant4(const __half *w, int N, int K, int group, uint8_t *canon, __half *scales,
                         uint8_t *kl, hipStream_t st)
{
    return launch_wq4(w, N, K, group, canon, scales, kl, st);
}

// Eq. 2 as printed and / or per-tensor granularity; amax_scratch: 4 bytes of device memory (per-tensor only)
int launch_weight_quant_opt(const __half *w, int N, int K, int bits, int group, int range, bool per_tensor,
                            unsigned *amax_scratch, void *canon, void *scales, void *kl, hipStream_t st)
{
    if (per_tensor) {
        const size_t nchunks = (size_t)N * K / CHUNK;
        const int blocks = (int)((nchunks + 255) / 256 < 2048 ? (nchunks + 255) / 256 : 2048);
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(1), 0, st, amax_scratch, 0u);
        hipLaunchKernelGGL(tensor_absmax_kernel<__half>, dim3(blocks), dim3(256), 0, st, w, nchunks, amax_scratch);
        QL_TRY(check_hip(hipGetLastError(), "tensor_absmax launch"));
    }
    const unsigned *ta = per_tensor ? amax_scratch : nullptr;
    if (bits == 8)
        return launch_wq8(w, N, K, static_cast<int8_t *>(canon), static_cast<float *>(scales),
                          static_cast<int8_t *>(kl), st, range, ta);
    return launch_wq4(w, N, K, group, static_cast<uint8_t *>(canon), static_cast<__half *>(scales),
                      static_cast<uint8_t *>(kl), st, range, ta);
}

// the same quantizers on fp32 weights (the output of a transform, Eq. 3-4)
int launch_weight_quant8_f32(const float *w, int N, int K, int8_t *canon, float *scales, int8_t *kl,
                             hipStream_t st)
{
    return launch_wq8(w, N, K, canon, scales, kl, st);
}

int launch_weight_quant4_f32(const float *w, int N, int K, int group, uint8_t *canon, __half *scales,
                             uint8_t *kl, hipStream_t st)
{
    return launch_wq4(w, N, K, group, canon, scales, kl, st);
}

int launch_export8(const int8_t *kl, int N, int K, int8_t *canon, hipStream_t st)
{
    hipLaunchKernelGGL(export8_kernel, dim3(N), dim3(256), 0, st, kl, K, canon);
    return check_hip(hipGetLastError(), "export8 launch");
}

int launch_export4(const uint8_t *kl, int N, int K, int group, uint8_t *canon, __half *scales,
                   hipStream_t st)
{
    (void)group;
    const int Npad = round_up(N, TILE_ROWS);
    const __half *kls = reinterpret_cast<const __half *>(kl + w4_scales_offset(N, K));
    hipLaunchKernelGGL(export4_kernel, dim3(N), dim3(256), 0, st, kl, kls, Npad, K, canon, scales);
    return check_hip(hipGetLastError(), "export4 launch");
}

}  // namespace ql
