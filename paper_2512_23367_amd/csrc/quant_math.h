// Arithmetic of the per-token int8 activation quantizer (paper Eq. 1-2 with n = 8), shared by the
// stand-alone quantization kernel and the decode GEMM that quantizes its few tokens in its prologue.
// Every step is a single correctly rounded fp32 operation:
//   amax = max_k |x|            sx = amax / 127          inv = 127 / amax
//   code = clamp(rne(x * inv), -127, 127)                (all-zero token: sx = 1, codes 0)
#ifndef QL_QUANT_MATH_H
#define QL_QUANT_MATH_H

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

namespace ql {

constexpr int CHUNK = 16;               // elements per lane per step: 32 B in, 16 B out

struct alignas(16) Half16 {
    uint4 lo, hi;                       // 16 fp16 values
};

__device__ inline unsigned abs_max_bits(const Half16 &v, unsigned m)
{
    // |h| as an integer is monotonic in |value| for finite fp16, so the maximum can be taken on bits
    const unsigned w[8] = {v.lo.x, v.lo.y, v.lo.z, v.lo.w, v.hi.x, v.hi.y, v.hi.z, v.hi.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        m = max(m, w[i] & 0x7fffu);
        m = max(m, (w[i] >> 16) & 0x7fffu);
    }
    return m;
}

__device__ inline float half_bits_to_float(unsigned bits)
{
    return __half2float(__ushort_as_half((unsigned short)bits));
}

__device__ inline int quant_code(unsigned hbits, float inv)
{
    const float t = half_bits_to_float(hbits) * inv;    // one fp32 multiply
    float r = rintf(t);                                 // round half to even
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

__device__ inline unsigned quant_word(unsigned w0, unsigned w1, float inv)   // 4 halves -> 4 codes
{
    const unsigned a = quant_code(w0 & 0xffffu, inv) & 0xff;
    const unsigned b = quant_code(w0 >> 16, inv) & 0xff;
    const unsigned c = quant_code(w1 & 0xffffu, inv) & 0xff;
    const unsigned d = quant_code(w1 >> 16, inv) & 0xff;
    return a | (b << 8) | (c << 16) | (d << 24);
}

__device__ inline uint4 quant_chunk(const Half16 &v, float inv)
{
    uint4 q;
    q.x = quant_word(v.lo.x, v.lo.y, inv);
    q.y = quant_word(v.lo.z, v.lo.w, inv);
    q.z = quant_word(v.hi.x, v.hi.y, inv);
    q.w = quant_word(v.hi.z, v.hi.w, inv);
    return q;
}

// the same code decision for an fp32 value (operands after one of the paper's transforms, Eq. 3-4)
__device__ inline int quant_code_f32(float x, float inv)
{
    float r = rintf(x * inv);                           // one fp32 multiply, round half to even
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

__device__ inline uint4 quant_chunk_f32(const float (&v)[16], float inv)
{
    unsigned q[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 16; ++i) q[i / 4] |= (unsigned)(quant_code_f32(v[i], inv) & 0xff) << (8 * (i % 4));
    return make_uint4(q[0], q[1], q[2], q[3]);
}

__device__ inline void token_scales_f32(float amax, float &scale, float &inv)
{
    const bool zero = (amax == 0.0f);
    scale = zero ? 1.0f : amax / 127.0f;    // IEEE fp32 division
    inv = zero ? 0.0f : 127.0f / amax;      // IEEE fp32 division
}

// SwiGLU of the gated MLP in front of the quantizer (textbook definition: h = silu(gate) * up, silu(g) = g / (1 +
// exp(-g)); the paper names no activation function).  Every step is one correctly rounded fp32 operation, the
// exponential included -- clamp, range reduction by n = rint(t log2 e) with a two-constant ln 2, degree-7 Horner
// polynomial (multiply, then add), exact scaling by 2^n -- so that the codes are a function of the inputs alone.
__device__ inline float exp_steps(float t)      // t in [-80, 80]
{
    const float n = rintf(t * 1.4426950408889634f);
    float r = t - n * 0.693359375f;
    r = r - n * -2.12194440e-4f;
    float p = (float)(1.0 / 5040);
    p = p * r + (float)(1.0 / 720);
    p = p * r + (float)(1.0 / 120);
    p = p * r + (float)(1.0 / 24);
    p = p * r + (float)(1.0 / 6);
    p = p * r + 0.5f;
    p = p * r + 1.0f;
    p = p * r + 1.0f;
    return p * __int_as_float(((int)n + 127) << 23);   // times 2^n, exact: |n| <= 116
}

__device__ inline float swiglu_f32(float g, float u)
{
    const float t = fminf(fmaxf(-g, -80.0f), 80.0f);
    const float d = 1.0f + exp_steps(t);
    const float sg = 1.0f / d;                          // IEEE fp32 division
    return (g * sg) * u;
}

// token scale and its reciprocal from the bit pattern of the largest |x|
__device__ inline void token_scales(unsigned amax_bits, float &scale, float &inv)
{
    const float amax = half_bits_to_float(amax_bits);
    const bool zero = (amax_bits == 0);
    scale = zero ? 1.0f : amax / 127.0f;    // IEEE fp32 division
    inv = zero ? 0.0f : 127.0f / amax;      // IEEE fp32 division
}

}  // namespace ql
#endif
