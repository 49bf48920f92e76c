// Per-token dynamic int8 activation quantization (paper Eq. 1-2 with n = 8; one scale per token
// over its whole feature dimension, Preliminary section) for gfx950.
//
// One workgroup per 8 tokens (per token when there are at most 512).  The rows are read once: each lane
// keeps its 16-element chunks in registers, the row maxima are reduced across lanes and wavefronts, then the codes are produced
// from the registers and written row-major and/or in the GEMM's tile order, whole 128-byte lines
// at a time.
//
// Arithmetic (every step a single correctly rounded fp32 operation):
//   amax = max_k |x|            sx = amax / 127          inv = 127 / amax
//   code = clamp(rne(x * inv), -127, 127)                (all-zero token: sx = 1, codes 0)
#include "common.h"
#include "quant_math.h"

namespace ql {
namespace {

// One workgroup quantizes RPB consecutive tokens.  RPB = 8 (prefill): a wavefront covers 8 tokens x 8
// chunks per step (lane = token % 8 + 8 * chunk), so that in the GEMM's tile order the 8 lanes of one
// chunk write one whole 128-byte line (8 token slots x 16 bytes) and in the row-major copy each token
// gets 128 contiguous bytes per step.  RPB = 1 (decode, short prefill): all 64 lanes of a wavefront
// work on the same token, 64 chunks per step, so that a single token is not left to 8 lanes.
// The NW wavefronts split K; the row maxima meet in LDS.
// NIT: steps per wavefront kept in registers; NIT == 0: the row is read twice.
// Up to this many tokens one workgroup per token is faster (2.5-8 us against 5-11 us at K = 4096..11008): the
// 8-token workgroups are too few to cover the memory latency; beyond it their whole-line writes win.
constexpr int SINGLE_TOKEN_MAX_M = 512;
constexpr int MAX_RPB = 8;
constexpr int MAX_WAVES = 8;

// SM: the SmoothQuant variant (paper Eq. 3): every element is first multiplied by inv_smooth[k] = 1 / s_k (one
// fp32 multiply, done again when the codes are produced -- cheaper than keeping fp32 copies in registers), the
// row maximum is taken on those fp32 products (non-negative floats order like their bit patterns).
template <int NIT, int RPB, bool SM>
__global__ __launch_bounds__(MAX_WAVES * 64) void act_quant_kernel(const __half *__restrict__ x, int64_t ldx,
                                                                    int M, int K, int per_wave,
                                                                    const float *__restrict__ inv_smooth,
                                                                    int8_t *__restrict__ xq_rm,
                                                                    int8_t *__restrict__ xq_kl,
                                                                    float *__restrict__ sx)
{
    auto smoothed = [&](const Half16 &h, int c, float (&f)[16]) {
        const unsigned w[8] = {h.lo.x, h.lo.y, h.lo.z, h.lo.w, h.hi.x, h.hi.y, h.hi.z, h.hi.w};
#pragma unroll
        for (int i = 0; i < 16; i += 4) {
            const float4 s4 = *reinterpret_cast<const float4 *>(inv_smooth + (size_t)c * CHUNK + i);
            f[i] = half_bits_to_float(w[i / 2] & 0xffffu) * s4.x;
            f[i + 1] = half_bits_to_float(w[i / 2] >> 16) * s4.y;
            f[i + 2] = half_bits_to_float(w[i / 2 + 1] & 0xffffu) * s4.z;
            f[i + 3] = half_bits_to_float(w[i / 2 + 1] >> 16) * s4.w;
        }
    };
    auto row_max = [&](const Half16 &h, int c, unsigned m) {
        if (!SM) return abs_max_bits(h, m);
        float f[16];
        smoothed(h, c, f);
#pragma unroll
        for (int i = 0; i < 16; ++i) m = max(m, __float_as_uint(fabsf(f[i])));
        return m;
    };
    __shared__ unsigned red[MAX_RPB][MAX_WAVES];
    constexpr int CPS = 64 / RPB;                       // chunks per wavefront per step
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int r = lane % RPB, cl = lane / RPB;
    const int m = blockIdx.x * RPB + r;
    const bool valid = m < M;
    const int nchunks = K / CHUNK;
    const Half16 *row = reinterpret_cast<const Half16 *>(x + (size_t)(valid ? m : 0) * ldx);
    const int s0 = wave * per_wave;

    Half16 v[NIT > 0 ? NIT : 1];
    unsigned mx = 0;
    if (NIT > 0) {
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = (s0 + i) * CPS + cl;
            if (i < per_wave && c < nchunks && valid) {
                v[i] = row[c];
                mx = row_max(v[i], c, mx);
            }
        }
    } else {
        for (int i = 0; i < per_wave; ++i) {
            const int c = (s0 + i) * CPS + cl;
            if (c < nchunks && valid) mx = row_max(row[c], c, mx);
        }
    }
#pragma unroll
    for (int off = 32; off >= RPB; off >>= 1) mx = max(mx, (unsigned)__shfl_xor((int)mx, off, 64));
    if (cl == 0) red[r][wave] = mx;
    __syncthreads();
    mx = 0;
    for (int w = 0; w < nwaves; ++w) mx = max(mx, red[r][w]);

    float scale, inv;
    if (SM) token_scales_f32(__uint_as_float(mx), scale, inv);
    else token_scales(mx, scale, inv);
    if (wave == 0 && cl == 0 && valid) sx[m] = scale;

    auto emit = [&](int c, const Half16 &h) {
        uint4 q;
        if (SM) {
            float f[16];
            smoothed(h, c, f);
            q = quant_chunk_f32(f, inv);
        } else {
            q = quant_chunk(h, inv);
        }
        if (xq_rm) *reinterpret_cast<uint4 *>(xq_rm + (size_t)m * K + (size_t)c * CHUNK) = q;
        if (xq_kl) *reinterpret_cast<uint4 *>(xq_kl + tile_offset_i8(m, c * CHUNK, K)) = q;
    };
    if (NIT > 0) {
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = (s0 + i) * CPS + cl;
            if (i < per_wave && c < nchunks && valid) emit(c, v[i]);
        }
    } else {
        for (int i = 0; i < per_wave; ++i) {
            const int c = (s0 + i) * CPS + cl;
            if (c < nchunks && valid) emit(c, row[c]);
        }
    }
}

__global__ void act_repack_kernel(const int8_t *__restrict__ xq_rm, int M, int K,
                                  int8_t *__restrict__ xq_kl)
{
    const int nchunks = K / CHUNK;
    const size_t total = (size_t)M * nchunks;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        const int m = (int)(i / nchunks), c = (int)(i % nchunks);
        const uint4 q = *reinterpret_cast<const uint4 *>(xq_rm + (size_t)m * K + (size_t)c * CHUNK);
        *reinterpret_cast<uint4 *>(xq_kl + tile_offset_i8(m, c * CHUNK, K)) = q;
    }
}

}  // namespace

template <int RPB, bool SM>
static void launch_aq(const __half *x, int64_t ldx, int M, int K, const float *inv_smooth, int8_t *xq_rm,
                      int8_t *xq_kl, float *sx, hipStream_t st)
{
    const int steps = ceil_div(K / CHUNK, 64 / RPB);
    const int nw = steps < MAX_WAVES ? steps : MAX_WAVES;
    const int per_wave = ceil_div(steps, nw);
    dim3 grid(ceil_div(M, RPB)), block(nw * 64);
#define QL_LAUNCH_AQ(NIT) \
    hipLaunchKernelGGL((act_quant_kernel<NIT, RPB, SM>), grid, block, 0, st, x, ldx, M, K, per_wave, inv_smooth, xq_rm, \
                       xq_kl, sx)
    if (per_wave <= 1) QL_LAUNCH_AQ(1);
    else if (per_wave <= 2) QL_LAUNCH_AQ(2);
    else if (per_wave <= 4) QL_LAUNCH_AQ(4);
    else if (per_wave <= 8) QL_LAUNCH_AQ(8);
    else if (per_wave <= 12) QL_LAUNCH_AQ(12);
    else QL_LAUNCH_AQ(0);
#undef QL_LAUNCH_AQ
}

int launch_act_quant(const __half *x, int64_t ldx, int M, int K, int8_t *xq_rm, int8_t *xq_kl,
                     float *sx, hipStream_t st)
{
    if (M == 0) return QL_OK;
    if (M <= SINGLE_TOKEN_MAX_M) launch_aq<1, false>(x, ldx, M, K, nullptr, xq_rm, xq_kl, sx, st);
    else launch_aq<8, false>(x, ldx, M, K, nullptr, xq_rm, xq_kl, sx, st);
    return check_hip(hipGetLastError(), "act_quant launch");
}

int launch_act_quant_smooth(const __half *x, int64_t ldx, int M, int K, const float *inv_smooth, int8_t *xq_rm,
                            int8_t *xq_kl, float *sx, hipStream_t st)
{
    if (M == 0) return QL_OK;
    if (M <= SINGLE_TOKEN_MAX_M) launch_aq<1, true>(x, ldx, M, K, inv_smooth, xq_rm, xq_kl, sx, st);
    else launch_aq<8, true>(x, ldx, M, K, inv_smooth, xq_rm, xq_kl, sx, st);
    return check_hip(hipGetLastError(), "act_quant (smooth) launch");
}

int launch_act_repack(const int8_t *xq_rm, int M, int K, int8_t *xq_kl, hipStream_t st)
{
    if (M == 0) return QL_OK;
    const size_t total = (size_t)M * (K / CHUNK);
    int blocks = (int)((total + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(act_repack_kernel, dim3(blocks), dim3(256), 0, st, xq_rm, M, K, xq_kl);
    return check_hip(hipGetLastError(), "act_repack launch");
}

}  // namespace ql
