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

typedef unsigned v4u __attribute__((ext_vector_type(4)));

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

// MODE 1: the SmoothQuant variant (paper Eq. 3): every element is first multiplied by inv_smooth[k] = 1 / s_k (one
// fp32 multiply, done again when the codes are produced -- cheaper than keeping fp32 copies in registers), the
// row maximum is taken on those fp32 products (non-negative floats order like their bit patterns).
// MODE 2: RMSNorm in front of the quantizer (textbook definition; the normalisation a decoder layer applies to the
// input of its QKV and gate/up projections):  h_k = x_k / sqrt(mean(x^2) + eps) * gamma_k, then Eq. 1-2 on h.
//   ss = fp32(sum x^2): the squares are exact in fp32, they are added in fp64 (per lane in k order, a butterfly
//        across the lanes, the wavefronts in order) and rounded to fp32 once -- the fp64 sum is within ~1e-13 of the
//        exact one, so this is the correctly rounded exact sum except within that distance of a rounding boundary;
//   mean = ss / K,  r = 1 / sqrt(mean + eps),  h = (x * r) * gamma: one correctly rounded fp32 operation each.
// MODE 3: SwiGLU in front of the quantizer: x is the fused gate+up projection output [M, 2K] (gate = columns 0..K-1,
// up = columns K..2K-1), the quantized value is h_k = silu(gate_k) * up_k in fp32 (swiglu_f32: a fixed sequence of
// single fp32 operations), recomputed when the codes are produced; the up half is re-read then (it sits in L2).
template <int NIT, int RPB, int MODE>
__global__ __launch_bounds__(MAX_WAVES * 64) void act_quant_kernel(const __half *__restrict__ x, int64_t ldx,
                                                                    int M, int K, int per_wave,
                                                                    const float *__restrict__ inv_smooth,
                                                                    const __half *__restrict__ gamma, float eps,
                                                                    int8_t *__restrict__ xq_rm,
                                                                    int8_t *__restrict__ xq_kl,
                                                                    float *__restrict__ sx)
{
    constexpr bool SM = MODE != 0;   // the codes come from fp32 values
    // MODE 2, up to 4 steps: the lane's chunks of gamma are requested with the row's and kept in registers (as
    // conditional loads inside the maximum and the code loops each of them was a trip to L2 of its own, twice)
    constexpr bool GREG = MODE == 2 && NIT > 0 && NIT <= 4;
    const Half16 no_gamma = Half16{uint4{0, 0, 0, 0}, uint4{0, 0, 0, 0}};
    float rnorm = 0.0f;              // MODE 2: 1 / sqrt(mean(x^2) + eps) of this lane's token
    auto widen = [](const Half16 &h, float (&f)[16]) {
        const unsigned w[8] = {h.lo.x, h.lo.y, h.lo.z, h.lo.w, h.hi.x, h.hi.y, h.hi.z, h.hi.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            f[2 * i] = half_bits_to_float(w[i] & 0xffffu);
            f[2 * i + 1] = half_bits_to_float(w[i] >> 16);
        }
    };
    const Half16 *row_up = nullptr;    // MODE 3: the up half of this lane's token
    auto smoothed = [&](const Half16 &h, int c, float (&f)[16], const Half16 &gch) {
        if constexpr (MODE == 3) {
            float u[16];
            widen(h, f);
            widen(row_up[c], u);
#pragma unroll
            for (int i = 0; i < 16; ++i) f[i] = swiglu_f32(f[i], u[i]);
            return;
        }
        if constexpr (MODE == 2) {
            float g[16];
            widen(h, f);
            if constexpr (GREG) widen(gch, g);
            else widen(reinterpret_cast<const Half16 *>(gamma)[c], g);
#pragma unroll
            for (int i = 0; i < 16; ++i) f[i] = (f[i] * rnorm) * g[i];
            return;
        }
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
    auto row_max = [&](const Half16 &h, int c, unsigned m, const Half16 &gch) {
        if (!SM) return abs_max_bits(h, m);
        float f[16];
        smoothed(h, c, f, gch);
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
    if (MODE == 3) row_up = reinterpret_cast<const Half16 *>(x + (size_t)(valid ? m : 0) * ldx + K);
    const int s0 = wave * per_wave;

    Half16 v[NIT > 0 ? NIT : 1];
    Half16 gv[GREG ? NIT : 1];
    unsigned mx = 0;
    // Rows kept in registers: all NIT chunks of a lane are requested at once, through range-checked buffer loads
    // with no branch around them (a chunk beyond the row, the wavefront's share or the last token gets an offset behind
    // the buffer and reads zeros, which change neither a maximum nor a sum of squares).  With a conditional load per
    // step the compiler waits for each step's data before it issues the next step's loads: one memory round trip per
    // step instead of one per row.  The buffer is the workgroup's RPB rows, so the 32-bit offsets hold for any M.
    auto load_row_chunks = [&]() {
        const int rows = M - (int)blockIdx.x * RPB < RPB ? M - (int)blockIdx.x * RPB : RPB;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<__half *>(x + (size_t)blockIdx.x * RPB * ldx), 0,
            (int)(((size_t)(rows - 1) * ldx + K) * sizeof(__half)), 0x00020000);
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = (s0 + i) * CPS + cl;
            const bool ok = i < per_wave && c < nchunks && valid;
            const unsigned off = ok ? (unsigned)r * (unsigned)ldx * 2u + (unsigned)c * 32u : 0xFFFFFFE0u;
            const v4u lo = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));
            const v4u hi = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(rs, off + 16u, 0, 0));
            v[i].lo = uint4{lo[0], lo[1], lo[2], lo[3]};
            v[i].hi = uint4{hi[0], hi[1], hi[2], hi[3]};
        }
        if constexpr (GREG) {
            const __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc(const_cast<__half *>(gamma), 0,
                                                                                K * (int)sizeof(__half), 0x00020000);
#pragma unroll
            for (int i = 0; i < NIT; ++i) {
                const int c = (s0 + i) * CPS + cl;
                const unsigned off = (i < per_wave && c < nchunks && valid) ? (unsigned)c * 32u : 0xFFFFFFE0u;
                const v4u lo = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(rg, off, 0, 0));
                const v4u hi = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(rg, off + 16u, 0, 0));
                gv[i].lo = uint4{lo[0], lo[1], lo[2], lo[3]};
                gv[i].hi = uint4{hi[0], hi[1], hi[2], hi[3]};
            }
        }
    };
    // MODE 3 with the row in registers: the fp32 values themselves are kept (the transform costs ~45 vector
    // operations per element, twice that if it were recomputed for the codes: the kernel is ALU-bound)
    constexpr bool KEEP32 = MODE == 3 && NIT > 0;
    float hv[KEEP32 ? NIT : 1][16];
    if constexpr (KEEP32) {
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = (s0 + i) * CPS + cl;
            if (i < per_wave && c < nchunks && valid) {
                smoothed(row[c], c, hv[i], no_gamma);
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = max(mx, __float_as_uint(fabsf(hv[i][e])));
            }
        }
    } else if constexpr (MODE == 2) {
        // sum of squares first (the maximum needs the normalised values); the row goes to registers on the way
        __shared__ double red_ss[MAX_RPB][MAX_WAVES];
        double ss = 0.0;
        auto add_squares = [&](const Half16 &h) {
            float f[16];
            widen(h, f);
#pragma unroll
            for (int i = 0; i < 16; ++i) ss += (double)(f[i] * f[i]);   // the product is exact in fp32
        };
        if (NIT > 0) {
            load_row_chunks();
#pragma unroll
            for (int i = 0; i < NIT; ++i) add_squares(v[i]);   // absent chunks hold zeros
        } else {
            for (int i = 0; i < per_wave; ++i) {
                const int c = (s0 + i) * CPS + cl;
                if (c < nchunks && valid) add_squares(row[c]);
            }
        }
#pragma unroll
        for (int off = 32; off >= RPB; off >>= 1) ss += __shfl_xor(ss, off, 64);
        if (cl == 0) red_ss[r][wave] = ss;
        __syncthreads();
        double tot = 0.0;
        for (int w = 0; w < nwaves; ++w) tot += red_ss[r][w];
        const float mean = (float)tot / (float)K;
        rnorm = 1.0f / sqrtf(mean + eps);
        if (NIT > 0) {
#pragma unroll
            for (int i = 0; i < NIT; ++i) {
                const int c = (s0 + i) * CPS + cl;
                if (i < per_wave && c < nchunks && valid) mx = row_max(v[i], c, mx, gv[GREG ? i : 0]);
            }
        } else {
            for (int i = 0; i < per_wave; ++i) {
                const int c = (s0 + i) * CPS + cl;
                if (c < nchunks && valid) mx = row_max(row[c], c, mx, no_gamma);
            }
        }
    } else if (NIT > 0 && !SM) {
        load_row_chunks();
#pragma unroll
        for (int i = 0; i < NIT; ++i) mx = abs_max_bits(v[i], mx);   // absent chunks hold zeros
    } else if (NIT > 0) {
        // (SmoothQuant: a step's scale vector is requested together with its chunk; with the chunks requested ahead of
        // all the scale vectors the kernel measured 18 % slower at K = 11008)
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = (s0 + i) * CPS + cl;
            if (i < per_wave && c < nchunks && valid) {
                v[i] = row[c];
                mx = row_max(v[i], c, mx, no_gamma);
            }
        }
    } else {
        for (int i = 0; i < per_wave; ++i) {
            const int c = (s0 + i) * CPS + cl;
            if (c < nchunks && valid) mx = row_max(row[c], c, mx, no_gamma);
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

    auto emit = [&](int c, const Half16 &h, const Half16 &gch) {
        uint4 q;
        if (SM) {
            float f[16];
            smoothed(h, c, f, gch);
            q = quant_chunk_f32(f, inv);
        } else {
            q = quant_chunk(h, inv);
        }
        if (xq_rm) *reinterpret_cast<uint4 *>(xq_rm + (size_t)m * K + (size_t)c * CHUNK) = q;
        if (xq_kl) *reinterpret_cast<uint4 *>(xq_kl + tile_offset_i8(m, c * CHUNK, K)) = q;
    };
    if constexpr (KEEP32) {
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = (s0 + i) * CPS + cl;
            if (i < per_wave && c < nchunks && valid) {
                const uint4 q = quant_chunk_f32(hv[i], inv);
                if (xq_rm) *reinterpret_cast<uint4 *>(xq_rm + (size_t)m * K + (size_t)c * CHUNK) = q;
                if (xq_kl) *reinterpret_cast<uint4 *>(xq_kl + tile_offset_i8(m, c * CHUNK, K)) = q;
            }
        }
    } else if (NIT > 0) {
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const int c = (s0 + i) * CPS + cl;
            if (i < per_wave && c < nchunks && valid) emit(c, v[i], gv[GREG ? i : 0]);
        }
    } else {
        for (int i = 0; i < per_wave; ++i) {
            const int c = (s0 + i) * CPS + cl;
            if (c < nchunks && valid) emit(c, row[c], no_gamma);
        }
    }
}

// The other quantizer forms of the Preliminary section (not the hot path; one workgroup per token, the row is
// read twice).  Eq. 1 as printed: code = rne(x / s) with the stored fp32 scale s (IEEE division), then Eq. 2's
// clamp.  range 1 = Eq. 2 as printed (s = 2 amax / 255, codes in [-128, 127]); scope: the token's own maximum,
// the whole tensor's (tensor_amax: its bit pattern, found by a kernel before this one) or a calibrated scale
// supplied by the caller (static_scale).  sx still gets one entry per token, so the GEMM epilogue is unchanged.
__device__ inline float act_scale_of(float amax, int range)
{
    return range == QL_RANGE_EQ2 ? (2.0f * amax) / 255.0f : amax / 127.0f;   // one IEEE fp32 division
}

__global__ __launch_bounds__(256) void act_quant_opt_kernel(const __half *__restrict__ x, int64_t ldx, int M, int K,
                                                            int range, const unsigned *__restrict__ tensor_amax,
                                                            const float *__restrict__ static_scale,
                                                            int8_t *__restrict__ xq_rm, int8_t *__restrict__ xq_kl,
                                                            float *__restrict__ sx)
{
    __shared__ unsigned red[4];
    const int m = blockIdx.x;
    const int nchunks = K / CHUNK;
    const Half16 *row = reinterpret_cast<const Half16 *>(x + (size_t)m * ldx);
    float s;
    if (static_scale) {
        s = *static_scale;
    } else if (tensor_amax) {
        s = act_scale_of(__uint_as_float(*tensor_amax), range);
    } else {
        unsigned mx = 0;
        for (int c = threadIdx.x; c < nchunks; c += 256) mx = abs_max_bits(row[c], mx);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = max(mx, (unsigned)__shfl_xor((int)mx, off, 64));
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
        __syncthreads();
        mx = max(max(red[0], red[1]), max(red[2], red[3]));
        s = act_scale_of(half_bits_to_float(mx), range);
    }
    if (s == 0.0f) s = 1.0f;
    if (threadIdx.x == 0) sx[m] = s;
    const float lo = range == QL_RANGE_EQ2 ? -128.0f : -127.0f;
    for (int c = threadIdx.x; c < nchunks; c += 256) {
        const Half16 h = row[c];
        const unsigned w[8] = {h.lo.x, h.lo.y, h.lo.z, h.lo.w, h.hi.x, h.hi.y, h.hi.z, h.hi.w};
        unsigned q[4] = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float v = half_bits_to_float((w[i / 2] >> (16 * (i % 2))) & 0xffffu);
            const float r = fminf(fmaxf(rintf(v / s), lo), 127.0f);   // IEEE fp32 division, ties to even, clamp
            q[i / 4] |= (unsigned)((int)r & 0xff) << (8 * (i % 4));
        }
        const uint4 o = make_uint4(q[0], q[1], q[2], q[3]);
        if (xq_rm) *reinterpret_cast<uint4 *>(xq_rm + (size_t)m * K + (size_t)c * CHUNK) = o;
        if (xq_kl) *reinterpret_cast<uint4 *>(xq_kl + tile_offset_i8(m, c * CHUNK, K)) = o;
    }
}

// max |x| over all tokens, as a bit pattern (accumulates into *out) or, with `as_scale`, as Eq. 2's scale for
// the given range (the scale is a non-decreasing function of the maximum, so the largest scale any workgroup
// derives is the scale of the largest value): a calibrated scale is the running maximum over batches
__global__ __launch_bounds__(256) void act_absmax_kernel(const __half *__restrict__ x, int64_t ldx, int M, int K,
                                                         int range, bool as_scale, unsigned *__restrict__ out)
{
    __shared__ unsigned red[4];
    const int nchunks = K / CHUNK;
    unsigned mx = 0;
    for (int m = blockIdx.x; m < M; m += gridDim.x) {
        const Half16 *row = reinterpret_cast<const Half16 *>(x + (size_t)m * ldx);
        for (int c = threadIdx.x; c < nchunks; c += 256) mx = abs_max_bits(row[c], mx);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = max(mx, (unsigned)__shfl_xor((int)mx, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        mx = max(max(red[0], red[1]), max(red[2], red[3]));
        const float amax = half_bits_to_float(mx);
        const float v = as_scale ? act_scale_of(amax, range) : amax;
        if (v > 0.0f) atomicMax(out, __float_as_uint(v));
    }
}

__global__ void fill_word_kernel(unsigned *p, unsigned v) { *p = v; }

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

// the row-in-registers kernels address a workgroup's 8 rows with 32-bit byte offsets
static int check_row_stride(int64_t ldx)
{
    if (ldx > ((int64_t)1 << 27)) return fail(QL_ERR_SHAPE, "row stride %lld beyond 2^27 elements", (long long)ldx);
    return QL_OK;
}

template <int RPB, int MODE>
static void launch_aq(const __half *x, int64_t ldx, int M, int K, const float *inv_smooth, const __half *gamma, float eps,
                      int8_t *xq_rm, int8_t *xq_kl, float *sx, hipStream_t st)
{
    const int steps = ceil_div(K / CHUNK, 64 / RPB);
    const int nw = steps < MAX_WAVES ? steps : MAX_WAVES;
    const int per_wave = ceil_div(steps, nw);
    dim3 grid(ceil_div(M, RPB)), block(nw * 64);
#define QL_LAUNCH_AQ(NIT) \
    hipLaunchKernelGGL((act_quant_kernel<NIT, RPB, MODE>), grid, block, 0, st, x, ldx, M, K, per_wave, inv_smooth, gamma, \
                       eps, xq_rm, xq_kl, sx)
    if (per_wave <= 1) QL_LAUNCH_AQ(1);
    else if (per_wave <= 2) QL_LAUNCH_AQ(2);
    else if (per_wave <= 4) QL_LAUNCH_AQ(4);
    else if (per_wave <= 8) QL_LAUNCH_AQ(8);
    else if (per_wave <= 12 && MODE != 3) QL_LAUNCH_AQ(12);
    else QL_LAUNCH_AQ(0);
#undef QL_LAUNCH_AQ
}

int launch_act_quant(const __half *x, int64_t ldx, int M, int K, int8_t *xq_rm, int8_t *xq_kl,
                     float *sx, hipStream_t st)
{
    if (M == 0) return QL_OK;
    QL_TRY(check_row_stride(ldx));
    if (M <= SINGLE_TOKEN_MAX_M) launch_aq<1, 0>(x, ldx, M, K, nullptr, nullptr, 0.0f, xq_rm, xq_kl, sx, st);
    else launch_aq<8, 0>(x, ldx, M, K, nullptr, nullptr, 0.0f, xq_rm, xq_kl, sx, st);
    return check_hip(hipGetLastError(), "act_quant launch");
}

int launch_act_quant_smooth(const __half *x, int64_t ldx, int M, int K, const float *inv_smooth, int8_t *xq_rm,
                            int8_t *xq_kl, float *sx, hipStream_t st)
{
    if (M == 0) return QL_OK;
    QL_TRY(check_row_stride(ldx));
    if (M <= SINGLE_TOKEN_MAX_M) launch_aq<1, 1>(x, ldx, M, K, inv_smooth, nullptr, 0.0f, xq_rm, xq_kl, sx, st);
    else launch_aq<8, 1>(x, ldx, M, K, inv_smooth, nullptr, 0.0f, xq_rm, xq_kl, sx, st);
    return check_hip(hipGetLastError(), "act_quant (smooth) launch");
}

int launch_act_quant_opt(const __half *x, int64_t ldx, int M, int K, int range, int scope,
                         const float *static_scale, unsigned *amax_scratch, int8_t *xq_rm, int8_t *xq_kl, float *sx,
                         hipStream_t st)
{
    if (M == 0) return QL_OK;
    const unsigned *ta = nullptr;
    if (scope == QL_SCOPE_TENSOR) {
        hipLaunchKernelGGL(fill_word_kernel, dim3(1), dim3(1), 0, st, amax_scratch, 0u);
        hipLaunchKernelGGL(act_absmax_kernel, dim3(M < 1024 ? M : 1024), dim3(256), 0, st, x, ldx, M, K, range, false,
                           amax_scratch);
        QL_TRY(check_hip(hipGetLastError(), "act_absmax launch"));
        ta = amax_scratch;
    }
    hipLaunchKernelGGL(act_quant_opt_kernel, dim3(M), dim3(256), 0, st, x, ldx, M, K, range, ta,
                       scope == QL_SCOPE_STATIC ? static_scale : nullptr, xq_rm, xq_kl, sx);
    return check_hip(hipGetLastError(), "act_quant (options) launch");
}

int launch_act_calibrate(const __half *x, int64_t ldx, int M, int K, int range, float *scale, hipStream_t st)
{
    if (M == 0) return QL_OK;
    hipLaunchKernelGGL(act_absmax_kernel, dim3(M < 1024 ? M : 1024), dim3(256), 0, st, x, ldx, M, K, range, true,
                       reinterpret_cast<unsigned *>(scale));
    return check_hip(hipGetLastError(), "act_calibrate launch");
}

int launch_act_quant_rmsnorm(const __half *x, int64_t ldx, int M, int K, const __half *gamma, float eps, int8_t *xq_rm,
                             int8_t *xq_kl, float *sx, hipStream_t st)
{
    if (M == 0) return QL_OK;
    QL_TRY(check_row_stride(ldx));
    if (M <= SINGLE_TOKEN_MAX_M) launch_aq<1, 2>(x, ldx, M, K, nullptr, gamma, eps, xq_rm, xq_kl, sx, st);
    else launch_aq<8, 2>(x, ldx, M, K, nullptr, gamma, eps, xq_rm, xq_kl, sx, st);
    return check_hip(hipGetLastError(), "act_quant (rmsnorm) launch");
}

int launch_act_quant_swiglu(const __half *gate_up, int64_t ld, int M, int K, int8_t *xq_rm, int8_t *xq_kl, float *sx,
                            hipStream_t st)
{
    if (M == 0) return QL_OK;
    // 8 tokens per workgroup keep up to 8192 features per token in registers, 4 tokens up to 16384
    if (M <= SINGLE_TOKEN_MAX_M) launch_aq<1, 3>(gate_up, ld, M, K, nullptr, nullptr, 0.0f, xq_rm, xq_kl, sx, st);
    else if (K <= 8192) launch_aq<8, 3>(gate_up, ld, M, K, nullptr, nullptr, 0.0f, xq_rm, xq_kl, sx, st);
    else launch_aq<4, 3>(gate_up, ld, M, K, nullptr, nullptr, 0.0f, xq_rm, xq_kl, sx, st);
    return check_hip(hipGetLastError(), "act_quant (swiglu) launch");
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
