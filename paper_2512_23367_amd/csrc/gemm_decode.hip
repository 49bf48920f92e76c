// Decode-shaped GEMM (at most 32 tokens) + dequantization epilogue of the W8A8 / W4A8 linear layer
// for gfx950.  Same arithmetic as the prefill kernel (integer accumulation, Y = XW, per-token and
// per-channel / per-group scales), but the time goes into streaming the weights from HBM once, so:
//   * one workgroup owns 16 output channels and the whole K; its 8 wavefronts split K and add their
//     exact integer (W8A8) or fp32 (W4A8) partial sums through LDS -- no atomics, no second pass;
//   * weight fragments go global -> registers with 16-byte (int8) or 8-byte (int4) loads per lane,
//     several in flight per wavefront, straight into the 16x16x64 int8 matrix instruction; nothing is
//     reused, so nothing is staged in LDS;
//   * the (at most 32) quantized tokens are re-read from L2 in the same tile order.
#include "common.h"

namespace ql {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));

enum { EPI_F16 = 0, EPI_ACC = 1 };
constexpr int WAVES = 8;

struct DecodeParams {
    const int8_t *xq;
    const char *wq;
    const float *sx;
    const float *sw;
    const __half *wscales;
    const __half *bias;
    __half *y;
    int64_t ldy;
    int32_t *acc;
    int32_t *partials;
    int row0, nrows;
    int M, N, K, Npad;
};

template <bool W4, int MH, int EPI>
__global__ __launch_bounds__(WAVES * 64) void gemm_decode_kernel(DecodeParams p)
{
    __shared__ int red[WAVES][MH][4][64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rg = blockIdx.x;                    // group of 16 output channels
    const int r = lane & 15, ch = lane >> 4;      // operand row and 16-k chunk of the 16x16x64 instruction
    const int KB = p.K / 32;

    // token operand: rows 0..15 (and 16..31) of row-block 0; 64 k = two consecutive 32-k tiles
    const char *xb = reinterpret_cast<const char *>(p.xq) + (ch / 2) * 1024 + (r + 32 * (ch % 2)) * 16;
    const int wl = (rg % 2) * 16 + r + 32 * (ch % 2);   // lane slot inside the 32-row weight tile

    v4i acc[MH];
    float accf[MH][4];
    int tot[MH][4];
#pragma unroll
    for (int h = 0; h < MH; ++h) {
        acc[h] = v4i{0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            accf[h][e] = 0.0f;
            tot[h][e] = 0;
        }
    }

    if (!W4) {
        const int nchunks = p.K / 64;
        const int per = (nchunks + WAVES - 1) / WAVES;
        const int c0 = wave * per, c1 = (c0 + per < nchunks) ? c0 + per : nchunks;
        const char *wb = p.wq + (size_t)(rg / 2) * KB * 1024 + (ch / 2) * 1024 + wl * 16;
        constexpr int U = 8;
        for (int c = c0; c < c1; c += U) {
            v4i wv[U], xv[MH][U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (c + u < c1) {
                    wv[u] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(wb + (size_t)(c + u) * 2048));
#pragma unroll
                    for (int h = 0; h < MH; ++h)
                        xv[h][u] = *reinterpret_cast<const v4i *>(xb + (size_t)(c + u) * 2048 + h * 256);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (c + u < c1) {
#pragma unroll
                    for (int h = 0; h < MH; ++h)
                        acc[h] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wv[u], xv[h][u], acc[h], 0, 0, 0);
                }
            }
        }
    } else {
        const int G = p.K / 128;
        const int per = (G + WAVES - 1) / WAVES;
        const int g0 = wave * per, g1 = (g0 + per < G) ? g0 + per : G;
        const char *wb = p.wq + (size_t)(rg / 2) * (p.K / 64) * 1024 + wl * 16 + (ch / 2) * 8;
        const __half *sgp = p.wscales + rg * 16 + 4 * ch;
        constexpr int U = 4;                      // groups per batch = 8 fragments in flight
        for (int g = g0; g < g1; g += U) {
            v2i wv[U][2];
            v4i xv[MH][U][2];
            h4 sg[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (g + u < g1) {
                    sg[u] = *reinterpret_cast<const h4 *>(sgp + (size_t)(g + u) * p.Npad);
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const size_t c = 2 * (size_t)(g + u) + t;
                        wv[u][t] = __builtin_nontemporal_load(reinterpret_cast<const v2i *>(wb + c * 1024));
#pragma unroll
                        for (int h = 0; h < MH; ++h)
                            xv[h][u][t] = *reinterpret_cast<const v4i *>(xb + c * 2048 + h * 256);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (g + u < g1) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const unsigned w0 = (unsigned)wv[u][t][0], w1 = (unsigned)wv[u][t][1];
                        v4i wf;
                        wf[0] = (int)((w0 << 4) & 0xF0F0F0F0u);
                        wf[1] = (int)(w0 & 0xF0F0F0F0u);
                        wf[2] = (int)((w1 << 4) & 0xF0F0F0F0u);
                        wf[3] = (int)(w1 & 0xF0F0F0F0u);
#pragma unroll
                        for (int h = 0; h < MH; ++h)
                            acc[h] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, xv[h][u][t], acc[h], 0, 0, 0);
                    }
#pragma unroll
                    for (int h = 0; h < MH; ++h) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            if (EPI == EPI_F16) {
                                accf[h][e] = __builtin_fmaf((float)acc[h][e], (float)sg[u][e], accf[h][e]);
                            } else {
                                tot[h][e] += acc[h][e];
                                if (p.partials) {
                                    const int m = r + 16 * h, n = rg * 16 + 4 * ch + e;
                                    if (m >= p.row0 && m < p.row0 + p.nrows && m < p.M && n < p.N)
                                        p.partials[((size_t)(m - p.row0) * G + (g + u)) * p.N + n] = acc[h][e] >> 4;
                                }
                            }
                        }
                        acc[h] = v4i{0, 0, 0, 0};
                    }
                }
            }
        }
    }

    // add the 8 wavefronts' partial sums (fixed order: the result does not depend on timing)
#pragma unroll
    for (int h = 0; h < MH; ++h)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int v;
            if (!W4) v = acc[h][e];
            else if (EPI == EPI_F16) v = __float_as_int(accf[h][e]);
            else v = tot[h][e];
            red[wave][h][e][lane] = v;
        }
    __syncthreads();
    if (wave != 0) return;

    const int n0 = rg * 16 + 4 * ch;
#pragma unroll
    for (int h = 0; h < MH; ++h) {
        const int m = r + 16 * h;
        int si[4] = {0, 0, 0, 0};
        float sf[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < WAVES; ++w)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (W4 && EPI == EPI_F16) sf[e] += __int_as_float(red[w][h][e][lane]);
                else si[e] += red[w][h][e][lane];
            }
        if (m >= p.M || n0 >= p.N) continue;
        if (EPI == EPI_ACC) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (n0 + e < p.N) p.acc[(size_t)m * p.N + n0 + e] = W4 ? (si[e] >> 4) : si[e];
            continue;
        }
        const float sxm = p.sx[m] * (W4 ? 0.0625f : 1.0f);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (n0 + e >= p.N) break;
            const float b = p.bias ? __half2float(p.bias[n0 + e]) : 0.0f;
            float v;
            if (W4) v = __builtin_fmaf(sf[e], sxm, b);
            else v = __builtin_fmaf((float)si[e] * sxm, p.sw[n0 + e], b);
            p.y[(size_t)m * p.ldy + n0 + e] = __float2half_rn(v);
        }
    }
}

template <bool W4, int MH, int EPI>
int launch_one(const GemmArgs &a, hipStream_t st)
{
    DecodeParams p;
    p.xq = a.xq;
    p.wq = static_cast<const char *>(a.wq);
    p.sx = a.sx;
    p.sw = a.sw;
    p.bias = a.bias;
    p.y = a.y;
    p.ldy = a.ldy;
    p.acc = a.acc;
    p.partials = a.partials;
    p.row0 = a.row0;
    p.nrows = a.nrows;
    p.M = a.M;
    p.N = a.N;
    p.K = a.K;
    p.Npad = round_up(a.N, TILE_ROWS);
    p.wscales = W4 ? reinterpret_cast<const __half *>(p.wq + w4_scales_offset(a.N, a.K)) : nullptr;
    const int grid = p.Npad / 16;
    hipLaunchKernelGGL((gemm_decode_kernel<W4, MH, EPI>), dim3(grid), dim3(WAVES * 64), 0, st, p);
    return check_hip(hipGetLastError(), "gemm_decode launch");
}

template <bool W4, int EPI>
int by_m(const GemmArgs &a, hipStream_t st)
{
    return a.M <= 16 ? launch_one<W4, 1, EPI>(a, st) : launch_one<W4, 2, EPI>(a, st);
}

}  // namespace

int launch_gemm_decode(const GemmArgs &a, int variant, hipStream_t st)
{
    (void)variant;
    if (a.M == 0) return QL_OK;
    const bool dump = a.acc != nullptr;
    if (a.bits == 4) return dump ? by_m<true, EPI_ACC>(a, st) : by_m<true, EPI_F16>(a, st);
    return dump ? by_m<false, EPI_ACC>(a, st) : by_m<false, EPI_F16>(a, st);
}

}  // namespace ql
