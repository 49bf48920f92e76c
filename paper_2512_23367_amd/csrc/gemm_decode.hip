// Weight-streaming GEMM + dequantization epilogue of the W8A8 / W4A8 linear layer for gfx950: the decode
// shapes (up to 32 tokens per call) and, in blocks of 64 or 32 tokens, up to 1024 tokens where that is faster than
// the prefill tile kernels.  Same arithmetic as the prefill kernel (integer accumulation, Y = XW, per-token and
// per-channel / per-group scales), but the time goes into streaming the weights from HBM once, so:
//   * one workgroup owns 16 C output channels (C = 1..8) and the whole K; its 8 (or 16) wavefronts split K and add their
//     exact integer (W8A8) or fp32 (W4A8) partial sums through LDS -- no atomics, no second pass;
//   * weight fragments go global -> registers with 16-byte loads per lane, a ring of them in flight
//     per wavefront, straight into the 16x16x64 int8 matrix instruction (int4: after a shift/mask
//     unpack); nothing is reused, so nothing is staged in LDS;
//   * the quantized tokens (of the workgroup's block) are re-read from L2 in the same tile order, or staged in LDS when
//     they are few; for up to four tokens the linear-layer entry points skip the separate quantization
//     kernel and every workgroup quantizes the fp16 tokens itself on the way into LDS (paper Eq. 1-2,
//     same arithmetic as the stand-alone quantizer), while its first weight fragments are in flight.
#include "common.h"
#include "quant_math.h"

#ifndef QL_RING8
#define QL_RING8 8     // weight fragments (1 KiB each) a wavefront keeps in flight, int8 weights
#endif
#ifndef QL_RING4
#define QL_RING4 4     // the same for int4 weights
#endif

namespace ql {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));

enum { EPI_F16 = 0, EPI_ACC = 1 };

struct DecodeParams {
    const __half *x;         // fused quantization: fp16 tokens [M, ldx]
    int64_t ldx;
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
    unsigned x_bytes, w_bytes;   // sizes of the quantized tokens and of the weight codes (range-checked loads)
};

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// C: groups of 16 output channels per workgroup (they share every token fragment that is loaded).
// XL: the (few) quantized tokens are staged once per workgroup in LDS, [k-tile half][token] with one extra
// all-zero token row that the lanes of absent tokens read; the ring then holds weights only.
// FQ > 0: the tokens arrive as fp16 and are quantized here (XL staging with the quantizer in front of it); a lane
// keeps FQ (= 2) pieces of 16 k in registers.
// Measured: up to 4 tokens and K <= 4096 (8192 for two, 12288 for one) the fused form wins 0.7-2.4 us per
// linear; at 8 tokens, or with twice the pieces per lane, every workgroup re-quantizing all tokens costs more
// than the separate launch.
constexpr int FQ_MAX_M = 4;
constexpr size_t FQ_MAX_LDS = 24576;   // staged tokens (M + 1) * K bytes: four workgroups per CU still fit
// OVL (fused quantizer only): the first ring of weights is loaded without conditions, see the int8 loop.
template <bool W4, int MH, int C, int EPI, int WAVES, bool XL, int FQ, bool OVL>
__global__ __launch_bounds__(WAVES * 64) void gemm_decode_kernel(DecodeParams p)
{
    static_assert(!FQ || (XL && EPI == EPI_F16), "fused quantization stages the tokens in LDS");
    constexpr int RH = MH < 2 ? MH : (C > 4 ? 1 : 2);     // token halves that meet in LDS at a time (at most 64 KiB)
    __shared__ int red[WAVES][C][RH][4][64];
    __shared__ unsigned amax_red[FQ ? WAVES : 1][FQ_MAX_M];
    extern __shared__ __attribute__((aligned(16))) char dyn_lds[];
    // W4A8: the group scales of this workgroup's C*16 channels, [C][K/128][16] fp16, then
    // XL: the staged tokens, (M + 1) * K bytes
    char *ss = dyn_lds;
    char *xs = dyn_lds + (W4 ? (size_t)C * (p.K / 128) * 32 : 0);
    static_assert(!XL || MH == 1, "LDS-staged tokens: at most 16 tokens");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (MH >= 2) {   // more tokens than the kernel's 16 * MH: blockIdx.y picks a block of them
        const int t0 = 16 * MH * blockIdx.y;
        p.xq += (size_t)t0 * p.K;
        p.x_bytes -= (unsigned)t0 * p.K;
        if (p.sx) p.sx += t0;
        if (p.y) p.y += (size_t)t0 * p.ldy;
        if (p.acc) p.acc += (size_t)t0 * p.N;
        p.row0 -= t0;
        p.M = p.M - t0 < 16 * MH ? p.M - t0 : 16 * MH;
    }
    const int rg0 = blockIdx.x * C;               // first group of 16 output channels
    const int r = lane & 15, ch = lane >> 4;      // operand row and 16-k chunk of the 16x16x64 instruction
    const int KB = p.K / 32;
    const int ngroups = p.Npad / 16;

    // token operand: rows 0..15 (16..31, then the same of row-block 1); 64 k = two consecutive 32-k tiles.
    // Rows >= M hold nothing: their lanes load nothing, which keeps the L2 traffic at M/16 of the weights'.
    const char *xb = reinterpret_cast<const char *>(p.xq) + (ch / 2) * 1024 + (r + 32 * (ch % 2)) * 16;
    bool xlive[MH];
#pragma unroll
    for (int h = 0; h < MH; ++h) xlive[h] = r + 16 * h < p.M;
    const int wl = r + 32 * (ch % 2);             // lane slot inside the 32-row weight tile, + 16 for odd groups

    v4i acc[C][MH];
    float accf[C][MH][4];
    int tot[C][MH][4];
#pragma unroll
    for (int j = 0; j < C; ++j)
#pragma unroll
        for (int h = 0; h < MH; ++h) {
            acc[j][h] = v4i{0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                accf[j][h][e] = 0.0f;
                tot[j][h][e] = 0;
            }
        }

    // The scales and bias the finishing wavefronts (w < C handles channel group w) will need are requested before the
    // main loop and stay in registers as loaded: the epilogue does not end with a dependent trip to memory, and nothing
    // waits for them before it (a conversion or a branch around a load would).  Range-checked buffer loads: tokens
    // beyond M, channels beyond N and absent operands (zero-length buffers) read 0 without a branch.  Where the ring is
    // refilled through counted buffer loads (17 tokens and more) they go out first, so that the loop's wait counts stay
    // exact; in the other loops right behind the first ring of weights -- in front of it, a register that one of them
    // loads into can be wanted for a weight address, which costs the finishing wavefronts a memory round trip.
    constexpr bool COUNTED_RING = !XL && MH >= 2 && (!W4 || WAVES == 8);
    int e_sx_raw[MH], e_sw_raw[4];
    int e_b_raw[4];         // fp16 bits, zero-extended
    float e_sx_fq = 0.0f;   // fused quantizer: the token scale is computed below
#pragma unroll
    for (int h = 0; h < MH; ++h) e_sx_raw[h] = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) e_sw_raw[e] = 0, e_b_raw[e] = 0;
    auto request_finish_operands = [&]() {
        // (fused quantizer overlapping the first ring: every wavefront requests them, first of all -- without a branch
        // around them the compiler can count them, so that the wait for the tokens does not include the weights)
        if (EPI == EPI_F16 && ((FQ > 0 && OVL) || wave < C)) {   // wave-uniform
            const unsigned n0 = (unsigned)((rg0 + wave) * 16 + 4 * ch);
            const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.sx, (!FQ && p.sx) ? (unsigned)p.M * 4u : 0u);
            const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.sw, (!W4 && p.sw) ? (unsigned)p.N * 4u : 0u);
            const __amdgpu_buffer_rsrc_t rb = make_rsrc(p.bias, p.bias ? (unsigned)p.N * 2u : 0u);
#pragma unroll
            for (int h = 0; h < MH; ++h) e_sx_raw[h] = __builtin_amdgcn_raw_buffer_load_b32(rx, (unsigned)(r + 16 * h) * 4u, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                e_sw_raw[e] = __builtin_amdgcn_raw_buffer_load_b32(rw, (n0 + e) * 4u, 0, 0);
                e_b_raw[e] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rb, (n0 + e) * 2u, 0, 0);
            }
        }
    };
    if (COUNTED_RING || (FQ > 0 && OVL)) request_finish_operands();

    // byte offset of channel group rg0+j inside the weight blob, for this lane
    size_t wgo[C];
    bool glive[C];
#pragma unroll
    for (int j = 0; j < C; ++j) {
        const int rg = rg0 + j;
        glive[j] = rg < ngroups;
        const int g2 = glive[j] ? rg : 0;
        if (!W4) wgo[j] = (size_t)(g2 / 2) * KB * 1024 + (ch / 2) * 1024 + ((g2 % 2) * 16 + wl) * 16;
        else wgo[j] = (size_t)(g2 / 2) * (p.K / 64) * 1024 + (ch / 2) * 1024 + ((g2 % 2) * 16 + wl) * 16;
    }

    // XL: copy tokens 0..M-1 from the tile order into xs[(k-tile * 2 + half) * (M + 1) + token] and clear row M
    const int xrows = p.M + 1;
    const int xrow = (r < p.M) ? r : p.M;
    // Every wavefront stages only the k-range it multiplies (tile-halves th0 .. th1-1), so no workgroup
    // barrier is needed: a wavefront's LDS operations complete in order.
    auto stage_tokens = [&](int th0, int th1) {
        const int pieces = (th1 - th0) * xrows;
        for (int i = lane; i < pieces; i += 64) {
            const int th = th0 + i / xrows, row = i % xrows;
            v4i v = v4i{0, 0, 0, 0};
            if (row < p.M)
                v = *reinterpret_cast<const v4i *>(reinterpret_cast<const char *>(p.xq) + (size_t)(th / 2) * 1024 +
                                                   (row + 32 * (th % 2)) * 16);
            *reinterpret_cast<v4i *>(xs + ((size_t)th * xrows + row) * 16) = v;
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_wave_barrier();
    };

    // FQ: quantize tokens 0..M-1 (M <= FQ_MAX_M) over this wavefront's 16-k pieces th0 .. th1-1 into the same
    // LDS layout.  The fp16 pieces are loaded BEFORE the first weight fragments are requested and stay in
    // registers (loads return in order: behind the weight stream they would arrive an HBM latency late);
    // the row maxima of the wavefronts' k-ranges meet in LDS (one workgroup barrier, reached by every
    // wavefront), then the codes are produced from the registers while the weights are still in flight.
    // With Mp = M rounded up to a power of two, lane l works on token l % Mp (always the same one: a token's
    // maximum needs no bookkeeping) and, in slot sl, on piece th0 + sl * (64 / Mp) + l / Mp; the host makes sure
    // that FQ slots cover the wavefront's pieces.
    constexpr int FQ_SLOTS = FQ > 0 ? FQ : 1;
    Half16 keep[FQ_SLOTS];
    const int fq_lg = p.M <= 1 ? 0 : p.M <= 2 ? 1 : 2;   // log2(Mp)
    const int fq_m = lane & ((1 << fq_lg) - 1);        // this lane's token (absent when >= M)
    const int fq_ppr = 64 >> fq_lg;                     // pieces per slot
    auto load_tokens = [&](int th0, int th1) {
#pragma unroll
        for (int sl = 0; sl < FQ_SLOTS; ++sl) {
            const int i = th0 + sl * fq_ppr + (lane >> fq_lg);
            keep[sl] = Half16{uint4{0, 0, 0, 0}, uint4{0, 0, 0, 0}};
            if (i < th1 && fq_m < p.M) keep[sl] = *reinterpret_cast<const Half16 *>(p.x + (size_t)fq_m * p.ldx + (size_t)i * 16);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto quantize_tokens = [&](int th0, int th1) {
        unsigned mx = 0;
#pragma unroll
        for (int sl = 0; sl < FQ_SLOTS; ++sl) mx = abs_max_bits(keep[sl], mx);   // pieces beyond the range hold zeros
        for (int off = 32; off >= (1 << fq_lg); off >>= 1) mx = max(mx, (unsigned)__shfl_xor((int)mx, off, 64));
        if (lane < (1 << fq_lg)) amax_red[wave][lane] = mx;
        __syncthreads();
        unsigned a = 0;
        for (int w = 0; w < WAVES; ++w) a = max(a, amax_red[w][fq_m]);
        float scale, inv;
        token_scales(a, scale, inv);
        // the finishing lanes want the scale of token r: for r < M that is this lane's own token (Mp divides 16)
        e_sx_fq = (r < p.M) ? scale * (W4 ? 0.0625f : 1.0f) : 0.0f;
#pragma unroll
        for (int sl = 0; sl < FQ_SLOTS; ++sl) {
            const int i = th0 + sl * fq_ppr + (lane >> fq_lg);
            if (i < th1 && fq_m < p.M) {
                *reinterpret_cast<uint4 *>(xs + ((size_t)i * xrows + fq_m) * 16) = quant_chunk(keep[sl], inv);
                if (fq_m == 0) *reinterpret_cast<uint4 *>(xs + ((size_t)i * xrows + p.M) * 16) = uint4{0, 0, 0, 0};
            }
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_wave_barrier();
    };

    // Both loops keep a ring of U weight fragments (1 KiB each per wavefront) in flight: slot u is
    // consumed, then immediately refilled with the fragment U steps ahead.
    if (!W4) {
        const int nchunks = p.K / 64;
        const int per = (nchunks + WAVES - 1) / WAVES;
        const int c0 = wave * per, c1 = (c0 + per < nchunks) ? c0 + per : nchunks;
        constexpr int U = C >= QL_RING8 ? 1 : (QL_RING8 + C - 1) / C;
        v4i wv[U][C], xv[XL ? 1 : U][MH];
        const int th0 = 4 * c0, th1 = c0 < c1 ? 4 * c1 : 4 * c0;
        if constexpr (!XL && MH >= 2) {
            // Tokens from L2, 17 tokens and more (measured on one box against conditional pointer loads: 1-9 % faster
            // at 32 and 64 tokens, 1-5 % slower with 16 tokens or fewer, which keep the loop below): every ring slot takes C weight and MH token fragments through range-checked buffer
            // loads.  Absent channel groups and token rows get a lane offset behind the buffer, and chunks past this
            // wavefront's range a buffer of zero length: such loads return zeros and cost no traffic.  Every slot
            // therefore issues the same loads in the same order with no branch around them, and the waits the
            // compiler inserts count exactly: U - 1 slots stay in flight while one is multiplied (with conditional
            // loads it waited for all of them before every slot).
            constexpr unsigned OOB = 0xFFFFF000u;
            unsigned wo[C], xo[MH];
#pragma unroll
            for (int j = 0; j < C; ++j) wo[j] = glive[j] ? (unsigned)wgo[j] : OOB;
#pragma unroll
            for (int h = 0; h < MH; ++h)
                xo[h] = xlive[h] ? (unsigned)((size_t)(h / 2) * KB * 1024 + (ch / 2) * 1024 + (r + 32 * (ch % 2)) * 16 + (h % 2) * 256)
                                 : OOB;
            auto fetch = [&](int u, int c) {
                const bool in = c < c1;
                const __amdgpu_buffer_rsrc_t wr = make_rsrc(p.wq, in ? p.w_bytes : 0u);
                const __amdgpu_buffer_rsrc_t xr = make_rsrc(p.xq, in ? p.x_bytes : 0u);
                const unsigned so = (unsigned)c * 2048u;   // scalar offset: added to the address, not range-checked
#pragma unroll
                for (int j = 0; j < C; ++j)
                    wv[u][j] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(wr, wo[j], so, 2));
#pragma unroll
                for (int h = 0; h < MH; ++h)
                    xv[u][h] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(xr, xo[h], so, 0));
            };
#pragma unroll
            for (int u = 0; u < U; ++u) fetch(u, c0 + u);
            auto multiply = [&](int u) {
#pragma unroll
                for (int j = 0; j < C; ++j)
#pragma unroll
                    for (int h = 0; h < MH; ++h)
                        acc[j][h] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wv[u][j], xv[u][h], acc[j][h], 0, 0, 0);
            };
            int c = c0;
            for (; c + U <= c1; c += U) {   // whole rounds of the ring: no branch inside
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    multiply(u);
                    __builtin_amdgcn_sched_barrier(0);   // keep the refill right behind its slot's last use:
                    fetch(u, c + U + u);                 // the scheduler would sink all refills to the loop's end
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int u = 0; u < U - 1; ++u)   // the last, partial round (its chunks are already on their way)
                if (c + u < c1) multiply(u);
        } else {
            auto fetch = [&](int u, int c) {
                if (c < c1) {
#pragma unroll
                    for (int j = 0; j < C; ++j)
                        wv[u][j] = glive[j] ? __builtin_nontemporal_load(
                                                  reinterpret_cast<const v4i *>(p.wq + wgo[j] + (size_t)c * 2048))
                                            : v4i{0, 0, 0, 0};
                    if (!XL) {
#pragma unroll
                        for (int h = 0; h < MH; ++h)
                            xv[u][h] = xlive[h] ? *reinterpret_cast<const v4i *>(xb + (size_t)(h / 2) * KB * 1024 + (size_t)c * 2048 + (h % 2) * 256)
                                                : v4i{0, 0, 0, 0};
                    }
                }
            };
            if (FQ) load_tokens(th0, th1);
            if constexpr (FQ > 0 && OVL) {
                // Fused quantizer, at most one workgroup per CU (the host's choice): the first ring is loaded without
                // conditions (a chunk past the wavefront's range repeats the last chunk of the matrix, an absent channel
                // group reads group 0; neither is multiplied into anything that is stored).  With a branch around a load
                // the compiler cannot count the loads in flight and waits for all of them -- the weights included --
                // before the tokens are quantized; counted, the quantizer runs while the weights are on their way
                // (O projection, one token: 6.7 -> 5.5 us).  With several workgroups per CU the conditional form
                // measured faster (a CU then overlaps one workgroup's quantizer with another's wait anyway).
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = c0 + u < nchunks ? c0 + u : nchunks - 1;
#pragma unroll
                    for (int j = 0; j < C; ++j)
                        wv[u][j] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(p.wq + wgo[j] + (size_t)c * 2048));
                }
                quantize_tokens(th0, th1);
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) fetch(u, c0 + u);
                if (!COUNTED_RING) request_finish_operands();
                if (FQ) quantize_tokens(th0, th1);
                else if (XL && c0 < c1) stage_tokens(4 * c0, 4 * c1);
            }
            for (int c = c0; c < c1; c += U) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (c + u < c1) {
                        if (XL) xv[0][0] = *reinterpret_cast<const v4i *>(xs + ((size_t)(4 * (c + u) + ch) * xrows + xrow) * 16);
#pragma unroll
                        for (int j = 0; j < C; ++j)
#pragma unroll
                            for (int h = 0; h < MH; ++h)
                                acc[j][h] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wv[u][j], xv[XL ? 0 : u][h], acc[j][h], 0, 0, 0);
                    }
                    fetch(u, c + U + u);
                }
            }
        }
    } else {
        // One 16-byte load per lane covers one scale group (128 k): words 0,1 feed the first matrix
        // instruction (k-blocks 4g, 4g+2 over the four lane chunks), words 2,3 the second (4g+1, 4g+3).
        const int G = p.K / 128;
        const int per = (G + WAVES - 1) / WAVES;
        const int g0 = wave * per, g1 = (g0 + per < G) ? g0 + per : G;
        const char *xb4 = reinterpret_cast<const char *>(p.xq) + (2 * (ch / 2)) * 1024 + (r + 32 * (ch % 2)) * 16;
                // a short ring keeps the register count low: more resident workgroups hide a workgroup's serial
        // load -> unpack -> multiply -> fold -> reduce chain better than a deeper ring does
        constexpr int U = C >= QL_RING4 ? 1 : (QL_RING4 + C - 1) / C;   // without XL a slot also holds token fragments
        v4i wv[U][C], xv[XL ? 1 : U][2][MH];
        // 17 tokens and more (8 wavefronts; the accumulator dump runs the same loop): branch-free refills through range-checked buffer loads, as
        // in the int8 loop above (absent rows and channel groups: lane offset behind the buffer; groups past this
        // wavefront's range: a buffer of zero length).  Measured on one box against the conditional pointer loads:
        // 2-10 % faster at 64 tokens, 1-4 % at 128, 3-5 % slower with 16 wavefronts (kept on the old loop).
        constexpr bool BR = !XL && MH >= 2 && WAVES == 8;
        constexpr unsigned OOB = 0xFFFFF000u;
        unsigned wo[C], xo[MH];
#pragma unroll
        for (int j = 0; j < C; ++j) wo[j] = glive[j] ? (unsigned)wgo[j] : OOB;
#pragma unroll
        for (int h = 0; h < MH; ++h)
            xo[h] = xlive[h] ? (unsigned)((size_t)(h / 2) * KB * 1024 + (2 * (ch / 2)) * 1024 + (r + 32 * (ch % 2)) * 16 + (h % 2) * 256)
                             : OOB;
        auto fetch = [&](int u, int g) {
            if constexpr (BR) {
                const bool in = g < g1;
                const __amdgpu_buffer_rsrc_t wr = make_rsrc(p.wq, in ? p.w_bytes : 0u);
                const __amdgpu_buffer_rsrc_t xr = make_rsrc(p.xq, in ? p.x_bytes : 0u);
#pragma unroll
                for (int j = 0; j < C; ++j)
                    wv[u][j] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(wr, wo[j], (unsigned)g * 2048u, 2));
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int h = 0; h < MH; ++h)
                        xv[u][t][h] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(
                                                                   xr, xo[h], ((unsigned)4 * g + t) * 1024u, 0));
                return;
            }
            if (g < g1) {
#pragma unroll
                for (int j = 0; j < C; ++j) {
                    wv[u][j] = glive[j] ? __builtin_nontemporal_load(
                                              reinterpret_cast<const v4i *>(p.wq + wgo[j] + (size_t)g * 2048))
                                        : v4i{0, 0, 0, 0};

                }
                if (!XL) {
#pragma unroll
                    for (int t = 0; t < 2; ++t)
#pragma unroll
                        for (int h = 0; h < MH; ++h)
                            xv[u][t][h] = xlive[h] ? *reinterpret_cast<const v4i *>(xb4 + (size_t)(h / 2) * KB * 1024 + ((size_t)4 * g + t) * 1024 + (h % 2) * 256)
                                                   : v4i{0, 0, 0, 0};
                }
            }
        };
        const int th0 = 8 * g0, th1 = g0 < g1 ? 8 * g1 : 8 * g0;
        if (FQ) load_tokens(th0, th1);
        // The group scales of this wavefront's groups g0..g1-1 for the C channel groups ((g1-g0)*32 contiguous bytes
        // each in the blob's decode-ordered copy [channel group][K/128][16]) and, with XL, the quantized tokens of its
        // k-range are requested BEFORE the first weight fragments and parked in registers: loads return in order, so
        // they arrive first and are copied to LDS while the weights are still on their way.  (Requested after the
        // weights, each staging step was one more full trip to memory in front of the first multiply.)
        constexpr int SREG = 2, TREG = 3;              // 16-byte pieces per lane parked in registers
        const int n16 = (g1 - g0) * 2;                 // 16-byte scale pieces per channel group
        const int spieces = g0 < g1 ? C * n16 : 0;
        const int tpieces = (XL && !FQ && g0 < g1) ? (th1 - th0) * xrows : 0;
        const bool s_regs = spieces <= 64 * SREG, t_regs = tpieces <= 64 * TREG;
        v4i sreg[SREG], treg[TREG];
        if (s_regs) {
#pragma unroll
            for (int q = 0; q < SREG; ++q) {
                const int i = lane + 64 * q;
                sreg[q] = v4i{0, 0, 0, 0};
                if (i < spieces && rg0 + i / n16 < ngroups)
                    sreg[q] = *reinterpret_cast<const v4i *>(reinterpret_cast<const char *>(p.wscales) +
                                                             ((size_t)(rg0 + i / n16) * G + g0) * 32 + (size_t)(i % n16) * 16);
            }
        }
        if (XL && !FQ && t_regs) {
#pragma unroll
            for (int q = 0; q < TREG; ++q) {
                const int i = lane + 64 * q;
                treg[q] = v4i{0, 0, 0, 0};
                if (i < tpieces && i % xrows < p.M) {
                    const int th = th0 + i / xrows, row = i % xrows;
                    treg[q] = *reinterpret_cast<const v4i *>(reinterpret_cast<const char *>(p.xq) + (size_t)(th / 2) * 1024 +
                                                             (row + 32 * (th % 2)) * 16);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);             // keep these requests in front of the weights'
        if constexpr (FQ > 0 && OVL) {   // unconditional first ring, as in the int8 loop
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int g = g0 + u < G ? g0 + u : G - 1;
#pragma unroll
                for (int j = 0; j < C; ++j)
                    wv[u][j] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(p.wq + wgo[j] + (size_t)g * 2048));
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) fetch(u, g0 + u);
        }
        if (!COUNTED_RING && !(FQ > 0 && OVL)) request_finish_operands();
        if (g0 < g1) {
            if (s_regs) {
#pragma unroll
                for (int q = 0; q < SREG; ++q) {
                    const int i = lane + 64 * q;
                    if (i < spieces)
                        *reinterpret_cast<v4i *>(ss + ((size_t)(i / n16) * G + g0) * 32 + (size_t)(i % n16) * 16) = sreg[q];
                }
            } else {
                for (int i = lane; i < spieces; i += 64) {
                    const int j = i / n16, o = i % n16;
                    v4i v = v4i{0, 0, 0, 0};
                    if (rg0 + j < ngroups)
                        v = *reinterpret_cast<const v4i *>(reinterpret_cast<const char *>(p.wscales) +
                                                           ((size_t)(rg0 + j) * G + g0) * 32 + (size_t)o * 16);
                    *reinterpret_cast<v4i *>(ss + ((size_t)j * G + g0) * 32 + (size_t)o * 16) = v;
                }
            }
            if (XL && !FQ) {
                if (t_regs) {
#pragma unroll
                    for (int q = 0; q < TREG; ++q) {
                        const int i = lane + 64 * q;
                        if (i < tpieces)
                            *reinterpret_cast<v4i *>(xs + ((size_t)(th0 + i / xrows) * xrows + i % xrows) * 16) = treg[q];
                    }
                } else {
                    stage_tokens(8 * g0, 8 * g1);
                }
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
        }
        if (FQ) quantize_tokens(th0, th1);
        auto consume = [&](int u, int gg) {   // scale group gg from ring slot u: unpack, multiply, fold
            if (XL) {
#pragma unroll
                for (int t = 0; t < 2; ++t)   // k-tile 4g + 2(ch/2) + t, half ch%2
                    xv[0][t][0] = *reinterpret_cast<const v4i *>(
                        xs + ((size_t)((4 * gg + 2 * (ch / 2) + t) * 2 + (ch % 2)) * xrows + xrow) * 16);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int j = 0; j < C; ++j) {
                    const unsigned w0 = (unsigned)wv[u][j][2 * t], w1 = (unsigned)wv[u][j][2 * t + 1];
                    v4i wf;
                    wf[0] = (int)((w0 << 4) & 0xF0F0F0F0u);
                    wf[1] = (int)(w0 & 0xF0F0F0F0u);
                    wf[2] = (int)((w1 << 4) & 0xF0F0F0F0u);
                    wf[3] = (int)(w1 & 0xF0F0F0F0u);
#pragma unroll
                    for (int h = 0; h < MH; ++h)
                        acc[j][h] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, xv[XL ? 0 : u][t][h], acc[j][h], 0, 0, 0);
                }
            h4 sgv[C];
#pragma unroll
            for (int j = 0; j < C; ++j)
                sgv[j] = *reinterpret_cast<const h4 *>(ss + ((size_t)(j * G + gg) * 16 + 4 * ch) * 2);
#pragma unroll
            for (int j = 0; j < C; ++j)
#pragma unroll
                for (int h = 0; h < MH; ++h) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (EPI == EPI_F16) {
                            accf[j][h][e] = __builtin_fmaf((float)acc[j][h][e], (float)sgv[j][e], accf[j][h][e]);
                        } else {
                            tot[j][h][e] += acc[j][h][e];
                            if (p.partials) {
                                const int m = r + 16 * h, n = (rg0 + j) * 16 + 4 * ch + e;
                                if (m >= p.row0 && m < p.row0 + p.nrows && m < p.M && n < p.N)
                                    p.partials[((size_t)(m - p.row0) * G + gg) * p.N + n] = acc[j][h][e] >> 4;
                            }
                        }
                    }
                    acc[j][h] = v4i{0, 0, 0, 0};
                }
        };
        if constexpr (BR) {
            int g = g0;
            for (; g + U <= g1; g += U) {   // whole rounds of the ring: no branch inside
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    consume(u, g + u);
                    __builtin_amdgcn_sched_barrier(0);
                    fetch(u, g + U + u);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int u = 0; u < U - 1; ++u)
                if (g + u < g1) consume(u, g + u);
        } else {
            for (int g = g0; g < g1; g += U) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (g + u < g1) consume(u, g + u);
                    fetch(u, g + U + u);
                }
            }
        }
    }

    // add the wavefronts' partial sums (fixed order: the result does not depend on timing), RH token halves
    // at a time; wavefront w finishes channel group w (C <= WAVES)
#pragma unroll
    for (int hb = 0; hb < MH; hb += RH) {
        if (hb) __syncthreads();                          // the previous halves have been read
#pragma unroll
        for (int j = 0; j < C; ++j)
#pragma unroll
            for (int hh = 0; hh < RH; ++hh)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    int v;
                    if (!W4) v = acc[j][hb + hh][e];
                    else if (EPI == EPI_F16) v = __float_as_int(accf[j][hb + hh][e]);
                    else v = tot[j][hb + hh][e];
                    red[wave][j][hh][e][lane] = v;
                }
        __syncthreads();
        if (wave < C) {
            const int j = wave;
            const int n0 = (rg0 + j) * 16 + 4 * ch;
#pragma unroll
            for (int hh = 0; hh < RH; ++hh) {
                const int h = hb + hh;
                const int m = r + 16 * h;
                int si[4] = {0, 0, 0, 0};
                float sf[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int w = 0; w < WAVES; ++w)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (W4 && EPI == EPI_F16) sf[e] += __int_as_float(red[w][j][hh][e][lane]);
                        else si[e] += red[w][j][hh][e][lane];
                    }
                if (m >= p.M || n0 >= p.N) continue;
                if (EPI == EPI_ACC) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n0 + e < p.N) p.acc[(size_t)m * p.N + n0 + e] = W4 ? (si[e] >> 4) : si[e];
                    continue;
                }
                const float sxm = FQ ? e_sx_fq : __int_as_float(e_sx_raw[h]) * (W4 ? 0.0625f : 1.0f);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (n0 + e >= p.N) break;
                    const float be = __half2float(__ushort_as_half((unsigned short)e_b_raw[e]));
                    float v;
                    if (W4) v = __builtin_fmaf(sf[e], sxm, be);
                    else v = __builtin_fmaf((float)si[e] * sxm, __int_as_float(e_sw_raw[e]), be);
                    asm("" : "+v"(v));   // rounded to fp32, then to fp16, as in the tile kernels' epilogue
                    p.y[(size_t)m * p.ldy + n0 + e] = __float2half_rn(v);
                }
            }
        }
    }
}

template <bool W4, int MH, int C, int EPI, int WAVES, bool XL = false, int FQ = 0, bool OVL = false>
int launch_one(const GemmArgs &a, hipStream_t st)
{
    DecodeParams p;
    p.x = a.x;
    p.ldx = a.ldx;
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
    p.x_bytes = (unsigned)act_kernel_bytes(a.M, a.K);
    p.w_bytes = (unsigned)(W4 ? (size_t)p.Npad * a.K / 2 : w8_kernel_bytes(a.N, a.K));
    p.wscales = W4 ? reinterpret_cast<const __half *>(p.wq + w4_scales_dec_offset(a.N, a.K, a.group)) : nullptr;
    const int grid = ceil_div(p.Npad / 16, C);
    const size_t xs_bytes = (XL ? (size_t)(a.M + 1) * a.K : 0) + (W4 ? (size_t)C * (a.K / 128) * 32 : 0);
    if (XL || W4) {   // static reduction buffer + staged tokens/scales can exceed the default 64 KB limit
        // once per kernel and process; the initialisation of a function-local static is thread-safe
        static const hipError_t attr_status = hipFuncSetAttribute(
            reinterpret_cast<const void *>(gemm_decode_kernel<W4, MH, C, EPI, WAVES, XL, FQ, OVL>),
            hipFuncAttributeMaxDynamicSharedMemorySize, 40960 + 32768);
        QL_TRY(check_hip(attr_status, "hipFuncSetAttribute(max dynamic LDS)"));
    }
    hipLaunchKernelGGL((gemm_decode_kernel<W4, MH, C, EPI, WAVES, XL, FQ, OVL>), dim3(grid, MH >= 2 ? ceil_div(a.M, 16 * MH) : 1),
                       dim3(WAVES * 64), xs_bytes, st, p);
    return check_hip(hipGetLastError(), "gemm_decode launch");
}

// From 33 tokens on the kernels work on blocks of 64 or 32 tokens (blockIdx.y).  Every workgroup pulls its token
// block and its C*16 channels over the whole K through its CU's L1 -- measured ~50 GB/s per CU with a ring of
// at least two fragments per channel group (C <= 4), ~40 GB/s with one (C = 6, 8).  Its registers allow one
// workgroup per CU, so workgroups beyond 256 run in further passes, each paying its own first round trip to
// HBM and its reduction (2.5 us): 1 us + passes x (2.5 us + bytes per workgroup / rate).  Blocks of 32 tokens
// read the weights twice (the second time from L2) but halve the tokens a workgroup pulls: they win when N is
// small (N = 4096, 64 tokens: 256 workgroups of 32 channels x 32 tokens instead of 16 x 64).  On 16 layer
// shapes of 1.5B..70B models at 33..256 tokens the C this picks for blocks of 64 was the fastest measured one;
// the time is within ~20 % of the measured one and is what the caller compares with the tile kernels' estimate.
struct BlockedPlan {
    int block, c;
    double us;
};

inline BlockedPlan plan_blocked(int M, int N, int K, bool w4, int force_block = 0)
{
    const int groups = round_up(N, TILE_ROWS) / 16;
    static const int cs[] = {1, 2, 3, 4, 6, 8};
    BlockedPlan best = {64, 1, 1e30};
    for (int block = 64; block >= 32; block /= 2) {
        if (force_block && block != force_block) continue;
        const int blocks = ceil_div(M, block);
        const int tokens = M >= block ? block : round_up(M, 16);
        for (int c : cs) {
            if (c > 4 && (w4 || block == 32)) continue;   // int4: register budget; 32-token kernels: 6 or 8 measured no faster
            if (w4 && (size_t)c * (K / 128) * 32 > 16384) continue;            // int4: staged scales
            const double passes = (double)ceil_div(ceil_div(groups, c) * blocks, 256);
            const double us = 1.0 + passes * (2.5 + K * ((w4 ? 8.0 : 16.0) * c + tokens) / (c <= 4 ? 50e3 : 40e3));
            if (us < best.us) best = {block, c, us};
        }
    }
    return best;
}

// Token block and channel groups per workgroup of the automatic choice.
// The token fragments are re-read from L2 by every workgroup; their traffic relative to the weight
// stream is (tokens rounded up to 16) / (16 * C).  More channel groups per workgroup cut it, at the
// price of fewer workgroups, so C grows with M and shrinks again when N is too small to fill 256 CUs.
inline void auto_shape(int M, int N, int K, bool w4, int force_block, int &block, int &c)
{
    const int groups = round_up(N, TILE_ROWS) / 16;
    if (M <= 16) {
        // Every workgroup streams c channel groups (16 c channels x K weight bytes) plus the tokens (M x K bytes); all
        // workgroups are resident at once up to two per CU, beyond that the rest is handed out as CUs free up.  The
        // busiest CU decides: rounds x bytes per workgroup, in units of one channel group's weights.  Measured on the
        // 7B shapes: the pick is the fastest or within 3 % of it (e.g. QKV: 256 workgroups of 48 channels instead of
        // 384 of 32, which left half the CUs with twice the work; int4 gate+up at 8 tokens 12.3 -> 10.3 us).
        block = 16;
        const double tokens = (double)M / (w4 ? 8.0 : 16.0);
        double best = 1e30;
        c = 1;
        for (int cand = 1; cand <= 4; ++cand) {
            if (w4 && (size_t)cand * (K / 128) * 32 > 16384) break;      // int4: staged scales
            const int wgs = ceil_div(groups, cand);
            const double rounds = wgs <= 512 ? (double)ceil_div(wgs, 256) : wgs / 256.0 + 1.0;
            const double cost = rounds * (cand + tokens);
            if (cost < best * 0.999) best = cost, c = cand;
        }
    } else if (M <= 32) {
        // 17..32 tokens: one block of 32 in the same model as the larger token counts (measured at 20 and 32 tokens on
        // five wide layers: the C it picks was the fastest of those tried, up to 27 % ahead of a fixed rule by N)
        block = 32, c = plan_blocked(M, N, K, w4, 32).c;
    } else {   // blocks of 64 or 32 tokens
        const BlockedPlan plan = plan_blocked(M, N, K, w4, force_block);
        c = plan.c, block = plan.block;
    }
    if (w4) {   // the staged scales (C * K/128 * 32 bytes of LDS) must stay small
        while (c > 1 && (size_t)c * (K / 128) * 32 > 16384) --c;
    }
}

template <bool W4, int EPI>
int by_m(const GemmArgs &a, int variant, hipStream_t st)
{
    const int groups = round_up(a.N, TILE_ROWS) / 16;
    int block, c;
    auto_shape(a.M, a.N, a.K, W4, variant == 122 ? 32 : variant == 123 ? 64 : 0, block, c);
    if (variant == 101 || variant == 111) c = 1;
    if (variant == 102 && (!W4 || (size_t)2 * (a.K / 128) * 32 <= 16384)) c = 2;
    if (variant == 103 && (!W4 || (size_t)3 * (a.K / 128) * 32 <= 16384)) c = 3;
    if (variant == 104 && (!W4 || (size_t)4 * (a.K / 128) * 32 <= 16384)) c = 4;
    if ((variant == 106 || variant == 108) && !W4 && a.M > 32 && block == 64) c = variant - 100;
    // 16 wavefronts (K split 16 ways) when there is at most one workgroup per CU: twice the bytes in flight
    const bool wide = c == 1 && (groups <= 256 || variant == 111) && variant != 101 && a.M <= 32;
    // few tokens can be staged in LDS (ring slots then hold weights only).  Measured: it pays for int4 weights
    // with 8 wavefronts (gate+up at up to 5 tokens 13.5 -> 11.4 us: the short int4 ring no longer shares its
    // registers with token fragments), makes no difference for int8 weights, and costs 0.7-1.1 us with 16
    // wavefronts -- so it is used there, and as the vehicle of the fused quantization below.
    const bool fits = (size_t)(a.M + 1) * a.K <= FQ_MAX_LDS && a.M <= 16 && variant != 121;   // keeps 4 workgroups per CU
    if (a.x && !W4 && variant == 100) {
        // fused quantization, int8 weights: measured faster with at most 32 channels per workgroup (QKV, one token:
        // 10.4 us against 11.6 with 48) -- every workgroup quantizes all tokens before its first multiply
        c = 2;
        while (c > 1 && ceil_div(groups, c) < 320) c /= 2;
    }
    if (a.x) {   // fp16 tokens: quantize in the prologue (the caller checked decode_fuses_quant); always 8 wavefronts
        if (EPI != EPI_F16 || !fits || a.M > FQ_MAX_M) return fail(QL_ERR_UNSUPPORTED, "fused quantization: unsupported shape");
        // 16-k pieces of a wavefront's k-range x tokens (rounded up to a power of two) <= 64 lanes x 2 slots
        const int pieces = W4 ? 8 * ceil_div(a.K / 128, 8) : 4 * ceil_div(a.K / 64, 8);
        const int mp = a.M <= 1 ? 1 : a.M <= 2 ? 2 : 4;
        if (pieces * mp > 128) return fail(QL_ERR_UNSUPPORTED, "fused quantization: unsupported shape");
        if constexpr (EPI == EPI_F16) {
            // at most one workgroup per CU: the quantizer overlaps the first ring of weights (OVL)
            if (ceil_div(round_up(a.N, TILE_ROWS) / 16, c) <= 256) {
                if (c == 1) return launch_one<W4, 1, 1, EPI, 8, true, 2, true>(a, st);
                if (c == 2) return launch_one<W4, 1, 2, EPI, 8, true, 2, true>(a, st);
                if (c == 3) return launch_one<W4, 1, 3, EPI, 8, true, 2, true>(a, st);
                return launch_one<W4, 1, 4, EPI, 8, true, 2, true>(a, st);
            }
            if (c == 1) return launch_one<W4, 1, 1, EPI, 8, true, 2>(a, st);
            if (c == 2) return launch_one<W4, 1, 2, EPI, 8, true, 2>(a, st);
            if (c == 3) return launch_one<W4, 1, 3, EPI, 8, true, 2>(a, st);
            return launch_one<W4, 1, 4, EPI, 8, true, 2>(a, st);
        }
    }
    const bool xl = fits && ((W4 && !wide) || variant == 111 || (variant >= 101 && variant <= 104));
    if (xl) {
        if (wide) return launch_one<W4, 1, 1, EPI, 16, true>(a, st);
        if (c == 1) return launch_one<W4, 1, 1, EPI, 8, true>(a, st);
        if (c == 2) return launch_one<W4, 1, 2, EPI, 8, true>(a, st);
        if (c == 3) return launch_one<W4, 1, 3, EPI, 8, true>(a, st);
        return launch_one<W4, 1, 4, EPI, 8, true>(a, st);
    }
    if (a.M <= 16) {
        if (wide) return launch_one<W4, 1, 1, EPI, 16>(a, st);
        if (c == 1) return launch_one<W4, 1, 1, EPI, 8>(a, st);
        if (c == 2) return launch_one<W4, 1, 2, EPI, 8>(a, st);
        if (c == 3) return launch_one<W4, 1, 3, EPI, 8>(a, st);
        return launch_one<W4, 1, 4, EPI, 8>(a, st);
    }
    if (a.M > 32 && block == 64) {
        if (c == 1) return launch_one<W4, 4, 1, EPI, 8>(a, st);
        if (c == 2) return launch_one<W4, 4, 2, EPI, 8>(a, st);
        if (c == 3) return launch_one<W4, 4, 3, EPI, 8>(a, st);
        if constexpr (!W4) {
            if (c == 6) return launch_one<W4, 4, 6, EPI, 8>(a, st);
            if (c == 8) return launch_one<W4, 4, 8, EPI, 8>(a, st);
        }
        return launch_one<W4, 4, 4, EPI, 8>(a, st);
    }
    if (wide) return launch_one<W4, 2, 1, EPI, 16>(a, st);
    if (c == 1) return launch_one<W4, 2, 1, EPI, 8>(a, st);
    if (c == 2) return launch_one<W4, 2, 2, EPI, 8>(a, st);
    if (c == 3) return launch_one<W4, 2, 3, EPI, 8>(a, st);
    return launch_one<W4, 2, 4, EPI, 8>(a, st);
}

}  // namespace

// The linear-layer entry points hand fp16 tokens straight to the decode GEMM when this holds (the same
// condition that stages the tokens in LDS, and few enough tokens that every workgroup re-reading and
// re-quantizing all of them costs less than a kernel launch).
bool decode_fuses_quant(int M, int K, int variant)
{
    // a wavefront (of at least 8) keeps its k-range in registers: at most 2 x 64 pieces of 16 k, tokens rounded up
    // to a power of two (int4 splits whole 128-k groups, int8 64-k chunks: bound both)
    const int pieces = ceil_div(ceil_div(K, 128), 8) * 8;
    const int mp = M <= 1 ? 1 : M <= 2 ? 2 : 4;
    return M >= 1 && M <= FQ_MAX_M && (size_t)(M + 1) * K <= FQ_MAX_LDS && pieces * mp <= 128 && variant != 121 &&
           variant != 130;
}

double decode_estimate_us(const GemmArgs &a)
{
    // up to 32 tokens: launch, first round trip and reduction + the weight stream at 90 % of nominal HBM bandwidth
    // (fits the measured 7B decode GEMMs within 10 %); from 33 tokens the blocked plan's model
    if (a.M <= 32) return 3.5 + (double)a.N * a.K * a.bits / 8.0 / 7.2e6;
    return plan_blocked(a.M, a.N, a.K, a.bits == 4).us;
}

void decode_plan(const GemmArgs &a, int *token_block, int *channel_groups)
{
    auto_shape(a.M, a.N, a.K, a.bits == 4, 0, *token_block, *channel_groups);
}

int launch_gemm_decode(const GemmArgs &a, int variant, hipStream_t st)
{
    if (a.M == 0) return QL_OK;
    const bool dump = a.acc != nullptr;
    if (a.bits == 4) return dump ? by_m<true, EPI_ACC>(a, variant, st) : by_m<true, EPI_F16>(a, variant, st);
    return dump ? by_m<false, EPI_ACC>(a, variant, st) : by_m<false, EPI_F16>(a, variant, st);
}

}  // namespace ql
